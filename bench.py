#!/usr/bin/env python3
"""Benchmark of the optimizer-step hot path on one MI355X.

One step = the whole path over one batch of synthetic state: gradient scan (overflow flag +
sum of squares), device-side gate and clip, AdamW update of fp32 p/m/v with the low-precision
parameter copy.  Inputs are resident in HBM before the timed region starts.  Prints ONE JSON
line: whole-job Gparam/s, the HBM roofline of the dominant (update) kernel measured with
stream events inside the timed region, and the CPU oracle timed on the host cores on a
bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--also none]

With no --workload the line describes the 8B-shaped list (K timed steps) and carries, measured in the
same process after the timed region: "also" = the other workloads below (their own short runs),
roofline.frac_plain = the same kernel with the state in an ordinary allocation,
check_fp32_by_model = the fused overflow / norm check alone over fp32 flat gradient buffers of four model sizes, and
roofline.mix_ceiling_GBps = what a trivial kernel with the same stream mix reaches on the same buffers.

Workloads: llama3_8b (default; 290-tensor Llama-3-8B-shaped list, 8.03e9 elements, bf16
gradients, clip 1.0; --layout tensor|streams), flat_1e8, fp16_5e7, share8_8b (a flat slice of 1/8 of the 8B list: one data-parallel rank's share over eight GPUs),
c1, c1_onecall (c1 through the whole-step call), c1_graph (those calls replayed as one HIP graph), qwen14b_4sub (12.57e9 elements as 4 flat
sub-groups streamed on one stream); rows beyond the basic step at the 8B element count:
fp32grad_8b (the 8B list with fp32 gradients: the accumulated flat buffer of Sec. III-C as input,
4 + 30 B/param), bf16_states_8b (p/m/v held in bf16, truncating stores, 14 B/param), accumulate_8b (4 bf16
micro-batch gradients into the fp32 flat buffer, 6 / 10 B/param), accumulate1_8b (one micro-batch per
step: the overwrite fused with the scan), iteration_8b (that pass followed by the gated update reading
the fp32 buffer: one whole iteration in the order of Sec. IV-A, 6 + 30 B/param), auto_fp16_8b (fp16
gradients, loss scale, update number and gate all read on the device).
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2505_23254_amd import hbm, synth  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
STEP_BYTES_PER_PARAM = 28.0    # update kernel: read p,m,v (12) + g (2), write p,m,v (12) + p_lp (2)
SCAN_BYTES_PER_PARAM = 2.0     # scan kernel: read g


# HBM bytes per launch of each workload's dominant kernel from hardware counters (rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE, scaled by a plain copy of known size; summaries under profiles/).  Valid
# only for the kernel sources they were taken with: when the digest of the sources a workload's
# kernels are built from differs, the figure is reported as null.
STEP_SOURCES = ("ma_device.h", "ma_internal.h", "ma_norm.hip", "ma_adamw.hip")
ACCUM_SOURCES = ("ma_device.h", "ma_internal.h", "ma_norm.hip", "ma_accum.hip")
STEP_SHA256 = "89c2b05c0092404313d34a01e6d704e58e6833b33dc7fa1c83da8aa9318592f1"
ACCUM_SHA256 = "db74af454226034f9c1f11421ec1510a983596dffcaefeabd12dfe2997cc1086"
MEASURED_TRAFFIC = {      # workload: (bytes per launch, sources, their digest when measured)
    "llama3_8b": (224847131614, STEP_SOURCES, STEP_SHA256),
    "flat_1e8": (2800277378, STEP_SOURCES, STEP_SHA256),
    "fp16_5e7": (1400285898, STEP_SOURCES, STEP_SHA256),
    "fp32grad_8b": (240908399879, STEP_SOURCES, STEP_SHA256),
    "auto_fp16_8b": (224847117850, STEP_SOURCES, STEP_SHA256),
    "qwen14b_4sub": (87973259267, STEP_SOURCES, STEP_SHA256),
    "bf16_states_8b": (112423952863, STEP_SOURCES, STEP_SHA256),
    "accumulate_8b": (80301678360, ACCUM_SOURCES, ACCUM_SHA256),
    "iteration_8b": (240908599968, STEP_SOURCES, STEP_SHA256),
    "share8_8b": (28105993608, STEP_SOURCES, STEP_SHA256),
    "accumulate1_8b": (48182763199, ACCUM_SOURCES, ACCUM_SHA256),
}


TRAFFIC_SOURCE = {
    "llama3_8b": "profiles/step_and_norm_multi_kernels__llama3_8b.txt",
    "flat_1e8": "profiles/step_and_norm_flat_kernels__flat_1e8.txt",
    "fp16_5e7": "profiles/step_and_norm_flat_kernels__fp16_5e7.txt",
    "fp32grad_8b": "profiles/step_and_norm_multi_kernels__fp32grad_8b.txt",
    "auto_fp16_8b": "profiles/step_and_norm_multi_kernels__auto_fp16_8b.txt",
    "qwen14b_4sub": "profiles/step_and_norm_flat_kernels__qwen14b_4sub.txt",
    "bf16_states_8b": "profiles/step_flat_kernel_bf16_states__bf16_states_8b.txt",
    "accumulate_8b": "profiles/accumulate_kernel__accumulate_8b.txt",
    "iteration_8b": "profiles/accumulate_scan_and_step_multi_kernels__iteration_8b.txt",
    "share8_8b": "profiles/step_and_norm_flat_kernels__share8_8b.txt",
    "accumulate1_8b": "profiles/accumulate_kernel_overwrite_scan__accumulate1_8b.txt",
}


def kernel_digest(sources=STEP_SOURCES):
    import hashlib
    h = hashlib.sha256()
    for f in sources:
        with open(os.path.join(ROOT, "paper_2505_23254_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload):
    if workload in MEASURED_TRAFFIC:
        nbytes, sources, digest = MEASURED_TRAFFIC[workload]
        if kernel_digest(sources) == digest:
            return nbytes
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Workload:
    """Holds device state and enqueues one step; records (scan, update) event pairs."""

    def __init__(self, name, ma, layout="streams", arena=None, rotate=1):
        # arena: an hbm.StitchedArena (placement "stitched": the state is cut from a range that the
        # library mapped from physical blocks of known HBM region: p | m | v | g at the offset that splits
        # their traffic evenly over two of the three 96 GiB regions, the write-only parameter copy in
        # the third), an hbm.DeviceArena (placement "region": the same cut from one whole-device
        # allocation), or None (placement "plain": a fresh allocation of just the state's size,
        # wherever the driver puts it)
        self.name, self.ma, self.layout = name, ma, "flat"
        self.placement = arena.placement if arena is not None else "plain"
        self.device_arena = arena
        def place(nbytes, traffic):
            if self.device_arena is None:
                return None
            try:
                return self.device_arena.window(nbytes, traffic)
            except ValueError as e:        # the arena is smaller than the state
                log("bench.py: %s; falling back to a plain allocation" % e)
                self.device_arena = None
                self.placement = "plain"
                torch.cuda.empty_cache()
                return None

        def place_state(parts, traffic):
            """p | m | v | g and p_lp as two views (see hbm.DeviceArena.split_window)."""
            if self.device_arena is None:
                return None
            try:
                return self.device_arena.split_window(parts[0], traffic[:4], parts[1])
            except ValueError as e:
                log("bench.py: %s; falling back to a plain allocation" % e)
                self.device_arena = None
                self.placement = "plain"
                torch.cuda.empty_cache()
                return None

        self.ws = ma.workspace()
        self.res = ma.new_result()
        self.t = 100
        self.events = []
        self.step_bytes = STEP_BYTES_PER_PARAM
        self.kernel_label = "AdamW update (+ low-precision copy)"
        if name in ("llama3_8b", "fp32grad_8b"):
            cfg = synth.FlatConfig(name, 0, seed=3, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
            if name == "fp32grad_8b":      # the accumulated fp32 flat gradient buffer as the step's input
                cfg.gdt = "f32"
                self.step_bytes = 30.0      # read p, m, v (12) + g (4), write p, m, v (12) + p_lp (2)
            self.cfg = cfg
            self.layout = layout
            shapes = synth.llama3_8b_shapes()
            where = (place_state(synth.list_state_parts(shapes, gdt=cfg.gdt), synth.list_traffic(shapes, gdt=cfg.gdt))
                     if layout == "streams" else
                     place(synth.list_state_bytes(shapes, layout, gdt=cfg.gdt), None))
            self.state = synth.make_list(shapes, cfg, device="cuda", layout=layout, arena=where)
            self.plan = ma.MultiPlan(self.state.p, self.state.m, self.state.v, self.state.g,
                                     self.state.p_lp)
            self.n = self.plan.total
            self.kind = "multi"
            self.desc = ("290-tensor Llama-3-8B-shaped list, %d elements, fp32 p/m/v, %s grads "
                         "~N(0,1e-3), clip 1.0; layout '%s', placement '%s'"
                         % (self.n, cfg.gdt, layout, self.placement))
        elif name == "qwen14b_4sub":
            cfg = synth.FlatConfig(name, 0, seed=4, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
            self.cfg = cfg
            total = sum(n for _, n in synth.qwen14b_class_shapes())
            self.flat = synth.make_flat(cfg, device="cuda", n=total,
                                        arena=place_state(synth.flat_state_parts(total), synth.flat_traffic(total)))
            self.n = total
            self.kind = "sub"
            self.parts = ma.new_result(4)
            self.desc = ("14B-class list (%d elements) as 4 equal flat sub-groups streamed on one "
                         "stream, bf16 grads, clip 1.0" % total)
        elif name in ("bf16_states_8b", "accumulate_8b", "accumulate1_8b"):
            # flat sub-groups of the 8B element count for the rows beyond the basic step
            n = sum(k for _, k in synth.llama3_8b_shapes())
            cfg = synth.FlatConfig(name, n, seed=5, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
            self.cfg, self.n = cfg, n
            up = lambda x: (x + synth.ARENA_ALIGN - 1) // synth.ARENA_ALIGN * synth.ARENA_ALIGN
            if name == "bf16_states_8b":
                sizes, weights = [up(2 * n)] * 4, (2.0, 2.0, 2.0, 1.0)
                self.step_bytes, self.kind = 14.0, "bf16"
                self.kernel_label = "AdamW update, bf16 p/m/v stored by truncation"
                self.desc = "flat sub-group n=%d, bf16 p/m/v (truncating stores), bf16 grads, clip 1.0" % n
            else:
                sizes, weights = [up(4 * n), up(2 * n)], (2.0, 1.0)
                self.step_bytes, self.kind = 10.0, "accum"
                self.micro = 4 if name == "accumulate_8b" else 1
                self.kernel_label = "gradient accumulation into the fp32 flat buffer (2nd and later micro-batches)"
                self.desc = ("fp32 flat gradient buffer n=%d, %d bf16 micro-batch gradients per step "
                             "(first overwrites, the others add, the last add is fused with the "
                             "overflow / norm scan of the buffer)" % (n, self.micro))
                if self.micro == 1:      # one micro-batch per iteration: the overwrite itself carries the scan
                    self.step_bytes = 6.0
                    self.kernel_label = "overwrite of the fp32 flat buffer fused with the overflow / norm scan"
                    self.desc = ("fp32 flat gradient buffer n=%d, one bf16 micro-batch gradient per step: "
                                 "overwrite fused with the overflow / norm scan of the buffer" % n)
            buf = place(sum(sizes), list(zip(sizes, weights)))
            if buf is None:
                buf = torch.empty(sum(sizes), dtype=torch.uint8, device="cuda")
            self.raw = buf
            offs = [sum(sizes[:i]) for i in range(len(sizes))]
            gen = torch.Generator(device="cuda")
            gen.manual_seed(cfg.seed)
            if name == "bf16_states_8b":
                self.bp, self.bm, self.bv, self.bg = (buf[o:o + 2 * n].view(torch.bfloat16) for o in offs)
                for t, std in ((self.bp, cfg.p_std), (self.bm, cfg.m_std), (self.bv, cfg.v_std), (self.bg, cfg.g_std)):
                    synth._fill_grad(t, std, 1.0, gen)
                self.bv.abs_()
            else:
                self.acc = buf[offs[0]:offs[0] + 4 * n].view(torch.float32)
                self.bg = buf[offs[1]:offs[1] + 2 * n].view(torch.bfloat16)
                synth._fill_grad(self.bg, cfg.g_std, 1.0, gen)
        elif name == "iteration_8b":
            # Sec. IV-A's order: the micro-batch gradient goes into the fp32 flat gradient buffer, the
            # overflow / norm check is fused into that pass, the gated step reads the buffer (fp32)
            cfg = synth.FlatConfig(name, 0, seed=3, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
            cfg.gdt = "f32"
            self.cfg, self.layout = cfg, "streams"
            shapes = synth.llama3_8b_shapes()
            n = sum(k for _, k in shapes)
            parts, traffic = synth.list_state_parts(shapes, gdt="f32"), synth.list_traffic(shapes, gdt="f32")
            up = lambda x: (x + synth.ARENA_ALIGN - 1) // synth.ARENA_ALIGN * synth.ARENA_ALIGN
            where, mb = None, None
            if self.device_arena is not None:      # the 16-bit micro-batch gradient lies behind the copy
                try:
                    main, side = self.device_arena.split_window(parts[0], traffic[:4], up(parts[1]) + 2 * n)
                    where = (main, side[:parts[1]])
                    mb = side[up(parts[1]):up(parts[1]) + 2 * n].view(torch.bfloat16)
                except ValueError as e:
                    log("bench.py: %s; falling back to a plain allocation" % e)
                    self.device_arena, self.placement = None, "plain"
            self.state = synth.make_list(shapes, cfg, device="cuda", layout="streams", arena=where)
            self.mb = mb if mb is not None else torch.empty(n, dtype=torch.bfloat16, device="cuda")
            gen = torch.Generator(device="cuda")
            gen.manual_seed(cfg.seed + 1)
            synth._fill_grad(self.mb, cfg.g_std, 1.0, gen)
            self.plan = ma.MultiPlan(self.state.p, self.state.m, self.state.v, self.state.g, self.state.p_lp)
            self.n = self.plan.total
            assert self.state.flat.g.numel() == self.n
            self.kind, self.step_bytes = "iter", 30.0
            self.desc = ("one iteration on the 8B-shaped list: a bf16 micro-batch gradient is written into the "
                         "fp32 flat gradient buffer with the overflow / norm check fused into that pass, then "
                         "the gated update reads the buffer as fp32 gradients; placement '%s'" % self.placement)
        elif name == "auto_fp16_8b":
            cfg = synth.FlatConfig(name, 0, seed=7, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0,
                                   gdt="f16", loss_scale=65536.0)
            self.cfg = cfg
            self.layout = layout
            shapes = synth.llama3_8b_shapes()
            where = (place_state(synth.list_state_parts(shapes), synth.list_traffic(shapes))
                     if layout == "streams" else place(synth.list_state_bytes(shapes, layout), None))
            self.state = synth.make_list(shapes, cfg, device="cuda", layout=layout, arena=where)
            self.plan = ma.MultiPlan(self.state.p, self.state.m, self.state.v, self.state.g,
                                     self.state.p_lp)
            self.n = self.plan.total
            self.kind = "auto"
            self.scaler = ma.new_scaler(cfg.loss_scale, 99)
            self.scaler_cfg = ma.scaler_config(window=1000)
            self.desc = ("8B-shaped list, fp16 grads at loss scale 65536 kept on the device: scan, gated "
                         "update and loss-scale update without host round trip; layout '%s'" % layout)
        else:
            # c1_onecall: the same sub-group through ma_optimizer_step (two launches instead of three)
            # c1_graph: those calls for all the rotating sub-groups captured once as a HIP graph; a step
            # is then one replay
            self.onecall = name in ("c1_onecall", "c1_graph")
            if name == "share8_8b":      # one data-parallel rank's share of the 8B list over eight GPUs, as a flat slice
                cfg = synth.FlatConfig(name, sum(k for _, k in synth.llama3_8b_shapes()) // 8, seed=9, m_std=1e-4,
                                       v_std=1e-8, step=100, max_norm=1.0)
            else:
                cfg = synth.config({"flat_1e8": "c2", "fp16_5e7": "c3a", "c1": "c1", "c1_onecall": "c1", "c1_graph": "c1"}[name])
            self.cfg = cfg
            self.flat = synth.make_flat(cfg, device="cuda",
                                        arena=place_state(synth.flat_state_parts(cfg.n, cfg.gdt),
                                                          synth.flat_traffic(cfg.n, cfg.gdt)))
            # --rotate K: K distinct sub-groups of this shape, one per step in turn, so that a small
            # sub-group is measured from HBM and not from the caches (256 MB of Infinity Cache)
            self.flats = [self.flat]
            for k in range(1, rotate):
                other = synth.FlatConfig(**{**cfg.__dict__, "seed": cfg.seed + 1000 * k})
                self.flats.append(synth.make_flat(other, device="cuda"))
            self.n = cfg.n
            self.t = cfg.step
            self.kind = "flat"
            if self.onecall:
                self.kernel_label = "AdamW update that adds up the scan's partials itself (no finalize launch)"
            self.graph = None
            if name == "c1_graph":
                h = ma.hyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)
                one = lambda f: ma.optimizer_step(f.p, f.m, f.v, f.g, f.p_lp, h, self.t, cfg.loss_scale,
                                                  cfg.max_norm, self.res, self.ws)
                one(self.flats[0])                 # the kernels are loaded before the capture
                torch.cuda.synchronize()
                self.graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(self.graph):
                    for f in self.flats:
                        one(f)
                # one step = one replay = a step of every sub-group (update number fixed at capture; a
                # training loop keeps it on the device instead: the *_auto calls)
                self.graph_steps = len(self.flats)
                self.n = cfg.n * self.graph_steps
                self.kernel_label = "scan + update launches of %d sub-groups replayed as one HIP graph" % self.graph_steps
            self.desc = "%sflat sub-group n=%d, %s grads, loss_scale %g, max_norm %g%s" % (
                "" if self.graph is None else "one HIP graph of %d whole-step calls, one per " % self.graph_steps,
                cfg.n, cfg.gdt, cfg.loss_scale, cfg.max_norm,
                "" if rotate == 1 else "; %d distinct sub-groups in rotation (%.0f MB of state)" % (
                    rotate, rotate * synth.flat_state_bytes(cfg.n) / 1e6))
        c = self.cfg
        self.h = ma.hyper(c.lr, c.beta1, c.beta2, c.eps, c.weight_decay, 1)

    def step(self, record):
        ma, c = self.ma, self.cfg
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if record else None
        if record:
            ev[0].record()
        if self.kind == "multi":
            ma.multi_overflow_norm(self.plan, c.loss_scale, self.res, self.ws)
            if record:
                ev[1].record()
            ma.multi_adamw_step_gated(self.plan, self.h, self.t, c.loss_scale, self.res, c.max_norm)
        elif self.kind == "iter":
            ma.grad_accumulate_scan(self.state.flat.g, self.mb, True, c.loss_scale, self.res, self.ws)
            if record:
                ev[1].record()
            ma.multi_adamw_step_gated(self.plan, self.h, self.t, c.loss_scale, self.res, c.max_norm)
        elif self.kind == "auto":
            ma.multi_overflow_norm_auto(self.plan, self.scaler, self.res, self.ws)
            if record:
                ev[1].record()
            ma.multi_adamw_step_auto(self.plan, self.h, self.scaler, self.res, c.max_norm)
            ma.scaler_update(self.scaler, self.res, self.scaler_cfg)
        elif self.kind == "bf16":
            ma.overflow_norm(self.bg, c.loss_scale, self.res, self.ws)
            if record:
                ev[1].record()
            ma.adamw_step_bf16_gated(self.bp, self.bm, self.bv, self.bg, self.h, self.t, c.loss_scale,
                                     self.res, c.max_norm)
        elif self.kind == "accum" and self.micro == 1:
            if record:
                ev[1].record()
            ma.grad_accumulate_scan(self.acc, self.bg, True, c.loss_scale, self.res, self.ws)
        elif self.kind == "accum":
            ma.grad_accumulate(self.acc, self.bg, first=True)
            if record:
                ev[1].record()
            for _ in range(self.micro - 2):
                ma.grad_accumulate(self.acc, self.bg, first=False)
            # the last micro-batch of an iteration is accumulated and scanned in one pass
            ma.grad_accumulate_scan(self.acc, self.bg, False, c.loss_scale, self.res, self.ws)
        elif self.kind == "flat" and self.graph is not None:
            if record:
                ev[1].record()
            self.graph.replay()
        elif self.kind == "flat" and self.onecall:
            f = self.flats[self.t % len(self.flats)]
            if record:      # both launches fall into the second interval
                ev[1].record()
            ma.optimizer_step(f.p, f.m, f.v, f.g, f.p_lp, self.h, self.t, c.loss_scale, c.max_norm,
                              self.res, self.ws)
        elif self.kind == "flat":
            f = self.flats[self.t % len(self.flats)]
            ma.overflow_norm(f.g, c.loss_scale, self.res, self.ws)
            if record:
                ev[1].record()
            ma.adamw_step_gated(f.p, f.m, f.v, f.g, f.p_lp, self.h, self.t, c.loss_scale, self.res,
                                c.max_norm)
        else:
            f, sub = self.flat, self.n // 4
            for k in range(4):
                ma.overflow_norm(f.g[k * sub:(k + 1) * sub], c.loss_scale, self.parts, self.ws, index=k)
            ma.norm_combine(self.parts, 4, self.res)
            if record:
                ev[1].record()
            for k in range(4):
                s = slice(k * sub, (k + 1) * sub)
                ma.adamw_step_gated(f.p[s], f.m[s], f.v[s], f.g[s], f.p_lp[s], self.h, self.t,
                                    c.loss_scale, self.res, c.max_norm)
        if record:
            ev[2].record()
            self.events.append(ev)
        self.t += 1


def host_threads():
    """Threads for the host baseline: this process's share of the box (its affinity mask, and the
    thread count the box sets for worker pools), not every core the machine has."""
    n = os.cpu_count() or 1
    try:
        n = min(n, len(os.sched_getaffinity(0)))
    except AttributeError:
        pass
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return n


def cpu_baseline(wl, sample_elems, passes):
    """The CPU oracle, as it stands, on the first `sample_elems` elements of the workload's state
    (copied to the host), on this process's share of the host cores; also one thread on a smaller piece."""
    import oracle
    c = wl.cfg
    if wl.kind == "multi":      # the list's first tensor (the embedding) is larger than any sample
        st = wl.state
        src = synth.FlatState(st.p[0], st.m[0], st.v[0], st.g[0], st.p_lp[0])
    else:
        src = wl.flat
    n = min(sample_elems, src.p.numel())
    p, m, v = (t[:n].cpu().numpy().copy() for t in (src.p, src.m, src.v))
    g = synth.bits16(src.g[:n])
    lp = synth.bits16(src.p_lp[:n])
    h = oracle.hyper(c.lr, c.beta1, c.beta2, c.eps, c.weight_decay, 1)
    cores = host_threads()
    oracle.optimizer_step(p, m, v, g, c.gdt, lp, c.pdt, h, 100, c.loss_scale, c.max_norm, nthreads=cores)
    t0 = time.perf_counter()
    for k in range(passes):
        oracle.optimizer_step(p, m, v, g, c.gdt, lp, c.pdt, h, 101 + k, c.loss_scale, c.max_norm,
                              nthreads=cores)
    dt = (time.perf_counter() - t0) / passes
    n1 = min(n, 1 << 24)
    t0 = time.perf_counter()
    oracle.optimizer_step(p[:n1], m[:n1], v[:n1], g[:n1], c.gdt, lp[:n1], c.pdt, h, 200, c.loss_scale,
                          c.max_norm, nthreads=1)
    dt1 = time.perf_counter() - t0
    return {
        "value": n / dt / 1e9, "unit": "Gparam/s", "cores": cores, "kind": "oracle",
        "host_cores_visible": os.cpu_count(),
        "sample": "first %d elements of the workload, %d full passes (scan+gate+update) over %d "
                  "threads (this process's share of the host: the machine shows %s cores); single "
                  "thread on %d elements: %.4f Gparam/s"
                  % (n, passes, cores, os.cpu_count(), n1, n1 / dt1 / 1e9),
        "single_thread_value": n1 / dt1 / 1e9,
    }


def run(wl, steps, warmup, events_in_region=True):
    """W untimed and K timed steps of one workload; returns ms per step (wall clock between two device
    synchronisations) and leaves per-step stream events in wl.events.  events_in_region=False: the
    timed steps carry no events and the events come from a second pass of the same steps (for steps
    of tens of microseconds, where recording three events per step costs as much as the step:
    n = 2^20 measured 21 us per step without and 40 us with events)."""
    for _ in range(warmup):
        wl.step(False)
    torch.cuda.synchronize()
    wl.events = []
    t0 = time.perf_counter()
    for _ in range(steps):
        wl.step(events_in_region)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    if not events_in_region:
        for _ in range(min(steps, 100)):
            wl.step(True)
        torch.cuda.synchronize()
    return ms


def summarise(wl, ma, ms_per_step, quiet=False):
    """value (Gparam/s) and the roofline of the workload's dominant kernel from the stream events."""
    first_ms = sum(e[0].elapsed_time(e[1]) for e in wl.events) / len(wl.events)
    rest_ms = sum(e[1].elapsed_time(e[2]) for e in wl.events) / len(wl.events)
    if not quiet:
        log("2nd phase ms per step: " + " ".join("%.3f" % e[1].elapsed_time(e[2]) for e in wl.events))
        log("1st phase ms per step: " + " ".join("%.3f" % e[0].elapsed_time(e[1]) for e in wl.events))
    if wl.kind != "accum" or wl.micro == 1:
        ov, ss = ma.read_result(wl.res)
        if ov:
            sys.exit("bench.py: unexpected overflow flag on clean synthetic gradients (%s)" % wl.name)
    else:
        ss = None
    # launches of the dominant kernel in the second phase of a step, and what precedes them
    launches = {"sub": 4, "accum": max(1, wl.micro - 1) if wl.kind == "accum" else 1}.get(wl.kind, 1)
    if getattr(wl, "graph", None) is not None:
        launches = wl.graph_steps
    passes = launches if wl.kind == "accum" else 1          # times the second phase sweeps all n elements
    achieved = wl.step_bytes * wl.n * passes / (rest_ms * 1e-3) / 1e9
    gdt_bytes = 4.0 if wl.cfg.gdt == "f32" else 2.0
    if wl.kind == "accum" and wl.micro == 1:
        first = None
        value = wl.n / (ms_per_step * 1e-3) / 1e9
        whole = 6.0 * wl.n / (ms_per_step * 1e-3) / 1e9
    elif wl.kind == "iter":
        first = {"kernel": "micro-batch gradient into the fp32 flat buffer, fused with the overflow / norm check",
                 "avg_ms": first_ms, "bytes_per_param": 6.0, "achieved": 6.0 * wl.n / (first_ms * 1e-3) / 1e9}
        value = wl.n / (ms_per_step * 1e-3) / 1e9
        whole = (6.0 + wl.step_bytes) * wl.n / (ms_per_step * 1e-3) / 1e9
    elif wl.kind == "accum":
        first = {"kernel": "first micro-batch (overwrite)", "avg_ms": first_ms, "bytes_per_param": 6.0,
                 "achieved": 6.0 * wl.n / (first_ms * 1e-3) / 1e9}
        value = wl.n * wl.micro / (ms_per_step * 1e-3) / 1e9       # micro-batch elements accumulated
        whole = (6.0 + 10.0 * (wl.micro - 1)) * wl.n / (ms_per_step * 1e-3) / 1e9
    else:
        onecall = getattr(wl, "onecall", False)      # no event between its two launches
        first = None if onecall else {"kernel": "gradient scan (+ finalize)", "avg_ms": first_ms,
                                      "bytes_per_param": gdt_bytes,
                                      "achieved": gdt_bytes * wl.n / (first_ms * 1e-3) / 1e9}
        value = wl.n / (ms_per_step * 1e-3) / 1e9
        whole = (gdt_bytes + wl.step_bytes) * wl.n / (ms_per_step * 1e-3) / 1e9
    traffic = measured_traffic(wl.name)
    roofline = {
        "bound": "hbm", "kernel": wl.kernel_label,
        "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
        "traffic_source": (TRAFFIC_SOURCE.get(wl.name) if traffic is not None else
                           "none: no counter run for this workload" if wl.name not in MEASURED_TRAFFIC else
                           "none: the kernel sources changed since the counters under profiles/ were taken"),
        "algorithmic_bytes_per_launch": wl.step_bytes * wl.n / (launches if wl.kind in ("sub", "flat") else 1),
        "bytes_per_param": wl.step_bytes,
        "params_per_launch": wl.n / (launches if wl.kind in ("sub", "flat") else 1),
        "avg_launch_ms": rest_ms / launches,
        "first_phase": first,
        "whole_step_GBps": whole,
    }
    return value, roofline, ss


def mix_ceiling(wl, ma, reps=5):
    """GB/s of the library's trivial same-mix kernel over the workload's own five flat buffers, where
    they lie (destroys their contents): the ceiling of a 1:1 read/write mix for this placement."""
    if wl.kind == "bf16":
        bufs, per, item = (wl.bp, wl.bm, wl.bv, wl.bg, None), 14.0, 8192
    else:
        f = wl.state.flat if wl.kind in ("multi", "auto") else getattr(wl, "flat", None)
        if f is None or f.g.element_size() != 2:
            return None
        bufs, per, item = (f.p, f.m, f.v, f.g, f.p_lp), 28.0, 4096
    ma.probe_update_mix(*bufs)
    best = 0.0
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        ma.probe_update_mix(*bufs)
        b.record()
        b.synchronize()
        n = bufs[0].numel() // item * item
        best = max(best, per * n / (a.elapsed_time(b) * 1e-3) / 1e9)
    return best


def release(wl):
    import gc
    for a in ("graph", "state", "plan", "flat", "flats", "raw", "bp", "bm", "bv", "bg", "acc", "mb", "device_arena"):
        if hasattr(wl, a):
            setattr(wl, a, None)
    gc.collect()
    torch.cuda.empty_cache()


def region_arena(ma):
    """The whole-device arena and its placement check, or (None, check) when the check fails."""
    try:
        arena = hbm.DeviceArena("cuda")
    except RuntimeError as e:      # e.g. another process holds most of the device
        log("bench.py: whole-device arena not available (%s)" % e)
        return None, None
    _, total = torch.cuda.mem_get_info()
    if arena.nbytes < 2 * hbm.REGION_BYTES + 16 * hbm.GIB:
        log("bench.py: the arena (%.0f GiB of %.0f) does not reach the third HBM region; its offsets "
            "may not map onto the regions as assumed" % (arena.nbytes / hbm.GIB, total / hbm.GIB))
    verify = arena.verify_regions(ma.probe_two_writes)
    log("placement check of the whole-device allocation (two write streams, GB/s): same region %s, different "
        "regions %s -> %s" % (verify["same_GBps"], verify["cross_GBps"], "verified" if verify["verified"] else "NOT verified"))
    if not verify["verified"]:
        arena.release()
        arena = None
        torch.cuda.empty_cache()
    return arena, verify


def stitched_arena(ma):
    """The library-built range (ma_arena_create) and its placement check, or (None, None)."""
    st = None
    # 84 + 84 + 32 GiB hold every workload (iteration_8b needs 30 GiB in the side part, the 14B-class
    # state 164 in the main part); 64 + 64 + 16 still hold the 8B-shaped list when less memory is free
    for half, side in ((84, 32), (64, 16)):
        try:
            st = hbm.StitchedArena(ma.Arena, half_bytes=half * hbm.GIB, side_bytes=side * hbm.GIB)
            break
        except Exception as e:      # noqa: BLE001 - any failure here means: try smaller, then a plain allocation
            log("bench.py: stitched arena of %d + %d + %d GiB not available (%r)" % (half, half, side, e))
    if st is None:
        return None, None
    verify = st.verify_regions(ma.probe_two_writes)
    verify["blocks_in_place"] = st.in_place
    log("stitched arena %s; check (two write streams, GB/s): same part %s, different parts %s -> %s"
        % (st.report, verify["same_GBps"], verify["cross_GBps"], "verified" if verify["verified"] else "NOT verified"))
    settle()
    return st, verify


# Sec. VI-B reports the fused overflow check per model size, on the fp32 flat gradient buffer.  The same
# here: the check (fp32 mask of Algorithm 1, fused with the sum of squares) over fp32 buffers with the
# element counts of four decoder shapes of the sizes the paper evaluates (embedding, per layer q / k /
# v / o, gate / up / down, two norm vectors, LM head; no biases).
CHECK_SHAPES = (("7B-class", (3584, 18944, 28, 4, 128, 152064)), ("8B-class", (4096, 14336, 32, 8, 128, 128256)),
                ("14B-class", (5120, 13824, 48, 8, 128, 152064)), ("32B-class", (5120, 27648, 64, 8, 128, 152064)))


def check_by_model(ma, arena, reps=5):
    ws, res = ma.workspace(), ma.new_result()
    rows = []
    for label, dims in CHECK_SHAPES:
        n = sum(k for _, k in synth.decoder_shapes(*dims))
        try:
            g = arena.window(4 * n, None).view(torch.float32)
        except ValueError:
            continue
        for a in range(0, n, 1 << 30):
            g[a:a + (1 << 30)].fill_(1e-3)
        ma.overflow_norm(g, 1.0, res, ws)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for k in range(reps):
            ma.overflow_norm(g, 1.0, res, ws)
            ev[k + 1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[reps]) / reps
        ov, ss = ma.read_result(res)
        if ov or abs(ss - 1e-6 * n) > 1e-6 * (1e-6 * n):
            sys.exit("bench.py: the check over the %s buffer returned overflow=%s, sumsq=%r" % (label, ov, ss))
        rows.append({"shape": label, "elements": n, "buffer_GiB": 4 * n / hbm.GIB, "ms": ms,
                     "GBps": 4.0 * n / (ms * 1e-3) / 1e9, "frac": 4.0 * n / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS})
        log("fused check, fp32 flat gradient buffer, %-9s %14d elements (%6.2f GiB): %7.3f ms  %.0f GB/s (%.1f %%)"
            % (label, n, 4 * n / hbm.GIB, ms, rows[-1]["GBps"], 100 * rows[-1]["frac"]))
    return rows


def settle():
    """Waits until the driver has wiped the device's free memory.  Memory that a process gave back
    (this one or the one before it) is wiped in the background, at 26 GB/s as measured, and while that
    runs every kernel is about 0.5 % slower (the scan 3 %).  Only free memory can be waiting for its
    wipe, so free bytes / 20 GB/s bounds the time."""
    free, _ = torch.cuda.mem_get_info()
    wait = free / hbm.StitchedArena.WIPE_BYTES_PER_S
    log("waiting %.1f s: the driver may still be wiping the %.0f GiB of free device memory" % (wait, free / hbm.GIB))
    time.sleep(wait)


# The other workloads a default run reports under "also": (name, timed steps, warm-up steps, rotate).
ALSO = (("c1", 400, 40, 32), ("c1_onecall", 400, 40, 32), ("c1_graph", 40, 5, 32), ("flat_1e8", 100, 10, 1), ("fp16_5e7", 100, 10, 1), ("share8_8b", 20, 4, 1), ("qwen14b_4sub", 8, 2, 1),
        ("fp32grad_8b", 8, 2, 1), ("iteration_8b", 8, 2, 1), ("auto_fp16_8b", 8, 2, 1), ("bf16_states_8b", 10, 2, 1),
        ("accumulate_8b", 5, 2, 1), ("accumulate1_8b", 8, 2, 1))


def extras_of(out, roofline, wl, ma, arena, name, args):
    """What a default run measures after the timed region (see the module docstring)."""
    t_extra = time.perf_counter()
    ceil = mix_ceiling(wl, ma)
    if ceil is not None:
        roofline["mix_ceiling_GBps"] = ceil
        roofline["frac_of_mix_ceiling"] = roofline["achieved"] / ceil
        log("mix ceiling (%s placement): %.0f GB/s" % (wl.placement, ceil))
    release(wl)
    also = out["also"] = []
    for other, steps, warmup, rotate in ALSO:
        if other == name:
            continue
        w2 = Workload(other, ma, "streams", arena, rotate)
        ms2 = run(w2, steps, warmup, events_in_region=w2.n >= 10 ** 9)
        v2, r2, _ = summarise(w2, ma, ms2, quiet=True)
        also.append({"workload": other, "description": w2.desc, "placement": w2.placement,
                     "steps": steps, "ms_per_step": ms2, "value": v2,
                     "kernel_events": "in the timed steps" if w2.n >= 10 ** 9 else "from a second pass",
                     "unit": "Gparam/s" if w2.kind != "accum" else "G micro-batch elements/s",
                     "roofline": {k: r2[k] for k in ("kernel", "achieved", "frac", "bytes_per_param",
                                                     "avg_launch_ms", "first_phase", "traffic")}})
        if getattr(w2, "graph", None) is not None:
            also[-1]["sub_group_steps_per_step"] = w2.graph_steps
            also[-1]["us_per_sub_group_step"] = 1e3 * ms2 / w2.graph_steps
        if w2.kind in ("bf16", "sub") or (w2.kind == "flat" and w2.n >= 10 ** 7 and getattr(w2, "graph", None) is None):
            also[-1]["roofline"]["mix_ceiling_GBps"] = mix_ceiling(w2, ma)
        log("also %-15s %9.4f ms/step  %8.2f %s  dominant kernel %.4f ms = %.0f GB/s (%.1f %%)  mix ceiling %s"
            % (other, ms2, v2, also[-1]["unit"], r2["avg_launch_ms"], r2["achieved"], 100 * r2["frac"],
               also[-1]["roofline"].get("mix_ceiling_GBps")))
        release(w2)
    if arena is not None:
        out["check_fp32_by_model"] = check_by_model(ma, arena)
    if name == "llama3_8b" and arena is not None:
        # the same list in an ordinary allocation: what a caller sees who does not place the state
        arena.release()
        arena = None
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        w3 = Workload(name, ma, args.layout, None, 1)
        torch.cuda.synchronize()
        settle()
        ms3 = run(w3, 8, 2)
        v3, r3, _ = summarise(w3, ma, ms3, quiet=True)
        roofline["frac_plain"] = r3["frac"]
        roofline["plain"] = {"placement": "plain", "ms_per_step": ms3, "value": v3,
                             "achieved": r3["achieved"], "avg_launch_ms": r3["avg_launch_ms"],
                             "mix_ceiling_GBps": mix_ceiling(w3, ma)}
        log("plain placement: %.3f ms/step, update %.0f GB/s (%.1f %%), mix ceiling %s GB/s"
            % (ms3, r3["achieved"], 100 * r3["frac"], roofline["plain"]["mix_ceiling_GBps"]))
        release(w3)
    log("extras took %.1f s" % (time.perf_counter() - t_extra))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    choices=["llama3_8b", "fp32grad_8b", "flat_1e8", "fp16_5e7", "share8_8b", "c1", "c1_onecall", "c1_graph", "qwen14b_4sub",
                             "bf16_states_8b", "accumulate_8b", "accumulate1_8b", "auto_fp16_8b", "iteration_8b"],
                    help="default: llama3_8b, followed by short runs of all the others (see --also)")
    ap.add_argument("--also", default=None, choices=["all", "none"],
                    help="after the timed region also run the other workloads, the plain-placement run and "
                         "the mix-ceiling probe ('all': the default when no --workload is given)")
    ap.add_argument("--layout", default="streams", choices=["streams", "tensor"],
                    help="llama3_8b only: how the list's buffers lie in the state: 'streams' = five flat "
                         "buffers p|m|v|g|p_lp (default), 'tensor' = the five buffers of each tensor adjacent")
    ap.add_argument("--placement", default="stitched", choices=["stitched", "region", "plain"],
                    help="'stitched' (default): the state lies in a range that ma_arena_create maps from "
                         "1-GiB physical blocks whose HBM region it finds by timing, so that the traffic of "
                         "p | m | v | g splits evenly over two 96 GiB regions and the write-only copy lies in "
                         "the third; 'region': the same split cut from one whole-device allocation, which maps "
                         "linearly onto the regions on a device whose memory has not been churned (checked; "
                         "falls back to 'stitched'); 'plain': a fresh allocation")
    ap.add_argument("--rotate", type=int, default=1, metavar="K",
                    help="flat_1e8 / fp16_5e7 / c1 only: step K distinct sub-groups of the workload's shape in "
                         "turn, so that a small sub-group is read from HBM rather than from the caches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=1 << 28)
    ap.add_argument("--cpu-passes", type=int, default=4)
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="after the timed region, run one plain device copy of BYTES bytes (reads "
                         "BYTES, writes BYTES): the known-size reference for hardware byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU's share of the optimizer step; "
                 "--gpus must be 1 (no collectives or sharding are part of it)")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    extras = (args.also or ("all" if args.workload is None else "none")) == "all"
    name = args.workload or "llama3_8b"

    from paper_2505_23254_amd import binding as ma  # fails loudly if the library is not built

    torch.cuda.set_device(0)
    arena, verify = None, None
    if args.placement == "region":
        arena, verify = region_arena(ma)
        if arena is None:
            log("bench.py: switching to the stitched placement (ma_arena_create)")
    if args.placement == "stitched" or (args.placement == "region" and arena is None):
        arena, verify = stitched_arena(ma)
        if arena is None:
            log("bench.py: falling back to a plain allocation")
    t_setup = time.perf_counter()
    wl = Workload(name, ma, args.layout, arena, max(1, args.rotate))
    torch.cuda.synchronize()
    log("setup %.1f s: %s" % (time.perf_counter() - t_setup, wl.desc))
    if wl.placement == "plain":
        settle()

    ms_per_step = run(wl, args.steps, args.warmup, events_in_region=wl.n >= 10 ** 9)

    if args.copy_calibration > 0:
        nb = args.copy_calibration
        if wl.placement == "region":         # the arena holds the device's memory: use its unused tail
            buf = wl.device_arena.buf
            fl = wl.state.flat if wl.kind in ("multi", "auto") else getattr(wl, "flat", None)
            used = [wl.raw] if wl.kind in ("bf16", "accum") else \
                [wl.state.arena] if fl is None else [fl.p, fl.m, fl.v, fl.g, fl.p_lp]
            end = max(t.data_ptr() + t.numel() * t.element_size() for t in used) - buf.data_ptr()
            tail = buf.numel() - end
            if tail < 2 * nb:
                sys.exit("bench.py: --copy-calibration needs %d free bytes behind the state" % (2 * nb))
            src, dst = buf[-2 * nb:-nb], buf[-nb:]
            src.fill_(1)
        else:
            src = torch.ones(nb, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        log("copy calibration: %d bytes read, %d bytes written" % (src.numel(), dst.numel()))
        del src, dst
    value, roofline, ss = summarise(wl, ma, ms_per_step)
    out = {
        "metric": "optimizer-step Gparam/s and achieved HBM GB/s (% of peak), 8B-shaped, 1 GPU",
        "value": value,
        "unit": "Gparam/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "description": wl.desc, "elements": wl.n,
                   "layout": wl.layout, "placement": wl.placement,
                   "placement_verified": None if verify is None or wl.placement == "plain" else verify["verified"],
                   "placement_check": verify,
                   "stitched_arena": wl.device_arena.report if wl.placement == "stitched" else None,
                   "rotating_sets": len(getattr(wl, "flats", None) or [None]),
                   "grad_dtype": wl.cfg.gdt, "param_copy_dtype": wl.cfg.pdt,
                   "max_norm": wl.cfg.max_norm, "loss_scale": wl.cfg.loss_scale,
                   "sumsq_last_step": ss},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline and wl.kind in ("multi", "flat", "sub"):
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample, args.cpu_passes)
    if extras:
        # whatever happens in the extras, the line with the headline is printed
        try:
            extras_of(out, roofline, wl, ma, arena, name, args)
        except (Exception, SystemExit) as e:      # noqa: BLE001
            log("bench.py: the extras stopped early: %r" % (e,))
            out["extras_error"] = repr(e)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
