"""The placement helper (ma_arena_*): the stitched range is ordinary device memory, every byte of it
mapped exactly once; it puts its parts into different HBM regions, which an independent timing
confirms; and it gives everything back."""
import pytest
import torch

from paper_2505_23254_amd import synth

pytestmark = pytest.mark.gpu
GIB = 1 << 30
MIB = 1 << 20


def test_small_arena_is_plain_memory_and_steps_identically():
    from paper_2505_23254_amd import binding as ma, hbm
    free0, _ = torch.cuda.mem_get_info()
    block = 64 * MIB
    a = ma.Arena(5 * block + 12345, 2 * block, block // 2, block_bytes=block, max_transient_bytes=GIB)
    rep = a.report
    assert rep["main_bytes"] == 6 * block and rep["side_bytes"] == block and rep["first_region_bytes"] == 2 * block
    assert 7 <= rep["blocks_created"] <= 16 and rep["regions_seen"] >= 1
    assert a.main.numel() == 5 * block + 12345 and a.side.numel() == block // 2
    assert a.side.data_ptr() == a.main.data_ptr() + 6 * block
    # every block is mapped once: a distinct value per MiB over the whole range, read back in full
    whole = torch.as_tensor(ma._RawDeviceBytes(a.main.data_ptr(), 7 * block, a), device="cuda").view(torch.int32)
    ids = torch.arange(7 * block // MIB, dtype=torch.int32, device="cuda").repeat_interleave(MIB // 4)
    whole.copy_(ids)
    assert torch.equal(whole, ids)
    del whole, ids
    a.close()
    # the blocks go back to the driver: a second arena of the same size, built and closed, leaves the
    # free memory where the first left it (the first may have loaded the library's kernels)
    torch.cuda.empty_cache()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 >= free0 - 7 * block                # (kernels and events of a first use: some tens of MB)
    ma.Arena(6 * block, 2 * block, block, block_bytes=block, max_transient_bytes=GIB).close()
    assert torch.cuda.mem_get_info()[0] >= free1 - 8 * MIB
    # no side part, everything in the second part: the degenerate request is served too
    b = ma.Arena(2 * block, 0, 0, block_bytes=block, max_transient_bytes=0)
    assert b.side is None and b.report["first_region_bytes"] == 0 and b.report["blocks_created"] == 2
    b.main.fill_(3)
    assert int(b.main[-1]) == 3
    b.close()
    # one step of a flat sub-group placed through the placement interface: bit-identical to the same
    # step in ordinary memory
    cfg = synth.config("c1")
    parts, traffic = synth.flat_state_parts(cfg.n, cfg.gdt), synth.flat_traffic(cfg.n, cfg.gdt)
    st = hbm.StitchedArena(ma.Arena, half_bytes=2 * block, side_bytes=block, max_transient_bytes=GIB, block_bytes=block)
    assert st.half == 2 * block and st.settle_seconds >= 0.0
    assert st.verify_regions(ma.probe_two_writes)["verified"] is False       # too small to probe, and says so
    main, side = st.split_window(parts[0], traffic[:4], parts[1])
    assert main.numel() == parts[0] and side.numel() == parts[1]
    # the window straddles the boundary between the two halves, half of its traffic on each side
    lo = main.data_ptr() - st.arena.main.data_ptr()
    assert lo < st.half < lo + parts[0] and abs((st.half - lo) - hbm.DeviceArena._midpoint(parts[0], traffic[:4])) <= hbm.ALIGN
    with pytest.raises(ValueError):
        st.window(5 * block)
    with pytest.raises(ValueError):
        st.split_window(parts[0], traffic[:4], 2 * block)
    inside = synth.make_flat(cfg, device="cuda", arena=(main, side))
    plain = synth.make_flat(cfg, device="cuda")
    lo = main.data_ptr()
    assert lo <= inside.p.data_ptr() < lo + parts[0] and inside.p_lp.data_ptr() == side.data_ptr()
    h = ma.hyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)
    ws, out = ma.workspace(), ma.new_result(2)
    for k, fl in enumerate((inside, plain)):
        ma.optimizer_step(fl.p, fl.m, fl.v, fl.g, fl.p_lp, h, cfg.step, cfg.loss_scale, cfg.max_norm, out, ws, index=k)
    torch.cuda.synchronize()
    for name in ("p", "m", "v", "p_lp"):
        x, y = getattr(inside, name), getattr(plain, name)
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), name
    assert ma.read_result_raw(out, 0) == ma.read_result_raw(out, 1)
    del inside, main, side
    st.release()
    assert st.arena is None


def test_arena_parts_lie_in_three_regions():
    from paper_2505_23254_amd import binding as ma
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 250 * GIB:
        pytest.skip("needs a nearly empty device: the third region is reached only through the first two")
    a = ma.Arena(8 * GIB, 4 * GIB, 2 * GIB, max_transient_bytes=int(free) - 4 * GIB)
    rep = a.report
    assert rep["regions_seen"] >= 3, rep
    assert (rep["first_blocks_in_place"], rep["second_blocks_in_place"], rep["side_blocks_in_place"]) == (4, 4, 2), rep

    def rate(x, y):
        ma.probe_two_writes(x, y)
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ma.probe_two_writes(x, y)
            e1.record()
            e1.synchronize()
            best = max(best, 2 * x.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        return best

    m, s = a.main, a.side
    first = (m[0:2 * GIB], m[2 * GIB:4 * GIB])
    second = (m[4 * GIB:6 * GIB], m[6 * GIB:8 * GIB])
    same = [rate(*first), rate(*second)]
    cross = [rate(first[0], second[0]), rate(first[1], s), rate(second[1], s)]
    print("two write streams, GB/s: same region", [round(x) for x in same], "different regions", [round(x) for x in cross])
    assert min(cross) >= 1.08 * max(same)
    del m, s, first, second
    a.close()
    assert torch.cuda.mem_get_info()[0] >= free - GIB
    # max_transient_bytes = 0: not one block beyond the arena's own; the parts take whatever regions
    # come first, the report says which blocks are in place, and the timing never contradicts it
    from paper_2505_23254_amd import hbm
    st = hbm.StitchedArena(ma.Arena, half_bytes=6 * GIB, side_bytes=2 * GIB, max_transient_bytes=0)
    assert st.report["blocks_created"] == 14
    check = st.verify_regions(ma.probe_two_writes)
    print("tight arena:", st.report, check)
    assert check["verified"] or not st.in_place
    st.release()
