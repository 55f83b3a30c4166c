"""Do the oracle's pins notice a mistake?  Each entry below plants one plausible mistake (a dropped
term, a wrong sign or index, a swapped operand, a misplaced epsilon, a wrong tie rule ...) in a COPY
of the oracle's source, builds it, and runs the pin tests against that build in a child process:
the pins must fail.  An unmodified copy must pass, which shows that the failures come from the
planted mistakes and not from the mechanism.  Nothing here touches the GPU library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_TESTS = ["tests/test_oracle_adamw.py", "tests/test_oracle_casts.py", "tests/test_oracle_norm.py",
             "tests/test_oracle_next.py"]

MUTANTS = [
    ("decay dropped", "const float q = std::fmaf(-s.decay, p, p);", "const float q = p;"),
    ("eps inside the square root", "const float d = std::fmaf(std::sqrt(v1), s.inv_sqrt_bc2, s.eps);",
     "const float d = std::sqrt(v1 + s.eps) * s.inv_sqrt_bc2;"),
    ("eps added before the bias correction", "const float d = std::fmaf(std::sqrt(v1), s.inv_sqrt_bc2, s.eps);",
     "const float d = (std::sqrt(v1) + s.eps) * s.inv_sqrt_bc2;"),
    ("first correction from beta2",
     "bc1 = 1.0 - std::pow(b1, static_cast<double>(step));", "bc1 = 1.0 - std::pow(b2, static_cast<double>(step));"),
    ("no first bias correction", "s.step_size = static_cast<float>(lr / bc1);", "s.step_size = static_cast<float>(lr);"),
    ("second correction without the root", "s.inv_sqrt_bc2 = static_cast<float>(1.0 / std::sqrt(bc2));",
     "s.inv_sqrt_bc2 = static_cast<float>(1.0 / bc2);"),
    ("decay not scaled by lr", "s.decay = static_cast<float>(lr * wd);", "s.decay = static_cast<float>(wd);"),
    ("unscale multiplies", "static_cast<double>(clip_coef) / static_cast<double>(loss_scale));",
     "static_cast<double>(clip_coef) * static_cast<double>(loss_scale));"),
    ("ties round up", "} else if (frac == 0.5) {\n    if (std::fmod(r, 2.0) != 0.0) r += 1.0;",
     "} else if (frac == 0.5) {\n    r += 1.0;"),
    ("fp16 exponent off by one", "mag = std::ldexp(static_cast<float>(1024 + f), e - 25);",
     "mag = std::ldexp(static_cast<float>(1024 + f), e - 24);"),
    ("sum of values, not squares", "acc += y * y;", "acc += y;"),
    ("NaN not flagged", "if (std::isinf(x) || std::isnan(x)) ov = 1;", "if (std::isinf(x)) ov = 1;"),
    ("1 - beta1 dropped", "const float m1 = std::fmaf(s.beta1, m, s.omb1 * g);",
     "const float m1 = std::fmaf(s.beta1, m, g);"),
    ("second moment from g, not g squared", "const float v1 = std::fmaf(s.beta2, v, s.omb2 * (g * g));",
     "const float v1 = std::fmaf(s.beta2, v, s.omb2 * g);"),
    ("norm multiplies by the scale", "const double y = static_cast<double>(x) / scale;",
     "const double y = static_cast<double>(x) * scale;"),
    ("overflow does not skip", "  if (ov) {\n    if (clip_out) *clip_out = 0.0f;\n    return 1;\n  }",
     "  if (ov) {\n    if (clip_out) *clip_out = 0.0f;\n  }"),
    ("copy taken from the old parameter",
     "    adamw_element(s, widen(g, gdt, i), p[i], m[i], v[i]);\n    store_lp(p_lp, pdt, i, p[i]);",
     "    store_lp(p_lp, pdt, i, p[i]);\n    adamw_element(s, widen(g, gdt, i), p[i], m[i], v[i]);"),
    ("subnormal threshold off by one", "if (E < EMIN) E = EMIN;", "if (E < EMIN - 1) E = EMIN - 1;"),
    ("beta2 in the first moment", "const float m1 = std::fmaf(s.beta1, m, s.omb1 * g);",
     "const float m1 = std::fmaf(s.beta2, m, s.omb1 * g);"),
    ("update with the wrong sign", "const float p1 = std::fmaf(-s.step_size, u, q);",
     "const float p1 = std::fmaf(s.step_size, u, q);"),
    ("clip takes the maximum", "return static_cast<float>(c < 1.0 ? c : 1.0);",
     "return static_cast<float>(c > 1.0 ? c : 1.0);"),
    ("first micro-batch adds", "acc[i] = first ? g : acc[i] + g;", "acc[i] = acc[i] + g;"),
    ("accumulation subtracts", "acc[i] = first ? g : acc[i] + g;", "acc[i] = first ? g : acc[i] - g;"),
    ("truncation rounds", "uint16_t h = static_cast<uint16_t>(b >> 16);\n  if (std::isnan(x)) h |= 0x0040;",
     "uint16_t h = static_cast<uint16_t>((b + 0x8000u) >> 16);\n  if (std::isnan(x)) h |= 0x0040;"),
    ("truncation loses a NaN", "  if (std::isnan(x)) h |= 0x0040;\n  return h;", "  return h;"),
    ("bf16 second moment stored from the first", "v[i] = ora_truncate_bf16_one(vf);",
     "v[i] = ora_truncate_bf16_one(mf);"),
    ("scale grows one step late", "if (st.good_steps >= cfg.window) {", "if (st.good_steps > cfg.window) {"),
    ("skipped iteration counted as an update", "    st.good_steps = 0;\n    st.skipped += 1;",
     "    st.good_steps = 0;\n    st.step += 1;\n    st.skipped += 1;"),
    ("scale without a floor", "st.scale = s < cfg.min_scale ? cfg.min_scale : s;", "st.scale = s;"),
    ("clean-step count survives an overflow", "    st.good_steps = 0;\n    st.skipped += 1;", "    st.skipped += 1;"),
    ("update number not advanced", "hyper, st.step + 1, st.scale,", "hyper, st.step, st.scale,"),
]


def _build_and_run(workdir, name, source):
    tag = "".join(ch if ch.isalnum() else "_" for ch in name)
    src = os.path.join(workdir, tag + ".cpp")
    lib = os.path.join(workdir, tag + ".so")
    with open(src, "w") as f:
        f.write(source)
    subprocess.run(["g++", *oracle_build.FLAGS, src, "-o", lib], check=True, capture_output=True)
    env = dict(os.environ, MA_ORACLE_LIBRARY=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", *PIN_TESTS, "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    return name, r.returncode, r.stdout[-600:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    original = open(oracle_build.SRC).read()
    jobs = [("unmodified", original)]
    for name, find, replace in MUTANTS:
        assert original.count(find) >= 1, "the oracle no longer contains the text of mutant '%s'" % name
        jobs.append((name, original.replace(find, replace)))
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(lambda j: _build_and_run(str(tmp_path), *j), jobs))
    name, rc, tail = results[0]
    assert rc == 0, "the pins fail on an unmodified copy of the oracle:\n" + tail
    survivors = [name for name, rc, _ in results[1:] if rc == 0]
    broken = [(name, rc, tail) for name, rc, tail in results[1:] if rc not in (0, 1)]
    assert not broken, "pytest itself failed: %r" % (broken[:1],)
    assert not survivors, "planted mistakes that no pin noticed: %s" % survivors
