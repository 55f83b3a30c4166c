"""The measurement aids run, move what they say they move, and leave everything else alone."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_probes_touch_whole_work_items_only():
    from paper_2505_23254_amd import binding as ma, hbm
    n = 3 * 4096 + 123                                     # three work items and a rest the probe must leave alone
    a, b, c = (torch.full((n,), 2.0, dtype=torch.float32, device="cuda") for _ in range(3))
    d = torch.full((n,), 1.0, dtype=torch.bfloat16, device="cuda")
    e = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    ma.probe_update_mix(a, b, c, d, e)
    torch.cuda.synchronize()
    body = 3 * 4096
    assert torch.all(a[:body] == 3.0) and torch.all(a[body:] == 2.0)          # a + d inside, untouched outside
    assert torch.all(e[:body].float() == 2.0) and torch.all(e[body:] == 0)    # upper halves of the old a
    h = [torch.full((2 * 8192 + 77,), 1.0, dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    keep = [t.clone() for t in h]
    ma.probe_update_mix(*h)                                # states held in 16 bits: a, b, c rewritten, d only read
    torch.cuda.synchronize()
    assert torch.equal(h[3], keep[3])
    assert all(torch.equal(t[2 * 8192:], k[2 * 8192:]) for t, k in zip(h, keep))
    assert not torch.equal(h[0][:2 * 8192], keep[0][:2 * 8192])
    x = torch.zeros(3 * 32768 + 64, dtype=torch.uint8, device="cuda")
    y = torch.zeros_like(x)
    ma.probe_two_writes(x, y)
    torch.cuda.synchronize()
    assert x[:3 * 32768].view(torch.float32)[0].item() == 1.0 and int(x[3 * 32768:].sum()) == 0
    assert torch.equal(x, y)
    # an arena too small to reach a second region cannot be verified, and says so
    class Small(hbm.DeviceArena):
        def __init__(self):
            self.buf = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    assert Small().verify_regions(ma.probe_two_writes)["verified"] is False
