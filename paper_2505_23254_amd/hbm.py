"""Where optimizer state lies in the 288 GiB of HBM of one MI355X.

Measured on MI355X (two-stream write and mixed read/write probes over a whole-device allocation):

* the HBM behaves as three regions of 96 GiB each.  Streams that lie in ONE region share a lower
  ceiling (two write streams: ~5.7 TB/s inside a region, ~7.1 TB/s across two regions; the 1:1
  read/write mix of the update kernel: ~5.3 TB/s inside one region);
* one allocation that takes (nearly) all free device memory maps linearly onto the regions: byte
  offset x of the allocation lies in region x // 96 GiB;
* the update kernel is fastest when its traffic splits evenly over two regions (measured on the
  8B-shaped state: 6.4 TB/s with the state straddling a region boundary half and half, 5.85-6.0
  TB/s with 80 % of it inside one region; three-way splits were not better than the even two-way
  split).

Hence this helper: take the device's free memory as one arena and hand out, for a state of a given
size, the window of the arena whose traffic midpoint sits on a region boundary.  Only placement
lives here; nothing of the optimizer step.
"""
from typing import Optional, Sequence, Tuple

import torch

GIB = 1 << 30
REGION_BYTES = 96 * GIB
ALIGN = 2 << 20


class DeviceArena:
    """All free memory of one device as a single allocation (minus `reserve_gib` left to others)."""

    def __init__(self, device="cuda", reserve_gib: float = 3.0):
        dev = torch.device(device)
        free, _ = torch.cuda.mem_get_info(dev)
        nbytes = (int(free - reserve_gib * GIB) // ALIGN) * ALIGN
        if nbytes <= 0:
            raise RuntimeError("no free device memory for an arena")
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    @property
    def nbytes(self) -> int:
        return self.buf.numel()

    def window(self, nbytes: int,
               traffic: Optional[Sequence[Tuple[int, float]]] = None) -> torch.Tensor:
        """A uint8 view of `nbytes` bytes placed so that half of the traffic falls on each side of a
        region boundary.  `traffic`: (bytes, weight) of the state's pieces in address order, weight =
        bytes moved per byte stored (2 for a buffer read and written, 1 for read-only or write-only);
        None = uniform.  A state larger than two regions is centred on the middle region instead."""
        if nbytes > self.nbytes:
            raise ValueError("state of %d bytes does not fit the arena of %d" % (nbytes, self.nbytes))
        if nbytes > 2 * REGION_BYTES:
            start = REGION_BYTES + REGION_BYTES // 2 - nbytes // 2
        else:
            start = REGION_BYTES - self._midpoint(nbytes, traffic)
        start = max(0, min(start, self.nbytes - nbytes))
        start = start // ALIGN * ALIGN
        return self.buf[start:start + nbytes]

    def verify_regions(self, two_writes, gib_each: int = 2, reps: int = 3, margin: float = 1.08) -> dict:
        """Checks, by timing, that byte offset x of this allocation lies in region x // 96 GiB.

        `two_writes(x, y)` enqueues a kernel that writes the two uint8 views once (the library's
        ma_probe_two_writes).  Pairs of windows that the linear map puts into ONE region must be slower
        than pairs it puts into two different regions, by at least `margin`.  Run it before the arena
        holds data: the windows are overwritten.  Returns {"verified", "same_GBps", "cross_GBps"}."""
        nb = gib_each * GIB
        last = (self.nbytes - nb) // GIB                 # last whole-GiB offset a window can start at
        inside = lambda r: [o for o in (96 * r + 8, 96 * r + 56) if o + gib_each <= 96 * (r + 1) and o <= last]
        offs = [inside(r) for r in range(3)]
        same = [tuple(o) for o in offs if len(o) == 2]
        cross = [(offs[r][0], offs[r + 1][0]) for r in range(2) if offs[r] and offs[r + 1]]
        cross += [(offs[r][1], offs[r + 1][1]) for r in range(2) if len(offs[r]) == 2 and len(offs[r + 1]) == 2]
        if not same or not cross:
            return {"verified": False, "same_GBps": [], "cross_GBps": [], "note": "arena too small to probe"}

        def rate(pair):
            x, y = (self.buf[o * GIB:o * GIB + nb] for o in pair)
            two_writes(x, y)
            best = 0.0
            for _ in range(reps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                two_writes(x, y)
                b.record()
                b.synchronize()
                best = max(best, 2 * nb / (a.elapsed_time(b) * 1e-3) / 1e9)
            return best

        s, c = [rate(p) for p in same], [rate(p) for p in cross]
        return {"verified": bool(min(c) >= margin * max(s)), "same_GBps": [round(x) for x in s],
                "cross_GBps": [round(x) for x in c], "pairs_GiB": {"same": same, "cross": cross}}

    @staticmethod
    def _midpoint(nbytes: int, traffic) -> int:
        if not traffic:
            return nbytes // 2
        total = sum(b * w for b, w in traffic)
        acc, off = 0.0, 0
        for b, w in traffic:
            if b * w > 0 and acc + b * w >= total / 2:
                return off + int((total / 2 - acc) / w)
            acc += b * w
            off += b
        return nbytes // 2
