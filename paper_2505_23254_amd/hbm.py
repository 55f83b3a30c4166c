"""Where optimizer state lies in the 288 GiB of HBM of one MI355X.

Measured on MI355X (two-stream write and mixed read/write probes over a whole-device allocation):

* the HBM behaves as three regions of 96 GiB each.  Streams that lie in ONE region share a lower
  ceiling (two write streams: ~5.7 TB/s inside a region, ~7.1 TB/s across two regions; the 1:1
  read/write mix of the update kernel: ~5.3 TB/s inside one region);
* one allocation that takes (nearly) all free device memory maps linearly onto the regions (byte
  offset x of the allocation lies in region x // 96 GiB), but only on a device whose physical memory
  has not been handed out and taken back in pieces: after a process has created and released
  virtual-memory blocks, later whole-device allocations (of other processes too) no longer do;
* the update kernel is fastest when the traffic of the buffers it updates in place (p, m, v, read
  and written) splits evenly over two regions (measured on the 8B-shaped state: 6.4 TB/s with the
  state straddling a region boundary half and half, 5.85-6.0 TB/s with 80 % of it inside one region;
  three-way splits of p, m, v were not better than the even two-way split);
* a WRITE-ONLY stream (the 16-bit parameter copy) is best kept out of those two regions: with the copy
  in the third region the same kernel reaches 6.47 TB/s (34.75 instead of 35.15 ms on the 8B-shaped
  list; insensitive to shifts of +-4 GiB, to where in the third region the copy lies, and to whether
  the gradient lies before p or behind v).  A read-only stream there makes things worse (gradient in
  the third region: 6.26-6.35 TB/s).  A probe with separate output buffers says the same: what the
  memory system rewards is write traffic spread over more regions than the reads.

Hence two ways to place a state.  StitchedArena (the one bench.py uses) asks the library's
ma_arena_create for a range built from 1-GiB physical blocks whose region the library finds by
timing: it works whatever happened on the device before, and holds only what was asked for.
DeviceArena takes the device's free memory as one allocation and hands out the window whose traffic
midpoint sits on a region boundary; it needs the linear map, which verify_regions() checks.  Only
placement lives here; nothing of the optimizer step.
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

    def split_window(self, main_bytes: int, main_traffic, side_bytes: int):
        """Two views: `main_bytes` placed as window() places them (the buffers updated in place and the
        read-only ones), and `side_bytes` for write-only buffers in the region that `main` uses least
        (the third one, when main straddles the first boundary).  Falls back to one contiguous window
        (side right behind main) when no such room exists."""
        main = self.window(main_bytes, main_traffic)
        lo = main.data_ptr() - self.buf.data_ptr()
        hi = lo + main_bytes
        best = None
        for r in range(3):
            r0, r1 = r * REGION_BYTES, min((r + 1) * REGION_BYTES, self.nbytes)
            if r1 - r0 <= 0:
                continue
            covered = max(0, min(hi, r1) - max(lo, r0))
            # the largest free stretch of region r: before or behind main's part of it
            free = [(r0, max(r0, min(lo, r1))), (min(max(hi, r0), r1), r1)]
            a, b = max(free, key=lambda ab: ab[1] - ab[0])
            a = (a + ALIGN - 1) // ALIGN * ALIGN
            if b - a >= side_bytes and (best is None or covered < best[0]):
                # a little into the stretch, away from the region's edge, when there is room
                start = a + min(8 * GIB, (b - a - side_bytes) // 2) // ALIGN * ALIGN
                best = (covered, start)
        if best is None or best[0] > 0:
            whole = self.window(main_bytes + ALIGN + side_bytes,
                                list(main_traffic or [(main_bytes, 1.0)]) + [(ALIGN + side_bytes, 1.0)])
            off = (main_bytes + ALIGN - 1) // ALIGN * ALIGN
            return whole[:main_bytes], whole[off:off + side_bytes]
        return main, self.buf[best[1]:best[1] + side_bytes]

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
            return _pair_rate(two_writes, x, y, reps)

        s, c = [rate(p) for p in same], [rate(p) for p in cross]
        return {"verified": bool(min(c) >= margin * max(s)), "same_GBps": [round(x) for x in s],
                "cross_GBps": [round(x) for x in c], "pairs_GiB": {"same": same, "cross": cross}}

    placement = "region"

    def release(self):
        self.buf = None

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


class StitchedArena:
    """The placement of DeviceArena without holding the device: ONE address range of `2 * half_bytes`
    (+ `side_bytes`) built by the library's ma_arena_create (`make_arena` = the binding's Arena) out of
    1-GiB physical blocks whose HBM region it finds by timing: the first half from one region, the
    second half from another, the side part (for write-only buffers) from a third.  window() and
    split_window() then cut a state out of it so that its traffic midpoint lies on the boundary
    between the two halves.  While it searches, the library holds at most `max_transient_bytes`
    (default: all free memory but `reserve_gib`) for a fraction of a second; the blocks it does not
    use go back to the driver, which wipes them in the background (measured: ~26 GB/s, during which
    every kernel runs ~0.5 % slower); `settle_seconds` is how long that takes."""

    placement = "stitched"
    WIPE_BYTES_PER_S = 20e9          # a cautious figure for the driver's background wipe

    def __init__(self, make_arena, half_bytes: int = 84 * GIB, side_bytes: int = 24 * GIB,
                 max_transient_bytes: Optional[int] = None, reserve_gib: float = 3.0, block_bytes: int = 0):
        limit = max_transient_bytes
        if limit is None:
            free, _ = torch.cuda.mem_get_info()
            limit = max(0, int(free - reserve_gib * GIB))
        self.arena = make_arena(2 * half_bytes, half_bytes, side_bytes, block_bytes, limit)
        self.report = dict(self.arena.report)
        self.half = int(self.report["first_region_bytes"])          # whole blocks
        self.block = block_bytes or GIB
        released = int(self.report["blocks_created"]) * self.block - int(self.report["main_bytes"]) - int(self.report["side_bytes"])
        self.settle_seconds = max(0.0, released / self.WIPE_BYTES_PER_S)

    @property
    def in_place(self) -> bool:
        """True when every block lies in the region it was wanted in."""
        r, blk = self.report, self.block
        return bool(r["first_blocks_in_place"] * blk == r["first_region_bytes"]
                    and r["second_blocks_in_place"] * blk == r["main_bytes"] - r["first_region_bytes"]
                    and r["side_blocks_in_place"] * blk == r["side_bytes"])

    def window(self, nbytes: int, traffic=None) -> torch.Tensor:
        """A uint8 view of `nbytes` bytes with half of its traffic in each of the two main regions."""
        cap = self.arena.main.numel()
        if nbytes > cap:
            raise ValueError("state of %d bytes does not fit the stitched arena of %d" % (nbytes, cap))
        start = self.half - DeviceArena._midpoint(nbytes, traffic)
        start = max(0, min(start, cap - nbytes)) // ALIGN * ALIGN
        return self.arena.main[start:start + nbytes]

    def split_window(self, main_bytes: int, main_traffic, side_bytes: int):
        """window() for the buffers updated in place and the read-only ones, plus `side_bytes` for
        write-only buffers in the third region."""
        side = self.arena.side
        if side is None or side_bytes > side.numel():
            raise ValueError("side part of %d bytes does not fit the stitched arena" % side_bytes)
        return self.window(main_bytes, main_traffic), side[:side_bytes]

    def verify_regions(self, two_writes, gib_each: int = 2, reps: int = 3, margin: float = 1.08) -> dict:
        """An independent check of the finished range, by timing (see DeviceArena.verify_regions):
        two windows inside one part must be slower together than windows of two different parts.
        Overwrites the windows; run it before the arena holds data."""
        nb = gib_each * GIB
        main, side, half, cap = self.arena.main, self.arena.side, self.half, self.arena.main.numel()
        if half < 3 * nb or cap - half < 3 * nb:
            return {"verified": False, "same_GBps": [], "cross_GBps": [], "note": "arena too small to probe"}
        first = (main[0:nb], main[half - nb:half])
        second = (main[half:half + nb], main[cap - nb:cap])
        same, cross = [first, second], [(first[0], second[0]), (first[1], second[1])]
        if side is not None and side.numel() >= nb:
            cross += [(first[0], side[:nb]), (second[1], side[side.numel() - nb:])]
        s = [_pair_rate(two_writes, x, y, reps) for x, y in same]
        c = [_pair_rate(two_writes, x, y, reps) for x, y in cross]
        return {"verified": bool(min(c) >= margin * max(s)), "same_GBps": [round(x) for x in s],
                "cross_GBps": [round(x) for x in c]}

    def release(self):
        if self.arena is not None:
            self.arena.close()
            self.arena = None


def _pair_rate(two_writes, x, y, reps: int) -> float:
    """GB/s of two write streams over the uint8 views x and y (best of `reps` after a warm-up)."""
    two_writes(x, y)
    best = 0.0
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        two_writes(x, y)
        b.record()
        b.synchronize()
        best = max(best, 2 * x.numel() / (a.elapsed_time(b) * 1e-3) / 1e9)
    return best
