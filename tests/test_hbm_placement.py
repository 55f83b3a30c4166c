"""Placement arithmetic of hbm.DeviceArena (no GPU: the arena is a stand-in that only knows offsets)."""
from paper_2505_23254_amd import hbm, synth

GIB = 1 << 30


class _View:
    def __init__(self, lo, hi):
        self.lo, self.hi = lo, hi

    def numel(self):
        return self.hi - self.lo

    def data_ptr(self):
        return 0x7000_0000_0000 + self.lo

    def __getitem__(self, s):
        lo = self.lo + (s.start or 0)
        hi = self.hi if s.stop is None else self.lo + s.stop
        assert self.lo <= lo <= hi <= self.hi
        return _View(lo, hi)


class _Arena(hbm.DeviceArena):
    def __init__(self, gib):
        self.buf = _View(0, int(gib * GIB))


def _span(arena, v):
    lo = v.data_ptr() - arena.buf.data_ptr()
    return lo, lo + v.numel()


def _traffic_split(arena, main, traffic):
    """Share of the main window's traffic that lies below the first region boundary."""
    lo, _ = _span(arena, main)
    below = total = 0.0
    for nb, w in traffic:
        a, b = lo, lo + nb
        below += w * max(0, min(b, hbm.REGION_BYTES) - a)
        total += w * nb
        lo = b
    return below / total


def test_8b_list_goes_across_the_first_boundary_with_the_copy_in_the_third_region():
    shapes = synth.llama3_8b_shapes()
    arena = _Arena(283.6)
    parts, traffic = synth.list_state_parts(shapes), synth.list_traffic(shapes)[:4]
    main, side = arena.split_window(parts[0], traffic, parts[1])
    (a, b), (c, d) = _span(arena, main), _span(arena, side)
    assert a % hbm.ALIGN == 0 and c % hbm.ALIGN == 0
    assert a < hbm.REGION_BYTES < b < 2 * hbm.REGION_BYTES                    # two regions, not three
    assert abs(_traffic_split(arena, main, traffic) - 0.5) < 1e-3            # half of the traffic on each side
    assert 2 * hbm.REGION_BYTES <= c and d <= arena.nbytes                    # the copy: third region only
    assert d - c == parts[1] and b - a == parts[0]


def test_14b_class_state_still_leaves_the_third_region_to_the_copy():
    total = sum(n for _, n in synth.qwen14b_class_shapes())
    arena = _Arena(283.6)
    parts, traffic = synth.flat_state_parts(total), synth.flat_traffic(total)[:4]
    main, side = arena.split_window(parts[0], traffic, parts[1])
    (a, b), (c, d) = _span(arena, main), _span(arena, side)
    assert 0 <= a and b <= 2 * hbm.REGION_BYTES and c >= 2 * hbm.REGION_BYTES and d <= arena.nbytes
    assert abs(_traffic_split(arena, main, traffic) - 0.5) < 1e-3


def test_small_states_and_small_arenas():
    arena = _Arena(283.6)
    n = 10 ** 8
    parts, traffic = synth.flat_state_parts(n), synth.flat_traffic(n)[:4]
    main, side = arena.split_window(parts[0], traffic, parts[1])
    assert _span(arena, main)[0] < hbm.REGION_BYTES < _span(arena, main)[1]
    assert _span(arena, side)[0] >= 2 * hbm.REGION_BYTES or _span(arena, side)[1] <= hbm.REGION_BYTES
    # an arena that ends inside the second region: no region is free of the main window, so the copy
    # follows the main part in one contiguous window
    small = _Arena(150)
    shapes = synth.llama3_8b_shapes()
    parts, traffic = synth.list_state_parts(shapes), synth.list_traffic(shapes)[:4]
    main, side = small.split_window(parts[0], traffic, parts[1])
    (a, b), (c, d) = _span(small, main), _span(small, side)
    assert 0 <= a and b <= c and d <= small.nbytes and c - b < 2 * hbm.ALIGN


def test_stitched_arena_windows_straddle_its_internal_boundary():
    """StitchedArena asks the allocator once, for two halves and a side part, and cuts every state so
    that half of its traffic lies on each side of the boundary between the halves."""
    made, closed = [], []

    class _Made:
        def __init__(self, main_bytes, first, side_bytes, block, limit):
            made.append((main_bytes, first, side_bytes, block, limit))
            self.report = {"main_bytes": main_bytes, "side_bytes": side_bytes, "first_region_bytes": first,
                           "blocks_created": 213, "first_blocks_in_place": first // GIB,
                           "second_blocks_in_place": (main_bytes - first) // GIB,
                           "side_blocks_in_place": side_bytes // GIB, "regions_seen": 3}
            self.main, self.side = _View(0, main_bytes), _View(1 << 40, (1 << 40) + side_bytes)

        def close(self):
            closed.append(self)

    st = hbm.StitchedArena(_Made, max_transient_bytes=250 * GIB)
    assert made == [(168 * GIB, 84 * GIB, 24 * GIB, 0, 250 * GIB)]
    assert st.in_place and st.half == 84 * GIB
    assert abs(st.settle_seconds - (213 - 192) * GIB / hbm.StitchedArena.WIPE_BYTES_PER_S) < 1e-9
    shapes = synth.llama3_8b_shapes()
    parts, traffic = synth.list_state_parts(shapes), synth.list_traffic(shapes)
    main, side = st.split_window(parts[0], traffic[:4], parts[1])
    assert main.numel() == parts[0] and side.numel() == parts[1] and len(made) == 1
    lo = main.data_ptr() - st.arena.main.data_ptr()
    below = total = 0.0
    off = lo
    for nb, w in traffic[:4]:
        below += w * max(0, min(off + nb, st.half) - off)
        total += w * nb
        off += nb
    assert abs(below / total - 0.5) < 1e-3
    w = st.window(10 * GIB, None)                       # uniform traffic: centred on the boundary
    assert w.data_ptr() - st.arena.main.data_ptr() == 79 * GIB and len(made) == 1
    big = st.window(160 * GIB, [(150 * GIB, 2.0), (10 * GIB, 1.0)])      # clamped into the range
    assert big.data_ptr() - st.arena.main.data_ptr() + 160 * GIB <= 168 * GIB
    import pytest
    with pytest.raises(ValueError):
        st.window(169 * GIB)
    with pytest.raises(ValueError):
        st.split_window(GIB, None, 25 * GIB)
    st.report["side_blocks_in_place"] = 3               # a part that did not get its region is reported
    assert not st.in_place
    st.release()
    assert len(closed) == 1 and st.arena is None
    st.release()                                        # idempotent
    assert len(closed) == 1
