"""Host-only checks of the split-L schedule (integer work, bit-exact): the tile walk the kernels
run, reported by vista_summarize_schedule, against a brute-force statement of the same schedule."""
import numpy as np
import pytest

from paper_2510_22049_amd import binding as V
from paper_2510_22049_amd import inputs as I


def desc(B, N, seg=0, S=256, d=128, H=4):
    return V.summarize_desc(B, S, d, H, V.VISTA_BF16, N, segment_items=seg)


def brute_force_tiles(off, seg):
    """Segments of `seg` flat rows, cut at user boundaries, each piece cut into tiles of 32."""
    N, B = int(off[-1]), len(off) - 1
    owner = np.repeat(np.arange(B), np.diff(off))          # user of every flat row
    tiles = []
    for g in range((N + seg - 1) // seg):
        lo, hi = g * seg, min((g + 1) * seg, N)
        r = lo
        while r < hi:
            u = owner[r]
            piece_end = min(int(off[u + 1]), hi)
            t = r
            while t < piece_end:
                n = min(32, piece_end - t)
                tiles.append((g, u, t, n))
                t += n
            r = piece_end
    return np.array(tiles, dtype=np.int64).reshape(-1, 4)


@pytest.mark.parametrize("lens,seg", [
    ([700, 0, 1, 31, 32, 33, 2100, 64, 0, 95, 1029], 64),
    ([700, 0, 1, 31, 32, 33, 2100, 64, 0, 95, 1029], 992),
    ([700, 0, 1, 31, 32, 33, 2100, 64, 0, 95, 1029], 0),
    ([0, 0, 5], 32),
    ([1], 0),
    ([0, 0, 0], 0),
    ([40000, 3, 0, 0, 977, 12345], 4096),
])
def test_schedule_is_the_brute_force_tiling(lens, seg):
    off = I.offsets_from_lengths(lens)
    d_ = desc(len(lens), int(off[-1]), seg)
    got = V.vista_summarize_schedule(d_, off)
    want = brute_force_tiles(off, V.vista_summarize_segment_items(d_))
    assert np.array_equal(got, want)
    covered = np.zeros(int(off[-1]), dtype=np.int32)        # every row exactly once, under its own user
    for g, u, r, n in got:
        covered[r:r + n] += 1
        assert off[u] <= r and r + n <= off[u + 1]
    assert np.all(covered == 1)


def test_schedule_of_the_jagged_workload():
    c = I.CONFIGS[2]
    off = I.offsets_from_lengths(I.lengths(c))
    d_ = desc(c.B, int(off[-1]))
    got = V.vista_summarize_schedule(d_, off)
    assert np.array_equal(got, brute_force_tiles(off, V.vista_summarize_segment_items(d_)))
    assert got[:, 3].sum() == off[-1]


@pytest.mark.parametrize("seed", range(6))
def test_schedule_stays_in_bounds_for_any_offsets(seed):
    """Offsets that are decreasing, all zero, negative or beyond N: what the kernels walk is
    wrong but every tile stays inside [0, N) and every user index inside [0, B)."""
    g = np.random.default_rng(seed)
    B, N = 9, 5000
    kinds = [
        g.integers(-3 * N, 3 * N, size=B + 1),
        np.zeros(B + 1, dtype=np.int64),
        np.full(B + 1, 10 * N),
        np.sort(g.integers(0, N, size=B + 1))[::-1].copy(),
        np.concatenate([[0], np.sort(g.integers(0, 2 * N, size=B))]),
        np.concatenate([[7], g.integers(0, N, size=B - 1), [N]]),
    ]
    for off in kinds:
        for seg in (32, 256, 4096):
            t = V.vista_summarize_schedule(desc(B, N, seg), off.astype(np.int64))
            if len(t) == 0:
                continue
            assert t[:, 1].min() >= 0 and t[:, 1].max() < B
            assert t[:, 2].min() >= 0 and (t[:, 2] + t[:, 3]).max() <= N
            assert t[:, 3].min() >= 1 and t[:, 3].max() <= 32
            assert np.all(t[:, 2] >= t[:, 0] * seg) and np.all(t[:, 2] + t[:, 3] <= (t[:, 0] + 1) * seg)
            assert len(t) <= N + B * ((N + seg - 1) // seg)      # the walk ends


def test_schedule_rejects_bad_arguments():
    import ctypes as C
    L = V.lib()
    d_ = desc(2, 100)
    assert L.vista_summarize_schedule(C.byref(d_), None, None, 0) == -1
    off = np.array([0, 50, 100], dtype=np.int64)
    ptr = off.ctypes.data_as(C.POINTER(C.c_int64))
    assert L.vista_summarize_schedule(C.byref(d_), ptr, None, 5) == -1
    assert L.vista_summarize_schedule(C.byref(desc(0, 100)), ptr, None, 0) == -1
    assert L.vista_summarize_schedule(C.byref(d_), ptr, None, 0) == 4        # 50 rows = 2 tiles per user
