"""Host-side model of the rows the MFMA decode kernel asks memory for, over capacities, windows,
lengths and the launch plans the library chooses: every row index must lie inside the cache.
(With a window the ranges start at the 32-aligned base of the window, which is known only on the
device; the last ranges can then start at or beyond the capacity, and the kernel's fixed dummy
address for tiles it does not need has to be clamped like every other row.)  No GPU needed."""
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1911_02150_amd", "libmqa_decode.so")
pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="library not built (run __graft_entry__.build())")

NW = 4          # waves per workgroup; wave w owns the 32-position tiles w, w+NW, ... of its range


def rows_requested(cap, window, L, S, chunk):
    """Every cache row index the kernel forms for one sequence: (row, is_dummy) pairs."""
    L = min(max(L, 0), cap)
    lo = max(0, L - window) if window > 0 else 0
    base = (lo & ~31) if window > 0 else 0
    rmax = cap - 1
    out = []
    for srange in range(S):
        begin = srange * chunk + base
        end = min(begin + chunk, L)
        ntiles = (end - begin + 31) // 32 if end > begin else 0
        for wave in range(NW):
            # the first tile is requested before the length check
            tiles = [(wave, begin + 32 * wave <= rmax)]
            # later tiles: tile t + NW is requested while tile t is processed
            t = wave
            while t < ntiles:
                tiles.append((t + NW, t + NW < ntiles))
                t += NW
            for t, real in tiles:
                p0 = begin + 32 * t
                if real:
                    out += [(min(p0 + r, rmax), False) for r in range(32)]
                else:
                    out.append((min(begin, rmax), True))
    return out, base


@pytest.mark.parametrize("b,h,cap,window", [
    (1, 8, 4096, 1024),      # ranges of 128: the ninth starts at the capacity when the sequence is full
    (2, 32, 3000, 1024), (2, 32, 3000, 1500), (1, 8, 301, 32), (1, 8, 4096, 4096), (1, 32, 8192, 2048),
    (3, 16, 1024, 992), (1, 8, 160, 64), (64, 32, 8192, 32), (1, 64, 40000, 4000),
])
def test_every_requested_row_is_inside_the_cache(b, h, cap, window):
    import paper_1911_02150_amd as m
    S, chunk, _ = m.mqa_decode_plan(b, h, cap, 128, 128, m.MQA_BF16, window=window)
    assert chunk % 32 == 0 and S >= 1
    beyond = False
    lengths = sorted({0, 1, 31, 32, 33, cap // 2, cap - 33, cap - 32, cap - 1, cap, max(0, min(cap, window)),
                      max(0, min(cap, window + 31))} & set(range(cap + 1)))
    for L in lengths:
        rows, base = rows_requested(cap, window, L, S, chunk)
        assert all(0 <= r < cap for r, _ in rows), (cap, window, L, S, chunk)
        beyond = beyond or any(s * chunk + base >= cap for s in range(S))
        # the ranges cover the whole window
        lo = max(0, L - window)
        assert base <= lo and base + S * chunk >= L, (cap, window, L, S, chunk, base)
    if (b, h, cap, window) == (1, 8, 4096, 1024):
        assert S > 1 and beyond, "this case is meant to have a range that starts at the capacity"
