"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-side logic (argument checks that return before
any launch, key-tile box, token->tile window conversion, work model) agrees
with the oracle and the paper's counts.  No compute call is made here."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import paper_2502_04507_amd as sta
from oracle import sta_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
I3 = ctypes.c_int * 3


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sta.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sta_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = sta.load_library()
    names = _declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(sta.EXPORTED_SYMBOLS) == names
    assert sta.sta_version() >= 100


def test_strerror_covers_all_codes():
    msgs = {sta.sta_strerror(i) for i in range(8)}
    assert len(msgs) == 8 and "unknown status" not in msgs
    assert sta.sta_strerror(99) == "unknown status"


def test_host_key_tile_box_matches_oracle_lists():
    """Bit-exact: host box (ascending row-major enumeration) == oracle's collapsed token predicate."""
    cases = [((30, 48, 80), (6, 8, 8), (3, 3, 3)), ((30, 48, 80), (6, 8, 8), (5, 3, 5)),
             ((12, 48, 48), (6, 8, 8), (1, 3, 3)), ((1, 64, 64), (1, 8, 8), (1, 3, 3)),
             ((8, 8, 12), (2, 2, 2), (2, 4, 7)), ((4, 6, 6), (2, 2, 2), (9, 1, 2)),
             ((30, 48, 80), (6, 8, 8), (5, 6, 10))]
    for grid, tile, wt in cases:
        tg = [g // t for g, t in zip(grid, tile)]
        counts, lists = orc.key_tiles(grid, tile, orc.window_tiles_to_tokens(wt, tile))
        for qt, qc in enumerate(itertools.product(*[range(n) for n in tg])):
            lo, hi = sta.sta_key_tile_box(tg, wt, qc)
            ids = [int(np.ravel_multi_index(c, tg))
                   for c in itertools.product(*[range(lo[a], hi[a] + 1) for a in range(3)])]
            assert ids == lists[qt, :counts[qt]].tolist()


def test_window_tokens_to_tiles():
    assert sta.sta_window_tokens_to_tiles((18, 24, 24), (6, 8, 8)) == (3, 3, 3)     # Sec. 4.3
    assert sta.sta_window_tokens_to_tiles((30, 40, 40), (6, 8, 8)) == (5, 5, 5)
    with pytest.raises(sta.StaError) as e:
        sta.sta_window_tokens_to_tiles((19, 25, 25), (6, 8, 8))
    assert e.value.status == 3
    with pytest.raises(sta.StaError):
        sta.sta_window_tokens_to_tiles((0, 8, 8), (6, 8, 8))


def test_kept_flops_model_matches_paper_scaling():
    """Work is 4*P^2*D per kept pair; kept fractions 27/300 and 125/300 (Table 2 scales its
    work column by exactly these)."""
    grid, tile = (30, 48, 80), (6, 8, 8)
    dense = sta.sta_kept_flops(1, 24, 128, grid, tile, [(5, 6, 10)] * 24)
    assert dense == 4.0 * 115200 * 115200 * 128 * 24
    assert sta.sta_kept_flops(1, 24, 128, grid, tile, [(3, 3, 3)] * 24) == pytest.approx(dense * 27 / 300, rel=1e-12)
    assert sta.sta_kept_flops(1, 24, 128, grid, tile, [(5, 5, 5)] * 24) == pytest.approx(dense * 125 / 300, rel=1e-12)
    assert sta.sta_kept_flops(2, 24, 128, grid, tile, [(5, 3, 5)] * 24) == pytest.approx(2 * dense * 75 / 300, rel=1e-12)


def test_error_returns_before_any_launch():
    lib = sta.load_library()
    grid, tile = I3(4, 4, 4), I3(2, 2, 2)
    win = (ctypes.c_int * 3)(1, 1, 1)
    fake = ctypes.c_void_p(0x10000)
    fake2 = ctypes.c_void_p(0x90000000)
    # NULL pointers
    assert lib.sta_tile_permute(None, fake, 0, 0, 1, 1, 64, grid, tile, None) == 1
    assert lib.sta_forward(None, fake, fake, fake, 1, 1, 64, grid, tile, win, 0.0, None, 0, None) == 1
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 1, 64, grid, tile, None, 0.0, None, 0, None) == 1
    # shape: grid not a multiple of tile, non-positive dims
    assert lib.sta_tile_permute(fake, fake2, 0, 0, 1, 1, 64, I3(5, 4, 4), tile, None) == 2
    assert lib.sta_untile(fake, fake2, 0, 0, 0, 1, 64, grid, tile, None) == 2
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 1, 64, I3(4, 4, 3), tile, win, 0.0, None, 0, None) == 2
    # window < 1
    bad = (ctypes.c_int * 3)(1, 0, 1)
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 1, 64, grid, tile, bad, 0.0, None, 0, None) == 3
    # unsupported: P = 8 not a multiple of 32; D = 48; bad dtype; D not a multiple of 8
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 1, 64, grid, tile, win, 0.0, None, 0, None) == 4
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 1, 48, I3(8, 8, 8), I3(4, 4, 2), win, 0.0, None, 0, None) == 4
    assert lib.sta_tile_permute(fake, fake2, 2, 0, 1, 1, 64, grid, tile, None) == 4
    assert lib.sta_tile_permute(fake, fake2, 0, 0, 1, 1, 12, grid, tile, None) == 4
    # aliasing
    assert lib.sta_tile_permute(fake, fake, 0, 0, 1, 1, 64, grid, tile, None) == 5
    assert lib.sta_forward(fake, fake, fake, fake, 1, 1, 64, I3(8, 8, 8), I3(4, 4, 2), win, 0.0, None, 0, None) == 5
    # key-tile box argument checks
    lo, hi = I3(), I3()
    assert lib.sta_key_tile_box(I3(2, 2, 2), I3(1, 1, 1), I3(0, 0, 2), lo, hi) == 2
    assert lib.sta_key_tile_box(I3(2, 2, 2), I3(1, 0, 1), I3(0, 0, 1), lo, hi) == 3
    # workspace: a positive size for the shapes whose kernels split work, zero otherwise; too small is an error
    need = sta.sta_workspace_bytes(1, 24, 128, (30, 48, 80), (6, 8, 8))
    assert need > 0 and need % 16 == 0
    assert sta.sta_workspace_bytes(1, 8, 64, (1, 64, 64), (1, 8, 8)) == 0
    assert sta.sta_workspace_bytes(1, 1, 128, (4, 4, 6), (2, 2, 8)) == 0          # P = 32
    win24 = (ctypes.c_int * 72)(*([3] * 72))
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 24, 128, I3(30, 48, 80), I3(6, 8, 8), win24, 0.0,
                           ctypes.c_void_p(0x40000000), need - 16, None) == 6
    assert lib.sta_forward(fake, fake, fake, fake2, 1, 24, 128, I3(30, 48, 80), I3(6, 8, 8), win24, 0.0,
                           ctypes.c_void_p(0x40000008), need, None) == 6


@pytest.mark.parametrize("grid,tile,win", [
    ((1, 24, 24), (1, 4, 4), (1, 12, 12)),
    ((1, 24, 24), (1, 4, 4), (1, 11, 11)),
    ((6, 8, 8), (2, 2, 2), (2, 6, 6)),
    ((4, 6, 9), (2, 3, 3), (7, 5, 3)),
    ((6, 6, 6), (1, 2, 3), (4, 4, 6)),
    ((2, 3, 4), (1, 1, 2), (9, 9, 9)),
    ((12, 12, 12), (4, 4, 4), (11, 11, 11)),
])
def test_block_census_matches_brute_force(grid, tile, win):
    """The library counts blocks from per-axis interval tests; the oracle enumerates every token pair."""
    for kind, name in ((sta.STA_MASK_STA, "sta"), (sta.STA_MASK_NATTEN, "natten")):
        if name == "sta" and any(w // t < 1 for w, t in zip(win, tile)):
            continue
        dense, mixed, totals = sta.sta_block_census(kind, grid, tile, win)
        o_dense, o_mixed = orc.block_census_per_query(name, "tiled", grid, tile, win)
        assert dense == o_dense.tolist() and mixed == o_mixed.tolist()
        n = len(dense)
        assert totals == (o_dense.sum(), o_mixed.sum(), n * n - o_dense.sum() - o_mixed.sum())


def test_block_census_table1_at_full_size():
    """Table 1 at its own size (video 48^3, tile 4^3): STA windows 12^3 and 20^3 give 27 and 125 dense blocks for
    every query tile and none mixed; the tiled sliding window 11^3 gives 1 dense and 124 mixed in the interior."""
    grid, tile = (48, 48, 48), (4, 4, 4)
    for w, per_q in ((12, 27), (20, 125)):
        dense, mixed, totals = sta.sta_block_census(sta.STA_MASK_STA, grid, tile, (w, w, w))
        assert set(dense) == {per_q} and set(mixed) == {0}
        assert abs(100.0 * totals[0] / 1728 ** 2 - {12: 1.56, 20: 7.23}[w]) < 0.005
    dense, mixed, totals = sta.sta_block_census(sta.STA_MASK_NATTEN, grid, tile, (11, 11, 11))
    mid = (6 * 12 + 6) * 12 + 6
    assert (dense[mid], mixed[mid]) == (1, 124)
    assert totals[0] + totals[1] + totals[2] == 1728 ** 2


def test_block_census_errors():
    with pytest.raises(sta.StaError) as e:
        sta.sta_block_census(sta.STA_MASK_STA, (4, 4, 4), (2, 2, 2), (1, 2, 2))      # less than one tile
    assert e.value.status == 3
    with pytest.raises(sta.StaError) as e:
        sta.sta_block_census(sta.STA_MASK_NATTEN, (4, 4, 5), (2, 2, 2), (3, 3, 3))   # grid not a multiple
    assert e.value.status == 2
    with pytest.raises(sta.StaError) as e:
        sta.sta_block_census(7, (4, 4, 4), (2, 2, 2), (3, 3, 3))
    assert e.value.status == 4


def test_query_tile_box_is_the_transpose_of_the_key_tile_box():
    """For every key tile, the query tiles whose box contains it, by scanning all boxes, equal the closed form."""
    for n, w in itertools.product(range(1, 9), range(1, 19)):
        grid = (1, 1, n)
        for k in range(n):
            scan = [q for q in range(n)
                    if sta.sta_key_tile_box(grid, (1, 1, w), (0, 0, q))[0][2] <= k
                    <= sta.sta_key_tile_box(grid, (1, 1, w), (0, 0, q))[1][2]]
            lo, hi = sta.sta_query_tile_box(grid, (1, 1, w), (0, 0, k))
            assert scan == list(range(lo[2], hi[2] + 1)), (n, w, k)
    # three axes at once, against the oracle's key-tile lists
    grid, tile, win = (4, 6, 10), (1, 2, 2), (3, 1, 5)
    n = (4, 3, 5)
    counts, lists = orc.key_tiles(grid, tile, orc.window_tiles_to_tokens(win, tile))
    for kt in range(60):
        keepers = sorted(q for q in range(60) if kt in lists[q, :counts[q]])
        c = np.unravel_index(kt, n)
        lo, hi = sta.sta_query_tile_box(n, win, tuple(int(x) for x in c))
        box = sorted(int(np.ravel_multi_index((a, b, d), n)) for a in range(lo[0], hi[0] + 1)
                     for b in range(lo[1], hi[1] + 1) for d in range(lo[2], hi[2] + 1))
        assert keepers == box, kt
