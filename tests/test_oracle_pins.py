"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- values the paper prints, closed forms, library routines
on special cases, brute-force characterisations written differently.  No GPU.
"""
import itertools
import os

import numpy as np
import pytest

from oracle import sta_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


def _dense_softmax_attention(q, k, v, scale):
    """Library one-liner for unmasked attention (numpy fp64 matmuls)."""
    q, k, v = (x.astype(np.float64) for x in (q, k, v))
    s = (q @ k.T) * scale
    s = s - s.max(axis=1, keepdims=True)
    a = np.exp(s)
    a /= a.sum(axis=1, keepdims=True)
    return a @ v


# --------------------------------------------------------------------------
# Whole attention: special cases that reduce to a library routine
# --------------------------------------------------------------------------
@pytest.mark.parametrize("grid,tile", [((4, 6, 4), (2, 3, 2)), ((1, 8, 12), (1, 4, 4)), ((6, 4, 4), (2, 2, 2))])
def test_full_window_equals_dense_softmax_attention(grid, tile):
    """Window covering the whole grid => textbook softmax(QK^T/sqrt(d))V (Eq. 1 with M = 0)."""
    N, d = int(np.prod(grid)), 16
    q, k, v = _rand((N, d), 1), _rand((N, d), 2), _rand((N, d), 3)
    out = orc.attention(q, k, v, grid, tile, window_tokens=grid)
    ref = _dense_softmax_attention(q, k, v, 1.0 / np.sqrt(d))
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_full_window_when_window_exceeds_grid():
    grid, tile = (4, 4, 6), (2, 2, 2)
    N, d = int(np.prod(grid)), 8
    q, k, v = _rand((N, d), 4), _rand((N, d), 5), _rand((N, d), 6)
    out = orc.attention(q, k, v, grid, tile, window_tokens=(8, 12, 14))
    ref = _dense_softmax_attention(q, k, v, 1.0 / np.sqrt(d))
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_unit_window_is_block_diagonal_per_tile_attention():
    """Window of one tile: each tile attends only to itself => independent dense
    attention over the tile's own tokens, gathered by coordinates."""
    grid, tile = (4, 6, 6), (2, 3, 2)
    N, d = int(np.prod(grid)), 12
    q, k, v = _rand((N, d), 7), _rand((N, d), 8), _rand((N, d), 9)
    out = orc.attention(q, k, v, grid, tile, window_tokens=tile)
    coords = np.stack(np.unravel_index(np.arange(N), grid), axis=1)
    tile_of = coords // np.array(tile)
    for tc in itertools.product(*[range(g // t) for g, t in zip(grid, tile)]):
        idx = np.nonzero((tile_of == np.array(tc)).all(axis=1))[0]
        assert idx.size == np.prod(tile)
        ref = _dense_softmax_attention(q[idx], k[idx], v[idx], 1.0 / np.sqrt(d))
        np.testing.assert_allclose(out[idx], ref, rtol=1e-12, atol=1e-13)


def test_scale_argument_and_default():
    """Default scale is 1/sqrt(d_k) (Eq. 1); an explicit scale multiplies QK^T."""
    grid, tile = (2, 4, 4), (1, 2, 2)
    N, d = int(np.prod(grid)), 8
    q, k, v = _rand((N, d), 10), _rand((N, d), 11), _rand((N, d), 12)
    a = orc.attention(q, k, v, grid, tile, grid)
    b = orc.attention(q * 2.0, k, v, grid, tile, grid, scale=0.5 / np.sqrt(d))
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    c = orc.attention(q, k, v, grid, tile, grid, scale=0.3)
    np.testing.assert_allclose(c, _dense_softmax_attention(q, k, v, 0.3), rtol=1e-12, atol=1e-13)


def test_operands_not_transposed_or_swapped():
    """Distinct roles of Q, K, V: swapping K and V, or Q and K, changes the result
    in the way the dense library routine says."""
    grid, tile = (2, 2, 4), (1, 1, 2)
    N, d = int(np.prod(grid)), 4
    q, k, v = _rand((N, d), 13), _rand((N, d), 14), _rand((N, d), 15)
    np.testing.assert_allclose(orc.attention(k, q, v, grid, tile, grid),
                               _dense_softmax_attention(k, q, v, 0.5), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.attention(q, v, k, grid, tile, grid),
                               _dense_softmax_attention(q, v, k, 0.5), rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------
# Softmax invariants
# --------------------------------------------------------------------------
def test_softmax_rows_sum_to_one_and_vanish_outside_window():
    grid, tile, win = (4, 6, 6), (2, 2, 2), (2, 6, 2)
    N, d = int(np.prod(grid)), 8
    q, k = _rand((N, d), 16) * 3.0, _rand((N, d), 17) * 3.0
    for i in (0, 17, 71, N - 1):
        p, s = orc.probs(q, k, grid, tile, win, i)
        assert abs(s - 1.0) <= 1e-14
        assert abs(p.sum() - 1.0) <= 1e-13
        assert (p >= 0).all()
        qc = np.unravel_index(i, grid)
        for j in range(N):
            kc = np.unravel_index(j, grid)
            assert (p[j] > 0) == orc.keep(qc, kc, grid, win, tile)


def test_constant_v_and_convex_hull():
    grid, tile, win = (2, 6, 8), (1, 2, 2), (1, 6, 6)
    N, d = int(np.prod(grid)), 6
    q, k = _rand((N, d), 18), _rand((N, d), 19)
    vconst = np.tile(np.linspace(-1, 1, d, dtype=np.float32), (N, 1))
    out = orc.attention(q, k, vconst, grid, tile, win)
    np.testing.assert_allclose(out, vconst.astype(np.float64), rtol=0, atol=1e-14)
    v = _rand((N, d), 20)
    out = orc.attention(q, k, v, grid, tile, win)
    assert (out <= v.max(axis=0) + 1e-12).all() and (out >= v.min(axis=0) - 1e-12).all()


# --------------------------------------------------------------------------
# Kept set, read straight out of the attention output (Q = 0, one-hot V)
# --------------------------------------------------------------------------
def _axis_box_by_shifting(qt, n, w):
    """Independent characterisation of the border rule (Sec. 2.1: window centres
    shift at the borders so every query keeps a constant number of keys): the
    interval of 2*(w//2)+1 tiles centred on qt, slid the least distance needed
    to lie inside [0, n-1]; if it cannot fit, the whole axis."""
    half = w // 2
    size = 2 * half + 1
    if size >= n:
        return set(range(n))
    lo = qt - half
    while lo < 0:
        lo += 1
    while lo + size - 1 > n - 1:
        lo -= 1
    return set(range(lo, lo + size))


@pytest.mark.parametrize("grid,tile,win_tiles", [
    ((4, 6, 10), (1, 2, 2), (3, 3, 3)),
    ((4, 6, 10), (2, 2, 2), (1, 3, 5)),
    ((6, 4, 8), (1, 1, 2), (5, 1, 3)),
    ((1, 12, 12), (1, 2, 2), (1, 3, 3)),
    ((3, 6, 6), (1, 2, 2), (2, 4, 3)),      # even window entries: follow the algorithm literally
])
def test_kept_set_read_from_output_matches_shifted_window(grid, tile, win_tiles):
    tg = [g // t for g, t in zip(grid, tile)]
    n = int(np.prod(tg))
    N = int(np.prod(grid))
    coords = np.stack(np.unravel_index(np.arange(N), grid), axis=1)
    tile_id = np.ravel_multi_index((coords // np.array(tile)).T, tg)
    d = n
    q = np.zeros((N, d), np.float32)
    k = _rand((N, d), 21)
    v = np.zeros((N, d), np.float32)
    v[np.arange(N), tile_id] = 1.0
    win_tokens = orc.window_tiles_to_tokens(win_tiles, tile)
    out = orc.attention(q, k, v, grid, tile, win_tokens)
    for i in range(N):
        qt = np.unravel_index(tile_id[i], tg)
        boxes = [_axis_box_by_shifting(qt[a], tg[a], win_tiles[a]) for a in range(3)]
        kept = {int(np.ravel_multi_index(c, tg)) for c in itertools.product(*boxes)}
        expect = np.zeros(n)
        expect[list(kept)] = 1.0 / len(kept)
        np.testing.assert_allclose(out[i], expect, rtol=0, atol=1e-14)


# --------------------------------------------------------------------------
# Counts the paper prints
# --------------------------------------------------------------------------
def test_table1_sta_block_ratios():
    """Table 1 STA rows / Theorem 2 at video 48^3, tile 4^3."""
    grid, tile = (48, 48, 48), (4, 4, 4)
    for w, dense_pct, mixed_pct in _rows("table1_sta_block_ratios.txt"):
        w = int(w)
        counts, _ = orc.key_tiles(grid, tile, (w, w, w))
        n = counts.size
        assert n == 12 ** 3
        dense = int(counts.sum())
        assert dense == (w // 4) ** 3 * 12 ** 3                 # Theorem 2
        assert round(100.0 * dense / n ** 2, 2) == float(dense_pct)
        assert float(mixed_pct) == 0.0


def test_hunyuan_grid_sparsities():
    """91.00 / 58.33 / 75.00 % on the (30,48,80) grid with tile (6,8,8); every query
    tile keeps the same number of key tiles."""
    grid, tile = (30, 48, 80), (6, 8, 8)
    for wt, wh, ww, pct in _rows("sparsity_hunyuan_grid.txt"):
        win = (int(wt), int(wh), int(ww))
        counts, lists = orc.key_tiles(grid, tile, win)
        assert counts.size == 300
        per_q = (win[0] // 6) * (win[1] // 8) * (win[2] // 8)
        assert (counts == per_q).all()
        sparsity = 100.0 * (1.0 - counts.sum() / 300.0 ** 2)
        assert abs(sparsity - float(pct)) < 0.005
        for qt in range(300):                                       # a tile always keeps itself
            assert qt in lists[qt, :counts[qt]]


def test_fig4_nine_dense_blocks_per_query_tile():
    (th, tw, wh, ww, nblocks, br, bc), = _rows("fig4_2d_tile2_window6.txt")
    tile = (1, int(th), int(tw))
    grid = (1, 12, 16)
    counts, _ = orc.key_tiles(grid, tile, (1, int(wh), int(ww)))
    assert (counts == int(nblocks)).all()
    assert tile[1] * tile[2] == int(br) == int(bc)
    dense, mixed, empty = orc.block_census(grid, tile, (1, int(wh), int(ww)))
    assert dense == int(nblocks) * counts.size and mixed == 0


@pytest.mark.parametrize("grid,tile,win", [
    ((1, 24, 24), (1, 4, 4), (1, 12, 12)),      # Fig. 3 setting: image 24x24, window 12x12, tile 4x4
    ((6, 8, 8), (2, 2, 2), (2, 6, 6)),
    ((4, 6, 9), (2, 3, 3), (6, 6, 9)),
    ((6, 6, 6), (1, 2, 3), (4, 4, 6)),          # even tile-window
])
def test_no_mixed_blocks_by_brute_force(grid, tile, win):
    """Theorem 2: every block is dense or empty; dense count = sum of per-tile list sizes."""
    dense, mixed, empty = orc.block_census(grid, tile, win)
    counts, _ = orc.key_tiles(grid, tile, win)
    n = counts.size
    assert mixed == 0
    assert dense == counts.sum()
    assert dense + empty == n * n


def test_one_axis_border_placement_enumeration():
    """1-D enumeration: for every n <= 10, window w <= n + 2 and query tile, the kept
    interval is contiguous, has size min(n, 2*(w//2)+1), contains the query tile, lies
    in the grid, and equals [q-half, q+half] whenever that fits."""
    for n in range(1, 11):
        for w in range(1, n + 3):
            counts, lists = orc.key_tiles((1, 1, n), (1, 1, 1), (1, 1, w))
            half = w // 2
            for qt in range(n):
                ks = lists[qt, :counts[qt]].tolist()
                assert ks == list(range(ks[0], ks[0] + len(ks)))
                assert len(ks) == min(n, 2 * half + 1)
                assert qt in ks and ks[0] >= 0 and ks[-1] <= n - 1
                if qt - half >= 0 and qt + half <= n - 1:
                    assert ks == list(range(qt - half, qt + half + 1))
                assert set(ks) == _axis_box_by_shifting(qt, n, w)


def test_mask_is_not_symmetric_at_borders():
    """Border clamp: tile 0 keeps tile 2 (window 3 of 4 tiles) but tile 2 does not keep tile 0."""
    grid, tile, win = (1, 1, 4), (1, 1, 1), (1, 1, 3)
    assert orc.keep((0, 0, 0), (0, 0, 2), grid, win, tile)
    assert not orc.keep((0, 0, 2), (0, 0, 0), grid, win, tile)


def test_axes_are_not_mixed_up():
    """Different window per axis on a non-cubic grid: the kept box has the per-axis sizes
    in the right order."""
    grid, tile, win_tiles = (8, 10, 12), (2, 2, 2), (1, 3, 5)
    counts, lists = orc.key_tiles(grid, tile, orc.window_tiles_to_tokens(win_tiles, tile))
    tg = (4, 5, 6)
    for qt in range(counts.size):
        c = np.array(np.unravel_index(lists[qt, :counts[qt]], tg))
        spans = [int(c[a].max() - c[a].min() + 1) for a in range(3)]
        assert spans == [1, 3, 5]


# --------------------------------------------------------------------------
# Permutation
# --------------------------------------------------------------------------
def test_fig7_order_9x9_tile3x3():
    want = np.array([int(x) for row in _rows("fig7_9x9_tile3x3_order.txt") for x in row])
    got = orc.tile_order((1, 9, 9), (1, 3, 3))
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("grid,tile", [((4, 6, 8), (2, 3, 4)), ((18, 24, 24), (6, 8, 8)), ((1, 16, 8), (1, 8, 8)),
                                       ((3, 5, 7), (3, 5, 7)), ((3, 5, 7), (1, 1, 1))])
def test_permutation_is_bijection_tiles_contiguous_and_roundtrip(grid, tile):
    N = int(np.prod(grid))
    P = int(np.prod(tile))
    order = orc.tile_order(grid, tile)
    assert sorted(order.tolist()) == list(range(N))
    tg = [g // t for g, t in zip(grid, tile)]
    coords = np.stack(np.unravel_index(order, grid), axis=1)
    tid = np.ravel_multi_index((coords // np.array(tile)).T, tg)
    np.testing.assert_array_equal(tid, np.repeat(np.arange(N // P), P))      # tile tau occupies [tau*P, (tau+1)*P)
    intra = np.ravel_multi_index((coords % np.array(tile)).T, tile)
    np.testing.assert_array_equal(intra, np.tile(np.arange(P), N // P))      # row-major inside the tile
    x = _rand((2, 3, N, 4), 22)
    y = orc.tile_permute(x, grid, tile)
    np.testing.assert_array_equal(y, x[:, :, order, :])
    np.testing.assert_array_equal(orc.untile(y, grid, tile), x)
    xb = (np.arange(2 * N * 6, dtype=np.uint16)).reshape(2, N, 6)               # 2-byte rows move whole
    np.testing.assert_array_equal(orc.untile(orc.tile_permute(xb, grid, tile), grid, tile), xb)


def test_permutation_equivariance_of_attention():
    """Attention over tile-ordered tokens, computed by the dense library routine per
    kept set, equals the raster-order oracle gathered into tile order."""
    grid, tile, win = (2, 4, 6), (1, 2, 2), (1, 6, 2)
    N, d = int(np.prod(grid)), 8
    q, k, v = _rand((N, d), 23), _rand((N, d), 24), _rand((N, d), 25)
    out = orc.attention(q, k, v, grid, tile, win)
    order = orc.tile_order(grid, tile)
    counts, lists = orc.key_tiles(grid, tile, win)
    P = int(np.prod(tile))
    qt_, kt_, vt_ = q[order], k[order], v[order]
    for qt in range(counts.size):
        keys = np.concatenate([np.arange(t * P, (t + 1) * P) for t in lists[qt, :counts[qt]]])
        ref = _dense_softmax_attention(qt_[qt * P:(qt + 1) * P], kt_[keys], vt_[keys], 1.0 / np.sqrt(d))
        np.testing.assert_allclose(out[order][qt * P:(qt + 1) * P], ref, rtol=1e-12, atol=1e-13)


def test_non_multiple_grid_is_rejected():
    with pytest.raises(ValueError):
        orc.tile_order((5, 4, 4), (2, 2, 2))
    with pytest.raises(ValueError):
        orc.key_tiles((4, 4, 5), (2, 2, 2), (2, 2, 2))


# --------------------------------------------------------------------------
# Log of the softmax denominator, and the attention recall built from it
# --------------------------------------------------------------------------
def test_lse_full_window_is_library_logsumexp():
    from scipy.special import logsumexp
    grid, tile = (2, 6, 4), (1, 3, 2)
    N, d = int(np.prod(grid)), 16
    q, k, v = _rand((N, d), 31), _rand((N, d), 32), _rand((N, d), 33)
    out, lse = orc.attention(q, k, v, grid, tile, grid, return_lse=True)
    s = (q.astype(np.float64) @ k.astype(np.float64).T) / np.sqrt(d)
    np.testing.assert_allclose(lse, logsumexp(s, axis=1), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(out, _dense_softmax_attention(q, k, v, 1.0 / np.sqrt(d)), rtol=1e-12, atol=1e-13)


def test_lse_unit_window_is_per_tile_logsumexp():
    from scipy.special import logsumexp
    grid, tile = (4, 4, 6), (2, 2, 3)
    N, d = int(np.prod(grid)), 8
    q, k, v = _rand((N, d), 34), _rand((N, d), 35), _rand((N, d), 36)
    _, lse = orc.attention(q, k, v, grid, tile, tile, scale=0.7, return_lse=True)
    coords = np.stack(np.unravel_index(np.arange(N), grid), axis=1)
    tile_of = coords // np.array(tile)
    for tc in itertools.product(*[range(g // t) for g, t in zip(grid, tile)]):
        idx = np.nonzero((tile_of == np.array(tc)).all(axis=1))[0]
        s = (q[idx].astype(np.float64) @ k[idx].astype(np.float64).T) * 0.7
        np.testing.assert_allclose(lse[idx], logsumexp(s, axis=1), rtol=1e-13, atol=1e-13)


def test_recall_from_lse_equals_probability_mass_inside_the_window():
    """Attention recall (Sec. 1: the fraction of the total attention score that falls inside a local
    window) of query i is sum_{j kept} A_full[i, j].  It must equal exp(lse_window - lse_full)."""
    grid, tile, win = (2, 6, 6), (1, 2, 2), (1, 6, 2)
    N, d = int(np.prod(grid)), 8
    q, k, v = _rand((N, d), 37) * 2.0, _rand((N, d), 38) * 2.0, _rand((N, d), 39)
    _, lse_w = orc.attention(q, k, v, grid, tile, win, return_lse=True)
    _, lse_f = orc.attention(q, k, v, grid, tile, grid, return_lse=True)
    recall = np.exp(lse_w - lse_f)
    assert (recall > 0).all() and (recall <= 1 + 1e-14).all()
    for i in (0, 5, 33, N - 1):
        p_full, _ = orc.probs(q, k, grid, tile, grid, i)
        qc = np.unravel_index(i, grid)
        inside = np.array([orc.keep(qc, np.unravel_index(j, grid), grid, win, tile) for j in range(N)])
        np.testing.assert_allclose(recall[i], p_full[inside].sum(), rtol=1e-12)


# --------------------------------------------------------------------------
# Mask-search inner loop ("STA Mask Search")
# --------------------------------------------------------------------------
def test_head_mse_is_library_mean_squared_error():
    from sklearn.metrics import mean_squared_error
    a, b = _rand((2, 3, 10, 4), 41), _rand((2, 3, 10, 4), 42)
    got = orc.head_mse(a, b)
    for h in range(3):
        want = mean_squared_error(a[:, h].reshape(-1).astype(np.float64), b[:, h].reshape(-1).astype(np.float64))
        np.testing.assert_allclose(got[h], want, rtol=1e-13)


def test_mask_search_full_pattern_has_zero_loss_and_first_minimum_wins():
    grid, tile = (2, 4, 6), (1, 2, 2)
    N, d, H = int(np.prod(grid)), 8, 2
    q, k, v = _rand((1, H, N, d), 43), _rand((1, H, N, d), 44), _rand((1, H, N, d), 45)
    pats = [(1, 2, 2), (1, 4, 2), tuple(grid), (1, 2, 6), tuple(grid)]
    losses, best = orc.mask_search(q, k, v, grid, tile, pats)
    assert (losses[2] == 0).all() and (losses[4] == 0).all()
    assert (losses[[0, 1, 3]] > 0).all()
    assert (best == 2).all()                       # the second zero-loss entry does not replace the first
    # constant V: every window gives the same output up to rounding, so every loss vanishes
    vconst = np.ones_like(v)
    losses, _ = orc.mask_search(q, k, vconst, grid, tile, pats)
    assert np.abs(losses).max() <= 1e-28


def test_mask_search_losses_match_dense_library_attention():
    """Loss of a one-tile window against full attention, both computed by the dense library routine."""
    grid, tile = (1, 4, 4), (1, 2, 2)
    N, d = 16, 4
    q, k, v = _rand((1, 1, N, d), 46), _rand((1, 1, N, d), 47), _rand((1, 1, N, d), 48)
    losses, best = orc.mask_search(q, k, v, grid, tile, [tile])
    full = _dense_softmax_attention(q[0, 0], k[0, 0], v[0, 0], 0.5)
    coords = np.stack(np.unravel_index(np.arange(N), grid), axis=1)
    tid = np.ravel_multi_index((coords // np.array(tile)).T, (1, 2, 2))
    local = np.empty_like(full)
    for t in range(4):
        idx = np.nonzero(tid == t)[0]
        local[idx] = _dense_softmax_attention(q[0, 0][idx], k[0, 0][idx], v[0, 0][idx], 0.5)
    np.testing.assert_allclose(losses[0, 0], ((full - local) ** 2).mean(), rtol=1e-12)
    assert best[0] == 0


# ---- sliding-window (NATTEN) mask and the block census -------------------------------------------------------

def test_natten_mask_is_sta_mask_with_unit_tiles():
    """With tile (1,1,1) the STA mask algorithm reduces, line by line, to the sliding-window one."""
    grid = (3, 5, 6)
    for win in ((1, 1, 1), (3, 3, 3), (3, 5, 1), (5, 3, 7), (9, 9, 9), (2, 4, 6)):
        a_dense, a_mixed = orc.block_census_per_query("sta", "tiled", grid, (1, 1, 1), win)
        b_dense, b_mixed = orc.block_census_per_query("natten", "tiled", grid, (1, 1, 1), win)
        assert (a_dense == b_dense).all() and (a_mixed == 0).all() and (b_mixed == 0).all()
    # and pair by pair on one window
    coords = [np.unravel_index(i, grid) for i in range(int(np.prod(grid)))]
    for q in coords[::7]:
        for k in coords:
            t = tuple(int(abs(max(min(q[a], grid[a] - 1 - 1), 1) - k[a]) <= 1) for a in range(3))
            assert orc.natten_keep(q, k, grid, (3, 3, 3)) == bool(t[0] and t[1] and t[2])


def test_natten_every_query_attends_to_a_constant_number_of_keys():
    """Sec. 2.2: the window centre is shifted at the borders so that every query keeps the same number of keys."""
    grid = (4, 6, 7)
    for win in ((3, 3, 3), (1, 5, 3), (3, 5, 7), (9, 3, 5)):
        dense, _ = orc.block_census_per_query("natten", "tiled", grid, (1, 1, 1), win)
        expect = int(np.prod([min(grid[a], 2 * (win[a] // 2) + 1) for a in range(3)]))
        assert (dense == expect).all()


def test_theorem1_interior_counts_one_axis():
    """Theorem 1 per axis: an interior query tile has max(2*floor((W+1)/(2T)) - 1, 0) dense blocks and
    2*ceil((W-1)/(2T)) + 1 non-empty ones."""
    for T in (2, 3, 4, 8):
        for W in range(1, 4 * T + 4, 2):
            n = 2 * (-(-(W - 1) // (2 * T)) + 2) + 1          # enough tiles that the middle one sees no border
            dense, mixed = orc.block_census_per_query("natten", "tiled", (1, 1, n * T), (1, 1, T), (1, 1, W))
            mid = n // 2
            assert dense[mid] == max(2 * ((W + 1) // (2 * T)) - 1, 0), (T, W)
            assert dense[mid] + mixed[mid] == 2 * (-(-(W - 1) // (2 * T))) + 1, (T, W)


def test_table1_tiled_natten_row():
    """Table 1, Tiled NATTEN, tile 4^3, window 11^3: one dense and 124 mixed blocks per interior query tile, i.e.
    0.06 % and 7.17 % of the 12^3 key tiles of the 48^3 video."""
    (w, dense_pct, mixed_pct), = _rows("table1_tiled_natten_block_ratios.txt")
    w = int(w)
    dense, mixed = orc.block_census_per_query("natten", "tiled", (28, 28, 28), (4, 4, 4), (w, w, w))
    mid = (3 * 7 + 3) * 7 + 3                                   # tile (3,3,3) of the 7^3 tile grid
    assert (dense[mid], mixed[mid]) == (1, 124)
    n_tiles_48 = 12 ** 3
    assert abs(100.0 * dense[mid] / n_tiles_48 - float(dense_pct)) < 0.005
    assert abs(100.0 * mixed[mid] / n_tiles_48 - float(mixed_pct)) < 0.01
    # border tiles keep fewer blocks, which is what "ignoring boundary effects" leaves out
    assert mixed.sum() < 124 * mixed.size and dense.sum() >= dense.size


def test_fig3_block_types_for_the_three_orderings():
    """Fig. 3 (image 24x24, window 12x12, tile 4x4): the sliding window in raster order has only mixed blocks,
    tiling the tokens turns some of them dense, STA has no mixed block at all."""
    grid, tile, win = (1, 24, 24), (1, 4, 4), (1, 12, 12)
    rd, rm = orc.block_census_per_query("natten", "raster", grid, tile, win)
    td, tm = orc.block_census_per_query("natten", "tiled", grid, tile, win)
    sd, sm = orc.block_census_per_query("sta", "tiled", grid, tile, win)
    assert sm.sum() == 0 and sd.sum() == 36 * 9
    assert 0 < tm.sum() < rm.sum()
    assert td.sum() > rd.sum()
    # old and new census agree on STA
    assert orc.block_census(grid, tile, win)[:2] == (sd.sum(), 0)


def test_raster_block_census_on_countable_cases():
    """The raster-order census (blocks of P consecutive raster tokens) on cases that can be counted by hand.
    (a) In 1-D raster order and tile order are the same order, so both censuses agree block by block, for both masks
    (the tiled one is pinned to Theorem 1 above).  (b) A window that covers the whole grid keeps every pair: every
    block is dense in any order.  (c) Image 2 x 8, tile 2 x 2 (P = 4), STA window of one tile: a raster block is half
    an image row, i.e. the top (or bottom) halves of two tiles; each of its queries keeps the two columns of its own
    tile in both rows, so the block meets the two half-row key blocks of its own image half partially (mixed), the
    other two not at all, and none completely."""
    for T, W, n in ((4, 5, 9), (3, 9, 8), (8, 3, 5)):
        grid, tile, win = (1, 1, n * T), (1, 1, T), (1, 1, W)
        for mask in ("sta", "natten"):
            rd, rm = orc.block_census_per_query(mask, "raster", grid, tile, win)
            td, tm = orc.block_census_per_query(mask, "tiled", grid, tile, win)
            assert (rd == td).all() and (rm == tm).all(), (mask, T, W)
    grid, tile = (2, 4, 6), (1, 2, 3)
    for mask in ("sta", "natten"):
        for order in ("raster", "tiled"):
            d, m = orc.block_census_per_query(mask, order, grid, tile, (3, 9, 11))     # covers 2 x 4 x 6 from anywhere
            assert (d == 8).all() and (m == 0).all(), (mask, order)
    d, m = orc.block_census_per_query("sta", "raster", (1, 2, 8), (1, 2, 2), (1, 2, 2))
    assert d.tolist() == [0, 0, 0, 0] and m.tolist() == [2, 2, 2, 2]
    d, m = orc.block_census_per_query("sta", "tiled", (1, 2, 8), (1, 2, 2), (1, 2, 2))
    assert d.tolist() == [1, 1, 1, 1] and m.tolist() == [0, 0, 0, 0]


# ---- gradients of Eq. 1 under the STA mask ---------------------------------------------------------------

def _autograd_dense(q, k, v, g, scale, additive_mask=None):
    """Library automatic differentiation of softmax(QK^T*scale + mask)V in fp64."""
    import torch
    tq, tk, tv = [torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True) for x in (q, k, v)]
    s = tq @ tk.T * scale
    if additive_mask is not None:
        s = s + torch.tensor(additive_mask)
    o = torch.softmax(s, dim=-1) @ tv
    (o * torch.tensor(np.asarray(g, dtype=np.float64))).sum().backward()
    return tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


def test_backward_full_window_matches_library_autodiff():
    grid, tile = (2, 4, 6), (1, 2, 2)
    N, d = 48, 8
    q, k, v, g = (_rand((N, d), s) for s in (61, 62, 63, 64))
    dq, dk, dv = orc.attention_backward(q, k, v, g, grid, tile, grid, scale=0.3)
    for mine, ref in zip((dq, dk, dv), _autograd_dense(q, k, v, g, 0.3)):
        np.testing.assert_allclose(mine, ref, rtol=0, atol=1e-13)


def test_backward_unit_window_is_per_tile_dense_autodiff():
    grid, tile = (2, 4, 4), (1, 2, 2)
    N, d = 32, 4
    q, k, v, g = (_rand((N, d), s) for s in (65, 66, 67, 68))
    dq, dk, dv = orc.attention_backward(q, k, v, g, grid, tile, tile)
    coords = np.stack(np.unravel_index(np.arange(N), grid), axis=1)
    tid = np.ravel_multi_index((coords // np.array(tile)).T, (2, 2, 2))
    for t in range(8):
        idx = np.nonzero(tid == t)[0]
        refs = _autograd_dense(q[idx], k[idx], v[idx], g[idx], 0.5)
        for mine, ref in zip((dq, dk, dv), refs):
            np.testing.assert_allclose(mine[idx], ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("win", [(1, 6, 2), (2, 2, 6), (1, 2, 2)])
def test_backward_windowed_matches_finite_differences_of_the_forward(win):
    """Central differences of sum(O * G) computed with the (separately pinned) forward oracle."""
    grid, tile = (2, 4, 6), (1, 2, 2)
    N, d = 48, 8
    q, k, v, g = (_rand((N, d), s) for s in (71, 72, 73, 74))
    dq, dk, dv = orc.attention_backward(q, k, v, g, grid, tile, win)

    def loss(qq, kk, vv):
        return float((orc.attention(qq, kk, vv, grid, tile, win) * g).sum())

    eps = 2.0 ** -10                                            # exactly representable steps
    for which, grad in enumerate((dq, dk, dv)):
        for (i, c) in ((0, 0), (17, 3), (30, 5), (47, 7)):
            args_p, args_m = [q.copy(), k.copy(), v.copy()], [q.copy(), k.copy(), v.copy()]
            args_p[which][i, c] += eps
            args_m[which][i, c] -= eps
            fd = (loss(*args_p) - loss(*args_m)) / (float(args_p[which][i, c]) - float(args_m[which][i, c]))
            assert abs(fd - grad[i, c]) <= 2e-6 * max(1.0, abs(fd)), (which, i, c, fd, grad[i, c])


def test_backward_windowed_matches_library_autodiff_with_additive_mask():
    """The mask enters Eq. 1 as M (0 / -inf added to S): hand that matrix to the library's autodiff."""
    grid, tile, win = (2, 6, 6), (1, 2, 3), (1, 6, 3)           # even tile-window along h, borders on every axis
    N, d = 72, 8
    q, k, v, g = (_rand((N, d), s) for s in (75, 76, 77, 78))
    coords = [tuple(int(x) for x in np.unravel_index(i, grid)) for i in range(N)]
    M = np.array([[0.0 if orc.keep(qi, kj, grid, win, tile) else -np.inf for kj in coords] for qi in coords])
    dq, dk, dv = orc.attention_backward(q, k, v, g, grid, tile, win)
    for mine, ref in zip((dq, dk, dv), _autograd_dense(q, k, v, g, 1.0 / np.sqrt(d), M)):
        np.testing.assert_allclose(mine, ref, rtol=0, atol=1e-13)
    # a sample of rows gives the same rows
    qi, ki = np.array([3, 40, 71]), np.array([0, 35])
    sq, sk, sv = orc.attention_backward(q, k, v, g, grid, tile, win, query_idx=qi, key_idx=ki)
    np.testing.assert_array_equal(sq, dq[qi])
    np.testing.assert_array_equal(sk, dk[ki])
    np.testing.assert_array_equal(sv, dv[ki])


def test_backward_invariants():
    grid, tile, win = (2, 4, 6), (1, 2, 2), (1, 6, 2)
    N, d = 48, 8
    q, k, v, g = (_rand((N, d), s) for s in (81, 82, 83, 84))
    dq, dk, dv = orc.attention_backward(q, k, v, g, grid, tile, win)
    # adding one vector to every key shifts each score row by a constant: the loss does not move
    assert np.abs(dk.sum(axis=0)).max() < 1e-13
    # O is a convex combination of V rows: shifting all of V by c shifts O by c, so sum_j dV_j = sum_i G_i
    np.testing.assert_allclose(dv.sum(axis=0), g.astype(np.float64).sum(axis=0), atol=1e-13)
    # constant V: O does not depend on Q or K
    dq0, dk0, _ = orc.attention_backward(q, k, np.ones_like(v), g, grid, tile, win)
    assert np.abs(dq0).max() < 1e-13 and np.abs(dk0).max() < 1e-13
