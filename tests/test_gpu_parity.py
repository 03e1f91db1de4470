"""GPU parity tests: the HIP path, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Integer / byte work must be bit-exact;
attention output must meet the tolerances in gpu_util."""
import itertools

import numpy as np
import pytest
import torch

import paper_2502_04507_amd as sta
import synth_inputs as syn
from oracle import sta_oracle as orc
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _as_u16(t):
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------------------
# Permutation: bit-exact
# --------------------------------------------------------------------------
PERM_CASES = [
    ("C1grid", 1, 1, 64, (18, 24, 24), (6, 8, 8)),
    ("C2grid", 1, 8, 64, (1, 64, 64), (1, 8, 8)),
    ("C3grid", 1, 12, 128, (12, 48, 48), (6, 8, 8)),
    ("ragged", 2, 3, 40, (6, 10, 14), (3, 5, 7)),
    ("unit-tile", 1, 2, 8, (3, 5, 7), (1, 1, 1)),
    ("one-tile", 1, 2, 16, (2, 3, 4), (2, 3, 4)),
    ("wide-w", 1, 1, 128, (2, 4, 96), (1, 2, 32)),
]


@pytest.mark.parametrize("name,B,H,D,grid,tile", PERM_CASES)
def test_tile_permute_and_untile_bit_exact(name, B, H, D, grid, tile):
    N = int(np.prod(grid))
    g = torch.Generator().manual_seed(7)
    x = torch.randn((B, H, N, D), generator=g).to(torch.bfloat16)
    xd = x.to(DEV)
    y = torch.full_like(xd, float("nan"))
    sta.sta_tile_permute(xd, y, grid, tile)
    want = orc.tile_permute(_as_u16(x), grid, tile)
    np.testing.assert_array_equal(_as_u16(y.cpu()), want)
    z = torch.full_like(xd, float("nan"))
    sta.sta_untile(y, z, grid, tile)
    np.testing.assert_array_equal(_as_u16(z.cpu()), _as_u16(x))
    np.testing.assert_array_equal(_as_u16(z.cpu()), orc.untile(want, grid, tile))


def test_tile_permute_full_size_grid_bit_exact():
    """The 30x48x80 grid at full head dim; 4 heads keep the host side light."""
    w = syn.workload("C4")
    N, D = w.N, w.D
    g = torch.Generator().manual_seed(8)
    x = torch.randn((1, 4, N, D), generator=g).to(torch.bfloat16)
    xd = x.to(DEV)
    y = torch.empty_like(xd)
    sta.sta_tile_permute(xd, y, w.grid, w.tile)
    order = torch.from_numpy(orc.tile_order(w.grid, w.tile))
    assert torch.equal(y.cpu().view(torch.int16), x.view(torch.int16)[:, :, order, :])
    z = torch.empty_like(xd)
    sta.sta_untile(y, z, w.grid, w.tile)
    assert torch.equal(z.cpu().view(torch.int16), x.view(torch.int16))


def test_tile_permute_fused_casts_bit_exact():
    grid, tile = (18, 24, 24), (6, 8, 8)
    N = int(np.prod(grid))
    g = torch.Generator().manual_seed(9)
    x = torch.randn((1, 2, N, 64), generator=g)
    x[0, 0, 0, :8] = torch.tensor([0.0, -0.0, float("inf"), -float("inf"), 1e-40, 3.3895e38, 1.00390625, 1.01171875])
    xd = x.to(DEV)
    y = torch.empty((1, 2, N, 64), dtype=torch.bfloat16, device=DEV)
    sta.sta_tile_permute(xd, y, grid, tile)                       # f32 -> bf16, round to nearest even
    want = orc.tile_permute(_as_u16(x.to(torch.bfloat16)), grid, tile)
    np.testing.assert_array_equal(_as_u16(y.cpu()), want)
    z = torch.empty((1, 2, N, 64), dtype=torch.float32, device=DEV)
    sta.sta_untile(y, z, grid, tile)                              # bf16 -> f32, exact
    assert torch.equal(z.cpu(), x.to(torch.bfloat16).float())
    y32 = torch.empty_like(xd)
    sta.sta_tile_permute(xd, y32, grid, tile)                     # f32 -> f32
    np.testing.assert_array_equal(y32.cpu().numpy().view(np.uint32),
                                  orc.tile_permute(x.numpy().view(np.uint32), grid, tile))


# --------------------------------------------------------------------------
# Key-tile lists as the device computes them: bit-exact
# --------------------------------------------------------------------------
@pytest.mark.parametrize("grid,tile,windows", [
    ((30, 48, 80), (6, 8, 8), [(3, 3, 3), (1, 3, 3), (3, 3, 5), (5, 6, 10), (5, 3, 5), (5, 5, 5), (1, 1, 1)]),
    ((12, 48, 48), (6, 8, 8), [(1, 3, 3), (2, 2, 2), (7, 1, 4)]),
    ((1, 64, 64), (1, 8, 8), [(1, 3, 3), (1, 8, 8), (1, 5, 1), (4, 2, 9)]),
    ((4, 4, 4), (4, 4, 4), [(1, 1, 1), (3, 3, 3)]),
])
def test_device_key_tile_lists_bit_exact(grid, tile, windows):
    H = len(windows)
    n = int(np.prod([g // t for g, t in zip(grid, tile)]))
    counts = torch.full((H, n), -7, dtype=torch.int32, device=DEV)
    lists = torch.full((H, n, n), -7, dtype=torch.int32, device=DEV)
    sta.sta_dump_key_tiles(H, grid, tile, windows, counts, lists)
    torch.cuda.synchronize()
    for h, wt in enumerate(windows):
        oc, ol = orc.key_tiles(grid, tile, orc.window_tiles_to_tokens(wt, tile))
        np.testing.assert_array_equal(counts[h].cpu().numpy(), oc)
        np.testing.assert_array_equal(lists[h].cpu().numpy(), ol)


# --------------------------------------------------------------------------
# Attention: whole-problem parity on the small configurations
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_attention_parity_whole_problem(name):
    w = syn.workload(name)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for b in range(w.B):
        for h in range(w.H):
            ref = gu.oracle_rows(w, q, k, v, b, h, None)
            gu.assert_parity(out[b, h], ref, "%s b%d h%d" % (name, b, h))


EDGE_CASES = [
    # name, B, H, D, grid, tile, per-head windows (tiles)
    ("p32-d64", 1, 2, 64, (4, 8, 8), (2, 4, 4), [(1, 1, 1), (3, 3, 1)]),
    ("p96-d128", 1, 2, 128, (4, 8, 12), (4, 4, 6), [(1, 3, 3), (1, 2, 2)]),
    ("p64-d128", 2, 2, 128, (2, 16, 16), (1, 8, 8), [(3, 1, 3), (1, 2, 1)]),
    ("p128-d64", 1, 3, 64, (8, 8, 8), (2, 8, 8), [(3, 1, 1), (4, 1, 1), (9, 9, 9)]),
    ("p384-d128-mixed", 2, 3, 128, (6, 16, 24), (6, 8, 8), [(1, 1, 1), (1, 3, 3), (1, 2, 3)]),
    ("single-tile", 1, 1, 64, (6, 8, 8), (6, 8, 8), [(1, 1, 1)]),
    ("p256-d128", 1, 1, 128, (4, 16, 16), (4, 8, 8), [(1, 3, 1)]),
    # head dimension 64 on each of its DMA-staged shapes: 12 waves (P = 384), 4 waves (P = 256), 2 waves (P = 64, 192)
    ("p384-d64-mixed", 1, 3, 64, (6, 16, 24), (6, 8, 8), [(1, 1, 1), (1, 3, 3), (1, 2, 3)]),
    ("p256-d64", 1, 2, 64, (4, 16, 24), (4, 8, 8), [(1, 3, 1), (1, 1, 3)]),
    ("p64-d64-2d", 2, 2, 64, (1, 32, 40), (1, 8, 8), [(1, 3, 3), (1, 5, 2)]),
    ("p192-d64", 1, 2, 64, (6, 8, 16), (3, 8, 8), [(3, 1, 1), (1, 1, 3)]),
]


@pytest.mark.parametrize("name,B,H,D,grid,tile,windows", EDGE_CASES)
def test_attention_parity_edge_shapes(name, B, H, D, grid, tile, windows):
    w = syn.custom(name, B, H, D, grid, tile, windows, "bf16", seed=4242)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for b in range(B):
        for h in range(H):
            ref = gu.oracle_rows(w, q, k, v, b, h, None)
            gu.assert_parity(out[b, h], ref, "%s b%d h%d" % (name, b, h))


def test_attention_many_heads_chunked_launch():
    """More heads than one launch carries in its argument table (256): heads go out in chunks,
    each with its own window; every head must come back right."""
    H = 260
    windows = [((h % 3) + 1, 1, (h % 2) * 2 + 1) for h in range(H)]
    w = syn.custom("manyheads", 1, H, 128, (2, 8, 32), (1, 8, 16), windows, "bf16", seed=77)   # P = 128, 2x1x2 tiles
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for h in list(range(0, H, 37)) + [255, 256, 257, 259]:
        ref = gu.oracle_rows(w, q, k, v, 0, h, None)
        gu.assert_parity(out[0, h], ref, "manyheads h%d" % h)


def test_attention_tile_of_768_tokens():
    """P = 768: two 384-query workgroups share one query tile and must use the same key-tile box."""
    w = syn.custom("p768", 1, 2, 128, (12, 16, 16), (12, 8, 8), [(1, 1, 2), (1, 2, 1)], "bf16", seed=78)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for h in range(2):
        ref = gu.oracle_rows(w, q, k, v, 0, h, None)
        gu.assert_parity(out[0, h], ref, "p768 h%d" % h)


@pytest.mark.parametrize("tile,grid", [((6, 8, 8), (6, 16, 24)), ((2, 8, 8), (4, 16, 16))])
def test_attention_running_max_keeps_growing(tile, grid):
    """Keys are scaled so that the row maximum rises from sub-block to sub-block and from tile to tile
    (and large query norms make the steps big): the rescale path of the online softmax is taken many
    times, late in the loop, not only on the first block.  Both kernel shapes (384- and 128-token tiles)."""
    w = syn.custom("growmax", 1, 2, 128, grid, tile, [(1, 3, 3), (3, 3, 3)], "bf16", seed=79)
    q, k, v = syn.make_qkv(w)
    order = torch.from_numpy(orc.tile_order(w.grid, w.tile))
    ramp_tiled = torch.linspace(0.2, 6.0, w.N)                      # grows along the TILED sequence
    ramp = torch.empty(w.N)
    ramp[order] = ramp_tiled
    k = (k.float() * ramp[None, None, :, None]).to(torch.bfloat16)
    q = (q.float() * 2.0).to(torch.bfloat16)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for h in range(2):
        ref = gu.oracle_rows(w, q, k, v, 0, h, None)
        gu.assert_parity(out[0, h], ref, "growmax h%d" % h)


@pytest.mark.parametrize("tile,grid,D,windows", [
    ((6, 8, 8), (6, 16, 24), 128, [(1, 3, 3), (3, 3, 3)]), ((2, 8, 8), (4, 16, 16), 128, [(1, 3, 3), (3, 3, 3)]),
    ((6, 8, 8), (6, 16, 24), 64, [(1, 3, 3), (3, 3, 3)]), ((2, 8, 8), (4, 16, 16), 64, [(1, 3, 3), (3, 3, 3)]),
    ((1, 8, 8), (1, 32, 32), 64, [(1, 3, 3), (1, 3, 5)])])
def test_attention_scores_outgrow_the_first_offset(tile, grid, D, windows):
    """The first keys of every window give scores near zero, later ones scores of many tens: an exponent offset
    that is set by the first sub-block and then left alone lets the row sums leave the range of fp32 (2^100 and
    beyond).  The kernel has to notice and do such items again with offsets that follow the scores.  Every
    shape of the DMA-staged kernels (384-, 128- and 64-token tiles, head dimension 128 and 64)."""
    w = syn.custom("outgrow", 1, 2, D, grid, tile, windows, "bf16", seed=84)
    q, k, v = syn.make_qkv(w)
    order = torch.from_numpy(orc.tile_order(w.grid, w.tile))
    ramp_tiled = torch.linspace(0.02, 14.0, w.N)                    # grows along the TILED sequence
    ramp = torch.empty(w.N)
    ramp[order] = ramp_tiled
    k = (k.float() * ramp[None, None, :, None]).to(torch.bfloat16)
    q = (q.float() * 2.0).to(torch.bfloat16)
    refs = [gu.oracle_rows(w, q, k, v, 0, h, None) for h in range(2)]
    for workspace in (False, True):       # whole items, and (head dimension 128) items cut into parts along the keys
        out = gu.gpu_chain(w, q, k, v, workspace=workspace).float().numpy()
        assert np.isfinite(out).all()
        for h in range(2):
            gu.assert_parity(out[0, h], refs[h], "outgrow h%d workspace=%s" % (h, workspace))


@pytest.mark.parametrize("tile,grid,D", [((6, 8, 8), (6, 16, 24), 128), ((2, 8, 8), (4, 16, 16), 128), ((6, 8, 8), (6, 16, 24), 64)])
def test_attention_accumulators_outgrow_fp32_before_the_row_sums_do(tile, grid, D):
    """All queries are the all-ones vector; the keys of one tile are 4.875 * ones, all others zero, so that tile's
    scores exceed every other by 55 (2^79 as a factor): row sums stay below the bound at which the kernel repeats
    an item carefully, but with V scaled by 2^50 the unnormalised accumulators pass 2^128.  The kernel has to
    notice that as well.  Attention is linear in V and the scaling is by a power of two, so the result must be
    2^50 times the oracle's result for the unscaled V."""
    w = syn.custom("vhuge", 1, 2, D, grid, tile, [(3, 3, 3), (1, 3, 3)], "bf16", seed=85)
    _, _, v = syn.make_qkv(w)
    order = torch.from_numpy(orc.tile_order(w.grid, w.tile))
    q = torch.ones((1, 2, w.N, D), dtype=torch.bfloat16)
    k = torch.zeros((1, 2, w.N, D), dtype=torch.bfloat16)
    hot_tile = w.n_tiles - 1                                       # last tile in tiled order
    k[:, :, order[hot_tile * w.P:(hot_tile + 1) * w.P], :] = 4.875 * (128.0 / D) ** 0.5     # same score at both head dimensions
    big = (v.float() * 2.0 ** 50).to(torch.bfloat16)
    for workspace in (False, True):
        out = gu.gpu_chain(w, q, k, big, workspace=workspace).float().numpy() * 2.0 ** -50
        assert np.isfinite(out).all()
        for h in range(2):
            ref = gu.oracle_rows(w, q, k, v, 0, h, None)
            gu.assert_parity(out[0, h], ref, "vhuge h%d workspace=%s" % (h, workspace))


def test_attention_large_scores_stay_finite():
    """Scores of a few hundred before scaling: exponent offsets must keep everything finite."""
    w = syn.custom("bigscores", 1, 1, 128, (6, 8, 16), (6, 8, 8), [(1, 1, 3)], "bf16", seed=80)
    q, k, v = syn.make_qkv(w)
    q = (q.float() * 6.0).to(torch.bfloat16)
    k = (k.float() * 6.0).to(torch.bfloat16)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    ref = gu.oracle_rows(w, q, k, v, 0, 0, None)
    gu.assert_parity(out[0, 0], ref, "bigscores")


@pytest.mark.parametrize("tile,grid,D", [((6, 8, 8), (6, 16, 16), 128), ((2, 8, 8), (4, 16, 16), 128), ((6, 8, 8), (6, 8, 16), 64)])
def test_attention_all_scores_far_below_zero(tile, grid, D):
    """Every score of a row is a large negative number (positive queries, negative keys, a few hundred before
    scaling): an exponent offset that starts at zero and is not moved DOWN by the first keys makes every
    probability underflow and the row sum zero.  All three kernel shapes."""
    w = syn.custom("negscores", 1, 2, D, grid, tile, [(1, 1, 2), (1, 2, 2)], "bf16", seed=83)
    q, k, v = syn.make_qkv(w)
    q = (q.float().abs() * 3.0).to(torch.bfloat16)
    k = (-(k.float().abs()) * 3.0).to(torch.bfloat16)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for h in range(2):
        ref = gu.oracle_rows(w, q, k, v, 0, h, None)
        gu.assert_parity(out[0, h], ref, "negscores h%d" % h)


@pytest.mark.parametrize("tile,grid", [((6, 8, 8), (6, 16, 32)), ((2, 8, 8), (4, 16, 16)), ((1, 8, 8), (1, 16, 16))])
def test_forward_is_bit_reproducible(tile, grid):
    """The same call twice gives the same bits (a vector read of a matrix-instruction result issued too
    early once made the rescale decision, and with it the rounding, vary from run to run)."""
    D = 64 if tile[0] == 1 else 128
    w = syn.custom("repro", 1, 3, D, grid, tile, [(1, 1, 1), (1, 2, 3), (3, 3, 3)], "bf16", seed=81)
    q, k, v = syn.make_qkv(w)
    qd, kd, vd = (x.to(DEV) for x in (q, k, v))
    qt, kt, vt = (torch.empty_like(qd) for _ in range(3))
    sta.sta_tile_permute(qd, qt, w.grid, w.tile)
    sta.sta_tile_permute(kd, kt, w.grid, w.tile)
    sta.sta_tile_permute(vd, vt, w.grid, w.tile)
    ws = gu.forward_workspace(w, DEV)
    for workspace in (None, ws):          # without and with work splitting below one query tile
        outs = []
        for _ in range(4):
            o = torch.full_like(qt, float("nan"))
            sta.sta_forward(qt, kt, vt, o, w.grid, w.tile, w.window_tiles, workspace=workspace)
            outs.append(o)
        torch.cuda.synchronize()
        for o in outs[1:]:
            assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16))


@pytest.mark.parametrize("tile,grid,windows", [
    ((6, 8, 8), (12, 24, 32), [(1, 3, 3), (3, 1, 2), (2, 3, 4)]),      # 12-wave kernel, 24 items per head
    ((2, 8, 8), (4, 24, 32), [(2, 3, 4), (3, 3, 3), (2, 2, 2)]),       # 4-wave kernel; >= 8 kept tiles per head
])
def test_split_items_match_whole_items_and_the_oracle(tile, grid, windows):
    """With a workspace the last (here: all) work items are cut along the keys into parts whose partial results
    a second kernel merges; the result must agree with the one-workgroup-per-item run to rounding and with the
    oracle to the usual tolerance.  A workspace that is too small is an error, not a silent fallback."""
    w = syn.custom("split", 1, len(windows), 128, grid, tile, windows, "bf16", seed=4242)
    assert sta.sta_workspace_bytes(w.B, w.H, w.D, w.grid, w.tile) > 0
    q, k, v = syn.make_qkv(w)
    whole = gu.gpu_chain(w, q, k, v, workspace=False).float().numpy()
    split = gu.gpu_chain(w, q, k, v, workspace=True).float().numpy()
    assert np.isfinite(split).all()
    assert np.abs(split - whole).max() <= 2.0 ** -7 * np.abs(whole).max()      # both round the same value to bf16
    assert (split != whole).any(), "the split path was not taken"
    for h in range(w.H):
        ref = gu.oracle_rows(w, q, k, v, 0, h, None)
        gu.assert_parity(split[0, h], ref, "split h%d" % h)
    qd = q.to(DEV)
    small = torch.empty(64, dtype=torch.uint8, device=DEV)
    with pytest.raises(sta.StaError) as e:
        sta.sta_forward(qd, qd, qd, torch.empty_like(qd), w.grid, w.tile, w.window_tiles, workspace=small)
    assert e.value.status == 6


def test_attention_explicit_scale():
    w = syn.custom("scale", 1, 1, 64, (2, 8, 16), (1, 8, 8), [(1, 1, 3)], "bf16", seed=5)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v, scale=0.05).float().numpy()
    ref = gu.oracle_rows(w, q, k, v, 0, 0, None, scale=0.05)
    gu.assert_parity(out[0, 0], ref, "scale")


def test_full_window_equals_dense_attention_on_gpu():
    """Window = whole grid: the STA kernel is plain softmax attention."""
    w = syn.custom("dense", 1, 2, 128, (2, 16, 16), (1, 8, 8), [(2, 2, 2), (9, 9, 9)], "bf16", seed=6)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).double()
    for h in range(2):
        s = (q[0, h].double() @ k[0, h].double().T) / np.sqrt(128.0)
        ref = torch.softmax(s, dim=-1) @ v[0, h].double()
        gu.assert_parity(out[0, h].numpy(), ref.numpy(), "dense h%d" % h)


@pytest.mark.parametrize("D,grid,tile,workspace", [
    (64, (4, 16, 16), (2, 4, 4), False),           # general kernel (32-token tiles), ascending walk
    (64, (12, 24, 32), (6, 8, 8), False),          # 12-wave kernel at head dimension 64
    (64, (1, 40, 48), (1, 8, 8), False),           # 2-wave kernel (64-token tiles), 30 tiles
    (128, (12, 24, 32), (6, 8, 8), False),         # 12-wave kernel: residue-order walk of the box
    (128, (12, 24, 32), (6, 8, 8), True),          # ... with items split along the keys
    (128, (4, 24, 32), (2, 8, 8), False),          # 4-wave kernel
    (128, (4, 24, 32), (2, 8, 8), True),
    (128, (6, 40, 48), (6, 8, 8), False),          # 1x5x6 = 30 tiles: boxes that wrap along two axes
])
def test_kept_set_read_from_gpu_output(D, grid, tile, workspace):
    """Q = 0 and V = one-hot(tile id): O[i, tau] = [tau kept] / kept(q tile), which reads the
    kept set and its size straight out of the kernel's output, for every kernel that walks the box."""
    windows = [(1, 3, 3), (3, 1, 2), (1, 1, 1), (2, 3, 4), (1, 5, 3), (3, 9, 9)]
    w = syn.custom("onehot", 1, len(windows), D, grid, tile, windows, "bf16", seed=11)
    assert w.n_tiles <= D
    n = w.n_tiles
    order = orc.tile_order(grid, tile)
    tile_of_raster = np.empty(w.N, dtype=np.int64)
    tile_of_raster[order] = np.repeat(np.arange(n), w.P)
    q = torch.zeros((1, w.H, w.N, w.D), dtype=torch.bfloat16)
    _, k, _ = syn.make_qkv(w)
    v = torch.zeros((1, w.H, w.N, w.D), dtype=torch.bfloat16)
    v[0, :, torch.arange(w.N), torch.from_numpy(tile_of_raster)] = 1.0
    out = gu.gpu_chain(w, q, k, v, workspace=workspace).float().numpy()
    for h, wt in enumerate(windows):
        counts, lists = orc.key_tiles(grid, tile, orc.window_tiles_to_tokens(wt, tile))
        for qt in range(n):
            rows = out[0, h, order[qt * w.P:(qt + 1) * w.P]]
            kept = lists[qt, :counts[qt]]
            expect = np.zeros(w.D)
            expect[kept] = 1.0 / counts[qt]
            mask = expect > 0
            assert (rows[:, ~mask] == 0).all(), (h, qt)
            np.testing.assert_allclose(rows[:, mask], np.broadcast_to(expect[mask], rows[:, mask].shape),
                                       rtol=2.0 ** -7, atol=0)


def test_constant_v_gives_constant_output():
    w = syn.custom("constv", 1, 1, 128, (6, 16, 16), (6, 8, 8), [(1, 3, 3)], "bf16", seed=12)
    q, k, _ = syn.make_qkv(w)
    row = torch.linspace(-2, 2, 128).to(torch.bfloat16)
    v = row.expand(1, 1, w.N, 128).contiguous()
    out = gu.gpu_chain(w, q, k, v)
    assert (out.float() - row.float()).abs().max().item() <= 2.0 ** -7 * 2


# --------------------------------------------------------------------------
# Attention: sampled parity at the larger configurations
# --------------------------------------------------------------------------
def test_attention_parity_c3_sampled():
    w = syn.workload("C3")
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    tiles = gu.border_and_interior_tiles(w)
    for h in range(w.H):
        idx = gu.stratified_query_sample(w, 128, tiles[h % len(tiles):h % len(tiles) + 1], seed=100 + h)
        ref = gu.oracle_rows(w, q, k, v, 0, h, idx)
        gu.assert_parity(out[0, h, idx], ref, "C3 h%d" % h)


def _sampled_full_size(name, n_random, heads_with_full_tile, heads=None, rows_per_stratum=16, strata_per_head=3):
    """Full-size run in the launch configuration the benchmark times (workspace given, so the last round of work
    items is split).  Every head is checked on n_random random rows plus rows_per_stratum rows of each of
    strata_per_head query tiles taken in turn from the strata of the tile grid: the 8 corners, one tile per
    edge and face class, interior tiles."""
    w = syn.workload(name)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    assert np.isfinite(out).all()
    strata = gu.strata_tiles(w)
    order = orc.tile_order(w.grid, w.tile)
    stats, used = [], set()
    head_list = list(heads if heads is not None else range(w.H))
    for i, h in enumerate(head_list):
        rng = np.random.default_rng(300 + h)
        idx = [rng.integers(0, w.N, size=n_random)]
        for j in range(strata_per_head):
            t = strata[(i * strata_per_head + j) % len(strata)]
            used.add(t)
            rows = order[t * w.P:(t + 1) * w.P]
            idx.append(rows if h in heads_with_full_tile and j == 0 else rng.choice(rows, size=rows_per_stratum, replace=False))
        idx = np.unique(np.concatenate(idx)).astype(np.int64)
        ref = gu.oracle_rows(w, q, k, v, 0, h, idx)
        stats.append(gu.assert_parity(out[0, h, idx], ref, "%s h%d" % (name, h)))
    assert len(used) == min(len(strata), len(head_list) * strata_per_head)
    return stats


def test_attention_parity_c4_sampled():
    """HunyuanVideo-shaped layer, 3x3x3 window: 24 heads x 3 strata tiles cover all 8 corners, the edge and face
    classes and the interior tiles of the 5x6x10 tile grid."""
    _sampled_full_size("C4", n_random=16, heads_with_full_tile={0, 13})


def test_attention_parity_c5_mixed_windows_sampled():
    _sampled_full_size("C5", n_random=8, heads_with_full_tile=set(), rows_per_stratum=8)


def test_attention_parity_head_dimension_64_full_size_sampled():
    """The headline grid, tile and window at head dimension 64 (the 12-wave instance of the other attention kernel)."""
    _sampled_full_size("D64-3D", n_random=8, heads_with_full_tile=set(), heads=[0, 9, 17, 23], rows_per_stratum=8)


def test_attention_parity_c4_dense_sampled():
    _sampled_full_size("C4dense", n_random=16, heads_with_full_tile=set(), heads=[0, 7, 23], rows_per_stratum=16)


def test_many_batch_entries_take_the_head_chunk_limit():
    """B = 300: the number of heads per launch is cut to 65535 / B (the limit of the general kernel's grid, applied
    to every kernel), so the two heads go out in separate launches."""
    w = syn.custom("manybatch", 300, 2, 64, (1, 8, 16), (1, 8, 8), [(1, 1, 1), (1, 1, 3)], "bf16", seed=77)
    q, k, v = syn.make_qkv(w)
    out = gu.gpu_chain(w, q, k, v).float().numpy()
    for b in (0, 151, 299):
        for h in range(w.H):
            ref = gu.oracle_rows(w, q, k, v, b, h, None)
            gu.assert_parity(out[b, h], ref, "manybatch b%d h%d" % (b, h))


# --------------------------------------------------------------------------
# Error paths with real device buffers
# --------------------------------------------------------------------------
def test_errors_with_device_buffers():
    x = torch.zeros((1, 1, 64, 64), dtype=torch.bfloat16, device=DEV)
    y = torch.zeros_like(x)
    with pytest.raises(sta.StaError) as e:
        sta.sta_tile_permute(x, x, (1, 8, 8), (1, 8, 8))
    assert e.value.status == 5
    with pytest.raises(sta.StaError) as e:
        sta.sta_forward(x, x, x, x, (1, 8, 8), (1, 8, 8), [(1, 1, 1)])
    assert e.value.status == 5
    with pytest.raises(sta.StaError) as e:
        sta.sta_forward(x, x, x, y, (1, 8, 8), (1, 8, 8), [(1, 0, 1)])
    assert e.value.status == 3
    with pytest.raises(sta.StaError) as e:
        sta.sta_forward(x, x, x, y, (1, 8, 8), (1, 4, 4), [(1, 1, 1)])      # P = 16
    assert e.value.status == 4
    torch.cuda.synchronize()


# --------------------------------------------------------------------------
# A seeded sweep over shapes: every kernel instance, borders, windows of all kinds
# --------------------------------------------------------------------------
def _random_shapes(n_cases, seed):
    rng = np.random.default_rng(seed)
    tiles = [(6, 8, 8), (2, 8, 8), (1, 8, 8), (4, 4, 8), (2, 4, 4), (3, 8, 8), (1, 4, 8), (2, 6, 8)]
    cases = []
    while len(cases) < n_cases:
        tile = tiles[rng.integers(len(tiles))]
        n = tuple(int(rng.integers(1, 5)) for _ in range(3))
        grid = tuple(n[a] * tile[a] for a in range(3))
        N = grid[0] * grid[1] * grid[2]
        if N > 4608 or (tile[0] * tile[1] * tile[2]) % 32 != 0:
            continue
        D = int(rng.choice([64, 128]))
        H = int(rng.integers(1, 4))
        B = int(rng.integers(1, 3))
        windows = [tuple(int(rng.integers(1, 2 * n[a] + 2)) for a in range(3)) for _ in range(H)]
        cases.append((B, H, D, grid, tile, windows))
    return cases


@pytest.mark.parametrize("case", _random_shapes(24, seed=20250207), ids=lambda c: "B%d-H%d-D%d-g%s-t%s" % (c[0], c[1], c[2], "x".join(map(str, c[3])), "x".join(map(str, c[4]))))
def test_attention_parity_seeded_shape_sweep(case):
    B, H, D, grid, tile, windows = case
    w = syn.custom("sweep", B, H, D, grid, tile, windows, "bf16", seed=hash((grid, tile, D)) % 100000)
    q, k, v = syn.make_qkv(w)
    for workspace in (False, True):
        out = gu.gpu_chain(w, q, k, v, workspace=workspace).float().numpy()
        assert np.isfinite(out).all()
        for b in range(B):
            for h in range(H):
                gu.assert_parity(out[b, h], gu.oracle_rows(w, q, k, v, b, h, None), "sweep %s b%d h%d" % (case, b, h))
