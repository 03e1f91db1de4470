"""ctypes binding of the C oracle (oracle/sta_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  It never imports the HIP package and the HIP
package never imports it.  All windows here are in TOKENS, as the paper's
mask algorithm takes them ("kernel size"); `window_tiles_to_tokens` converts
from the tile units the GPU boundary uses.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsta_oracle.so")
_lib = None

_I3 = ctypes.c_int * 3


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build_oracle  # local build step: gcc only
        build_oracle.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    c_long, c_int, c_double, c_void = ctypes.c_long, ctypes.c_int, ctypes.c_double, ctypes.c_void_p
    lib.sta_oracle_keep.argtypes = [_I3, _I3, _I3, _I3, _I3]
    lib.sta_oracle_keep.restype = c_int
    lib.sta_oracle_attention.argtypes = [c_void, c_void, c_void, c_int, _I3, _I3, _I3, c_double,
                                         c_void, c_long, c_void]
    lib.sta_oracle_attention.restype = c_int
    lib.sta_oracle_attention_lse.argtypes = [c_void, c_void, c_void, c_int, _I3, _I3, _I3, c_double,
                                             c_void, c_long, c_void, c_void]
    lib.sta_oracle_attention_lse.restype = c_int
    lib.sta_oracle_probs.argtypes = [c_void, c_void, c_int, _I3, _I3, _I3, c_double, c_long,
                                     c_void, c_void]
    lib.sta_oracle_probs.restype = c_int
    lib.sta_oracle_tile_order.argtypes = [_I3, _I3, c_void]
    lib.sta_oracle_tile_order.restype = c_int
    for name in ("sta_oracle_tile_permute", "sta_oracle_untile"):
        fn = getattr(lib, name)
        fn.argtypes = [c_void, c_void, c_long, c_long, _I3, _I3]
        fn.restype = c_int
    lib.sta_oracle_key_tiles.argtypes = [_I3, _I3, _I3, c_void, c_void]
    lib.sta_oracle_key_tiles.restype = c_int
    lib.sta_oracle_block_census.argtypes = [_I3, _I3, _I3, c_void, c_void, c_void]
    lib.sta_oracle_block_census.restype = c_int
    lib.sta_oracle_natten_keep.argtypes = [_I3, _I3, _I3, _I3]
    lib.sta_oracle_natten_keep.restype = c_int
    lib.sta_oracle_block_census_per_query.argtypes = [c_int, c_int, _I3, _I3, _I3, c_void, c_void]
    lib.sta_oracle_block_census_per_query.restype = c_int
    lib.sta_oracle_num_threads.argtypes = []
    lib.sta_oracle_attention_backward.argtypes = [c_void, c_void, c_void, c_void, c_int, _I3, _I3, _I3, c_double,
                                                  c_void, c_long, c_void, c_long, c_void, c_void, c_void]
    lib.sta_oracle_attention_backward.restype = c_int
    lib.sta_oracle_num_threads.restype = c_int
    _lib = lib
    return lib


def _i3(x):
    x = [int(v) for v in x]
    assert len(x) == 3
    return _I3(*x)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def window_tiles_to_tokens(window_tiles, tile):
    """Window in tiles -> window in tokens (the algorithm's kernel size)."""
    return [int(w) * int(t) for w, t in zip(window_tiles, tile)]


def num_threads() -> int:
    return int(_load().sta_oracle_num_threads())


def keep(q, k, grid, window_tokens, tile) -> bool:
    """Mask predicate for one (query token, key token) pair of coordinates."""
    return bool(_load().sta_oracle_keep(_i3(q), _i3(k), _i3(grid), _i3(window_tokens), _i3(tile)))


def attention(q, k, v, grid, tile, window_tokens, scale=None, query_idx=None, return_lse=False):
    """Masked attention (Eq. 1) of ONE head in raster order.

    q, k, v: [N, d] arrays (any float type; values are taken exactly as fp32).
    query_idx: raster indices to evaluate (default: all).  Returns [nq, d] fp64, and with
    return_lse also [nq] fp64: the natural log of each row's softmax denominator.
    """
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    N, d = q.shape
    assert N == int(grid[0]) * int(grid[1]) * int(grid[2]) and k.shape == (N, d) and v.shape == (N, d)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    if query_idx is None:
        query_idx = np.arange(N, dtype=np.int64)
    query_idx = np.ascontiguousarray(query_idx, dtype=np.int64)
    assert query_idx.ndim == 1 and (query_idx >= 0).all() and (query_idx < N).all()
    out = np.empty((query_idx.shape[0], d), dtype=np.float64)
    lse = np.empty(query_idx.shape[0], dtype=np.float64)
    rc = lib.sta_oracle_attention_lse(q.ctypes.data, k.ctypes.data, v.ctypes.data, d, _i3(grid), _i3(tile),
                                      _i3(window_tokens), float(scale), query_idx.ctypes.data,
                                      query_idx.shape[0], out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise MemoryError("oracle attention failed")
    return (out, lse) if return_lse else out


def attention_backward(q, k, v, g, grid, tile, window_tokens, scale=None, query_idx=None, key_idx=None):
    """Gradients of masked attention (Eq. 1) of ONE head with respect to q, k, v, given g = dLoss/dO.

    q, k, v, g: [N, d] in raster order.  query_idx / key_idx: raster rows of dq / of dk and dv to return
    (default: all).  Returns (dq [nq, d], dk [nk, d], dv [nk, d]) in fp64."""
    lib = _load()
    q, k, v, g = _f32(q), _f32(k), _f32(v), _f32(g)
    N, d = q.shape
    assert N == int(grid[0]) * int(grid[1]) * int(grid[2])
    assert k.shape == (N, d) and v.shape == (N, d) and g.shape == (N, d)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    if query_idx is None:
        query_idx = np.arange(N, dtype=np.int64)
    if key_idx is None:
        key_idx = np.arange(N, dtype=np.int64)
    query_idx = np.ascontiguousarray(query_idx, dtype=np.int64)
    key_idx = np.ascontiguousarray(key_idx, dtype=np.int64)
    for idx in (query_idx, key_idx):
        assert idx.ndim == 1 and (idx >= 0).all() and (idx < N).all()
    dq = np.empty((query_idx.shape[0], d), dtype=np.float64)
    dk = np.empty((key_idx.shape[0], d), dtype=np.float64)
    dv = np.empty((key_idx.shape[0], d), dtype=np.float64)
    rc = lib.sta_oracle_attention_backward(q.ctypes.data, k.ctypes.data, v.ctypes.data, g.ctypes.data, d,
                                           _i3(grid), _i3(tile), _i3(window_tokens), float(scale),
                                           query_idx.ctypes.data, query_idx.shape[0], key_idx.ctypes.data,
                                           key_idx.shape[0], dq.ctypes.data, dk.ctypes.data, dv.ctypes.data)
    if rc != 0:
        raise MemoryError("oracle backward failed")
    return dq, dk, dv


def attention_bh(q, k, v, grid, tile, window_tokens_per_head, scale=None, query_idx=None):
    """[B, H, N, d] inputs, per-head windows (tokens) -> [B, H, nq, d] fp64."""
    B, H = q.shape[0], q.shape[1]
    outs = []
    for b in range(B):
        row = []
        for h in range(H):
            row.append(attention(q[b, h], k[b, h], v[b, h], grid, tile, window_tokens_per_head[h],
                                 scale=scale, query_idx=query_idx))
        outs.append(np.stack(row))
    return np.stack(outs)


def probs(q, k, grid, tile, window_tokens, i, scale=None):
    """Row i of A = softmax(S + M) over all N keys, and its sum."""
    lib = _load()
    q, k = _f32(q), _f32(k)
    N, d = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    p = np.empty(N, dtype=np.float64)
    s = ctypes.c_double(0.0)
    lib.sta_oracle_probs(q.ctypes.data, k.ctypes.data, d, _i3(grid), _i3(tile), _i3(window_tokens),
                         float(scale), int(i), p.ctypes.data, ctypes.addressof(s))
    return p, float(s.value)


def tile_order(grid, tile):
    """order[slot] = raster index of the token stored at tiled slot."""
    lib = _load()
    N = int(grid[0]) * int(grid[1]) * int(grid[2])
    order = np.empty(N, dtype=np.int64)
    if lib.sta_oracle_tile_order(_i3(grid), _i3(tile), order.ctypes.data) != 0:
        raise ValueError("grid is not a multiple of tile")
    return order


def _permute(fn_name, x, grid, tile):
    lib = _load()
    x = np.ascontiguousarray(x)
    N = int(grid[0]) * int(grid[1]) * int(grid[2])
    assert x.ndim >= 2 and x.shape[-2] == N, "expect [..., N, d]"
    row_bytes = x.shape[-1] * x.dtype.itemsize
    outer = int(np.prod(x.shape[:-2])) if x.ndim > 2 else 1
    out = np.empty_like(x)
    rc = getattr(lib, fn_name)(x.ctypes.data, out.ctypes.data, outer, row_bytes, _i3(grid), _i3(tile))
    if rc != 0:
        raise ValueError("grid is not a multiple of tile")
    return out


def tile_permute(x, grid, tile):
    """Raster [..., N, d] -> tile-contiguous [..., N, d] (whole rows move)."""
    return _permute("sta_oracle_tile_permute", x, grid, tile)


def untile(x, grid, tile):
    """Inverse of tile_permute."""
    return _permute("sta_oracle_untile", x, grid, tile)


def key_tiles(grid, tile, window_tokens):
    """(counts[n], lists[n][n]) from the collapsed token predicate; -1 padded."""
    lib = _load()
    n = (int(grid[0]) // int(tile[0])) * (int(grid[1]) // int(tile[1])) * (int(grid[2]) // int(tile[2]))
    counts = np.empty(n, dtype=np.int32)
    lists = np.empty((n, n), dtype=np.int32)
    if lib.sta_oracle_key_tiles(_i3(grid), _i3(tile), _i3(window_tokens), counts.ctypes.data,
                                lists.ctypes.data) != 0:
        raise ValueError("grid is not a multiple of tile")
    return counts, lists


def block_census(grid, tile, window_tokens):
    """(dense, mixed, empty) block counts by brute force over all token pairs."""
    lib = _load()
    vals = [ctypes.c_int64(0) for _ in range(3)]
    if lib.sta_oracle_block_census(_i3(grid), _i3(tile), _i3(window_tokens),
                                   *[ctypes.addressof(v) for v in vals]) != 0:
        raise ValueError("grid is not a multiple of tile")
    return tuple(int(v.value) for v in vals)


def natten_keep(q, k, grid, window_tokens):
    """Sliding-window predicate for one (query token, key token) pair, coordinates (t, h, w)
    (appendix algorithm "Mask Definition of 3D NATTEN")."""
    return bool(_load().sta_oracle_natten_keep(_i3(q), _i3(k), _i3(grid), _i3(window_tokens)))


def block_census_per_query(mask, order, grid, tile, window_tokens):
    """(dense[nb], mixed[nb]) per query block by brute force over all token pairs.
    mask: "sta" or "natten"; order: "tiled" (block = tile) or "raster" (block = P consecutive raster tokens)."""
    lib = _load()
    P = int(tile[0]) * int(tile[1]) * int(tile[2])
    nb = (int(grid[0]) * int(grid[1]) * int(grid[2])) // P
    dense = np.empty(nb, dtype=np.int64)
    mixed = np.empty(nb, dtype=np.int64)
    rc = lib.sta_oracle_block_census_per_query({"sta": 0, "natten": 1}[mask], {"raster": 0, "tiled": 1}[order],
                                               _i3(grid), _i3(tile), _i3(window_tokens), dense.ctypes.data,
                                               mixed.ctypes.data)
    if rc != 0:
        raise ValueError("grid is not a multiple of the block shape")
    return dense, mixed


def head_mse(o_ref, o_other):
    """MSE(O, O') per head over batch, tokens and channels ("STA Mask Search": loss <- MSE(O, O')).
    o_*: [B, H, n, d] arrays; returns [H] fp64."""
    a = np.asarray(o_ref, dtype=np.float64)
    b = np.asarray(o_other, dtype=np.float64)
    diff = a - b
    return (diff * diff).mean(axis=(0, 2, 3))


def mask_search(q, k, v, grid, tile, patterns_tokens, scale=None, query_idx=None):
    """Inner loop of the paper's mask-search algorithm for one layer: O <- original (full) attention output;
    for each pattern p in list order: O' <- output with window p, loss <- MSE(O, O'); a pattern replaces the
    best one only if its loss is strictly smaller.  q, k, v: [B, H, N, d].  Returns (losses [n_p, H], best [H]).
    query_idx restricts the MSE to a sample of query rows (same rows for every pattern)."""
    B, H = q.shape[0], q.shape[1]
    full = [list(grid)] * H
    o = attention_bh(q, k, v, grid, tile, full, scale=scale, query_idx=query_idx)
    losses = np.empty((len(patterns_tokens), H), dtype=np.float64)
    best = np.full(H, -1, dtype=np.int64)
    minimum = np.full(H, np.inf)
    for p, pat in enumerate(patterns_tokens):
        o_p = attention_bh(q, k, v, grid, tile, [list(pat)] * H, scale=scale, query_idx=query_idx)
        losses[p] = head_mse(o, o_p)
        for h in range(H):
            if losses[p, h] < minimum[h]:
                minimum[h] = losses[p, h]
                best[h] = p
    return losses, best
