"""ctypes binding of libsta.so.  Same names as the C entry points.

Tensors are torch tensors used purely as device-memory handles (data_ptr);
the stream is torch's current HIP stream unless one is given.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

STA_BF16, STA_F32 = 0, 1
STA_MASK_STA, STA_MASK_NATTEN = 0, 1
_I3 = ctypes.c_int * 3

EXPORTED_SYMBOLS = (
    "sta_tile_permute", "sta_untile", "sta_forward", "sta_forward_lse", "sta_workspace_bytes", "sta_key_tile_box",
    "sta_dump_key_tiles", "sta_window_tokens_to_tiles", "sta_kept_flops", "sta_strerror", "sta_version",
    "sta_head_mse_workspace_bytes", "sta_head_mse", "sta_mask_search", "sta_attention_recall", "sta_block_census", "sta_forward_general",
    "sta_backward_workspace_bytes", "sta_backward", "sta_query_tile_box", "sta_head_mse_static",
)


class StaError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("sta status %d: %s" % (status, message))
        self.status = status


def lib_path() -> str:
    return os.path.join(_HERE, "libsta.so")


def load_library():
    """Load libsta.so; raises if it has not been built (no fallback exists)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError("libsta.so is not built: run `python -m paper_2502_04507_amd.build_lib` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(path)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    for name in ("sta_tile_permute", "sta_untile"):
        fn = getattr(lib, name)
        fn.argtypes = [vp, vp, ci, ci, ci, ci, ci, _I3, _I3, vp]
        fn.restype = ci
    lib.sta_forward.argtypes = [vp, vp, vp, vp, ci, ci, ci, _I3, _I3, ctypes.POINTER(ci), cf, vp,
                                ctypes.c_size_t, vp]
    lib.sta_forward.restype = ci
    lib.sta_forward_lse.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, _I3, _I3, ctypes.POINTER(ci), cf, vp]
    lib.sta_forward_lse.restype = ci
    lib.sta_forward_general.argtypes = [vp, vp, vp, vp, ci, ci, ci, _I3, _I3, ci, ctypes.POINTER(ci), cf, vp]
    lib.sta_forward_general.restype = ci
    lib.sta_head_mse_workspace_bytes.argtypes = [ci, ci]
    lib.sta_head_mse_workspace_bytes.restype = ctypes.c_size_t
    lib.sta_head_mse.argtypes = [vp, vp, ci, ci, ci, _I3, vp, ctypes.c_size_t, vp, vp]
    lib.sta_head_mse.restype = ci
    lib.sta_head_mse_static.argtypes = [vp, vp, ci, ci, ci, _I3, vp, vp]
    lib.sta_head_mse_static.restype = ci
    lib.sta_mask_search.argtypes = [vp, vp, vp, ci, ci, ci, _I3, _I3, ctypes.POINTER(ci), ci, cf, vp, vp, vp,
                                    ctypes.c_size_t, vp, vp, vp]
    lib.sta_mask_search.restype = ci
    lib.sta_attention_recall.argtypes = [vp, vp, ci, ci, _I3, vp, ctypes.c_size_t, vp, vp, vp]
    lib.sta_attention_recall.restype = ci
    lib.sta_workspace_bytes.argtypes = [ci, ci, ci, _I3, _I3]
    lib.sta_workspace_bytes.restype = ctypes.c_size_t
    lib.sta_key_tile_box.argtypes = [_I3, _I3, _I3, _I3, _I3]
    lib.sta_key_tile_box.restype = ci
    lib.sta_dump_key_tiles.argtypes = [ci, _I3, _I3, ctypes.POINTER(ci), vp, vp, vp]
    lib.sta_dump_key_tiles.restype = ci
    lib.sta_window_tokens_to_tiles.argtypes = [_I3, _I3, _I3]
    lib.sta_window_tokens_to_tiles.restype = ci
    lib.sta_kept_flops.argtypes = [ci, ci, ci, _I3, _I3, ctypes.POINTER(ci)]
    lib.sta_kept_flops.restype = ctypes.c_double
    vp = ctypes.c_void_p
    lib.sta_backward_workspace_bytes.argtypes = [ci, ci, _I3]
    lib.sta_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.sta_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, _I3, _I3, ctypes.POINTER(ci),
                                 ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.sta_backward.restype = ci
    lib.sta_query_tile_box.argtypes = [_I3, _I3, _I3, _I3, _I3]
    lib.sta_query_tile_box.restype = ci
    lib.sta_block_census.argtypes = [ci, _I3, _I3, _I3, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.sta_block_census.restype = ci
    lib.sta_strerror.argtypes = [ci]
    lib.sta_strerror.restype = ctypes.c_char_p
    lib.sta_version.argtypes = []
    lib.sta_version.restype = ci
    _LIB = lib
    return lib


def sta_strerror(status: int) -> str:
    return load_library().sta_strerror(int(status)).decode()


def sta_version() -> int:
    return int(load_library().sta_version())


def _check(status):
    if status != 0:
        raise StaError(status, sta_strerror(status))


def _i3(x):
    x = [int(v) for v in x]
    if len(x) != 3:
        raise ValueError("expected 3 entries")
    return _I3(*x)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return STA_BF16
    if t.dtype == torch.float32:
        return STA_F32
    raise TypeError("only bfloat16 and float32 tensors are supported")


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t: torch.Tensor, name: str):
    if not t.is_cuda:
        raise ValueError("%s must live in device memory" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return ctypes.c_void_p(t.data_ptr())


def _windows(window_tiles, H):
    flat = [int(x) for w in window_tiles for x in w]
    if len(flat) != 3 * H:
        raise ValueError("window_tiles must have H entries of 3")
    return (ctypes.c_int * (3 * H))(*flat)


def _permute(fn_name, src, dst, grid, tile, stream):
    lib = load_library()
    if src.dim() != 4 or dst.shape != src.shape:
        raise ValueError("expect [B, H, N, D] tensors of equal shape")
    B, H, N, D = src.shape
    if N != int(grid[0]) * int(grid[1]) * int(grid[2]):
        raise ValueError("N does not match the grid")
    _check(getattr(lib, fn_name)(_dev(src, "src"), _dev(dst, "dst"), _dt(src), _dt(dst), B, H, D, _i3(grid),
                                 _i3(tile), _stream_ptr(stream)))
    return dst


def sta_tile_permute(src, dst, grid, tile, stream=None):
    """Raster [B,H,N,D] -> tiled [B,H,N,D] (dst preallocated; dtype may differ: fused cast)."""
    return _permute("sta_tile_permute", src, dst, grid, tile, stream)


def sta_untile(src, dst, grid, tile, stream=None):
    """Tiled -> raster."""
    return _permute("sta_untile", src, dst, grid, tile, stream)


def sta_workspace_bytes(B, H, D, grid, tile) -> int:
    return int(load_library().sta_workspace_bytes(B, H, D, _i3(grid), _i3(tile)))


def sta_forward(q_tiled, k_tiled, v_tiled, o_tiled, grid, tile, window_tiles, scale=0.0, workspace=None,
                stream=None):
    """STA forward on tiled bf16 [B,H,N,D] tensors; window_tiles: H entries of (t,h,w) in tiles."""
    lib = load_library()
    for t in (q_tiled, k_tiled, v_tiled, o_tiled):
        if t.dim() != 4 or t.shape != q_tiled.shape or t.dtype != torch.bfloat16:
            raise ValueError("expect four bf16 [B, H, N, D] tensors of equal shape")
    B, H, N, D = q_tiled.shape
    if N != int(grid[0]) * int(grid[1]) * int(grid[2]):
        raise ValueError("N does not match the grid")
    ws_ptr, ws_bytes = ctypes.c_void_p(0), 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev(workspace, "workspace"), workspace.numel() * workspace.element_size()
    _check(lib.sta_forward(_dev(q_tiled, "q"), _dev(k_tiled, "k"), _dev(v_tiled, "v"), _dev(o_tiled, "o"), B, H, D,
                           _i3(grid), _i3(tile), _windows(window_tiles, H), float(scale), ws_ptr, ws_bytes,
                           _stream_ptr(stream)))
    return o_tiled


def sta_forward_general(q_tiled, k_tiled, v_tiled, o_tiled, grid, tile, mask_kind, window, scale=0.0, stream=None):
    """Attention through the general kernel: mask_kind STA_MASK_STA (window: H entries of (t,h,w) in tiles) or
    STA_MASK_NATTEN (token-granular sliding window; window: H entries of (t,h,w) in tokens)."""
    lib = load_library()
    for t in (q_tiled, k_tiled, v_tiled, o_tiled):
        if t.dim() != 4 or t.shape != q_tiled.shape or t.dtype != torch.bfloat16:
            raise ValueError("expect four bf16 [B, H, N, D] tensors of equal shape")
    B, H, N, D = q_tiled.shape
    if N != int(grid[0]) * int(grid[1]) * int(grid[2]):
        raise ValueError("N does not match the grid")
    _check(lib.sta_forward_general(_dev(q_tiled, "q"), _dev(k_tiled, "k"), _dev(v_tiled, "v"), _dev(o_tiled, "o"), B, H,
                                   D, _i3(grid), _i3(tile), int(mask_kind), _windows(window, H), float(scale),
                                   _stream_ptr(stream)))
    return o_tiled


def sta_forward_lse(q_tiled, k_tiled, v_tiled, o_tiled, lse_tiled, grid, tile, window_tiles, scale=0.0, stream=None):
    """sta_forward that also writes lse_tiled (float32 [B,H,N], tiled order): ln of each row's softmax denominator."""
    lib = load_library()
    for t in (q_tiled, k_tiled, v_tiled, o_tiled):
        if t.dim() != 4 or t.shape != q_tiled.shape or t.dtype != torch.bfloat16:
            raise ValueError("expect four bf16 [B, H, N, D] tensors of equal shape")
    B, H, N, D = q_tiled.shape
    if lse_tiled.dtype != torch.float32 or tuple(lse_tiled.shape) != (B, H, N):
        raise ValueError("lse_tiled must be float32 [B, H, N]")
    if N != int(grid[0]) * int(grid[1]) * int(grid[2]):
        raise ValueError("N does not match the grid")
    _check(lib.sta_forward_lse(_dev(q_tiled, "q"), _dev(k_tiled, "k"), _dev(v_tiled, "v"), _dev(o_tiled, "o"),
                               _dev(lse_tiled, "lse"), B, H, D, _i3(grid), _i3(tile), _windows(window_tiles, H),
                               float(scale), _stream_ptr(stream)))
    return o_tiled, lse_tiled


def sta_backward_workspace_bytes(B, H, grid) -> int:
    return int(load_library().sta_backward_workspace_bytes(int(B), int(H), _i3(grid)))


def sta_backward(q_tiled, k_tiled, v_tiled, o_tiled, d_o_tiled, lse_tiled, d_q_tiled, d_k_tiled, d_v_tiled, grid, tile,
                 window_tiles, workspace, scale=0.0, stream=None):
    """Gradients of sta_forward.  All tensors bf16 [B,H,N,D] in tiled order except lse_tiled (float32 [B,H,N]) and
    workspace (any dtype, at least sta_backward_workspace_bytes bytes)."""
    lib = load_library()
    for t in (q_tiled, k_tiled, v_tiled, o_tiled, d_o_tiled, d_q_tiled, d_k_tiled, d_v_tiled):
        if t.dim() != 4 or t.shape != q_tiled.shape or t.dtype != torch.bfloat16:
            raise ValueError("expect bf16 [B, H, N, D] tensors of equal shape")
    B, H, N, D = q_tiled.shape
    if lse_tiled.dtype != torch.float32 or tuple(lse_tiled.shape) != (B, H, N):
        raise ValueError("lse_tiled must be float32 [B, H, N]")
    if N != int(grid[0]) * int(grid[1]) * int(grid[2]):
        raise ValueError("N does not match the grid")
    _check(lib.sta_backward(_dev(q_tiled, "q"), _dev(k_tiled, "k"), _dev(v_tiled, "v"), _dev(o_tiled, "o"),
                            _dev(d_o_tiled, "d_o"), _dev(lse_tiled, "lse"), _dev(d_q_tiled, "d_q"),
                            _dev(d_k_tiled, "d_k"), _dev(d_v_tiled, "d_v"), B, H, D, _i3(grid), _i3(tile),
                            _windows(window_tiles, H), float(scale), _dev(workspace, "workspace"),
                            workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
    return d_q_tiled, d_k_tiled, d_v_tiled


def sta_query_tile_box(grid_tiles, window_tiles, k_tile):
    """Host-side, pure integer: inclusive (lo, hi) box of the query tiles that keep key tile k_tile."""
    lo, hi = _I3(), _I3()
    _check(load_library().sta_query_tile_box(_i3(grid_tiles), _i3(window_tiles), _i3(k_tile), lo, hi))
    return tuple(lo), tuple(hi)


def sta_key_tile_box(grid_tiles, window_tiles, q_tile):
    """Host-side, pure integer: inclusive (lo, hi) box of kept key tiles."""
    lo, hi = _I3(), _I3()
    _check(load_library().sta_key_tile_box(_i3(grid_tiles), _i3(window_tiles), _i3(q_tile), lo, hi))
    return tuple(lo), tuple(hi)


def sta_dump_key_tiles(H, grid, tile, window_tiles, counts, lists, stream=None):
    """Test hook: device-computed key-tile lists into int32 tensors counts[H,n], lists[H,n,n]."""
    if counts.dtype != torch.int32 or lists.dtype != torch.int32:
        raise TypeError("counts and lists must be int32")
    n = 1
    for g, t in zip(grid, tile):
        n *= int(g) // int(t)
    if counts.numel() != H * n or lists.numel() != H * n * n:
        raise ValueError("counts must be [H,n] and lists [H,n,n]")
    _check(load_library().sta_dump_key_tiles(H, _i3(grid), _i3(tile), _windows(window_tiles, H),
                                             _dev(counts, "counts"), _dev(lists, "lists"), _stream_ptr(stream)))
    return counts, lists


def sta_window_tokens_to_tiles(window_tokens, tile):
    out = _I3()
    _check(load_library().sta_window_tokens_to_tiles(_i3(window_tokens), _i3(tile), out))
    return tuple(out)


def sta_block_census(mask_kind, grid, tile, window_tokens):
    """Returns (dense_per_q, mixed_per_q, (dense, mixed, empty)); the per-query arrays are lists of ints."""
    n = 1
    for g, t in zip(grid, tile):
        if int(t) <= 0:
            raise StaError(2, sta_strerror(2))
        n *= max(int(g) // int(t), 0)
    n = max(n, 1)
    dense = (ctypes.c_int64 * n)()
    mixed = (ctypes.c_int64 * n)()
    totals = (ctypes.c_int64 * 3)()
    _check(load_library().sta_block_census(int(mask_kind), _i3(grid), _i3(tile), _i3(window_tokens), dense, mixed,
                                           totals))
    return list(dense), list(mixed), tuple(totals)


def sta_kept_flops(B, H, D, grid, tile, window_tiles) -> float:
    return float(load_library().sta_kept_flops(B, H, D, _i3(grid), _i3(tile), _windows(window_tiles, H)))


def sta_head_mse_workspace_bytes(B, H) -> int:
    return int(load_library().sta_head_mse_workspace_bytes(int(B), int(H)))


def _nbytes(t):
    return t.numel() * t.element_size()


def sta_head_mse(a, b, grid, workspace, mse, stream=None):
    """Per-head MSE of two bf16 [B,H,N,D] tensors into mse (float32 [H]); workspace: device bytes."""
    if a.shape != b.shape or a.dtype != torch.bfloat16 or b.dtype != torch.bfloat16 or a.dim() != 4:
        raise ValueError("expect two bf16 [B, H, N, D] tensors of equal shape")
    B, H, N, D = a.shape
    if mse.dtype != torch.float32 or mse.numel() != H:
        raise ValueError("mse must be float32 [H]")
    _check(load_library().sta_head_mse(_dev(a, "a"), _dev(b, "b"), B, H, D, _i3(grid), _dev(workspace, "workspace"),
                                       _nbytes(workspace), _dev(mse, "mse"), _stream_ptr(stream)))
    return mse


def sta_head_mse_static(a, b, grid, mse, stream=None):
    """sta_head_mse without a workspace argument (partial sums in a fixed device array of the library)."""
    if a.shape != b.shape or a.dtype != torch.bfloat16 or b.dtype != torch.bfloat16 or a.dim() != 4:
        raise ValueError("expect two bf16 [B, H, N, D] tensors of equal shape")
    B, H, N, D = a.shape
    if mse.dtype != torch.float32 or mse.numel() != H:
        raise ValueError("mse must be float32 [H]")
    _check(load_library().sta_head_mse_static(_dev(a, "a"), _dev(b, "b"), B, H, D, _i3(grid), _dev(mse, "mse"),
                                              _stream_ptr(stream)))
    return mse


def sta_mask_search(q_tiled, k_tiled, v_tiled, grid, tile, patterns, o_full, o_pattern, workspace, losses, best,
                    scale=0.0, stream=None):
    """Mask-search inner loop: losses float32 [n_patterns, H], best int32 [H]; patterns: (t,h,w) in tiles."""
    B, H, N, D = q_tiled.shape
    flat = [int(x) for p in patterns for x in p]
    n_p = len(patterns)
    if len(flat) != 3 * n_p:
        raise ValueError("patterns must be triples")
    if losses.dtype != torch.float32 or losses.numel() != n_p * H or best.dtype != torch.int32 or best.numel() != H:
        raise ValueError("losses must be float32 [n_patterns, H] and best int32 [H]")
    arr = (ctypes.c_int * (3 * n_p))(*flat)
    _check(load_library().sta_mask_search(_dev(q_tiled, "q"), _dev(k_tiled, "k"), _dev(v_tiled, "v"), B, H, D,
                                          _i3(grid), _i3(tile), arr, n_p, float(scale), _dev(o_full, "o_full"),
                                          _dev(o_pattern, "o_pattern"), _dev(workspace, "workspace"),
                                          _nbytes(workspace), _dev(losses, "losses"), _dev(best, "best"),
                                          _stream_ptr(stream)))
    return losses, best


def sta_attention_recall(lse_window, lse_full, grid, workspace, mean, recall=None, stream=None):
    """recall = exp(lse_window - lse_full); mean: float32 [B*H]; recall: optional float32 [B,H,N];
    workspace: device bytes, at least sta_head_mse_workspace_bytes(B, H)."""
    if lse_window.shape != lse_full.shape or lse_window.dim() != 3 or lse_window.dtype != torch.float32:
        raise ValueError("expect two float32 [B, H, N] tensors")
    B, H, N = lse_window.shape
    if mean.dtype != torch.float32 or mean.numel() != B * H:
        raise ValueError("mean must be float32 [B*H]")
    rp = ctypes.c_void_p(0) if recall is None else _dev(recall, "recall")
    _check(load_library().sta_attention_recall(_dev(lse_window, "lse_window"), _dev(lse_full, "lse_full"), B, H,
                                               _i3(grid), _dev(workspace, "workspace"), _nbytes(workspace), rp,
                                               _dev(mean, "mean"), _stream_ptr(stream)))
    return mean
