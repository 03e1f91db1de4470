// C ABI of libsta: argument checking, host-side geometry, kernel dispatch.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <new>

#include "../../include/sta.h"
#include "sta_geometry.h"
#include "sta_internal.h"

namespace {

struct Shape {
    int64_t N, P, n_tiles;
    int n[3];
};

// Validates B, H, D, grid, tile and fills the derived sizes.
int check_shape(int B, int H, int D, const int grid[3], const int tile[3], Shape *s)
{
    if (!grid || !tile) return STA_ERR_NULL;
    if (B <= 0 || H <= 0 || D <= 0) return STA_ERR_SHAPE;
    int64_t N = 1, P = 1, nt = 1;
    for (int a = 0; a < 3; ++a) {
        if (grid[a] <= 0 || tile[a] <= 0 || grid[a] % tile[a] != 0) return STA_ERR_SHAPE;
        s->n[a] = grid[a] / tile[a];
        if (s->n[a] > 30000) return STA_ERR_SHAPE;
        N *= grid[a];
        P *= tile[a];
        nt *= s->n[a];
        if (N > (int64_t)1 << 30 || P > (int64_t)1 << 20) return STA_ERR_SHAPE;
    }
    // element count of one tensor must stay addressable with comfortable margin
    const long double total = (long double)B * H * (long double)N * D;
    if (total > 9.0e15L) return STA_ERR_SHAPE;
    if ((int64_t)B * H > 0x7fffffff / (nt > 0 ? nt : 1)) return STA_ERR_SHAPE;
    s->N = N;
    s->P = P;
    s->n_tiles = nt;
    return STA_OK;
}

bool valid_dtype(int dt) { return dt == STA_BF16 || dt == STA_F32; }

size_t elem_size(int dt) { return dt == STA_F32 ? 4 : 2; }

bool ranges_overlap(const void *a, size_t abytes, const void *b, size_t bbytes)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

uint32_t magic_of(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }

int permute_common(const void *src, void *dst, int src_dt, int dst_dt, int B, int H, int D, const int grid[3],
                   const int tile[3], void *hip_stream, bool to_tiled)
{
    if (!src || !dst) return STA_ERR_NULL;
    Shape s;
    if (int rc = check_shape(B, H, D, grid, tile, &s)) return rc;
    if (!valid_dtype(src_dt) || !valid_dtype(dst_dt)) return STA_ERR_UNSUPPORTED;
    if (D % 8 != 0) return STA_ERR_UNSUPPORTED;
    const size_t elems = (size_t)B * H * s.N * D;
    if (ranges_overlap(src, elems * elem_size(src_dt), dst, elems * elem_size(dst_dt))) return STA_ERR_ALIAS;

    sta::PermuteParams p;
    p.N = (uint32_t)s.N;
    p.cpr = (uint32_t)(D / 8);
    p.L_h = grid[1];
    p.L_w = grid[2];
    p.T_t = tile[0];
    p.T_h = tile[1];
    p.T_w = tile[2];
    p.n_h = s.n[1];
    p.n_w = s.n[2];
    p.n_tiles = (uint32_t)s.n_tiles;
    const uint64_t cpt = (uint64_t)s.P * p.cpr;
    p.seg = p.T_w * p.cpr;
    // exactness condition of the multiply-high division used by the kernel
    if (cpt * p.seg >= ((uint64_t)1 << 32) || cpt * p.T_h >= ((uint64_t)1 << 32)) return STA_ERR_SHAPE;
    p.chunks_per_tile = (uint32_t)cpt;
    p.seg_magic = magic_of(p.seg);
    p.T_h_magic = magic_of(p.T_h);
    // One workgroup moves at most kPermuteChunksPerBlock chunks, one pass of four 16-byte loads and stores per lane:
    // measured at the 115,200-token, 24-head tensor 5.0 TB/s with one workgroup per 384-token tile (six passes),
    // 5.2 / 5.4 / 5.5 TB/s with 2 / 3 / 6 workgroups per tile.
    const uint64_t tiles = (uint64_t)B * H * s.n_tiles;
    p.span = sta::kPermuteChunksPerBlock;
    p.parts = (uint32_t)((cpt + p.span - 1) / p.span);
    if (tiles * p.parts >= ((uint64_t)1 << 31)) return STA_ERR_SHAPE;
    const uint32_t blocks = (uint32_t)(tiles * p.parts);
    hipError_t e = sta::launch_permute(src, dst, src_dt == STA_F32, dst_dt == STA_F32, to_tiled, p, blocks,
                                       static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? STA_OK : STA_ERR_HIP;
}

int check_windows(int H, const int *window_tiles)
{
    if (!window_tiles) return STA_ERR_NULL;
    for (int i = 0; i < 3 * H; ++i)
        if (window_tiles[i] < 1) return STA_ERR_WINDOW;
    return STA_OK;
}

void fill_window_table(sta::WindowTable *t, const int *window_tiles, int head_base, int heads, const int n[3])
{
    for (int h = 0; h < heads; ++h)
        for (int a = 0; a < 3; ++a) {
            const int w = window_tiles[3 * (head_base + h) + a];
            t->w[h][a] = (uint16_t)(w < 2 * n[a] ? w : 2 * n[a]);   // >= 2n-1 already means the whole axis
        }
}

// Kept (query tile, key tile) pairs of one head: the box is a product of per-axis ranges, so the count factorises.
double kept_pairs_of_head(const int n[3], const int *window3)
{
    double per_head = 1.0;
    for (int a = 0; a < 3; ++a) {
        const int w = window3[a] < 2 * n[a] ? window3[a] : 2 * n[a];
        long sum = 0;
        for (int qa = 0; qa < n[a]; ++qa) {
            const StaAxisRange r = sta_axis_range(n[a], w, qa);
            sum += r.hi - r.lo + 1;
        }
        per_head *= (double)sum;
    }
    return per_head;
}

// Heads of the launch sorted by descending cost (stable, so equal heads keep their order).
void fill_head_order(sta::HeadOrder *o, const int *window_tiles, int head_base, int heads, const int n[3])
{
    double cost[sta::kMaxHeadsPerLaunch];
    for (int h = 0; h < heads; ++h) {
        o->h[h] = (uint16_t)h;
        cost[h] = kept_pairs_of_head(n, window_tiles + 3 * (head_base + h));
    }
    for (int i = 1; i < heads; ++i) {          // insertion sort: at most 256 entries
        const uint16_t hi = o->h[i];
        int j = i - 1;
        while (j >= 0 && cost[o->h[j]] < cost[hi]) { o->h[j + 1] = o->h[j]; --j; }
        o->h[j + 1] = hi;
    }
    for (int h = heads; h < sta::kMaxHeadsPerLaunch; ++h) o->h[h] = 0;
}

sta::FwdParams make_fwd_params(const Shape &s, int H, float scale_log2e)
{
    sta::FwdParams p;
    p.N = (uint32_t)s.N;
    p.P = (uint32_t)s.P;
    p.n_t = s.n[0];
    p.n_h = s.n[1];
    p.n_w = s.n[2];
    p.n_tiles = (uint32_t)s.n_tiles;
    p.H = H;
    p.head_base = 0;
    p.heads = 0;
    p.scale_log2e = scale_log2e;
    p.lse = nullptr;
    return p;
}

// Kept key-token interval [lo, hi] along one axis for query token x.
//  STA: the key-tile range of x's tile, in tokens.  Sliding window: centre x clamped into
//  [half, L-1-half] (upper clamp first), keys within half of it, clipped to the axis.
struct TokenRange {
    int lo, hi;
};

TokenRange kept_token_range(int mask_kind, int L, int T, int W, int x)
{
    TokenRange r;
    if (mask_kind == STA_MASK_STA) {
        const int n = L / T;
        int w = W / T;
        if (w > 2 * n) w = 2 * n;
        const StaAxisRange t = sta_axis_range(n, w, x / T);
        r.lo = t.lo * T;
        r.hi = t.hi * T + T - 1;
    } else {
        const int half = (W < 2 * L ? W : 2 * L) / 2;
        int c = x < (L - 1 - half) ? x : (L - 1 - half);
        c = c > half ? c : half;
        r.lo = (c - half) > 0 ? (c - half) : 0;
        r.hi = (c + half) < (L - 1) ? (c + half) : (L - 1);
    }
    return r;
}

// Per query tile along one axis: how many key tiles are fully kept by every query of the tile, and how many
// are touched by at least one.
void axis_census(int mask_kind, int L, int T, int W, int64_t *full, int64_t *touched)
{
    const int n = L / T;
    for (int i = 0; i < n; ++i) {
        int64_t f = 0, e = 0;
        for (int j = 0; j < n; ++j) {
            const int y0 = j * T, y1 = j * T + T - 1;
            bool all = true, any = false;
            for (int x = i * T; x < i * T + T; ++x) {
                const TokenRange r = kept_token_range(mask_kind, L, T, W, x);
                all = all && (r.lo <= y0 && y1 <= r.hi);
                any = any || (r.lo <= y1 && y0 <= r.hi);
            }
            f += all;
            e += any;
        }
        full[i] = f;
        touched[i] = e;
    }
}

}  // namespace

extern "C" {

int sta_tile_permute(const void *src, void *dst, int src_dt, int dst_dt, int B, int H, int D, const int grid[3],
                     const int tile[3], void *hip_stream)
{
    return permute_common(src, dst, src_dt, dst_dt, B, H, D, grid, tile, hip_stream, true);
}

int sta_untile(const void *src, void *dst, int src_dt, int dst_dt, int B, int H, int D, const int grid[3],
               const int tile[3], void *hip_stream)
{
    return permute_common(src, dst, src_dt, dst_dt, B, H, D, grid, tile, hip_stream, false);
}

size_t sta_workspace_bytes(int B, int H, int D, const int grid[3], const int tile[3])
{
    Shape s;
    if (check_shape(B, H, D, grid, tile, &s) != STA_OK) return 0;
    return sta::forward_split_workspace_bytes((int)s.P, D);
}

}  // extern "C"

namespace {

int forward_common(const void *q_tiled, const void *k_tiled, const void *v_tiled, void *o_tiled, float *lse_tiled,
                   int B, int H, int D, const int grid[3], const int tile[3], const int *window_tiles, float scale,
                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!q_tiled || !k_tiled || !v_tiled || !o_tiled) return STA_ERR_NULL;
    Shape s;
    if (int rc = check_shape(B, H, D, grid, tile, &s)) return rc;
    if (int rc = check_windows(H, window_tiles)) return rc;
    if (!sta::forward_supported((int)s.P, D)) return STA_ERR_UNSUPPORTED;
    const size_t bytes = (size_t)B * H * s.N * D * 2;
    if (ranges_overlap(o_tiled, bytes, q_tiled, bytes) || ranges_overlap(o_tiled, bytes, k_tiled, bytes) ||
        ranges_overlap(o_tiled, bytes, v_tiled, bytes))
        return STA_ERR_ALIAS;
    if (workspace != nullptr) {
        if (workspace_bytes < sta::forward_split_workspace_bytes((int)s.P, D) || ((uintptr_t)workspace & 15) != 0)
            return STA_ERR_WORKSPACE;
        const void *tensors[4] = {q_tiled, k_tiled, v_tiled, o_tiled};
        for (int i = 0; i < 4; ++i)
            if (workspace_bytes != 0 && ranges_overlap(workspace, workspace_bytes, tensors[i], bytes)) return STA_ERR_ALIAS;
    }
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);
    sta::FwdParams p = make_fwd_params(s, H, scale * 1.4426950408889634f);
    if (lse_tiled) {
        const size_t lse_bytes = (size_t)B * H * s.N * sizeof(float);
        if (ranges_overlap(lse_tiled, lse_bytes, q_tiled, bytes) || ranges_overlap(lse_tiled, lse_bytes, k_tiled, bytes) ||
            ranges_overlap(lse_tiled, lse_bytes, v_tiled, bytes) || ranges_overlap(lse_tiled, lse_bytes, o_tiled, bytes))
            return STA_ERR_ALIAS;
        p.lse = lse_tiled;
    }

    // Per-head windows travel in the kernel arguments; heads are launched in chunks.
    int max_heads = sta::kMaxHeadsPerLaunch;
    if ((int64_t)B * max_heads > 65535) max_heads = 65535 / B;
    if (max_heads < 1) return STA_ERR_SHAPE;
    for (int hb = 0; hb < H; hb += max_heads) {
        const int heads = (H - hb) < max_heads ? (H - hb) : max_heads;
        sta::WindowTable win;
        fill_window_table(&win, window_tiles, hb, heads, s.n);
        p.head_base = hb;
        p.heads = heads;
        sta::HeadOrder order;
        fill_head_order(&order, window_tiles, hb, heads, s.n);
        hipError_t e = sta::launch_forward(q_tiled, k_tiled, v_tiled, o_tiled, B, D, p, win, order,
                                           static_cast<float *>(workspace), workspace_bytes / sizeof(float),
                                           static_cast<hipStream_t>(hip_stream));
        if (e != hipSuccess) return STA_ERR_HIP;
    }
    return STA_OK;
}

}  // namespace

extern "C" {

int sta_forward(const void *q_tiled, const void *k_tiled, const void *v_tiled, void *o_tiled, int B, int H, int D,
                const int grid[3], const int tile[3], const int *window_tiles, float scale, void *workspace,
                size_t workspace_bytes, void *hip_stream)
{
    return forward_common(q_tiled, k_tiled, v_tiled, o_tiled, nullptr, B, H, D, grid, tile, window_tiles, scale,
                          workspace, workspace_bytes, hip_stream);
}

int sta_forward_lse(const void *q_tiled, const void *k_tiled, const void *v_tiled, void *o_tiled, float *lse_tiled,
                    int B, int H, int D, const int grid[3], const int tile[3], const int *window_tiles, float scale,
                    void *hip_stream)
{
    if (!lse_tiled) return STA_ERR_NULL;
    return forward_common(q_tiled, k_tiled, v_tiled, o_tiled, lse_tiled, B, H, D, grid, tile, window_tiles, scale,
                          nullptr, 0, hip_stream);
}

size_t sta_head_mse_workspace_bytes(int B, int H)
{
    if (B <= 0 || H <= 0) return 0;
    return (size_t)B * (size_t)H * sta::kMseSlices * sizeof(double);
}

int sta_head_mse(const void *a, const void *b, int B, int H, int D, const int grid[3], void *workspace,
                 size_t workspace_bytes, float *dev_mse, void *hip_stream)
{
    if (!a || !b || !dev_mse) return STA_ERR_NULL;
    const int unit[3] = {1, 1, 1};
    Shape s;
    if (int rc = check_shape(B, H, D, grid, unit, &s)) return rc;
    if (D % 8 != 0) return STA_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < sta_head_mse_workspace_bytes(B, H)) return STA_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 7) != 0) return STA_ERR_WORKSPACE;
    hipError_t e = sta::launch_head_mse(a, b, B, H, (size_t)s.N * D, static_cast<double *>(workspace), dev_mse,
                                        static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? STA_OK : STA_ERR_HIP;
}

int sta_head_mse_static(const void *a, const void *b, int B, int H, int D, const int grid[3], float *dev_mse,
                        void *hip_stream)
{
    if (!a || !b || !dev_mse) return STA_ERR_NULL;
    const int unit[3] = {1, 1, 1};
    Shape s;
    if (int rc = check_shape(B, H, D, grid, unit, &s)) return rc;
    if (D % 8 != 0) return STA_ERR_UNSUPPORTED;
    if ((int64_t)B * H > sta::kStaticMseMaxSlabs) return STA_ERR_WORKSPACE;
    double *partial = nullptr;
    if (sta::static_mse_scratch(&partial) != hipSuccess) return STA_ERR_HIP;
    hipError_t e = sta::launch_head_mse(a, b, B, H, (size_t)s.N * D, partial, dev_mse,
                                        static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? STA_OK : STA_ERR_HIP;
}

int sta_attention_recall(const float *lse_window, const float *lse_full, int B, int H, const int grid[3],
                         void *workspace, size_t workspace_bytes, float *dev_recall, float *dev_mean,
                         void *hip_stream)
{
    if (!lse_window || !lse_full || !dev_mean) return STA_ERR_NULL;
    const int unit[3] = {1, 1, 1};
    Shape s;
    if (int rc = check_shape(B, H, 8, grid, unit, &s)) return rc;
    if (!workspace || workspace_bytes < sta_head_mse_workspace_bytes(B, H)) return STA_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 7) != 0) return STA_ERR_WORKSPACE;
    hipError_t e = sta::launch_recall(lse_window, lse_full, B * H, (size_t)s.N, dev_recall,
                                      static_cast<double *>(workspace), dev_mean,
                                      static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? STA_OK : STA_ERR_HIP;
}

int sta_mask_search(const void *q_tiled, const void *k_tiled, const void *v_tiled, int B, int H, int D,
                    const int grid[3], const int tile[3], const int *patterns, int n_patterns, float scale,
                    void *o_full, void *o_pattern, void *workspace, size_t workspace_bytes, float *dev_losses,
                    int32_t *dev_best, void *hip_stream)
{
    if (!patterns || !o_full || !o_pattern || !dev_losses || !dev_best) return STA_ERR_NULL;
    if (n_patterns < 1 || n_patterns > 4096) return STA_ERR_SHAPE;
    if (H > 4096) return STA_ERR_SHAPE;
    if (int rc = check_windows(n_patterns, patterns)) return rc;
    Shape s;
    if (int rc = check_shape(B, H, D, grid, tile, &s)) return rc;
    if (!workspace || workspace_bytes < sta_head_mse_workspace_bytes(B, H)) return STA_ERR_WORKSPACE;
    const size_t bytes = (size_t)B * H * s.N * D * 2;
    if (ranges_overlap(o_full, bytes, o_pattern, bytes)) return STA_ERR_ALIAS;

    // Every head's output depends on that head's mask only, so one launch with the same pattern on all heads
    // yields the per-head losses the algorithm obtains by masking one head at a time.
    int win[3 * 4096];
    for (int h = 0; h < H; ++h)
        for (int a = 0; a < 3; ++a) win[3 * h + a] = s.n[a];                 // the original: full attention
    if (int rc = forward_common(q_tiled, k_tiled, v_tiled, o_full, nullptr, B, H, D, grid, tile, win, scale, nullptr, 0,
                                hip_stream))
        return rc;
    for (int p = 0; p < n_patterns; ++p) {
        for (int h = 0; h < H; ++h)
            for (int a = 0; a < 3; ++a) win[3 * h + a] = patterns[3 * p + a];
        if (int rc = forward_common(q_tiled, k_tiled, v_tiled, o_pattern, nullptr, B, H, D, grid, tile, win, scale,
                                    nullptr, 0, hip_stream))
            return rc;
        if (int rc = sta_head_mse(o_full, o_pattern, B, H, D, grid, workspace, workspace_bytes,
                                  dev_losses + (size_t)p * H, hip_stream))
            return rc;
    }
    hipError_t e = sta::launch_first_min(dev_losses, n_patterns, H, dev_best, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? STA_OK : STA_ERR_HIP;
}

int sta_key_tile_box(const int grid_tiles[3], const int window_tiles[3], const int q_tile[3], int lo[3], int hi[3])
{
    if (!grid_tiles || !window_tiles || !q_tile || !lo || !hi) return STA_ERR_NULL;
    for (int a = 0; a < 3; ++a) {
        if (grid_tiles[a] <= 0 || q_tile[a] < 0 || q_tile[a] >= grid_tiles[a]) return STA_ERR_SHAPE;
        if (window_tiles[a] < 1) return STA_ERR_WINDOW;
    }
    for (int a = 0; a < 3; ++a) {
        const int n = grid_tiles[a];
        const int w = window_tiles[a] < 2 * n ? window_tiles[a] : 2 * n;
        const StaAxisRange r = sta_axis_range(n, w, q_tile[a]);
        lo[a] = r.lo;
        hi[a] = r.hi;
    }
    return STA_OK;
}

int sta_query_tile_box(const int grid_tiles[3], const int window_tiles[3], const int k_tile[3], int lo[3], int hi[3])
{
    if (!grid_tiles || !window_tiles || !k_tile || !lo || !hi) return STA_ERR_NULL;
    for (int a = 0; a < 3; ++a) {
        if (grid_tiles[a] <= 0 || k_tile[a] < 0 || k_tile[a] >= grid_tiles[a]) return STA_ERR_SHAPE;
        if (window_tiles[a] < 1) return STA_ERR_WINDOW;
    }
    for (int a = 0; a < 3; ++a) {
        const int n = grid_tiles[a];
        const int w = window_tiles[a] < 2 * n ? window_tiles[a] : 2 * n;
        const StaAxisRange r = sta_axis_query_range(n, w, k_tile[a]);
        lo[a] = r.lo;
        hi[a] = r.hi;
    }
    return STA_OK;
}

size_t sta_backward_workspace_bytes(int B, int H, const int grid[3])
{
    if (!grid || B <= 0 || H <= 0 || grid[0] <= 0 || grid[1] <= 0 || grid[2] <= 0) return 0;
    return 2 * (size_t)B * H * (size_t)grid[0] * grid[1] * grid[2] * sizeof(float);     // two row statistics
}

int sta_backward(const void *q_tiled, const void *k_tiled, const void *v_tiled, const void *o_tiled,
                 const void *d_o_tiled, const float *lse_tiled, void *d_q_tiled, void *d_k_tiled, void *d_v_tiled, int B,
                 int H, int D, const int grid[3], const int tile[3], const int *window_tiles, float scale,
                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!q_tiled || !k_tiled || !v_tiled || !o_tiled || !d_o_tiled || !lse_tiled || !d_q_tiled || !d_k_tiled ||
        !d_v_tiled)
        return STA_ERR_NULL;
    Shape s;
    if (int rc = check_shape(B, H, D, grid, tile, &s)) return rc;
    if (int rc = check_windows(H, window_tiles)) return rc;
    if (!sta::backward_supported((int)s.P, D)) return STA_ERR_UNSUPPORTED;
    const size_t bytes = (size_t)B * H * s.N * D * 2;
    const size_t stat_bytes = (size_t)B * H * s.N * sizeof(float);
    const size_t ws_bytes = 2 * stat_bytes;
    if (!workspace || workspace_bytes < ws_bytes || ((uintptr_t)workspace & 15) != 0) return STA_ERR_WORKSPACE;
    if (((uintptr_t)lse_tiled & 15) != 0) return STA_ERR_SHAPE;
    const void *inputs[5] = {q_tiled, k_tiled, v_tiled, o_tiled, d_o_tiled};
    void *outputs[3] = {d_q_tiled, d_k_tiled, d_v_tiled};
    for (int i = 0; i < 3; ++i) {
        for (int j = 0; j < 5; ++j)
            if (ranges_overlap(outputs[i], bytes, inputs[j], bytes)) return STA_ERR_ALIAS;
        for (int j = i + 1; j < 3; ++j)
            if (ranges_overlap(outputs[i], bytes, outputs[j], bytes)) return STA_ERR_ALIAS;
        if (ranges_overlap(outputs[i], bytes, lse_tiled, stat_bytes) || ranges_overlap(outputs[i], bytes, workspace, ws_bytes))
            return STA_ERR_ALIAS;
    }
    for (int j = 0; j < 5; ++j)
        if (ranges_overlap(workspace, ws_bytes, inputs[j], bytes)) return STA_ERR_ALIAS;
    if (ranges_overlap(workspace, ws_bytes, lse_tiled, stat_bytes)) return STA_ERR_ALIAS;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);
    sta::FwdParams p = make_fwd_params(s, H, scale * 1.4426950408889634f);

    int max_heads = sta::kMaxHeadsPerLaunch;
    if ((int64_t)B * max_heads > 65535) max_heads = 65535 / B;
    if (max_heads < 1) return STA_ERR_SHAPE;
    for (int hb = 0; hb < H; hb += max_heads) {
        const int heads = (H - hb) < max_heads ? (H - hb) : max_heads;
        sta::WindowTable win;
        fill_window_table(&win, window_tiles, hb, heads, s.n);
        p.head_base = hb;
        p.heads = heads;
        hipError_t e = sta::launch_backward(q_tiled, k_tiled, v_tiled, o_tiled, d_o_tiled, lse_tiled,
                                            static_cast<float *>(workspace), hb == 0, d_q_tiled, d_k_tiled, d_v_tiled, B,
                                            D, p, win, static_cast<hipStream_t>(hip_stream));
        if (e != hipSuccess) return STA_ERR_HIP;
    }
    return STA_OK;
}

int sta_dump_key_tiles(int H, const int grid[3], const int tile[3], const int *window_tiles, int32_t *dev_counts,
                       int32_t *dev_lists, void *hip_stream)
{
    if (!dev_counts || !dev_lists) return STA_ERR_NULL;
    Shape s;
    if (int rc = check_shape(1, H, 8, grid, tile, &s)) return rc;
    if (int rc = check_windows(H, window_tiles)) return rc;
    sta::FwdParams p = make_fwd_params(s, H, 1.f);
    for (int hb = 0; hb < H; hb += sta::kMaxHeadsPerLaunch) {
        const int heads = (H - hb) < sta::kMaxHeadsPerLaunch ? (H - hb) : sta::kMaxHeadsPerLaunch;
        sta::WindowTable win;
        fill_window_table(&win, window_tiles, hb, heads, s.n);
        p.head_base = hb;
        p.heads = heads;
        if (sta::launch_dump_key_tiles(p, win, dev_counts, dev_lists, static_cast<hipStream_t>(hip_stream)) !=
            hipSuccess)
            return STA_ERR_HIP;
    }
    return STA_OK;
}

int sta_block_census(int mask_kind, const int grid[3], const int tile[3], const int window_tokens[3],
                     int64_t *dense_per_q, int64_t *mixed_per_q, int64_t totals[3])
{
    if (!window_tokens) return STA_ERR_NULL;
    Shape s;
    if (int rc = check_shape(1, 1, 8, grid, tile, &s)) return rc;
    if (mask_kind != STA_MASK_STA && mask_kind != STA_MASK_NATTEN) return STA_ERR_UNSUPPORTED;
    for (int a = 0; a < 3; ++a) {
        if (window_tokens[a] < 1) return STA_ERR_WINDOW;
        if (mask_kind == STA_MASK_STA && window_tokens[a] / tile[a] < 1) return STA_ERR_WINDOW;
    }
    int64_t *full[3], *touched[3];
    int64_t *buf = new (std::nothrow) int64_t[2 * (size_t)(s.n[0] + s.n[1] + s.n[2])];
    if (!buf) return STA_ERR_SHAPE;
    int64_t *cur = buf;
    for (int a = 0; a < 3; ++a) {
        full[a] = cur;
        touched[a] = cur + s.n[a];
        cur += 2 * s.n[a];
        axis_census(mask_kind, grid[a], tile[a], window_tokens[a], full[a], touched[a]);
    }
    int64_t dense_total = 0, mixed_total = 0;
    int64_t q = 0;
    for (int it = 0; it < s.n[0]; ++it)
        for (int ih = 0; ih < s.n[1]; ++ih)
            for (int iw = 0; iw < s.n[2]; ++iw, ++q) {
                const int64_t dense = full[0][it] * full[1][ih] * full[2][iw];
                const int64_t mixed = touched[0][it] * touched[1][ih] * touched[2][iw] - dense;
                if (dense_per_q) dense_per_q[q] = dense;
                if (mixed_per_q) mixed_per_q[q] = mixed;
                dense_total += dense;
                mixed_total += mixed;
            }
    delete[] buf;
    if (totals) {
        totals[0] = dense_total;
        totals[1] = mixed_total;
        totals[2] = s.n_tiles * s.n_tiles - dense_total - mixed_total;
    }
    return STA_OK;
}

int sta_forward_general(const void *q_tiled, const void *k_tiled, const void *v_tiled, void *o_tiled, int B, int H, int D,
                        const int grid[3], const int tile[3], int mask_kind, const int *window, float scale,
                        void *hip_stream)
{
    if (!q_tiled || !k_tiled || !v_tiled || !o_tiled) return STA_ERR_NULL;
    if (mask_kind != STA_MASK_STA && mask_kind != STA_MASK_NATTEN) return STA_ERR_UNSUPPORTED;
    Shape s;
    if (int rc = check_shape(B, H, D, grid, tile, &s)) return rc;
    if (!window) return STA_ERR_NULL;
    if (mask_kind == STA_MASK_STA) {
        if (int rc = check_windows(H, window)) return rc;
    } else {
        for (int i = 0; i < 3 * H; ++i)
            if (window[i] <= 0) return STA_ERR_WINDOW;
        if (s.P > sta::kMaxTokenWindowTile) return STA_ERR_UNSUPPORTED;
    }
    if (!sta::forward_supported((int)s.P, D)) return STA_ERR_UNSUPPORTED;
    const size_t bytes = (size_t)B * H * s.N * D * 2;
    if (ranges_overlap(o_tiled, bytes, q_tiled, bytes) || ranges_overlap(o_tiled, bytes, k_tiled, bytes) ||
        ranges_overlap(o_tiled, bytes, v_tiled, bytes))
        return STA_ERR_ALIAS;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);
    sta::FwdParams p = make_fwd_params(s, H, scale * 1.4426950408889634f);
    p.T_t = tile[0];
    p.T_h = tile[1];
    p.T_w = tile[2];
    int max_heads = sta::kMaxHeadsPerLaunch;
    if ((int64_t)B * max_heads > 65535) max_heads = 65535 / B;
    if (max_heads < 1) return STA_ERR_SHAPE;
    for (int hb = 0; hb < H; hb += max_heads) {
        const int heads = (H - hb) < max_heads ? (H - hb) : max_heads;
        sta::WindowTable win;
        if (mask_kind == STA_MASK_STA) {
            fill_window_table(&win, window, hb, heads, s.n);
        } else {
            for (int h = 0; h < heads; ++h)
                for (int a = 0; a < 3; ++a) {
                    const int w = window[3 * (hb + h) + a], cap = 2 * grid[a];       // 2L already covers the axis from anywhere
                    win.w[h][a] = (uint16_t)(w < cap ? (w < 65535 ? w : 65535) : (cap < 65535 ? cap : 65535));
                }
        }
        p.head_base = hb;
        p.heads = heads;
        if (sta::launch_forward_general(q_tiled, k_tiled, v_tiled, o_tiled, B, D, p, win, mask_kind == STA_MASK_NATTEN,
                                        static_cast<hipStream_t>(hip_stream)) != hipSuccess)
            return STA_ERR_HIP;
    }
    return STA_OK;
}

int sta_window_tokens_to_tiles(const int window_tokens[3], const int tile[3], int out_tiles[3])
{
    if (!window_tokens || !tile || !out_tiles) return STA_ERR_NULL;
    for (int a = 0; a < 3; ++a) {
        if (tile[a] <= 0) return STA_ERR_SHAPE;
        if (window_tokens[a] <= 0 || window_tokens[a] % tile[a] != 0) return STA_ERR_WINDOW;
    }
    for (int a = 0; a < 3; ++a) out_tiles[a] = window_tokens[a] / tile[a];
    return STA_OK;
}

double sta_kept_flops(int B, int H, int D, const int grid[3], const int tile[3], const int *window_tiles)
{
    Shape s;
    if (check_shape(B, H, D, grid, tile, &s) != STA_OK) return 0.0;
    if (check_windows(H, window_tiles) != STA_OK) return 0.0;
    double pairs = 0.0;
    for (int h = 0; h < H; ++h) pairs += kept_pairs_of_head(s.n, window_tiles + 3 * h);
    return 4.0 * (double)s.P * (double)s.P * (double)D * pairs * (double)B;
}

const char *sta_strerror(int status)
{
    switch (status) {
    case STA_OK: return "ok";
    case STA_ERR_NULL: return "required pointer is NULL";
    case STA_ERR_SHAPE: return "invalid shape: non-positive dimension, grid not a multiple of tile, or too large";
    case STA_ERR_WINDOW: return "invalid window: entries must be >= 1 (and multiples of the tile when given in tokens)";
    case STA_ERR_UNSUPPORTED: return "unsupported combination of tile size, head dim or dtype";
    case STA_ERR_ALIAS: return "source and destination buffers overlap";
    case STA_ERR_WORKSPACE: return "workspace missing or too small";
    case STA_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
    }
}

int sta_version(void) { return 100; }

}  // extern "C"
