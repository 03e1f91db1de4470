/*
 * sta.h -- C ABI of the Sliding Tile Attention (STA) forward path for AMD
 * MI355X (gfx950).
 *
 * Conventions that hold for every entry point
 *   - The return value is an sta_status.  Nothing throws, aborts or prints.
 *     Argument checks happen on the host before any launch; a failed check
 *     launches nothing.
 *   - Pointers named dev_* / *_tiled / src / dst are DEVICE pointers owned by
 *     the caller; `grid`, `tile`, `window_tiles` and friends are HOST pointers
 *     that are read during the call and may be freed on return.
 *   - Tensors are contiguous [B, H, N, D] (batch, head, token, channel) with
 *     N = grid[0]*grid[1]*grid[2].  "raster" order puts token (t,h,w) at
 *     n = (t*grid[1] + h)*grid[2] + w.  "tiled" order puts it at
 *     n = tile_id*P + intra_id with tile_id row-major over the tile grid
 *     (grid[a]/tile[a] per axis), intra_id row-major inside the tile and
 *     P = tile[0]*tile[1]*tile[2]  (Sec. 3.1: each tile occupies one
 *     contiguous run of the sequence; appendix "Tiling in STA").
 *   - All device work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = default stream) and is asynchronous.
 *   - The library allocates no device memory and keeps no state.
 *   - 2D (image) STA is the 3D case with grid[0] = tile[0] = window[0] = 1.
 */
#ifndef STA_H
#define STA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    STA_OK = 0,
    STA_ERR_NULL = 1,        /* a required pointer is NULL */
    STA_ERR_SHAPE = 2,       /* non-positive dimension, grid not a multiple of tile, size overflow */
    STA_ERR_WINDOW = 3,      /* a window entry is < 1 */
    STA_ERR_UNSUPPORTED = 4, /* (P, D, dtype) combination has no kernel */
    STA_ERR_ALIAS = 5,       /* src == dst, or the output aliases an input */
    STA_ERR_WORKSPACE = 6,   /* workspace missing or too small */
    STA_ERR_HIP = 7          /* a HIP call or kernel launch failed */
} sta_status;

typedef enum { STA_BF16 = 0, STA_F32 = 1 } sta_dtype;

/* Mask definitions of the paper's appendix: the tile-granular STA mask and the token-granular sliding
 * window with inward-shifted centre ("Mask Definition of 3D NATTEN") it is compared against. */
typedef enum { STA_MASK_STA = 0, STA_MASK_NATTEN = 1 } sta_mask_kind;

/*
 * Tile permutation (Sec. 3.1, appendix "Tiling in STA"): raster -> tiled.
 * src, dst: device, [B, H, N, D], element types src_dt / dst_dt.  Whole
 * token rows move; when the two types differ the value is converted on the
 * way (f32 -> bf16 rounds to nearest even; bf16 -> f32 is exact).  D must be a
 * multiple of 8.  src and dst must not overlap.
 */
int sta_tile_permute(const void *src, void *dst, int src_dt, int dst_dt,
                     int B, int H, int D, const int grid[3], const int tile[3],
                     void *hip_stream);

/* Inverse permutation: tiled -> raster.  Same arguments and rules. */
int sta_untile(const void *src, void *dst, int src_dt, int dst_dt,
               int B, int H, int D, const int grid[3], const int tile[3],
               void *hip_stream);

/*
 * STA forward (Eq. 1 with the mask of the appendix STA mask algorithm):
 * for every head h and query tile, softmax(Q K^T * scale) V over the key
 * tiles inside that head's window, the window being placed by the clamped
 * centre rule.  q/k/v/o_tiled: device, bf16, [B, H, N, D] in TILED order.
 * window_tiles: host, [H][3], window size in tiles per head (t, h, w), the
 * same for every batch entry; an entry larger than the tile grid means the
 * whole axis.  scale <= 0 selects 1/sqrt(D).  Arithmetic: bf16 inputs, fp32
 * scores, softmax statistics and output accumulator, probabilities rounded
 * to bf16 before the PV product, output rounded to bf16.
 * Supported: D in {64, 128}; P a multiple of 32.  Anything else returns
 * STA_ERR_UNSUPPORTED.
 * workspace: optional device scratch, 16-byte aligned, of at least
 * sta_workspace_bytes(...) bytes.  With it, the work items that would make up
 * the ragged last round of workgroups (the number of query tiles is rarely a
 * multiple of what the chip holds at once) are cut along the keys into parts
 * that fill the chip, each part leaving an unnormalised accumulator, exponent
 * offset and row sum there, and a second kernel merges them in a fixed order
 * (results stay repeatable bit for bit; they differ from the unsplit run by
 * rounding only).  NULL: every query tile is computed by one workgroup.  A
 * non-NULL workspace that is too small or misaligned is STA_ERR_WORKSPACE; one
 * that overlaps a tensor is STA_ERR_ALIAS.  Its contents are undefined after
 * the call.
 */
int sta_forward(const void *q_tiled, const void *k_tiled, const void *v_tiled,
                void *o_tiled, int B, int H, int D, const int grid[3],
                const int tile[3], const int *window_tiles, float scale,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * sta_forward that also returns, per query row, the natural log of the softmax
 * denominator of Eq. 1, ln(sum_j exp(S_ij + M_ij)).  lse_tiled: device, float32,
 * [B, H, N] in TILED token order; must not overlap the other buffers.  It is the
 * quantity from which the paper's attention recall (Sec. 1: the fraction of the
 * total attention score inside a local window) follows without another pass over
 * the scores: recall = exp(lse_window - lse_full).  Everything else as sta_forward.
 */
int sta_forward_lse(const void *q_tiled, const void *k_tiled, const void *v_tiled,
                    void *o_tiled, float *lse_tiled, int B, int H, int D,
                    const int grid[3], const int tile[3], const int *window_tiles,
                    float scale, void *hip_stream);

/*
 * Gradients of sta_forward (what finetuning through STA layers, Sec. 3.2, differentiates): the chain
 * rule of Eq. 1 under the same mask.  With P = softmax(S + M) row-wise and dO the gradient of the
 * loss with respect to O:  dV = P^T dO,  dP = dO V^T,  dS = P o (dP - rowsum(dO o O)),
 * dQ = dS K * scale,  dK = dS^T Q * scale, summed over kept (query tile, key tile) pairs only.
 * q/k/v/o/d_o: device, bf16, [B, H, N, D] in TILED order, o and lse_tiled as returned by
 * sta_forward_lse for the same q, k, v, windows and scale.  d_q/d_k/d_v: device, bf16, same shape,
 * written; they must not overlap any input or each other.  Arithmetic: P is recomputed from the
 * scores and lse in fp32, P and dS are rounded to bf16 for the matrix products, accumulation in
 * fp32, results rounded to bf16.  No atomics: repeated calls give identical bits.
 * workspace: device, 16-byte aligned, at least sta_backward_workspace_bytes(B, H, grid) bytes
 * (two floats per query row), else STA_ERR_WORKSPACE.  lse_tiled must be 16-byte aligned as well
 * (the kernels read it four rows at a time), else STA_ERR_SHAPE.
 * Supported: D in {64, 128}; P a multiple of 32 (D = 128 with P a multiple of 128 takes the fast
 * kernels, everything else simple one-wave kernels); anything else returns STA_ERR_UNSUPPORTED.
 */
size_t sta_backward_workspace_bytes(int B, int H, const int grid[3]);
int sta_backward(const void *q_tiled, const void *k_tiled, const void *v_tiled,
                 const void *o_tiled, const void *d_o_tiled, const float *lse_tiled,
                 void *d_q_tiled, void *d_k_tiled, void *d_v_tiled, int B, int H, int D,
                 const int grid[3], const int tile[3], const int *window_tiles, float scale,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Query-tile box of one key tile: the query tiles whose window (sta_key_tile_box) contains key tile
 * k_tile.  It is the set the gradient kernels walk per key tile; at the borders it is not the mirror
 * image of the key-tile box.  Host, pure integer, inclusive bounds.
 */
int sta_query_tile_box(const int grid_tiles[3], const int window_tiles[3],
                       const int k_tile[3], int lo[3], int hi[3]);

/*
 * Per-head mean squared error between two attention outputs, the loss of the
 * paper's mask-search algorithm ("STA Mask Search": loss <- MSE(O, O')).
 * a, b: device, bf16, [B, H, N, D] in the same token order.  dev_mse: device,
 * float32 [H]; entry h is the mean over batch, tokens and channels of
 * (a - b)^2 for head h, accumulated in fp32 per thread and fp64 across threads
 * in a fixed order (repeatable).  workspace: device, 8-byte aligned, at least
 * sta_head_mse_workspace_bytes(B, H) bytes, else STA_ERR_WORKSPACE.
 */
size_t sta_head_mse_workspace_bytes(int B, int H);
int sta_head_mse(const void *a, const void *b, int B, int H, int D,
                 const int grid[3], void *workspace, size_t workspace_bytes,
                 float *dev_mse, void *hip_stream);

/*
 * sta_head_mse for callers that cannot allocate or pass device scratch: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels, summation order and
 * result bits as sta_head_mse, but the partial sums go to a fixed 512 KB array inside the library's
 * device image (one copy per GPU, held until the process ends) instead of a workspace; the call itself
 * allocates and frees nothing.  Limit: B * H <= 1024, else STA_ERR_WORKSPACE.  Every partial sum the
 * second kernel reads is written by the first one in the same call, so nothing needs clearing between
 * calls; but all calls on one GPU share the array, so two calls that may overlap in time on the same GPU
 * (different streams) race and must be ordered by the caller.
 */
int sta_head_mse_static(const void *a, const void *b, int B, int H, int D,
                        const int grid[3], float *dev_mse, void *hip_stream);

/*
 * Inner loop of the paper's mask-search algorithm for one layer and one set of
 * activations: O <- full attention; for every pattern p of the list (window
 * sizes in tiles, host, [n_patterns][3]): O' <- STA with window p, loss <-
 * MSE(O, O') per head; the pattern kept for a head is the first one whose loss
 * is strictly smaller than every earlier one.  dev_losses: device float32
 * [n_patterns][H]; dev_best: device int32 [H] (index into the list).  o_full,
 * o_pattern: device scratch tensors, bf16 [B, H, N, D], caller-provided;
 * workspace as for sta_head_mse.  Averaging the losses over prompts and time
 * steps, as the paper does before the final choice, is left to the caller
 * (dev_losses is there for that).  H <= 4096.
 */
int sta_mask_search(const void *q_tiled, const void *k_tiled, const void *v_tiled,
                    int B, int H, int D, const int grid[3], const int tile[3],
                    const int *patterns, int n_patterns, float scale,
                    void *o_full, void *o_pattern, void *workspace,
                    size_t workspace_bytes, float *dev_losses, int32_t *dev_best,
                    void *hip_stream);

/*
 * Attention recall (Sec. 1: the fraction of the total attention score that
 * falls inside a local window) from the two log-denominators sta_forward_lse
 * returns for the window and for the full grid: recall = exp(lse_window -
 * lse_full) per query.  lse_*: device float32 [B, H, N] (same token order).
 * dev_recall: device float32 [B, H, N] or NULL; dev_mean: device float32
 * [B*H], the mean recall of each (batch, head), summed in a fixed order.
 * workspace: as for sta_head_mse (same size), else STA_ERR_WORKSPACE.
 */
int sta_attention_recall(const float *lse_window, const float *lse_full, int B,
                         int H, const int grid[3], void *workspace,
                         size_t workspace_bytes, float *dev_recall,
                         float *dev_mean, void *hip_stream);

/* Bytes of device scratch with which sta_forward splits work below one query tile on the current device
 * (0 when the kernels serving this shape do not split: D = 64, or P not a multiple of 128). */
size_t sta_workspace_bytes(int B, int H, int D, const int grid[3],
                           const int tile[3]);

/*
 * Key-tile box of one query tile (appendix STA mask algorithm, in tile
 * units): per axis a, half = window_tiles[a]/2 (integer), centre
 * c = max(min(q_tile[a], grid_tiles[a]-1-half), half), kept key tiles are
 * [c-half, c+half] clipped to the grid.  Host, pure integer.  lo/hi are
 * inclusive.  Note an even window entry w keeps min(n, w+1) tiles, exactly as
 * the algorithm's "<= W/2" test does.
 */
int sta_key_tile_box(const int grid_tiles[3], const int window_tiles[3],
                     const int q_tile[3], int lo[3], int hi[3]);

/*
 * Test hook: the key-tile lists as the DEVICE code computes them (the same
 * device function the attention kernel calls).  dev_counts: device int32
 * [H][n]; dev_lists: device int32 [H][n][n], ascending tile ids, -1 padded;
 * n = number of tiles.
 */
int sta_dump_key_tiles(int H, const int grid[3], const int tile[3],
                       const int *window_tiles, int32_t *dev_counts,
                       int32_t *dev_lists, void *hip_stream);

/*
 * Block census (Sec. 2.2: dense / mixed / empty attention blocks; Theorem 1 for the tiled sliding
 * window, Theorem 2 for STA; Table 1).  Tokens are taken in TILED order, so block (i, j) of the
 * attention map is (query tile i, key tile j), P x P scores.  A block is dense when the mask keeps
 * every score in it, empty when it keeps none, mixed otherwise.  mask_kind: sta_mask_kind;
 * window_tokens: window size in tokens per axis (for STA_MASK_STA converted to tiles by floor
 * division, as the STA mask algorithm does).  Exact counts including the borders (the theorems
 * ignore them).  Host only, pure integer: both masks are products of per-axis interval tests, so
 * the per-axis classifications are counted and multiplied; no token pair is enumerated.
 * dense_per_q, mixed_per_q: host int64 [number of tiles], counts per query tile, either may be
 * NULL.  totals: host int64 [3] = dense, mixed, empty over the whole map; may be NULL.
 */
int sta_block_census(int mask_kind, const int grid[3], const int tile[3],
                     const int window_tokens[3], int64_t *dense_per_q,
                     int64_t *mixed_per_q, int64_t totals[3]);

/*
 * Attention through the library's general (register-staged, untuned) kernel under either mask, for measuring on
 * one and the same kernel what blocks that are only partly kept cost (Sec. 2.2: dense, mixed and empty blocks;
 * the Tiled NATTEN line of Table 2).  Not part of the STA path.
 *   mask_kind = STA_MASK_STA:    window = H*3 window sizes in TILES; same result as sta_forward (to rounding).
 *   mask_kind = STA_MASK_NATTEN: window = H*3 window sizes in TOKENS; the token-granular sliding window of the
 *     appendix algorithm "Mask Definition of 3D NATTEN" on the tile-ordered tensors: per axis the window centre
 *     is the query coordinate clamped into [floor(W/2), L-1-floor(W/2)], kept keys lie within floor(W/2) of it.
 *     Key tiles no query of the tile keeps are skipped, tiles every query keeps in full run without a mask, the
 *     others evaluate the predicate per score.  Tiles of at most 1024 tokens.
 * Tensors, layout, scale, stream and errors as sta_forward.  Supported: D in {64, 128}, P a multiple of 32.
 */
int sta_forward_general(const void *q_tiled, const void *k_tiled, const void *v_tiled,
                        void *o_tiled, int B, int H, int D, const int grid[3],
                        const int tile[3], int mask_kind, const int *window, float scale,
                        void *hip_stream);

/*
 * Window in tokens (the paper's notation, e.g. (18,24,24)) -> window in
 * tiles.  STA_ERR_WINDOW unless every entry is a positive multiple of the
 * tile size (Sec. 3.1 assumes W is an integer multiple of T).
 */
int sta_window_tokens_to_tiles(const int window_tokens[3], const int tile[3],
                               int out_tiles[3]);

/*
 * Work model used for reporting (Sec. 4.1 counts only kept blocks):
 * 4 * P^2 * D flop per (query tile, key tile) pair, summed over heads and
 * batch.  Returns 0.0 on invalid arguments.
 */
double sta_kept_flops(int B, int H, int D, const int grid[3], const int tile[3],
                      const int *window_tiles);

const char *sta_strerror(int status);
int sta_version(void);

#ifdef __cplusplus
}
#endif
#endif /* STA_H */
