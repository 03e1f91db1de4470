// Internal declarations shared by the translation units of libsta (GPU side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sta {

// ---- permutation -----------------------------------------------------------
struct PermuteParams {
    uint32_t N;                 // tokens per (b,h) slice
    uint32_t cpr;               // 8-element chunks per token row (D / 8)
    uint32_t L_h, L_w;          // grid
    uint32_t T_t, T_h, T_w;     // tile
    uint32_t n_h, n_w;          // tile grid (h, w)
    uint32_t n_tiles;
    uint32_t chunks_per_tile;   // P * cpr
    uint32_t seg, seg_magic;    // T_w * cpr chunks per contiguous run, ceil(2^32/seg)
    uint32_t T_h_magic;         // ceil(2^32 / T_h)
    uint32_t parts;             // workgroups per tile
    uint32_t span;              // chunks per workgroup (the last one of a tile may get fewer)
};

constexpr uint32_t kPermuteChunksPerBlock = 1024;   // 256 lanes x 4 chunks of 16 bytes

hipError_t launch_permute(const void *src, void *dst, bool src_f32, bool dst_f32, bool to_tiled,
                          const PermuteParams &p, uint32_t blocks, hipStream_t stream);

// ---- attention -------------------------------------------------------------
constexpr int kMaxHeadsPerLaunch = 256;

struct WindowTable {
    uint16_t w[kMaxHeadsPerLaunch][3];   // window in tiles per head of this launch (clamped to 2*n)
};

// Heads of one launch in the order the kernel visits them (most expensive first).
struct HeadOrder {
    uint16_t h[kMaxHeadsPerLaunch];
};

struct FwdParams {
    uint32_t N;            // tokens per head
    uint32_t P;            // tokens per tile
    uint32_t n_t, n_h, n_w;
    uint32_t n_tiles;
    uint32_t H;            // heads in the tensor
    uint32_t head_base;    // first head of this launch
    uint32_t heads;        // heads in this launch
    float scale_log2e;     // softmax scale * log2(e)
    uint32_t T_t = 1, T_h = 1, T_w = 1;   // tile shape in tokens (used by the token-masked sliding-window kernel only)
    float *lse = nullptr;  // optional output [B,H,N] (tiled order): ln of each row's softmax denominator; may be null
    // work splitting below one query block (filled in by the launcher): item ids from split_first on are run
    // by split_parts workgroups each, which leave partial results in split_ws
    uint32_t split_first = 0xffffffffu;
    uint32_t split_parts = 1;
    float *split_ws = nullptr;
};

// Returns hipErrorInvalidValue if no kernel instance exists for (P, D).
// split_ws: optional device scratch for work splitting (null: every item is run by one workgroup).
hipError_t launch_forward(const void *q, const void *k, const void *v, void *o, int B, int D,
                          const FwdParams &p, const WindowTable &win, const HeadOrder &order, float *split_ws,
                          size_t split_ws_floats, hipStream_t stream);
size_t forward_split_workspace_bytes(int P, int D);    // upper bound of what the splitting ever uses
// The general (register-staged) kernel for any supported shape.  token_window = false: the STA mask, win in tiles
// (same results as launch_forward).  token_window = true: the token-granular sliding window, win in tokens.
hipError_t launch_forward_general(const void *q, const void *k, const void *v, void *o, int B, int D, const FwdParams &p,
                                  const WindowTable &win, bool token_window, hipStream_t stream);
constexpr uint32_t kMaxTokenWindowTile = 1024;         // tokens per tile the sliding-window kernel's table holds
bool forward_supported(int P, int D);

// ---- gradients ---------------------------------------------------------------
// delta: float [B, H, N] scratch (dO_i . O_i per query row), filled by the call when compute_delta is set.
hipError_t launch_backward(const void *q, const void *k, const void *v, const void *o, const void *d_o, const float *lse,
                           float *delta, bool compute_delta, void *d_q, void *d_k, void *d_v, int B, int D,
                           const FwdParams &p, const WindowTable &win, hipStream_t stream);
bool backward_supported(int P, int D);

// ---- reductions around the attention kernel ----------------------------------
constexpr int kMseSlices = 64;     // partial sums per (batch, head) slab
hipError_t launch_head_mse(const void *a, const void *b, int B, int H, size_t elems_per_head, double *partial,
                           float *mse_per_head, hipStream_t stream);
// Allocation-free variant: the partial sums live in a file-scope device array of kStaticMseMaxSlabs * kMseSlices
// doubles.  static_mse_scratch returns the current device's address of that array (looked up once per device).
constexpr int kStaticMseMaxSlabs = 1024;
hipError_t static_mse_scratch(double **out);
hipError_t launch_first_min(const float *losses, int n_patterns, int H, int32_t *best, hipStream_t stream);
hipError_t launch_recall(const float *lse_window, const float *lse_full, int BH, size_t N, float *recall,
                         double *partial, float *mean_bh, hipStream_t stream);

// 16 MFMAs per wave per iteration, 4 waves per workgroup; operands: 16 KB of bf16; sink: workgroups*256 floats.

hipError_t launch_dump_key_tiles(const FwdParams &p, const WindowTable &win, int32_t *counts,
                                 int32_t *lists, hipStream_t stream);

}  // namespace sta
