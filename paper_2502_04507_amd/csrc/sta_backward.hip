// Gradients of Sliding Tile Attention for gfx950 (MI355X): dQ, dK, dV of Eq. 1 under the STA mask, for the
// finetuning use of the paper (Sec. 3.2 trains through STA layers).  The paper gives no backward kernel; this
// is the chain rule of Eq. 1 evaluated block by block over the kept (query tile, key tile) pairs only:
//
//   P_ij  = exp(S_ij - lse_i)          S = Q K^T * scale, lse_i = ln sum_j exp(S_ij) from the forward pass
//   dV_j  = sum_i P_ij dO_i
//   dP_ij = dO_i . V_j
//   dS_ij = P_ij (dP_ij - delta_i)     delta_i = dO_i . O_i
//   dQ_i  = scale * sum_j dS_ij K_j    dK_j = scale * sum_i dS_ij Q_i
//
// Three kernels, no atomics, results repeatable:
//   sta_bwd_delta_kernel  -delta_i and -lse_i / scale for every query row (HBM-bound, reads O and dO once);
//   sta_bwd_dq_kernel     one workgroup per query block, walks the key tiles of its window (as the forward
//                         kernel does): 3 MFMA products per block (K Q^T, V dO^T, K^T dS^T);
//   sta_bwd_dkv_kernel    one workgroup per key block, walks the QUERY tiles that keep its key tile (the
//                         transposed box): 4 MFMA products per block (Q K^T, dO V^T, dO^T P, Q^T dS), split
//                         over pairs of waves.
// S and dP are thus computed twice (7 products against the 5 of a single-pass scheme with atomics on dQ).
//
// Same MFMA formulation as the forward kernel (v_mfma_f32_16x16x32_bf16, the shape that costs the least energy per
// flop on this power-limited chip): the block is held so that one lane owns one column (a query in the dQ kernel,
// a key in the dK/dV kernel), and the bf16-rounded P or dS goes from the accumulators straight into the B operand
// of the next product, the contraction index being fed in accumulator order.  Staged operands are brought in by
// global_load_lds; an operand may be read both by rows (A rows = tokens, 16-byte reads) and transposed (A rows =
// channels, ds_read_b64_tr_b16), and one LDS layout serves both without bank conflicts (described where the two
// products are defined).
// These kernels: head dimension 64 or 128, tokens per tile a multiple of 128.  Other shapes (tiles that are other
// multiples of 32 tokens) go through the simple kernels further down.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sta_device_util.h"
#include "sta_geometry.h"
#include "sta_internal.h"

namespace {

constexpr int kSub = 32;               // tokens per staged sub-block
constexpr int kNW = 4;                 // waves per workgroup, 32 columns each
constexpr int kCols = kNW * 32;        // queries (dQ kernel) or keys (dK/dV kernel) per workgroup
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Walks the sub-blocks of the tiles of a box; next_row is the first token row (tiled order, inside the head) of
// the sub-block to request next.  Along each axis the box [lo, hi] holds e = hi-lo+1 consecutive tiles, hence
// one tile of every residue class mod e; they are taken in the order of that residue, i.e. the walk starts
// inside the box and wraps from hi to lo.  Neighbouring workgroups, whose boxes are shifted by one tile, then
// reach the tiles they share at the same step of their walks and find them in their XCD's L2.
struct BoxWalk {
    StaBox box;
    int n_h, n_w, P, sub_per_tile;
    int e_h, e_w, start_h, start_w, left_h, left_w;
    int t, h, w, s;
    uint32_t next_row;
    __device__ __forceinline__ static int first_of(const StaAxisRange &r)      // the tile of the box with k mod e == 0
    {
        const int e = r.hi - r.lo + 1;
        return r.lo + (e - r.lo % e) % e;
    }
    __device__ __forceinline__ void start(const StaBox &b, int nh, int nw, int tokens_per_tile)
    {
        box = b; n_h = nh; n_w = nw; P = tokens_per_tile; sub_per_tile = tokens_per_tile / kSub;
        e_h = b.h.hi - b.h.lo + 1; e_w = b.w.hi - b.w.lo + 1;
        start_h = first_of(b.h); start_w = first_of(b.w);
        t = first_of(b.t); h = start_h; w = start_w; s = 0;
        left_h = e_h; left_w = e_w;
        next_row = tile_row();
    }
    __device__ __forceinline__ uint32_t tile_row() const { return (uint32_t)(((t * n_h + h) * n_w + w) * P); }
    __device__ __forceinline__ void advance()
    {
        next_row += kSub;
        if (++s == sub_per_tile) {
            s = 0;
            if (++w > box.w.hi) w = box.w.lo;
            if (--left_w == 0) {
                left_w = e_w;
                w = start_w;
                if (++h > box.h.hi) h = box.h.lo;
                if (--left_h == 0) {
                    left_h = e_h;
                    h = start_h;
                    if (++t > box.t.hi) t = box.t.lo;
                }
            }
            next_row = tile_row();
        }
    }
};

// Work item of a workgroup.  The hardware deals workgroup ids round-robin over the 8 XCDs (each with its own
// L2).  The launch's column blocks, taken head after head, are cut into chunks of `chunk` consecutive blocks and
// the chunks are dealt to the XCDs in turn: the blocks resident on one XCD at a time are then neighbours that
// share most of their windows, while all XCDs together still work on one region of one head.
// Returns false for the padding ids of the launch.
__device__ __forceinline__ bool work_item(uint32_t chunk, uint32_t blocks_per_head, uint32_t n_bh, uint32_t *block,
                                          uint32_t *bh_rank)
{
    const uint32_t xcd = blockIdx.x & 7, s = blockIdx.x >> 3;
    const uint32_t linear = ((s / chunk) * 8 + xcd) * chunk + s % chunk;
    if (linear >= blocks_per_head * n_bh) return false;
    *bh_rank = linear / blocks_per_head;
    *block = linear - *bh_rank * blocks_per_head;
    return true;
}

// ---------------------------------------------------------------------------------------------------------
// Row statistics in the form the two kernels below start their accumulators with: neg_delta_i = -(dO_i . O_i)
// and neg_lse_i = -lse_i / scale, so that the matrix instructions deliver dP - delta and S - lse / scale and
// neither a subtraction nor a fused multiply-add per element is left (P = 2^(scale * log2(e) * (S - lse / scale))).
// One group of D / 8 lanes per row (each lane 16 bytes of it).
// ---------------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void sta_bwd_delta_kernel(const uint4 *__restrict__ o, const uint4 *__restrict__ d_o,
                                                            const float *__restrict__ lse, float inv_scale,
                                                            float *__restrict__ neg_delta, float *__restrict__ neg_lse,
                                                            size_t rows)
{
    constexpr int LPR = D / 8;                          // lanes per row
    const size_t row = (size_t)blockIdx.x * (256 / LPR) + (threadIdx.x / LPR);
    const int part = threadIdx.x % LPR;
    float acc = 0.f;
    if (row < rows) {
        const uint4 a = o[row * LPR + part], b = d_o[row * LPR + part];
        const uint32_t as[4] = {a.x, a.y, a.z, a.w}, bs[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = fmaf(__uint_as_float(as[e] << 16), __uint_as_float(bs[e] << 16), acc);
            acc = fmaf(__uint_as_float(as[e] & 0xffff0000u), __uint_as_float(bs[e] & 0xffff0000u), acc);
        }
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, LPR);
    if (row < rows && part == 0) {
        neg_delta[row] = -acc;
        neg_lse[row] = -lse[row] * inv_scale;
    }
}

__device__ __forceinline__ void lds_write_b128(uint32_t addr, bf16x8 v)
{
    asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v) : "memory");
}

// ---------------------------------------------------------------------------------------------------------
// Staged operands and the two kinds of product.  Register layout of v_mfma_f32_16x16x32_bf16: a lane holds column
// c16 = lane & 15 of a 16x16 result and the rows 4*g4 .. 4*g4+3 (g4 = lane >> 4); of an operand it holds row/column
// c16 and the k-chunk 8*g4 .. 8*g4+7.  A wave's 32 columns are two blocks of 16, and every fragment read from LDS
// feeds both.
// LDS layout of a staged operand (32 token rows).  A DMA instruction fills 1 KB, and a lane's place in it is fixed
// (16 * lane), so any swizzle is applied on the global side: the lane fetches the chunk that belongs at its place.
//  Head dimension 128 (rows of 256 bytes = all 64 banks): groups of 4 rows, 1024 + 32 bytes apart, chunk c of row j
//  of a group at c ^ (j << 2).
//  - by rows (16-byte reads, served for lanes 0-7 together with 24-31, i.e. rows 0..7 at chunk x with rows 8..15
//    at chunk x ^ 1): the four rows of a group land in the four quarters of the 256 bytes, and consecutive groups
//    are turned by 32 bytes, which together with the odd chunk of the second half covers all sixteen positions;
//  - transposed (8-byte reads, served 32 lanes at a time: 8 consecutive rows, two neighbouring chunks each).
//  The stage, the operand, the row block of a row read and the odd channel blocks of a transposing read are
//  offsets inside the instructions: a wave keeps four row addresses (one per k-step) and four transposing ones.
//  Head dimension 64 (rows of 128 bytes, two rows span the banks): rows 128 bytes apart without padding, chunk c of
//  row r at c ^ (((r >> 1) & 3) << 1).
//  - by rows: even rows sit in the lower 128 bytes of a bank line and odd rows in the upper; rows 0, 2, 4, 6 at chunk
//    x take the four even positions of their half, rows 8, 10, 12, 14 at chunk x ^ 1 the four odd ones;
//  - transposed: rows 0, 2, 4, 6 take four different 32-byte pairs of their half, rows 1, 3, 5, 7 the same of theirs.
//  A wave keeps two row addresses (one per k-step) and four transposing ones (one per channel block).
// In both layouts no address is computed inside the loop.
// ---------------------------------------------------------------------------------------------------------
template <int D>
struct Staged {
    static_assert(D == 64 || D == 128, "head dimension");
    static constexpr int RowB = 2 * D;                          // bytes per token row
    static constexpr int KS = D / 32;                           // k-steps of a product over the channels
    static constexpr int CB = D / 16;                           // 16-channel blocks of an accumulator
    static constexpr int GroupRows = 1024 / RowB;               // rows per DMA instruction: 4 or 8
    static constexpr int Groups = kSub / GroupRows;             // DMA instructions per operand: 8 or 4
    static constexpr int Group = D == 128 ? 1024 + 32 : 1024;   // bytes from one group to the next
    static constexpr int Tile = Groups * Group;                 // one staged operand
    static constexpr int Rows16 = (16 / GroupRows) * Group;     // from row r to row r + 16

    // where the 16-byte chunk c of row r (0..31) of a staged operand sits, in bytes from its start
    static __device__ __forceinline__ uint32_t place(int r, int c)
    {
        if constexpr (D == 128) return (uint32_t)((r >> 2) * Group + (r & 3) * RowB + ((c ^ ((r & 3) << 2)) << 4));
        else return (uint32_t)(r * RowB + ((c ^ (((r >> 1) & 3) << 1)) << 4));
    }
    // byte offset, inside a DMA group of the source (GroupRows rows, contiguous), of what the lane fetches
    static __device__ __forceinline__ uint32_t dma_lane_offset(int lane)
    {
        constexpr int LPR = RowB / 16;                          // lanes (chunks) per row
        const int r = lane / LPR, pos = lane % LPR;             // row inside the group, place inside the row
        if constexpr (D == 128) return (uint32_t)(r * RowB + ((pos ^ (r << 2)) << 4));
        else return (uint32_t)(r * RowB + ((pos ^ (((r >> 1) & 3) << 1)) << 4));   // groups start at multiples of 8 rows
    }
    // Per-lane addresses of the operand reads, relative to the start of a staged operand at LDS address `base`.
    //  Row reads (A = 16 tokens x 32 channels): token row c16 (+16 for the second row block), chunk 4*ks + g4.
    //  Transposing reads (A = 16 channels x 32 tokens): within each block of 16 lanes, lane 4*j4 + s4 supplies
    //  channels 4*s4 .. 4*s4+3 of the block's 16 of token row 4*g4 + j4 (+16 for the second read); chunk
    //  2*cb + (s4 >> 1).  With 256-byte rows the XOR reaches cb >> 1 only (cb & 1 is 32 bytes in the instruction),
    //  with 128-byte rows it reaches all of cb: four addresses either way.
    static __device__ __forceinline__ void addresses(uint32_t base, int lane, uint32_t (&row_addr)[KS], uint32_t (&tr_addr)[4])
    {
        const int c16 = lane & 15, g4 = lane >> 4, j4 = c16 >> 2, s4 = lane & 3;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) row_addr[ks] = base + place(c16, 4 * ks + g4);
#pragma unroll
        for (int m = 0; m < 4; ++m)
            tr_addr[m] = base + place(4 * g4 + j4, (D == 128 ? 4 * m : 2 * m) + (s4 >> 1)) + 8 * (s4 & 1);
    }
    static constexpr int tr_index(int cb) { return D == 128 ? cb >> 1 : cb; }
    static constexpr int tr_offset(int cb) { return D == 128 ? (cb & 1) * 32 : 0; }
};

// X[rb][col] (16 staged rows x 16 resident columns) += A B: A = the staged operand at byte offset OFF read by rows
// (k = channels), B = resident fragments of the wave's 32 columns; the caller has set X to the value the sums start
// from.  Four reads in flight; a fragment feeds both column blocks, taken 0, 1, 1, 0, .. so that one operand changes
// from one matrix instruction to the next.
template <int D, int OFF>
__device__ __forceinline__ void staged_rows_times_resident(const uint32_t (&row_addr)[D / 32],
                                                           const bf16x8 (&resident)[2][D / 32], floatx4 (&X)[2][2])
{
    constexpr int ROWS16 = OFF + Staged<D>::Rows16;             // rows 16..31
    if constexpr (D == 128) {
        bf16x8 a0 = ds_read_b128_at<OFF>(row_addr[0]), a1 = ds_read_b128_at<OFF>(row_addr[1]);
        bf16x8 a2 = ds_read_b128_at<OFF>(row_addr[2]), a3 = ds_read_b128_at<OFF>(row_addr[3]);
        lds_wait2<2>(a0, a1);
#pragma unroll
        for (int col = 0; col < 2; ++col) X[0][col] = mfma_16x16x32(a0, resident[col][0], X[0][col]);
#pragma unroll
        for (int col = 1; col >= 0; --col) X[0][col] = mfma_16x16x32(a1, resident[col][1], X[0][col]);
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 b0 = ds_read_b128_at<ROWS16>(row_addr[0]), b1 = ds_read_b128_at<ROWS16>(row_addr[1]);
        lds_wait2<2>(a2, a3);
#pragma unroll
        for (int col = 0; col < 2; ++col) X[0][col] = mfma_16x16x32(a2, resident[col][2], X[0][col]);
#pragma unroll
        for (int col = 1; col >= 0; --col) X[0][col] = mfma_16x16x32(a3, resident[col][3], X[0][col]);
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 b2 = ds_read_b128_at<ROWS16>(row_addr[2]), b3 = ds_read_b128_at<ROWS16>(row_addr[3]);
        lds_wait2<2>(b0, b1);
#pragma unroll
        for (int col = 0; col < 2; ++col) X[1][col] = mfma_16x16x32(b0, resident[col][0], X[1][col]);
#pragma unroll
        for (int col = 1; col >= 0; --col) X[1][col] = mfma_16x16x32(b1, resident[col][1], X[1][col]);
        __builtin_amdgcn_sched_barrier(0);
        lds_wait2<0>(b2, b3);
#pragma unroll
        for (int col = 0; col < 2; ++col) X[1][col] = mfma_16x16x32(b2, resident[col][2], X[1][col]);
#pragma unroll
        for (int col = 1; col >= 0; --col) X[1][col] = mfma_16x16x32(b3, resident[col][3], X[1][col]);
        __builtin_amdgcn_sched_barrier(0);
    } else {
        bf16x8 a0 = ds_read_b128_at<OFF>(row_addr[0]), a1 = ds_read_b128_at<OFF>(row_addr[1]);
        bf16x8 b0 = ds_read_b128_at<ROWS16>(row_addr[0]), b1 = ds_read_b128_at<ROWS16>(row_addr[1]);
        lds_wait2<2>(a0, a1);
#pragma unroll
        for (int col = 0; col < 2; ++col) X[0][col] = mfma_16x16x32(a0, resident[col][0], X[0][col]);
#pragma unroll
        for (int col = 1; col >= 0; --col) X[0][col] = mfma_16x16x32(a1, resident[col][1], X[0][col]);
        __builtin_amdgcn_sched_barrier(0);
        lds_wait2<0>(b0, b1);
#pragma unroll
        for (int col = 0; col < 2; ++col) X[1][col] = mfma_16x16x32(b0, resident[col][0], X[1][col]);
#pragma unroll
        for (int col = 1; col >= 0; --col) X[1][col] = mfma_16x16x32(b1, resident[col][1], X[1][col]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// acc[cb][col] (16 channels x 16 resident columns) += A B: A = the staged operand at OFF read transposed (A rows =
// channels, k = its 32 rows: index 8*g4 + i is row 4*g4 + i of the first 16 for i < 4, of the second 16 otherwise),
// B = packed[col].  The reads of channel blocks 0..3 can go out before B exists.
template <int D, int OFF>
struct StagedTransposedProduct {
    static constexpr int CB = D / 16;                   // channel blocks: read four at a time
    static constexpr int NG = CB / 4;
    shortx4 frag[NG][4][2];
    template <int G>
    __device__ __forceinline__ void issue(const uint32_t (&tr_addr)[4])
    {
        static_for<0, 4>([&](auto i) {
            constexpr int cb = 4 * G + decltype(i)::value;
            constexpr int at = OFF + Staged<D>::tr_offset(cb);
            frag[G][cb & 3][0] = ds_read_tr16<at>(tr_addr[Staged<D>::tr_index(cb)]);
            frag[G][cb & 3][1] = ds_read_tr16<at + Staged<D>::Rows16>(tr_addr[Staged<D>::tr_index(cb)]);
        });
    }
    __device__ __forceinline__ void prefetch(const uint32_t (&tr_addr)[4]) { issue<0>(tr_addr); }
    __device__ __forceinline__ void run(const uint32_t (&tr_addr)[4], const bf16x8 (&packed)[2], floatx4 (&acc)[CB][2])
    {
        typedef short shortx8 __attribute__((ext_vector_type(8)));
        static_for<0, NG>([&](auto gi) {
            constexpr int g = decltype(gi)::value;
            if constexpr (g + 1 < NG) {
                issue<g + 1>(tr_addr);
                pv_wait<8>(frag[g]);
            } else {
                pv_wait<0>(frag[g]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const shortx8 a = __builtin_shufflevector(frag[g][i][0], frag[g][i][1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int col = (i & 1) ^ t;
                    acc[4 * g + i][col] = mfma_16x16x32(__builtin_bit_cast(bf16x8, a), packed[col], acc[4 * g + i][col]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    }
};

// ---------------------------------------------------------------------------------------------------------
// dQ.  One workgroup of 4 waves per 128 queries (two workgroups per CU at head dimension 128, 206 registers); a lane
// holds query column c16 of its wave's two 16-query blocks.  LDS stage: K (read by rows and transposed) and V (read by
// rows), in the layout described above.  Per wave and 32-key sub-block: S^T = K Q^T - lse / scale and
// dP^T = V dO^T - delta (the statistics of the lane's query as the initial value), dS^T = 2^(c S^T) o dP^T,
// dQ^T += K^T dS^T; 16 matrix instructions each at head dimension 128, 8 at 64.
// ---------------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kNW * 64, 2) void sta_bwd_dq_kernel(const bf16_raw *__restrict__ q,
                                                                 const bf16_raw *__restrict__ k,
                                                                 const bf16_raw *__restrict__ v,
                                                                 const bf16_raw *__restrict__ d_o,
                                                                 const float *__restrict__ neg_lse,
                                                                 const float *__restrict__ neg_delta,
                                                                 bf16_raw *__restrict__ d_q, sta::FwdParams p,
                                                                 sta::WindowTable win, uint32_t n_bh, uint32_t chunk)
{
    using L = Staged<D>;
    constexpr int KS = L::KS, CB = L::CB;
    constexpr int STAGE_B = 2 * L::Tile;
    constexpr int K_TILE = 0, V_TILE = L::Tile;
    constexpr int LOADS = L::Groups / kNW;              // DMA instructions per operand and wave: 2 or 1
    __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE_B];

    uint32_t qblock, bh_rank;
    if (!work_item(chunk, p.N / kCols, n_bh, &qblock, &bh_rank)) return;
    const uint32_t heads = p.heads;
    const uint32_t h_local = bh_rank % heads, b = bh_rank / heads;
    const size_t bh = (size_t)b * p.H + p.head_base + h_local;
    const uint32_t q_tile = (qblock * kCols) / p.P;
    const StaBox box = sta_key_tile_box_of(p.n_t, p.n_h, p.n_w, win.w[h_local][0], win.w[h_local][1], win.w[h_local][2],
                                           q_tile);
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, c16 = lane & 15, g4 = lane >> 4;

    const size_t my_row = bh * p.N + (size_t)qblock * kCols + (size_t)wave * 32;
    const char *kh = reinterpret_cast<const char *>(k + bh * p.N * D);
    const char *vh = reinterpret_cast<const char *>(v + bh * p.N * D);

    // DMA: each operand is L::Groups instructions of 1 KB; wave w issues the groups LOADS * w .. of each.
    const uint32_t src_lane_off = L::dma_lane_offset(lane);
    auto issue_loads = [&](int stage, uint32_t first_row) {
        uint32_t off = src_lane_off;
        asm volatile("" : "+v"(off));                   // keep the lane offset 32-bit next to a scalar base
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int group = LOADS * wave + i;
            const size_t base = (size_t)(first_row + L::GroupRows * group) * L::RowB;
            char *dst = smem + stage * STAGE_B + group * L::Group;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kh + base + off),
                                             STA_LDS_PTR(dst + K_TILE), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(vh + base + off),
                                             STA_LDS_PTR(dst + V_TILE), 16, 0, 0);
        }
    };

    uint32_t row_addr[KS], tr_addr[4];
    L::addresses((uint32_t)(uintptr_t)smem, lane, row_addr, tr_addr);

    // resident B fragments: query 16*qb + c16, channels 32*ks + 8*g4 ..
    bf16x8 Qr[2][KS], Gr[2][KS];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const size_t at = (my_row + 16 * qb + c16) * D + ks * 32 + g4 * 8;
            Qr[qb][ks] = *reinterpret_cast<const bf16x8 *>(q + at);
            Gr[qb][ks] = *reinterpret_cast<const bf16x8 *>(d_o + at);
        }
    const float c = p.scale_log2e;
    // a lane owns one query column per block: the four registers of an accumulator all start at that query's statistic
    floatx4 s_init[2], dp_init[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float a = neg_lse[my_row + 16 * qb + c16], d = neg_delta[my_row + 16 * qb + c16];
        s_init[qb] = floatx4{a, a, a, a};
        dp_init[qb] = floatx4{d, d, d, d};
    }

    floatx4 dQ[CB][2];                                  // [channel block][query block]
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) dQ[cb][qb] = floatx4{0.f, 0.f, 0.f, 0.f};

    BoxWalk walk;
    walk.start(box, p.n_h, p.n_w, p.P);
    const int n_iter = box.count() * walk.sub_per_tile;
    int issued = 0;
    auto issue_next = [&]() {
        if (issued < n_iter) {
            issue_loads(issued & 1, walk.next_row);
            walk.advance();
            ++issued;
        }
    };
    issue_next();

    auto sub_block = [&](auto stage_c) {
        constexpr int ST = decltype(stage_c)::value * STAGE_B;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        issue_next();
        floatx4 S[2][2], dP[2][2];                      // [key block][query block]
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                S[kb][qb] = s_init[qb];
                dP[kb][qb] = dp_init[qb];
            }
        staged_rows_times_resident<D, ST + K_TILE>(row_addr, Qr, S);    // K Q^T - lse / scale
        staged_rows_times_resident<D, ST + V_TILE>(row_addr, Gr, dP);   // V dO^T - delta
        StagedTransposedProduct<D, ST + K_TILE> k_t;
        k_t.prefetch(tr_addr);
        __builtin_amdgcn_sched_barrier(0);
        // dS^T, rounded to bf16 and packed as the B operand of the last product: k index 8*g4 + i is key 4*g4 + i
        // of the first key block (i < 4) or of the second
        bf16x8 dSb[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    dSb[qb][4 * kb + e] = static_cast<__bf16>(__builtin_amdgcn_exp2f(S[kb][qb][e] * c) * dP[kb][qb][e]);
        k_t.run(tr_addr, dSb, dQ);                                       // dQ^T += K^T dS^T
    };
    for (int iter = 0; iter < n_iter; iter += 2) {
        sub_block(std::integral_constant<int, 0>{});
        if (iter + 1 < n_iter) sub_block(std::integral_constant<int, 1>{});
    }
    // dQ[cb][qb][i] = channel 16*cb + 4*g4 + i of query 16*qb + c16
    const float mul = c * kLn2;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            bf16x4 ov;
#pragma unroll
            for (int t = 0; t < 4; ++t) ov[t] = static_cast<__bf16>(dQ[cb][qb][t] * mul);
            *reinterpret_cast<bf16x4 *>(d_q + (my_row + 16 * qb + c16) * D + 16 * cb + 4 * g4) = ov;
        }
}

// ---------------------------------------------------------------------------------------------------------
// dK, dV.  One workgroup of 2 * NPAIR waves per 32 * NPAIR keys.  Each 32-key column block is served by a PAIR of
// waves: the first holds K and accumulates dV (S = Q K^T, P, dV^T += dO^T P), the second holds V and accumulates dK
// (dP = dO V^T, dS = P o (dP - delta), dK^T += Q^T dS).  P, rounded to bf16 and packed as the MFMA B operand, goes
// from the first to the second through 2 KB of LDS.  Four matrix products per block, no duplicate work inside the
// kernel, and each wave keeps one accumulator set: at head dimension 128, per wave and 32-query sub-block 32 matrix
// instructions, 40 vector instructions and 26 LDS reads in 158 registers, so that three waves per SIMD fit (six pairs:
// 192 keys per workgroup); at head dimension 64 it is 106 registers and two workgroups of four pairs share a CU.
// LDS stage: Q and dO (each read by rows and transposed) and the row statistics of the 32 queries.
// A lane holds key column c16 of its wave's two 16-key blocks and the query rows 4*g4 .. 4*g4+3 of a result.
// ---------------------------------------------------------------------------------------------------------
template <int D, int NPAIR>
__global__ __launch_bounds__(NPAIR * 128, (D == 64 && NPAIR == 4) ? 2 : 1) void sta_bwd_dkv_kernel(const bf16_raw *__restrict__ q,
                                                                     const bf16_raw *__restrict__ k,
                                                                     const bf16_raw *__restrict__ v,
                                                                     const bf16_raw *__restrict__ d_o,
                                                                     const float *__restrict__ neg_lse,
                                                                     const float *__restrict__ neg_delta,
                                                                     bf16_raw *__restrict__ d_k,
                                                                     bf16_raw *__restrict__ d_v, sta::FwdParams p,
                                                                     sta::WindowTable win, uint32_t n_bh, uint32_t chunk)
{
    using L = Staged<D>;
    constexpr int KS = L::KS, CB = L::CB;
    constexpr int COLS = NPAIR * 32;                    // keys per workgroup
    constexpr int STAGE_B = 2 * L::Tile;
    constexpr int Q_TILE = 0, G_TILE = L::Tile;
    constexpr int P_XCHG = 2 * STAGE_B;                 // per pair: 2 key blocks x 64 lanes x 16 B
    constexpr int STATS = P_XCHG + NPAIR * 2048;        // per stage: -lse / scale then -delta of the 32 staged query rows
    constexpr int STAT_B = 2 * kSub * 4;
    constexpr int DMA_WAVES = 8;                        // waves that bring the operands in
    constexpr int STAT_WAVE = 2 * NPAIR > DMA_WAVES ? DMA_WAVES : DMA_WAVES - 1;   // a wave of its own where there is one
    static_assert(2 * NPAIR >= DMA_WAVES, "eight loading waves");
    __shared__ __attribute__((aligned(1024))) char smem[STATS + 2 * STAT_B];

    uint32_t kblock, bh_rank;
    if (!work_item(chunk, p.N / COLS, n_bh, &kblock, &bh_rank)) return;
    const uint32_t heads = p.heads;
    const uint32_t h_local = bh_rank % heads, b = bh_rank / heads;
    const size_t bh = (size_t)b * p.H + p.head_base + h_local;
    const uint32_t k_tile = (kblock * COLS) / p.P;
    const StaBox box = sta_query_tile_box_of(p.n_t, p.n_h, p.n_w, win.w[h_local][0], win.w[h_local][1],
                                             win.w[h_local][2], k_tile);
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, c16 = lane & 15, g4 = lane >> 4;
    const bool probs_role = wave < NPAIR;               // S, P, dV; the other role: dP, dS, dK
    const int pair = probs_role ? wave : wave - NPAIR;

    const size_t head_row = bh * p.N;
    const size_t my_row = head_row + (size_t)kblock * COLS + (size_t)pair * 32;
    const char *qh = reinterpret_cast<const char *>(q + head_row * D);
    const char *gh = reinterpret_cast<const char *>(d_o + head_row * D);

    // DMA: each operand is L::Groups instructions of 1 KB.  Head dimension 128 (8 per operand): wave w < 8 issues
    // instruction w of each operand; head dimension 64 (4 per operand): waves 0..3 bring Q, waves 4..7 dO.  Wave 8
    // brings the row statistics of the sub-block (32 + 32 floats) with one 4-byte-per-lane instruction (wave 7 where
    // there are eight).
    const uint32_t src_lane_off = L::dma_lane_offset(lane);
    const uint32_t stat_lane_off = (uint32_t)((lane & (kSub - 1)) * 4);
    const char *stat_base = reinterpret_cast<const char *>((lane < kSub ? neg_lse : neg_delta) + head_row);
    auto issue_loads = [&](int stage, uint32_t first_row) {
        uint32_t off = src_lane_off, soff = stat_lane_off;
        asm volatile("" : "+v"(off), "+v"(soff));       // keep the lane offsets 32-bit next to a scalar base
        if (wave < DMA_WAVES) {
            const int group = D == 128 ? wave : (wave & 3);
            const size_t base = (size_t)(first_row + L::GroupRows * group) * L::RowB;
            char *dst = smem + stage * STAGE_B + group * L::Group;
            if (D == 128 || wave < 4)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(qh + base + off),
                                                 STA_LDS_PTR(dst + Q_TILE), 16, 0, 0);
            if (D == 128 || wave >= 4)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gh + base + off),
                                                 STA_LDS_PTR(dst + G_TILE), 16, 0, 0);
        }
        if (wave == STAT_WAVE)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(stat_base + (size_t)first_row * 4 + soff),
                STA_LDS_PTR(smem + STATS + stage * STAT_B), 4, 0, 0);
    };

    const uint32_t smem_addr = (uint32_t)(uintptr_t)smem;
    uint32_t row_addr[KS], tr_addr[4];
    L::addresses(smem_addr, lane, row_addr, tr_addr);
    const uint32_t xchg_addr = smem_addr + P_XCHG + pair * 2048 + lane * 16;   // two planes of 1 KB per pair
    const uint32_t stat_addr = smem_addr + STATS + (probs_role ? 0 : kSub * 4) + 16 * g4;

    // resident B fragments: K rows (first role) or V rows (second role) of key 16*kb + c16, channels 32*ks + 8*g4 ..
    bf16x8 resident[2][KS];
    {
        const bf16_raw *rows = (probs_role ? k : v) + my_row * D;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                resident[kb][ks] = *reinterpret_cast<const bf16x8 *>(rows + (size_t)(16 * kb + c16) * D + ks * 32 + g4 * 8);
    }
    const float c = p.scale_log2e;

    floatx4 acc[CB][2];                                 // dV^T (first role) or dK^T (second role): [channel block][key block]
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) acc[cb][kb] = floatx4{0.f, 0.f, 0.f, 0.f};

    BoxWalk walk;
    walk.start(box, p.n_h, p.n_w, p.P);
    const int n_iter = box.count() * walk.sub_per_tile;
    int issued = 0;
    auto issue_next = [&]() {
        if (issued < n_iter) {
            issue_loads(issued & 1, walk.next_row);
            walk.advance();
            ++issued;
        }
    };
    issue_next();

    // One sub-block in one role.  (The role is a compile-time argument and each role has its own loop: with the
    // branch inside a common loop the register allocator serves both paths at once and spills.)
    auto sub_block = [&](auto role_c, auto stage_c) {
        constexpr bool PROBS = decltype(role_c)::value;
        constexpr int ST = decltype(stage_c)::value * STAGE_B;
        constexpr int ST_STATS = decltype(stage_c)::value * STAT_B;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();       // the stage is complete; the other stage and the exchange buffer are free
        issue_next();
        // the accumulators of the first product start at the statistics of their query rows 16*qb + 4*g4 ..
        floatx4 init[2];
        {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            u32x4 r0, r1;
            asm volatile("ds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(r0), "=&v"(r1)
                         : "v"(stat_addr), "n"(ST_STATS), "n"(ST_STATS + 64));
            init[0] = __builtin_bit_cast(floatx4, r0);
            init[1] = __builtin_bit_cast(floatx4, r1);
        }
        floatx4 X[2][2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) X[qb][kb] = init[qb];
        if constexpr (PROBS) {
            staged_rows_times_resident<D, ST + Q_TILE>(row_addr, resident, X);      // Q K^T - lse / scale
            StagedTransposedProduct<D, ST + G_TILE> g_t;
            g_t.prefetch(tr_addr);
            __builtin_amdgcn_sched_barrier(0);
            bf16x8 Pb[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        Pb[kb][4 * qb + e] = static_cast<__bf16>(__builtin_amdgcn_exp2f(X[qb][kb][e] * c));
            lds_write_b128(xchg_addr, Pb[0]);
            lds_write_b128(xchg_addr + 1024, Pb[1]);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            g_t.run(tr_addr, Pb, acc);                                              // dV^T += dO^T P
        } else {
            staged_rows_times_resident<D, ST + G_TILE>(row_addr, resident, X);      // dO V^T - delta
            StagedTransposedProduct<D, ST + Q_TILE> q_t;
            q_t.prefetch(tr_addr);
            __builtin_amdgcn_s_barrier();
            bf16x8 Pb[2];
            Pb[0] = ds_read_b128_at<0>(xchg_addr);
            Pb[1] = ds_read_b128_at<1024>(xchg_addr);
            lds_wait2<0>(Pb[0], Pb[1]);
            bf16x8 dSb[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        dSb[kb][4 * qb + e] = static_cast<__bf16>(static_cast<float>(Pb[kb][4 * qb + e]) * X[qb][kb][e]);
            q_t.run(tr_addr, dSb, acc);                                             // dK^T += Q^T dS
        }
    };
    auto all_sub_blocks = [&](auto role_c) {
        for (int iter = 0; iter < n_iter; iter += 2) {
            sub_block(role_c, std::integral_constant<int, 0>{});
            if (iter + 1 < n_iter) sub_block(role_c, std::integral_constant<int, 1>{});
        }
    };
    if (probs_role) all_sub_blocks(std::true_type{});
    else all_sub_blocks(std::false_type{});
    // acc[cb][kb][i] = channel 16*cb + 4*g4 + i of key 16*kb + c16
    bf16_raw *dst = (probs_role ? d_v : d_k) + my_row * D;
    const float mul = probs_role ? 1.0f : c * kLn2;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            bf16x4 ov;
#pragma unroll
            for (int t = 0; t < 4; ++t) ov[t] = static_cast<__bf16>(acc[cb][kb][t] * mul);
            *reinterpret_cast<bf16x4 *>(dst + (size_t)(16 * kb + c16) * D + 16 * cb + 4 * g4) = ov;
        }
}


// ---------------------------------------------------------------------------------------------------------
// General shapes: head dimension 64 or 128, any tile size that is a multiple of 32 tokens.  Same mathematics and
// the same MFMA formulation (one lane owns one column, P or dS goes from the accumulators into the B operand),
// kept simple: one wave per workgroup and 32 columns, staged operands copied through registers into a
// row-major LDS block without swizzle (the row reads take bank conflicts), one sub-block at a time.  The fast
// kernels above take over where they apply.
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ void pack16(const float (&x)[16], bf16x8 (&out)[2])
{
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) out[j][e] = static_cast<__bf16>(x[8 * j + e]);
}

template <int D>
struct GenericOps {
    static constexpr int RowB = 2 * D;             // bytes per token row
    static constexpr int SubB = kSub * RowB;       // one staged operand
    static constexpr int KS = D / 16;              // k-steps of a product over the channels
    static constexpr int DB = D / 32;              // 32-channel blocks of an accumulator over the channels

    // One wave copies a 32-row sub-block (contiguous in global memory) to LDS, 16 bytes per lane and step.
    static __device__ __forceinline__ void copy_in(char *dst, const char *src, int lane)
    {
#pragma unroll
        for (int i = 0; i < SubB / 1024; ++i)
            *reinterpret_cast<uint4 *>(dst + i * 1024 + lane * 16) = *reinterpret_cast<const uint4 *>(src + i * 1024 + lane * 16);
    }
    // acc(32 x 32) = A B, A = staged sub-block read by rows (k = channels), B = resident fragments.
    static __device__ __forceinline__ floatx16 rows_times(const char *sub, int lane, const bf16x8 (&resident)[KS])
    {
        const int lo = lane & 31, hb = lane >> 5;
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(sub + lo * RowB + (2 * ks + hb) * 16);
            acc = mfma_32x32x16(a, resident[ks], acc);
        }
        return acc;
    }
    // acc[db](32 channels x 32 columns) += A B, A = staged sub-block read transposed (rows = channels, k = its 32
    // tokens in accumulator order), B = the two packed halves of an accumulator.
    static __device__ __forceinline__ void transposed_times(uint32_t sub_addr, int lane, const bf16x8 (&packed)[2],
                                                            floatx16 (&acc)[DB])
    {
        typedef short shortx8 __attribute__((ext_vector_type(8)));
        const int hb = lane >> 5, j4 = (lane & 15) >> 2, s4 = lane & 3, blk = (lane >> 4) & 1;
        const uint32_t base = sub_addr + (uint32_t)((4 * hb + j4) * RowB + (16 * blk + 4 * s4) * 2);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                shortx4 f0, f1;
                const uint32_t a = base + (uint32_t)(16 * j * RowB + 64 * db);
                asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %2 offset:%3\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(f0), "=&v"(f1)
                             : "v"(a), "n"(8 * RowB));
                const shortx8 a01 = __builtin_shufflevector(f0, f1, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[db] = mfma_32x32x16(__builtin_bit_cast(bf16x8, a01), packed[j], acc[db]);
            }
    }
    static __device__ __forceinline__ void load_resident(const bf16_raw *rows, int lane, bf16x8 (&frag)[KS])
    {
        const int lo = lane & 31, hb = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) frag[ks] = *reinterpret_cast<const bf16x8 *>(rows + (size_t)lo * D + ks * 16 + hb * 8);
    }
    static __device__ __forceinline__ void store_columns(bf16_raw *dst, int lane, const floatx16 (&acc)[DB], float mul)
    {
        const int lo = lane & 31, hb = lane >> 5;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 ov;
#pragma unroll
                for (int t = 0; t < 4; ++t) ov[t] = static_cast<__bf16>(acc[db][4 * g + t] * mul);
                *reinterpret_cast<bf16x4 *>(dst + (size_t)lo * D + db * 32 + g * 8 + hb * 4) = ov;
            }
    }
};

template <int D>
__global__ __launch_bounds__(256) void sta_bwd_delta_generic_kernel(const uint4 *__restrict__ o,
                                                                    const uint4 *__restrict__ d_o,
                                                                    float *__restrict__ delta, size_t rows)
{
    constexpr int LPR = D / 8;                     // lanes per row, 16 bytes each
    const size_t row = (size_t)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
    const int part = threadIdx.x % LPR;
    float acc = 0.f;
    if (row < rows) {
        const uint4 a = o[row * LPR + part], b = d_o[row * LPR + part];
        const uint32_t as[4] = {a.x, a.y, a.z, a.w}, bs[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = fmaf(__uint_as_float(as[e] << 16), __uint_as_float(bs[e] << 16), acc);
            acc = fmaf(__uint_as_float(as[e] & 0xffff0000u), __uint_as_float(bs[e] & 0xffff0000u), acc);
        }
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, LPR);
    if (row < rows && part == 0) delta[row] = acc;
}

// dQ of 32 queries: grid (N / 32, batch x heads of the launch).
template <int D>
__global__ __launch_bounds__(64) void sta_bwd_dq_generic_kernel(const bf16_raw *__restrict__ q,
                                                                const bf16_raw *__restrict__ k,
                                                                const bf16_raw *__restrict__ v,
                                                                const bf16_raw *__restrict__ d_o,
                                                                const float *__restrict__ lse,
                                                                const float *__restrict__ delta,
                                                                bf16_raw *__restrict__ d_q, sta::FwdParams p,
                                                                sta::WindowTable win)
{
    using G = GenericOps<D>;
    __shared__ __attribute__((aligned(1024))) char smem[2 * G::SubB];         // K, V
    const uint32_t qblock = blockIdx.x, bh_rank = blockIdx.y;
    const uint32_t h_local = bh_rank % p.heads, b = bh_rank / p.heads;
    const size_t bh = (size_t)b * p.H + p.head_base + h_local;
    const uint32_t q_tile = (qblock * kSub) / p.P;
    const StaBox box = sta_key_tile_box_of(p.n_t, p.n_h, p.n_w, win.w[h_local][0], win.w[h_local][1], win.w[h_local][2],
                                           q_tile);
    const int lane = threadIdx.x, lo = lane & 31;
    const size_t my_row = bh * p.N + (size_t)qblock * kSub;
    const char *kh = reinterpret_cast<const char *>(k + bh * p.N * D);
    const char *vh = reinterpret_cast<const char *>(v + bh * p.N * D);
    const uint32_t smem_addr = (uint32_t)(uintptr_t)smem;

    bf16x8 Qr[G::KS], Gr[G::KS];
    G::load_resident(q + my_row * D, lane, Qr);
    G::load_resident(d_o + my_row * D, lane, Gr);
    const float c = p.scale_log2e;
    const float lse2 = lse[my_row + lo] * kLog2e;
    const float dl = delta[my_row + lo];
    floatx16 dQ[G::DB];
#pragma unroll
    for (int db = 0; db < G::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dQ[db][r] = 0.f;

    BoxWalk walk;
    walk.start(box, p.n_h, p.n_w, p.P);
    const int n_iter = box.count() * walk.sub_per_tile;
    for (int iter = 0; iter < n_iter; ++iter) {
        __syncthreads();                                   // the previous sub-block has been read
        G::copy_in(smem, kh + (size_t)walk.next_row * G::RowB, lane);
        G::copy_in(smem + G::SubB, vh + (size_t)walk.next_row * G::RowB, lane);
        walk.advance();
        __syncthreads();
        const floatx16 S = G::rows_times(smem, lane, Qr);                      // S^T  = K Q^T (keys x queries)
        const floatx16 dP = G::rows_times(smem + G::SubB, lane, Gr);           // dP^T = V dO^T
        float ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) ds[r] = __builtin_amdgcn_exp2f(fmaf(S[r], c, -lse2)) * (dP[r] - dl);
        bf16x8 dSb[2];
        pack16(ds, dSb);
        G::transposed_times(smem_addr, lane, dSb, dQ);                         // dQ^T += K^T dS^T
    }
    G::store_columns(d_q + my_row * D, lane, dQ, c * kLn2);
}

// dK and dV of 32 keys: grid (N / 32, batch x heads of the launch); walks the query tiles that keep the key tile.
template <int D>
__global__ __launch_bounds__(64) void sta_bwd_dkv_generic_kernel(const bf16_raw *__restrict__ q,
                                                                 const bf16_raw *__restrict__ k,
                                                                 const bf16_raw *__restrict__ v,
                                                                 const bf16_raw *__restrict__ d_o,
                                                                 const float *__restrict__ lse,
                                                                 const float *__restrict__ delta,
                                                                 bf16_raw *__restrict__ d_k,
                                                                 bf16_raw *__restrict__ d_v, sta::FwdParams p,
                                                                 sta::WindowTable win)
{
    using G = GenericOps<D>;
    __shared__ __attribute__((aligned(1024))) char smem[2 * G::SubB];         // Q, dO
    const uint32_t kblock = blockIdx.x, bh_rank = blockIdx.y;
    const uint32_t h_local = bh_rank % p.heads, b = bh_rank / p.heads;
    const size_t bh = (size_t)b * p.H + p.head_base + h_local;
    const uint32_t k_tile = (kblock * kSub) / p.P;
    const StaBox box = sta_query_tile_box_of(p.n_t, p.n_h, p.n_w, win.w[h_local][0], win.w[h_local][1],
                                             win.w[h_local][2], k_tile);
    const int lane = threadIdx.x, hb = lane >> 5;
    const size_t head_row = bh * p.N;
    const size_t my_row = head_row + (size_t)kblock * kSub;
    const char *qh = reinterpret_cast<const char *>(q + head_row * D);
    const char *gh = reinterpret_cast<const char *>(d_o + head_row * D);
    const uint32_t smem_addr = (uint32_t)(uintptr_t)smem;

    bf16x8 Kr[G::KS], Vr[G::KS];
    G::load_resident(k + my_row * D, lane, Kr);
    G::load_resident(v + my_row * D, lane, Vr);
    const float c = p.scale_log2e;
    floatx16 dK[G::DB], dV[G::DB];
#pragma unroll
    for (int db = 0; db < G::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            dK[db][r] = 0.f;
            dV[db][r] = 0.f;
        }

    BoxWalk walk;
    walk.start(box, p.n_h, p.n_w, p.P);
    const int n_iter = box.count() * walk.sub_per_tile;
    for (int iter = 0; iter < n_iter; ++iter) {
        __syncthreads();
        const uint32_t first_row = walk.next_row;
        G::copy_in(smem, qh + (size_t)first_row * G::RowB, lane);
        G::copy_in(smem + G::SubB, gh + (size_t)first_row * G::RowB, lane);
        walk.advance();
        // statistics of the query rows this lane's accumulator registers belong to: rows 8*g + 4*hb + t
        float ls[16], dl[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const floatx4 a = *reinterpret_cast<const floatx4 *>(lse + head_row + first_row + 8 * g + 4 * hb);
            const floatx4 d = *reinterpret_cast<const floatx4 *>(delta + head_row + first_row + 8 * g + 4 * hb);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                ls[4 * g + t] = a[t] * kLog2e;
                dl[4 * g + t] = d[t];
            }
        }
        __syncthreads();
        const floatx16 S = G::rows_times(smem, lane, Kr);                      // S  = Q K^T (queries x keys)
        const floatx16 dP = G::rows_times(smem + G::SubB, lane, Vr);           // dP = dO V^T
        float prob[16], ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            prob[r] = __builtin_amdgcn_exp2f(fmaf(S[r], c, -ls[r]));
            ds[r] = prob[r] * (dP[r] - dl[r]);
        }
        bf16x8 Pb[2], dSb[2];
        pack16(prob, Pb);
        pack16(ds, dSb);
        G::transposed_times(smem_addr + G::SubB, lane, Pb, dV);                // dV^T += dO^T P
        G::transposed_times(smem_addr, lane, dSb, dK);                         // dK^T += Q^T dS
    }
    G::store_columns(d_v + my_row * D, lane, dV, 1.0f);
    G::store_columns(d_k + my_row * D, lane, dK, c * kLn2);
}

template <int D>
hipError_t launch_backward_generic(const bf16_raw *q, const bf16_raw *k, const bf16_raw *v, const void *o, const void *d_o,
                                   const float *lse, float *delta, bool compute_delta, void *d_q, void *d_k, void *d_v,
                                   int B, const sta::FwdParams &p, const sta::WindowTable &win, hipStream_t stream)
{
    if (compute_delta) {
        const size_t rows = (size_t)B * p.H * p.N;   // all heads of the tensor at once
        const unsigned per_block = 256 / (D / 8);
        sta_bwd_delta_generic_kernel<D><<<dim3((unsigned)((rows + per_block - 1) / per_block)), dim3(256), 0, stream>>>(
            static_cast<const uint4 *>(o), static_cast<const uint4 *>(d_o), delta, rows);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const dim3 grid(p.N / kSub, (uint32_t)B * p.heads), block(64);
    const bf16_raw *gg = static_cast<const bf16_raw *>(d_o);
    sta_bwd_dq_generic_kernel<D><<<grid, block, 0, stream>>>(q, k, v, gg, lse, delta, static_cast<bf16_raw *>(d_q), p, win);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    sta_bwd_dkv_generic_kernel<D><<<grid, block, 0, stream>>>(q, k, v, gg, lse, delta, static_cast<bf16_raw *>(d_k),
                                                              static_cast<bf16_raw *>(d_v), p, win);
    return hipGetLastError();
}

}  // namespace

namespace sta {

bool backward_supported(int P, int D) { return (D == 64 || D == 128) && P > 0 && P % kSub == 0; }

// The three tuned kernels for head dimension D: tokens per tile a multiple of 128.
template <int D>
hipError_t launch_backward_staged(const bf16_raw *qq, const bf16_raw *kk, const bf16_raw *vv, const void *o, const bf16_raw *gg,
                                  const float *lse, float *delta, bool compute_delta, void *d_q, void *d_k, void *d_v, int B,
                                  const FwdParams &p, const WindowTable &win, hipStream_t stream)
{
    // the workspace holds two floats per row here: -delta, then -lse / scale
    const size_t rows = (size_t)B * p.H * p.N;       // all heads of the tensor at once
    float *neg_delta = delta, *neg_lse = delta + rows;
    if (compute_delta) {
        constexpr unsigned per_block = 256 / (D / 8);
        sta_bwd_delta_kernel<D><<<dim3((unsigned)((rows + per_block - 1) / per_block)), dim3(256), 0, stream>>>(
            static_cast<const uint4 *>(o), reinterpret_cast<const uint4 *>(gg), lse, kLog2e / p.scale_log2e, neg_delta,
            neg_lse, rows);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const uint32_t n_bh = (uint32_t)B * p.heads;
    const uint32_t total = (p.N / kCols) * n_bh;
    auto grid_for = [&](uint32_t chunk) { return dim3(8 * chunk * ((((total + chunk - 1) / chunk) + 7) / 8)); };
    // One chunk = the column blocks of one row of tiles along w.  Measured at the 30x48x80 grid (chunk sizes 1, 3,
    // 6, 30, 60, 120 in one session): dK/dV kernel 32.7, 31.5, 31.6, 31.0, 31.1, 34.0 ms; dQ kernel 18.9, 18.8, 18.7,
    // 18.5, 18.5, 19.3 ms.
    const uint32_t chunk = p.n_w * (p.P / kCols);
    dim3 block(kNW * 64);
    sta_bwd_dq_kernel<D><<<grid_for(chunk), block, 0, stream>>>(qq, kk, vv, gg, neg_lse, neg_delta, static_cast<bf16_raw *>(d_q), p,
                                                               win, n_bh, chunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // Head dimension 128: six pairs (192 keys per workgroup, three waves per SIMD) where the tile allows.  Head
    // dimension 64 needs 106 registers, so two workgroups of four pairs share a CU (four waves per SIMD); measured on
    // the 30x48x80 grid with 384-token tiles: 21.7 ms for the entry point against 24.9-25.1 ms with six pairs.
    if (D == 128 && p.P % 192 == 0) {
        // the chunk is again one row of tiles along w
        const uint32_t total6 = (p.N / 192) * n_bh, chunk6 = p.n_w * (p.P / 192);
        const dim3 grid6(8 * chunk6 * ((((total6 + chunk6 - 1) / chunk6) + 7) / 8));
        sta_bwd_dkv_kernel<D, 6><<<grid6, dim3(768), 0, stream>>>(qq, kk, vv, gg, neg_lse, neg_delta, static_cast<bf16_raw *>(d_k),
                                                                 static_cast<bf16_raw *>(d_v), p, win, n_bh, chunk6);
    } else {
        sta_bwd_dkv_kernel<D, 4><<<grid_for(chunk), dim3(512), 0, stream>>>(qq, kk, vv, gg, neg_lse, neg_delta,
                                                                           static_cast<bf16_raw *>(d_k),
                                                                           static_cast<bf16_raw *>(d_v), p, win, n_bh, chunk);
    }
    return hipGetLastError();
}

hipError_t launch_backward(const void *q, const void *k, const void *v, const void *o, const void *d_o, const float *lse,
                           float *delta, bool compute_delta, void *d_q, void *d_k, void *d_v, int B, int D,
                           const FwdParams &p, const WindowTable &win, hipStream_t stream)
{
    if (!backward_supported((int)p.P, D)) return hipErrorInvalidValue;
    const bf16_raw *qq = static_cast<const bf16_raw *>(q), *kk = static_cast<const bf16_raw *>(k);
    const bf16_raw *vv = static_cast<const bf16_raw *>(v), *gg = static_cast<const bf16_raw *>(d_o);
    const bool staged = p.P % kCols == 0;
    if (D == 64)
        return staged ? launch_backward_staged<64>(qq, kk, vv, o, gg, lse, delta, compute_delta, d_q, d_k, d_v, B, p, win, stream)
                      : launch_backward_generic<64>(qq, kk, vv, o, d_o, lse, delta, compute_delta, d_q, d_k, d_v, B, p, win, stream);
    return staged ? launch_backward_staged<128>(qq, kk, vv, o, gg, lse, delta, compute_delta, d_q, d_k, d_v, B, p, win, stream)
                  : launch_backward_generic<128>(qq, kk, vv, o, d_o, lse, delta, compute_delta, d_q, d_k, d_v, B, p, win, stream);
}

}  // namespace sta
