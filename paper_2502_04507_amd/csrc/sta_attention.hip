// Sliding Tile Attention forward kernel for gfx950 (MI355X).
//
// What is computed: Eq. 1 of the paper (S = QK^T/sqrt(d), A = softmax(S + M),
// O = AV) where M keeps, for each query tile, exactly the key tiles inside the
// clamped tile window of the appendix algorithm "Mask Definition of 3D STA".
// Tokens arrive in tile order, so each kept (query tile, key tile) pair is a
// fully dense block and no element-level mask exists anywhere in this file.
//
// Formulation.  The kernel works on the TRANSPOSED score block
// S^T = K Q^T (keys along the MFMA M dimension, queries along N), so that one
// lane owns one query column: its running max / sum are per-lane scalars and
// the only cross-lane traffic in the softmax is one exchange between the two
// 32-lane halves of a wave.  The output is accumulated transposed as well,
// O^T += V^T P^T, which lets P^T go from the S^T accumulators straight into the
// B operand of the second MFMA with no data movement: the MFMA contraction
// index is only a summation index, so the keys are fed in the order the
// accumulator layout holds them and V^T is stored in LDS in that same order.
//
// MFMA: v_mfma_f32_32x32x16_bf16.  Operand layout (lane l, lo = l%32, hb = l/32):
//   A (32 x 16): row lo,  k = 8*hb .. 8*hb+7
//   B (16 x 32): col lo,  k = 8*hb .. 8*hb+7
//   C (32 x 32): col lo,  row = 8*g + 4*hb + t for register r = 4*g + t.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sta_geometry.h"
#include "sta_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_raw;

__device__ __forceinline__ floatx16 mfma_32x32x16(bf16x8 a, bf16x8 b, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Position inside a group of 16 keys at which key `k16` (0..15) is stored in the
// transposed V buffer: the accumulator of S^T holds, for half hb, keys
// {4*hb + t} and {8 + 4*hb + t}; they are made adjacent so one 16-byte LDS read
// yields the 8 keys a lane feeds to the PV MFMA.
__device__ __forceinline__ int vt_pos(int k16)
{
    const int a = k16 >> 3, hb = (k16 >> 2) & 1, t = k16 & 3;
    return 8 * hb + 4 * a + t;
}

template <int D, int NW, int NQ, int KB>
struct FwdCfg {
    static constexpr int kThreads = NW * 64;
    static constexpr int kQB = NW * NQ * 32;          // queries per workgroup
    static constexpr int kKStride = D + 8;            // elements; 16 B pad => conflict-free b128 reads
    static constexpr int kVStride = KB + 8;           // elements (keys) per d row of V^T
    static constexpr int kKElems = KB * kKStride;
    static constexpr int kVElems = D * kVStride;
    static constexpr int kChunks = KB * D / 8;        // 16-byte chunks per K (or V) sub-block
    static constexpr int kChunksPerThread = kChunks / kThreads;
    static_assert(kChunks % kThreads == 0, "sub-block must split evenly over the workgroup");
    static_assert(KB % 32 == 0 && D % 32 == 0, "MFMA tiling");
};

template <int D, int NW, int NQ, int KB>
__global__ __launch_bounds__(NW * 64) void sta_fwd_kernel(const bf16_raw *__restrict__ q,
                                                          const bf16_raw *__restrict__ k,
                                                          const bf16_raw *__restrict__ v,
                                                          bf16_raw *__restrict__ o, sta::FwdParams p,
                                                          sta::WindowTable win)
{
    using C = FwdCfg<D, NW, NQ, KB>;
    constexpr int MB = KB / 32;       // 32-key blocks per sub-block
    constexpr int KS = D / 16;        // MFMA k-steps over the head dim
    constexpr int DB = D / 32;        // 32-row blocks of O^T

    __shared__ __attribute__((aligned(16))) bf16_raw Ks[C::kKElems];
    __shared__ __attribute__((aligned(16))) bf16_raw Vt[C::kVElems];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int lo = lane & 31;
    const int hb = lane >> 5;

    const uint32_t qblock = blockIdx.x;                       // index of this QB-query block inside the head
    const uint32_t bh_local = blockIdx.y;                     // b * heads + h_local
    const uint32_t h_local = bh_local % p.heads;
    const uint32_t b = bh_local / p.heads;
    const size_t bh = (size_t)b * p.H + p.head_base + h_local;
    const uint32_t q_tile = (qblock * C::kQB) / p.P;

    const StaBox box = sta_key_tile_box_of(p.n_t, p.n_h, p.n_w, win.w[h_local][0], win.w[h_local][1],
                                           win.w[h_local][2], q_tile);

    const bf16_raw *qh = q + (bh * p.N + (size_t)qblock * C::kQB + (size_t)wave * NQ * 32) * D;
    const bf16_raw *kh = k + bh * p.N * D;
    const bf16_raw *vh = v + bh * p.N * D;

    // Q fragments stay in registers for the whole kernel (B operand of S^T = K Q^T).
    bf16x8 Qr[NQ][KS];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            Qr[nq][ks] = *reinterpret_cast<const bf16x8 *>(qh + (size_t)(nq * 32 + lo) * D + ks * 16 + hb * 8);

    floatx16 Oacc[NQ][DB];
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_run[nq] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) Oacc[nq][db][r] = 0.f;
    }

    const int sub_per_tile = p.P / KB;
    const int n_iter = box.count() * sub_per_tile;

    // Iteration state: (kt_t, kt_h, kt_w, sub-block) walked in ascending tile id order.
    int it_t = box.t.lo, it_h = box.h.lo, it_w = box.w.lo, it_s = 0;
    auto key_base = [&]() -> size_t {
        const size_t kt = ((size_t)it_t * p.n_h + it_h) * p.n_w + it_w;
        return (kt * p.P + (size_t)it_s * KB) * D;
    };
    auto advance = [&]() {
        if (++it_s == sub_per_tile) {
            it_s = 0;
            if (++it_w > box.w.hi) {
                it_w = box.w.lo;
                if (++it_h > box.h.hi) { it_h = box.h.lo; ++it_t; }
            }
        }
    };

    uint4 kreg[C::kChunksPerThread], vreg[C::kChunksPerThread];
    auto fetch = [&](size_t base) {
#pragma unroll
        for (int i = 0; i < C::kChunksPerThread; ++i) {
            const int ci = tid + i * C::kThreads;
            kreg[i] = *reinterpret_cast<const uint4 *>(kh + base + (size_t)ci * 8);
            vreg[i] = *reinterpret_cast<const uint4 *>(vh + base + (size_t)ci * 8);
        }
    };

    fetch(key_base());

    for (int iter = 0; iter < n_iter; ++iter) {
        __syncthreads();                       // everyone is done reading the previous sub-block
#pragma unroll
        for (int i = 0; i < C::kChunksPerThread; ++i) {
            const int ci = tid + i * C::kThreads;
            const int row = ci / (D / 8);      // key inside the sub-block
            const int c = ci % (D / 8);        // 8-element chunk along d
            *reinterpret_cast<uint4 *>(&Ks[row * C::kKStride + c * 8]) = kreg[i];
            const int col = (row & ~15) + vt_pos(row & 15);
            const bf16_raw *ve = reinterpret_cast<const bf16_raw *>(&vreg[i]);
#pragma unroll
            for (int e = 0; e < 8; ++e) Vt[(c * 8 + e) * C::kVStride + col] = ve[e];
        }
        __syncthreads();
        advance();
        if (iter + 1 < n_iter) fetch(key_base());   // next sub-block in flight during the math

        // ---- S^T = K Q^T -------------------------------------------------------
        floatx16 S[NQ][MB];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) S[nq][mb][r] = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&Ks[(mb * 32 + lo) * C::kKStride + ks * 16 + hb * 8]);
#pragma unroll
                for (int nq = 0; nq < NQ; ++nq) S[nq][mb] = mfma_32x32x16(a, Qr[nq][ks], S[nq][mb]);
            }

        // ---- online softmax (one query column per lane) -------------------------
        bf16x8 Pb[NQ][MB][2];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            float mx = S[nq][0][0];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[nq][mb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[nq], mx);
            const float alpha = exp2f((m_run[nq] - m_new) * p.scale_log2e);
            const float mneg = -m_new * p.scale_log2e;
            m_run[nq] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        // register 8*j + e  <->  key 16*j + 8*(e/4) + 4*hb + e%4 of this 32-key block
                        const float pe = exp2f(fmaf(S[nq][mb][8 * j + e], p.scale_log2e, mneg));
                        const __bf16 pb = static_cast<__bf16>(pe);
                        Pb[nq][mb][j][e] = pb;
                        psum += static_cast<float>(pb);
                    }
                }
            l_run[nq] = l_run[nq] * alpha + psum;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) Oacc[nq][db][r] *= alpha;
        }

        // ---- O^T += V^T P^T ----------------------------------------------------
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&Vt[(db * 32 + lo) * C::kVStride + (mb * 2 + j) * 16 + hb * 8]);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq) Oacc[nq][db] = mfma_32x32x16(a, Pb[nq][mb][j], Oacc[nq][db]);
                }
    }

    // ---- finalize: O = O / l, bf16, tiled layout ----------------------------------
    bf16_raw *oh = o + (bh * p.N + (size_t)qblock * C::kQB + (size_t)wave * NQ * 32) * D;
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const float l_tot = l_run[nq] + __shfl_xor(l_run[nq], 32);
        const float inv = 1.f / l_tot;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 ov;
#pragma unroll
                for (int t = 0; t < 4; ++t) ov[t] = static_cast<__bf16>(Oacc[nq][db][4 * g + t] * inv);
                // rows of O^T are channels: d = 32*db + 8*g + 4*hb + t
                *reinterpret_cast<bf16x4 *>(oh + (size_t)(nq * 32 + lo) * D + db * 32 + g * 8 + hb * 4) = ov;
            }
    }
}

// Test hook: the key-tile list of every (head, query tile) from the same box function.
__global__ void sta_dump_key_tiles_kernel(sta::FwdParams p, sta::WindowTable win, int32_t *counts, int32_t *lists)
{
    const uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= p.heads * p.n_tiles) return;
    const uint32_t h_local = idx / p.n_tiles;
    const uint32_t q_tile = idx % p.n_tiles;
    const StaBox box = sta_key_tile_box_of(p.n_t, p.n_h, p.n_w, win.w[h_local][0], win.w[h_local][1],
                                           win.w[h_local][2], q_tile);
    const size_t row = (size_t)(p.head_base + h_local) * p.n_tiles + q_tile;
    int32_t *out = lists + row * p.n_tiles;
    uint32_t c = 0;
    for (int a = box.t.lo; a <= box.t.hi; ++a)
        for (int bq = box.h.lo; bq <= box.h.hi; ++bq)
            for (int cq = box.w.lo; cq <= box.w.hi; ++cq) out[c++] = (a * (int)p.n_h + bq) * (int)p.n_w + cq;
    counts[row] = (int32_t)c;
    for (; c < p.n_tiles; ++c) out[c] = -1;
}

template <int D, int NW, int NQ, int KB>
hipError_t launch_cfg(const void *q, const void *k, const void *v, void *o, int B, const sta::FwdParams &p,
                      const sta::WindowTable &win, hipStream_t stream)
{
    using C = FwdCfg<D, NW, NQ, KB>;
    dim3 grid(p.N / C::kQB, (uint32_t)B * p.heads);
    dim3 block(C::kThreads);
    sta_fwd_kernel<D, NW, NQ, KB><<<grid, block, 0, stream>>>(
        static_cast<const bf16_raw *>(q), static_cast<const bf16_raw *>(k), static_cast<const bf16_raw *>(v),
        static_cast<bf16_raw *>(o), p, win);
    return hipGetLastError();
}

template <int D>
hipError_t launch_d(const void *q, const void *k, const void *v, void *o, int B, const sta::FwdParams &p,
                    const sta::WindowTable &win, hipStream_t stream)
{
    const uint32_t P = p.P;
    if (P % 128 == 0) return launch_cfg<D, 4, 1, 64>(q, k, v, o, B, p, win, stream);
    if (P % 64 == 0) return launch_cfg<D, 2, 1, 64>(q, k, v, o, B, p, win, stream);
    if (P % 32 == 0) return launch_cfg<D, 1, 1, 32>(q, k, v, o, B, p, win, stream);
    return hipErrorInvalidValue;
}

}  // namespace

namespace sta {

bool forward_supported(int P, int D) { return (D == 64 || D == 128) && P > 0 && P % 32 == 0; }

hipError_t launch_forward(const void *q, const void *k, const void *v, void *o, int B, int D, const FwdParams &p,
                          const WindowTable &win, hipStream_t stream)
{
    if (!forward_supported((int)p.P, D)) return hipErrorInvalidValue;
    if (D == 64) return launch_d<64>(q, k, v, o, B, p, win, stream);
    return launch_d<128>(q, k, v, o, B, p, win, stream);
}

hipError_t launch_dump_key_tiles(const FwdParams &p, const WindowTable &win, int32_t *counts, int32_t *lists,
                                 hipStream_t stream)
{
    const uint32_t total = p.heads * p.n_tiles;
    sta_dump_key_tiles_kernel<<<dim3((total + 255) / 256), dim3(256), 0, stream>>>(p, win, counts, lists);
    return hipGetLastError();
}

}  // namespace sta
