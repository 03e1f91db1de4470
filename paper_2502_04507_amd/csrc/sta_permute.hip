// Tile / untile permutation kernels (HBM-bound).
//
// STA orders tokens so that each (T_t, T_h, T_w) tile occupies one contiguous
// run of the sequence (Sec. 3.1; appendix "Tiling in STA").  In
// raster order a tile is T_t*T_h runs of T_w consecutive tokens, so both sides
// of the copy are made of contiguous segments of T_w*D elements: a workgroup
// moves one tile of one (batch, head) slice, or an even share of it when the
// tensor has too few tiles to fill the chip, each lane moving 8 elements (16 B
// of bf16) at a time with the tiled side fully linear.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sta_internal.h"

namespace {

struct alignas(16) Chunk8bf16 { uint32_t w[4]; };
struct alignas(16) Chunk8f32 { float4 lo, hi; };

__device__ __forceinline__ uint32_t pack2_bf16(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v;
    v[0] = static_cast<__bf16>(a);   // round to nearest even
    v[1] = static_cast<__bf16>(b);
    return __builtin_bit_cast(uint32_t, v);
}

// Load 8 elements as raw bf16 bits (4 dwords) or as 8 floats.
template <bool SRC_F32>
__device__ __forceinline__ void load8(const void *base, size_t chunk, Chunk8bf16 &b, Chunk8f32 &f)
{
    if constexpr (SRC_F32) {
        f = reinterpret_cast<const Chunk8f32 *>(base)[chunk];
    } else {
        b = reinterpret_cast<const Chunk8bf16 *>(base)[chunk];
    }
}

// 16-byte store that does not leave a dirty line in L2.  The outputs are written once and read by a later kernel;
// with ordinary stores the dirty lines are written back when the kernel ends, which at small sizes costs more than
// the copy itself (measured: 4 MB tensor 17 -> 2.7 us per launch, 85 MB tensor 33 -> 25.6 us, 1.4 GB 261 -> 247 us).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store16_streaming(void *base, size_t chunk16, u32x4_t v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(base) + chunk16);
}

template <bool SRC_F32, bool DST_F32>
__device__ __forceinline__ void store8(void *base, size_t chunk, const Chunk8bf16 &b, const Chunk8f32 &f)
{
    if constexpr (!DST_F32) {
        u32x4_t o;
        if constexpr (SRC_F32) {                 // f32 -> bf16
            o[0] = pack2_bf16(f.lo.x, f.lo.y);
            o[1] = pack2_bf16(f.lo.z, f.lo.w);
            o[2] = pack2_bf16(f.hi.x, f.hi.y);
            o[3] = pack2_bf16(f.hi.z, f.hi.w);
        } else {
            o[0] = b.w[0]; o[1] = b.w[1]; o[2] = b.w[2]; o[3] = b.w[3];
        }
        store16_streaming(base, chunk, o);
    } else {
        u32x4_t lo, hi;
        if constexpr (SRC_F32) {
            lo[0] = __float_as_uint(f.lo.x); lo[1] = __float_as_uint(f.lo.y);
            lo[2] = __float_as_uint(f.lo.z); lo[3] = __float_as_uint(f.lo.w);
            hi[0] = __float_as_uint(f.hi.x); hi[1] = __float_as_uint(f.hi.y);
            hi[2] = __float_as_uint(f.hi.z); hi[3] = __float_as_uint(f.hi.w);
        } else {                                 // bf16 -> f32 (exact)
            lo[0] = b.w[0] << 16; lo[1] = b.w[0] & 0xffff0000u; lo[2] = b.w[1] << 16; lo[3] = b.w[1] & 0xffff0000u;
            hi[0] = b.w[2] << 16; hi[1] = b.w[2] & 0xffff0000u; hi[2] = b.w[3] << 16; hi[3] = b.w[3] & 0xffff0000u;
        }
        store16_streaming(base, 2 * chunk, lo);
        store16_streaming(base, 2 * chunk + 1, hi);
    }
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t magic)
{
    // magic = ceil(2^32 / d) for d > 1; exact while n * d < 2^32 (checked on the host).
    return d == 1 ? n : __umulhi(n, magic);
}

constexpr int kPermuteThreads = 256;
constexpr int kUnroll = 4;
static_assert(kPermuteThreads * kUnroll == (int)sta::kPermuteChunksPerBlock, "one pass per workgroup");

// TO_TILED: src is raster, dst is tiled.  Otherwise the reverse.
template <bool SRC_F32, bool DST_F32, bool TO_TILED>
__global__ __launch_bounds__(kPermuteThreads) void sta_permute_kernel(const void *__restrict__ src,
                                                                     void *__restrict__ dst,
                                                                     sta::PermuteParams p)
{
    const uint32_t part = blockIdx.x % p.parts;
    const uint32_t tile_linear = blockIdx.x / p.parts;
    const uint32_t tile_id = tile_linear % p.n_tiles;
    const uint32_t outer = tile_linear / p.n_tiles;         // b*H + h
    const uint32_t tw = tile_id % p.n_w;
    const uint32_t th = (tile_id / p.n_w) % p.n_h;
    const uint32_t tt = tile_id / (p.n_w * p.n_h);

    const size_t slice = (size_t)outer * p.N * p.cpr;       // chunk offset of this (b,h) slice
    const size_t tiled_base = slice + (size_t)tile_id * p.chunks_per_tile;
    // raster chunk index of the tile's first token
    const size_t raster_tile = slice + (((size_t)tt * p.T_t * p.L_h + (size_t)th * p.T_h) * p.L_w + (size_t)tw * p.T_w) * p.cpr;
    const uint32_t row_stride_h = p.L_w * p.cpr;            // chunks per raster row of tokens (fixed t,h)
    const uint32_t row_stride_t = p.L_h * row_stride_h;

    const uint32_t first = part * p.span;
    const uint32_t end = first + p.span < p.chunks_per_tile ? first + p.span : p.chunks_per_tile;
    for (uint32_t i0 = first + threadIdx.x; i0 < end; i0 += kPermuteThreads * kUnroll) {
        Chunk8bf16 b[kUnroll];
        Chunk8f32 f[kUnroll];
        size_t dst_idx[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t idx = i0 + u * kPermuteThreads;
            if (idx < end) {
                const uint32_t seg = fast_div(idx, p.seg, p.seg_magic);      // which (i_t, i_h) run
                const uint32_t off = idx - seg * p.seg;
                const uint32_t it = fast_div(seg, p.T_h, p.T_h_magic);
                const uint32_t ih = seg - it * p.T_h;
                const size_t raster = raster_tile + (size_t)it * row_stride_t + (size_t)ih * row_stride_h + off;
                const size_t tiled = tiled_base + idx;
                load8<SRC_F32>(src, TO_TILED ? raster : tiled, b[u], f[u]);
                dst_idx[u] = TO_TILED ? tiled : raster;
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t idx = i0 + u * kPermuteThreads;
            if (idx < end) store8<SRC_F32, DST_F32>(dst, dst_idx[u], b[u], f[u]);
        }
    }
}

template <bool TO_TILED>
hipError_t launch(const void *src, void *dst, bool src_f32, bool dst_f32, const sta::PermuteParams &p,
                  uint32_t blocks, hipStream_t stream)
{
    dim3 g(blocks), b(kPermuteThreads);
    if (!src_f32 && !dst_f32) sta_permute_kernel<false, false, TO_TILED><<<g, b, 0, stream>>>(src, dst, p);
    else if (src_f32 && !dst_f32) sta_permute_kernel<true, false, TO_TILED><<<g, b, 0, stream>>>(src, dst, p);
    else if (!src_f32 && dst_f32) sta_permute_kernel<false, true, TO_TILED><<<g, b, 0, stream>>>(src, dst, p);
    else sta_permute_kernel<true, true, TO_TILED><<<g, b, 0, stream>>>(src, dst, p);
    return hipGetLastError();
}

}  // namespace

namespace sta {

hipError_t launch_permute(const void *src, void *dst, bool src_f32, bool dst_f32, bool to_tiled,
                          const PermuteParams &p, uint32_t blocks, hipStream_t stream)
{
    return to_tiled ? launch<true>(src, dst, src_f32, dst_f32, p, blocks, stream)
                    : launch<false>(src, dst, src_f32, dst_f32, p, blocks, stream);
}

}  // namespace sta
