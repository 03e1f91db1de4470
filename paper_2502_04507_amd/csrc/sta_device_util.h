// Device-side helpers shared by the attention kernels: vector types, the MFMA wrapper, compile-time loops,
// hand-issued LDS operand reads and the half-wave exchange.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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

__device__ __forceinline__ floatx4 mfma_16x16x32(bf16x8 a, bf16x8 b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

typedef short shortx4 __attribute__((ext_vector_type(4)));
#define STA_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// max(a, b, c).  Written with fmaxf so that the compiler sees the reads of MFMA results and inserts the wait
// states the hardware needs between a matrix instruction and a vector read of its result (it does not do that
// for inline assembly).  The translation unit is built with -fno-honor-nans, which lets this become a single
// v_max3_f32 without a canonicalising max per operand.
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

__device__ __forceinline__ float half_swap_max(float x)
{
    // v_permlane32_swap exchanges the upper half of the first operand with the lower half of the
    // second: afterwards r[0] holds lanes 0..31 of x in both halves and r[1] lanes 32..63.
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float a = __uint_as_float(r[0]), b = __uint_as_float(r[1]);
    return max3(a, b, b);
}

__device__ __forceinline__ float half_swap_sum(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Maximum / sum over the four lanes l, l^16, l^32, l^48 (the lanes that hold one column of a 16x16 MFMA result):
// v_permlane32_swap pairs lanes 32 apart, v_permlane16_swap lanes 16 apart; every lane ends with the same value.
__device__ __forceinline__ float quad_lane_max(float x)
{
    const float a = half_swap_max(x);
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(a), false, false);
    const float u = __uint_as_float(r[0]), w = __uint_as_float(r[1]);
    return max3(u, w, w);
}

__device__ __forceinline__ float quad_lane_sum(float x)
{
    const float a = half_swap_sum(x);
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(a), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// The value, usable by hand-written vector instructions: the compiler does not see into inline assembly and so
// cannot give such an instruction the wait state the hardware needs behind a transcendental one that produced x.
__device__ __forceinline__ float settled_after_transcendental(float x)
{
    asm volatile("s_nop 1" : "+v"(x));
    return x;
}

// x *= a with the result forced into the registers of x.
__device__ __forceinline__ void scale_in_place(floatx4 &x, float a)
{
    asm volatile("v_mul_f32_e32 %0, %4, %0\n\tv_mul_f32_e32 %1, %4, %1\n\tv_mul_f32_e32 %2, %4, %2\n\tv_mul_f32_e32 %3, %4, %3"
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])
                 : "v"(a));
}

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// One transposing LDS read with a compile-time byte offset.
template <int OFF>
__device__ __forceinline__ shortx4 ds_read_tr16(uint32_t addr)
{
    shortx4 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

// Issue the 2*DB transposing reads of one 16-key group (A operands of DB PV MFMAs).
template <int BASE, int DB, int ROWB>
__device__ __forceinline__ void pv_issue(shortx4 (&va)[DB][2], const uint32_t (&v_addr)[DB])
{
    static_for<0, DB>([&](auto dbi) {
        constexpr int db = decltype(dbi)::value;
        va[db][0] = ds_read_tr16<BASE>(v_addr[db]);
        va[db][1] = ds_read_tr16<BASE + 8 * ROWB>(v_addr[db]);
    });
}

// One 16-byte LDS read with a compile-time byte offset.
template <int OFF>
__device__ __forceinline__ bf16x8 ds_read_b128_at(uint32_t addr)
{
    bf16x8 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}

// Issue the K-operand reads of one group of 4 MFMA k-steps (A operands of S^T = K Q^T).
// k_addr[ks] is the lane's LDS address of its chunk for k-step ks in stage 0, row block 0; BASE (a compile-time
// byte offset, e.g. the stage) goes into the instruction's immediate.  GPM: groups per 32-row block (k-steps / 4).
template <int G, int ROWB, int BASE, int GPM = 2, int KS>
__device__ __forceinline__ void k_issue(bf16x8 (&ka)[4], const uint32_t (&k_addr)[KS])
{
    static_assert(KS == 4 * GPM, "k-steps per row block");
    constexpr int mb = G / GPM, ks0 = 4 * (G % GPM);
    static_for<0, 4>([&](auto i) {
        constexpr int ks = ks0 + decltype(i)::value;
        ka[decltype(i)::value] = ds_read_b128_at<BASE + mb * 32 * ROWB>(k_addr[ks]);
    });
}

template <int PENDING>
__device__ __forceinline__ void k_wait(bf16x8 (&ka)[4])
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]) : "n"(PENDING));
}

template <int PENDING>
__device__ __forceinline__ void lds_wait2(bf16x8 &a, bf16x8 &b)
{
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(PENDING));
}

// Wait until at most PENDING LDS reads are outstanding; the operands are tied to the wait so that
// their consumers cannot be scheduled above it.
template <int PENDING>
__device__ __forceinline__ void pv_wait(shortx4 (&va)[4][2])
{
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(va[0][0]), "+v"(va[0][1]), "+v"(va[1][0]), "+v"(va[1][1]), "+v"(va[2][0]), "+v"(va[2][1]),
                   "+v"(va[3][0]), "+v"(va[3][1])
                 : "n"(PENDING));
}

template <int PENDING>
__device__ __forceinline__ void pv_wait(shortx4 (&va)[2][2])
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(va[0][0]), "+v"(va[0][1]), "+v"(va[1][0]), "+v"(va[1][1]) : "n"(PENDING));
}

}  // namespace
