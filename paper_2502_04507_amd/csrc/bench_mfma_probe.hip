// Measurement aid for the benchmark, NOT part of the attention library: what the matrix pipes deliver on THIS chip
// for the instructions the attention kernels use.  Built into its own shared object (libsta_mfma_probe.so) which only
// the benchmark loads.
//
// mfma_probe: each wave runs `iters` rounds of 16 v_mfma_f32_32x32x16_bf16 (8 chained into one accumulator like a
// QK^T block, 8 into four accumulators like a PV block), 2 waves per SIMD: the shape and occupancy of the head
// dimension 64 and gradient kernels.
// mfma_probe_16x16x32: each wave runs `iters` rounds of 32 v_mfma_f32_16x16x32_bf16 in the order of the head
// dimension 128 forward kernel (16 into four accumulators with the A operand kept for two instructions, 16 into
// sixteen accumulators with one operand changing at a time), 3 waves per SIMD.
// Operands are taken from `operands`, so their bit patterns, and with them the power drawn and the clock the chip
// settles at, are the caller's choice; nothing else is executed.
#include <hip/hip_runtime.h>

namespace {

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(const probe_bf16x8 *__restrict__ operands, int iters,
                                                            float *__restrict__ sink)
{
    probe_bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = operands[(threadIdx.x & 63) + 64 * i];
        b[i] = operands[(threadIdx.x & 63) + 64 * (8 + i)];
    }
    probe_floatx16 s, o[4];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        s[r] = 0.f;
#pragma unroll
        for (int d = 0; d < 4; ++d) o[d][r] = 0.f;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], s, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[i], a[i], o[i & 3], 0, 0, 0);
        asm volatile("" : "+v"(a[0]));      // nothing is loop-invariant
    }
    float acc = s[0] + s[7];
#pragma unroll
    for (int d = 0; d < 4; ++d) acc += o[d][3];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

typedef float probe_floatx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(768, 1) void mfma_probe_16x16x32_kernel(const probe_bf16x8 *__restrict__ operands, int iters,
                                                                     float *__restrict__ sink)
{
    probe_bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = operands[(threadIdx.x & 63) + 64 * i];
        b[i] = operands[(threadIdx.x & 63) + 64 * (8 + i)];
    }
    probe_floatx4 s[4], o[16];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
        for (int d = 0; d < 4; ++d) s[d][r] = 0.f;
#pragma unroll
        for (int d = 0; d < 16; ++d) o[d][r] = 0.f;
    }
    for (int it = 0; it < iters; ++it) {
        // scores: per key block four k-steps, each feeding the two query blocks (0, 1, 1, 0, ..)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int step = i >> 1, qb = ((i >> 1) & 1) ^ (i & 1);
            s[2 * (step >> 2) + qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[step], b[4 * qb + (step & 3)], s[2 * (step >> 2) + qb], 0, 0, 0);
        }
        // output: eight channel blocks x two query blocks, one operand changing at a time
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int cb = i >> 1, qb = ((i >> 1) & 1) ^ (i & 1);
            o[2 * cb + qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[cb], a[qb], o[2 * cb + qb], 0, 0, 0);
        }
        asm volatile("" : "+v"(a[0]));      // nothing is loop-invariant
    }
    float acc = 0.f;
#pragma unroll
    for (int d = 0; d < 4; ++d) acc += s[d][1];
#pragma unroll
    for (int d = 0; d < 16; ++d) acc += o[d][3];
    sink[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

}  // namespace

// dev_operands: device, >= 8192 bf16 values, read.  dev_sink: device, float32 [workgroups * 256], written.
// Work = workgroups * 4 waves * iters * 16 instructions * 32768 flop.  Returns 0, or 1 on a bad argument,
// or 2 when the launch failed.
extern "C" int mfma_probe(const void *dev_operands, int iters, int workgroups, float *dev_sink, void *hip_stream)
{
    if (!dev_operands || !dev_sink || iters < 1 || workgroups < 1 || workgroups > 65536) return 1;
    mfma_probe_kernel<<<dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const probe_bf16x8 *>(dev_operands), iters, dev_sink);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Same arguments; dev_sink: float32 [workgroups * 768].  Work = workgroups * 12 waves * iters * 32 instructions *
// 16384 flop.
extern "C" int mfma_probe_16x16x32(const void *dev_operands, int iters, int workgroups, float *dev_sink, void *hip_stream)
{
    if (!dev_operands || !dev_sink || iters < 1 || workgroups < 1 || workgroups > 65536) return 1;
    mfma_probe_16x16x32_kernel<<<dim3(workgroups), dim3(768), 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const probe_bf16x8 *>(dev_operands), iters, dev_sink);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
