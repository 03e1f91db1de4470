// Small HBM-bound kernels around the attention kernel:
//   - per-head mean squared error between two attention outputs (the loss of the paper's mask-search
//     algorithm, "STA Mask Search": loss <- MSE(O, O')),
//   - first-minimum selection over a list of patterns per head (same algorithm: keep the pattern whose
//     loss is strictly smaller than the best so far),
//   - attention recall from two log-denominators (Sec. 1: fraction of the attention score that falls
//     inside a local window).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "sta_internal.h"

namespace {

constexpr int kThreads = 256;

// Partial sums of the allocation-free per-head MSE entry point: kMseSlices doubles per (batch, head) slab, for
// at most kStaticMseMaxSlabs slabs (512 KB).  Every GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; kernels
// receive the device address that call returns.
static __device__ __align__(256) double scratch[sta::kStaticMseMaxSlabs * sta::kMseSlices];
constexpr int kMaxDevices = 64;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Sum over a workgroup of one double per thread; result valid in thread 0.
__device__ __forceinline__ double block_sum(double x)
{
    __shared__ double part[kThreads / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0)
#pragma unroll
        for (int i = 0; i < kThreads / 64; ++i) s += part[i];
    return s;
}

// grid = (slices, B*H).  Slice s of slice count S sums the squared differences of 16-byte chunks
// s, s+S, s+2S, ... of one (b,h) slab and writes one double.  chunks = N*D/8 per slab.
__global__ __launch_bounds__(kThreads) void sta_sq_diff_partial_kernel(const uint4 *__restrict__ a,
                                                                       const uint4 *__restrict__ b, size_t chunks,
                                                                       double *__restrict__ partial)
{
    const size_t slab = (size_t)blockIdx.y * chunks;
    const size_t stride = (size_t)gridDim.x * kThreads;
    float acc0 = 0.f, acc1 = 0.f;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < chunks; i += stride) {
        const uint4 x = a[slab + i], y = b[slab + i];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float d0 = bf16_lo(xs[e]) - bf16_lo(ys[e]);
            const float d1 = bf16_hi(xs[e]) - bf16_hi(ys[e]);
            acc0 = fmaf(d0, d0, acc0);
            acc1 = fmaf(d1, d1, acc1);
        }
    }
    const double s = block_sum((double)acc0 + (double)acc1);
    if (threadIdx.x == 0) partial[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = s;
}

// One thread per head: sums the slices of every batch entry in a fixed order and divides by the element count.
__global__ void sta_mse_finish_kernel(const double *__restrict__ partial, int slices, int B, int H, double inv_count,
                                      float *__restrict__ mse_per_head)
{
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= H) return;
    double s = 0.0;
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < slices; ++i) s += partial[((size_t)b * H + h) * slices + i];
    mse_per_head[h] = (float)(s * inv_count);
}

// losses: [n_patterns][H].  best[h] = index of the first pattern with the smallest loss.
__global__ void sta_first_min_kernel(const float *__restrict__ losses, int n_patterns, int H, int32_t *__restrict__ best)
{
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= H) return;
    float minimum = INFINITY;
    int32_t arg = -1;
    for (int p = 0; p < n_patterns; ++p) {
        const float loss = losses[(size_t)p * H + h];
        if (loss < minimum) {
            minimum = loss;
            arg = p;
        }
    }
    best[h] = arg;
}

// grid = (slices, B*H).  recall_i = exp(lse_window_i - lse_full_i); optional per-query output; one partial sum
// per workgroup.
__global__ __launch_bounds__(kThreads) void sta_recall_partial_kernel(const float *__restrict__ lse_window,
                                                                      const float *__restrict__ lse_full, size_t N,
                                                                      float *__restrict__ recall,
                                                                      double *__restrict__ partial)
{
    const size_t base = (size_t)blockIdx.y * N;
    const size_t stride = (size_t)gridDim.x * kThreads;
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < N; i += stride) {
        const float r = __expf(lse_window[base + i] - lse_full[base + i]);
        if (recall) recall[base + i] = r;
        acc += r;
    }
    const double s = block_sum((double)acc);
    if (threadIdx.x == 0) partial[(size_t)blockIdx.y * gridDim.x + blockIdx.x] = s;
}

// One thread per (batch, head): fixed-order sum of the slices.
__global__ void sta_recall_finish_kernel(const double *__restrict__ partial, int slices, int BH, double inv_n,
                                         float *__restrict__ mean_bh)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= BH) return;
    double s = 0.0;
    for (int k = 0; k < slices; ++k) s += partial[(size_t)i * slices + k];
    mean_bh[i] = (float)(s * inv_n);
}

}  // namespace

namespace sta {

hipError_t launch_head_mse(const void *a, const void *b, int B, int H, size_t elems_per_head, double *partial,
                           float *mse_per_head, hipStream_t stream)
{
    const size_t chunks = elems_per_head / 8;
    dim3 grid(kMseSlices, (uint32_t)B * H), block(kThreads);
    sta_sq_diff_partial_kernel<<<grid, block, 0, stream>>>(static_cast<const uint4 *>(a), static_cast<const uint4 *>(b),
                                                           chunks, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    sta_mse_finish_kernel<<<dim3((H + 63) / 64), dim3(64), 0, stream>>>(partial, kMseSlices, B, H,
                                                                        1.0 / ((double)B * (double)elems_per_head),
                                                                        mse_per_head);
    return hipGetLastError();
}

hipError_t static_mse_scratch(double **out)
{
    static std::mutex mu;
    static double *per_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (per_device[dev] == nullptr) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        per_device[dev] = static_cast<double *>(ptr);
    }
    *out = per_device[dev];
    return hipSuccess;
}

hipError_t launch_first_min(const float *losses, int n_patterns, int H, int32_t *best, hipStream_t stream)
{
    sta_first_min_kernel<<<dim3((H + 63) / 64), dim3(64), 0, stream>>>(losses, n_patterns, H, best);
    return hipGetLastError();
}

hipError_t launch_recall(const float *lse_window, const float *lse_full, int BH, size_t N, float *recall, double *partial,
                         float *mean_bh, hipStream_t stream)
{
    sta_recall_partial_kernel<<<dim3(kMseSlices, BH), dim3(kThreads), 0, stream>>>(lse_window, lse_full, N, recall, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    sta_recall_finish_kernel<<<dim3((BH + 63) / 64), dim3(64), 0, stream>>>(partial, kMseSlices, BH, 1.0 / (double)N, mean_bh);
    return hipGetLastError();
}

}  // namespace sta
