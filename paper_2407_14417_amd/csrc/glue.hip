// 16-bit glue around the expert kernels: weighted average of the selected experts' outputs
// (paper §1) with the residual add of the chained configuration (§3: non-expert parts are
// always 16-bit).  The RMSNorm of that configuration lives in the gating kernel.
#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

// out[t, c] = fp16( residual[t, c] + sum_s gate[t, s] * sum_p y[p][inv[t*k+s], c] ), slots and partials added in order.
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ y, int splits, size_t split_stride,
                                                       const float* __restrict__ gate, const int32_t* __restrict__ inv,
                                                       int d, int k, const half_t* __restrict__ residual,
                                                       half_t* __restrict__ out) {
    const int t = blockIdx.y;
    const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c >= d) return;
    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < k; ++s) {
        const int r = inv[t * k + s];
        if (r < 0) continue;
        const float g = gate[t * k + s];
        float4_t v = *(const float4_t*)(y + (size_t)r * d + c);
        for (int p = 1; p < splits; ++p) v += *(const float4_t*)(y + p * split_stride + (size_t)r * d + c);
        acc += g * v;
    }
    if (residual) {
        const half4_t rv = *(const half4_t*)(residual + (size_t)t * d + c);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] += (float)rv[j];
    }
    half4_t o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (half_t)acc[j];
    *(half4_t*)(out + (size_t)t * d + c) = o;
}

void launch_combine(const float* y, int splits, size_t split_stride, const float* gate, const int32_t* inv, int T, int d,
                    int k, const half_t* residual, half_t* out, hipStream_t st) {
    TraceScope trace(kKernelCombine, st);
    dim3 grid((d / 4 + 255) / 256, T);
    combine_kernel<<<grid, 256, 0, st>>>(y, splits, split_stride, gate, inv, d, k, residual, out);
}

// dst[i] = sum_p y[p][i], partials added in order
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ y, int splits, size_t split_stride,
                                                             size_t n4, float* __restrict__ dst) {
    for (size_t i = blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        float4_t v = ((const float4_t*)y)[i];
        for (int p = 1; p < splits; ++p) v += *(const float4_t*)(y + p * split_stride + i * 4);
        ((float4_t*)dst)[i] = v;
    }
}

void launch_reduce_splits(const float* y, int splits, size_t split_stride, size_t n, float* dst, hipStream_t st) {
    if (n == 0) return;
    const size_t n4 = n / 4;
    const int blocks = (int)((n4 + 255) / 256 < 2048 ? (n4 + 255) / 256 : 2048);
    reduce_splits_kernel<<<blocks, 256, 0, st>>>(y, splits, split_stride, n4, dst);
}

// Fill kernel used instead of a memset node so that every launch sequence stays graph-capturable.
__global__ void zero_words_kernel(int32_t* p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

void launch_zero_words(int32_t* p, int n, hipStream_t st) {
    if (n > 0) zero_words_kernel<<<(n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024, 256, 0, st>>>(p, n);
}

}  // namespace moemix
