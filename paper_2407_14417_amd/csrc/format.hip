// The 4-bit weight format on the device: dequantizer (check hook, 4-bit -> 16-bit switch),
// quantizer (16-bit -> 4-bit switch when the expert table is re-planned, paper §3), and the seeded
// synthetic-tensor fill.
#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

// One thread per 8 weights (one 32-bit word of codes).
__global__ __launch_bounds__(256) void dequant_int4_kernel(DevMat m, size_t n_words, int in, half_t* __restrict__ w) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_words) return;
    const size_t col0 = (i * 8) % (size_t)in, row = (i * 8) / (size_t)in;
    const size_t g = row * (size_t)(in >> 6) + (col0 >> 6);
    const float s = (float)m.scale[g], z = (float)m.zero[g];
    const uint32_t word = ((const uint32_t*)m.data)[i];
    half8_t o;
#pragma unroll
    for (int n = 0; n < 8; ++n) o[n] = dequant_one((word >> (4 * n)) & 0xFu, s, z);
    *(half8_t*)(w + i * 8) = o;
}

void launch_dequant_int4(const DevMat& m, int out, int in, half_t* w, hipStream_t st) {
    const size_t n_words = (size_t)out * in / 8;
    if (n_words == 0) return;
    dequant_int4_kernel<<<(unsigned)((n_words + 255) / 256), 256, 0, st>>>(m, n_words, in, w);
}

// One wavefront per group of 64 weights: lane = column.  Min and max by shuffles, every fp32 step
// rounded on its own (division is the correctly rounded one), codes packed by lane pairs.
__global__ __launch_bounds__(256) void quantize_int4_kernel(const half_t* __restrict__ w, size_t n_groups,
                                                             uint8_t* __restrict__ packed, half_t* __restrict__ scale,
                                                             half_t* __restrict__ zero) {
    const size_t g = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= n_groups) return;
    const int lane = threadIdx.x & 63;
    const float v = (float)w[g * 64 + lane];
    float mn = v, mx = v;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, m, kWave));
    }
    const float range = __fsub_rn(mx, mn);
    const half_t s16 = f32_to_f16_rne(__fdiv_rn(range, 15.0f));
    const float s = (float)s16;
    uint32_t q = 0;
    if (s != 0.0f) {
        float r = rintf(__fdiv_rn(__fsub_rn(v, mn), s));
        r = fminf(fmaxf(r, 0.0f), 15.0f);
        q = (uint32_t)r;
    }
    const uint32_t hi = __shfl_down(q, 1, kWave);
    if ((lane & 1) == 0) packed[g * 32 + (lane >> 1)] = (uint8_t)(q | (hi << 4));
    if (lane == 0) {
        scale[g] = s16;
        zero[g] = (half_t)mn;
    }
}

void launch_quantize_int4(const half_t* w, int out, int in, uint8_t* packed, half_t* scale, half_t* zero,
                          hipStream_t st) {
    const size_t n_groups = (size_t)out * in / 64;
    if (n_groups == 0) return;
    quantize_int4_kernel<<<(unsigned)((n_groups + 3) / 4), 256, 0, st>>>(w, n_groups, packed, scale, zero);
}

// 8-bit form: one thread per 4 weights (one 32-bit word of codes).
__global__ __launch_bounds__(256) void dequant_int8_kernel(DevMat m, size_t n_words, int in, half_t* __restrict__ w) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_words) return;
    const size_t col0 = (i * 4) % (size_t)in, row = (i * 4) / (size_t)in;
    const size_t g = row * (size_t)(in >> 6) + (col0 >> 6);
    const float s = (float)m.scale[g], z = (float)m.zero[g];
    const uint32_t word = ((const uint32_t*)m.data)[i];
    half4_t o;
#pragma unroll
    for (int n = 0; n < 4; ++n) o[n] = dequant_one((word >> (8 * n)) & 0xFFu, s, z);
    *(half4_t*)(w + i * 4) = o;
}

void launch_dequant_int8(const DevMat& m, int out, int in, half_t* w, hipStream_t st) {
    const size_t n_words = (size_t)out * in / 4;
    if (n_words == 0) return;
    dequant_int8_kernel<<<(unsigned)((n_words + 255) / 256), 256, 0, st>>>(m, n_words, in, w);
}

// One wavefront per group of 64 weights, as in the 4-bit quantizer; one code per byte.
__global__ __launch_bounds__(256) void quantize_int8_kernel(const half_t* __restrict__ w, size_t n_groups,
                                                             uint8_t* __restrict__ codes, half_t* __restrict__ scale,
                                                             half_t* __restrict__ zero) {
    const size_t g = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= n_groups) return;
    const int lane = threadIdx.x & 63;
    const float v = (float)w[g * 64 + lane];
    float mn = v, mx = v;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, m, kWave));
    }
    const float range = __fsub_rn(mx, mn);
    const half_t s16 = f32_to_f16_rne(__fdiv_rn(range, 255.0f));
    const float s = (float)s16;
    uint32_t q = 0;
    if (s != 0.0f) {
        float r = rintf(__fdiv_rn(__fsub_rn(v, mn), s));
        r = fminf(fmaxf(r, 0.0f), 255.0f);
        q = (uint32_t)r;
    }
    codes[g * 64 + lane] = (uint8_t)q;
    if (lane == 0) {
        scale[g] = s16;
        zero[g] = (half_t)mn;
    }
}

void launch_quantize_int8(const half_t* w, int out, int in, uint8_t* codes, half_t* scale, half_t* zero, hipStream_t st) {
    const size_t n_groups = (size_t)out * in / 64;
    if (n_groups == 0) return;
    quantize_int8_kernel<<<(unsigned)((n_groups + 3) / 4), 256, 0, st>>>(w, n_groups, codes, scale, zero);
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Element i = pure function of (key, first + i); see the generator module for the recipe.
__global__ __launch_bounds__(256) void synth_fill_kernel(half_t* __restrict__ dst, size_t n, size_t first, uint64_t key,
                                                          float scale, int kind) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t j = (size_t)blockIdx.x * 256 + threadIdx.x; j < n; j += stride) {
        const uint64_t i = (uint64_t)first + j;
        const uint64_t h0 = mix64(key + 2 * i);
        int32_t c;
        if (kind == 0) {
            const uint64_t h1 = mix64(key + 2 * i + 1);
            uint32_t s = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                s += (uint32_t)((h0 >> (16 * b)) & 0xFFFFu);
                s += (uint32_t)((h1 >> (16 * b)) & 0xFFFFu);
            }
            c = 2 * (int32_t)s - 8 * 65535;
        } else {
            c = 2 * (int32_t)(h0 >> 40) - ((1 << 24) - 1);
        }
        dst[j] = f32_to_f16_rne(__fmul_rn((float)c, scale));
    }
}

void launch_synth_fill(half_t* dst, size_t n, size_t first, uint64_t seed, uint64_t stream_id, float scale, int kind,
                       hipStream_t st) {
    if (n == 0) return;
    // host-side key derivation (same two mixing steps as on the device)
    auto hmix = [](uint64_t z) {
        z += 0x9E3779B97F4A7C15ull;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    };
    const uint64_t key = hmix(hmix(seed) + stream_id);
    const size_t blocks = (n + 255) / 256;
    synth_fill_kernel<<<(unsigned)(blocks < 65536 ? blocks : 65536), 256, 0, st>>>(dst, n, first, key, scale, kind);
}

}  // namespace moemix
