// Gating network for one token, evaluated by one wavefront at a time (paper §1 gating, §2.1 top-k): shared by the
// gating kernel (any number of tokens) and by the batch-1 up-projection launch, which evaluates the gating
// network for its one token inside every workgroup instead of waiting for a separate launch.  Both use exactly
// the functions below, so both give the same bits for the same token.
//
// Order of the arithmetic (what makes the result reproducible): lane L of the wavefront owns the 8-column chunks
// L, L + 64, L + 128, ... of the row; sums run over its chunks in that order, element pairs in column order, in one
// fp32 accumulator; lane sums are added over the wavefront by wave_total.
#pragma once

#include "common.hpp"

namespace moemix {

#if defined(__HIPCC__)

constexpr int kGateMaxChunks = 16;     // d_model <= 8192: at most 16 chunks of 8 columns per lane

// The lane's chunks of one fp16 row of length d (d a multiple of 8): chunk j holds columns (lane + 64 j) * 8 .. + 8.
// Chunks past the end of the row are zero.
struct GateRow {
    uint4_t v[kGateMaxChunks];
};

template <int NCHUNK>
__device__ __forceinline__ void gate_load_row(const half_t* __restrict__ row, int d, int lane, uint4_t (&v)[NCHUNK]) {
#pragma unroll
    for (int j = 0; j < NCHUNK; ++j) {
        const int c = (lane + 64 * j) * 8;
        v[j] = c < d ? *(const uint4_t*)(row + c) : uint4_t{0u, 0u, 0u, 0u};
    }
}

// RMSNorm of the row held in v (non-expert part of the chained configuration, always 16-bit: paper §3):
// v <- fp16( v / sqrt(mean(v^2) + eps) * gain ), every wavefront for itself.
template <int NCHUNK>
__device__ __forceinline__ void gate_rmsnorm(uint4_t (&v)[NCHUNK], const half_t* __restrict__ gain, int d, float eps,
                                             int lane) {
    float ss = 0.0f;
#pragma unroll
    for (int j = 0; j < NCHUNK; ++j) {
        const half8_t x = __builtin_bit_cast(half8_t, v[j]);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += (float)x[i] * (float)x[i];
    }
    ss = wave_total(ss);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int j = 0; j < NCHUNK; ++j) {
        const int c = (lane + 64 * j) * 8;
        if (c < d) {
            const half8_t x = __builtin_bit_cast(half8_t, v[j]), g = *(const half8_t*)(gain + c);
            half8_t o;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (half_t)((float)x[i] * inv * (float)g[i]);
            v[j] = __builtin_bit_cast(uint4_t, o);
        }
    }
}

// Router logit of one expert: sum over the row of x * w_gate[e], (+ bias), returned to every lane.
template <int NCHUNK>
__device__ __forceinline__ float gate_logit(const uint4_t (&xv)[NCHUNK], const half_t* __restrict__ wrow, int d,
                                            int lane) {
    uint4_t wv[NCHUNK];
    gate_load_row<NCHUNK>(wrow, d, lane, wv);
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < NCHUNK; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc = __builtin_amdgcn_fdot2(as_half2(xv[j][i]), as_half2(wv[j][i]), acc, false);
    return wave_total(acc);
}

// Top-k by k selection passes over the E logits (strict ">" keeps the lower index among equal logits), in
// descending order of the logit.  Every thread that calls it gets the same result.
__device__ __forceinline__ void gate_select(const float* __restrict__ logit, int E, int k, int (&sel)[MOE_MAX_TOPK],
                                            float (&lsel)[MOE_MAX_TOPK]) {
    uint32_t taken = 0;
#pragma unroll
    for (int s = 0; s < MOE_MAX_TOPK; ++s) {
        if (s < k) {
            int best = -1;
            float lb = 0.0f;
            for (int e = 0; e < E; ++e) {
                if (taken & (1u << e)) continue;
                const float l = logit[e];
                if (best < 0 || l > lb) { best = e; lb = l; }
            }
            taken |= 1u << best;
            sel[s] = best;
            lsel[s] = lb;
        }
    }
}

// Softmax over the k selected logits: the weights of the weighted average.
__device__ __forceinline__ void gate_weights(const float (&lsel)[MOE_MAX_TOPK], int k, float (&g)[MOE_MAX_TOPK]) {
    float denom = 0.0f;
#pragma unroll
    for (int s = 0; s < MOE_MAX_TOPK; ++s)
        if (s < k) { g[s] = expf(lsel[s] - lsel[0]); denom += g[s]; }
#pragma unroll
    for (int s = 0; s < MOE_MAX_TOPK; ++s)
        if (s < k) g[s] = g[s] / denom;
}

#endif  // __HIPCC__

}  // namespace moemix
