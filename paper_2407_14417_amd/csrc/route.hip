// Gating network with top-k selection (paper §1, §2.1) and the grouping of (token, slot)
// pairs by expert.
#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

// One workgroup per token.  Each thread takes 8-column chunks of the token row and of every
// gate row (one 128-bit load each), accumulates E partial logits in fp32, the partials are
// summed with wavefront shuffles and a 4-entry LDS step in a fixed order, then lane 0 runs
// top_k selection passes (strict ">" keeps the lower index among equal logits) and the softmax
// over the selected logits.
template <int EMAX>
__global__ __launch_bounds__(512) void route_kernel(const half_t* __restrict__ x, const half_t* __restrict__ wg,
                                                     const float* __restrict__ bias, int d, int E, int k,
                                                     int32_t* __restrict__ idx, float* __restrict__ gate,
                                                     int32_t* __restrict__ idx2, float* __restrict__ gate2,
                                                     int32_t* __restrict__ status, const half_t* __restrict__ rms_gain,
                                                     float eps, half_t* __restrict__ xn) {
    __shared__ float part[8][EMAX];
    __shared__ float logit[EMAX];
    __shared__ float sq[8];
    const int t = blockIdx.x;
    const int tid = threadIdx.x, n_waves = blockDim.x >> 6;
    const int wave = tid >> 6, lane = tid & 63;
    if (t == 0 && tid == 0 && status) *status = 0;   // status word describes the call that starts here
    float acc[EMAX];
#pragma unroll
    for (int e = 0; e < EMAX; ++e) acc[e] = 0.0f;
    const half_t* xr = x + (size_t)t * d;
    // chained configuration: the block input is RMSNorm(x) * gain, rounded to fp16; it is written to xn for the
    // expert kernels and used for the logits in the same pass
    float inv = 1.0f;
    if (rms_gain) {
        float ss = 0.0f;
        for (int c = tid * 8; c < d; c += blockDim.x * 8) {
            const half8_t v = *(const half8_t*)(xr + c);
#pragma unroll
            for (int j = 0; j < 8; ++j) ss += (float)v[j] * (float)v[j];
        }
        ss = wave_total(ss);
        if (lane == 0) sq[wave] = ss;
        __syncthreads();
        float total = 0.0f;
        for (int w = 0; w < n_waves; ++w) total += sq[w];
        inv = 1.0f / sqrtf(total / (float)d + eps);
    }
    for (int c = tid * 8; c < d; c += blockDim.x * 8) {
        uint4_t xv = *(const uint4_t*)(xr + c);
        if (rms_gain) {
            const half8_t v = __builtin_bit_cast(half8_t, xv), g = *(const half8_t*)(rms_gain + c);
            half8_t o;
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = (half_t)((float)v[j] * inv * (float)g[j]);
            *(half8_t*)(xn + (size_t)t * d + c) = o;
            xv = __builtin_bit_cast(uint4_t, o);
        }
        uint4_t wv[EMAX];
#pragma unroll
        for (int e = 0; e < EMAX; ++e)
            if (e < E) wv[e] = *(const uint4_t*)(wg + (size_t)e * d + c);
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if (e < E) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[e] = __builtin_amdgcn_fdot2(as_half2(xv[j]), as_half2(wv[e][j]), acc[e], false);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
        if (e < E) {
            const float s = wave_total(acc[e]);
            if (lane == 0) part[wave][e] = s;
        }
    }
    __syncthreads();
    if (tid < E) {
        float s = 0.0f;
        for (int w = 0; w < n_waves; ++w) s += part[w][tid];
        logit[tid] = s + (bias ? bias[tid] : 0.0f);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t taken = 0;
        int sel[MOE_MAX_TOPK];
        float lsel[MOE_MAX_TOPK];
        for (int s = 0; s < k; ++s) {
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
        float u[MOE_MAX_TOPK];
        float denom = 0.0f;
        for (int s = 0; s < k; ++s) { u[s] = expf(lsel[s] - lsel[0]); denom += u[s]; }
        for (int s = 0; s < k; ++s) {
            const float g = u[s] / denom;
            idx[(size_t)t * k + s] = sel[s];
            gate[(size_t)t * k + s] = g;
            if (idx2) idx2[(size_t)t * k + s] = sel[s];
            if (gate2) gate2[(size_t)t * k + s] = g;
        }
    }
}

void launch_route(const half_t* x, const half_t* wg, const float* bias, int T, int d, int E, int k, int32_t* idx,
                  float* gate, int32_t* idx2, float* gate2, int32_t* status, hipStream_t st, const half_t* rms_gain,
                  float eps, half_t* xn) {
    TraceScope trace(kKernelRoute, st);
    int threads = (d / 8 + 63) / 64 * 64;      // one 8-column chunk per thread when the row fits
    threads = threads < 64 ? 64 : (threads > 512 ? 512 : threads);
    if (E <= 8)
        route_kernel<8><<<T, threads, 0, st>>>(x, wg, bias, d, E, k, idx, gate, idx2, gate2, status, rms_gain, eps, xn);
    else
        route_kernel<MOE_MAX_EXPERTS><<<T, threads, 0, st>>>(x, wg, bias, d, E, k, idx, gate, idx2, gate2, status, rms_gain, eps,
                                                               xn);
}

// One workgroup.  Wave w owns experts w, w+16: it walks all pairs in order, 64 at a time, and a
// ballot + popcount gives every pair routed to its expert a rank in increasing pair order, so the
// grouping is the unique stable one.
__global__ __launch_bounds__(1024) void permute_kernel(const int32_t* __restrict__ idx, int P, int E,
                                                        int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                                        int32_t* __restrict__ perm, int32_t* __restrict__ inv,
                                                        int32_t* __restrict__ status) {
    __shared__ int32_t cnt[MOE_MAX_EXPERTS];
    __shared__ int32_t off[MOE_MAX_EXPERTS + 1];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int e = wave; e < E; e += 16) {
        int c = 0;
        for (int i0 = 0; i0 < P; i0 += 64) {
            const int i = i0 + lane;
            const int v = (i < P) ? idx[i] : -1;
            c += __popcll(__ballot(v == e));
        }
        if (lane == 0) cnt[e] = c;
    }
    // pairs with an index outside [0, E) belong to no expert: flag them
    for (int i = tid; i < P; i += 1024) {
        const int v = idx[i];
        if (v < 0 || v >= E) {
            inv[i] = -1;
            atomicOr(status, kStatusBadIndex);
        }
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) { off[e] = run; run += cnt[e]; }
        off[E] = run;
    }
    __syncthreads();
    if (tid <= E) offsets[tid] = off[tid];
    if (tid < E) counts[tid] = cnt[tid];
    for (int e = wave; e < E; e += 16) {
        int base = off[e];
        for (int i0 = 0; i0 < P; i0 += 64) {
            const int i = i0 + lane;
            const int v = (i < P) ? idx[i] : -1;
            const unsigned long long m = __ballot(v == e);
            if (v == e) {
                const int r = base + __popcll(m & ((1ull << lane) - 1ull));
                perm[r] = i;
                inv[i] = r;
            }
            base += __popcll(m);
        }
    }
}

void launch_permute(const int32_t* idx, int P, int E, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                    int32_t* status, hipStream_t st) {
    TraceScope trace(kKernelPermute, st);
    permute_kernel<<<1, 1024, 0, st>>>(idx, P, E, counts, offsets, perm, inv, status);
}

}  // namespace moemix
