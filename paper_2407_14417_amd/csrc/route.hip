// Gating network with top-k selection (paper §1, §2.1) and the grouping of (token, slot)
// pairs by expert.
#include "common.hpp"
#include "gating.hpp"
#include "kernels.hpp"

namespace moemix {

// One workgroup of four wavefronts per token.  Every wavefront holds the whole token row (lane L the 8-column
// chunks L, L + 64, ...), normalises it when the block input is RMSNorm(x) * gain, and evaluates the experts
// w, w + 4, ... of the gate matrix, each as one wavefront-wide dot product (gating.hpp); thread 0 then runs the
// top_k selection passes and the softmax over the selected logits.
template <int NCHUNK>
__global__ __launch_bounds__(256) void route_kernel(const half_t* __restrict__ x, const half_t* __restrict__ wg,
                                                     const float* __restrict__ bias, int d, int E, int k,
                                                     int32_t* __restrict__ idx, float* __restrict__ gate,
                                                     int32_t* __restrict__ idx2, float* __restrict__ gate2,
                                                     int32_t* __restrict__ status, const half_t* __restrict__ rms_gain,
                                                     float eps, half_t* __restrict__ xn) {
    __shared__ float logit[MOE_MAX_EXPERTS];
    const int t = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (t == 0 && tid == 0 && status) *status = 0;   // status word describes the call that starts here
    uint4_t xv[NCHUNK];
    gate_load_row<NCHUNK>(x + (size_t)t * d, d, lane, xv);
    if (rms_gain) {
        // chained configuration: the block input is RMSNorm(x) * gain, rounded to fp16; it is written to xn for the
        // expert kernels and used for the logits in the same pass
        gate_rmsnorm<NCHUNK>(xv, rms_gain, d, eps, lane);
        if (wave == 0) {
#pragma unroll
            for (int j = 0; j < NCHUNK; ++j) {
                const int c = (lane + 64 * j) * 8;
                if (c < d) *(uint4_t*)(xn + (size_t)t * d + c) = xv[j];
            }
        }
    }
    for (int e = wave; e < E; e += 4) {
        const float l = gate_logit<NCHUNK>(xv, wg + (size_t)e * d, d, lane);
        if (lane == 0) logit[e] = l + (bias ? bias[e] : 0.0f);
    }
    __syncthreads();
    if (tid == 0) {
        int sel[MOE_MAX_TOPK];
        float lsel[MOE_MAX_TOPK], g[MOE_MAX_TOPK];
        gate_select(logit, E, k, sel, lsel);
        gate_weights(lsel, k, g);
#pragma unroll
        for (int s = 0; s < MOE_MAX_TOPK; ++s) {
            if (s < k) {
                idx[(size_t)t * k + s] = sel[s];
                gate[(size_t)t * k + s] = g[s];
                if (idx2) idx2[(size_t)t * k + s] = sel[s];
                if (gate2) gate2[(size_t)t * k + s] = g[s];
            }
        }
    }
}

void launch_route(const half_t* x, const half_t* wg, const float* bias, int T, int d, int E, int k, int32_t* idx,
                  float* gate, int32_t* idx2, float* gate2, int32_t* status, hipStream_t st, const half_t* rms_gain,
                  float eps, half_t* xn) {
    TraceScope trace(kKernelRoute, st);
    if (d <= 2048)
        route_kernel<4><<<T, 256, 0, st>>>(x, wg, bias, d, E, k, idx, gate, idx2, gate2, status, rms_gain, eps, xn);
    else if (d <= 4096)
        route_kernel<8><<<T, 256, 0, st>>>(x, wg, bias, d, E, k, idx, gate, idx2, gate2, status, rms_gain, eps, xn);
    else
        route_kernel<kGateMaxChunks><<<T, 256, 0, st>>>(x, wg, bias, d, E, k, idx, gate, idx2, gate2, status, rms_gain, eps,
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
