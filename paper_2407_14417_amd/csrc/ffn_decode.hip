// Batch-1 decode path of the expert feed-forward layers (paper §1, §3): one token, top_k routed
// experts, each 16-bit or 4-bit.  Both projections are bandwidth-bound GEMVs:
//   up  : h_s[r] = silu(W1_s[r,:] . x) * (W3_s[r,:] . x)           for every routed slot s
//   down: out[r] = fp16( residual[r] + sum_s gate_s * (W2_s[r,:] . h_s) )    (weighted average fused)
// The token (or the hidden row) sits in registers in the order the weight loads deliver columns, so
// the inner loop is: one coalesced 128-bit load per lane -> bit-trick unpack -> packed dot products
// with fp32 accumulation.  4-bit rows use the factored form of the group-wise dequantization,
//   sum_c (q_c*s + z) x_c = s * sum_c q_c x_c + z * sum_c x_c,
// with the per-lane sums of x precomputed once, so a weight costs about 1.3 vector instructions.
#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

namespace {

// ---------------------------------------------------------------- activations in registers

// 4-bit layout.  A lane's 128-bit load holds 32 consecutive codes: 4 words of 8 nibbles.  Masking a word
// with 0x000F000F / 0x00F000F0 (before and after a shift by 8) yields the code pairs of columns (0,4),
// (1,5), (2,6), (3,7) inside the mantissa of fp16 1024.0, so the activations are kept in that pairing.
struct ActI4 {
    half2_t p[4][4];   // [word][pair]
    float c1;          // 1024 * (sum of even-column x + sum of odd-column x / 16): offset of the biased codes
    float c2;          // sum of the 32 x: multiplies the group zero
};

__device__ __forceinline__ void load_act_i4(const half_t* __restrict__ src, ActI4& a) {
    float se = 0.0f, so = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const half8_t v = *(const half8_t*)(src + 8 * j);
#pragma unroll
        for (int q = 0; q < 4; ++q) a.p[j][q] = half2_t{v[q], v[q + 4]};
        se += ((float)v[0] + (float)v[2]) + ((float)v[4] + (float)v[6]);
        so += ((float)v[1] + (float)v[3]) + ((float)v[5] + (float)v[7]);
    }
    a.c1 = 1024.0f * se + 64.0f * so;
    a.c2 = se + so;
}

// s * sum_c q_c x_c + z * sum_c x_c over the lane's 32 columns of one row.
__device__ __forceinline__ float dot_i4(const uint4_t pk, const ActI4& a, float s, float z) {
    constexpr uint32_t kMagic = 0x64006400u;   // fp16 pair (1024, 1024)
    float lo = 0.0f, hi = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t w = pk[j], w8 = w >> 8;
        const half2_t q04 = as_half2((w & 0x000F000Fu) | kMagic);    // 1024 + q
        const half2_t q15 = as_half2((w & 0x00F000F0u) | kMagic);    // 1024 + 16 q
        const half2_t q26 = as_half2((w8 & 0x000F000Fu) | kMagic);
        const half2_t q37 = as_half2((w8 & 0x00F000F0u) | kMagic);
        lo = __builtin_amdgcn_fdot2(q04, a.p[j][0], lo, false);
        hi = __builtin_amdgcn_fdot2(q15, a.p[j][1], hi, false);
        lo = __builtin_amdgcn_fdot2(q26, a.p[j][2], lo, false);
        hi = __builtin_amdgcn_fdot2(q37, a.p[j][3], hi, false);
    }
    const float t = fmaf(hi, 0.0625f, lo) - a.c1;
    return fmaf(s, t, z * a.c2);
}

// 16-bit layout: a lane's 128-bit load holds 8 consecutive weights, natural pairs.
struct ActF16 {
    half2_t p[4];
};

__device__ __forceinline__ void load_act_f16(const half_t* __restrict__ src, ActF16& a) {
    const half8_t v = *(const half8_t*)src;
#pragma unroll
    for (int q = 0; q < 4; ++q) a.p[q] = half2_t{v[2 * q], v[2 * q + 1]};
}

__device__ __forceinline__ float dot_f16(const uint4_t w, const ActF16& a, float acc) {
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_fdot2(as_half2(w[q]), a.p[q], acc, false);
    return acc;
}

__device__ __forceinline__ uint4_t load_stream(const void* p) {
    return __builtin_nontemporal_load((const uint4_t*)p);
}

// ---------------------------------------------------------------- up-projection

// Rows of all routed slots are laid end to end, weighted by their stored bytes (9 units per 4-bit row
// pair, 32 per 16-bit one), and cut into equal shares, one per wavefront: every wavefront streams the
// same number of bytes whatever the precision mix.
template <int NCH>   // d_model / 2048
__global__ __launch_bounds__(256) void decode_up_kernel(DevExperts ex, const int32_t* __restrict__ idx,
                                                         const half_t* __restrict__ x, int f, int k,
                                                         half_t* __restrict__ h, int32_t* status) {
    constexpr int d = NCH * 2048;
    const int lane = threadIdx.x & 63;
    const long n_waves = (long)gridDim.x * 4, gw = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    long total = 0;
    for (int s = 0; s < k; ++s) total += (long)f * (ex.e[idx[s]].prec == MOE_PREC_INT4G64 ? 9 : 32);
    const long lo = total * gw / n_waves, hi = total * (gw + 1) / n_waves;
    long base = 0;
    for (int s = 0; s < k; ++s) {
        const DevExpert& ee = ex.e[idx[s]];
        const bool int4 = ee.prec == MOE_PREC_INT4G64;
        const long cost = int4 ? 9 : 32;
        // rows whose first cost unit falls in [lo, hi)
        long r0 = (lo - base + cost - 1) / cost, r1 = (hi - base + cost - 1) / cost;
        r0 = r0 < 0 ? 0 : (r0 > f ? f : r0);
        r1 = r1 < 0 ? 0 : (r1 > f ? f : r1);
        base += (long)f * cost;
        if (r0 >= r1) continue;
        if (!ee.resident || !ee.w1.data) {
            if (lane == 0) atomicOr(status, kStatusNotResident);
            continue;
        }
        half_t* hs = h + (size_t)s * f;
        if (int4) {
            ActI4 act[NCH];
#pragma unroll
            for (int c = 0; c < NCH; ++c) load_act_i4(x + c * 2048 + lane * 32, act[c]);
            constexpr int gpr = d / 64;
            const uint8_t* q1 = ee.w1.data + lane * 16;
            const uint8_t* q3 = ee.w3.data + lane * 16;
            const half_t *s1 = ee.w1.scale + (lane >> 1), *z1 = ee.w1.zero + (lane >> 1);
            const half_t *s3 = ee.w3.scale + (lane >> 1), *z3 = ee.w3.zero + (lane >> 1);
            for (long r = r0; r < r1; r += 2) {
                uint4_t pk1[2][NCH], pk3[2][NCH];
                half_t sc1[2][NCH], zr1[2][NCH], sc3[2][NCH], zr3[2][NCH];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const long row = (r + i < r1) ? r + i : r1 - 1;
#pragma unroll
                    for (int c = 0; c < NCH; ++c) {
                        pk1[i][c] = load_stream(q1 + row * (d / 2) + c * 1024);
                        pk3[i][c] = load_stream(q3 + row * (d / 2) + c * 1024);
                        sc1[i][c] = s1[row * gpr + c * 32];
                        zr1[i][c] = z1[row * gpr + c * 32];
                        sc3[i][c] = s3[row * gpr + c * 32];
                        zr3[i][c] = z3[row * gpr + c * 32];
                    }
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    float a = 0.0f, b = 0.0f;
#pragma unroll
                    for (int c = 0; c < NCH; ++c) {
                        a += dot_i4(pk1[i][c], act[c], (float)sc1[i][c], (float)zr1[i][c]);
                        b += dot_i4(pk3[i][c], act[c], (float)sc3[i][c], (float)zr3[i][c]);
                    }
                    a = wave_total(a);
                    b = wave_total(b);
                    if (lane == 0 && r + i < r1) hs[r + i] = (half_t)silu_mul(a, b);
                }
            }
        } else {
            constexpr int NL = d / 512;   // 128-bit loads per row
            ActF16 act[NL];
#pragma unroll
            for (int c = 0; c < NL; ++c) load_act_f16(x + c * 512 + lane * 8, act[c]);
            const half_t* w1 = (const half_t*)ee.w1.data + lane * 8;
            const half_t* w3 = (const half_t*)ee.w3.data + lane * 8;
            for (long r = r0; r < r1; ++r) {
                uint4_t v1[NL], v3[NL];
#pragma unroll
                for (int c = 0; c < NL; ++c) {
                    v1[c] = load_stream(w1 + r * d + c * 512);
                    v3[c] = load_stream(w3 + r * d + c * 512);
                }
                float a = 0.0f, b = 0.0f;
#pragma unroll
                for (int c = 0; c < NL; ++c) {
                    a = dot_f16(v1[c], act[c], a);
                    b = dot_f16(v3[c], act[c], b);
                }
                a = wave_total(a);
                b = wave_total(b);
                if (lane == 0) hs[r] = (half_t)silu_mul(a, b);
            }
        }
    }
}

// ---------------------------------------------------------------- down-projection + weighted average

// One workgroup per 8 output rows; wavefront w owns columns [2048 w, 2048 w + 2048) of every row, for
// every slot in turn, with that slice of the slot's hidden row in registers.  Partial sums meet in LDS
// and are added in wavefront order, so the result does not depend on scheduling.
constexpr int kDownRows = 8;

__global__ __launch_bounds__(512) void decode_down_kernel(DevExperts ex, const int32_t* __restrict__ idx,
                                                           const float* __restrict__ gate,
                                                           const half_t* __restrict__ h, int d, int f, int k,
                                                           const half_t* __restrict__ residual,
                                                           half_t* __restrict__ out, int32_t* status) {
    __shared__ float part[8][kDownRows];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int row0 = blockIdx.x * kDownRows;
    float acc[kDownRows];
#pragma unroll
    for (int r = 0; r < kDownRows; ++r) acc[r] = 0.0f;
    for (int s = 0; s < k; ++s) {
        const DevExpert& ee = ex.e[idx[s]];
        if (!ee.resident || !ee.w2.data) {
            if (threadIdx.x == 0 && blockIdx.x == 0) atomicOr(status, kStatusNotResident);
            continue;
        }
        const float g = gate[s];
        const half_t* hs = h + (size_t)s * f + wave * 2048;
        if (ee.prec == MOE_PREC_INT4G64) {
            ActI4 act;
            load_act_i4(hs + lane * 32, act);
            const int gpr = f >> 6;
            const uint8_t* q = ee.w2.data + (size_t)row0 * (f >> 1) + wave * 1024 + lane * 16;
            const half_t* sc = ee.w2.scale + (size_t)row0 * gpr + wave * 32 + (lane >> 1);
            const half_t* zr = ee.w2.zero + (size_t)row0 * gpr + wave * 32 + (lane >> 1);
            uint4_t pk[kDownRows];
            half_t sv[kDownRows], zv[kDownRows];
#pragma unroll
            for (int r = 0; r < kDownRows; ++r) {
                pk[r] = load_stream(q + (size_t)r * (f >> 1));
                sv[r] = sc[(size_t)r * gpr];
                zv[r] = zr[(size_t)r * gpr];
            }
#pragma unroll
            for (int r = 0; r < kDownRows; ++r) acc[r] = fmaf(g, dot_i4(pk[r], act, (float)sv[r], (float)zv[r]), acc[r]);
        } else {
            ActF16 act[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) load_act_f16(hs + c * 512 + lane * 8, act[c]);
            const half_t* w = (const half_t*)ee.w2.data + (size_t)row0 * f + wave * 2048 + lane * 8;
#pragma unroll
            for (int rb = 0; rb < kDownRows; rb += 4) {
                uint4_t v[4][4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[r][c] = load_stream(w + (size_t)(rb + r) * f + c * 512);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float p = 0.0f;
#pragma unroll
                    for (int c = 0; c < 4; ++c) p = dot_f16(v[r][c], act[c], p);
                    acc[rb + r] = fmaf(g, p, acc[rb + r]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kDownRows; ++r) {
        const float t = wave_total(acc[r]);
        if (lane == 0) part[wave][r] = t;
    }
    __syncthreads();
    if (threadIdx.x < kDownRows) {
        const int row = row0 + threadIdx.x;
        float t = residual ? (float)residual[row] : 0.0f;
        float sum = 0.0f;
        for (int w = 0; w < n_waves; ++w) sum += part[w][threadIdx.x];
        out[row] = (half_t)(t + sum);
    }
}

}  // namespace

bool decode_shape_ok(int d, int f) { return d % 2048 == 0 && d <= 8192 && f % 2048 == 0 && f <= 16384 && d % kDownRows == 0; }

void launch_decode_up(const DevExperts& ex, const int32_t* idx, const half_t* x, int d, int f, int k, half_t* h,
                      int32_t* status, int blocks, hipStream_t st) {
    TraceScope trace(kKernelUp, st);
    switch (d / 2048) {
        case 1: decode_up_kernel<1><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status); break;
        case 2: decode_up_kernel<2><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status); break;
        case 3: decode_up_kernel<3><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status); break;
        default: decode_up_kernel<4><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status); break;
    }
}

void launch_decode_down(const DevExperts& ex, const int32_t* idx, const float* gate, const half_t* h, int d, int f,
                        int k, const half_t* residual, half_t* out, int32_t* status, hipStream_t st) {
    TraceScope trace(kKernelDown, st);
    decode_down_kernel<<<d / kDownRows, (f / 2048) * 64, 0, st>>>(ex, idx, gate, h, d, f, k, residual, out, status);
}

}  // namespace moemix
