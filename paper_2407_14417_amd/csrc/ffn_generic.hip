// Expert feed-forward layer, any number of rows per expert (paper §1: experts are parallel FF
// layers; §3: each is 16-bit or 4-bit).  One wavefront per weight row; activations of up to NT
// rows are staged in LDS and every weight is dequantized to its exact fp16 value in registers.
// This is the shape-agnostic path; decode and large-batch shapes have their own kernels.
#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

namespace {

constexpr int kRowsPerBlock = 16;

struct Span {
    int e, begin, end;
};

__device__ __forceinline__ Span block_span(const RowMap& rows) {
    Span s;
    if (rows.direct_expert >= 0) {
        s.e = rows.direct_expert;
        s.begin = 0;
        s.end = rows.direct_n;
    } else {
        s.e = blockIdx.y;
        s.begin = rows.offsets[s.e];
        s.end = rows.offsets[s.e + 1];
    }
    return s;
}

// acc[t] += sum_c w[c] * act[t][c] over this lane's share of one weight row of length K.
template <int NT>
__device__ __forceinline__ void row_dot_fp16(const half_t* __restrict__ wrow, const half_t* __restrict__ act, int K,
                                             int nt, int lane, float (&acc)[NT]) {
    for (int c = lane * 8; c < K; c += kWave * 8) {
        const half8_t wv = *(const half8_t*)(wrow + c);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (t < nt) {
                const half8_t xv = *(const half8_t*)(act + (size_t)t * K + c);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[t] += (float)wv[j] * (float)xv[j];
            }
        }
    }
}

template <int NT>
__device__ __forceinline__ void row_dot_int4(const uint8_t* __restrict__ qrow, const half_t* __restrict__ srow,
                                             const half_t* __restrict__ zrow, const half_t* __restrict__ act, int K,
                                             int nt, int lane, float (&acc)[NT]) {
    for (int c = lane * 32; c < K; c += kWave * 32) {
        const uint4_t pk = *(const uint4_t*)(qrow + (c >> 1));
        const float s = (float)srow[c >> 6], z = (float)zrow[c >> 6];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half8_t wv;
#pragma unroll
            for (int n = 0; n < 8; ++n) wv[n] = dequant_one((pk[j] >> (4 * n)) & 0xFu, s, z);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (t < nt) {
                    const half8_t xv = *(const half8_t*)(act + (size_t)t * K + c + j * 8);
#pragma unroll
                    for (int n = 0; n < 8; ++n) acc[t] += (float)wv[n] * (float)xv[n];
                }
            }
        }
    }
}

// 8-bit rows: a lane's 128-bit load holds 16 codes, all of one group of 64 columns.
template <int NT>
__device__ __forceinline__ void row_dot_int8(const uint8_t* __restrict__ qrow, const half_t* __restrict__ srow,
                                             const half_t* __restrict__ zrow, const half_t* __restrict__ act, int K,
                                             int nt, int lane, float (&acc)[NT]) {
    for (int c = lane * 16; c < K; c += kWave * 16) {
        const uint4_t pk = *(const uint4_t*)(qrow + c);
        const float s = (float)srow[c >> 6], z = (float)zrow[c >> 6];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            half4_t wv;
#pragma unroll
            for (int n = 0; n < 4; ++n) wv[n] = dequant_one((pk[j] >> (8 * n)) & 0xFFu, s, z);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (t < nt) {
                    const half4_t xv = *(const half4_t*)(act + (size_t)t * K + c + j * 4);
#pragma unroll
                    for (int n = 0; n < 4; ++n) acc[t] += (float)wv[n] * (float)xv[n];
                }
            }
        }
    }
}

template <int NT>
__global__ __launch_bounds__(256) void ffn_up_generic(DevExperts ex, RowMap rows, const half_t* __restrict__ x, int d,
                                                       int f, half_t* __restrict__ h, int32_t* status) {
    extern __shared__ half_t act[];   // [NT][d]
    const Span sp = block_span(rows);
    if (sp.begin >= sp.end) return;
    const DevExpert& ee = ex.e[sp.e];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (ee.resident == kDeferred) return;
    if (!ee.resident || !ee.w1.data) {
        if (tid == 0 && blockIdx.x == 0) atomicOr(status, kStatusNotResident);
        return;
    }
    const bool int4 = ee.prec == MOE_PREC_INT4G64, int8 = ee.prec == MOE_PREC_INT8G64;
    const int row0 = blockIdx.x * kRowsPerBlock;
    for (int rc = sp.begin; rc < sp.end; rc += NT) {
        const int nt = min(NT, sp.end - rc);
        __syncthreads();
        for (int t = 0; t < nt; ++t) {
            const int src = rows.perm ? rows.perm[rc + t] / rows.top_k : rc + t;
            for (int c = tid * 8; c < d; c += 256 * 8)
                *(half8_t*)(act + (size_t)t * d + c) = *(const half8_t*)(x + (size_t)src * d + c);
        }
        __syncthreads();
        for (int rp = wave; rp < kRowsPerBlock; rp += 4) {
            const int row = row0 + rp;
            if (row >= f) break;
            float a[NT], b[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) a[t] = b[t] = 0.0f;
            if (int4) {
                const int gpr = d >> 6;
                row_dot_int4<NT>(ee.w1.data + (size_t)row * (d >> 1), ee.w1.scale + (size_t)row * gpr,
                                 ee.w1.zero + (size_t)row * gpr, act, d, nt, lane, a);
                row_dot_int4<NT>(ee.w3.data + (size_t)row * (d >> 1), ee.w3.scale + (size_t)row * gpr,
                                 ee.w3.zero + (size_t)row * gpr, act, d, nt, lane, b);
            } else if (int8) {
                const int gpr = d >> 6;
                row_dot_int8<NT>(ee.w1.data + (size_t)row * d, ee.w1.scale + (size_t)row * gpr,
                                 ee.w1.zero + (size_t)row * gpr, act, d, nt, lane, a);
                row_dot_int8<NT>(ee.w3.data + (size_t)row * d, ee.w3.scale + (size_t)row * gpr,
                                 ee.w3.zero + (size_t)row * gpr, act, d, nt, lane, b);
            } else {
                row_dot_fp16<NT>((const half_t*)ee.w1.data + (size_t)row * d, act, d, nt, lane, a);
                row_dot_fp16<NT>((const half_t*)ee.w3.data + (size_t)row * d, act, d, nt, lane, b);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (t < nt) {
                    const float sa = wave_sum(a[t]), sb = wave_sum(b[t]);
                    if (lane == 0) h[(size_t)(rc + t) * f + row] = (half_t)silu_mul(sa, sb);
                }
            }
        }
    }
}

template <int NT>
__global__ __launch_bounds__(256) void ffn_down_generic(DevExperts ex, RowMap rows, const half_t* __restrict__ h, int d,
                                                         int f, float* __restrict__ y, int32_t* status) {
    extern __shared__ half_t act[];   // [NT][f]
    const Span sp = block_span(rows);
    if (sp.begin >= sp.end) return;
    const DevExpert& ee = ex.e[sp.e];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    if (ee.resident == kDeferred) return;
    if (!ee.resident || !ee.w2.data) {
        if (tid == 0 && blockIdx.x == 0) atomicOr(status, kStatusNotResident);
        // rows of an expert that cannot run contribute nothing
        for (int r = sp.begin; r < sp.end; ++r)
            for (int c = blockIdx.x * kRowsPerBlock + tid; c < min(d, (int)(blockIdx.x + 1) * kRowsPerBlock); c += 256)
                y[(size_t)r * d + c] = 0.0f;
        return;
    }
    const bool int4 = ee.prec == MOE_PREC_INT4G64, int8 = ee.prec == MOE_PREC_INT8G64;
    const int row0 = blockIdx.x * kRowsPerBlock;
    for (int rc = sp.begin; rc < sp.end; rc += NT) {
        const int nt = min(NT, sp.end - rc);
        __syncthreads();
        for (int t = 0; t < nt; ++t)
            for (int c = tid * 8; c < f; c += 256 * 8)
                *(half8_t*)(act + (size_t)t * f + c) = *(const half8_t*)(h + (size_t)(rc + t) * f + c);
        __syncthreads();
        for (int rp = wave; rp < kRowsPerBlock; rp += 4) {
            const int row = row0 + rp;
            if (row >= d) break;
            float a[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) a[t] = 0.0f;
            if (int4) {
                const int gpr = f >> 6;
                row_dot_int4<NT>(ee.w2.data + (size_t)row * (f >> 1), ee.w2.scale + (size_t)row * gpr,
                                 ee.w2.zero + (size_t)row * gpr, act, f, nt, lane, a);
            } else if (int8) {
                const int gpr = f >> 6;
                row_dot_int8<NT>(ee.w2.data + (size_t)row * f, ee.w2.scale + (size_t)row * gpr,
                                 ee.w2.zero + (size_t)row * gpr, act, f, nt, lane, a);
            } else {
                row_dot_fp16<NT>((const half_t*)ee.w2.data + (size_t)row * f, act, f, nt, lane, a);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (t < nt) {
                    const float sa = wave_sum(a[t]);
                    if (lane == 0) y[(size_t)(rc + t) * d + row] = sa;
                }
            }
        }
    }
}

}  // namespace

void launch_ffn_up(const DevExperts& ex, int E, const RowMap& rows, const half_t* x, int d, int f, half_t* h,
                   int32_t* status, hipStream_t st) {
    constexpr int NT = 4;
    TraceScope trace(kKernelUp, st);
    dim3 grid((f + kRowsPerBlock - 1) / kRowsPerBlock, rows.direct_expert >= 0 ? 1 : E);
    ffn_up_generic<NT><<<grid, 256, (size_t)NT * d * sizeof(half_t), st>>>(ex, rows, x, d, f, h, status);
}

void launch_ffn_down(const DevExperts& ex, int E, const RowMap& rows, const half_t* h, int d, int f, float* y,
                     int32_t* status, hipStream_t st) {
    constexpr int NT = 2;
    TraceScope trace(kKernelDown, st);
    dim3 grid((d + kRowsPerBlock - 1) / kRowsPerBlock, rows.direct_expert >= 0 ? 1 : E);
    ffn_down_generic<NT><<<grid, 256, (size_t)NT * f * sizeof(half_t), st>>>(ex, rows, h, d, f, y, status);
}

}  // namespace moemix
