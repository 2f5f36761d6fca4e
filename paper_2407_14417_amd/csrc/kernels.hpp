// Host-callable launchers of the moemix kernels (internal to the library).
#pragma once

#include "common.hpp"

namespace moemix {

// How the matrix kernels find their rows.
//   grouped: rows [offsets[e], offsets[e+1]) of the grouped order belong to expert e; grouped row r
//            reads token perm[r] / top_k of x.
//   direct : one given expert, rows 0..n-1 of x in order (moe_expert_ffn_mixed).
struct RowMap {
    const int32_t* offsets;  // device [E+1] or nullptr (direct)
    const int32_t* perm;     // device [P] or nullptr (direct)
    int top_k;
    int direct_expert;       // >= 0: direct mode
    int direct_n;
};

// rms_gain != null: the gating input is RMSNorm(x) * rms_gain (fp16), which is also written to xn [T, d].
void launch_route(const half_t* x, const half_t* wg, const float* bias, int T, int d, int E, int k, int32_t* idx,
                  float* gate, int32_t* idx2, float* gate2, int32_t* status, hipStream_t st,
                  const half_t* rms_gain = nullptr, float eps = 0.0f, half_t* xn = nullptr);
void launch_permute(const int32_t* idx, int P, int E, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv,
                    int32_t* status, hipStream_t st);

// h[r, :] = silu(W1 x_r) * (W3 x_r) for every row of every expert that has rows.
void launch_ffn_up(const DevExperts& ex, int E, const RowMap& rows, const half_t* x, int d, int f, half_t* h,
                   int32_t* status, hipStream_t st);
// y[r, :] = W2 h[r, :]
void launch_ffn_down(const DevExperts& ex, int E, const RowMap& rows, const half_t* h, int d, int f, float* y,
                     int32_t* status, hipStream_t st);

// Matrix-core path for many rows (contraction lengths multiples of 128).  `ct` = 16-row activation tiles per
// chunk (1, 2, 4 or 8); the down-projection splits the contraction `splits` ways and writes one partial
// y per split (`split_stride` elements apart), which launch_combine adds up.
struct MfmaPlan {
    int ct;
    int down_splits;
};
bool mfma_shape_ok(int d, int f);
bool mfma_rows_ok(int rows, int d, int f);
MfmaPlan plan_mfma(int P, int d, int f, int E);
void launch_ffn_up_mfma(const DevExperts& ex, int E, const RowMap& rows, int P, const half_t* x, int d, int f, half_t* h,
                        int ct, int32_t* status, hipStream_t st);
void launch_ffn_down_mfma(const DevExperts& ex, int E, const RowMap& rows, int P, const half_t* h, int d, int f, float* y,
                          int ct, int splits, size_t split_stride, int32_t* status, hipStream_t st);

// Batch-1 decode path (one token): shapes it covers, and its two kernels.
bool decode_shape_ok(int d, int f);
// Gating network evaluated inside the up-projection launch (one token): gate matrix [E, d], optional bias,
// optional RMSNorm of the token first (rms_gain != null); the routing result goes to idx_ws / gate_ws [top_k] for
// the down-projection launch and, if wanted, to idx_out / gate_out.  The launch then also clears the status word.
struct GateArgs {
    const half_t* wg;
    const float* bias;
    int E;
    const half_t* rms_gain;
    float eps;
    int32_t* idx_ws;
    float* gate_ws;
    int32_t* idx_out;
    float* gate_out;
};
// gating == null: the routing result is read from idx [top_k].
void launch_decode_up(const DevExperts& ex, const int32_t* idx, const half_t* x, int d, int f, int k, half_t* h,
                      int32_t* status, int blocks, hipStream_t st, const GateArgs* gating = nullptr);
// out32 != null: the result is written there unrounded (fp32) instead of to `out`.
void launch_decode_down(const DevExperts& ex, const int32_t* idx, const float* gate, const half_t* h, int d, int f,
                        int k, const half_t* residual, half_t* out, int32_t* status, hipStream_t st,
                        float* out32 = nullptr);
// idx[0] = expert, gate[0] = 1: one expert alone through the batch-1 kernels.
void launch_single_route(int32_t* idx, float* gate, int expert, hipStream_t st);

// out[t, :] = fp16( (residual ? residual[t, :] : 0) + sum_s gate[t, s] * sum_p y[p][inv[t*k + s], :] ),
// p over the `splits` partial results, `split_stride` elements apart.
void launch_combine(const float* y, int splits, size_t split_stride, const float* gate, const int32_t* inv, int T, int d,
                    int k, const half_t* residual, half_t* out, hipStream_t st);
// dst[i] = sum_p y[p][i] for i < n (n a multiple of 4), p over the `splits` partial results `split_stride` elements apart
void launch_reduce_splits(const float* y, int splits, size_t split_stride, size_t n, float* dst, hipStream_t st);
void launch_zero_words(int32_t* p, int n, hipStream_t st);

void launch_dequant_int4(const DevMat& m, int out, int in, half_t* w, hipStream_t st);
void launch_quantize_int4(const half_t* w, int out, int in, uint8_t* packed, half_t* scale, half_t* zero,
                          hipStream_t st);
// Reads `bytes` (a multiple of 16) of device memory once with streamed 128-bit loads.
void launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int blocks, hipStream_t st);
void launch_dequant_int8(const DevMat& m, int out, int in, half_t* w, hipStream_t st);
void launch_quantize_int8(const half_t* w, int out, int in, uint8_t* codes, half_t* scale, half_t* zero, hipStream_t st);
void launch_synth_fill(half_t* dst, size_t n, size_t first, uint64_t seed, uint64_t stream_id, float scale, int kind,
                       hipStream_t st);

}  // namespace moemix

namespace moemix {

// Kernel ids for moe_trace_kernel (same values as MOE_KERNEL_* in the public header).
enum KernelId { kKernelRoute = 0, kKernelPermute = 1, kKernelUp = 2, kKernelDown = 3, kKernelCombine = 4,
                kKernelStreamRead = 5, kKernelCount = 6 };

// One-shot event bracket around the next launch of a given kernel on this thread.
void trace_arm(int kernel, hipEvent_t start, hipEvent_t stop);
void trace_disarm(int kernel);
struct TraceScope {
    int kernel;
    hipStream_t st;
    TraceScope(int kernel, hipStream_t st);
    ~TraceScope();
};

}  // namespace moemix
