// C-ABI entry points of libmoemix (declared and documented in include/moemix.h): argument
// checks, workspace carving, kernel sequencing.  No allocation, no synchronization except in
// moe_read_status.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "common.hpp"
#include "kernels.hpp"

using namespace moemix;

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_hip(hipStream_t) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
    return MOE_OK;
}

int check_layer(const moe_layer* L) {
    if (!L) return fail(MOE_EINVAL, "layer is NULL");
    if (!L->w_gate || !L->experts) return fail(MOE_EINVAL, "layer.w_gate / layer.experts is NULL");
    if (L->d_model < 64 || L->d_ff < 64 || L->d_model % MOE_GROUP || L->d_ff % MOE_GROUP)
        return fail(MOE_ESHAPE, "d_model=%d and d_ff=%d must be positive multiples of %d", L->d_model, L->d_ff, MOE_GROUP);
    if (L->d_model > 8192 || L->d_ff > 16384)
        return fail(MOE_ESHAPE, "d_model=%d > 8192 or d_ff=%d > 16384 not supported", L->d_model, L->d_ff);
    if (L->n_experts < 1 || L->n_experts > MOE_MAX_EXPERTS)
        return fail(MOE_ESHAPE, "n_experts=%d outside [1, %d]", L->n_experts, MOE_MAX_EXPERTS);
    if (L->top_k < 1 || L->top_k > L->n_experts || L->top_k > MOE_MAX_TOPK)
        return fail(MOE_ESHAPE, "top_k=%d outside [1, min(n_experts, %d)]", L->top_k, MOE_MAX_TOPK);
    for (int e = 0; e < L->n_experts; ++e) {
        const moe_expert& x = L->experts[e];
        if (x.prec != MOE_PREC_FP16 && x.prec != MOE_PREC_INT4G64 && x.prec != MOE_PREC_INT8G64)
            return fail(MOE_EINVAL, "expert %d: unknown precision %d", e, x.prec);
        if (x.resident && x.prec != MOE_PREC_FP16 &&
            (!x.w1.scale || !x.w1.zero || !x.w3.scale || !x.w3.zero || !x.w2.scale || !x.w2.zero))
            return fail(MOE_EINVAL, "expert %d: quantized matrices need scale and zero", e);
        if (x.resident) {   // the kernels read weights, scales and zeros with 128-bit loads
            const moe_mat* mats[3] = {&x.w1, &x.w3, &x.w2};
            for (const moe_mat* m : mats)
                if (((uintptr_t)m->data | (uintptr_t)m->scale | (uintptr_t)m->zero) & 15)
                    return fail(MOE_EINVAL, "expert %d: data, scale and zero must be 16-byte aligned", e);
        }
    }
    return MOE_OK;
}

// Workgroups of the batch-1 up-projection: four per compute unit, each wavefront taking an equal share of the
// routed experts' stored bytes.
constexpr int kDecodeUpBlocks = 1024;

// Which kernels serve T tokens of a block: T == 1 the batch-1 kernels, otherwise the matrix-core path when
// the shape allows it, else the shape-agnostic kernels.
bool use_decode(const moe_layer* L, int T) { return T == 1 && decode_shape_ok(L->d_model, L->d_ff); }
bool use_mfma(const moe_layer* L, int rows) {
    return rows > 1 && mfma_shape_ok(L->d_model, L->d_ff) && mfma_rows_ok(rows, L->d_model, L->d_ff);
}

MfmaPlan plan_for(const moe_layer* L, int rows) { return plan_mfma(rows, L->d_model, L->d_ff, L->n_experts); }

int y_splits_for(const moe_layer* L, int T) {
    if (!use_mfma(L, T * L->top_k)) return 1;
    return plan_for(L, T * L->top_k).down_splits;
}

bool expert_resident(const moe_expert& x) { return x.resident && x.w1.data && x.w3.data && x.w2.data; }

DevExperts device_table(const moe_layer* L) {
    DevExperts t;
    memset(&t, 0, sizeof(t));
    for (int e = 0; e < L->n_experts; ++e) {
        const moe_expert& x = L->experts[e];
        DevExpert& y = t.e[e];
        y.prec = x.prec;
        y.resident = expert_resident(x) ? 1 : 0;
        auto cp = [](const moe_mat& m) { return DevMat{(const uint8_t*)m.data, (const half_t*)m.scale, (const half_t*)m.zero}; };
        y.w1 = cp(x.w1);
        y.w3 = cp(x.w3);
        y.w2 = cp(x.w2);
    }
    return t;
}

int check_ws(const moe_layer* L, int T, void* ws, size_t ws_bytes, Workspace* out) {
    if (!ws) return fail(MOE_EWORKSPACE, "workspace is NULL");
    if ((uintptr_t)ws % 256) return fail(MOE_EWORKSPACE, "workspace must be 256-byte aligned");
    *out = carve_workspace(ws, T, L->d_model, L->d_ff, L->n_experts, L->top_k, y_splits_for(L, T));
    if (ws_bytes < out->bytes)
        return fail(MOE_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, out->bytes);
    return MOE_OK;
}

// (RMSNorm +) gating -> grouping -> experts -> weighted average (+ residual), all on `st`.
// rms_gain != null: the block input is RMSNorm(x) * rms_gain, computed by the gating kernel into ws.xn.
int layer_body(const moe_layer* L, const DevExperts& table, const half_t* x, int T, const half_t* rms_gain, float eps,
               const half_t* residual, half_t* out, int32_t* idx_out, float* gate_out, const Workspace& w,
               bool reset_status, hipStream_t st) {
    const int d = L->d_model, f = L->d_ff, E = L->n_experts, k = L->top_k;
    if (use_decode(L, T)) {
        // batch-1 decode: two launches.  The gating network (and the RMSNorm of the chain) runs inside the
        // up-projection launch, no grouping is needed, the weighted average is fused into the down-projection.
        // The up-projection launch clears the word it is given: the status word for the first block of a call, a
        // spare word of the status region for later blocks of a chain, which must keep what earlier blocks raised.
        const GateArgs ga{(const half_t*)L->w_gate, L->gate_bias, E, rms_gain, eps, w.idx, w.gate, idx_out, gate_out};
        launch_decode_up(table, nullptr, x, d, f, k, w.h, reset_status ? w.status : w.status + 1, kDecodeUpBlocks, st, &ga);
        launch_decode_down(table, w.idx, w.gate, w.h, d, f, k, residual, out, w.status, st);
        return check_hip(st);
    }
    launch_route(x, (const half_t*)L->w_gate, L->gate_bias, T, d, E, k, w.idx, w.gate, idx_out, gate_out,
                 reset_status ? w.status : nullptr, st, rms_gain, eps, w.xn);
    if (rms_gain) x = w.xn;
    launch_permute(w.idx, T * k, E, w.counts, w.offsets, w.perm, w.inv, w.status, st);
    RowMap rows{w.offsets, w.perm, k, -1, 0};
    const size_t split_stride = (size_t)T * k * d;
    if (use_mfma(L, T * k)) {
        const MfmaPlan p = plan_for(L, T * k);
        launch_ffn_up_mfma(table, E, rows, T * k, x, d, f, w.h, p.ct, w.status, st);
        launch_ffn_down_mfma(table, E, rows, T * k, w.h, d, f, w.y, p.ct, p.down_splits, split_stride, w.status, st);
        launch_combine(w.y, p.down_splits, split_stride, w.gate, w.inv, T, d, k, residual, out, st);
    } else {
        launch_ffn_up(table, E, rows, x, d, f, w.h, w.status, st);
        launch_ffn_down(table, E, rows, w.h, d, f, w.y, w.status, st);
        launch_combine(w.y, 1, split_stride, w.gate, w.inv, T, d, k, residual, out, st);
    }
    return check_hip(st);
}

}  // namespace

namespace moemix {

namespace {
struct Trace {
    bool armed = false;
    hipEvent_t start = nullptr, stop = nullptr;
};
thread_local Trace g_trace[kKernelCount];   // one slot per kernel id: several kernels of one call can be armed
}  // namespace

void trace_arm(int kernel, hipEvent_t start, hipEvent_t stop) { g_trace[kernel] = Trace{true, start, stop}; }
void trace_disarm(int kernel) { g_trace[kernel] = Trace{}; }

TraceScope::TraceScope(int kernel_, hipStream_t st_) : kernel(kernel_), st(st_) {
    if (g_trace[kernel].armed) (void)hipEventRecord(g_trace[kernel].start, st);
}

TraceScope::~TraceScope() {
    if (g_trace[kernel].armed) {
        (void)hipEventRecord(g_trace[kernel].stop, st);
        g_trace[kernel].armed = false;
    }
}

}  // namespace moemix

extern "C" {

int moe_trace_kernel(int kernel, void* start_event, void* stop_event) {
    if (kernel < 0 || kernel >= kKernelCount) return fail(MOE_EINVAL, "moe_trace_kernel: bad kernel id %d", kernel);
    if (!start_event && !stop_event) {
        trace_disarm(kernel);
        return MOE_OK;
    }
    if (!start_event || !stop_event) return fail(MOE_EINVAL, "moe_trace_kernel: one event is NULL");
    trace_arm(kernel, (hipEvent_t)start_event, (hipEvent_t)stop_event);
    return MOE_OK;
}

size_t moe_workspace_bytes(const moe_layer* layer, int n_tokens) {
    if (!layer || n_tokens < 1 || layer->d_model < 1 || layer->d_ff < 1 || layer->n_experts < 1 || layer->top_k < 1)
        return 0;
    return carve_workspace(nullptr, n_tokens, layer->d_model, layer->d_ff, layer->n_experts, layer->top_k, y_splits_for(layer, n_tokens)).bytes;
}

int moe_route(const moe_layer* layer, const void* x, int T, int32_t* topk_idx, float* topk_gate, moe_stream_t stream) {
    if (int rc = check_layer(layer)) return rc;
    if (!x || !topk_idx || !topk_gate) return fail(MOE_EINVAL, "moe_route: NULL argument");
    if (T < 1) return fail(MOE_ESHAPE, "moe_route: T=%d < 1", T);
    launch_route((const half_t*)x, (const half_t*)layer->w_gate, layer->gate_bias, T, layer->d_model, layer->n_experts,
                 layer->top_k, topk_idx, topk_gate, nullptr, nullptr, nullptr, (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_permute(const moe_layer* layer, const int32_t* topk_idx, int T, int32_t* counts, int32_t* offsets,
                int32_t* perm, void* ws, size_t ws_bytes, moe_stream_t stream) {
    if (int rc = check_layer(layer)) return rc;
    if (!topk_idx || !counts || !offsets || !perm) return fail(MOE_EINVAL, "moe_permute: NULL argument");
    if (T < 1) return fail(MOE_ESHAPE, "moe_permute: T=%d < 1", T);
    Workspace w;
    if (int rc = check_ws(layer, T, ws, ws_bytes, &w)) return rc;
    hipStream_t st = (hipStream_t)stream;
    launch_zero_words(w.status, 1, st);   // the status word describes this call
    launch_permute(topk_idx, T * layer->top_k, layer->n_experts, counts, offsets, perm, w.inv, w.status, st);
    return check_hip(st);
}

int moe_expert_ffn_mixed(const moe_layer* layer, int expert, const void* x_rows, int n, float* y, void* ws,
                         size_t ws_bytes, moe_stream_t stream) {
    if (int rc = check_layer(layer)) return rc;
    if (!x_rows || !y) return fail(MOE_EINVAL, "moe_expert_ffn_mixed: NULL argument");
    if (expert < 0 || expert >= layer->n_experts) return fail(MOE_EINVAL, "expert %d outside [0, %d)", expert, layer->n_experts);
    if (n < 1) return fail(MOE_ESHAPE, "moe_expert_ffn_mixed: n=%d < 1", n);
    if (!expert_resident(layer->experts[expert])) return fail(MOE_ENOTRESIDENT, "expert %d is not resident", expert);
    // the hidden rows need n*d_ff halves: a workspace sized for ceil(n / top_k) tokens holds them
    const int T_equiv = (n + layer->top_k - 1) / layer->top_k;
    Workspace w;
    if (int rc = check_ws(layer, T_equiv, ws, ws_bytes, &w)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const DevExperts table = device_table(layer);
    RowMap rows{nullptr, nullptr, layer->top_k, expert, n};
    const int d = layer->d_model, f = layer->d_ff;
    launch_zero_words(w.status, 1, st);   // the status word describes this call
    if (use_decode(layer, n)) {
        // one row: the batch-1 kernels, with the routing result "this expert, weight 1" written to the workspace
        launch_single_route(w.idx, w.gate, expert, st);
        launch_decode_up(table, w.idx, (const half_t*)x_rows, d, f, 1, w.h, w.status, kDecodeUpBlocks, st);
        launch_decode_down(table, w.idx, w.gate, w.h, d, f, 1, nullptr, nullptr, w.status, st, y);
    } else if (use_mfma(layer, n)) {
        MfmaPlan p = plan_mfma(n, d, f, 1);       // all n rows belong to the one expert
        launch_ffn_up_mfma(table, layer->n_experts, rows, n, (const half_t*)x_rows, d, f, w.h, p.ct, w.status, st);
        // few rows: the contraction of the down-projection is split over as many workgroups as the workspace's
        // partial-result region was sized for, and the partials are added in order
        const int splits = p.down_splits < w.y_splits ? p.down_splits : w.y_splits;
        if (splits > 1) {
            const size_t stride = (size_t)n * d;
            launch_ffn_down_mfma(table, layer->n_experts, rows, n, w.h, d, f, w.y, p.ct, splits, stride, w.status, st);
            launch_reduce_splits(w.y, splits, stride, stride, y, st);
        } else {
            launch_ffn_down_mfma(table, layer->n_experts, rows, n, w.h, d, f, y, p.ct, 1, 0, w.status, st);
        }
    } else {
        launch_ffn_up(table, layer->n_experts, rows, (const half_t*)x_rows, d, f, w.h, w.status, st);
        launch_ffn_down(table, layer->n_experts, rows, w.h, d, f, y, w.status, st);
    }
    return check_hip(st);
}

int moe_layer_forward(const moe_layer* layer, const void* x, int T, void* out, int32_t* topk_idx_out,
                      float* topk_gate_out, void* ws, size_t ws_bytes, moe_stream_t stream) {
    if (int rc = check_layer(layer)) return rc;
    if (!x || !out) return fail(MOE_EINVAL, "moe_layer_forward: NULL argument");
    if (T < 1) return fail(MOE_ESHAPE, "moe_layer_forward: T=%d < 1", T);
    Workspace w;
    if (int rc = check_ws(layer, T, ws, ws_bytes, &w)) return rc;
    const DevExperts table = device_table(layer);
    return layer_body(layer, table, (const half_t*)x, T, nullptr, 0.0f, nullptr, (half_t*)out, topk_idx_out, topk_gate_out, w, true,
                      (hipStream_t)stream);
}

// ---------------------------------------------------------------- the block without a caller workspace

namespace {

// Scratch of moe_layer_forward_static: one array per GPU, held until the process ends.
constexpr size_t kStaticScratchBytes = MOE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on each GPU (the array's name is only a host-side handle).  Looked up once per
// device, with that device current; 0 = not looked up yet.
constexpr int kMaxDevices = 64;
std::atomic<uintptr_t> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(MOE_EHIP, "device %d outside [0, %d)", dev, kMaxDevices);
    uintptr_t p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void* sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !sym)
            return fail(MOE_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        p = (uintptr_t)sym;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread finds the same address
    }
    *out = (void*)p;
    return MOE_OK;
}

}  // namespace

size_t moe_static_scratch_bytes(void) { return kStaticScratchBytes; }

int moe_layer_forward_static(const moe_layer* layer, const void* x, int T, void* out, int32_t* topk_idx_out,
                             float* topk_gate_out, moe_stream_t stream) {
    if (int rc = check_layer(layer)) return rc;
    if (!x || !out) return fail(MOE_EINVAL, "moe_layer_forward_static: NULL argument");
    if (T < 1) return fail(MOE_ESHAPE, "moe_layer_forward_static: T=%d < 1", T);
    const size_t need = moe_workspace_bytes(layer, T);
    if (need == 0 || need > kStaticScratchBytes)
        return fail(MOE_EWORKSPACE, "moe_layer_forward_static: %d tokens of this layer need %zu bytes of scratch, the "
                    "library holds %zu; use moe_layer_forward with a workspace", T, need, kStaticScratchBytes);
    void* ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    Workspace w;
    if (int rc = check_ws(layer, T, ws, kStaticScratchBytes, &w)) return rc;
    const DevExperts table = device_table(layer);
    // the scratch keeps the last call's contents: the status word is cleared by the gating kernel, every other
    // region is written before it is read
    return layer_body(layer, table, (const half_t*)x, T, nullptr, 0.0f, nullptr, (half_t*)out, topk_idx_out, topk_gate_out, w,
                      true, (hipStream_t)stream);
}

// ---------------------------------------------------------------- expert-miss path

namespace {

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// Bytes of one matrix [out, in] in the given precision: codes or halves, then scales, then zeros, each piece
// starting on a 256-byte boundary inside a swap slot.
struct MatBytes {
    size_t data, scale, zero;
    size_t total() const { return align256(data) + align256(scale) + align256(zero); }
};
MatBytes mat_bytes(int prec, int out, int in) {
    if (prec == MOE_PREC_INT4G64 || prec == MOE_PREC_INT8G64) {
        const size_t g = (size_t)out * (in / MOE_GROUP) * 2;
        return MatBytes{prec == MOE_PREC_INT4G64 ? (size_t)out * in / 2 : (size_t)out * in, g, g};
    }
    return MatBytes{(size_t)out * in * 2, 0, 0};
}

// Enqueues the host-to-device copies of one matrix into a slot and returns where the pieces landed.
hipError_t copy_mat(const moe_mat& src, const MatBytes& b, char*& cursor, DevMat* dst, hipStream_t st) {
    hipError_t e = hipMemcpyAsync(cursor, src.data, b.data, hipMemcpyHostToDevice, st);
    dst->data = (const uint8_t*)cursor;
    cursor += align256(b.data);
    dst->scale = dst->zero = nullptr;
    if (b.scale && e == hipSuccess) {
        e = hipMemcpyAsync(cursor, src.scale, b.scale, hipMemcpyHostToDevice, st);
        dst->scale = (const half_t*)cursor;
        cursor += align256(b.scale);
        if (e == hipSuccess) e = hipMemcpyAsync(cursor, src.zero, b.zero, hipMemcpyHostToDevice, st);
        dst->zero = (const half_t*)cursor;
        cursor += align256(b.zero);
    }
    return e;
}

// Up- and down-projection of every expert the table marks runnable (deferred ones are skipped silently).
void run_experts(const moe_layer* L, const DevExperts& table, const half_t* x, int T, const Workspace& w,
                 const half_t* decode_residual, half_t* out, hipStream_t st) {
    const int d = L->d_model, f = L->d_ff, E = L->n_experts, k = L->top_k;
    if (use_decode(L, T)) {
        launch_decode_up(table, w.idx, x, d, f, k, w.h, w.status, kDecodeUpBlocks, st);
        launch_decode_down(table, w.idx, w.gate, w.h, d, f, k, decode_residual, out, w.status, st);
        return;
    }
    RowMap rows{w.offsets, w.perm, k, -1, 0};
    const size_t split_stride = (size_t)T * k * d;
    if (use_mfma(L, T * k)) {
        const MfmaPlan p = plan_for(L, T * k);
        launch_ffn_up_mfma(table, E, rows, T * k, x, d, f, w.h, p.ct, w.status, st);
        launch_ffn_down_mfma(table, E, rows, T * k, w.h, d, f, w.y, p.ct, p.down_splits, split_stride, w.status, st);
    } else {
        launch_ffn_up(table, E, rows, x, d, f, w.h, w.status, st);
        launch_ffn_down(table, E, rows, w.h, d, f, w.y, w.status, st);
    }
}

}  // namespace

size_t moe_swap_slot_bytes(const moe_layer* layer) {
    if (!layer || layer->d_model < 1 || layer->d_ff < 1 || !layer->experts) return 0;
    size_t worst = 0;
    for (int e = 0; e < layer->n_experts; ++e) {
        const int prec = layer->experts[e].prec;
        const size_t b = 2 * mat_bytes(prec, layer->d_ff, layer->d_model).total() +
                         mat_bytes(prec, layer->d_model, layer->d_ff).total();
        worst = b > worst ? b : worst;
    }
    return worst;
}

int moe_layer_forward_swap(const moe_layer* layer, const moe_swap* swap, const void* x, int T, void* out,
                           int32_t* topk_idx_out, float* topk_gate_out, void* ws, size_t ws_bytes, moe_stream_t stream,
                           int32_t* n_missed) {
    if (int rc = check_layer(layer)) return rc;
    if (!swap || !x || !out) return fail(MOE_EINVAL, "moe_layer_forward_swap: NULL argument");
    if (!swap->host_experts || !swap->swap || !swap->host_idx || !swap->copied_event || !swap->computed_event)
        return fail(MOE_EINVAL, "moe_layer_forward_swap: incomplete swap descriptor");
    if (T < 1) return fail(MOE_ESHAPE, "moe_layer_forward_swap: T=%d < 1", T);
    if (swap->n_slots < 1 || swap->slot_bytes < moe_swap_slot_bytes(layer) || (uintptr_t)swap->swap % 256 ||
        swap->slot_bytes % 256)
        return fail(MOE_EWORKSPACE, "swap space: %d slots of %zu bytes, %zu bytes per slot needed (256-byte aligned)",
                    swap->n_slots, swap->slot_bytes, moe_swap_slot_bytes(layer));
    Workspace w;
    if (int rc = check_ws(layer, T, ws, ws_bytes, &w)) return rc;
    hipStream_t st = (hipStream_t)stream, cst = (hipStream_t)swap->copy_stream;
    const int d = layer->d_model, f = layer->d_ff, E = layer->n_experts, k = layer->top_k;
    const half_t* xin = (const half_t*)x;

    // gating, then the one host round trip of this path: which experts were chosen?
    launch_route(xin, (const half_t*)layer->w_gate, layer->gate_bias, T, d, E, k, w.idx, w.gate, topk_idx_out, topk_gate_out,
                 w.status, st);
    hipError_t e = hipMemcpyAsync(swap->host_idx, w.idx, (size_t)T * k * sizeof(int32_t), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
    int missed[MOE_MAX_EXPERTS], n_miss = 0;
    uint32_t seen = 0;
    for (int i = 0; i < T * k; ++i) {
        const int32_t ex = swap->host_idx[i];
        if (ex < 0 || ex >= E || (seen & (1u << ex))) continue;
        seen |= 1u << ex;
        const moe_expert& he = swap->host_experts[ex];
        if (expert_resident(layer->experts[ex]) || !he.w1.data || !he.w3.data || !he.w2.data) continue;
        if (layer->experts[ex].prec != MOE_PREC_FP16 &&
            (!he.w1.scale || !he.w1.zero || !he.w3.scale || !he.w3.zero || !he.w2.scale || !he.w2.zero))
            return fail(MOE_EINVAL, "host expert %d: quantized matrices need scale and zero", ex);
        missed[n_miss++] = ex;
    }
    if (n_missed) *n_missed = n_miss;

    // pass over the resident experts; the missed ones wait for their copies
    DevExperts table = device_table(layer);
    for (int i = 0; i < n_miss; ++i) table.e[missed[i]].resident = kDeferred;
    const bool decode = use_decode(layer, T);
    if (!decode) launch_permute(w.idx, T * k, E, w.counts, w.offsets, w.perm, w.inv, w.status, st);
    run_experts(layer, table, xin, T, w, nullptr, (half_t*)out, st);

    // rounds of at most n_slots copies, each followed by a pass over the experts it brought in
    for (int first = 0; first < n_miss; first += swap->n_slots) {
        const int n_round = n_miss - first < swap->n_slots ? n_miss - first : swap->n_slots;
        DevExperts round = device_table(layer);
        for (int i = 0; i < E; ++i) round.e[i].resident = kDeferred;
        if (first > 0) {      // the slots are reused: the pass that read them must have finished
            e = hipStreamWaitEvent(cst, (hipEvent_t)swap->computed_event, 0);
            if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
        }
        for (int i = 0; i < n_round; ++i) {
            const int ex = missed[first + i];
            const moe_expert& he = swap->host_experts[ex];
            const int prec = layer->experts[ex].prec;
            char* cursor = (char*)swap->swap + (size_t)i * swap->slot_bytes;
            DevExpert& de = round.e[ex];
            de.prec = prec;
            e = copy_mat(he.w1, mat_bytes(prec, f, d), cursor, &de.w1, cst);
            if (e == hipSuccess) e = copy_mat(he.w3, mat_bytes(prec, f, d), cursor, &de.w3, cst);
            if (e == hipSuccess) e = copy_mat(he.w2, mat_bytes(prec, d, f), cursor, &de.w2, cst);
            if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
            de.resident = 1;
        }
        e = hipEventRecord((hipEvent_t)swap->copied_event, cst);
        if (e == hipSuccess) e = hipStreamWaitEvent(st, (hipEvent_t)swap->copied_event, 0);
        if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
        // at one token the weighted average is fused into the down-projection: this pass adds to the last one's output
        run_experts(layer, round, xin, T, w, (const half_t*)out, (half_t*)out, st);
        e = hipEventRecord((hipEvent_t)swap->computed_event, st);
        if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
    }
    if (!decode) {
        const int splits = use_mfma(layer, T * k) ? plan_for(layer, T * k).down_splits : 1;
        launch_combine(w.y, splits, (size_t)T * k * d, w.gate, w.inv, T, d, k, nullptr, (half_t*)out, st);
    }
    return check_hip(st);
}

int moe_chain_forward(const moe_layer* layers, const void* const* rms_gain, int n_layers, float eps, void* h, int T,
                      int32_t* topk_idx_out, void* ws, size_t ws_bytes, moe_stream_t stream) {
    if (!layers || !rms_gain || !h) return fail(MOE_EINVAL, "moe_chain_forward: NULL argument");
    if (n_layers < 1 || T < 1) return fail(MOE_ESHAPE, "moe_chain_forward: n_layers=%d, T=%d", n_layers, T);
    for (int l = 0; l < n_layers; ++l) {
        if (int rc = check_layer(&layers[l])) return rc;
        if (!rms_gain[l]) return fail(MOE_EINVAL, "rms_gain[%d] is NULL", l);
        if (layers[l].d_model != layers[0].d_model || layers[l].d_ff != layers[0].d_ff ||
            layers[l].n_experts != layers[0].n_experts || layers[l].top_k != layers[0].top_k)
            return fail(MOE_ESHAPE, "layer %d differs in shape from layer 0", l);
    }
    Workspace w;
    if (int rc = check_ws(&layers[0], T, ws, ws_bytes, &w)) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int k = layers[0].top_k;
    for (int l = 0; l < n_layers; ++l) {
        const DevExperts table = device_table(&layers[l]);
        int32_t* idx_out = topk_idx_out ? topk_idx_out + (size_t)l * T * k : nullptr;
        if (int rc = layer_body(&layers[l], table, (const half_t*)h, T, (const half_t*)rms_gain[l], eps, (const half_t*)h,
                                (half_t*)h, idx_out, nullptr, w, l == 0, st))
            return rc;
    }
    return MOE_OK;
}

int moe_dequant_int4(const moe_mat* m, int out, int in, void* w_fp16, moe_stream_t stream) {
    if (!m || !m->data || !m->scale || !m->zero || !w_fp16) return fail(MOE_EINVAL, "moe_dequant_int4: NULL argument");
    if (out < 0 || in < 0) return fail(MOE_EINVAL, "moe_dequant_int4: negative size");
    if (in % MOE_GROUP) return fail(MOE_ESHAPE, "moe_dequant_int4: in=%d not a multiple of %d", in, MOE_GROUP);
    launch_dequant_int4(DevMat{(const uint8_t*)m->data, (const half_t*)m->scale, (const half_t*)m->zero}, out, in,
                        (half_t*)w_fp16, (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_quantize_int4(const void* w_fp16, int out, int in, void* packed, void* scale, void* zero, moe_stream_t stream) {
    if (!w_fp16 || !packed || !scale || !zero) return fail(MOE_EINVAL, "moe_quantize_int4: NULL argument");
    if (out < 0 || in < 0) return fail(MOE_EINVAL, "moe_quantize_int4: negative size");
    if (in % MOE_GROUP) return fail(MOE_ESHAPE, "moe_quantize_int4: in=%d not a multiple of %d", in, MOE_GROUP);
    launch_quantize_int4((const half_t*)w_fp16, out, in, (uint8_t*)packed, (half_t*)scale, (half_t*)zero,
                         (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_dequant_int8(const moe_mat* m, int out, int in, void* w_fp16, moe_stream_t stream) {
    if (!m || !m->data || !m->scale || !m->zero || !w_fp16) return fail(MOE_EINVAL, "moe_dequant_int8: NULL argument");
    if (out < 0 || in < 0) return fail(MOE_EINVAL, "moe_dequant_int8: negative size");
    if (in % MOE_GROUP) return fail(MOE_ESHAPE, "moe_dequant_int8: in=%d not a multiple of %d", in, MOE_GROUP);
    launch_dequant_int8(DevMat{(const uint8_t*)m->data, (const half_t*)m->scale, (const half_t*)m->zero}, out, in,
                        (half_t*)w_fp16, (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_quantize_int8(const void* w_fp16, int out, int in, void* codes, void* scale, void* zero, moe_stream_t stream) {
    if (!w_fp16 || !codes || !scale || !zero) return fail(MOE_EINVAL, "moe_quantize_int8: NULL argument");
    if (out < 0 || in < 0) return fail(MOE_EINVAL, "moe_quantize_int8: negative size");
    if (in % MOE_GROUP) return fail(MOE_ESHAPE, "moe_quantize_int8: in=%d not a multiple of %d", in, MOE_GROUP);
    launch_quantize_int8((const half_t*)w_fp16, out, in, (uint8_t*)codes, (half_t*)scale, (half_t*)zero,
                         (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_synth_fill_f16(void* dst, size_t n, size_t first, uint64_t seed, uint64_t stream_id, float scale, int kind,
                       moe_stream_t stream) {
    if (!dst && n) return fail(MOE_EINVAL, "moe_synth_fill_f16: NULL destination");
    if (kind != 0 && kind != 1) return fail(MOE_EINVAL, "moe_synth_fill_f16: kind=%d", kind);
    launch_synth_fill((half_t*)dst, n, first, seed, stream_id, scale, kind, (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_stream_read(const void* src, size_t bytes, void* sink, moe_stream_t stream) {
    if (!src || !sink) return fail(MOE_EINVAL, "moe_stream_read: NULL argument");
    if (bytes % 16 || (uintptr_t)src % 16) return fail(MOE_EINVAL, "moe_stream_read: bytes and src must be multiples of 16");
    if (bytes) launch_stream_read(src, bytes, (uint32_t*)sink, 512, (hipStream_t)stream);
    return check_hip((hipStream_t)stream);
}

int moe_read_status(void* ws, moe_stream_t stream, int* status_bits) {
    if (!status_bits) return fail(MOE_EINVAL, "moe_read_status: NULL argument");
    if (!ws) {      // the library's own scratch on the current device (moe_layer_forward_static)
        if (int rc = static_scratch(&ws)) return rc;
    }
    int32_t v = 0;
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess) e = hipMemcpy(&v, ws, sizeof(v), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(MOE_EHIP, "HIP: %s", hipGetErrorString(e));
    *status_bits = v;
    return MOE_OK;
}

const char* moe_last_error(void) { return g_err; }

int moe_version(void) { return 1000; }

}  // extern "C"
