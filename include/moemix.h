/*
 * moemix -- one Mixture-of-Experts feed-forward block in which every expert is
 * held either in 16-bit or in 4-bit form, for AMD MI355X (gfx950).
 *
 * Method: "Mixture of Experts with Mixture of Precisions for Tuning Quality of
 * Service" (arXiv 2407.14417).  The paper serves an MoE model whose experts are
 * partially quantized (§3): an expert table carries two attributes per expert,
 * "quantized?" and "on the GPU?"; the number of 4-bit experts is the knob that
 * trades quality for memory/throughput.  This library is the compute under that
 * policy: the gating network with top-k selection (§1, §2.1), the experts as
 * parallel feed-forward layers of Mixtral shape (§1, §4.1), each evaluated in
 * the precision its table entry names, and the weighted average of the selected
 * experts' outputs (§1).  The policy itself (how many experts to quantize,
 * which to keep resident) stays with the caller and reaches the library as the
 * per-expert `prec` and `resident` fields.
 *
 * Conventions
 *   - Every pointer argument documented "device" is GPU memory owned by the
 *     caller; "host" is ordinary host memory.  The library never frees or keeps
 *     a caller's pointer beyond the call, and allocates nothing.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as
 *     void*) and returns; nothing synchronizes except moe_read_status.
 *     All launches are capturable into a HIP graph.
 *   - Return value: MOE_OK or a negative moe_status.  No call throws or exits.
 *     moe_last_error() gives a host string for the last failure on this thread.
 *   - Matrices are row-major [out, in]; `in` is the contraction dimension.
 *   - 16-bit means IEEE fp16.  4-bit means: asymmetric uint4, groups of 64
 *     consecutive columns of one row share an fp16 scale and an fp16 zero,
 *     two codes per byte, the even column in the low nibble;
 *     dequantized weight = fp16_rne( fp32(code) * fp32(scale) + fp32(zero) ).
 *     moe_dequant_int4 and the kernels for shapes outside the tiled paths produce exactly these bits.  The
 *     tiled matrix kernels evaluate the same expression inside their products without materialising the
 *     weight: the multi-token kernels with one fp16 multiply-add (a single rounding), the one-token kernels
 *     in the factored form scale * sum(code * x) + zero * sum(x) in fp32 (no rounding of the weight); both
 *     stay within the tolerance stated for the block outputs, not bit-exact per weight.
 *   - 8-bit (the precision of the paper's homogeneous 8-bit comparison model, §4 Table 1) follows the same scheme:
 *     asymmetric uint8, groups of 64 columns with an fp16 scale and an fp16 zero, one code per byte;
 *     dequantized weight = fp16_rne( fp32(code) * fp32(scale) + fp32(zero) ).
 *   - d_model and d_ff must be multiples of 64, d_model <= 8192, d_ff <= 16384 (else MOE_ESHAPE);
 *     n_experts <= MOE_MAX_EXPERTS; 1 <= top_k <= min(n_experts, MOE_MAX_TOPK).
 */
#ifndef MOEMIX_H
#define MOEMIX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_GROUP 64
#define MOE_MAX_EXPERTS 32
#define MOE_MAX_TOPK 8
#define MOE_STATIC_SCRATCH_BYTES (8u << 20) /* scratch held by the library for moe_layer_forward_static */

typedef enum {
    MOE_OK = 0,
    MOE_EINVAL = -1,       /* null pointer, negative size */
    MOE_ESHAPE = -2,       /* shape outside what the kernels support (see above) */
    MOE_ENOTRESIDENT = -3, /* an expert that had to run is not in device memory */
    MOE_EWORKSPACE = -4,   /* workspace missing or smaller than moe_workspace_bytes */
    MOE_EHIP = -5          /* a HIP runtime call failed */
} moe_status;

/* The "quantized?" attribute of the paper's expert table (§3). */
typedef enum { MOE_PREC_FP16 = 0, MOE_PREC_INT4G64 = 1, MOE_PREC_INT8G64 = 2 } moe_prec;

/* One weight matrix [out, in] in device memory, rows end to end; every pointer 16-byte aligned (MOE_EINVAL otherwise). */
typedef struct {
    const void* data;  /* device: fp16 [out,in]; uint8 [out,in/2] of packed 4-bit codes; or uint8 [out,in] of 8-bit codes */
    const void* scale; /* device: fp16 [out,in/64]; NULL for a 16-bit matrix */
    const void* zero;  /* device: fp16 [out,in/64]; NULL for a 16-bit matrix */
} moe_mat;

/* One expert = SwiGLU feed-forward layer y = W2 ( silu(W1 x) * (W3 x) ).
 * w1, w3: [d_ff, d_model]; w2: [d_model, d_ff]; all three in precision `prec`. */
typedef struct {
    int32_t prec;     /* moe_prec */
    int32_t resident; /* location attribute of the expert table (§3): 1 = matrices are in device memory */
    moe_mat w1, w3, w2;
} moe_expert;

/* One MoE block.  `experts` is a HOST array of n_experts descriptors holding device pointers. */
typedef struct {
    int32_t d_model, d_ff, n_experts, top_k;
    const void* w_gate;        /* device: fp16 [n_experts, d_model], always 16-bit (§3: non-expert parts stay 16-bit) */
    const float* gate_bias;    /* device: fp32 [n_experts] added to the router logits, or NULL */
    const moe_expert* experts; /* host */
} moe_layer;

typedef void* moe_stream_t; /* hipStream_t; NULL = the default stream */

/* Bytes of scratch that the calls below need for `n_tokens` tokens of `layer`.  Host-only arithmetic.
 * The caller allocates that many bytes of device memory (256-byte aligned) and passes them as `ws`;
 * one workspace must not be used by two calls that may overlap in time.  Returns 0 on bad arguments. */
size_t moe_workspace_bytes(const moe_layer* layer, int n_tokens);

/*
 * Gating network (§1) with top-k selection (§2.1), one fused kernel.
 *   logit[t,e] = sum_j x[t,j] * w_gate[e,j] (+ gate_bias[e])       fp32 accumulation
 *   topk_idx[t,:]  = the top_k experts by logit, descending; equal logits: lower index first
 *   topk_gate[t,:] = softmax over those top_k logits (weights of the weighted average, sum to 1)
 * x: device fp16 [T, d_model]; topk_idx: device int32 [T, top_k]; topk_gate: device fp32 [T, top_k].
 */
int moe_route(const moe_layer* layer, const void* x, int T, int32_t* topk_idx, float* topk_gate,
              moe_stream_t stream);

/*
 * Grouping of the T*top_k (token, slot) pairs by expert (the scatter of tokens to experts that
 * top-k gating implies, §2.1).  Flat pair index p = t*top_k + s.
 *   counts[e]  = pairs routed to expert e;  offsets = exclusive prefix sum, offsets[E] = T*top_k
 *   perm[r]    = flat pair index held by grouped row r; one expert's rows are contiguous and keep
 *                increasing pair index (the result is unique).
 * topk_idx: device int32 [T, top_k]; counts: device int32 [E]; offsets: device int32 [E+1];
 * perm: device int32 [T*top_k].  An index outside [0, E) sets the MOE_EINVAL bit readable with
 * moe_read_status on `ws` and its pair is dropped.
 */
int moe_permute(const moe_layer* layer, const int32_t* topk_idx, int T, int32_t* counts, int32_t* offsets,
                int32_t* perm, void* ws, size_t ws_bytes, moe_stream_t stream);

/*
 * One expert's feed-forward layer on n rows (§1: experts are parallel FF layers), in the precision
 * its descriptor names (§3), 4-bit weights being dequantized inside the matrix kernels:
 *   y[i,:] = W2 ( silu(W1 x_i) * (W3 x_i) )                        fp32 accumulation
 * x_rows: device fp16 [n, d_model]; y: device fp32 [n, d_model] (overwritten).
 * ws: at least moe_workspace_bytes(layer, ceil(n / top_k)) bytes (the hidden rows live there).
 * Fails with MOE_ENOTRESIDENT on the host if the expert is not resident.
 * n == 1 runs the same one-token kernels as moe_layer_forward with T == 1 (when the shape is one they
 * take), n > 1 the multi-token kernels, so each can be checked alone, before gating and weighted average.
 */
int moe_expert_ffn_mixed(const moe_layer* layer, int expert, const void* x_rows, int n, float* y, void* ws,
                         size_t ws_bytes, moe_stream_t stream);

/*
 * The whole block on T tokens: gating, top-k, grouping, every selected expert in its own precision,
 * weighted average (§1, §2.1, §3):
 *   out[t,:] = fp16_rne( sum_s topk_gate[t,s] * FFN_{topk_idx[t,s]}(x[t,:]) )
 * x: device fp16 [T, d_model]; out: device fp16 [T, d_model];
 * topk_idx_out / topk_gate_out: device [T, top_k], nullable.
 * Routing happens on the device, so a routed expert that is not resident cannot fail the call on the
 * host: its contribution is left out and the MOE_ENOTRESIDENT bit is set in the workspace status
 * (moe_read_status).  No host synchronization inside.
 */
int moe_layer_forward(const moe_layer* layer, const void* x, int T, void* out, int32_t* topk_idx_out,
                      float* topk_gate_out, void* ws, size_t ws_bytes, moe_stream_t stream);

/*
 * moe_layer_forward for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same kernels and same
 * results as moe_layer_forward, minus `ws`: the scratch is a fixed array of MOE_STATIC_SCRATCH_BYTES inside
 * the library, one per GPU, held until the process ends.  The call allocates nothing and frees nothing.
 * Fails with MOE_EWORKSPACE when moe_workspace_bytes(layer, T) exceeds MOE_STATIC_SCRATCH_BYTES (at the
 * Mixtral shape, d_model 4096, d_ff 14336, top-2: up to 32 tokens fit).
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (two streams, two
 * threads) race; serialize them or use moe_layer_forward with separate workspaces.  The status bits of the
 * most recent call are read with moe_read_status(NULL, stream, &bits) while that GPU is current.
 */
size_t moe_static_scratch_bytes(void);
int moe_layer_forward_static(const moe_layer* layer, const void* x, int T, void* out, int32_t* topk_idx_out,
                             float* topk_gate_out, moe_stream_t stream);

/*
 * Expert-miss path (§3: device memory is set aside as a swap space that receives an expert from the host when
 * a token is routed to an expert that is not on the device; §4.1: the copy of an expert is what offloading costs).  Experts of `layer` with resident == 0 live in PINNED
 * host memory; when the gating network routes a token to one of them it is copied into a slot of a device-side
 * swap space on `copy_stream` while the resident experts of the same call already compute on `stream`, then the
 * swapped-in experts run and their contribution is added.  The result equals moe_layer_forward on the same
 * layer with every expert resident (T > 1: bit for bit; T == 1: the output is rounded to fp16 once more between
 * the two passes).
 *   host_experts: HOST array [n_experts]; entry e is read only if layer->experts[e].resident == 0 and then
 *                 names the expert's matrices (same layouts, `prec` as in the layer) in pinned host memory;
 *                 a missed expert whose entry has no data keeps the behaviour of moe_layer_forward (left out,
 *                 MOE_ENOTRESIDENT status bit)
 *   swap:         device memory, n_slots slots of slot_bytes >= moe_swap_slot_bytes(layer) each, 256-byte aligned;
 *                 more misses than slots are served in rounds that reuse the slots
 *   host_idx:     pinned host int32 [T * top_k]: the routing result is handed to the host through it
 *   copied_event, computed_event: hipEvent_t created by the caller (timing not needed)
 * Unlike every other call this one waits for `stream` once (the host must see the routing result to know what
 * to copy), so it cannot be captured into a graph.  *n_missed (host, nullable) = experts copied by this call.
 */
typedef struct {
    const moe_expert* host_experts;
    void* swap;
    size_t slot_bytes;
    int32_t n_slots;
    int32_t* host_idx;
    moe_stream_t copy_stream;
    void* copied_event;
    void* computed_event;
} moe_swap;
size_t moe_swap_slot_bytes(const moe_layer* layer);
int moe_layer_forward_swap(const moe_layer* layer, const moe_swap* swap, const void* x, int T, void* out,
                           int32_t* topk_idx_out, float* topk_gate_out, void* ws, size_t ws_bytes, moe_stream_t stream,
                           int32_t* n_missed);

/*
 * Chain of n_layers blocks as in a decoder stack whose non-expert parts are reduced to the 16-bit
 * glue (§3: non-expert layers are always 16-bit):  for each layer
 *   n = fp16_rne( h / sqrt(mean(h^2) + eps) * rms_gain[layer] );   h <- fp16_rne( h + MoE_layer(n) )
 * layers: host array [n_layers]; rms_gain: host array of n_layers device pointers to fp16 [d_model];
 * h: device fp16 [T, d_model], updated in place; topk_idx_out: device int32 [n_layers, T, top_k] or NULL.
 * All layers must share d_model, d_ff, n_experts, top_k.  ws sized by moe_workspace_bytes(&layers[0], T).
 */
int moe_chain_forward(const moe_layer* layers, const void* const* rms_gain, int n_layers, float eps, void* h,
                      int T, int32_t* topk_idx_out, void* ws, size_t ws_bytes, moe_stream_t stream);

/*
 * Dequantize one 4-bit matrix to fp16 (check hook for the format; also what a switch of an expert
 * from 4-bit to 16-bit form needs when the table is re-planned for new constraints, §3):
 *   w_fp16[r,c] = fp16_rne( fp32(code[r,c]) * fp32(scale[r,c/64]) + fp32(zero[r,c/64]) )
 * m: 4-bit matrix [out,in]; w_fp16: device fp16 [out,in].
 */
int moe_dequant_int4(const moe_mat* m, int out, int in, void* w_fp16, moe_stream_t stream);

/*
 * Quantize one fp16 matrix to the 4-bit form on the device (switching an expert from 16-bit to
 * 4-bit without a host round trip; §3 has experts change format when the constraints change).
 * Per group of 64 columns: zero = min; scale = fp16_rne((fp32(max) - fp32(min)) / 15);
 * code = clamp(rint((fp32(w) - fp32(zero)) / fp32(scale)), 0, 15), all codes 0 when scale == 0.
 * w_fp16: device fp16 [out,in]; packed: device uint8 [out,in/2]; scale, zero: device fp16 [out,in/64].
 */
int moe_quantize_int4(const void* w_fp16, int out, int in, void* packed, void* scale, void* zero,
                      moe_stream_t stream);

/*
 * The same two hooks for the 8-bit form: codes: device uint8 [out,in]; scale, zero: device fp16 [out,in/64];
 * scale = fp16_rne((fp32(max) - fp32(min)) / 255), code = clamp(rint((fp32(w) - fp32(zero)) / fp32(scale)), 0, 255).
 * Both are bit-exact against the definition.
 */
int moe_dequant_int8(const moe_mat* m, int out, int in, void* w_fp16, moe_stream_t stream);
int moe_quantize_int8(const void* w_fp16, int out, int in, void* codes, void* scale, void* zero, moe_stream_t stream);

/*
 * Seeded synthetic tensors written directly in device memory (stand-ins for trained weights and real
 * activations): element i of the stream is a pure function of (seed, stream_id, first + i).
 * kind 0: sum-of-eight-uniforms "normal" stream, kind 1: uniform stream; `scale` is the fp32 factor
 * applied to the integer draw before rounding to fp16.  dst: device fp16 [n].
 */
int moe_synth_fill_f16(void* dst, size_t n, size_t first, uint64_t seed, uint64_t stream_id, float scale,
                       int kind, moe_stream_t stream);

/* Waits for `stream`, then reads the status word of `ws` (NULL: of the library's own scratch on the current GPU,
 * as used by moe_layer_forward_static): OR of (1 << -code) over the device-side conditions
 * raised by the most recent moe_layer_forward / moe_chain_forward / moe_permute call that used `ws`
 * (bit 3: a routed expert was not resident; bit 1: an expert index outside [0, n_experts)). */
int moe_read_status(void* ws, moe_stream_t stream, int* status_bits);

/*
 * Measurement hook: the next launch of kernel `kernel` made by this thread is bracketed by
 * hipEventRecord(start_event) / hipEventRecord(stop_event) on the stream it is launched on (one shot;
 * arm again for the next launch).  Events are hipEvent_t created by the caller with timing enabled.
 * Both events NULL: a bracket that has been armed and not used yet is dropped.  A call on one token launches no
 * separate gating kernel (the gating network runs inside the up-projection launch): MOE_KERNEL_ROUTE then never
 * fires.  An armed bracket must not meet a launch that is being captured into a graph.
 */
enum { MOE_KERNEL_ROUTE = 0,   /* gating (with the RMSNorm of the chained configuration) */
       MOE_KERNEL_PERMUTE = 1, /* grouping */
       MOE_KERNEL_UP = 2,      /* up-projection + SiLU gate */
       MOE_KERNEL_DOWN = 3,    /* down-projection (with the weighted average at one token) */
       MOE_KERNEL_COMBINE = 4, /* weighted average of a multi-token call */
       MOE_KERNEL_STREAM_READ = 5 /* the plain read of moe_stream_read */ };
int moe_trace_kernel(int kernel, void* start_event, void* stop_event);

/*
 * Measurement hook: one kernel that reads `bytes` (multiple of 16) of device memory at `src` (16-byte aligned)
 * once, with the same streamed 128-bit loads as the expert kernels and no arithmetic.  Timed by the caller, it
 * gives the streaming-read ceiling of the GPU at a given size, beside which the bandwidth-bound kernels are
 * reported.  sink: device, 4 bytes, practically never written.
 */
int moe_stream_read(const void* src, size_t bytes, void* sink, moe_stream_t stream);

/*
 * Partitioner / planner (§3, Eq. 1): host-only arithmetic, no device work.  From the GPU memory available and the
 * task's preference it fills the expert table's two attributes for all `num_experts` experts of a model:
 *   throughput preference: the number of 16-bit experts is Eq. 1,
 *       Num_E,16 = floor((mem_gpu - size_non_expert - num_experts * size_e4) / (3 * size_e4))
 *                  if mem_gpu > size_non_expert + num_experts * size_e4, else 0     (clamped to num_experts);
 *   quality preference: `num_e4` experts are 4-bit, as the task asks.
 * Which experts are 4-bit is a seeded random choice (§3: the quantized attribute is assigned at random).  The
 * location attribute is then given out while the budget mem_gpu - size_non_expert - swap_bytes lasts, 4-bit
 * experts first, then 16-bit ones, each class in expert order (§3: 4-bit experts go to the GPU first, a swap
 * space is kept for expert misses).
 * quantized, resident: HOST arrays of num_experts bytes (1 = 4-bit / 1 = in device memory), written by the call.
 * Returns MOE_EINVAL on NULL arguments, size_e4 == 0, num_experts < 1 or num_e4 outside [0, num_experts].
 */
typedef enum { MOE_PREFER_THROUGHPUT = 0, MOE_PREFER_QUALITY = 1 } moe_preference;
typedef struct {
    uint64_t mem_gpu;         /* bytes of device memory the job may use */
    uint64_t size_non_expert; /* bytes of the non-expert layers, always 16-bit and resident */
    uint64_t size_e16;        /* bytes of one expert in 16-bit form */
    uint64_t size_e4;         /* bytes of one expert in 4-bit form */
    uint64_t swap_bytes;      /* device memory set aside for expert misses */
    uint64_t seed;            /* of the random choice of 4-bit experts */
    int32_t num_experts;      /* all experts of the model (layers x experts per layer) */
    int32_t preference;       /* moe_preference */
    int32_t num_e4;           /* quality preference only: requested number of 4-bit experts */
} moe_plan_request;
typedef struct {
    int32_t num_e16, num_e4;           /* experts per precision */
    int32_t resident_e16, resident_e4; /* of those, in device memory */
    uint64_t bytes_resident;           /* size_non_expert + resident experts */
} moe_plan_result;
int moe_plan(const moe_plan_request* req, moe_plan_result* res, uint8_t* quantized, uint8_t* resident);

/* Host string describing the last error returned on this thread ("" if none). */
const char* moe_last_error(void);

/* Library version, 1000*major + minor. */
int moe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOEMIX_H */
