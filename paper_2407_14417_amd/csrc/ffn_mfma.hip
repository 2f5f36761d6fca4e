// Expert feed-forward layers on many rows (prefill, batched decode): grouped matrix products on the
// matrix cores (paper §1: experts are parallel FF layers; §3: each is 16-bit or 4-bit).
//
//   up  : h[r, n] = silu(sum_c W1[n,c] x_r[c]) * (sum_c W3[n,c] x_r[c])      rows r of one expert, grouped order
//   down: y[s][r, n] = sum_{c in split s} W2[n,c] h[r,c]                      partial sums of the contraction splits
//
// One workgroup = 4 wavefronts = one (expert, tile of weight rows, chunk of activation rows, contraction split).
// Weights are the A operand of v_mfma_f32_16x16x32_f16: lane (r, c) holds 8 contraction elements of weight row r.
// Activations are the B operand, staged in LDS and shared by the 4 wavefronts.  Each lane's 4 accumulators of one
// 16x16 product are 4 consecutive weight rows of one activation row, so results are stored as 8-byte (fp16) or
// 16-byte (fp32) pieces.  4-bit weights travel as codes and are expanded in registers (codes masked into the
// mantissa of an fp16 constant, the constant subtracted, one packed fp16 multiply-add with the group's scale and
// zero); 8-bit codes likewise, with a byte permute in place of the masks.
// Four bodies, chosen per chunk:
//   tile_body    launches with chunks of at most 64 rows, ranges with an odd number of 128-column steps, 8-bit
//                experts, one-tile chunks.  Weights are read in whole 128-byte lines (8 lanes per row, 8 rows per
//                load instruction, streamed) and turned into operand layout through a small wavefront-private LDS
//                region; activations as a [16*CT, 128*SPB] tile per stage, double-buffered, one barrier per stage.
//   direct_body  16-bit experts in launches with 128-row chunks: weights straight into operand registers, chunks of
//                up to 256 rows, the order of loads, LDS reads and products pinned by hand.
//   quant4_body  4-bit experts in those launches, chunks of 2 .. 8 tiles: the same schedule with the expansion of the
//                codes folded in.
//   quant4_wide_body  the same for chunks of 9 .. 12 tiles (a 4-bit expert's chunks hold up to 192 rows).
#include <atomic>

#include "common.hpp"
#include "kernels.hpp"

namespace moemix {

namespace {

// Weights of launches with few activation rows per expert are read once, in whole lines: streamed past the caches'
// replacement order.
constexpr int kTemporalNA = 4;     // A operands per wavefront from which on weight lines are kept for sibling chunks
constexpr int kDirectNCT = 5;      // activation tiles per chunk from which on 16-bit weights go straight to registers
                                   // (launches with 128-row chunks only)
constexpr int kNASmall = 2;        // A operands per wavefront of launches with at most 32 rows per chunk
constexpr int kSPBMax = 2;         // most 128-column steps per LDS stage
constexpr int spb_for(int ct) { return (8 / ct) < kSPBMax ? (8 / ct) : kSPBMax; }
constexpr int kKTile = 128;                 // contraction elements per LDS tile
constexpr int kDirectRows = 256;            // most activation rows of a chunk of a 16-bit expert (direct_body)
constexpr unsigned kComputeUnits = 256;     // of the MI355X
constexpr int kQuantRows = 192;             // ... of a 4-bit expert (quant4_wide_body: 12 tiles leave it the registers it needs)

struct MfmaArgs {
    DevExperts ex;
    const int32_t* offsets;   // [E+1] grouped rows per expert, or null in direct mode
    const int32_t* perm;      // up, grouped: grouped row -> flat pair (token = pair / top_k); null: rows in order
    int top_k;
    int direct_expert, direct_n;
    const half_t* in;         // up: x [T, K]; down: h [rows, K]
    void* out;                // up: h [rows, N] fp16; down: y [splits][rows_total, N] fp32
    int K, N, E;
    int k_per_split;          // contraction elements per split (multiple of 128)
    int tiles;                // tiles of weight rows (grid.x = tiles * splits)
    size_t split_stride;      // elements of y between two splits
    int unit_bytes;           // LDS bytes per A operand for weight staging: 4096 if any expert is 16-bit, else 2048
    uint8_t order[MOE_MAX_EXPERTS];   // the experts in the order their chunks are handed out
    int32_t* status;
};

// Pointers into device (global) memory, typed as such, and a pin that keeps a uniform pointer in scalar
// registers so that "uniform base + 32-bit lane offset" compiles to the scalar-base addressing form.
#define MOEMIX_GLOBAL __attribute__((address_space(1)))
typedef const char MOEMIX_GLOBAL* gptr_t;
__device__ __forceinline__ gptr_t scalar_ptr(const void* p) {
    gptr_t g = (gptr_t)p;
    asm volatile("" : "+s"(g));
    return g;
}

__device__ __forceinline__ float4_t mfma16(half8_t a, half8_t b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Nothing moves across this point when the compiler schedules instructions: the pipelined bodies below lay out
// their loads, LDS accesses and products by hand.
__device__ __forceinline__ void pin_schedule() { __builtin_amdgcn_sched_barrier(0); }

// The same product with the accumulator tied to one register tuple by construction: in long straight-line loops the
// compiler otherwise unties some products (writes the sum to a new tuple), leaves every accumulator somewhere else
// at the end of an iteration and copies them all back at its head.  The instruction is opaque to the compiler's
// hazard handling: a reader of the accumulators that is not such a product has to follow mfma_settle().
__device__ __forceinline__ void mfma16_tied(float4_t& c, half8_t a, half8_t b) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}
// More wait states than the longest interval the hardware wants between a matrix product and a read of its result.
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

// (a & mask) | bits in one instruction: the mask travels in a scalar register, the OR-ed bits in a vector one
// (the instruction may read a single scalar operand, which is why the compiler does not form it by itself).
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t bits) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(bits));
    return r;
}

// fp16 pairs (1024, 1024) and (64, 64) held in vector registers (not volatile: identical copies are merged).
// A 32-bit lane offset as a value the compiler has not seen before: its widening to 64 bits then stays next to the
// load that uses it (scalar base + 32-bit lane offset in one instruction) instead of being hoisted out of the loop
// as a register pair per offset.
__device__ __forceinline__ uint32_t fresh_offset(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}
__device__ __forceinline__ uint32_t vreg_const(uint32_t v) {
    uint32_t m;
    asm("v_mov_b32 %0, %1" : "=v"(m) : "s"(v));
    return m;
}

// Eight 4-bit codes of one word -> their dequantized fp16 values, in the order (0,4,1,5,2,6,3,7).
__device__ __forceinline__ half8_t expand_word(uint32_t w, half2_t s2, half2_t z2, uint32_t m1024, uint32_t m64) {
    const uint32_t w8 = w >> 8;
    // low nibbles land in the mantissa of 1024 (ulp 1), high nibbles in the mantissa of 64 (ulp 1/16, code << 4)
    const half2_t q04 = as_half2(and_or(w, 0x000F000Fu, m1024)) - as_half2(m1024);
    const half2_t q15 = as_half2(and_or(w, 0x00F000F0u, m64)) - as_half2(m64);
    const half2_t q26 = as_half2(and_or(w8, 0x000F000Fu, m1024)) - as_half2(m1024);
    const half2_t q37 = as_half2(and_or(w8, 0x00F000F0u, m64)) - as_half2(m64);
    const half2_t a = __builtin_elementwise_fma(q04, s2, z2), b = __builtin_elementwise_fma(q15, s2, z2);
    const half2_t c = __builtin_elementwise_fma(q26, s2, z2), d = __builtin_elementwise_fma(q37, s2, z2);
    return half8_t{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

// Eight 8-bit codes (two words) -> their dequantized fp16 values, in column order.
__device__ __forceinline__ half8_t expand_bytes(uint32_t w0, uint32_t w1, half2_t s2, half2_t z2, uint32_t m1024,
                                                uint32_t m64x4) {
    // a byte permute puts each code into the low byte of an fp16 whose high byte is 0x64: 1024 + code, exactly
    const half2_t q01 = as_half2(__builtin_amdgcn_perm(m64x4, w0, 0x04010400u)) - as_half2(m1024);
    const half2_t q23 = as_half2(__builtin_amdgcn_perm(m64x4, w0, 0x04030402u)) - as_half2(m1024);
    const half2_t q45 = as_half2(__builtin_amdgcn_perm(m64x4, w1, 0x04010400u)) - as_half2(m1024);
    const half2_t q67 = as_half2(__builtin_amdgcn_perm(m64x4, w1, 0x04030402u)) - as_half2(m1024);
    const half2_t a = __builtin_elementwise_fma(q01, s2, z2), b = __builtin_elementwise_fma(q23, s2, z2);
    const half2_t c = __builtin_elementwise_fma(q45, s2, z2), d = __builtin_elementwise_fma(q67, s2, z2);
    return half8_t{a[0], a[1], b[0], b[1], c[0], c[1], d[0], d[1]};
}

// What one workgroup works on, set up once by the kernel and handed to the precision-specific body.
struct TileCtx {
    const half_t* in;        // activations
    const int32_t* perm;     // up, grouped: grouped row -> flat pair; else null
    int top_k;
    int K, N;
    int begin, m0, rows;     // grouped rows [begin + m0, begin + m0 + rows)
    int n0;                  // first weight row of the workgroup
    int k_begin, n_steps;    // contraction range [k_begin, k_begin + 128 n_steps)
    int rot;                 // the workgroup walks the range from step rot on, wrapping around (a multiple of 4; see below)
    int mc;                  // rows per LDS buffer (16 * ct of the launch)
    int unit_bytes;          // LDS bytes per A operand of the weight staging regions (2048: 4-bit only, 4096)
    uint8_t* lds;
};

// Results of one workgroup: lane (r16, c4) holds, for activation row 16 j + r16, weight rows
// 16 tile + 4 c4 + (0..3) of the wavefront's NT/4 rows.
template <bool UP, int NCT, int NA>
__device__ __forceinline__ void store_results(const TileCtx& c, const float4_t (&acc)[NA][NCT], void* out_base, int wave,
                                              int r16, int c4) {
    constexpr int NT = UP ? 32 * NA : 64 * NA;
    const int N = c.N;
#pragma unroll
    for (int j = 0; j < NCT; ++j) {
        const int rr = 16 * j + r16;
        if (rr < c.rows) {
            const size_t g = (size_t)(c.begin + c.m0 + rr);
            if (UP) {
                half_t* h = (half_t*)out_base + g * N;
#pragma unroll
                for (int tile = 0; tile < NA / 2; ++tile) {
                    const int col = c.n0 + wave * (NT / 4) + tile * 16 + c4 * 4;
                    if (col < N) {
                        half4_t o;
#pragma unroll
                        for (int v = 0; v < 4; ++v) o[v] = (half_t)silu_mul(acc[2 * tile][j][v], acc[2 * tile + 1][j][v]);
                        *(half4_t*)(h + col) = o;
                    }
                }
            } else {
                float* y = (float*)out_base + g * N;
#pragma unroll
                for (int tile = 0; tile < NA; ++tile) {
                    const int col = c.n0 + wave * (NT / 4) + tile * 16 + c4 * 4;
                    if (col < N) *(float4_t*)(y + col) = acc[tile][j];
                }
            }
        }
    }
}

// A wavefront holds NA A operands (16-row tiles of weights) per step.  UP: two matrices (w1, w3), NA/2 tiles each
// (workgroup of 4 wavefronts: 32 NA rows); down: one matrix (w2), NA tiles (workgroup: 64 NA rows).  NA = 4 for
// chunks of many activation rows (each B operand read from LDS feeds 4 products), NA = 2 when a chunk holds at
// most 32 rows: the kernel is then bound by the expansion of the codes, and half the registers per wavefront
// buy twice the wavefronts per SIMD to hide its latencies.
// NCT = 16-row activation tiles computed (exactly the tiles that hold rows), so the inner loops are
// straight-line code.  SPB = 128-column steps per LDS stage (and per barrier): a launch with few activation
// rows per chunk stages more columns at a time, so that the LDS buffers always hold 128 x 128 elements.
template <bool UP, int PREC, int NCT, int SPB, int NA>   // PREC: moe_prec of the expert
__device__ __forceinline__ void tile_body(const TileCtx& c, const DevExpert& ee, void* out_base) {
    constexpr bool INT4 = PREC == MOE_PREC_INT4G64, INT8 = PREC == MOE_PREC_INT8G64, QUANT = INT4 || INT8;
    constexpr int NT = UP ? 32 * NA : 64 * NA;     // weight rows per workgroup: 16 NA / (matrices) per wavefront
    constexpr int kStride = SPB * kKTile * 2 + 16;     // bytes per activation row of an LDS stage (16 bytes of padding)
    constexpr int PPR = 16 * SPB;                      // 16-byte pieces per row of a stage
    constexpr int RPP = 256 / PPR;                     // rows the 256 threads cover in one pass
    constexpr int NP = NCT * SPB;                      // pieces per thread and stage
    const int tid = threadIdx.x, lane = tid & 63, r16 = lane & 15, c4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = c.K, N = c.N, n_steps = c.n_steps;
    const int last = n_steps - 1;    // loads that would run past the contraction range repeat the last step instead
    const int buf_bytes = c.mc * kStride;

    // ---- activation pieces this thread stages: column piece tid % PPR of rows tid / PPR + RPP i.
    // Rows past the end of the chunk repeat its last row: their products are computed and never stored.
    const int pcol = tid % PPR, pstep = pcol >> 4;     // pstep: which 128-column step of the stage the piece is in
    const gptr_t xbase = scalar_ptr(c.in + c.k_begin);
    uint32_t xoff[NP];                                 // byte offsets: the input rows of a launch span less than 4 GB
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        int rr = tid / PPR + RPP * i;
        rr = rr < c.rows ? rr : c.rows - 1;
        const int g = c.begin + c.m0 + rr;
        const uint32_t src = (UP && c.perm) ? (uint32_t)(c.perm[g] / c.top_k) : (uint32_t)g;
        xoff[i] = src * (uint32_t)K * 2 + (pcol & 15) * 16;
    }
    uint4_t xr[NP];
    auto load_x = [&](int stage) {
        int step = stage * SPB + pstep;
        step = step < last ? step : last;
        step = step + c.rot < n_steps ? step + c.rot : step + c.rot - n_steps;
#pragma unroll
        for (int i = 0; i < NP; ++i)
            xr[i] = *(const uint4_t MOEMIX_GLOBAL*)(xbase + step * (kKTile * 2) + fresh_offset(xoff[i]));
    };
    auto store_x = [&](int buf) {
        uint8_t* base = c.lds + buf * buf_bytes + (tid / PPR) * kStride + pcol * 16;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            uint4_t v = xr[i];
            if (INT4) {   // element order (0,4,1,5,2,6,3,7) inside each group of 8, as expand_word delivers codes
                const half8_t h = __builtin_bit_cast(half8_t, v);
                v = __builtin_bit_cast(uint4_t, half8_t{h[0], h[4], h[1], h[5], h[2], h[6], h[3], h[7]});
            }
            *(uint4_t*)(base + i * RPP * kStride) = v;
        }
    };

    // ---- scales and zeros of this lane's weight rows (4-bit): the wavefront owns NT/4 rows from n0 + wave * NT/4,
    // in tiles of 16; lane (r16, c4) looks after row r16 of each tile
    gptr_t sbase[NA], zbase[NA];                       // uniform bases, one lane offset for both
    uint32_t soff[NA];
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        const int tile = UP ? (t >> 1) : t;                        // up: operands (w1 tile0, w3 tile0, w1 tile1, w3 tile1)
        const DevMat& m = UP ? ((t & 1) ? ee.w3 : ee.w1) : ee.w2;
        int row = c.n0 + wave * (NT / 4) + tile * 16 + r16;
        row = row < N ? row : N - 1;                               // rows past the end repeat the last row, never stored
        sbase[t] = QUANT ? scalar_ptr(m.scale + (c.k_begin >> 6)) : nullptr;
        zbase[t] = QUANT ? scalar_ptr(m.zero + (c.k_begin >> 6)) : nullptr;
        soff[t] = (uint32_t)row * (uint32_t)(K >> 6) * 2;
    }
    bool sz_aligned16 = true;                          // (what the 128-bit scale loads below ask of the arrays)
#pragma unroll
    for (int t = 0; t < NA; ++t)
        sz_aligned16 = sz_aligned16 && !(((uintptr_t)sbase[t] | (uintptr_t)zbase[t]) & 15);

    float4_t acc[NA][NCT];
#pragma unroll
    for (int t = 0; t < NA; ++t)
#pragma unroll
        for (int j = 0; j < NCT; ++j) acc[t][j] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // B operand of activation tile j, step q of the stage, sub-step s: lane (r16, c4) reads 8 elements of
    // activation row 16 j + r16
    // (quantized weights: a lane owns 32 consecutive columns of the 128-column step, sub-step s its s-th eight of
    // them -- a permutation of the contraction index that the activations follow)
    const int b_lane = r16 * kStride + (QUANT ? c4 * 64 : c4 * 16);
    constexpr int b_sub = QUANT ? 16 : 64;

    // Pipeline: at the first step of a stage the activation data of the next stage goes to the other LDS buffer
    // (its loads were issued a stage earlier) and the loads of the stage after that are issued; weights run three
    // steps (4-bit) or three 32-column sub-steps (16-bit) ahead in a ring of four register buffers; one barrier
    // closes each stage.  Steps are processed in groups of G = max(4, SPB) so that ring slots, the quarter of the
    // scale loads and the place of the barriers are compile-time constants.
    constexpr int G = SPB > 4 ? SPB : 4;
    uint32_t sz_cur[NA][2], sz_next[NA][2];
    const uint32_t sel = (c4 >> 1) ? 0x03020302u : 0x01000100u;   // which of the two groups of a 128-column step
    const uint32_t m1024 = vreg_const(0x64006400u), m64 = vreg_const(INT8 ? 0x64646464u : 0x54005400u);
    // scales and zeros of four steps with one load: lane (r16, c4) fetches the pair of groups of step 4 S + c4
    auto load_sz = [&](uint32_t (&dst)[NA][2], int S) {
        int step = 4 * S + c4;
        step = step < last ? step : last;
        step = step + c.rot < n_steps ? step + c.rot : step + c.rot - n_steps;
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            dst[t][0] = *(const uint32_t MOEMIX_GLOBAL*)(sbase[t] + step * 4 + fresh_offset(soff[t]));
            dst[t][1] = *(const uint32_t MOEMIX_GLOBAL*)(zbase[t] + step * 4 + fresh_offset(soff[t]));
        }
    };
    // 4-bit, at most 32 rows per chunk (the launch is bound by device memory), ranges of a multiple of 4 steps: scales
    // and zeros of sixteen steps with one 128-bit load per lane and array (lane (r16, c4) fetches the eight groups of
    // steps 16 S + 4 c4 .. + 3), so a row's 128-byte line of scales is asked for in two 64-byte requests instead of
    // eight of 16 bytes; with the narrow requests the lines left L2 between requests and a launch fetched 29 % more
    // than its algorithmic bytes.
    constexpr bool kWideSz = INT4 && NA == kNASmall;
    const bool wide_sz = kWideSz && !(n_steps & 3) && sz_aligned16;
    uint4_t sq_cur[NA][2], sq_next[NA][2];
    auto load_sq = [&](uint4_t (&dst)[NA][2], int S) {
        int step = 16 * S + 4 * c4;
        step = step < n_steps - 4 ? step : n_steps - 4;            // groups past the end repeat the last one (never used)
        step = step + c.rot < n_steps ? step + c.rot : step + c.rot - n_steps;   // (the rotation is a multiple of 4 steps)
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            dst[t][0] = *(const uint4_t MOEMIX_GLOBAL*)(sbase[t] + step * 4 + fresh_offset(soff[t]));
            dst[t][1] = *(const uint4_t MOEMIX_GLOBAL*)(zbase[t] + step * 4 + fresh_offset(soff[t]));
        }
    };
    auto load_sz_narrow = [&](uint4_t (&dst)[NA][2], int S) {      // the narrow form, kept in word 0 of the same registers
        int step = 4 * S + c4;
        step = step < last ? step : last;
        step = step + c.rot < n_steps ? step + c.rot : step + c.rot - n_steps;
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            dst[t][0][0] = *(const uint32_t MOEMIX_GLOBAL*)(sbase[t] + step * 4 + fresh_offset(soff[t]));
            dst[t][1][0] = *(const uint32_t MOEMIX_GLOBAL*)(zbase[t] + step * 4 + fresh_offset(soff[t]));
        }
    };
    // Weights take a detour through LDS so that device memory is read in whole 128-byte lines: one load instruction
    // fetches, for 8 weight rows, one 128-byte line of each row with 8 lanes per row; the 16-byte pieces are written
    // to a wavefront-private LDS region (slots XOR-swizzled by row so that neither side has bank conflicts) and read
    // back in operand layout.  A staging unit is UB bytes of every row: 4-bit, one line = 256 columns = two steps,
    // lane (r16, c4) takes slot 4 * (step & 1) + c4 as its 32 codes of a step; 16-bit, two lines = 128 columns = one
    // step, lane (r16, c4) takes slot 4 * sb + c4 as its 8 weights of sub-step sb.
    // 8-bit, one line = 128 columns = one step, lane (r16, c4) takes slots 2 c4 and 2 c4 + 1 as its 32 codes.
    constexpr int UL = QUANT ? 1 : 2;    // lines per row and unit
    constexpr int UB = UL * 128;         // bytes per row and unit
    constexpr int UA = QUANT ? 2 : 4;    // operand registers (128-bit) per A operand and unit
    uint4_t stg[NA][2 * UL];             // staged loads of the next unit
    uint4_t apc[NA][UA];                 // the current unit in operand layout
    uint32_t goff[NA][2];                // per-lane byte offsets of the staged rows inside the weight matrix
    gptr_t cbase[NA];                    // uniform: start of the contraction range in the weight matrix
    uint8_t* const wreg = c.lds + 2 * buf_bytes + wave * (NA * c.unit_bytes);
    const int w_wr = (lane >> 3) * UB + (((lane & 7) ^ (lane >> 3)) * 16);
    const int w_rd = r16 * UB;
    const int last_unit = INT4 ? (n_steps + 1) / 2 - 1 : n_steps - 1;
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        const int tile = UP ? (t >> 1) : t;
        const DevMat& m = UP ? ((t & 1) ? ee.w3 : ee.w1) : ee.w2;
        cbase[t] = scalar_ptr(m.data + (INT4 ? (c.k_begin >> 1) : INT8 ? c.k_begin : c.k_begin * 2));
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            int row = c.n0 + wave * (NT / 4) + tile * 16 + 8 * hb + (lane >> 3);
            row = row < N ? row : N - 1;                           // rows past the end repeat the last row, never stored
            goff[t][hb] = (uint32_t)row * (uint32_t)(INT4 ? (K >> 1) : INT8 ? K : 2 * K) + (lane & 7) * 16;
        }
    }
    auto load_unit = [&](int unit) {
        // No loads for a unit past the end (the registers keep what they hold; it is never used).  Repeating the last
        // unit instead looked free and was not: a streamed line has left L2 once it has been read, so every workgroup
        // fetched its last line of every row three times (batched decode: + 11 % of the code bytes).
        if (unit > last_unit) return;
        {   // (a rotated range has an even number of steps: whole units)
            const int urot = INT4 ? c.rot >> 1 : c.rot, units = INT4 ? n_steps >> 1 : n_steps;
            if (c.rot) unit = unit + urot < units ? unit + urot : unit + urot - units;
        }
        // 4-bit, odd number of steps: the last pair's second half would leave the row only in the last row of the
        // last split, so the pair is moved back by one step there (its second half is then never used)
        const int byte0 = (!INT4 || 2 * unit + 2 <= n_steps) ? unit * UB : unit * UB - 64;
#pragma unroll
        for (int t = 0; t < NA; ++t)
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int q = 0; q < UL; ++q)
                {
                    const uint4_t MOEMIX_GLOBAL* src =
                        (const uint4_t MOEMIX_GLOBAL*)(cbase[t] + (byte0 + q * 128) + fresh_offset(goff[t][hb]));
                    // launches with many activation rows per expert run several chunks of one expert side by side on
                    // the same XCD: the second reader of a weight line should find it in L2, so the line is not
                    // marked as used once there
                    stg[t][hb * UL + q] = NA >= kTemporalNA ? *src : __builtin_nontemporal_load(src);
                }
    };
    auto stage_to_lds = [&]() {
        wave_lds_handover();   // the previous unit has been read by every lane
#pragma unroll
        for (int t = 0; t < NA; ++t)
#pragma unroll
            for (int hb = 0; hb < 2; ++hb)
#pragma unroll
                for (int q = 0; q < UL; ++q)
                    *(uint4_t*)(wreg + t * (16 * UB) + hb * (8 * UB) + q * 128 + w_wr) = stg[t][hb * UL + q];
        wave_lds_handover();
    };
    auto lds_to_operands = [&](int unit) {
        // (4-bit: for the moved-back last pair of an odd range the wanted step sits in the second half)
        const int shift = (!INT4 || 2 * unit + 2 <= n_steps) ? 0 : 4;
#pragma unroll
        for (int t = 0; t < NA; ++t)
#pragma unroll
            for (int h = 0; h < UA; ++h) {
                const int slot = INT8 ? 2 * c4 + h : (4 * h + c4 + shift) & (8 * UL - 1);
                // the XOR touches the low three bits of the slot only: a piece stays inside its 128-byte line
                apc[t][h] = *(const uint4_t*)(wreg + t * (16 * UB) + w_rd + ((slot ^ (r16 & 7)) * 16));
            }
    };

    load_x(0);
    if (kWideSz && wide_sz) load_sq(sq_cur, 0);
    else if (kWideSz) load_sz_narrow(sq_cur, 0);
    else if (QUANT) load_sz(sz_cur, 0);
    load_unit(0);
    stage_to_lds();
    load_unit(1);
    store_x(0);
    load_x(1);
    __syncthreads();

    for (int base = 0; base < n_steps; base += G) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int step = base + g;
            if (step < n_steps) {                                   // uniform; false only in the last group
                const int stage = step / SPB;
                const uint8_t* xb = c.lds + (stage & 1) * buf_bytes + b_lane + (g % SPB) * (kKTile * 2);
                if (g % SPB == 0) {
                    store_x((stage + 1) & 1);                       // past the last stage this writes data nobody reads
                    load_x(stage + 2);
                    // 4-bit, two steps per stage = one unit of codes per stage: the unit that takes the place of the
                    // one used up in the last stage is asked for here, after the activation loads.  Loads return in
                    // the order of their issue, so an activation load (a hit in L2) issued behind a load of weights
                    // from device memory is held back as long as that one takes.
                    if (INT4 && SPB == 2 && step > 0) load_unit(((step - 1) >> 1) + 2);
                }
                if (INT4) {
                    if (kWideSz && wide_sz) {
                        if (g % 4 == 0 && (step & 15) == 0) {
                            if (step > 0) {
#pragma unroll
                                for (int t = 0; t < NA; ++t) { sq_cur[t][0] = sq_next[t][0]; sq_cur[t][1] = sq_next[t][1]; }
                            }
                            if (step + 16 < n_steps) load_sq(sq_next, step / 16 + 1);   // (nothing past the end: see load_unit)
                        }
                    } else if (g % 4 == 0) {
                        if (step > 0) {
#pragma unroll
                            for (int t = 0; t < NA; ++t) {
                                if (kWideSz) { sq_cur[t][0][0] = sq_next[t][0][0]; sq_cur[t][1][0] = sq_next[t][1][0]; }
                                else { sz_cur[t][0] = sz_next[t][0]; sz_cur[t][1] = sz_next[t][1]; }
                            }
                        }
                        if (step + 4 < n_steps) {                   // (nothing past the end: see load_unit)
                            if (kWideSz) load_sz_narrow(sq_next, step / 4 + 1);
                            else load_sz(sz_next, step / 4 + 1);
                        }
                    }
                    if (g % 2 == 0) lds_to_operands(step >> 1);
                    half2_t s2[NA], z2[NA];
                    // the lane of this row that fetched this step's scales: the step's place among four, or (wide
                    // requests) its group of four steps' place among four, where the step's word is g & 3
                    const int src = (r16 + 16 * ((kWideSz && wide_sz) ? (step >> 2) & 3 : g & 3)) * 4;
#pragma unroll
                    for (int t = 0; t < NA; ++t) {
                        const uint32_t sw = !kWideSz ? sz_cur[t][0] : wide_sz ? sq_cur[t][0][g & 3] : sq_cur[t][0][0];
                        const uint32_t zw = !kWideSz ? sz_cur[t][1] : wide_sz ? sq_cur[t][1][g & 3] : sq_cur[t][1][0];
                        const uint32_t sd = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)sw);
                        const uint32_t zd = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)zw);
                        s2[t] = as_half2(__builtin_amdgcn_perm(sd, sd, sel));
                        z2[t] = as_half2(__builtin_amdgcn_perm(zd, zd, sel));
                    }
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
                        half8_t af[NA];
#pragma unroll
                        for (int t = 0; t < NA; ++t) af[t] = expand_word(apc[t][g & 1][sb], s2[t], z2[t], m1024, m64);
#pragma unroll
                        for (int j2 = 0; j2 < NCT; ++j2) {
                            const half8_t b = *(const half8_t*)(xb + j2 * 16 * kStride + sb * b_sub);
#pragma unroll
                            for (int t = 0; t < NA; ++t) acc[t][j2] = mfma16(af[t], b, acc[t][j2]);
                        }
                    }
                    if (g % 2 == 1 || step == last) {               // the pair is used up: the next one takes its place
                        stage_to_lds();
                        if (SPB != 2) load_unit((step >> 1) + 2);   // (two steps per stage: at the next stage's start)
                    }
                } else if (INT8) {
                    if (g % 4 == 0) {
                        if (step > 0) {
#pragma unroll
                            for (int t = 0; t < NA; ++t) { sz_cur[t][0] = sz_next[t][0]; sz_cur[t][1] = sz_next[t][1]; }
                        }
                        if (step + 4 < n_steps) load_sz(sz_next, step / 4 + 1);
                    }
                    lds_to_operands(step);
                    half2_t s2[NA], z2[NA];
                    const int src = (r16 + 16 * (g & 3)) * 4;       // the lane of this row that fetched this step's scales
#pragma unroll
                    for (int t = 0; t < NA; ++t) {
                        const uint32_t sd = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)sz_cur[t][0]);
                        const uint32_t zd = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)sz_cur[t][1]);
                        s2[t] = as_half2(__builtin_amdgcn_perm(sd, sd, sel));
                        z2[t] = as_half2(__builtin_amdgcn_perm(zd, zd, sel));
                    }
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
                        half8_t af[NA];
#pragma unroll
                        for (int t = 0; t < NA; ++t)
                            af[t] = expand_bytes(apc[t][sb >> 1][2 * (sb & 1)], apc[t][sb >> 1][2 * (sb & 1) + 1], s2[t], z2[t],
                                                 m1024, m64);
#pragma unroll
                        for (int j2 = 0; j2 < NCT; ++j2) {
                            const half8_t b = *(const half8_t*)(xb + j2 * 16 * kStride + sb * b_sub);
#pragma unroll
                            for (int t = 0; t < NA; ++t) acc[t][j2] = mfma16(af[t], b, acc[t][j2]);
                        }
                    }
                    stage_to_lds();                                 // the step is used up: the next one takes its place
                    load_unit(step + 2);
                } else {
                    lds_to_operands(step);
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
#pragma unroll
                        for (int j2 = 0; j2 < NCT; ++j2) {
                            const half8_t b = *(const half8_t*)(xb + j2 * 16 * kStride + sb * b_sub);
#pragma unroll
                            for (int t = 0; t < NA; ++t)
                                acc[t][j2] = mfma16(__builtin_bit_cast(half8_t, apc[t][sb]), b, acc[t][j2]);
                        }
                    }
                    stage_to_lds();                                 // the step is used up: the next one takes its place
                    load_unit(step + 2);
                }
                if (g % SPB == SPB - 1 || step == last) __syncthreads();
            }
        }
    }

    store_results<UP, NCT, NA>(c, acc, out_base, wave, r16, c4);
}

// 16-bit weights against chunks of many activation rows.  A compute unit cannot draw more than about 25 GB/s of
// weights out of device memory (measured with a bare read kernel of the same access pattern), and a 16-bit weight
// brings only 2 products per activation row, so such a workgroup is bound by its weight stream unless it has some
// hundred rows to multiply: chunks of 16-bit experts therefore hold up to 256 rows (NCT <= 16 tiles, all 256
// accumulation registers), which halves the number of times an expert's weights are read.
// A operands skip LDS: lane (r16, c4) loads its 8 weights of every 32-column sub-step straight from device memory
// (16 rows x 64 bytes per instruction) into a ring of R sub-step slots, R sub-steps ahead of their use.
// Activations are staged through registers into an LDS stage of [rows][128 columns] without padding: piece p
// (16 bytes) of row r sits in slot p ^ (r & 15) of the row, so that the 16 lanes of a B operand read (rows r .. r + 15
// at one piece index) hit 16 different slots, as do the 16 lanes that write one row.
// B operands are read from LDS one unit (at most 8 tiles of one sub-step) ahead into a second register set, also
// across the end of a step: the workgroup's one barrier per step sits before the last unit, whose reads were issued
// before it; after it the stage just read out is free for the stage after the next one, and the other stage
// (written before the barrier) is read for the next step's first unit.
// The order of loads, LDS reads and products is pinned group by group (one B operand read per NA products); left
// to itself the compiler issues the weight loads at the end of the step that precedes their use and waits for
// every B operand it has just asked for.
template <bool UP, int NCT>
__device__ __forceinline__ void direct_body(const TileCtx& c, const DevExpert& ee, void* out_base) {
    constexpr int NA = 4;
    constexpr int NT = UP ? 32 * NA : 64 * NA;
    constexpr int R = NCT > 8 ? 4 : 8;                 // ring slots = sub-steps of weights in flight
    constexpr int U = NCT > 8 ? 2 : 1;                 // units (B register sets' worth of tiles) per sub-step
    constexpr int NU0 = NCT > 8 ? 8 : NCT;             // tiles in a sub-step's first unit; the second holds the rest
    constexpr int kRowBytes = kKTile * 2;              // one activation row of a stage: 256 bytes, 16 slots
    constexpr int kStageBytes = kDirectRows * kRowBytes;
    const int tid = threadIdx.x, lane = tid & 63, r16 = lane & 15, c4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = c.K, N = c.N, n_steps = c.n_steps;
    const int last = n_steps - 1, last_sub = 4 * n_steps - 1;

    // ---- activation pieces this thread stages: 16-byte piece tid & 15 of rows (tid >> 4) + 16 i, into slot
    // (tid & 15) ^ (tid >> 4) of the row.  Rows past the end of the chunk repeat its last row (their products are
    // computed and never stored).  At most 8 pieces are in registers at a time: chunks of more than 8 tiles stage
    // a stage in two batches.
    constexpr int XB = NCT > 8 ? 8 : NCT;              // pieces per batch
    const gptr_t xbase = scalar_ptr(c.in + c.k_begin);
    uint32_t xoff[NCT];                                // byte offsets: the activations of one call stay below 4 GB
#pragma unroll
    for (int i = 0; i < NCT; ++i) {
        int rr = (tid >> 4) + 16 * i;
        rr = rr < c.rows ? rr : c.rows - 1;
        const int g = c.begin + c.m0 + rr;
        const uint32_t src = (UP && c.perm) ? (uint32_t)(c.perm[g] / c.top_k) : (uint32_t)g;
        xoff[i] = src * (uint32_t)K * 2 + (tid & 15) * 16;
    }
    uint4_t xr[XB];
    uint8_t* const xst = c.lds + (tid >> 4) * kRowBytes + (((tid & 15) ^ (tid >> 4)) * 16);
    auto load_x1 = [&](int i, int stage) {             // piece i of the thread, stage `stage` of the contraction
        int phys = stage < last ? stage : last;
        phys = phys + c.rot < n_steps ? phys + c.rot : phys + c.rot - n_steps;
        xr[i % XB] = *(const uint4_t MOEMIX_GLOBAL*)(xbase + phys * kRowBytes + fresh_offset(xoff[i]));
    };
    auto store_x1 = [&](int i, int stage) {            // ... into LDS buffer stage & 1
        *(uint4_t*)(xst + (stage & 1) * kStageBytes + i * (16 * kRowBytes)) = xr[i % XB];
    };

    // ---- weights: row r16 of each of the wavefront's NA tiles, 16 bytes at c4 * 16 of every 64-byte sub-step
    gptr_t cbase[NA];
    uint32_t doff[NA];
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        const int tile = UP ? (t >> 1) : t;                        // up: operands (w1 tile0, w3 tile0, w1 tile1, w3 tile1)
        const DevMat& m = UP ? ((t & 1) ? ee.w3 : ee.w1) : ee.w2;
        cbase[t] = scalar_ptr(m.data + c.k_begin * 2);
        int row = c.n0 + wave * (NT / 4) + tile * 16 + r16;
        row = row < N ? row : N - 1;                               // rows past the end repeat the last row, never stored
        doff[t] = (uint32_t)row * (uint32_t)(2 * K) + c4 * 16;
    }
    uint4_t ar[R][NA];
    // (sub-steps past the end repeat the last one: a branch around the loads costs more than the loads -- the
    // compiler then waits as if they had not been issued, which drains the ring: prefill step + 5 %)
    auto load_a = [&](int slot, int sub) {
        sub = sub < last_sub ? sub : last_sub;
        sub = sub + 4 * c.rot <= last_sub ? sub + 4 * c.rot : sub + 4 * c.rot - 4 * n_steps;
#pragma unroll
        for (int t = 0; t < NA; ++t) ar[slot][t] = *(const uint4_t MOEMIX_GLOBAL*)(cbase[t] + sub * 64 + fresh_offset(doff[t]));
    };

    float4_t acc[NA][NCT];
#pragma unroll
    for (int t = 0; t < NA; ++t)
#pragma unroll
        for (int j = 0; j < NCT; ++j) acc[t][j] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // B operand of tile j, sub-step sb: row 16 j + r16, piece 4 sb + c4, which sits in slot (4 sb + c4) ^ r16
    int b_off[4];
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) b_off[sb] = r16 * kRowBytes + (((4 * sb + c4) ^ r16) * 16);
    half8_t bq[2][8];
    auto read_unit = [&](half8_t (&dst)[8], const uint8_t* stage_base, int sb, int h) {
#pragma unroll
        for (int j = 0; j < (h ? NCT - NU0 : NU0); ++j)
            dst[j] = *(const half8_t*)(stage_base + b_off[sb] + (8 * h + j) * (16 * kRowBytes));
    };

    // Stage 0 (and, for chunks of more than 8 tiles, the second batch of it) goes to LDS here; the batch that is in
    // registers when the loop starts is what the loop's schedule expects there: all of stage 1 (one batch per stage),
    // or the second batch of stage 1 (two).  The ring's loads go out last.
    if (U == 1) {
#pragma unroll
        for (int i = 0; i < NCT; ++i) load_x1(i, 0);
#pragma unroll
        for (int i = 0; i < NCT; ++i) { store_x1(i, 0); load_x1(i, 1); }
    } else {
#pragma unroll
        for (int i = 0; i < XB; ++i) load_x1(i, 0);
#pragma unroll
        for (int i = 0; i < XB; ++i) { store_x1(i, 0); if (XB + i < NCT) load_x1(XB + i, 0); }
#pragma unroll
        for (int i = 0; i < XB; ++i) { if (XB + i < NCT) store_x1(XB + i, 0); load_x1(i, 1); }
#pragma unroll
        for (int i = 0; i < XB; ++i) { store_x1(i, 1); if (XB + i < NCT) load_x1(XB + i, 1); }
    }
    pin_schedule();
#pragma unroll
    for (int u = 0; u < R; ++u) load_a(u, u);
    pin_schedule();
    __syncthreads();
    read_unit(bq[0], c.lds, 0, 0);
    pin_schedule();

    for (int base = 0; base < n_steps; base += R / 4) {            // (the number of steps is even here)
#pragma unroll
        for (int g = 0; g < R / 4; ++g) {
            const int step = base + g;
            const uint8_t* const cur = c.lds + (step & 1) * kStageBytes;
            const uint8_t* const nxt = c.lds + ((step + 1) & 1) * kStageBytes;
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                const int slot = (4 * g + sb) % R;
#pragma unroll
                for (int h = 0; h < U; ++h) {
                    const int v = sb * U + h;                      // unit of the step; B register set v & 1
                    const bool last_unit = v == 4 * U - 1;
                    // Before the step's last unit: every wavefront has read this stage out (its last reads were
                    // issued a unit ago) and has written its pieces of the next one.
                    if (last_unit) __syncthreads();
                    const int nsb = h + 1 < U ? sb : sb + 1, nh = h + 1 < U ? h + 1 : 0;
                    const int ntiles = h ? NCT - NU0 : NU0;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (j < ntiles) {
                            // the next unit's operand j (the units of a sub-step may differ in size: the rest below)
                            if (j < (nh ? NCT - NU0 : NU0))
                                bq[(v + 1) & 1][j] = *(const half8_t*)((last_unit ? nxt : cur) + b_off[nsb & 3] +
                                                                        (8 * nh + j) * (16 * kRowBytes));
#pragma unroll
                            for (int t = 0; t < NA; ++t)
                                mfma16_tied(acc[t][8 * h + j], __builtin_bit_cast(half8_t, ar[slot][t]), bq[v & 1][j]);
                            // Activation staging, one piece per group.  One batch per stage: stage step + 1 goes
                            // to LDS during the first sub-step (the buffer has been free since the last barrier) and
                            // stage step + 2 takes its place in the registers.  Two batches: the second batch of
                            // stage step + 1 goes to LDS in unit 2; the first batch of stage step + 2 is loaded in
                            // unit 3 and written after the barrier, in the last unit, into the stage just read out,
                            // where the second batch is loaded.
                            if (U == 1) {
                                if (v == 0) { store_x1(j, step + 1); load_x1(j, step + 2); }
                            } else {
                                if (v == 2 && XB + j < NCT) store_x1(XB + j, step + 1);
                                if (v == 3) {
#pragma unroll
                                    for (int i = j; i < XB; i += ntiles) load_x1(i, step + 2);
                                }
                                if (last_unit) {
#pragma unroll
                                    for (int i = j; i < XB; i += ntiles) {
                                        store_x1(i, step + 2);
                                        if (XB + i < NCT) load_x1(XB + i, step + 2);
                                    }
                                }
                            }
                            pin_schedule();
                        }
                    }
                    if ((nh ? NCT - NU0 : NU0) > ntiles) {         // operands of the next unit this one had no group for
#pragma unroll
                        for (int j = ntiles; j < (nh ? NCT - NU0 : NU0); ++j)
                            bq[(v + 1) & 1][j] = *(const half8_t*)((last_unit ? nxt : cur) + b_off[nsb & 3] +
                                                                    (8 * nh + j) * (16 * kRowBytes));
                        pin_schedule();
                    }
                }
                load_a(slot, 4 * step + sb + R);
                pin_schedule();
            }
        }
    }
    mfma_settle();
    store_results<UP, NCT, NA>(c, acc, out_base, wave, r16, c4);
}

// 4-bit weights against chunks of 17 .. 128 activation rows (launches with 128-row chunks): the same pinned schedule
// as direct_body, with the expansion of the codes folded in.  The codes skip LDS too: lane (r16, c4) loads the 16
// bytes that hold its 32 codes of a 128-column step (16 rows x 64 bytes per instruction) into a ring of R steps;
// word sb of the 16 bytes is its operand of sub-step sb (columns 32 c4 + 8 sb .. + 7 in the order
// (0,4,1,5,2,6,3,7), which the staged activations follow).  The A operands of a sub-step are expanded during the
// products of the sub-step before it, into a second register set; the scales and zeros of a step are fetched with
// the loads of four steps (lane (r16, c4) fetches the two groups of step 4 S + c4) and handed out through the
// lane-permute network during the step before (asked for in its first sub-step, picked up in its third).
// The number of steps is a multiple of 4 here.
template <bool UP, int NCT>
__device__ __forceinline__ void quant4_body(const TileCtx& c, const DevExpert& ee, void* out_base) {
    constexpr int NA = 4;
    constexpr int NT = UP ? 32 * NA : 64 * NA;
    constexpr int R = 4;                               // ring slots = steps of codes in flight
    constexpr int kRowBytes = kKTile * 2;              // one activation row of a stage: 256 bytes, 16 slots
    constexpr int kStageBytes = 128 * kRowBytes;
    const int tid = threadIdx.x, lane = tid & 63, r16 = lane & 15, c4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = c.K, N = c.N, n_steps = c.n_steps;
    const int last = n_steps - 1;
    auto phys_step = [&](int step) {                   // steps past the end repeat the last one
        step = step < last ? step : last;
        return step + c.rot < n_steps ? step + c.rot : step + c.rot - n_steps;
    };

    // ---- activation pieces this thread stages: 16-byte piece tid & 15 of rows (tid >> 4) + 16 i, into slot
    // (tid & 15) ^ (tid >> 4) of the row, its 8 elements in the order the expanded codes have
    const gptr_t xbase = scalar_ptr(c.in + c.k_begin);
    uint32_t xoff[NCT];
#pragma unroll
    for (int i = 0; i < NCT; ++i) {
        int rr = (tid >> 4) + 16 * i;
        rr = rr < c.rows ? rr : c.rows - 1;
        const int g = c.begin + c.m0 + rr;
        const uint32_t src = (UP && c.perm) ? (uint32_t)(c.perm[g] / c.top_k) : (uint32_t)g;
        xoff[i] = src * (uint32_t)K * 2 + (tid & 15) * 16;
    }
    // Chunks of at most 6 tiles have the registers for two stages of activations under way (XD = 2: a piece is asked
    // for two steps before it goes to LDS, in the register set of its stage's parity); their steps are short (1.6 us
    // at 3 tiles), and a piece that has left L2 takes longer than that.
    constexpr int XD = NCT <= 6 ? 2 : 1;
    uint4_t xr[XD][NCT];
    uint8_t* const xst = c.lds + (tid >> 4) * kRowBytes + (((tid & 15) ^ (tid >> 4)) * 16);
    auto load_x1 = [&](int i, int stage) {
        xr[stage & (XD - 1)][i] = *(const uint4_t MOEMIX_GLOBAL*)(xbase + phys_step(stage) * kRowBytes + fresh_offset(xoff[i]));
    };
    auto store_x1 = [&](int i, int stage) {
        const half8_t h = __builtin_bit_cast(half8_t, xr[stage & (XD - 1)][i]);
        *(half8_t*)(xst + (stage & 1) * kStageBytes + i * (16 * kRowBytes)) =
            half8_t{h[0], h[4], h[1], h[5], h[2], h[6], h[3], h[7]};
    };

    // ---- weights: row r16 of each of the wavefront's NA tiles: codes, scales, zeros
    gptr_t cbase[NA];
    uint32_t doff[NA];
    gptr_t sbase[NA], zbase[NA];                       // scales and zeros: uniform bases, one lane offset for both
    uint32_t soff[NA];
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        const int tile = UP ? (t >> 1) : t;                        // up: operands (w1 tile0, w3 tile0, w1 tile1, w3 tile1)
        const DevMat& m = UP ? ((t & 1) ? ee.w3 : ee.w1) : ee.w2;
        cbase[t] = scalar_ptr(m.data + (c.k_begin >> 1));
        int row = c.n0 + wave * (NT / 4) + tile * 16 + r16;
        row = row < N ? row : N - 1;                               // rows past the end repeat the last row, never stored
        doff[t] = (uint32_t)row * (uint32_t)(K >> 1) + c4 * 16;
        sbase[t] = scalar_ptr(m.scale + (c.k_begin >> 6));
        zbase[t] = scalar_ptr(m.zero + (c.k_begin >> 6));
        soff[t] = (uint32_t)row * (uint32_t)(K >> 6) * 2;
    }
    uint4_t ar[R][NA];
    auto load_a = [&](int slot, int step) {
        const int ps = phys_step(step);
#pragma unroll
        for (int t = 0; t < NA; ++t) ar[slot][t] = *(const uint4_t MOEMIX_GLOBAL*)(cbase[t] + ps * 64 + fresh_offset(doff[t]));
    };
    uint32_t sz_a[NA][2], sz_b[NA][2];                 // scales / zeros of the four steps under way, of the next four
    auto load_sz = [&](uint32_t (&dst)[NA][2], int S) {
        const int ps = phys_step(4 * S + c4);          // (rotation and range are multiples of 4 steps: no wrap inside)
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            dst[t][0] = *(const uint32_t MOEMIX_GLOBAL*)(sbase[t] + ps * 4 + fresh_offset(soff[t]));
            dst[t][1] = *(const uint32_t MOEMIX_GLOBAL*)(zbase[t] + ps * 4 + fresh_offset(soff[t]));
        }
    };
    const uint32_t sel = (c4 >> 1) ? 0x03020302u : 0x01000100u;   // which of the two groups of a 128-column step
    const uint32_t m1024 = vreg_const(0x64006400u), m64 = vreg_const(0x54005400u);
    half2_t s2[NA], z2[NA];
    uint32_t hs[NA], hz[NA];                           // a step's scale and zero words on their way through the network
    auto hand_ask = [&](const uint32_t (&src)[NA][2], int g, int t0) {   // tiles t0, t0 + 1
        const int from = (r16 + 16 * (g & 3)) * 4;     // the lane of this row that fetched step g's scales
#pragma unroll
        for (int t = t0; t < t0 + 2; ++t) {
            hs[t] = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)src[t][0]);
            hz[t] = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)src[t][1]);
        }
    };
    auto hand_take = [&](half2_t (&so)[NA], half2_t (&zo)[NA]) {
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            so[t] = as_half2(__builtin_amdgcn_perm(hs[t], hs[t], sel));
            zo[t] = as_half2(__builtin_amdgcn_perm(hz[t], hz[t], sel));
        }
    };

    float4_t acc[NA][NCT];
#pragma unroll
    for (int t = 0; t < NA; ++t)
#pragma unroll
        for (int j = 0; j < NCT; ++j) acc[t][j] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // B operand of tile j, sub-step sb: row 16 j + r16, piece 4 c4 + sb, which sits in slot (4 c4 + sb) ^ r16
    int b_off[4];
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) b_off[sb] = r16 * kRowBytes + (((4 * c4 + sb) ^ r16) * 16);
    half8_t bq[2][NCT];
    uint32_t af[2][NA][4];                             // A operands as words: codes (0,4) (1,5) (2,6) (3,7) dequantized
    // The expansion of a sub-step's NA words (see expand_word) as a list of 52 single instructions, stage by stage
    // over all tiles, so that no instruction stands next to the one it depends on: 4 shifts, 16 mask-and-or into the
    // mantissa of 1024 or 64, 16 subtractions of that constant, 16 multiply-adds with scale and zero.
    uint32_t xw8[NA], xq[NA][4];
    auto expand_op = [&](int k, int slot, int word, uint32_t (&dst)[NA][4], const half2_t (&sc)[NA], const half2_t (&ze)[NA]) {
        if (k < 4) { xw8[k] = ar[slot][k][word] >> 8; return; }
        const int t = ((k - 4) & 15) >> 2, q = (k - 4) & 3;
        const uint32_t magic = (q & 1) ? m64 : m1024;
        if (k < 20) xq[t][q] = and_or(q >= 2 ? xw8[t] : ar[slot][t][word], (q & 1) ? 0x00F000F0u : 0x000F000Fu, magic);
        else if (k < 36) xq[t][q] = __builtin_bit_cast(uint32_t, as_half2(xq[t][q]) - as_half2(magic));
        else dst[t][q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(as_half2(xq[t][q]), sc[t], ze[t]));
    };

    // stage 0 to LDS, stage 1 in registers; scales of the first four steps; the ring
#pragma unroll
    for (int i = 0; i < NCT; ++i) load_x1(i, 0);
    load_sz(sz_a, 0);
#pragma unroll
    for (int i = 0; i < NCT; ++i) { store_x1(i, 0); load_x1(i, 1); }
    if (XD == 2) {
#pragma unroll
        for (int i = 0; i < NCT; ++i) load_x1(i, 2);
    }
    pin_schedule();
#pragma unroll
    for (int u = 0; u < R; ++u) load_a(u, u);
    pin_schedule();
    hand_ask(sz_a, 0, 0);
    hand_ask(sz_a, 0, 2);
    hand_take(s2, z2);
#pragma unroll
    for (int k = 0; k < 52; ++k) expand_op(k, 0, 0, af[0], s2, z2);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NCT; ++j) bq[0][j] = *(const half8_t*)(c.lds + b_off[0] + j * (16 * kRowBytes));
    pin_schedule();

    // Two things shape the order of the memory instructions of a step.  A wavefront can have 16 LDS instructions
    // under way and stalls at the 17th: the step's LDS writes (staged activations) and lane permutes (scales) are
    // spread over its first three sub-steps instead of standing with the first one's B operand reads.  And loads
    // retire in the order of their issue: a load of weights (device memory, some 2.4 us under this kernel's own
    // traffic) holds back the activation loads behind it (L2 hits) that long, so everything that comes from device
    // memory goes out right after the step's last activation loads, most of a step before the next ones are
    // waited for.
    constexpr int PPS = (NCT + 2) / 3;                 // activation pieces staged per sub-step
    for (int base = 0; base < n_steps; base += 4) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int step = base + g;
            const uint8_t* const cur = c.lds + (step & 1) * kStageBytes;
            const uint8_t* const nxt = c.lds + ((step + 1) & 1) * kStageBytes;
            half2_t s2n[NA], z2n[NA];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                const int u = 4 * g + sb;                          // parity of the B and A register sets
                if (sb == 3) __syncthreads();                      // stage step + 1 is in LDS, this stage is read out
                // what the next sub-step multiplies: word sb + 1 of this step's codes, or word 0 of the next step's
                const int nslot = sb < 3 ? g : (g + 1) & 3, nword = (sb + 1) & 3;
#pragma unroll
                for (int j = 0; j < NCT; ++j) {
                    if (sb < 3 && j < PPS && sb * PPS + j < NCT) {   // stage step + 1 to LDS, stage step + 2 on its way
                        store_x1(sb * PPS + j, step + 1);
                        load_x1(sb * PPS + j, step + 1 + XD);
                    }
                    bq[(u + 1) & 1][j] = *(const half8_t*)((sb < 3 ? cur : nxt) + b_off[nword] + j * (16 * kRowBytes));
                    // The sub-step's 4 NCT products and, spread evenly between them, the 52 instructions that expand
                    // the next sub-step's A operands: a product of this wavefront hides one or two vector
                    // instructions that follow it, a run of products hides nothing and a run of vector instructions
                    // leaves the matrix cores idle (bare loops: 4 products then 12 vector instructions 30.8 cycles
                    // per product, one product then 3 vector instructions 23.8).
#pragma unroll
                    for (int t = 0; t < NA; ++t) {
                        mfma16_tied(acc[t][j],
                                    __builtin_bit_cast(half8_t, uint4_t{af[u & 1][t][0], af[u & 1][t][1], af[u & 1][t][2],
                                                                        af[u & 1][t][3]}),
                                    bq[u & 1][j]);
                        constexpr int NM = 4 * NCT;                 // products per sub-step
                        const int m = 4 * j + t;                    // this one
#pragma unroll
                        for (int k = (m * 52 + NM - 1) / NM; k < ((m + 1) * 52 + NM - 1) / NM; ++k) {
                            if (sb < 3) expand_op(k, nslot, nword, af[(u + 1) & 1], s2, z2);
                            else expand_op(k, nslot, nword, af[(u + 1) & 1], s2n, z2n);
                        }
                        pin_schedule();
                    }
                }
                if (sb < 2) {                                      // the next step's scales and zeros: asked for ...
                    if (g < 3) hand_ask(sz_a, g + 1, 2 * sb);
                    else hand_ask(sz_b, 0, 2 * sb);
                    pin_schedule();
                }
                if (sb == 2) {
                    hand_take(s2n, z2n);                           // ... and picked up
                    // the codes of three steps on, into the slot the last step used up (at step 0 this fetches step
                    // 3 once more); every fourth step the scales and zeros of the next four
                    load_a((g + 3) & 3, step + R - 1);
                    if (g == 0) load_sz(sz_b, base / 4 + 1);
                    pin_schedule();
                }
                if (sb == 3) {
#pragma unroll
                    for (int t = 0; t < NA; ++t) { s2[t] = s2n[t]; z2[t] = z2n[t]; }
                    pin_schedule();
                }
            }
        }
#pragma unroll
        for (int t = 0; t < NA; ++t) { sz_a[t][0] = sz_b[t][0]; sz_a[t][1] = sz_b[t][1]; }
    }
    mfma_settle();
    store_results<UP, NCT, NA>(c, acc, out_base, wave, r16, c4);
}

// 4-bit weights against chunks of 129 .. 192 activation rows (9 .. 12 tiles): quant4_body's expansion and scale
// hand-out in direct_body's two-unit schedule.  A workgroup's time is 35 us for expanding its 256 x 4096 codes plus
// 6 us per tile of 16 rows (prefill workload, per-workgroup device clock stamps), so one chunk of 9 tiles costs 89 us
// where chunks of 8 tiles and 1 tile cost 87 + 49 us.  A sub-step's products run in two units (tiles 0 .. 7, then the
// rest), each with its own B register set; the 52 instructions that expand the next sub-step's A operands are spread
// over the products of both.  Activations are staged in two batches of at most 8 pieces per thread, as in direct_body.
// Codes and scales of later steps are asked for at the end of a step, right after its last activation loads (loads
// retire in the order of their issue).  The number of steps is a multiple of 4 here.
template <bool UP, int NCT>
__device__ __forceinline__ void quant4_wide_body(const TileCtx& c, const DevExpert& ee, void* out_base) {
    static_assert(NCT > 8 && 16 * NCT <= kQuantRows, "two units of at most 8 tiles");
    constexpr int NA = 4;
    constexpr int NT = UP ? 32 * NA : 64 * NA;
    constexpr int R = 4;                               // ring slots = steps of codes in flight
    constexpr int NU0 = 8;                             // tiles in a sub-step's first unit; the second holds the rest
    constexpr int XB = 8;                              // activation pieces per batch (the second holds the rest)
    static_assert(NCT - XB <= XB, "two batches");
    constexpr int kRowBytes = kKTile * 2;              // one activation row of a stage: 256 bytes, 16 slots
    constexpr int kStageBytes = kDirectRows * kRowBytes;
    const int tid = threadIdx.x, lane = tid & 63, r16 = lane & 15, c4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = c.K, N = c.N, n_steps = c.n_steps;
    const int last = n_steps - 1;
    auto phys_step = [&](int step) {                   // steps past the end repeat the last one
        step = step < last ? step : last;
        return step + c.rot < n_steps ? step + c.rot : step + c.rot - n_steps;
    };

    // ---- activation pieces this thread stages (see quant4_body), at most XB of them in registers at a time
    const gptr_t xbase = scalar_ptr(c.in + c.k_begin);
    uint32_t xoff[NCT];
#pragma unroll
    for (int i = 0; i < NCT; ++i) {
        int rr = (tid >> 4) + 16 * i;
        rr = rr < c.rows ? rr : c.rows - 1;
        const int g = c.begin + c.m0 + rr;
        const uint32_t src = (UP && c.perm) ? (uint32_t)(c.perm[g] / c.top_k) : (uint32_t)g;
        xoff[i] = src * (uint32_t)K * 2 + (tid & 15) * 16;
    }
    uint4_t xr[XB];
    uint8_t* const xst = c.lds + (tid >> 4) * kRowBytes + (((tid & 15) ^ (tid >> 4)) * 16);
    auto load_x1 = [&](int i, int stage) {
        xr[i % XB] = *(const uint4_t MOEMIX_GLOBAL*)(xbase + phys_step(stage) * kRowBytes + fresh_offset(xoff[i]));
    };
    auto store_x1 = [&](int i, int stage) {
        const half8_t h = __builtin_bit_cast(half8_t, xr[i % XB]);
        *(half8_t*)(xst + (stage & 1) * kStageBytes + i * (16 * kRowBytes)) =
            half8_t{h[0], h[4], h[1], h[5], h[2], h[6], h[3], h[7]};
    };

    // ---- weights: row r16 of each of the wavefront's NA tiles: codes, scales, zeros
    gptr_t cbase[NA];
    uint32_t doff[NA];
    gptr_t sbase[NA], zbase[NA];                       // scales and zeros: uniform bases, one lane offset for both
    uint32_t soff[NA];
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        const int tile = UP ? (t >> 1) : t;                        // up: operands (w1 tile0, w3 tile0, w1 tile1, w3 tile1)
        const DevMat& m = UP ? ((t & 1) ? ee.w3 : ee.w1) : ee.w2;
        cbase[t] = scalar_ptr(m.data + (c.k_begin >> 1));
        int row = c.n0 + wave * (NT / 4) + tile * 16 + r16;
        row = row < N ? row : N - 1;                               // rows past the end repeat the last row, never stored
        doff[t] = (uint32_t)row * (uint32_t)(K >> 1) + c4 * 16;
        sbase[t] = scalar_ptr(m.scale + (c.k_begin >> 6));
        zbase[t] = scalar_ptr(m.zero + (c.k_begin >> 6));
        soff[t] = (uint32_t)row * (uint32_t)(K >> 6) * 2;
    }
    uint4_t ar[R][NA];
    auto load_a = [&](int slot, int step) {
        const int ps = phys_step(step);
#pragma unroll
        for (int t = 0; t < NA; ++t) ar[slot][t] = *(const uint4_t MOEMIX_GLOBAL*)(cbase[t] + ps * 64 + fresh_offset(doff[t]));
    };
    uint32_t sz_a[NA][2], sz_b[NA][2];                 // scales / zeros of the four steps under way, of the next four
    auto load_sz = [&](uint32_t (&dst)[NA][2], int S) {
        const int ps = phys_step(4 * S + c4);          // (rotation and range are multiples of 4 steps: no wrap inside)
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            dst[t][0] = *(const uint32_t MOEMIX_GLOBAL*)(sbase[t] + ps * 4 + fresh_offset(soff[t]));
            dst[t][1] = *(const uint32_t MOEMIX_GLOBAL*)(zbase[t] + ps * 4 + fresh_offset(soff[t]));
        }
    };
    const uint32_t sel = (c4 >> 1) ? 0x03020302u : 0x01000100u;   // which of the two groups of a 128-column step
    const uint32_t m1024 = vreg_const(0x64006400u), m64 = vreg_const(0x54005400u);
    half2_t s2[NA], z2[NA];
    uint32_t hs[NA], hz[NA];
    auto hand_ask = [&](const uint32_t (&src)[NA][2], int g, int t0) {   // tiles t0, t0 + 1
        const int from = (r16 + 16 * (g & 3)) * 4;
#pragma unroll
        for (int t = t0; t < t0 + 2; ++t) {
            hs[t] = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)src[t][0]);
            hz[t] = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)src[t][1]);
        }
    };
    auto hand_take = [&](half2_t (&so)[NA], half2_t (&zo)[NA]) {
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            so[t] = as_half2(__builtin_amdgcn_perm(hs[t], hs[t], sel));
            zo[t] = as_half2(__builtin_amdgcn_perm(hz[t], hz[t], sel));
        }
    };

    float4_t acc[NA][NCT];
#pragma unroll
    for (int t = 0; t < NA; ++t)
#pragma unroll
        for (int j = 0; j < NCT; ++j) acc[t][j] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // B operand of tile j, sub-step sb: row 16 j + r16, piece 4 c4 + sb, which sits in slot (4 c4 + sb) ^ r16
    int b_off[4];
#pragma unroll
    for (int sb = 0; sb < 4; ++sb) b_off[sb] = r16 * kRowBytes + (((4 * c4 + sb) ^ r16) * 16);
    half8_t bq[2][8];
    uint32_t af[2][NA][4];
    uint32_t xw8[NA];
    // the 52 instructions of quant4_body's expansion; the intermediate values live in the destination registers
    auto expand_op = [&](int k, int slot, int word, uint32_t (&dst)[NA][4], const half2_t (&sc)[NA], const half2_t (&ze)[NA]) {
        if (k < 4) { xw8[k] = ar[slot][k][word] >> 8; return; }
        const int t = ((k - 4) & 15) >> 2, q = (k - 4) & 3;
        const uint32_t magic = (q & 1) ? m64 : m1024;
        if (k < 20) dst[t][q] = and_or(q >= 2 ? xw8[t] : ar[slot][t][word], (q & 1) ? 0x00F000F0u : 0x000F000Fu, magic);
        else if (k < 36) dst[t][q] = __builtin_bit_cast(uint32_t, as_half2(dst[t][q]) - as_half2(magic));
        else dst[t][q] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(as_half2(dst[t][q]), sc[t], ze[t]));
    };

    // Both batches of stage 0 and the first of stage 1 go to LDS here; the second batch of stage 1 is in registers
    // when the loop starts.  Scales of the first four steps; the ring.
#pragma unroll
    for (int i = 0; i < XB; ++i) load_x1(i, 0);
    load_sz(sz_a, 0);
#pragma unroll
    for (int i = 0; i < XB; ++i) { store_x1(i, 0); if (XB + i < NCT) load_x1(XB + i, 0); }
#pragma unroll
    for (int i = 0; i < XB; ++i) { if (XB + i < NCT) store_x1(XB + i, 0); load_x1(i, 1); }
#pragma unroll
    for (int i = 0; i < XB; ++i) { store_x1(i, 1); if (XB + i < NCT) load_x1(XB + i, 1); }
    pin_schedule();
#pragma unroll
    for (int u = 0; u < R; ++u) load_a(u, u);
    pin_schedule();
    hand_ask(sz_a, 0, 0);
    hand_ask(sz_a, 0, 2);
    hand_take(s2, z2);
#pragma unroll
    for (int k = 0; k < 52; ++k) expand_op(k, 0, 0, af[0], s2, z2);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NU0; ++j) bq[0][j] = *(const half8_t*)(c.lds + b_off[0] + j * (16 * kRowBytes));
    pin_schedule();

    for (int base = 0; base < n_steps; base += 4) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int step = base + g;
            const uint8_t* const cur = c.lds + (step & 1) * kStageBytes;
            const uint8_t* const nxt = c.lds + ((step + 1) & 1) * kStageBytes;
            half2_t s2n[NA], z2n[NA];
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                const int u = 4 * g + sb;                          // parity of the A register sets
                // what the next sub-step multiplies: word sb + 1 of this step's codes, or word 0 of the next step's
                const int nslot = sb < 3 ? g : (g + 1) & 3, nword = (sb + 1) & 3;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int v = 2 * sb + h;                      // unit of the step; B register set v & 1
                    const bool last_unit = v == 7;
                    // Before the step's last unit: every wavefront has read this stage out (its last reads were
                    // issued a unit ago) and has written its pieces of the next one.
                    if (last_unit) __syncthreads();
                    const int nh = 1 - h;
                    const int ntiles = h ? NCT - NU0 : NU0, next_tiles = nh ? NCT - NU0 : NU0;
                    // the next unit's operands: the same sub-step's second unit, or the next sub-step's first
                    const uint8_t* const nb = (last_unit ? nxt : cur) + b_off[h ? nword : sb] + 8 * nh * (16 * kRowBytes);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        if (j < ntiles) {
                            if (j < next_tiles) bq[(v + 1) & 1][j] = *(const half8_t*)(nb + j * (16 * kRowBytes));
#pragma unroll
                            for (int t = 0; t < NA; ++t) {
                                mfma16_tied(acc[t][8 * h + j],
                                            __builtin_bit_cast(half8_t, uint4_t{af[u & 1][t][0], af[u & 1][t][1],
                                                                                af[u & 1][t][2], af[u & 1][t][3]}),
                                            bq[v & 1][j]);
                                constexpr int NM = 4 * NCT;         // products per sub-step
                                const int m = 4 * (8 * h + j) + t;  // this one
#pragma unroll
                                for (int k = (m * 52 + NM - 1) / NM; k < ((m + 1) * 52 + NM - 1) / NM; ++k) {
                                    if (sb < 3) expand_op(k, nslot, nword, af[(u + 1) & 1], s2, z2);
                                    else expand_op(k, nslot, nword, af[(u + 1) & 1], s2n, z2n);
                                }
                                pin_schedule();
                            }
                            // Activation staging, one piece per group (direct_body's two-batch order): the second
                            // batch of stage step + 1 goes to LDS in unit 2; the first batch of stage step + 2 is
                            // loaded in unit 3 and written after the barrier, in the last unit, into the stage just
                            // read out, where the second batch is loaded.
                            if (v == 2 && XB + j < NCT) store_x1(XB + j, step + 1);
                            if (v == 3) {
#pragma unroll
                                for (int i = j; i < XB; i += ntiles) load_x1(i, step + 2);
                            }
                            if (last_unit) {
#pragma unroll
                                for (int i = j; i < XB; i += ntiles) {
                                    store_x1(i, step + 2);
                                    if (XB + i < NCT) load_x1(XB + i, step + 2);
                                }
                            }
                            pin_schedule();
                        }
                    }
                    if (next_tiles > ntiles) {                     // operands of the next unit this one had no group for
#pragma unroll
                        for (int j = ntiles; j < next_tiles; ++j) bq[(v + 1) & 1][j] = *(const half8_t*)(nb + j * (16 * kRowBytes));
                        pin_schedule();
                    }
                }
                if (sb < 2) {                                      // the next step's scales and zeros: asked for ...
                    if (g < 3) hand_ask(sz_a, g + 1, 2 * sb);
                    else hand_ask(sz_b, 0, 2 * sb);
                    pin_schedule();
                }
                if (sb == 2) {
                    hand_take(s2n, z2n);                           // ... and picked up
                    pin_schedule();
                }
                if (sb == 3) {
                    // the codes of four steps on, into the slot this step has used up; every fourth step the scales
                    // and zeros of the next four
                    load_a(g, step + R);
                    if (g == 0) load_sz(sz_b, base / 4 + 1);
#pragma unroll
                    for (int t = 0; t < NA; ++t) { s2[t] = s2n[t]; z2[t] = z2n[t]; }
                    pin_schedule();
                }
            }
        }
#pragma unroll
        for (int t = 0; t < NA; ++t) { sz_a[t][0] = sz_b[t][0]; sz_a[t][1] = sz_b[t][1]; }
    }
    mfma_settle();
    store_results<UP, NCT, NA>(c, acc, out_base, wave, r16, c4);
}

// WIDE: the block holds 8-bit experts as well.  The 8-bit body needs more registers than the other two, and a
// kernel's register count is that of its largest body, so blocks without 8-bit experts get a kernel without it
// (and keep four wavefronts per SIMD at few rows per expert).  The wide kernel has bodies for 1, 2, 4 and 8 tiles.
template <bool UP, int CT, bool WIDE>
__global__ __launch_bounds__(256) void grouped_mfma_kernel(const MfmaArgs a) {
    constexpr int MC = 16 * CT;                  // activation rows per chunk
    constexpr int NA = CT <= 2 ? kNASmall : 4;   // A operands per wavefront
    constexpr int NT = UP ? 32 * NA : 64 * NA;   // weight rows per workgroup
    constexpr int SPB = spb_for(CT);          // 128-column steps per LDS stage
    extern __shared__ __align__(16) uint8_t lds[];   // [2][MC][SPB * 256 + 16]
    const int tid = threadIdx.x;
    // grid: x = tile of weight rows + tiles * contraction split, y = chunk: workgroups are handed out chunk by
    // chunk, in expert order
    // Workgroups go to the 8 XCDs (each with an L2 of its own) in turn, in launch order: with 2, 4 or 8 contraction
    // splits those of one chunk and split, which read the same slice of the activations, get the indices that
    // land on the same 4, 2 or 1 XCDs.
    int tile_x, split_z;
    {
        const int sp = gridDim.x / a.tiles, i = blockIdx.x, xcd = i & 7, slot = i >> 3;
        if (sp > 1 && (a.tiles * sp) % 8 == 0 && 8 % sp == 0) {
            const int q = 8 / sp;                                  // XCDs per split
            split_z = xcd / q; tile_x = slot * q + xcd % q;
        } else {
            tile_x = i % a.tiles; split_z = i / a.tiles;
        }
    }

    // ---- which expert, which rows.  Chunks hold at most MC rows, those of 16-bit experts in launches with 128-row
    // chunks up to kDirectRows (direct_body), split evenly in whole tiles.
    const int n_steps = a.k_per_split / kKTile;
    // (launches with 128-row chunks have LDS for two 256-row stages)
    const bool wide_ok = CT >= 8 && !(n_steps & 1);
    // (4-bit chunks of more than 128 rows save compute-unit time, not latency: one expert alone whose launch does not
    // fill the chip twice over is faster with more, smaller workgroups side by side -- 148 rows: 73 us in chunks of
    // 128 + 20 rows, 89 us in one chunk)
    const bool quant4_ok = wide_ok && !(n_steps & 3);
    const bool wide4_ok = quant4_ok && (a.direct_expert < 0 || gridDim.x * gridDim.y >= 2 * kComputeUnits);
    auto chunk_rows = [&](int expert, int n) {   // rows per chunk of an expert with n rows
        const int prec = a.ex.e[expert].prec;
        if (!((wide_ok && prec == MOE_PREC_FP16 && n > 16 * (kDirectNCT - 1)) ||
              (wide4_ok && prec == MOE_PREC_INT4G64 && n > MC)))
            return MC;
        const int cap = prec == MOE_PREC_FP16 ? kDirectRows : kQuantRows;
        const int nch = (n + cap - 1) / cap;
        return (((n + nch - 1) / nch) + 15) & ~15;
    };
    int e, begin, cnt, per, chunk = blockIdx.y;
    if (a.direct_expert >= 0) {
        e = a.direct_expert; begin = 0; cnt = a.direct_n; per = chunk_rows(e, cnt);
    } else {
        // Chunks are handed out expert by expert in the order the host has put the experts in (launch_order)
        e = -1; begin = 0; cnt = 0; per = MC;
        for (int j = 0; j < a.E; ++j) {
            const int i = a.order[j];
            const int b = a.offsets[i], n = a.offsets[i + 1] - b, pr = chunk_rows(i, n), nch = (n + pr - 1) / pr;
            if (chunk < nch) { e = i; begin = b; cnt = n; per = pr; break; }
            chunk -= nch;
        }
        if (e < 0) return;
    }
    TileCtx c;
    c.m0 = chunk * per;
    if (c.m0 >= cnt) return;
    c.in = a.in; c.perm = a.perm; c.top_k = a.top_k; c.K = a.K; c.N = a.N;
    c.begin = begin;
    c.rows = min(per, cnt - c.m0);
    c.n0 = tile_x * NT;
    c.k_begin = split_z * a.k_per_split;
    c.n_steps = n_steps;
    // Workgroups that work on different weight rows start at different places of the contraction range and wrap
    // around: walking it in step, every workgroup of the launch would ask for the same columns of rows that lie a
    // power of two apart at the same time, which lands on a fraction of the memory channels (measured with a bare
    // read kernel of the same access pattern: 4.3 TB/s in step, 6.0 TB/s staggered).  The offset depends on the
    // tile of weight rows, the expert and the split only, so a given output element is summed in the same order in
    // every launch shape.
    // Up-projection: one starting place per tile.  Down-projection (rows 7 x 4 KB apart in the Mixtral shape, less
    // prone to the effect): one per expert and contraction split, so that the workgroups which share a slice of the
    // hidden rows walk it in step and find it in L2 (fetched bytes of the prefill down-projection: 1060 MB with one
    // starting place per tile, 781 MB per slice, 637 MB with the slice's workgroups on two XCDs as well).
    c.rot = (c.n_steps & 3) ? 0 : 4 * ((UP ? tile_x * 5 : e * 3 + split_z * 5) % (c.n_steps >> 2));
    c.mc = MC;
    c.unit_bytes = a.unit_bytes;
    c.lds = lds;
    const DevExpert& ee = a.ex.e[e];
    void* out_base = UP ? a.out : (void*)((float*)a.out + split_z * a.split_stride);
    if (ee.resident == kDeferred) return;
    if (!(ee.resident && ee.w1.data && ee.w3.data && ee.w2.data)) {
        if (tid == 0 && tile_x == 0) atomicOr(a.status, kStatusNotResident);
        if (!UP) {   // rows of an expert that cannot run contribute nothing
            float* y = (float*)out_base;
            for (int i = tid; i < c.rows * NT; i += 256) {
                const int rr = i / NT, cc = c.n0 + i % NT;
                if (cc < c.N) y[(size_t)(begin + c.m0 + rr) * c.N + cc] = 0.0f;
            }
        }
        return;
    }
    const int prec = ee.prec;
    const int nct = (c.rows + 15) >> 4;          // 16-row tiles that hold any rows
    // the straight-line body for exactly the chunk's tiles where the launch can have that many (the clamp keeps
    // the smaller launches from instantiating bodies they never run)
#define MOEMIX_BODY(n)                                                                                          \
    do {                                                                                                        \
        if (prec == MOE_PREC_INT4G64) tile_body<UP, MOE_PREC_INT4G64, ((n) <= CT ? (n) : CT), SPB, NA>(c, ee, out_base); \
        else if (WIDE && prec == MOE_PREC_INT8G64) tile_body<UP, WIDE ? MOE_PREC_INT8G64 : MOE_PREC_FP16, ((n) <= CT ? (n) : CT), SPB, NA>(c, ee, out_base); \
        else tile_body<UP, MOE_PREC_FP16, ((n) <= CT ? (n) : CT), SPB, NA>(c, ee, out_base);                    \
    } while (0)
#define MOEMIX_DIRECT(n) direct_body<UP, CT >= 8 ? (n) : 8>(c, ee, out_base)
    if (CT >= 8 && wide_ok && prec == MOE_PREC_FP16 && nct >= kDirectNCT) {
        switch (nct) {
            case 5: MOEMIX_DIRECT(5); break;
            case 6: MOEMIX_DIRECT(6); break;
            case 7: MOEMIX_DIRECT(7); break;
            case 8: MOEMIX_DIRECT(8); break;
            case 9: MOEMIX_DIRECT(9); break;
            case 10: MOEMIX_DIRECT(10); break;
            case 11: MOEMIX_DIRECT(11); break;
            case 12: MOEMIX_DIRECT(12); break;
            case 13: MOEMIX_DIRECT(13); break;
            case 14: MOEMIX_DIRECT(14); break;
            case 15: MOEMIX_DIRECT(15); break;
            default: MOEMIX_DIRECT(16); break;
        }
        return;
    }
#undef MOEMIX_DIRECT
#define MOEMIX_QUANT4(n) quant4_body<UP, CT >= 8 ? (n) : 8>(c, ee, out_base)
#define MOEMIX_QUANT4W(n) quant4_wide_body<UP, CT >= 8 ? (n) : 12>(c, ee, out_base)
    if (quant4_ok && prec == MOE_PREC_INT4G64 && nct >= 2) {
        switch (nct) {
            case 2: MOEMIX_QUANT4(2); break;
            case 3: MOEMIX_QUANT4(3); break;
            case 4: MOEMIX_QUANT4(4); break;
            case 5: MOEMIX_QUANT4(5); break;
            case 6: MOEMIX_QUANT4(6); break;
            case 7: MOEMIX_QUANT4(7); break;
            case 8: MOEMIX_QUANT4(8); break;
            case 9: MOEMIX_QUANT4W(9); break;
            case 10: MOEMIX_QUANT4W(10); break;
            case 11: MOEMIX_QUANT4W(11); break;
            default: MOEMIX_QUANT4W(12); break;
        }
        return;
    }
#undef MOEMIX_QUANT4
#undef MOEMIX_QUANT4W
    if (WIDE) {
        if (CT >= 8 && nct > 4) MOEMIX_BODY(8);
        else if (CT >= 4 && nct > 2) MOEMIX_BODY(4);
        else if (CT >= 2 && nct > 1) MOEMIX_BODY(2);
        else MOEMIX_BODY(1);
    } else
    if (CT >= 8 && nct > 7) MOEMIX_BODY(8);
    else if (CT >= 8 && nct > 6) MOEMIX_BODY(7);
    else if (CT >= 8 && nct > 5) MOEMIX_BODY(6);
    else if (CT >= 8 && nct > 4) MOEMIX_BODY(5);
    else if (CT >= 4 && nct > 3) MOEMIX_BODY(4);
    else if (CT >= 4 && nct > 2) MOEMIX_BODY(3);
    else if (CT >= 2 && nct > 1) MOEMIX_BODY(2);
    else MOEMIX_BODY(1);
#undef MOEMIX_BODY
}

template <bool UP, int CT, bool WIDE>
void launch_one(const MfmaArgs& a, dim3 grid, hipStream_t st) {
    constexpr int NA = CT <= 2 ? kNASmall : 4;
    // activation stages + 4 wavefronts x NA operands of weight staging
    // (launches with 128-row chunks: at least two unpadded 256-row stages for the pipelined bodies)
    constexpr size_t lds_wide = CT >= 8 ? 2u * kDirectRows * kKTile * 2 : 0;
    const size_t lds_max = 2u * 16 * CT * (spb_for(CT) * kKTile * 2 + 16) + 4 * NA * 4096;
    const size_t lds_plain = 2u * 16 * CT * (spb_for(CT) * kKTile * 2 + 16) + 4 * NA * (size_t)a.unit_bytes;
    const size_t lds_bytes = lds_plain > lds_wide ? lds_plain : lds_wide;
    // the attribute belongs to (kernel, device): set it once per device of the process (bit d of the mask; devices
    // past the 64th set it on every launch)
    static std::atomic<unsigned long long> configured{0};
    int dev = 0;
    (void)hipGetDevice(&dev);
    const unsigned long long bit = dev < 64 ? 1ull << dev : 0ull;
    if (!(configured.load(std::memory_order_relaxed) & bit) || !bit) {
        (void)hipFuncSetAttribute((const void*)grouped_mfma_kernel<UP, CT, WIDE>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds_max);
        configured.fetch_or(bit, std::memory_order_relaxed);
    }
    grouped_mfma_kernel<UP, CT, WIDE><<<grid, 256, lds_bytes, st>>>(a);
}

template <bool UP, bool WIDE>
void launch_ct_w(const MfmaArgs& a, int ct, dim3 grid, hipStream_t st) {
    switch (ct) {
        case 1: launch_one<UP, 1, WIDE>(a, grid, st); break;
        case 2: launch_one<UP, 2, WIDE>(a, grid, st); break;
        case 4: launch_one<UP, 4, WIDE>(a, grid, st); break;
        default: launch_one<UP, 8, WIDE>(a, grid, st); break;
    }
}

// Launches with 128-row chunks hand out the chunks of the 16-bit experts first, then the others, each in expert
// order: a 16-bit workgroup runs 110-130 us (bound by its weight stream) against 45-100 us for a 4-bit one, and the
// launch ends when the last workgroup does, so the long ones must not start last.
void launch_order(const DevExperts& ex, int E, int ct, uint8_t (&order)[MOE_MAX_EXPERTS]) {
    int n = 0;
    for (int pass = 0; pass < 2; ++pass)
        for (int e = 0; e < E; ++e)
            if (ct >= 8 ? (ex.e[e].prec == MOE_PREC_FP16) == (pass == 0) : pass == 0) order[n++] = (uint8_t)e;
    for (; n < MOE_MAX_EXPERTS; ++n) order[n] = 0;
}

bool any_int8(const DevExperts& ex, int E) {
    for (int e = 0; e < E; ++e)
        if (ex.e[e].prec == MOE_PREC_INT8G64) return true;
    return false;
}

template <bool UP>
void launch_ct(const MfmaArgs& a, int ct, dim3 grid, hipStream_t st) {
    if (any_int8(a.ex, a.E)) launch_ct_w<UP, true>(a, ct, grid, st);
    else launch_ct_w<UP, false>(a, ct, grid, st);
}

// Weight staging needs 4 KB of LDS per A operand for 16-bit experts, 2 KB for 4-bit ones.
int staging_unit_bytes(const DevExperts& ex, int E, const RowMap& rows) {
    if (rows.direct_expert >= 0) return ex.e[rows.direct_expert].prec == MOE_PREC_FP16 ? 4096 : 2048;
    for (int e = 0; e < E; ++e)
        if (ex.e[e].resident == 1 && ex.e[e].prec == MOE_PREC_FP16) return 4096;
    return 2048;
}

int chunk_slots(const RowMap& rows, int P, int E, int ct) {
    const int mc = 16 * ct;
    if (rows.direct_expert >= 0) return (rows.direct_n + mc - 1) / mc;
    // every expert may end with one ragged chunk
    const int full = P / mc + E;
    return full;
}

}  // namespace

// every contraction range must hold at least two 128-column steps (4-bit codes are fetched in pairs of steps)
// (and a weight matrix spans less than 4 GB: rows are addressed with 32-bit byte offsets from the matrix)
bool mfma_shape_ok(int d, int f) {
    return d % kKTile == 0 && f % kKTile == 0 && d >= 2 * kKTile && f >= 2 * kKTile && (uint64_t)d * (uint64_t)f * 2u < (1ull << 32);
}

// The kernels address the rows of their input (tokens, hidden rows) with 32-bit byte offsets from its start.
bool mfma_rows_ok(int rows, int d, int f) {
    return (uint64_t)rows * (uint64_t)(d > f ? d : f) * 2u < (1ull << 32);
}

MfmaPlan plan_mfma(int P, int d, int f, int E) {
    MfmaPlan p;
    const int avg = (P + E - 1) / E;              // rows per expert if the load were even
    p.ct = avg <= 16 ? 1 : avg <= 32 ? 2 : avg <= 64 ? 4 : 8;
    // down-projection: split the contraction until there are enough workgroups for 256 compute units
    const int steps = f / kKTile;
    const int down_rows = 64 * (p.ct <= 2 ? kNASmall : 4);
    const int base = ((d + down_rows - 1) / down_rows) * (P / (16 * p.ct) + 1);
    int best = 1, best4 = 0;
    for (int s = 1; s <= 16; ++s)
        if (steps % s == 0 && steps / s >= 2 && base * s <= 640) {
            best = s;
            if ((steps / s) % 4 == 0) best4 = s;
        }
    // launches with 128-row chunks have pipelined bodies for ranges of a multiple of 4 steps: a split that gives
    // such ranges is preferred if it keeps at least half the workgroups
    p.down_splits = (p.ct == 8 && best4 * 2 >= best) ? best4 : best;
    return p;
}

void launch_ffn_up_mfma(const DevExperts& ex, int E, const RowMap& rows, int P, const half_t* x, int d, int f, half_t* h,
                        int ct, int32_t* status, hipStream_t st) {
    TraceScope trace(kKernelUp, st);
    MfmaArgs a;
    a.ex = ex; a.offsets = rows.offsets; a.perm = rows.perm; a.top_k = rows.top_k;
    a.direct_expert = rows.direct_expert; a.direct_n = rows.direct_n;
    a.in = x; a.out = h; a.K = d; a.N = f; a.E = E; a.k_per_split = d; a.split_stride = 0; a.status = status;
    a.unit_bytes = staging_unit_bytes(ex, E, rows);
    launch_order(ex, E, ct, a.order);
    const int up_rows = 32 * (ct <= 2 ? kNASmall : 4);
    a.tiles = (f + up_rows - 1) / up_rows;
    dim3 grid(a.tiles, chunk_slots(rows, P, E, ct), 1);
    launch_ct<true>(a, ct, grid, st);
}

void launch_ffn_down_mfma(const DevExperts& ex, int E, const RowMap& rows, int P, const half_t* h, int d, int f, float* y,
                          int ct, int splits, size_t split_stride, int32_t* status, hipStream_t st) {
    TraceScope trace(kKernelDown, st);
    MfmaArgs a;
    a.ex = ex; a.offsets = rows.offsets; a.perm = nullptr; a.top_k = rows.top_k;
    a.direct_expert = rows.direct_expert; a.direct_n = rows.direct_n;
    a.in = h; a.out = y; a.K = f; a.N = d; a.E = E; a.k_per_split = f / splits; a.split_stride = split_stride;
    a.status = status;
    a.unit_bytes = staging_unit_bytes(ex, E, rows);
    launch_order(ex, E, ct, a.order);
    const int down_rows = 64 * (ct <= 2 ? kNASmall : 4);
    a.tiles = (d + down_rows - 1) / down_rows;
    dim3 grid(a.tiles * splits, chunk_slots(rows, P, E, ct), 1);
    launch_ct<false>(a, ct, grid, st);
}

}  // namespace moemix
