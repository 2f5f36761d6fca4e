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
#include "gating.hpp"
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

// The 32 activations of a lane as loaded (four 128-bit pieces), before they are paired up.
struct RawI4 {
    half8_t v[4];
};

__device__ __forceinline__ void request_act_i4(const half_t* __restrict__ src, RawI4& raw) {
#pragma unroll
    for (int j = 0; j < 4; ++j) raw.v[j] = *(const half8_t*)(src + 8 * j);
}

__device__ __forceinline__ void pair_act_i4(const RawI4& raw, ActI4& a) {
    float se = 0.0f, so = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const half8_t v = raw.v[j];
#pragma unroll
        for (int q = 0; q < 4; ++q) a.p[j][q] = half2_t{v[q], v[q + 4]};
        se += ((float)v[0] + (float)v[2]) + ((float)v[4] + (float)v[6]);
        so += ((float)v[1] + (float)v[3]) + ((float)v[5] + (float)v[7]);
    }
    a.c1 = 1024.0f * se + 64.0f * so;
    a.c2 = se + so;
}

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

// (a & mask) | bits in one instruction.  The compiler keeps two instructions here because the fused form
// may read only one scalar operand: the mask goes in a scalar register, the OR-ed bits in a vector one.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t bits) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(bits));
    return r;
}

__device__ __forceinline__ uint32_t bias_magic() {
    uint32_t m;
    asm("v_mov_b32 %0, 0x64006400" : "=v"(m));   // not volatile: identical copies are merged and hoisted
    return m;
}

// s * sum_c q_c x_c + z * sum_c x_c over the lane's 32 columns of one row.
__device__ __forceinline__ float dot_i4(const uint4_t pk, const ActI4& a, float s, float z) {
    const uint32_t magic = bias_magic();   // fp16 pair (1024, 1024), held in a vector register
    float lo = 0.0f, hi = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t w = pk[j], w8 = w >> 8;
        const half2_t q04 = as_half2(and_or(w, 0x000F000Fu, magic));    // 1024 + q
        const half2_t q15 = as_half2(and_or(w, 0x00F000F0u, magic));    // 1024 + 16 q
        const half2_t q26 = as_half2(and_or(w8, 0x000F000Fu, magic));
        const half2_t q37 = as_half2(and_or(w8, 0x00F000F0u, magic));
        lo = __builtin_amdgcn_fdot2(q04, a.p[j][0], lo, false);
        hi = __builtin_amdgcn_fdot2(q15, a.p[j][1], hi, false);
        lo = __builtin_amdgcn_fdot2(q26, a.p[j][2], lo, false);
        hi = __builtin_amdgcn_fdot2(q37, a.p[j][3], hi, false);
    }
    const float t = fmaf(hi, 0.0625f, lo) - a.c1;
    return fmaf(s, t, z * a.c2);
}

// 8-bit layout.  A lane's 128-bit load holds 16 consecutive codes, all of one group of 64 columns.  A byte
// permute puts each code into the mantissa of fp16 1024.0 (0x64 in the high byte), in natural column pairs.
struct ActI8 {
    half2_t p[8];   // the lane's 16 activations of one 1024-column chunk, natural pairs
    float k1;       // 1024 * (sum of the 16 x): offset of the biased codes
    float sx;       // sum of the 16 x: multiplies the group zero
};

__device__ __forceinline__ void load_act_i8(const half_t* __restrict__ src, ActI8& a) {
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const half8_t v = *(const half8_t*)(src + 8 * j);
#pragma unroll
        for (int q = 0; q < 4; ++q) a.p[4 * j + q] = half2_t{v[2 * q], v[2 * q + 1]};
        sum += (((float)v[0] + (float)v[1]) + ((float)v[2] + (float)v[3])) +
               (((float)v[4] + (float)v[5]) + ((float)v[6] + (float)v[7]));
    }
    a.sx = sum;
    a.k1 = 1024.0f * sum;
}

// s * sum_c q_c x_c + z * sum_c x_c over the lane's 16 columns of one row.
__device__ __forceinline__ float dot_i8(const uint4_t pk, const ActI8& a, float s, float z) {
    uint32_t magic;
    asm("v_mov_b32 %0, 0x64646464" : "=v"(magic));   // not volatile: identical copies are merged and hoisted
    float lo = 0.0f, hi = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const half2_t q01 = as_half2(__builtin_amdgcn_perm(magic, pk[j], 0x04010400u));    // (1024 + q0, 1024 + q1)
        const half2_t q23 = as_half2(__builtin_amdgcn_perm(magic, pk[j], 0x04030402u));
        lo = __builtin_amdgcn_fdot2(q01, a.p[2 * j], lo, false);
        hi = __builtin_amdgcn_fdot2(q23, a.p[2 * j + 1], hi, false);
    }
    return fmaf(s, (lo + hi) - a.k1, z * a.sx);
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

// Pointers into device (global) memory, typed as such: after the register pin below the compiler can no
// longer infer the address space by itself and would fall back to generic (flat) loads.
#define MOEMIX_GLOBAL __attribute__((address_space(1)))
typedef const char MOEMIX_GLOBAL* gptr_t;

// Pins a uniform pointer in a scalar register pair at this point.  Without it the loop optimizer turns
// "row base + lane offset" into per-lane 64-bit pointer recurrences, one vector register pair per load.
__device__ __forceinline__ gptr_t scalar_ptr(const void* p) {
    gptr_t g = (gptr_t)p;
    asm volatile("" : "+s"(g));
    return g;
}

// Uniform base pointer + 32-bit per-lane byte offset: compiles to the scalar-base addressing form, so a
// whole set of loads shares one offset register instead of one 64-bit address register pair each.
__device__ __forceinline__ gptr_t at(gptr_t uniform_base, uint32_t lane_offset_bytes) {
    return uniform_base + lane_offset_bytes;
}

__device__ __forceinline__ uint4_t load_stream(gptr_t p) {
    return __builtin_nontemporal_load((const uint4_t MOEMIX_GLOBAL*)p);
}

__device__ __forceinline__ half_t load_half(gptr_t p) { return *(const half_t MOEMIX_GLOBAL*)p; }

// Index of the wavefront inside its workgroup, as a scalar (the compiler cannot see that
// threadIdx.x >> 6 is the same for all 64 lanes).
__device__ __forceinline__ uint32_t wave_index() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

// ---------------------------------------------------------------- up-projection

// Rows of all routed slots are laid end to end, weighted by their stored bytes (9 units per 4-bit row
// pair, 17 per 8-bit one, 32 per 16-bit one), and cut into equal shares, one per wavefront: every wavefront
// streams the same number of bytes whatever the precision mix.
__device__ __forceinline__ uint32_t row_units(int prec) {
    return prec == MOE_PREC_INT4G64 ? 9u : (prec == MOE_PREC_INT8G64 ? 17u : 32u);
}
constexpr int kUpRowsI4 = 2;                    // rows per register buffer of the 4-bit path
constexpr int kUpBufsI4 = 2;                    // register buffers in the ring of the 4-bit path
constexpr uint32_t kMinUnitsPerWave = 100;      // cost units (9 per 4-bit row, 32 per 16-bit row) below which a share is too short

// ROUTE: the gating network (with the RMSNorm of the chained configuration) runs inside this launch.  A separate
// gating launch is a chain of latencies (token -> logits -> reduction -> top-k -> launch boundary) during which
// device memory sits idle; here every workgroup evaluates the gating network for the one token by itself, from
// the 64 KB gate matrix that all of them read out of L2, and goes straight on to its share of the weights.
// Workgroup 0 also writes the routing result for the down-projection launch and for the caller.
// WIDE: the block holds 8-bit experts as well; blocks without them get a kernel without that branch (the code the
// compiler makes for the other two precisions is then exactly what it is without the third).
template <int NCH, bool ROUTE, bool WIDE>   // NCH = d_model / 2048
__global__ __launch_bounds__(256, 2) void decode_up_kernel(DevExperts ex, const int32_t* __restrict__ idx,
                                                         const half_t* __restrict__ x, int f, int k,
                                                         half_t* __restrict__ h, int32_t* status, const GateArgs ga) {
    constexpr int d = NCH * 2048;
    const int lane = threadIdx.x & 63;
    __shared__ __align__(16) half_t xs[ROUTE ? d : 8];      // block input (after the RMSNorm, if any)
    __shared__ float logit_s[MOE_MAX_EXPERTS];
    // the routed experts, 5 bits per slot (k <= 8 slots, E <= 32 experts), uniform
    uint64_t routed = 0;
    if (ROUTE) {
        // nothing of this launch raises status bits (the down-projection launch reports experts that cannot run),
        // so the word can be cleared here without a race
        if (blockIdx.x == 0 && threadIdx.x == 0) *status = 0;
        uint4_t xv[4 * NCH];
        gate_load_row<4 * NCH>(x, d, lane, xv);
        if (ga.rms_gain) gate_rmsnorm<4 * NCH>(xv, ga.rms_gain, d, ga.eps, lane);
        if (wave_index() == 0) {
#pragma unroll
            for (int j = 0; j < 4 * NCH; ++j) *(uint4_t*)(xs + (lane + 64 * j) * 8) = xv[j];
        }
        for (int e = wave_index(); e < ga.E; e += 4) {
            const float l = gate_logit<4 * NCH>(xv, ga.wg + (size_t)e * d, d, lane);
            if (lane == 0) logit_s[e] = l + (ga.bias ? ga.bias[e] : 0.0f);
        }
        __syncthreads();
        int sel[MOE_MAX_TOPK];
        float lsel[MOE_MAX_TOPK];
        gate_select(logit_s, ga.E, k, sel, lsel);
#pragma unroll
        for (int s = 0; s < MOE_MAX_TOPK; ++s)
            if (s < k) routed |= (uint64_t)(uint32_t)sel[s] << (5 * s);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            float g[MOE_MAX_TOPK];
            gate_weights(lsel, k, g);
#pragma unroll
            for (int s = 0; s < MOE_MAX_TOPK; ++s) {
                if (s < k) {
                    ga.idx_ws[s] = sel[s];
                    ga.gate_ws[s] = g[s];
                    if (ga.idx_out) ga.idx_out[s] = sel[s];
                    if (ga.gate_out) ga.gate_out[s] = g[s];
                }
            }
        }
    } else {
        for (int s = 0; s < k; ++s) routed |= (uint64_t)(uint32_t)idx[s] << (5 * s);
    }
    routed = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(routed >> 32)) << 32) |
             (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)routed);
    auto expert_of = [&](int s) { return (int)((routed >> (5 * s)) & 31u); };
    const half_t* xin = ROUTE ? xs : x;
    // 32-bit arithmetic throughout: total <= 8 slots * 16384 rows * 32 units
    // the wavefront index goes through a scalar register: everything derived from it (row ranges, row base
    // addresses) is then uniform, and the loads below take the scalar-base + 32-bit lane-offset form
    uint32_t total = 0;
    for (int s = 0; s < k; ++s) total += (uint32_t)f * (WIDE ? row_units(ex.e[expert_of(s)].prec) : (ex.e[expert_of(s)].prec == MOE_PREC_INT4G64 ? 9u : 32u));
    // A wavefront needs a dozen rows or so for its load pipeline to reach a steady state.  When the routed
    // experts are small (all 4-bit), half the workgroups take all the work and the others leave at once: the
    // launch shape is fixed on the host before the routing result exists, the work is only known here.
    const uint32_t blocks = (gridDim.x >= 2 && total / (gridDim.x * 4) < kMinUnitsPerWave) ? gridDim.x / 2 : gridDim.x;
    if (blockIdx.x >= blocks) return;
    const uint32_t n_waves = blocks * 4, gw = blockIdx.x * 4 + wave_index();
    // balanced cut: the first (total % n_waves) wavefronts take one unit more
    const uint32_t share = total / n_waves, extra = total % n_waves;
    const uint32_t lo = gw * share + (gw < extra ? gw : extra);
    const uint32_t hi = lo + share + (gw < extra ? 1u : 0u);
    uint32_t base = 0;
    for (int s = 0; s < k; ++s) {
        const DevExpert& ee = ex.e[expert_of(s)];
        const bool int4 = ee.prec == MOE_PREC_INT4G64, int8 = WIDE && ee.prec == MOE_PREC_INT8G64;
        const uint32_t cost = WIDE ? row_units(ee.prec) : (int4 ? 9u : 32u), span = (uint32_t)f * cost;
        // rows whose first cost unit falls in [lo, hi): ceil((lo - base) / cost) .. ceil((hi - base) / cost)
        const uint32_t l = lo > base ? (lo - base < span ? lo - base : span) : 0u;
        const uint32_t u = hi > base ? (hi - base < span ? hi - base : span) : 0u;
        // (the divisions run on the vector unit; move the uniform results back to scalar registers)
        const int r0 = __builtin_amdgcn_readfirstlane(
            (int)(WIDE ? (l + cost - 1u) / cost : (int4 ? (l + 8u) / 9u : (l + 31u) / 32u)));
        const int r1 = __builtin_amdgcn_readfirstlane(
            (int)(WIDE ? (u + cost - 1u) / cost : (int4 ? (u + 8u) / 9u : (u + 31u) / 32u)));
        base += span;
        // an expert that cannot run is left out here and reported by the down-projection launch
        if (r0 >= r1 || ee.resident != 1 || !ee.w1.data) continue;
        half_t* hs = h + (size_t)s * f;
        if (int4) {
            ActI4 act[NCH];
            constexpr int gpr = d / 64;
            constexpr int RB = kUpRowsI4;
            const uint32_t lane_q = lane * 16;   // byte offset of the lane's codes inside a 1 KB piece of a row
            // Scales and zeros.  Read as 2-byte (or even 256-byte) pieces per row they cost more device-memory time
            // than the codes: four extra streams of small scattered requests, measured to cap the kernel at 4.4 TB/s
            // (6.3 TB/s with the same loads served from cache).  The rows of a matrix lie end to end, so the wavefront
            // fetches them for G rows at a time as ONE 1 KB run per array (a 128-bit load per lane, like the codes),
            // parks the run in a wavefront-private LDS region and picks its 2-byte values from there.  The run of group
            // g is written when group g starts (the wavefront's LDS accesses stay in program order, so group g-1 has
            // been read by then) and the run of group g+1 is requested at the same moment.
            constexpr int DPR = 16 * NCH;                        // dwords of scales per row
            constexpr int G = ((256 / DPR) / RB) * RB;           // rows per group (8 at d = 4096)
            __shared__ __align__(16) uint8_t sz_lds[4][4][1024];      // [wavefront][array][run]
            uint8_t* const my_lds = &sz_lds[wave_index()][0][0];
            const gptr_t szm[4] = {scalar_ptr(ee.w1.scale), scalar_ptr(ee.w1.zero), scalar_ptr(ee.w3.scale),
                                   scalar_ptr(ee.w3.zero)};
            uint4_t sg[4];                                       // the run on its way to LDS
            auto load_group = [&](int rg) {
                int i = (4 * lane) / DPR;                        // the lane's four dwords belong to row rg + i
                i = i < G ? i : G - 1;
                const int row = (rg + i < r1) ? rg + i : r1 - 1; // rows past the end repeat the last one
                const uint32_t off = (uint32_t)row * (gpr * 2) + (uint32_t)((4 * lane) % DPR) * 4;
#pragma unroll
                for (int a = 0; a < 4; ++a) sg[a] = load_stream(at(szm[a], off));
            };
            auto publish_group = [&]() {
                wave_lds_handover();   // the previous run has been read by every lane
#pragma unroll
                for (int a = 0; a < 4; ++a) *(uint4_t*)(my_lds + a * 1024 + lane * 16) = sg[a];
                wave_lds_handover();
            };
            struct Rows {
                uint4_t pk1[RB][NCH], pk3[RB][NCH];
            };
            // RB rows starting at r; rows past the end repeat the last one (loaded, never stored)
            auto load_rows = [&](Rows& B, int r) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int row = (r + i < r1) ? r + i : r1 - 1;
                    const gptr_t q1 = scalar_ptr(ee.w1.data + (size_t)row * (d / 2));      // uniform row bases
                    const gptr_t q3 = scalar_ptr(ee.w3.data + (size_t)row * (d / 2));
#pragma unroll
                    for (int c = 0; c < NCH; ++c) {
                        B.pk1[i][c] = load_stream(at(q1, lane_q + c * 1024));
                        B.pk3[i][c] = load_stream(at(q3, lane_q + c * 1024));
                    }
                }
            };
            // scale or zero (array a) of row `in_group` of the current group, chunk c, for this lane's group of
            // columns 32 c + lane / 2
            const int lane_half = (lane >> 1) * 2;
            auto pick = [&](int a, int in_group, int c) {
                return (float)*(const half_t*)(my_lds + a * 1024 + (in_group * DPR + 16 * c) * 4 + lane_half);
            };
            auto compute_rows = [&](const Rows& B, int r) {
                const int in_group = (r - r0) % G;
                float am = 0.0f, bm = 0.0f;   // lane i keeps the totals of row r + i
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    float a = 0.0f, b = 0.0f;
#pragma unroll
                    for (int c = 0; c < NCH; ++c) {
                        a += dot_i4(B.pk1[i][c], act[c], pick(0, in_group + i, c), pick(1, in_group + i, c));
                        b += dot_i4(B.pk3[i][c], act[c], pick(2, in_group + i, c), pick(3, in_group + i, c));
                    }
                    a = wave_total(a);
                    b = wave_total(b);
                    am = lane == i ? a : am;
                    bm = lane == i ? b : bm;
                }
                if (lane < RB && r + lane < r1) hs[r + lane] = (half_t)silu_mul(am, bm);
            };
            // a ring of NB register buffers: NB - 1 sets of rows are in flight while one is used (a set of 4-bit
            // rows is used up in well under a microsecond, less than a trip to device memory under load)
            constexpr int NB = kUpBufsI4;
            Rows buf[NB];
#pragma unroll
            for (int j = 0; j < NB - 1; ++j)
                if (r0 + j * RB < r1) load_rows(buf[j], r0 + j * RB);
            load_group(r0);
            __builtin_amdgcn_sched_barrier(0);
            // the first weight rows are requested before the token: they come from HBM, the token from L2
#pragma unroll
            for (int c = 0; c < NCH; ++c) load_act_i4(xin + c * 2048 + lane * 32, act[c]);
            publish_group();
            load_group(r0 + G);
            __builtin_amdgcn_sched_barrier(0);
            for (int r = r0; r < r1; r += NB * RB) {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int rj = r + j * RB;
                    if (rj < r1) {
                        if (rj > r0 && (rj - r0) % G == 0) {     // a new group starts: its run goes to LDS, the next is requested
                            publish_group();
                            load_group(rj + G);
                        }
                        if (r + (j + NB - 1) * RB < r1) load_rows(buf[(j + NB - 1) % NB], r + (j + NB - 1) * RB);
                        __builtin_amdgcn_sched_barrier(0);
                        compute_rows(buf[j], rj);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        } else if (WIDE && int8) {
            // 8-bit rows: one register buffer = one row of w1 and one of w3 (2 x d bytes), two buffers; scales and
            // zeros travel as in the 4-bit path, as 1 KB runs of G rows through a wavefront-private LDS region.
            constexpr int NL8 = d / 1024;                        // 128-bit loads per row
            constexpr int gpr = d / 64;
            constexpr int DPR = 16 * NCH;                        // dwords of scales per row
            constexpr int G = ((256 / DPR) / 2) * 2;             // rows per run (8 at d = 4096), even
            ActI8 act[NL8];
            __shared__ __align__(16) uint8_t sz8_lds[4][4][1024];     // [wavefront][array][run]
            uint8_t* const my_lds = &sz8_lds[wave_index()][0][0];
            const gptr_t szm[4] = {scalar_ptr(ee.w1.scale), scalar_ptr(ee.w1.zero), scalar_ptr(ee.w3.scale),
                                   scalar_ptr(ee.w3.zero)};
            uint4_t sg[4];                                       // the run on its way to LDS
            auto load_group = [&](int rg) {
                int i = (4 * lane) / DPR;                        // the lane's four dwords belong to row rg + i
                i = i < G ? i : G - 1;
                const int row = (rg + i < r1) ? rg + i : r1 - 1; // rows past the end repeat the last one
                const uint32_t off = (uint32_t)row * (gpr * 2) + (uint32_t)((4 * lane) % DPR) * 4;
#pragma unroll
                for (int a = 0; a < 4; ++a) sg[a] = load_stream(at(szm[a], off));
            };
            auto publish_group = [&]() {
                wave_lds_handover();   // the previous run has been read by every lane
#pragma unroll
                for (int a = 0; a < 4; ++a) *(uint4_t*)(my_lds + a * 1024 + lane * 16) = sg[a];
                wave_lds_handover();
            };
            // scale or zero (array a) of row `in_group` of the current run for this lane's group of 64 columns in
            // chunk c: half 16 c + lane / 4 of the row
            const int lane_grp = (lane >> 2) * 2;
            auto pick = [&](int a, int in_group, int c) {
                return (float)*(const half_t*)(my_lds + a * 1024 + (in_group * DPR) * 4 + 32 * c + lane_grp);
            };
            struct Row8 {
                uint4_t v1[NL8], v3[NL8];
            };
            const uint32_t lane_q = lane * 16;
            auto load_row = [&](Row8& B, int r) {
                const int row = r < r1 ? r : r1 - 1;             // a row past the end repeats the last one (never stored)
                const gptr_t q1 = scalar_ptr(ee.w1.data + (size_t)row * d);      // uniform row bases
                const gptr_t q3 = scalar_ptr(ee.w3.data + (size_t)row * d);
#pragma unroll
                for (int c = 0; c < NL8; ++c) {
                    B.v1[c] = load_stream(at(q1, lane_q + c * 1024));
                    B.v3[c] = load_stream(at(q3, lane_q + c * 1024));
                }
            };
            auto compute_row = [&](const Row8& B, int r) {
                const int in_group = (r - r0) % G;
                float a = 0.0f, b = 0.0f;
#pragma unroll
                for (int c = 0; c < NL8; ++c) {
                    a += dot_i8(B.v1[c], act[c], pick(0, in_group, c), pick(1, in_group, c));
                    b += dot_i8(B.v3[c], act[c], pick(2, in_group, c), pick(3, in_group, c));
                }
                a = wave_total(a);
                b = wave_total(b);
                if (lane == 0 && r < r1) hs[r] = (half_t)silu_mul(a, b);
            };
            Row8 A, B;
            load_row(A, r0);
            load_group(r0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < NL8; ++c) load_act_i8(xin + c * 1024 + lane * 16, act[c]);
            publish_group();
            load_group(r0 + G);
            __builtin_amdgcn_sched_barrier(0);
            for (int r = r0; r < r1; r += 2) {
                if (r > r0 && (r - r0) % G == 0) {               // a new run starts: it goes to LDS, the next is requested
                    publish_group();
                    load_group(r + G);
                }
                load_row(B, r + 1);
                __builtin_amdgcn_sched_barrier(0);
                compute_row(A, r);
                __builtin_amdgcn_sched_barrier(0);
                if (r + 2 < r1) load_row(A, r + 2);
                __builtin_amdgcn_sched_barrier(0);
                compute_row(B, r + 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            constexpr int NL = d / 512;   // 128-bit loads per row
            ActF16 act[NL];
            const uint8_t* w1 = ee.w1.data;
            const uint8_t* w3 = ee.w3.data;
            const uint32_t lane_w = lane * 16;
            // one register buffer = one matrix row (w1 and w3 rows alternate between the two buffers)
            struct Row {
                uint4_t v[NL];
            };
            auto load_row = [&](Row& B, const uint8_t* w, int r) {
                const gptr_t rowp = scalar_ptr(w + (size_t)r * (d * 2));   // uniform row base
#pragma unroll
                for (int c = 0; c < NL; ++c) B.v[c] = load_stream(at(rowp, lane_w + c * 1024));
            };
            auto dot_row = [&](const Row& B) {
                float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
                for (int c = 0; c < NL; c += 2) {
                    a0 = dot_f16(B.v[c], act[c], a0);
                    a1 = dot_f16(B.v[c + 1], act[c + 1], a1);
                }
                return wave_total(a0 + a1);
            };
            Row A, B;
            load_row(A, w1, r0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < NL; ++c) load_act_f16(xin + c * 512 + lane * 8, act[c]);
            for (int r = r0; r < r1; ++r) {
                load_row(B, w3, r);
                __builtin_amdgcn_sched_barrier(0);
                const float a = dot_row(A);
                __builtin_amdgcn_sched_barrier(0);
                if (r + 1 < r1) load_row(A, w1, r + 1);
                __builtin_amdgcn_sched_barrier(0);
                const float b = dot_row(B);
                if (lane == 0) hs[r] = (half_t)silu_mul(a, b);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

// ---------------------------------------------------------------- down-projection + weighted average

// One workgroup per kDownRows output rows; wavefront w owns columns [2048 w, 2048 w + 2048) of every row,
// for every slot in turn, with that slice of the slot's hidden row in registers.  Rows go through two
// register buffers of kDownBatch rows, so the next batch is in flight while the current one is used.
// Partial sums meet in LDS and are added in wavefront order: the result does not depend on scheduling.
constexpr int kDownRows = 16;
constexpr int kDownBatch = 4;

template <bool WIDE>   // WIDE: with the branch for 8-bit experts
__global__ __launch_bounds__(512) void decode_down_kernel(DevExperts ex, const int32_t* __restrict__ idx,
                                                           const float* __restrict__ gate,
                                                           const half_t* __restrict__ h, int d, int f, int k,
                                                           const half_t* __restrict__ residual,
                                                           half_t* __restrict__ out, float* __restrict__ out32,
                                                           int32_t* status) {
    __shared__ float part[8][kDownRows];
    const int lane = threadIdx.x & 63, n_waves = blockDim.x >> 6;
    const uint32_t wave = wave_index();
    const int row0 = blockIdx.x * kDownRows;
    float acc[kDownRows];
#pragma unroll
    for (int r = 0; r < kDownRows; ++r) acc[r] = 0.0f;
    for (int s = 0; s < k; ++s) {
        const DevExpert& ee = ex.e[idx[s]];
        if (ee.resident == kDeferred) continue;
        if (!ee.resident || !ee.w2.data) {
            if (threadIdx.x == 0 && blockIdx.x == 0) atomicOr(status, kStatusNotResident);
            continue;
        }
        const float g = gate[s];
        const half_t* hs = h + (size_t)s * f + wave * 2048;
        if (ee.prec == MOE_PREC_INT4G64) {
            ActI4 act;
            load_act_i4(hs + lane * 32, act);
            const size_t gpr = f >> 6, qpr = f >> 1;
            const uint8_t* q = ee.w2.data + (size_t)row0 * qpr + wave * 1024;        // uniform
            const half_t* sc = ee.w2.scale + (size_t)row0 * gpr + wave * 32;
            const half_t* zr = ee.w2.zero + (size_t)row0 * gpr + wave * 32;
            const uint32_t lane_q = lane * 16, lane_g = (lane >> 1) * 2;
            struct Batch {
                uint4_t pk[kDownBatch];
                half_t sv[kDownBatch], zv[kDownBatch];
            };
            auto load_batch = [&](Batch& B, int rb) {
#pragma unroll
                for (int r = 0; r < kDownBatch; ++r) {
                    B.pk[r] = load_stream(at(scalar_ptr(q + (size_t)(rb + r) * qpr), lane_q));
                    B.sv[r] = load_half(at(scalar_ptr(sc + (size_t)(rb + r) * gpr), lane_g));
                    B.zv[r] = load_half(at(scalar_ptr(zr + (size_t)(rb + r) * gpr), lane_g));
                }
            };
            Batch A, B;
            load_batch(A, 0);
#pragma unroll
            for (int rb = 0; rb < kDownRows; rb += 2 * kDownBatch) {
                load_batch(B, rb + kDownBatch);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < kDownBatch; ++r)
                    acc[rb + r] = fmaf(g, dot_i4(A.pk[r], act, (float)A.sv[r], (float)A.zv[r]), acc[rb + r]);
                __builtin_amdgcn_sched_barrier(0);
                if (rb + 2 * kDownBatch < kDownRows) load_batch(A, rb + 2 * kDownBatch);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < kDownBatch; ++r)
                    acc[rb + kDownBatch + r] =
                        fmaf(g, dot_i4(B.pk[r], act, (float)B.sv[r], (float)B.zv[r]), acc[rb + kDownBatch + r]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if (WIDE && ee.prec == MOE_PREC_INT8G64) {
            // 8-bit rows: the wavefront's 2048 columns are two 128-bit loads per lane and row
            ActI8 act[2];
#pragma unroll
            for (int c = 0; c < 2; ++c) load_act_i8(hs + c * 1024 + lane * 16, act[c]);
            const size_t gpr = f >> 6;
            const uint8_t* q = ee.w2.data + (size_t)row0 * f + wave * 2048;           // uniform
            const half_t* sc = ee.w2.scale + (size_t)row0 * gpr + wave * 32;
            const half_t* zr = ee.w2.zero + (size_t)row0 * gpr + wave * 32;
            const uint32_t lane_q = lane * 16, lane_g = (lane >> 2) * 2;
            struct Batch {
                uint4_t pk[kDownBatch][2];
                half_t sv[kDownBatch][2], zv[kDownBatch][2];
            };
            auto load_batch = [&](Batch& B, int rb) {
#pragma unroll
                for (int r = 0; r < kDownBatch; ++r) {
                    const gptr_t qr = scalar_ptr(q + (size_t)(rb + r) * f);
                    const gptr_t sr = scalar_ptr(sc + (size_t)(rb + r) * gpr), zq = scalar_ptr(zr + (size_t)(rb + r) * gpr);
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        B.pk[r][c] = load_stream(at(qr, lane_q + c * 1024));
                        B.sv[r][c] = load_half(at(sr, lane_g + c * 32));
                        B.zv[r][c] = load_half(at(zq, lane_g + c * 32));
                    }
                }
            };
            auto use_batch = [&](const Batch& B, int rb) {
#pragma unroll
                for (int r = 0; r < kDownBatch; ++r) {
                    const float p = dot_i8(B.pk[r][0], act[0], (float)B.sv[r][0], (float)B.zv[r][0]) +
                                    dot_i8(B.pk[r][1], act[1], (float)B.sv[r][1], (float)B.zv[r][1]);
                    acc[rb + r] = fmaf(g, p, acc[rb + r]);
                }
            };
            Batch A, B;
            load_batch(A, 0);
#pragma unroll
            for (int rb = 0; rb < kDownRows; rb += 2 * kDownBatch) {
                load_batch(B, rb + kDownBatch);
                __builtin_amdgcn_sched_barrier(0);
                use_batch(A, rb);
                __builtin_amdgcn_sched_barrier(0);
                if (rb + 2 * kDownBatch < kDownRows) load_batch(A, rb + 2 * kDownBatch);
                __builtin_amdgcn_sched_barrier(0);
                use_batch(B, rb + kDownBatch);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            ActF16 act[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) load_act_f16(hs + c * 512 + lane * 8, act[c]);
            const uint8_t* w = ee.w2.data + ((size_t)row0 * f + wave * 2048) * 2;       // uniform
            const uint32_t lane_w = lane * 16;
            struct Batch {
                uint4_t v[2][4];     // two rows, four 128-bit loads each
            };
            auto load_batch = [&](Batch& B, int rb) {
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const gptr_t rowp = scalar_ptr(w + (size_t)(rb + r) * f * 2);
#pragma unroll
                    for (int c = 0; c < 4; ++c) B.v[r][c] = load_stream(at(rowp, lane_w + c * 1024));
                }
            };
            auto use_batch = [&](const Batch& B, int rb) {
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    float p0 = 0.0f, p1 = 0.0f;
                    p0 = dot_f16(B.v[r][0], act[0], p0);
                    p1 = dot_f16(B.v[r][1], act[1], p1);
                    p0 = dot_f16(B.v[r][2], act[2], p0);
                    p1 = dot_f16(B.v[r][3], act[3], p1);
                    acc[rb + r] = fmaf(g, p0 + p1, acc[rb + r]);
                }
            };
            Batch A, B;
            load_batch(A, 0);
#pragma unroll
            for (int rb = 0; rb < kDownRows; rb += 4) {
                load_batch(B, rb + 2);
                __builtin_amdgcn_sched_barrier(0);
                use_batch(A, rb);
                __builtin_amdgcn_sched_barrier(0);
                if (rb + 4 < kDownRows) load_batch(A, rb + 4);
                __builtin_amdgcn_sched_barrier(0);
                use_batch(B, rb + 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    float mine = 0.0f;    // lane r keeps the total of row r
#pragma unroll
    for (int r = 0; r < kDownRows; ++r) {
        const float t = wave_total(acc[r]);
        mine = lane == r ? t : mine;
    }
    if (lane < kDownRows) part[wave][lane] = mine;
    __syncthreads();
    if (threadIdx.x < kDownRows) {
        const int row = row0 + threadIdx.x;
        float t = residual ? (float)residual[row] : 0.0f;
        float sum = 0.0f;
        for (int w = 0; w < n_waves; ++w) sum += part[w][threadIdx.x];
        if (out32) out32[row] = t + sum;      // one expert alone: the unrounded result
        else out[row] = (half_t)(t + sum);
    }
}

// Routing result "this one expert with weight 1", for a single expert run through the batch-1 kernels.
__global__ void single_route_kernel(int32_t* idx, float* gate, int expert) {
    idx[0] = expert;
    gate[0] = 1.0f;
}

}  // namespace

bool decode_shape_ok(int d, int f) { return d % 2048 == 0 && d <= 8192 && f % 2048 == 0 && f <= 16384 && d % kDownRows == 0; }

static bool any_int8(const DevExperts& ex) {
    for (int e = 0; e < MOE_MAX_EXPERTS; ++e)
        if (ex.e[e].prec == MOE_PREC_INT8G64 && ex.e[e].w1.data) return true;
    return false;
}

template <bool ROUTE, bool WIDE>
static void launch_up(const DevExperts& ex, const int32_t* idx, const half_t* x, int d, int f, int k, half_t* h,
                      int32_t* status, int blocks, const GateArgs& ga, hipStream_t st) {
    switch (d / 2048) {
        case 1: decode_up_kernel<1, ROUTE, WIDE><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status, ga); break;
        case 2: decode_up_kernel<2, ROUTE, WIDE><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status, ga); break;
        case 3: decode_up_kernel<3, ROUTE, WIDE><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status, ga); break;
        default: decode_up_kernel<4, ROUTE, WIDE><<<blocks, 256, 0, st>>>(ex, idx, x, f, k, h, status, ga); break;
    }
}

void launch_decode_up(const DevExperts& ex, const int32_t* idx, const half_t* x, int d, int f, int k, half_t* h,
                      int32_t* status, int blocks, hipStream_t st, const GateArgs* gating) {
    TraceScope trace(kKernelUp, st);
    const bool wide = any_int8(ex);
    if (gating) {
        if (wide) launch_up<true, true>(ex, idx, x, d, f, k, h, status, blocks, *gating, st);
        else launch_up<true, false>(ex, idx, x, d, f, k, h, status, blocks, *gating, st);
    } else {
        if (wide) launch_up<false, true>(ex, idx, x, d, f, k, h, status, blocks, GateArgs{}, st);
        else launch_up<false, false>(ex, idx, x, d, f, k, h, status, blocks, GateArgs{}, st);
    }
}

void launch_decode_down(const DevExperts& ex, const int32_t* idx, const float* gate, const half_t* h, int d, int f,
                        int k, const half_t* residual, half_t* out, int32_t* status, hipStream_t st, float* out32) {
    TraceScope trace(kKernelDown, st);
    if (any_int8(ex))
        decode_down_kernel<true><<<d / kDownRows, (f / 2048) * 64, 0, st>>>(ex, idx, gate, h, d, f, k, residual, out, out32, status);
    else
        decode_down_kernel<false><<<d / kDownRows, (f / 2048) * 64, 0, st>>>(ex, idx, gate, h, d, f, k, residual, out, out32, status);
}

void launch_single_route(int32_t* idx, float* gate, int expert, hipStream_t st) {
    single_route_kernel<<<1, 1, 0, st>>>(idx, gate, expert);
}

}  // namespace moemix
