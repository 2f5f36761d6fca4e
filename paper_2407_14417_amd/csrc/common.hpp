// Shared device/host declarations of the moemix HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/moemix.h"

namespace moemix {

constexpr int kWave = 64;
constexpr int kGroup = MOE_GROUP;

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

// Device-side copy of the expert table, passed by value as a kernel argument (2.5 KB).
struct DevMat {
    const uint8_t* data;
    const half_t* scale;
    const half_t* zero;
};
// `resident` of a device-side table entry: 0 = not in device memory (a launch that meets it raises the status
// bit and leaves its contribution out), 1 = run it, kDeferred = another launch of the same call runs it (no work,
// no status bit, nothing written for its rows).
constexpr int32_t kDeferred = 2;
struct DevExpert {
    int32_t prec;
    int32_t resident;
    DevMat w1, w3, w2;
};
struct DevExperts {
    DevExpert e[MOE_MAX_EXPERTS];
};

// Status word bits, set by kernels with atomicOr (bit index = -moe_status).
constexpr int kStatusBadIndex = 1 << 1;
constexpr int kStatusNotResident = 1 << 3;

// Workspace layout, computed identically by moe_workspace_bytes and the entry points.
struct Workspace {
    int32_t* status;    // [64] first word is the status word
    int32_t* idx;       // [T, k]
    float* gate;        // [T, k]
    int32_t* counts;    // [E]
    int32_t* offsets;   // [E + 1]
    int32_t* perm;      // [T * k]   grouped row -> flat pair
    int32_t* inv;       // [T * k]   flat pair -> grouped row (-1: dropped)
    int32_t* tiles;     // [kMaxTiles * 4] work list of the grouped matrix kernels (+ counter)
    half_t* xn;         // [T, d]    normed input of the chain
    half_t* h;          // [T * k, f]  SwiGLU hidden rows, grouped order
    float* y;           // [y_splits][T * k, d]  expert outputs, grouped order, one partial per contraction split
    int y_splits;
    size_t bytes;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline Workspace carve_workspace(void* base, int T, int d, int f, int E, int k, int y_splits = 1) {
    Workspace w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* p = base ? (char*)base + off : nullptr;
        off += align_up(bytes, 256);
        return (void*)p;
    };
    const size_t P = (size_t)T * k;
    w.status = (int32_t*)take(64 * sizeof(int32_t));
    w.idx = (int32_t*)take(P * sizeof(int32_t));
    w.gate = (float*)take(P * sizeof(float));
    w.counts = (int32_t*)take((size_t)E * sizeof(int32_t));
    w.offsets = (int32_t*)take((size_t)(E + 1) * sizeof(int32_t));
    w.perm = (int32_t*)take(P * sizeof(int32_t));
    w.inv = (int32_t*)take(P * sizeof(int32_t));
    w.tiles = (int32_t*)take(256);
    w.xn = (half_t*)take((size_t)T * d * sizeof(half_t));
    w.h = (half_t*)take(P * f * sizeof(half_t));
    w.y = (float*)take((size_t)y_splits * P * d * sizeof(float));
    w.y_splits = y_splits;
    w.bytes = off;
    return w;
}

// ---------------------------------------------------------------- device helpers
#if defined(__HIPCC__)

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// ---------------------------------------------------------------- wavefront reduction on the DPP network

template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, true));
}

// Sum over the 64 lanes; the total is returned to every lane through a scalar register.
__device__ __forceinline__ float wave_total(float v) {
    v += dpp_move<0xB1>(v);          // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);          // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);         // row_half_mirror
    v += dpp_move<0x140>(v);         // row_mirror: every lane of a row of 16 holds the row sum
    v += dpp_move<0x142, 0xA>(v);    // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xC>(v);    // row_bcast31 into rows 2 and 3: lane 63 holds the total
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Lanes of one wavefront hand data to each other through a wavefront-private LDS region without a workgroup
// barrier.  This orders the wavefront's LDS writes before its later reads of what other lanes wrote (the hardware
// keeps one wavefront's LDS accesses in program order; the fences keep the compiler from reordering them and
// cost no instruction).
__device__ __forceinline__ void wave_lds_handover() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Reinterpret a 32-bit word as two halves.  The argument is taken by value on purpose: the bit-cast
// builtin applied directly to an element of a vector lvalue (v[j]) reads element 0 whatever j is.
__device__ __forceinline__ half2_t as_half2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }

__device__ __forceinline__ float silu_mul(float a, float b) { return a / (1.0f + __expf(-a)) * b; }

// Exact dequantized weight: fp16_rne( fp32(q) * fp32(s) + fp32(z) ).  q*s is exact in fp32, so
// whether the compiler fuses the multiply-add or not the fp32 sum is the same.
// fp32 -> fp16, round to nearest even, of a value that has already been rounded to fp32.  The empty
// asm keeps the compiler from folding the producing multiply/add into a mixed-precision instruction
// that would round the exact result once, straight to fp16 (different on ties).
__device__ __forceinline__ half_t f32_to_f16_rne(float v) {
    asm volatile("" : "+v"(v));
    return (half_t)v;
}

__device__ __forceinline__ half_t dequant_one(uint32_t q, float s, float z) {
    return f32_to_f16_rne((float)q * s + z);
}

#endif  // __HIPCC__

}  // namespace moemix
