/*
 * Host side of the seeded synthetic-input generator (stand-in for trained
 * Mixtral weights and real activations, which the paper's evaluation, §4.1,
 * takes from a checkpoint and from text corpora).
 *
 * This file holds no arithmetic of the MoE method: it only turns
 * (seed, stream, element index) into an fp16 bit pattern.  The device-side
 * fill kernel implements the same counter-based recipe so that a tensor can
 * be produced on either side and be bit-identical.
 *
 * Recipe (element i of stream `stream` under `seed`):
 *   key   = mix64(mix64(seed) + stream)
 *   h0,h1 = mix64(key + 2i), mix64(key + 2i + 1)          (splitmix64 finalizer)
 *   normal : S = sum of the eight 16-bit fields of h0,h1;  c = 2S - 8*65535
 *            value = fp16_rne( (float)c * scale )          (one fp32 multiply)
 *            with scale = sigma / sqrt((8/3)*(65536^2-1)) rounded to fp32 by
 *            the caller, so the stream has variance sigma^2 and is cut at
 *            about +-4.9 sigma (sum of eight uniforms).
 *   uniform: c = 2*(h0 >> 40) - (2^24 - 1);  value = fp16_rne( (float)c * scale )
 *            with scale = a / 2^24 for U(-a, a).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* fp32 -> fp16 bits, round to nearest even, written out by hand so the file
 * needs no compiler half type. */
static inline uint16_t f32_to_f16_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t absu = u & 0x7FFFFFFFu;
    if (absu >= 0x7F800000u) {                       /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((absu > 0x7F800000u) ? 0x200u : 0u));
    }
    if (absu >= 0x477FF000u) {                       /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7C00u);
    }
    if (absu < 0x33000001u) {                        /* <= 2^-25 rounds to zero */
        return (uint16_t)sign;
    }
    int32_t e = (int32_t)(absu >> 23) - 127;
    uint32_t m = (absu & 0x7FFFFFu) | 0x800000u;     /* 24-bit significand */
    int shift;
    uint32_t base;
    if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; m &= 0x7FFFFFu; }
    else          { shift = 13 + (-14 - e); base = 0; }
    uint32_t q = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (q & 1u))) q += 1u;
    return (uint16_t)(sign | (base + q));            /* carry into exponent is correct */
}

uint64_t synth_key(uint64_t seed, uint64_t stream) {
    return mix64(mix64(seed) + stream);
}

void synth_fill_normal_f16(uint16_t* dst, size_t n, size_t first, uint64_t seed,
                           uint64_t stream, float scale) {
    const uint64_t key = synth_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (ptrdiff_t j = 0; j < (ptrdiff_t)n; ++j) {
        uint64_t i = (uint64_t)first + (uint64_t)j;
        uint64_t h0 = mix64(key + 2 * i), h1 = mix64(key + 2 * i + 1);
        uint32_t s = 0;
        for (int b = 0; b < 4; ++b) {
            s += (uint32_t)((h0 >> (16 * b)) & 0xFFFFu);
            s += (uint32_t)((h1 >> (16 * b)) & 0xFFFFu);
        }
        int32_t c = 2 * (int32_t)s - 8 * 65535;
        dst[j] = f32_to_f16_bits((float)c * scale);
    }
}

void synth_fill_uniform_f16(uint16_t* dst, size_t n, size_t first, uint64_t seed,
                            uint64_t stream, float scale) {
    const uint64_t key = synth_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (ptrdiff_t j = 0; j < (ptrdiff_t)n; ++j) {
        uint64_t i = (uint64_t)first + (uint64_t)j;
        uint64_t h0 = mix64(key + 2 * i);
        int32_t c = 2 * (int32_t)(h0 >> 40) - ((1 << 24) - 1);
        dst[j] = f32_to_f16_bits((float)c * scale);
    }
}
