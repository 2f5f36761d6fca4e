/*
 * CPU ORACLE -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Stand-alone driver that runs every entry point of the oracle once on a tiny block with heap buffers of
 * exactly the documented sizes, meant to be compiled together with the oracle under
 * -fsanitize=address,undefined (tests/test_oracle_sanitize.py): an access outside a buffer, a signed
 * overflow or a misaligned access in the oracle ends the run with a non-zero status.  Prints one checksum
 * line so that the run cannot be optimized away.
 */
#include <stdio.h>

#include "moe_oracle.c"

static uint32_t lcg_state = 12345u;
static double lcg_unit(void) { /* (-1, 1) */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((double)(lcg_state >> 8) / 8388608.0) - 1.0;
}

static uint16_t* random_halves(size_t n, double scale) {
    uint16_t* p = (uint16_t*)malloc(sizeof(uint16_t) * n);
    for (size_t i = 0; i < n; ++i) p[i] = orc_double_to_half(scale * lcg_unit());
    return p;
}

int main(void) {
    enum { D = 128, F = 192, E = 3, K = 2, T = 5 };
    uint16_t* x = random_halves((size_t)T * D, 1.0);
    uint16_t* wg = random_halves((size_t)E * D, 0.05);
    float bias[E] = {0.0f, -0.5f, 0.25f};
    orc_expert ex[E];
    uint16_t* w[E][3];
    uint8_t* q[3] = {0, 0, 0};
    uint16_t *sc[3] = {0, 0, 0}, *ze[3] = {0, 0, 0};
    for (int e = 0; e < E; ++e) {
        w[e][0] = random_halves((size_t)F * D, 0.05);
        w[e][1] = random_halves((size_t)F * D, 0.05);
        w[e][2] = random_halves((size_t)D * F, 0.05);
        ex[e].prec_int4 = 0;
        ex[e].resident = 1;
        ex[e].w1 = (orc_mat){w[e][0], NULL, NULL};
        ex[e].w3 = (orc_mat){w[e][1], NULL, NULL};
        ex[e].w2 = (orc_mat){w[e][2], NULL, NULL};
    }
    /* expert 1 becomes 4-bit */
    const int outs[3] = {F, F, D}, ins[3] = {D, D, F};
    for (int m = 0; m < 3; ++m) {
        q[m] = (uint8_t*)malloc((size_t)outs[m] * ins[m] / 2);
        sc[m] = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)outs[m] * ins[m] / ORC_GROUP);
        ze[m] = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)outs[m] * ins[m] / ORC_GROUP);
        if (orc_quantize_int4(w[1][m], outs[m], ins[m], q[m], sc[m], ze[m]) != 0) return 2;
    }
    ex[1].prec_int4 = 1;
    ex[1].w1 = (orc_mat){q[0], sc[0], ze[0]};
    ex[1].w3 = (orc_mat){q[1], sc[1], ze[1]};
    ex[1].w2 = (orc_mat){q[2], sc[2], ze[2]};

    /* expert 2 becomes 8-bit */
    uint8_t* q8[3] = {0, 0, 0};
    uint16_t *sc8[3] = {0, 0, 0}, *ze8[3] = {0, 0, 0};
    for (int m = 0; m < 3; ++m) {
        q8[m] = (uint8_t*)malloc((size_t)outs[m] * ins[m]);
        sc8[m] = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)outs[m] * ins[m] / ORC_GROUP);
        ze8[m] = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)outs[m] * ins[m] / ORC_GROUP);
        if (orc_quantize_int8(w[2][m], outs[m], ins[m], q8[m], sc8[m], ze8[m]) != 0) return 2;
    }
    ex[2].prec_int4 = 2;
    ex[2].w1 = (orc_mat){q8[0], sc8[0], ze8[0]};
    ex[2].w3 = (orc_mat){q8[1], sc8[1], ze8[1]};
    ex[2].w2 = (orc_mat){q8[2], sc8[2], ze8[2]};

    double sum = 0.0;
    uint16_t* w_hat = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)F * D);
    if (orc_dequant_int8(q8[0], sc8[0], ze8[0], F, D, w_hat) != 0) return 3;
    for (size_t i = 0; i < (size_t)F * D; ++i) sum += orc_half_to_float(w_hat[i]);
    if (orc_dequant_int4(q[0], sc[0], ze[0], F, D, w_hat) != 0) return 3;
    for (size_t i = 0; i < (size_t)F * D; ++i) sum += orc_half_to_float(w_hat[i]);

    int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * T * K);
    float* gate = (float*)malloc(sizeof(float) * T * K);
    double* logits = (double*)malloc(sizeof(double) * T * E);
    if (orc_route(x, T, D, wg, bias, E, K, idx, gate, logits) != 0) return 4;
    int32_t counts[E], offsets[E + 1];
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * T * K);
    if (orc_permute(idx, T, K, E, counts, offsets, perm) != 0) return 5;
    for (int i = 0; i < T * K; ++i) sum += idx[i] + gate[i] + perm[i];

    double* y = (double*)malloc(sizeof(double) * (size_t)T * D);
    double* h = (double*)malloc(sizeof(double) * (size_t)T * F);
    for (int e = 0; e < E; ++e) {
        if (orc_expert_ffn(ex[e].prec_int4, &ex[e].w1, &ex[e].w3, &ex[e].w2, x, T, D, F, y, h) != 0) return 6;
        for (size_t i = 0; i < (size_t)T * D; ++i) sum += y[i];
    }
    double* out = (double*)malloc(sizeof(double) * (size_t)T * D);
    if (orc_layer_forward(x, T, D, F, E, K, wg, bias, ex, out, idx, gate) != 0) return 7;
    for (size_t i = 0; i < (size_t)T * D; ++i) sum += out[i];

    uint16_t* gain = (uint16_t*)malloc(sizeof(uint16_t) * D);
    for (int i = 0; i < D; ++i) gain[i] = orc_double_to_half(1.0);
    uint16_t* normed = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * D);
    uint16_t* hh = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * D);
    memcpy(hh, x, sizeof(uint16_t) * (size_t)T * D);
    for (int l = 0; l < 2; ++l)
        if (orc_chain_layer(hh, T, D, F, E, K, gain, 1e-5, wg, NULL, ex, idx, gate, normed) != 0) return 8;
    for (size_t i = 0; i < (size_t)T * D; ++i) sum += orc_half_to_float(hh[i]);

    /* the second mode (fp32 accumulators, fp16 intermediates), every precision */
    float* y32 = (float*)malloc(sizeof(float) * (size_t)T * D);
    uint16_t* h16 = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * F);
    for (int e = 0; e < E; ++e) {
        if (orc_expert_ffn_f32(ex[e].prec_int4, &ex[e].w1, &ex[e].w3, &ex[e].w2, x, T, D, F, e & 1, y32, h16) != 0) return 10;
        for (size_t i = 0; i < (size_t)T * D; ++i) sum += y32[i];
    }
    uint16_t* out16 = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)T * D);
    if (orc_layer_forward_f32(x, T, D, F, E, K, wg, bias, ex, 1, x, out16, idx, gate) != 0) return 11;
    memcpy(hh, x, sizeof(uint16_t) * (size_t)T * D);
    if (orc_chain_layer_f32(hh, T, D, F, E, K, gain, 1e-5f, wg, NULL, ex, 0, idx, gate) != 0) return 12;
    for (size_t i = 0; i < (size_t)T * D; ++i) sum += orc_half_to_float(out16[i]) + orc_half_to_float(hh[i]);
    free(y32); free(h16); free(out16);

    /* a routed expert that is not resident must be reported, not read */
    ex[idx[0]].resident = 0;
    memcpy(hh, x, sizeof(uint16_t) * (size_t)T * D);
    const int rc = orc_layer_forward(hh, T, D, F, E, K, wg, NULL, ex, out, NULL, NULL);
    if (rc != -3 && rc != 0) return 9;

    printf("checksum %.6f threads %d\n", sum, orc_max_threads());
    free(x); free(wg); free(w_hat); free(idx); free(gate); free(logits); free(perm); free(y); free(h); free(out);
    free(gain); free(normed); free(hh);
    for (int m = 0; m < 3; ++m) { free(q[m]); free(sc[m]); free(ze[m]); free(q8[m]); free(sc8[m]); free(ze8[m]); }
    for (int e = 0; e < E; ++e) for (int m = 0; m < 3; ++m) free(w[e][m]);
    return 0;
}
