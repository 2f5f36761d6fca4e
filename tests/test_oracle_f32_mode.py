"""Pins for the oracle's second mode (fp32 accumulators, hidden row and block output rounded to fp16).

The mode is pinned against things other than itself: the double functions (pinned in test_oracle_block.py)
within the textbook forward-error bound of recursive fp32 summation plus the fp16 roundings the mode states;
bit-equality with the double functions on inputs where every operation is exact; numpy float32 arithmetic
written out as the same recursion."""
import numpy as np

from paper_2407_14417_amd import synth
from tests.common import MEDIUM, TINY, build_workload

U32 = 2.0 ** -24          # unit roundoff fp32
U16 = 2.0 ** -11          # unit roundoff fp16


def _dense(m, orc):
    return orc.dequant_int4(m).astype(np.float64) if m.int4 else m.data.astype(np.float64)


def test_expert_f32_within_forward_error_bound_of_the_double_expert(orc):
    """|y32 - y64| <= W2_abs . (|dh| ) + gamma terms: the hidden row differs from the double one by its own
    fp32 summation error and one fp16 rounding; the output by fp32 summation error on top."""
    wl = build_workload(TINY, orc)
    cfg = wl.cfg
    for e in (0, 1):                                   # one 16-bit, one 4-bit expert
        ex = wl.experts[e]
        y64, h64 = orc.expert_ffn(ex, wl.x, want_h=True)
        y32, h16 = orc.expert_ffn_f32(ex, wl.x, want_h=True)
        w1, w3, w2 = (_dense(m, orc) for m in (ex.w1, ex.w3, ex.w2))
        x = wl.x.astype(np.float64)
        # a, b: recursive summation of d terms, each product rounded once: |err| <= (d + 1) u sum|terms|
        g1 = (cfg.d + 1) * U32
        a_abs, b_abs = np.abs(x) @ np.abs(w1).T, np.abs(x) @ np.abs(w3).T
        a, b = x @ w1.T, x @ w3.T
        da, db = g1 * a_abs, g1 * b_abs
        # silu'(a) lies in (-0.1, 1.1); expf, the division and two products add a few fp32 roundings
        sil = np.abs(a / (1 + np.exp(-a)))
        dh = 1.1 * da * (np.abs(b) + db) + sil * db + 8 * U32 * np.abs(h64)
        dh = dh + U16 * (np.abs(h64) + dh) + 2.0 ** -25          # the fp16 rounding (and the subnormal spacing)
        assert (np.abs(h16.astype(np.float64) - h64) <= dh).all()
        g2 = (cfg.f + 1) * U32
        bound = dh @ np.abs(w2).T + g2 * ((np.abs(h64) + dh) @ np.abs(w2).T)
        assert (np.abs(y32.astype(np.float64) - y64) <= bound).all()
        # and the bound is not vacuous: it sits orders of magnitude below the values themselves
        assert bound.max() < 2e-2 * np.abs(y64).max()


def test_expert_f32_equals_numpy_float32_recursion(orc):
    """The same recursion written with numpy float32 scalars on a small expert: every bit must agree (exp is
    checked through the hidden row with a one-ulp allowance for the library's expf)."""
    d, f, n = 64, 128, 3
    w1 = synth.normal_f16((f, d), 0.1, 3, 1)
    w3 = synth.normal_f16((f, d), 0.1, 3, 2)
    w2 = synth.normal_f16((d, f), 0.1, 3, 3)
    x = synth.normal_f16((n, d), 1.0, 3, 4)
    ex = orc.Expert(orc.Mat(w1), orc.Mat(w3), orc.Mat(w2))
    y32, h16 = orc.expert_ffn_f32(ex, x, want_h=True)
    f32 = np.float32
    h_ref = np.zeros((n, f), dtype=np.float16)
    for i in range(n):
        for r in range(f):
            a, b = f32(0), f32(0)
            for j in range(d):
                a = f32(a + f32(f32(w1[r, j]) * f32(x[i, j])))
                b = f32(b + f32(f32(w3[r, j]) * f32(x[i, j])))
            h_ref[i, r] = np.float16(f32(f32(a / f32(f32(1) + np.exp(-a, dtype=f32))) * b))
    ulp = np.abs(np.spacing(h_ref.astype(np.float16))).astype(np.float64)
    assert (np.abs(h16.astype(np.float64) - h_ref.astype(np.float64)) <= ulp).all()
    # the down-projection from the mode's own rounded hidden row: exact bit equality
    for i in range(n):
        for r in range(d):
            acc = f32(0)
            for j in range(f):
                acc = f32(acc + f32(f32(w2[r, j]) * f32(h16[i, j])))
            assert acc == y32[i, r]


def test_f32_mode_is_bit_equal_to_double_mode_when_every_operation_is_exact(orc):
    """Small-integer weights and tokens with W1 x = 0: silu(0) * b = 0 exactly, so h = 0 and y = 0 in both modes;
    with the gate logits exact as well, routing and gates agree to the last bit where fp32 can hold them."""
    d, f, E, k, T = 64, 64, 4, 2, 5
    rng = np.random.default_rng(0)
    x = rng.integers(-3, 4, size=(T, d)).astype(np.float16)
    wg = rng.integers(-2, 3, size=(E, d)).astype(np.float16)
    experts = []
    for e in range(E):
        w1 = np.zeros((f, d), dtype=np.float16)
        w3 = rng.integers(-2, 3, size=(f, d)).astype(np.float16)
        w2 = rng.integers(-2, 3, size=(d, f)).astype(np.float16)
        experts.append(orc.Expert(orc.Mat(w1), orc.Mat(w3), orc.Mat(w2)))
    out64, idx64, gate64 = orc.layer_forward(x, wg, experts, k)
    out16, idx32, gate32 = orc.layer_forward_f32(x, wg, experts, k)
    assert np.array_equal(idx64, idx32)
    assert np.allclose(gate64, gate32, rtol=0, atol=2e-7)
    assert (out64 == 0).all() and (out16 == 0).all()
    # residual passes through exactly
    res = rng.integers(-5, 6, size=(T, d)).astype(np.float16)
    out_res, _, _ = orc.layer_forward_f32(x, wg, experts, k, residual=res)
    assert np.array_equal(out_res, res)


def test_layer_f32_is_close_to_double_layer_and_exact_weights_move_it_by_half_an_ulp_of_the_weights(orc):
    wl = build_workload(MEDIUM, orc)
    cfg = wl.cfg
    ref, ref_idx, ref_gate = orc.layer_forward(wl.x, wl.wg, wl.experts, cfg.k)
    for exact in (False, True):
        out, idx, gate = orc.layer_forward_f32(wl.x, wl.wg, wl.experts, cfg.k, exact_weights=exact)
        assert np.array_equal(idx, ref_idx)
        assert np.allclose(gate, ref_gate, rtol=0, atol=2e-6)
        err = out.astype(np.float64) - ref
        # three fp16 roundings per path (hidden row, output; weights when exact): well inside the block tolerance
        assert np.abs(err).max() <= 2e-3 * np.abs(ref).max()
        assert np.linalg.norm(err) / np.linalg.norm(ref) <= 1e-3


def test_exact_weights_only_touch_4bit_experts(orc):
    wl = build_workload(TINY, orc)
    x = wl.x[:4]
    a = orc.expert_ffn_f32(wl.experts[0], x, exact_weights=False)      # expert 0 is 16-bit
    b = orc.expert_ffn_f32(wl.experts[0], x, exact_weights=True)
    assert np.array_equal(a, b)
    a = orc.expert_ffn_f32(wl.experts[1], x, exact_weights=False)      # expert 1 is 4-bit
    b = orc.expert_ffn_f32(wl.experts[1], x, exact_weights=True)
    assert not np.array_equal(a, b)
    assert np.abs(a - b).max() <= 2e-3 * np.abs(a).max()


def test_chain_layer_f32_follows_the_double_chain_layer(orc):
    wl = build_workload(TINY, orc)
    cfg = wl.cfg
    g = synth.normal_f16((cfg.d,), 0.1, 9, 7) + np.float16(1.0)
    h0 = wl.x
    h64, idx64, _, _ = orc.chain_layer(h0, g, 1e-5, wl.wg, wl.experts, cfg.k)
    h16, idx32, _ = orc.chain_layer_f32(h0, g, 1e-5, wl.wg, wl.experts, cfg.k)
    assert np.array_equal(idx64, idx32)
    d = h16.astype(np.float64) - h64.astype(np.float64)
    assert np.abs(d).max() <= 2.0 ** -9 * np.abs(h64.astype(np.float64)).max()
    # all-zero w2: the residual path alone, the hidden state comes back unchanged
    zero_experts = [orc.Expert(e.w1, e.w3, orc.Mat(np.zeros((cfg.d, cfg.f), dtype=np.float16)))
                    if not e.int4 else e for e in wl.experts]
    only16 = [e for e in zero_experts if not e.int4]
    wg2 = wl.wg[: len(only16)]
    h_same, _, _ = orc.chain_layer_f32(h0, g, 1e-5, wg2, only16, 2)
    assert np.array_equal(h_same, h0)
