"""Pins for the oracle's gating, grouping, expert FFN, whole block and chain glue."""
import itertools
import math

import numpy as np
import pytest
from scipy.special import softmax

from paper_2407_14417_amd import synth
from tests.common import TINY, build_workload


def _onehot_x(d, rows):
    """Tokens that are unit vectors: logits of token t are then column t of Wg, exactly."""
    x = np.zeros((rows, d), dtype=np.float16)
    x[np.arange(rows), np.arange(rows)] = 1.0
    return x


# ---------------------------------------------------------------- gating

def test_topk_against_full_sort_over_all_permutations(orc):
    base = np.array([-1.5, 0.25, 0.75, 2.0, 3.5], dtype=np.float16)
    perms = list(itertools.permutations(range(5)))
    T, E = len(perms), 5
    wg = np.zeros((E, T), dtype=np.float16)
    for t, p in enumerate(perms):
        wg[:, t] = base[list(p)]
    x = _onehot_x(T, T)
    for k in (1, 2, 3, 5):
        idx, gate, logits = orc.route(x, wg, k, want_logits=True)
        for t, p in enumerate(perms):
            l = base[list(p)].astype(np.float64)
            assert np.array_equal(logits[t], l)
            want = sorted(range(E), key=lambda e: (-l[e], e))[:k]
            assert list(idx[t]) == want
            sel = np.exp(l[want] - l[want].max())
            assert np.allclose(gate[t], sel / sel.sum(), rtol=0, atol=1e-7)


def test_topk_ties_take_lower_index_first(orc):
    wg = np.array([[1.0], [2.0], [2.0], [0.5], [2.0]], dtype=np.float16)
    idx, gate = orc.route(np.ones((1, 1), dtype=np.float16), wg, 3)
    assert list(idx[0]) == [1, 2, 4]
    assert np.allclose(gate[0], 1 / 3, atol=1e-7)


def test_logits_match_library_matmul_and_bias(orc):
    wg = synth.normal_f16((8, 320), 0.02, 5, 2)
    x = synth.normal_f16((7, 320), 1.0, 5, 1)
    bias = synth.zipf_bias(8)
    _, _, l0 = orc.route(x, wg, 2, want_logits=True)
    _, _, l1 = orc.route(x, wg, 2, bias=bias, want_logits=True)
    ref = x.astype(np.float64) @ wg.astype(np.float64).T
    assert np.allclose(l0, ref, rtol=1e-13, atol=1e-15)
    assert np.allclose(l1, ref + bias.astype(np.float64), rtol=1e-13, atol=1e-15)


def test_gates_sum_to_one_k_equals_E_is_softmax_k1_is_one_shift_invariant(orc):
    wg = synth.normal_f16((8, 256), 0.05, 6, 2)
    x = synth.normal_f16((33, 256), 1.0, 6, 1)
    _, _, logits = orc.route(x, wg, 2, want_logits=True)
    for k in (1, 2, 3, 8):
        idx, gate = orc.route(x, wg, k)
        assert np.allclose(gate.astype(np.float64).sum(axis=1), 1.0, atol=1e-6)
        assert (np.diff(gate, axis=1) <= 0).all()                      # descending logits -> descending gates
        # S2 identity: softmax over the selected logits == full softmax renormalised over the selection
        p = softmax(logits, axis=1)
        sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
        assert np.allclose(gate, sel / sel.sum(axis=1, keepdims=True), atol=1e-7)
    idx, gate = orc.route(x, wg, 8)
    assert np.allclose(np.take_along_axis(softmax(logits, axis=1), idx.astype(np.int64), axis=1), gate, atol=1e-7)
    idx1, gate1 = orc.route(x, wg, 1)
    assert (gate1 == 1.0).all() and np.array_equal(idx1[:, 0], logits.argmax(axis=1))
    # a constant added to every logit changes neither the choice nor the gates
    idx_a, gate_a = orc.route(x, wg, 2)
    idx_b, gate_b = orc.route(x, wg, 2, bias=np.full(8, 3.25, dtype=np.float32))
    assert np.array_equal(idx_a, idx_b) and np.allclose(gate_a, gate_b, atol=1e-7)


# ---------------------------------------------------------------- grouping

def test_permute_is_a_stable_grouping(orc):
    rng = np.random.default_rng(4)
    for T, k, E in ((1, 2, 8), (16, 2, 4), (37, 3, 8), (5, 1, 2)):
        idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        counts, offsets, perm = orc.permute(idx, E)
        flat = idx.reshape(-1)
        assert counts.sum() == T * k and np.array_equal(counts, np.bincount(flat, minlength=E))
        assert offsets[0] == 0 and np.array_equal(offsets[1:], np.cumsum(counts))
        assert sorted(perm) == list(range(T * k))
        assert np.array_equal(perm, np.argsort(flat, kind="stable"))
        v = rng.standard_normal(T * k)
        back = np.empty_like(v)
        back[perm] = v[perm]
        assert np.array_equal(back, v)


# ---------------------------------------------------------------- expert

def _silu(a):
    return a / (1.0 + np.exp(-a))


def test_fp16_expert_against_library_matmul_and_python_loops(orc):
    d, f, n = 64, 128, 3
    w1 = synth.normal_f16((f, d), 0.2, 7, 10)
    w3 = synth.normal_f16((f, d), 0.2, 7, 11)
    w2 = synth.normal_f16((d, f), 0.2, 7, 12)
    x = synth.normal_f16((n, d), 1.0, 7, 1)
    y, h = orc.expert_ffn(orc.Expert(orc.Mat(w1), orc.Mat(w3), orc.Mat(w2)), x, want_h=True)
    X, W1, W3, W2 = (a.astype(np.float64) for a in (x, w1, w3, w2))
    a, b = X @ W1.T, X @ W3.T
    href = _silu(a) * b
    assert np.allclose(h, href, rtol=1e-12, atol=1e-14)
    assert np.allclose(y, href @ W2.T, rtol=1e-11, atol=1e-13)
    # brute force with scalar Python loops on the first row
    xl, w1l, w3l, w2l = X[0].tolist(), W1.tolist(), W3.tolist(), W2.tolist()
    hl = []
    for r in range(f):
        aa = math.fsum(w1l[r][j] * xl[j] for j in range(d))
        bb = math.fsum(w3l[r][j] * xl[j] for j in range(d))
        hl.append(aa / (1.0 + math.exp(-aa)) * bb)
    yl = [math.fsum(w2l[r][j] * hl[j] for j in range(f)) for r in range(d)]
    assert np.allclose(y[0], yl, rtol=1e-11, atol=1e-13)


def test_operands_are_not_transposed_or_swapped(orc):
    """w1 is the gated (SiLU) branch, w3 the linear one, w2 maps f -> d: each checked with a one-entry matrix."""
    d, f = 64, 128
    x = np.zeros((1, d), dtype=np.float16)
    x[0, 5] = 2.0
    w1 = np.zeros((f, d), dtype=np.float16); w1[9, 5] = 1.5          # a[9] = 3
    w3 = np.zeros((f, d), dtype=np.float16); w3[9, 5] = 0.25         # b[9] = 0.5
    w2 = np.zeros((d, f), dtype=np.float16); w2[17, 9] = 4.0
    y = orc.expert_ffn(orc.Expert(orc.Mat(w1), orc.Mat(w3), orc.Mat(w2)), x)
    want = 3.0 / (1.0 + math.exp(-3.0)) * 0.5 * 4.0
    assert abs(y[0, 17] - want) < 1e-14 and np.count_nonzero(y) == 1
    # swapping the roles of w1 and w3 gives silu(0.5) * 3 instead
    y2 = orc.expert_ffn(orc.Expert(orc.Mat(w3), orc.Mat(w1), orc.Mat(w2)), x)
    assert abs(y2[0, 17] - 0.5 / (1.0 + math.exp(-0.5)) * 3.0 * 4.0) < 1e-14


def test_silu_identities_and_zero_w3(orc):
    d, f = 64, 64
    eye = np.eye(64, dtype=np.float16)
    ones_w3 = eye.copy()
    x = np.zeros((3, d), dtype=np.float16)
    x[0, :] = 0.0
    x[1, :] = 12.0            # silu(a) -> a for large a
    x[2, :] = -3.0
    # w1 = I, w3 = I, w2 = I: y = silu(x) * x
    y = orc.expert_ffn(orc.Expert(orc.Mat(eye), orc.Mat(ones_w3), orc.Mat(eye)), x)
    assert not y[0].any()
    assert np.allclose(y[1], 12.0 * 12.0 / (1 + math.exp(-12.0)), rtol=1e-14)
    assert np.allclose(y[2], (-3.0 * (1 / (1 + math.exp(3.0)))) * -3.0, rtol=1e-14)   # silu(-a) = -a*sigma(-a)
    zero = np.zeros((f, d), dtype=np.float16)
    assert not orc.expert_ffn(orc.Expert(orc.Mat(eye), orc.Mat(zero), orc.Mat(eye)), x).any()


def test_int4_expert_equals_fp16_expert_of_dequantized_weights(orc):
    d, f, n = 128, 192, 4
    ws = [synth.normal_f16(s, 0.02, 8, 20 + i) for i, s in enumerate(((f, d), (f, d), (d, f)))]
    x = synth.normal_f16((n, d), 1.0, 8, 1)
    q = [orc.quantize_int4(w) for w in ws]
    y4 = orc.expert_ffn(orc.Expert(*q), x)
    y16 = orc.expert_ffn(orc.Expert(*[orc.Mat(orc.dequant_int4(m)) for m in q]), x)
    assert np.array_equal(y4, y16)
    # and against a library matmul on the materialised weights
    W1, W3, W2 = (orc.dequant_int4(m).astype(np.float64) for m in q)
    X = x.astype(np.float64)
    assert np.allclose(y4, (_silu(X @ W1.T) * (X @ W3.T)) @ W2.T, rtol=1e-10, atol=1e-14)


# ---------------------------------------------------------------- whole block

def test_layer_equals_gate_weighted_sum_of_expert_outputs(orc):
    wl = build_workload(TINY, orc)
    out, idx, gate = orc.layer_forward(wl.x, wl.wg, wl.experts, TINY.k)
    idx2, gate2 = orc.route(wl.x, wl.wg, TINY.k)
    assert np.array_equal(idx, idx2) and np.array_equal(gate, gate2)
    ref = np.zeros_like(out)
    for t in range(TINY.T):
        for s in range(TINY.k):
            ref[t] += float(gate[t, s]) * orc.expert_ffn(wl.experts[idx[t, s]], wl.x[t:t + 1])[0]
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-16)
    assert set(np.unique(idx)) <= set(range(TINY.E)) and (idx[:, 0] != idx[:, 1]).all()


def test_one_hot_gate_reduces_to_single_expert(orc):
    wl = build_workload(TINY, orc)
    # k = 1: the gate is exactly 1, the block is the chosen expert's FFN
    out, idx, gate = orc.layer_forward(wl.x, wl.wg, wl.experts, 1)
    assert (gate == 1.0).all()
    for t in range(TINY.T):
        assert np.array_equal(out[t], orc.expert_ffn(wl.experts[idx[t, 0]], wl.x[t:t + 1])[0])
    # k = 2 with a bias that makes expert 2 win by 40: gate -> 1 up to exp(-40)
    bias = np.array([0, 0, 60, 0], dtype=np.float32)
    out, idx, gate = orc.layer_forward(wl.x, wl.wg, wl.experts, 2, bias=bias)
    assert (idx[:, 0] == 2).all() and (gate[:, 0] == 1.0).all()
    y2 = orc.expert_ffn(wl.experts[2], wl.x)
    assert np.allclose(out, y2, rtol=1e-9, atol=1e-12)


def test_identical_experts_make_routing_irrelevant(orc):
    wl = build_workload(TINY, orc)
    same = [wl.experts[1]] * TINY.E
    out, idx, gate = orc.layer_forward(wl.x, wl.wg, same, TINY.k)
    assert np.allclose(out, orc.expert_ffn(wl.experts[1], wl.x), rtol=1e-6, atol=1e-9)   # gates are fp32: sum to 1 within 1e-7


def test_non_resident_routed_expert_is_an_error(orc):
    wl = build_workload(TINY, orc)
    idx, _ = orc.route(wl.x, wl.wg, TINY.k)
    victim = int(idx[0, 0])
    e = wl.experts[victim]
    wl.experts[victim] = orc.Expert(e.w1, e.w3, e.w2, resident=False)
    with pytest.raises(LookupError):
        orc.layer_forward(wl.x, wl.wg, wl.experts, TINY.k)


# ---------------------------------------------------------------- chain glue

def test_rmsnorm_closed_form_on_constant_vector(orc):
    d, eps = 256, 1e-5
    g = synth.normal_f16((d,), 1.0, 9, 3)
    for c in (0.5, -2.0, 0.01):
        h = np.full((1, d), c, dtype=np.float16)
        cf = float(np.float16(c))
        want = (np.sign(cf) * g.astype(np.float64) / math.sqrt(1 + eps / cf ** 2)).astype(np.float16)
        assert np.array_equal(orc.rmsnorm(h, g, eps).view(np.uint16)[0], want.view(np.uint16))
    # against a float64 library evaluation on random rows
    h = synth.normal_f16((5, d), 3.0, 9, 4)
    H = h.astype(np.float64)
    want = (H / np.sqrt((H * H).mean(axis=1, keepdims=True) + eps) * g.astype(np.float64)).astype(np.float16)
    got = orc.rmsnorm(h, g, eps)
    assert (np.abs(got.view(np.int16).astype(np.int64) - want.view(np.int16).astype(np.int64)) <= 1).all()
    assert (got == want).mean() > 0.99


def test_chain_layer_with_zero_w2_leaves_h_unchanged_and_residual_rounds_once(orc):
    wl = build_workload(TINY, orc)
    g = np.ones(TINY.d, dtype=np.float16)
    def zero_like(e):          # a w2 whose dequantized value is all zero, in the expert's own precision
        if e.int4:
            return orc.Mat(np.zeros((TINY.d, TINY.f // 2), dtype=np.uint8),
                           np.zeros((TINY.d, TINY.f // 64), dtype=np.float16),
                           np.zeros((TINY.d, TINY.f // 64), dtype=np.float16))
        return orc.Mat(np.zeros((TINY.d, TINY.f), dtype=np.float16))
    fixed = [orc.Expert(e.w1, e.w3, zero_like(e)) for e in wl.experts]
    h0 = wl.x.copy()
    h1, idx, gate, normed = orc.chain_layer(h0, g, 1e-5, wl.wg, fixed, TINY.k)
    assert np.array_equal(h1.view(np.uint16), h0.view(np.uint16))
    assert np.array_equal(normed.view(np.uint16), orc.rmsnorm(h0, g, 1e-5).view(np.uint16))
    # full block: h1 = fp16(h0 + MoE(norm(h0))) with the MoE output unrounded
    h1, idx, gate, normed = orc.chain_layer(h0, g, 1e-5, wl.wg, wl.experts, TINY.k)
    out, idx2, _ = orc.layer_forward(normed, wl.wg, wl.experts, TINY.k)
    assert np.array_equal(idx, idx2)
    want = (h0.astype(np.float64) + out).astype(np.float16)
    assert np.array_equal(h1.view(np.uint16), want.view(np.uint16))
