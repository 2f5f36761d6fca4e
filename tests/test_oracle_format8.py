"""Pins for the oracle's 8-bit format (the paper's homogeneous 8-bit model, Table 1; here: asymmetric uint8,
group 64, fp16 scale and zero, one code per byte): quantizer, dequantizer, expert built from it."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2407_14417_amd import synth
from tests.common import float_rne_exact, half_rne_exact

pytestmark = pytest.mark.filterwarnings("ignore::RuntimeWarning")


def test_hand_written_codes(orc):
    q = np.zeros((1, 64), dtype=np.uint8)
    q[0, :6] = [0, 1, 2, 100, 254, 255]
    m = orc.Mat(q, np.array([[0.5]], dtype=np.float16), np.array([[-2.0]], dtype=np.float16), bits=8)
    w = orc.dequant_int8(m).astype(np.float64)[0]
    assert list(w[:6]) == [-2.0, -1.5, -1.0, 48.0, 125.0, 125.5] and (w[6:] == -2.0).all()
    # a ramp 0, 1/4 .. 63.75 has range 63.75 = 255 * 0.25: scale 0.25, zero 0, code = 4 * value ... one per byte
    ramp = (np.arange(64) * 0.25).astype(np.float16)[None, :]
    ramp[0, -1] = 63.75
    m = orc.quantize_int8(ramp)
    assert m.scale[0, 0] == 0.25 and m.zero[0, 0] == 0.0 and m.bits == 8 and m.data.shape == (1, 64)
    assert list(m.data[0, :5]) == [0, 1, 2, 3, 4] and m.data[0, -1] == 255


def test_dequant_against_exact_rational_arithmetic(orc):
    """w_hat = fp16_rne(fp32_rne(q*s + z)) recomputed with rationals for sampled (s, z) and all 256 codes."""
    rng = np.random.default_rng(5)
    n_groups = 64
    s_bits = (np.abs(rng.standard_normal(n_groups)) * 5e-4).astype(np.float16).view(np.uint16)
    z_bits = (-np.abs(rng.standard_normal(n_groups)) * 5e-2).astype(np.float16).view(np.uint16)
    s_bits[:8] = rng.integers(0, 0x7BFF, 8).astype(np.uint16)             # arbitrary magnitudes too
    z_bits[:8] = rng.integers(0, 0x7BFF, 8).astype(np.uint16) | 0x8000
    q = np.tile(np.arange(256, dtype=np.uint8), (n_groups, 1))            # 4 groups of 64 columns per row
    sc = np.repeat(s_bits.view(np.float16)[:, None], 4, axis=1).copy()
    ze = np.repeat(z_bits.view(np.float16)[:, None], 4, axis=1).copy()
    got = orc.dequant_int8(orc.Mat(q, sc, ze, bits=8)).view(np.uint16)
    for g in range(n_groups):
        s = Fraction(float(s_bits[g:g + 1].view(np.float16)[0]))
        z = Fraction(float(z_bits[g:g + 1].view(np.float16)[0]))
        for code in range(256):
            want = half_rne_exact(float_rne_exact(code * s + z))
            if (want & 0x7FFF) == 0 and (int(got[g, code]) & 0x7FFF) == 0:
                continue                                   # +0 / -0 of an exact cancellation: sign is not pinned
            assert int(got[g, code]) == want, (g, code, float(s), float(z))


def test_quantizer_roundtrip_bound_min_exact_and_ranges(orc):
    w = synth.normal_f16((64, 512), 0.02, 12, 78)
    m = orc.quantize_int8(w)
    w_hat = orc.dequant_int8(m)
    out, inn = w.shape
    wg = w.astype(np.float64).reshape(out, inn // 64, 64)
    hg = w_hat.astype(np.float64).reshape(out, inn // 64, 64)
    s = m.scale.astype(np.float64)
    mn, mx = wg.min(axis=2), wg.max(axis=2)
    assert np.array_equal(m.zero.view(np.uint16), mn.astype(np.float16).view(np.uint16))
    assert np.array_equal(hg.min(axis=2), mn)                             # the group minimum comes back exactly
    want_s = ((mx.astype(np.float32) - mn.astype(np.float32)) / np.float32(255)).astype(np.float16)
    assert np.array_equal(m.scale.view(np.uint16), want_s.view(np.uint16))
    # half a step (the fp16 rounding of the step moves code 255 by at most 255 * 2^-11 steps: the clamp may bite by
    # that much at the top of the range), fp32 slack, final fp16 rounding
    bound = s * (0.5 + 255 * 2.0 ** -11 + 2.0 ** -10) + 2.0 ** -11 * np.maximum(np.abs(mn), np.abs(mx))
    assert (np.abs(wg - hg) <= bound[:, :, None] + 1e-12).all()
    # and for everything below the top code the plain half-step bound holds
    q = m.data.reshape(out, inn // 64, 64).astype(np.int64)
    inner = q < 255
    plain = s * (0.5 + 2.0 ** -10) + 2.0 ** -11 * np.maximum(np.abs(mn), np.abs(mx))
    assert (np.abs(wg - hg)[inner] <= np.broadcast_to(plain[:, :, None], wg.shape)[inner] + 1e-12).all()
    assert q.min() >= 0 and q.max() <= 255
    order = np.argsort(wg, axis=2, kind="stable")
    assert (np.diff(np.take_along_axis(q, order, axis=2), axis=2) >= 0).all()       # monotone in w within a group
    assert (q.min(axis=2) == 0).all() and (q.max(axis=2) >= 254).all()
    # 8 bits are 16 times finer than 4: the round-trip error shrinks accordingly
    m4 = orc.quantize_int4(w)
    e8 = np.abs(w.astype(np.float64) - w_hat.astype(np.float64)).mean()
    e4 = np.abs(w.astype(np.float64) - orc.dequant_int4(m4).astype(np.float64)).mean()
    assert 8 < e4 / e8 < 24


def test_constant_group_and_ragged_shape(orc):
    w = np.full((2, 128), 0.0123, dtype=np.float16)
    w[1, 64:] = -3.5
    m = orc.quantize_int8(w)
    assert not m.scale.any() and not m.data.any()
    assert np.array_equal(orc.dequant_int8(m).view(np.uint16), w.view(np.uint16))
    with pytest.raises(ValueError):
        orc.quantize_int8(np.zeros((2, 96), dtype=np.float16))


def test_8bit_expert_is_the_16bit_expert_of_its_dequantized_weights(orc):
    """The expert built from 8-bit matrices equals, bit for bit, the 16-bit expert made of the dequantized weights
    (both evaluate the same doubles), and sits much closer to the unquantized expert than the 4-bit one."""
    d, f, n = 128, 192, 5
    w1 = synth.normal_f16((f, d), 0.05, 21, 1)
    w3 = synth.normal_f16((f, d), 0.05, 21, 2)
    w2 = synth.normal_f16((d, f), 0.05, 21, 3)
    x = synth.normal_f16((n, d), 1.0, 21, 4)
    e8 = orc.Expert(orc.quantize_int8(w1), orc.quantize_int8(w3), orc.quantize_int8(w2))
    assert e8.int8 and not e8.int4 and e8.prec == 2
    ed = orc.Expert(orc.Mat(orc.dequant_int8(e8.w1)), orc.Mat(orc.dequant_int8(e8.w3)), orc.Mat(orc.dequant_int8(e8.w2)))
    y8, yd = orc.expert_ffn(e8, x), orc.expert_ffn(ed, x)
    assert np.array_equal(y8, yd)
    y16 = orc.expert_ffn(orc.Expert(orc.Mat(w1), orc.Mat(w3), orc.Mat(w2)), x)
    e4 = orc.Expert(orc.quantize_int4(w1), orc.quantize_int4(w3), orc.quantize_int4(w2))
    y4 = orc.expert_ffn(e4, x)
    err8 = np.linalg.norm(y8 - y16) / np.linalg.norm(y16)
    err4 = np.linalg.norm(y4 - y16) / np.linalg.norm(y16)
    assert err8 < 0.02 and err4 > 5 * err8
    # the second mode takes the same codes
    y32 = orc.expert_ffn_f32(e8, x)
    assert np.linalg.norm(y32.astype(np.float64) - y8) / np.linalg.norm(y8) < 1e-3
    assert not np.array_equal(orc.expert_ffn_f32(e8, x, exact_weights=True), y32)
