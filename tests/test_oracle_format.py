"""Pins for the oracle's fp16 conversions and the 4-bit format (quantizer, dequantizer, nibble order)."""
from fractions import Fraction

import numpy as np
import pytest

from tests.common import half_rne_exact, float_rne_exact
from paper_2407_14417_amd import synth

pytestmark = pytest.mark.filterwarnings("ignore::RuntimeWarning")


def test_half_to_float_all_patterns_match_numpy(orc):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([orc.half_to_float(int(b)) for b in bits], dtype=np.float32)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite].view(np.uint32), ref[finite].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isinf(got), np.isinf(ref)) and np.array_equal(np.sign(got[np.isinf(ref)]), np.sign(ref[np.isinf(ref)]))


def test_float_to_half_matches_numpy_on_random_and_halfway_values(orc):
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(5000) * 1e-5).astype(np.float32),       # subnormal range
        (rng.standard_normal(5000) * 3e4).astype(np.float32),        # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.996, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
                  np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 2.0 ** -14, 6.0975552e-05], dtype=np.float32),
    ])
    # exact halfway points between neighbouring halves (tie cases), all representable in fp32
    hb = rng.integers(0, 0x7BFF, 4000).astype(np.uint16)
    lo = hb.view(np.float16).astype(np.float32)
    hi = (hb + 1).astype(np.uint16).view(np.float16).astype(np.float32)
    vals = np.concatenate([vals, (lo + hi) / 2, -(lo + hi) / 2])
    ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([orc.float_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_double_to_half_matches_exact_rational_rounding(orc):
    rng = np.random.default_rng(2)
    vals = np.concatenate([rng.standard_normal(3000), rng.standard_normal(1000) * 1e-6, rng.standard_normal(1000) * 2e4,
                           [1.0 + 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -40, 1.0 + 3 * 2.0 ** -11, 2.0 ** -24 * 0.5,
                            2.0 ** -24 * 1.5, 2.0 ** -24 * 2.5]])
    for v in vals:
        assert orc.double_to_half(float(v)) == half_rne_exact(Fraction(float(v))), v


def test_pack_order_hand_written_vector(orc):
    # One row, one group: bytes 0x21, 0x43, ... mean q[0]=1, q[1]=2, q[2]=3, q[3]=4 (low nibble = even column).
    packed = np.zeros((1, 32), dtype=np.uint8)
    packed[0, :8] = [0x21, 0x43, 0x65, 0x87, 0xA9, 0xCB, 0xED, 0x0F]
    m = orc.Mat(packed, np.array([[1.0]], dtype=np.float16), np.array([[0.0]], dtype=np.float16))
    w = orc.dequant_int4(m).astype(np.float64)[0]
    assert list(w[:16]) == [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 0]
    assert not w[16:].any()
    # scale 0.5, zero -1: q*0.5 - 1 is exact in fp16
    m = orc.Mat(packed, np.array([[0.5]], dtype=np.float16), np.array([[-1.0]], dtype=np.float16))
    w = orc.dequant_int4(m).astype(np.float64)[0]
    assert list(w[:4]) == [-0.5, 0.0, 0.5, 1.0] and w[15] == -1.0


def test_quantizer_packs_low_nibble_first(orc):
    # a ramp 0..15 repeated: scale 1, zero 0 -> q equals the value; check raw bytes
    w = np.tile(np.arange(16, dtype=np.float16), 4)[None, :]
    m = orc.quantize_int4(w)
    assert m.scale[0, 0] == 1.0 and m.zero[0, 0] == 0.0
    assert list(m.data[0, :8]) == [0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE]


def test_dequant_against_exact_rational_arithmetic(orc):
    """w_hat = fp16_rne(fp32_rne(q*s + z)): recomputed with integers/rationals for sampled (s, z), all 16 q."""
    rng = np.random.default_rng(3)
    n_groups = 300
    s_bits = rng.integers(0, 0x7BFF, n_groups).astype(np.uint16)
    z_bits = rng.integers(0, 0x7BFF, n_groups).astype(np.uint16) | (rng.integers(0, 2, n_groups).astype(np.uint16) << 15)
    # typical magnitudes too: s ~ 7e-3, z ~ -5e-2
    s_bits[:150] = (np.abs(rng.standard_normal(150)) * 7e-3).astype(np.float16).view(np.uint16)
    z_bits[:150] = (-np.abs(rng.standard_normal(150)) * 5e-2).astype(np.float16).view(np.uint16)
    packed = np.zeros((n_groups, 32), dtype=np.uint8)
    for j in range(32):                        # columns 0..63 carry q = c mod 16
        packed[:, j] = ((2 * j) % 16) | (((2 * j + 1) % 16) << 4)
    m = orc.Mat(packed, s_bits.view(np.float16)[:, None].copy(), z_bits.view(np.float16)[:, None].copy())
    got = orc.dequant_int4(m).view(np.uint16)
    for g in range(n_groups):
        s = Fraction(float(s_bits[g:g + 1].view(np.float16)[0]))
        z = Fraction(float(z_bits[g:g + 1].view(np.float16)[0]))
        for q in range(16):
            want = half_rne_exact(float_rne_exact(q * s + z))
            if (want & 0x7FFF) == 0 and (int(got[g, q]) & 0x7FFF) == 0:
                continue                                   # +0 / -0 of an exact cancellation: sign is not pinned
            assert int(got[g, q]) == want, (g, q, float(s), float(z))


def _roundtrip(orc, w):
    m = orc.quantize_int4(w)
    return m, orc.dequant_int4(m)


def test_quantizer_roundtrip_bound_min_exact_and_ranges(orc):
    w = synth.normal_f16((96, 512), 0.02, 11, 77)
    m, w_hat = _roundtrip(orc, w)
    out, inn = w.shape
    wd, hd = w.astype(np.float64), w_hat.astype(np.float64)
    wg = wd.reshape(out, inn // 64, 64)
    hg = hd.reshape(out, inn // 64, 64)
    s = m.scale.astype(np.float64)
    z = m.zero.astype(np.float64)
    mn, mx = wg.min(axis=2), wg.max(axis=2)
    # zero is the group minimum, bit for bit, and the minimum is reproduced exactly
    assert np.array_equal(m.zero.view(np.uint16), mn.astype(np.float16).view(np.uint16))
    assert np.array_equal(hg.min(axis=2), mn)
    # scale = fp16((max-min)/15) computed in fp32
    want_s = ((mx.astype(np.float32) - mn.astype(np.float32)) / np.float32(15)).astype(np.float16)
    assert np.array_equal(m.scale.view(np.uint16), want_s.view(np.uint16))
    # closed-form error bound: half a step, fp32 slack, final fp16 rounding
    bound = s * (0.5 + 2.0 ** -10) + 2.0 ** -11 * np.maximum(np.abs(mn), np.abs(mx))
    assert (np.abs(wg - hg) <= bound[:, :, None] + 1e-12).all()
    # group maximum within 15 * 2^-11 * s + one fp16 ulp of it
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(mx), 2.0 ** -14))) - 10)
    assert (np.abs(hg.max(axis=2) - mx) <= 15 * 2.0 ** -11 * s + ulp).all()
    # codes: in range and monotone in w within a group
    q = np.stack([m.data & 0xF, m.data >> 4], axis=2).reshape(out, inn // 64, 64)
    assert q.min() >= 0 and q.max() <= 15
    order = np.argsort(wg, axis=2, kind="stable")
    assert (np.diff(np.take_along_axis(q.astype(np.int64), order, axis=2), axis=2) >= 0).all()
    # every group uses code 0 (its minimum) and code 15 (its maximum)
    assert (q.min(axis=2) == 0).all() and (q.max(axis=2) == 15).all()


def test_quantizer_constant_group_is_exact(orc):
    w = np.full((2, 128), 0.0123, dtype=np.float16)
    w[1, 64:] = -3.5
    m, w_hat = _roundtrip(orc, w)
    assert not m.scale.any() and not m.data.any()
    assert np.array_equal(w_hat.view(np.uint16), w.view(np.uint16))


def test_quantize_rejects_ragged_group(orc):
    with pytest.raises(ValueError):
        orc.quantize_int4(np.zeros((2, 96), dtype=np.float16))


def test_expert_sizes_match_paper():
    consts = {}
    from pathlib import Path
    for line in (Path(__file__).parent / "golden" / "paper_constants.txt").read_text().splitlines():
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            consts[k.strip()] = float(v)
    d, f = 4096, 14336
    fp16_bytes = 3 * d * f * 2
    assert fp16_bytes == int(consts["expert_size_MB"]) * 2 ** 20               # 336 MiB, the paper's expert size
    int4_bytes = 3 * d * f // 2 + 3 * d * f // 64 * 4
    assert int4_bytes == 99_090_432
    assert consts["n_layers"] * consts["experts_per_layer"] == consts["total_experts"]
