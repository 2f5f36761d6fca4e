"""The seeded input generator: C accelerator == numpy recipe, moments, stream independence."""
import numpy as np

from paper_2407_14417_amd import synth


def test_c_and_numpy_generators_agree_bit_for_bit():
    for sigma, stream in ((1.0, synth.x_stream()), (0.02, synth.expert_stream(3, 5, 2))):
        a = synth.normal_f16((3, 1000), sigma, 42, stream)
        b = synth.normal_f16((3, 1000), sigma, 42, stream, use_numpy=True)
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    a = synth.uniform_f16((777,), 0.0346, 1, synth.STREAM_WG)
    b = synth.uniform_f16((777,), 0.0346, 1, synth.STREAM_WG, use_numpy=True)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_first_offset_addresses_the_same_stream():
    full = synth.normal_f16((4096,), 1.0, 0, 1)
    part = synth.normal_f16((100,), 1.0, 0, 1, first=1234)
    assert np.array_equal(full[1234:1334].view(np.uint16), part.view(np.uint16))


def test_moments_and_range():
    a = synth.normal_f16((1 << 20,), 0.02, 0, 99).astype(np.float64)
    assert abs(a.mean()) < 1e-4 and abs(a.std() / 0.02 - 1) < 5e-3
    assert np.abs(a).max() < 4.9 * 0.02 * 1.01
    # fourth moment of a sum of eight uniforms: kurtosis 3 - 1.2/8 = 2.85
    assert abs((a ** 4).mean() / a.var() ** 2 - 2.85) < 0.03
    u = synth.uniform_f16((1 << 20,), 0.5, 0, 98).astype(np.float64)
    assert abs(u.mean()) < 2e-3 and abs(u.std() - 0.5 / 3 ** 0.5) < 2e-3 and np.abs(u).max() <= 0.5


def test_streams_and_seeds_are_independent():
    a = synth.normal_f16((1 << 16,), 1.0, 0, 1).astype(np.float64)
    b = synth.normal_f16((1 << 16,), 1.0, 0, 2).astype(np.float64)
    c = synth.normal_f16((1 << 16,), 1.0, 1, 1).astype(np.float64)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.02 and abs(np.corrcoef(a, c)[0, 1]) < 0.02
    assert abs(np.corrcoef(a[:-1], a[1:])[0, 1]) < 0.02


def test_precision_mask_counts_and_seed_dependence():
    m0 = synth.precision_mask(256, 128, 0)
    m1 = synth.precision_mask(256, 128, 1)
    assert m0.sum() == 128 and m1.sum() == 128 and (m0 != m1).any()
    assert np.array_equal(m0, synth.precision_mask(256, 128, 0))
    assert synth.precision_mask(8, 0, 0).sum() == 0 and synth.precision_mask(8, 8, 0).sum() == 8


def test_zipf_bias_is_log_of_normalised_power_law():
    b = synth.zipf_bias(8, 1.2).astype(np.float64)
    assert abs(np.exp(b).sum() - 1) < 1e-6
    assert np.allclose(b[0] - b, 1.2 * np.log(np.arange(1, 9)), atol=1e-6)
