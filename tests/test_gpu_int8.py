"""8-bit experts (the precision of the paper's homogeneous 8-bit model, Table 1) through the library: the format
hooks bit for bit, the expert alone, the block with 16-bit, 8-bit and 4-bit experts side by side, one token and many."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2407_14417_amd import binding as mm
from paper_2407_14417_amd import synth
from tests import common
from tests.common import assert_ffn_close, build_workload
from tests.gpu_common import dev, device_layer, device_mat

pytestmark = pytest.mark.gpu
GATE_ATOL = 2e-6


@pytest.mark.parametrize("shape,sigma", [((64, 256), 0.02), ((301, 1088), 0.02), ((17, 64), 1.0), ((4, 4096), 3e-4)])
def test_device_quantizer_and_dequantizer_bit_exact(orc, shape, sigma):
    w = synth.normal_f16(shape, sigma, 9, 5)
    ref = orc.quantize_int8(w)
    m = mm.quantize_mat8(dev(w))
    assert np.array_equal(m.data.cpu().numpy(), ref.data)
    assert np.array_equal(m.scale.cpu().numpy().view(np.uint16), ref.scale.view(np.uint16))
    assert np.array_equal(m.zero.cpu().numpy().view(np.uint16), ref.zero.view(np.uint16))
    out = torch.empty(shape, dtype=torch.float16, device="cuda")
    mm.moe_dequant_int8(m, shape[0], shape[1], out)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), orc.dequant_int8(ref).view(np.uint16))


def test_dequant_all_codes_sampled_scales(orc):
    rng = np.random.default_rng(3)
    n = 128
    q = np.tile(np.arange(256, dtype=np.uint8), (n, 1))
    s = np.repeat((np.abs(rng.standard_normal(n)) * 5e-4).astype(np.float16)[:, None], 4, axis=1).copy()
    z = np.repeat((-np.abs(rng.standard_normal(n)) * 5e-2).astype(np.float16)[:, None], 4, axis=1).copy()
    ref = orc.dequant_int8(orc.Mat(q, s, z, bits=8))
    out = torch.empty((n, 256), dtype=torch.float16, device="cuda")
    mm.moe_dequant_int8(device_mat(orc.Mat(q, s, z, bits=8)), n, 256, out)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), ref.view(np.uint16))


CASES = [
    common.Config("int8_tiny", 256, 512, 4, 2, 16, (1,), int8_experts=(0, 3)),
    common.Config("int8_medium", 1024, 2816, 8, 2, 24, (1, 5), int8_experts=(0, 2, 7)),
    common.Config("int8_odd_steps", 640, 896, 8, 2, 40, (0, 4), int8_experts=(1, 3, 6)),
    common.Config("int8_generic", 192, 320, 4, 2, 9, (1,), int8_experts=(2,)),
    common.Config("int8_many_rows", 1024, 2048, 4, 2, 300, (), int8_experts=(0, 1, 2, 3)),
    # launches with 128-row chunks of the kernel variant that holds the 8-bit body: the 16-bit experts (most of the
    # rows) run the pipelined direct-operand body with chunks of up to 256 rows, the others the plain one
    common.Config("int8_three_precisions_zipf", 1024, 2048, 8, 2, 420, (2, 3), int8_experts=(4, 5, 6, 7), zipf=1.2),
    common.Config("int8_decode_small", 2048, 4096, 8, 2, 1, (1, 5), int8_experts=(0, 2, 4, 7)),
    common.Config("int8_decode_all", 4096, 2048, 4, 2, 1, (), int8_experts=(0, 1, 2, 3)),
    common.Config("int8_decode_top3", 2048, 6144, 6, 3, 1, (0,), int8_experts=(1, 2, 4)),
]


@pytest.mark.parametrize("cfg", CASES, ids=lambda c: c.name)
def test_layer_forward_with_8bit_experts(orc, cfg):
    wl = build_workload(cfg, orc)
    layer = device_layer(wl)
    tokens = [wl.x] if cfg.T > 1 else [synth.normal_f16((1, cfg.d), 1.0, cfg.seed, synth.x_stream(r)) for r in range(5)]
    ws = mm.alloc_workspace(layer, cfg.T)
    seen = set()
    for x in tokens:
        if cfg.T == 1:
            lg = np.sort(common.logits_f64(x, wl.wg, None)[0])[::-1]
            if (lg[:cfg.k] - lg[1:cfg.k + 1]).min() < 1e-3:
                continue
        print(f"{cfg.name} T={x.shape[0]}", flush=True)
        out = torch.full((x.shape[0], cfg.d), float("nan"), dtype=torch.float16, device="cuda")
        idx = torch.empty((x.shape[0], cfg.k), dtype=torch.int32, device="cuda")
        gate = torch.empty((x.shape[0], cfg.k), dtype=torch.float32, device="cuda")
        mm.moe_layer_forward(layer, dev(x), out, ws, idx, gate)
        assert mm.moe_read_status(ws) == 0
        ref, ref_idx, ref_gate = orc.layer_forward(x, wl.wg, wl.experts, cfg.k, bias=wl.bias)
        assert np.array_equal(idx.cpu().numpy(), ref_idx)
        assert np.allclose(gate.cpu().numpy(), ref_gate, rtol=0, atol=GATE_ATOL)
        assert_ffn_close(out.cpu().numpy(), ref, cfg.name)
        seen.update(int(e) for e in ref_idx.reshape(-1))
    assert seen & set(cfg.int8_experts), "no token met an 8-bit expert"


@pytest.mark.parametrize("cfg", [CASES[0], CASES[1], CASES[5]], ids=lambda c: c.name)
@pytest.mark.parametrize("n", [1, 3, 17, 40])
def test_expert_ffn_8bit_alone(orc, cfg, n):
    e = cfg.int8_experts[0]
    wl = build_workload(cfg, orc, experts_needed=(e,))
    layer = device_layer(wl)
    x = synth.normal_f16((n, cfg.d), 1.0, 31, synth.x_stream(0))
    ws = mm.alloc_workspace(layer, (n + cfg.k - 1) // cfg.k)
    y = torch.full((n, cfg.d), float("nan"), dtype=torch.float32, device="cuda")
    mm.moe_expert_ffn_mixed(layer, e, dev(x), y, ws)
    assert_ffn_close(y.cpu().numpy(), orc.expert_ffn(wl.experts[e], x), f"{cfg.name} n={n}")
