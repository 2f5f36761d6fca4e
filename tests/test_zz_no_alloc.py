"""moe_layer_forward_static: the block call whose scratch is a fixed array inside the library (for callers that
cannot allocate).  Two calls in a row through the C-ABI, the second on a smaller input, each compared with
moe_layer_forward on a caller workspace (same kernels: bit for bit) and with the oracle at the block tolerance."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2407_14417_amd import binding as mm
from tests import common
from tests.common import MEDIUM, TINY, assert_ffn_close
from tests.gpu_common import dev, device_layer

pytestmark = pytest.mark.gpu


def _both(layer, x_host, k):
    """(static outputs, workspace outputs) of one block call on x_host."""
    T, d = x_host.shape
    x = dev(x_host)
    res = []
    for static in (True, False):
        out = torch.full((T, d), float("nan"), dtype=torch.float16, device="cuda")
        idx = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
        gate = torch.full((T, k), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            mm.moe_layer_forward_static(layer, x, out, idx, gate)
            assert mm.moe_read_status(None) == 0
        else:
            ws = mm.alloc_workspace(layer, T)
            mm.moe_layer_forward(layer, x, out, ws, idx, gate)
            assert mm.moe_read_status(ws) == 0
        torch.cuda.synchronize()
        res.append((out, idx, gate))
    return res


@pytest.mark.parametrize("cfg", [MEDIUM, TINY], ids=lambda c: c.name)
def test_static_scratch_two_calls_second_smaller(orc, cfg):
    wl = common.build_workload(cfg, orc)
    layer = device_layer(wl)
    assert mm.workspace_bytes(layer, cfg.T) <= mm.moe_static_scratch_bytes()
    for n_tok in (cfg.T, max(1, cfg.T // 3)):          # the second call is smaller and reuses the same scratch
        x = np.ascontiguousarray(wl.x[cfg.T - n_tok:])
        print(f"static scratch: {cfg.name} T={n_tok}", flush=True)
        (out_s, idx_s, gate_s), (out_w, idx_w, gate_w) = _both(layer, x, cfg.k)
        assert torch.equal(idx_s, idx_w)
        assert torch.equal(gate_s, gate_w)
        assert torch.equal(out_s, out_w)
        ref, ref_idx, ref_gate = orc.layer_forward(x, wl.wg, wl.experts, cfg.k, wl.bias)
        assert np.array_equal(idx_s.cpu().numpy(), ref_idx)
        assert np.allclose(gate_s.cpu().numpy(), ref_gate, rtol=0, atol=2e-6)
        assert_ffn_close(out_s.cpu().numpy(), ref, f"static {cfg.name} T={n_tok}")


def test_static_scratch_rejects_what_does_not_fit(orc):
    wl = common.build_workload(TINY, orc)
    layer = device_layer(wl)
    T = 1
    while mm.workspace_bytes(layer, T) <= mm.moe_static_scratch_bytes():
        T *= 2
    x = torch.zeros((T, TINY.d), dtype=torch.float16, device="cuda")
    out = torch.empty_like(x)
    with pytest.raises(mm.MoeError) as err:
        mm.moe_layer_forward_static(layer, x, out)
    assert err.value.code == mm.MOE_EWORKSPACE


def test_static_scratch_status_of_a_missing_expert(orc):
    """A routed expert that is not resident raises the status bit in the library's scratch, and the next call
    clears it."""
    wl = common.build_workload(TINY, orc)
    layer_ok = device_layer(wl)
    experts = list(wl.experts)
    saved = experts[0]
    wl.experts = [None] + experts[1:]
    layer_missing = device_layer(wl)
    wl.experts = experts
    assert saved is wl.experts[0]
    x = dev(wl.x)
    out = torch.empty_like(x)
    mm.moe_layer_forward_static(layer_missing, x, out)
    routed = orc.route(wl.x, wl.wg, TINY.k, wl.bias)[0]
    assert (routed == 0).any()
    assert mm.moe_read_status(None) == mm.STATUS_NOT_RESIDENT
    mm.moe_layer_forward_static(layer_ok, x, out)
    assert mm.moe_read_status(None) == 0
