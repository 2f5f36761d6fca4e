"""Expert-miss path (paper section 3: swap space for experts that live in host memory): moe_layer_forward_swap
against moe_layer_forward with every expert resident, and against the oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2407_14417_amd import binding as mm
from tests import common
from tests.common import TINY, MEDIUM, STEPS4_ZIPF, STEPS4_ZIPF_Q, DECODE_SMALL, build_workload, assert_ffn_close
from tests.gpu_common import dev, device_layer, device_layer_with_offloaded

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _forward(layer, x, cfg):
    out = torch.empty_like(x)
    idx = torch.empty((x.shape[0], cfg.k), dtype=torch.int32, device="cuda")
    ws = mm.alloc_workspace(layer, x.shape[0])
    mm.moe_layer_forward(layer, x, out, ws, idx, None)
    assert mm.moe_read_status(ws) == 0
    return out.cpu().numpy(), idx.cpu().numpy()


# (STEPS4_ZIPF: launches with 128-row chunks; the 16-bit experts 0 and 1 hold most rows and run in chunks of up to
# 256 rows on the pipelined bodies, whether they are resident or come through the swap space; STEPS4_ZIPF_Q: the same
# for 4-bit experts in chunks of 9 tiles)
@pytest.mark.parametrize("cfg", [TINY, MEDIUM, STEPS4_ZIPF, STEPS4_ZIPF_Q], ids=lambda c: c.name)
@pytest.mark.parametrize("offloaded,n_slots", [((0, 3), 1), ((0, 3), 2), ((1, 2, 3), 2), ((0, 1, 2, 3), 4), ((), 1)])
def test_swap_many_tokens_equals_all_resident_bit_for_bit(orc, cfg, offloaded, n_slots):
    wl = build_workload(cfg, orc)
    x = dev(wl.x)
    want, want_idx = _forward(device_layer(wl), x, cfg)
    layer, hosts = device_layer_with_offloaded(wl, set(offloaded))
    swap = mm.Swap(layer, hosts, n_slots, cfg.T)
    ws = mm.alloc_workspace(layer, cfg.T)
    out = torch.empty_like(x)
    idx = torch.empty((cfg.T, cfg.k), dtype=torch.int32, device="cuda")
    _say(f"swap cfg={cfg.name} offloaded={offloaded} slots={n_slots}")
    missed = mm.moe_layer_forward_swap(layer, swap, x, out, ws, idx, None)
    assert mm.moe_read_status(ws) == 0
    routed = set(int(e) for e in want_idx.reshape(-1))
    assert missed == len(routed & set(offloaded))
    assert np.array_equal(idx.cpu().numpy(), want_idx)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), want.view(np.uint16))
    ref, _, _ = orc.layer_forward(wl.x, wl.wg, wl.experts, cfg.k, bias=wl.bias)
    assert_ffn_close(out.cpu().numpy(), ref, f"swap {cfg.name}")


@pytest.mark.parametrize("which", ["first", "second", "both", "none"])
@pytest.mark.parametrize("n_slots", [1, 2])
def test_swap_one_token_decode_kernels(orc, which, n_slots):
    cfg = DECODE_SMALL
    wl = build_workload(cfg, orc)
    x = dev(wl.x)
    want, want_idx = _forward(device_layer(wl), x, cfg)
    pair = [int(e) for e in want_idx[0]]
    offloaded = {"first": {pair[0]}, "second": {pair[1]}, "both": set(pair), "none": set(range(cfg.E)) - set(pair)}[which]
    layer, hosts = device_layer_with_offloaded(wl, offloaded)
    swap = mm.Swap(layer, hosts, n_slots, 1)
    ws = mm.alloc_workspace(layer, 1)
    out = torch.empty_like(x)
    _say(f"swap decode which={which} slots={n_slots} routed={pair} offloaded={sorted(offloaded)}")
    missed = mm.moe_layer_forward_swap(layer, swap, x, out, ws)
    assert mm.moe_read_status(ws) == 0
    assert missed == len(set(pair) & offloaded)
    got = out.cpu().numpy()
    # the first pass's partial sum is rounded to fp16 before the second pass adds to it: one more rounding, at
    # the magnitude of that partial sum (at most about the output's own scale, 2^-11 relative each)
    bound = 2.0 ** -9 * np.abs(want.astype(np.float64)).max()
    assert np.abs(got.astype(np.float64) - want.astype(np.float64)).max() <= bound
    ref, _, _ = orc.layer_forward(wl.x, wl.wg, wl.experts, cfg.k)
    assert_ffn_close(got, ref, f"swap decode {which}")


def test_swap_missed_expert_without_host_copy_keeps_the_status_bit(orc):
    wl = build_workload(TINY, orc)
    ref_idx, _ = orc.route(wl.x, wl.wg, TINY.k)
    victim = int(ref_idx[0, 0])
    layer, hosts = device_layer_with_offloaded(wl, {victim})
    hosts[victim] = None                                  # nothing to copy from
    swap = mm.Swap(layer, hosts, 1, TINY.T)
    ws = mm.alloc_workspace(layer, TINY.T)
    x = dev(wl.x)
    out = torch.empty_like(x)
    missed = mm.moe_layer_forward_swap(layer, swap, x, out, ws)
    assert missed == 0 and mm.moe_read_status(ws) == mm.STATUS_NOT_RESIDENT
    assert np.isfinite(out.cpu().numpy().astype(np.float64)).all()


def test_swap_rejects_small_slots(orc):
    wl = build_workload(TINY, orc)
    layer, hosts = device_layer_with_offloaded(wl, {0})
    swap = mm.Swap(layer, hosts, 1, TINY.T)
    swap.c.slot_bytes = 256
    ws = mm.alloc_workspace(layer, TINY.T)
    x = dev(wl.x)
    with pytest.raises(mm.MoeError) as ei:
        mm.moe_layer_forward_swap(layer, swap, x, torch.empty_like(x), ws)
    assert ei.value.code == mm.MOE_EWORKSPACE
