"""ramp_fused_moe_static (the entry point for callers that cannot allocate: its workspace is a device array inside
the library image) against ramp_fused_moe with a caller-provided workspace, through the C ABI: same bits, on two
calls in a row that share the built-in array, the second with a smaller input; sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

from paper_2604_26039_amd import ramp, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(s, T, beta, seed):
    ids, w = synth.routing(T, s, beta, seed=seed)
    return (torch.from_numpy(np.ascontiguousarray(ids, np.int32)).to(DEV),
            torch.from_numpy(np.ascontiguousarray(w, np.float32)).to(DEV))


def test_static_workspace_entry_point_matches_fused_moe():
    s = synth.SHAPES["olmoe"]
    T_max = 192
    X, Wg, Wu, Wd = synth.layer_tensors(s, T_max, seed=11, device=DEV, x_std=1.0)
    rs_max = ramp.Shape(T_max, s.k, s.E, s.H, s.I)
    packed = torch.empty(ramp.pack_bytes(rs_max), dtype=torch.uint8, device=DEV)
    ramp.pack_weights(rs_max, Wg, Wu, Wd, packed)
    torch.cuda.synchronize()
    checked = 0
    for cfg in ramp.configs(rs_max):
        if ramp.fused_moe_workspace_bytes(rs_max, cfg) > ramp.STATIC_WS_BYTES:
            continue
        if checked % 4 and not (cfg.mode & 0x400):   # every fourth configuration plus the ping-pong ones
            checked += 1
            continue
        checked += 1
        # two calls in a row on the shared built-in array: a larger batch, then a smaller one with other routing
        for T, beta, seed in ((T_max, 0.5, 1), (40, 0.2, 2)):
            rs = ramp.Shape(T, s.k, s.E, s.H, s.I)
            d_ids, d_w = _inputs(s, T, beta, seed)
            got = torch.full((T + 1, s.H), 777.0, dtype=torch.bfloat16, device=DEV)
            ramp.fused_moe_static(rs, cfg, X[:T], d_ids, d_w, packed, got)
            ref = torch.zeros((T, s.H), dtype=torch.bfloat16, device=DEV)
            ws = torch.full((ramp.fused_moe_workspace_bytes(rs, cfg),), 0xFF, dtype=torch.uint8, device=DEV)
            ramp.fused_moe(rs, cfg, X[:T], d_ids, d_w, packed, ref, ws)
            torch.cuda.synchronize()
            assert (got[T] == 777.0).all(), "write past the output"
            assert torch.isfinite(ref.float()).all() and ref.float().abs().max() > 0
            assert torch.equal(got[:T].view(torch.int16), ref.view(torch.int16)), f"{cfg} T={T}"
    assert checked >= 8


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    s = synth.SHAPES["olmoe"]
    T = 4096                                         # per-pair rows alone are 128 MB
    rs = ramp.Shape(T, s.k, s.E, s.H, s.I)
    cfg = ramp.configs(rs)[0]
    assert ramp.fused_moe_workspace_bytes(rs, cfg) > ramp.STATIC_WS_BYTES
    small = torch.zeros(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(ramp.RampError) as ei:
        ramp.fused_moe_static(rs, cfg, small, small, small, small, small)
    assert ei.value.status == ramp.ENOSPC
    assert "built-in" in ramp.last_error()
    with pytest.raises(ramp.RampError) as ei:        # configuration not in the family: refused before anything else
        ramp.fused_moe_static(rs, ramp.Config(24, 64, 128, 2, 2, 0), small, small, small, small, small)
    assert ei.value.status == ramp.EUNSUPPORTED
