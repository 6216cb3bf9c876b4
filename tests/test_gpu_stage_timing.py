"""Stage timing: a call reports only the stages it ran; stages of an earlier call read 0."""
import numpy as np
import pytest

from paper_2605_05899_amd import synth
from tests import helpers as Hp

pytestmark = pytest.mark.gpu


def test_standalone_calls_do_not_report_stale_stages():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_05899_amd import moe
    inp = synth.make_small(301, 300, 256, 8, 2, 128, 1, n_text=30)
    d = Hp.DeviceLayer(inp, torch, moe)
    ref = Hp.oracle_layer(inp)
    T, k, E, H = inp.T, inp.k, inp.E, inp.H
    off = torch.from_numpy(ref["expert_offsets"]).cuda()
    st = torch.from_numpy(ref["sorted_token"]).cuda()
    y = torch.zeros((T * k, H), dtype=torch.bfloat16, device="cuda")
    sh = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    moe.moe_stage_timing_enable(True)
    try:
        d.forward()
        fused = moe.moe_stage_timing_read()
        assert all(v > 0 for v in fused), fused
        moe.moe_expert_ffn(d.cfg, d.x, inp.T_in, d.keep, T, off, st, d.w_gate, d.w_up, d.w_down, y, d.ws)
        ffn = moe.moe_stage_timing_read()
        assert ffn[0] == 0 and ffn[1] == 0 and ffn[4] == 0 and ffn[2] > 0 and ffn[3] > 0, ffn
        moe.moe_shared_ffn(d.cfg, d.x, inp.T_in, d.keep, T, d.ws_gate, d.ws_up, d.ws_down, sh, d.ws)
        shared = moe.moe_stage_timing_read()
        assert shared[0] == 0 and shared[1] == 0 and shared[2] > 0 and shared[3] > 0 and shared[4] > 0, shared
        moe.moe_route(d.cfg, d.x, inp.T_in, d.keep, T, d.w_router, d.ids, d.w, d.ws)
        route = moe.moe_stage_timing_read()
        assert route[0] > 0 and not any(route[1:]), route
    finally:
        moe.moe_stage_timing_enable(False)
    torch.cuda.synchronize()
