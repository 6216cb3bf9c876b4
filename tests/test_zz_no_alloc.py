"""The fused layer with library-owned static scratch (moe_layer_forward_static) against the entry point it is a
variant of (moe_layer_forward with a caller workspace): bit-identical outputs and routing, on two calls in a row,
the second with a smaller input, plus the oracle's tolerances and the size limit."""
import numpy as np
import pytest

from paper_2605_05899_amd import synth
from tests import helpers as Hp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_05899_amd import moe
    return torch, moe


def _both(torch, moe, inp):
    d = Hp.DeviceLayer(inp, torch, moe)
    out_ws, ids_ws, w_ws = d.forward()
    out2 = torch.full_like(d.out, 7.0)
    ids2 = torch.full_like(d.ids, -1)
    w2 = torch.full_like(d.w, -1.0)
    moe.moe_layer_forward_static(d.cfg, d.x, inp.T_in, d.keep, inp.T, d.w_router, d.w_gate, d.w_up, d.w_down, d.ws_gate,
                                 d.ws_up, d.ws_down, out2, ids2, w2)
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int16), d.out.view(torch.int16)), "outputs differ from moe_layer_forward"
    assert torch.equal(ids2, d.ids) and torch.equal(w2, d.w), "routing differs from moe_layer_forward"
    return Hp.bf16_host(out2, torch), ids2.cpu().numpy(), w2.cpu().numpy()


# (seed, T, H, E, k, I, S, keep_visual, n_text): a tiled prefill with shared experts and a retained-index list,
# then a smaller decode-like batch on the same GPU's scratch (which still holds the first call's contents)
CASES = [(201, 500, 256, 8, 3, 320, 1, 150, 50), (202, 48, 512, 64, 4, 128, 0, None, 48)]


def test_static_scratch_matches_workspace_entry_point_twice_in_a_row(gpu):
    torch, moe = gpu
    for case in CASES:
        seed, T, H, E, k, I, S, keep, n_text = case
        print(f"[case] seed={seed} T={T} H={H} E={E} k={k} I={I} S={S} keep={keep}", flush=True)
        inp = synth.make_small(seed, T, H, E, k, I, S, n_text=n_text, keep_visual=keep)
        out, ids, w = _both(torch, moe, inp)
        ref = Hp.oracle_layer(inp)
        ok = Hp.check_routing(ids, w, ref, k, f"static s{seed}")
        Hp.check_out(out, ref["out"], ok, f"static s{seed}")


def test_static_scratch_rejects_a_config_beyond_its_size(gpu):
    torch, moe = gpu
    cfg = moe.MoEConfig(H=2048, I=768, E=128, k=8, S=0, max_tokens=8192)       # needs 368 MB
    assert moe.moe_workspace_bytes(cfg) > moe.moe_static_scratch_bytes()
    x = torch.zeros((8, 2048), dtype=torch.bfloat16, device="cuda")
    st = moe.moe_layer_forward_static(cfg, x, 8, None, 8, x, x, x, x, None, None, None, x, None, None, check=False)
    assert st == moe.MOE_ERR_WORKSPACE
