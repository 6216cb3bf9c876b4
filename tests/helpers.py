"""Shared plumbing of the GPU parity tests: upload seeded inputs, call the C-ABI through the binding, fetch
results, and the tolerance checks. No arithmetic of the method lives here."""
import numpy as np

ID_GAP = 1e-5            # tokens whose k-th / (k+1)-th oracle logit gap is below this are excluded from id parity
MAX_ERR_FRAC = 2e-2      # max|err| <= 2e-2 * max|ref|
MEAN_REL_ERR = 5e-3      # mean|err| / mean|ref| <= 5e-3


def bf16_dev(u16, torch):
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_host(t, torch):
    u = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_f32(a):
    """Round an fp32 array to bf16 precision (RNE) and widen again: used to hand oracle intermediates to a call."""
    from paper_2605_05899_amd import synth
    return synth.f32_to_bf16(np.asarray(a, dtype=np.float32))


class DeviceLayer:
    """Device copies of one synthetic layer plus workspace and output buffers."""

    def __init__(self, inp, torch, moe, max_tokens=None):
        self.inp, self.torch, self.moe = inp, torch, moe
        self.cfg = moe.MoEConfig(H=inp.H, I=inp.I, E=inp.E, k=inp.k, S=inp.S, norm_topk=inp.norm_topk,
                                 max_tokens=max_tokens if max_tokens is not None else max(inp.T, 1))
        d = lambda a: None if a is None else bf16_dev(a, torch)
        self.x = d(inp.x)
        self.keep = None if inp.keep_idx is None else torch.from_numpy(inp.keep_idx).cuda()
        self.w_router, self.w_gate, self.w_up, self.w_down = d(inp.w_router), d(inp.w_gate), d(inp.w_up), d(inp.w_down)
        self.ws_gate, self.ws_up, self.ws_down = d(inp.ws_gate), d(inp.ws_up), d(inp.ws_down)
        self.ws = moe.alloc_workspace(self.cfg)
        T, k, H = inp.T, inp.k, inp.H
        self.out = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
        self.ids = torch.zeros((T, k), dtype=torch.int32, device="cuda")
        self.w = torch.zeros((T, k), dtype=torch.float32, device="cuda")

    def forward(self, want_routing=True):
        i = self.inp
        self.moe.moe_layer_forward(self.cfg, self.x, i.T_in, self.keep, i.T, self.w_router, self.w_gate, self.w_up,
                                   self.w_down, self.ws_gate, self.ws_up, self.ws_down, self.out,
                                   self.ids if want_routing else None, self.w if want_routing else None, self.ws)
        self.torch.cuda.synchronize()
        return bf16_host(self.out, self.torch), self.ids.cpu().numpy(), self.w.cpu().numpy()


def oracle_layer(inp, dtype=np.float32):
    from oracle import moe_oracle as O
    return O.moe_layer_forward(inp.x, inp.keep_idx, inp.w_router, inp.w_gate, inp.w_up, inp.w_down, inp.k,
                               inp.norm_topk, inp.ws_gate, inp.ws_up, inp.ws_down, dtype=dtype)


def id_mask(ref, k):
    """True for tokens that take part in bit-exact id comparison."""
    from oracle import moe_oracle as O
    return O.topk_gap(ref["logits"], k) >= ID_GAP


def gate_weight_rtol(ref):
    """Relative tolerance of a gate weight. Both sides add the same H exact bf16 products in fp32, in different orders:
    each of the H additions rounds a partial sum of size at most about P = max(1, max|logit|) by at most 2^-24
    relative, independently, so a logit differs between the sides by at most about 2 sqrt(H) 2^-24 P (six standard
    deviations of the random walk of two sums). A weight is exp(logit - max) normalised, so its relative error is at
    most twice the largest logit error, plus a dozen roundings of the exponential (argument scaling, exp2, sum over
    E <= 512 terms, two divisions): 2e-6."""
    H = ref["xt"].shape[1]
    P = max(1.0, float(np.abs(ref["logits"]).max()))
    return 2e-6 + 4.0 * np.sqrt(H) * 2.0 ** -24 * P


def check_routing(ids, w, ref, k, where=""):
    """ids as per-token sets (bit-exact outside near-ties), weights matched through the expert id."""
    ok = id_mask(ref, k)
    rid, rw = ref["topk_ids"], ref["topk_w"]
    a, b = np.sort(ids[ok], axis=1), np.sort(rid[ok], axis=1)
    assert np.array_equal(a, b), f"{where}: expert ids differ on {int((a != b).any(axis=1).sum())} tokens"
    oa, ob = np.argsort(ids[ok], axis=1), np.argsort(rid[ok], axis=1)
    wa, wb = np.take_along_axis(w[ok], oa, axis=1), np.take_along_axis(rw[ok], ob, axis=1)
    rtol = gate_weight_rtol(ref)
    np.testing.assert_allclose(wa, wb, rtol=rtol, atol=1e-7, err_msg=f"{where}: gate weights")
    np.testing.assert_allclose(w[ok].sum(axis=1), 1.0, atol=1e-5)
    assert np.all(np.diff(w, axis=1) <= 1e-6), f"{where}: slots not in descending order"
    return ok


def check_out(got, ref_out, ok_rows=None, where=""):
    ref_out = np.asarray(ref_out, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ok_rows is not None:
        got, ref_out = got[ok_rows], ref_out[ok_rows]
    if ref_out.size == 0:
        return 0.0, 0.0
    err = np.abs(got - ref_out)
    max_frac = err.max() / np.abs(ref_out).max()
    mean_rel = err.mean() / np.abs(ref_out).mean()
    assert max_frac <= MAX_ERR_FRAC, f"{where}: max|err|/max|ref| = {max_frac:.3e}"
    assert mean_rel <= MEAN_REL_ERR, f"{where}: mean|err|/mean|ref| = {mean_rel:.3e}"
    return max_frac, mean_rel
