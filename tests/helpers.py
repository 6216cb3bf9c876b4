"""Shared plumbing of the GPU parity tests: upload seeded inputs, call the C-ABI through the binding, fetch
results, and the tolerance checks. No arithmetic of the method lives here."""
import numpy as np

from paper_2605_05899_amd.harness import DeviceLayer, bf16_dev, bf16_host  # noqa: F401  (device plumbing, re-exported)

ID_GAP = 1e-5            # tokens whose k-th / (k+1)-th oracle logit gap is below this are excluded from id parity
MAX_ERR_FRAC = 2e-2      # max|err| <= 2e-2 * max|ref|
MEAN_REL_ERR = 5e-3      # mean|err| / mean|ref| <= 5e-3


def f32_to_bf16_f32(a):
    """Round an fp32 array to bf16 precision (RNE) and widen again: used to hand oracle intermediates to a call."""
    from paper_2605_05899_amd import synth
    return synth.f32_to_bf16(np.asarray(a, dtype=np.float32))


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
