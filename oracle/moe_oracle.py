"""CPU oracle for one top-k MoE layer forward -- TEST INFRASTRUCTURE, not part of the product path.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file. It shares no code with
the HIP library and never imports it.

What it computes is the plain definition of the layer the paper treats as a black box (Sec. 2.1: feed-forward
blocks replaced by sparse MoE layers where each token activates a few experts; Table 2: E=128/top-8, E=72/top-6
plus 2 shared experts; Sec. 3.4.1: shared experts serve every token; Sec. 3.2 / 3.4.1: after pruning, layers run
on the retained-token stream I_keep). The paper gives no formula, so the definition below is the standard one:

  0. xt[j] = x[keep_idx[j]]                       (or x[j] when there is no index list)
  1. logit[j,e] = <xt[j], Wr[e]>
  2. top-k experts by logit; ties go to the lower expert index; listed in descending logit order
  3. p = softmax(logit[j,:]) over all E; w[j,s] = p[e_s] / sum_s' p[e_s']  (or p[e_s] if norm_topk == 0)
  4. counts per expert, expert_offsets = exclusive prefix sum
  5. the assignment (j,s) of expert e sits at offsets[e] + #{assignments of e from tokens j' < j}
  6. per assignment: hm = silu(Wg[e] xt[j]) * (Wu[e] xt[j]),  y = Wd[e] hm,   silu(a) = a / (1 + exp(-a))
  7. out[j] = sum_s w[j,s] * y[pos(j,s)] + sum_shared FFN_shared(xt[j])

All inputs are bf16 (uint16 storage); bf16 -> float is exact. Arithmetic is in `dtype`: np.float32 by default
(the precision the task fixes for the reference), np.float64 as the oracle's own error bar. No intermediate is
rounded to bf16 and the output stays in `dtype`. Matrix products are numpy matmuls (a library primitive used as
one step); there is no blocking, fusion or reordering beyond the steps above.

Pins (tests/test_oracle_pins.py): brute-force dense all-experts evaluation in pure Python, a hand-worked tiny
layer (tests/golden/), top-k against a full sort, weights against the softmax over the selected logits, the
permutation's bijection/ordering invariants, the E=1,k=1 identity against textbook GEMVs, shared experts against
the concatenated FFN, silu identities, gather identities. The absolute output values on the five benchmark
configs have no printed example to compare with: beyond the pins above that part is "parity unpinned".
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def bf16_to_float(u16: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Exact widening of bf16 storage to float."""
    u = np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(dtype, copy=False)


def gather_tokens(x_bf16: np.ndarray, keep_idx: Optional[np.ndarray], dtype=np.float32) -> np.ndarray:
    """Step 0. Returns xt [T, H]."""
    x = bf16_to_float(x_bf16, dtype)
    if keep_idx is None:
        return x
    return x[np.asarray(keep_idx, dtype=np.int64)]


def router_logits(xt: np.ndarray, w_router_bf16: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Step 1. logits [T, E]."""
    wr = bf16_to_float(w_router_bf16, dtype)
    return (xt @ wr.T).astype(dtype, copy=False)


def topk_experts(logits: np.ndarray, k: int) -> np.ndarray:
    """Step 2. ids [T, k] int32, descending logit, ties to the lower expert index."""
    order = np.argsort(-logits, axis=1, kind="stable")      # stable: equal logits keep ascending index
    return order[:, :k].astype(np.int32)


def gate_weights(logits: np.ndarray, ids: np.ndarray, norm_topk: int = 1) -> np.ndarray:
    """Step 3. w [T, k] in the dtype of logits."""
    dtype = logits.dtype
    m = logits.max(axis=1, keepdims=True)
    ex = np.exp(logits - m)
    p = ex / ex.sum(axis=1, keepdims=True, dtype=dtype)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    if norm_topk:
        w = w / w.sum(axis=1, keepdims=True, dtype=dtype)
    return w.astype(dtype, copy=False)


def dispatch(ids: np.ndarray, E: int):
    """Steps 4-5. Returns (expert_offsets [E+1], sorted_token [T*k], inv_perm [T*k]), all int32.

    sorted_token[pos] is the (compact) token row feeding position pos of the expert-grouped order;
    inv_perm[j*k+s] is the position of assignment (j, s)."""
    T, k = ids.shape
    counts = np.zeros(E, dtype=np.int64)
    for e in ids.reshape(-1):
        counts[e] += 1
    offsets = np.zeros(E + 1, dtype=np.int64)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:-1].copy()
    sorted_token = np.empty(T * k, dtype=np.int32)
    inv_perm = np.empty(T * k, dtype=np.int32)
    for j in range(T):                      # ascending token index => ascending order inside each group
        for s in range(k):
            e = ids[j, s]
            pos = cursor[e]
            cursor[e] += 1
            sorted_token[pos] = j
            inv_perm[j * k + s] = pos
    return offsets.astype(np.int32), sorted_token, inv_perm


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def swiglu_ffn(X: np.ndarray, wg_bf16: np.ndarray, wu_bf16: np.ndarray, wd_bf16: np.ndarray, dtype=np.float32):
    """One expert on a block of rows X [n, H]: Wd (silu(Wg x) * (Wu x)). Weights are [I,H], [I,H], [H,I]."""
    Wg = bf16_to_float(wg_bf16, dtype)
    Wu = bf16_to_float(wu_bf16, dtype)
    Wd = bf16_to_float(wd_bf16, dtype)
    G = X @ Wg.T
    U = X @ Wu.T
    Hm = silu(G) * U
    return (Hm @ Wd.T).astype(dtype, copy=False)


def expert_ffn(xt: np.ndarray, expert_offsets: np.ndarray, sorted_token: np.ndarray,
               w_gate: np.ndarray, w_up: np.ndarray, w_down: np.ndarray, dtype=np.float32) -> np.ndarray:
    """Step 6. y_sorted [T*k, H] in expert-grouped order."""
    E = w_gate.shape[0]
    H = xt.shape[1]
    y = np.zeros((len(sorted_token), H), dtype=dtype)
    for e in range(E):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        rows = sorted_token[lo:hi].astype(np.int64)
        y[lo:hi] = swiglu_ffn(xt[rows], w_gate[e], w_up[e], w_down[e], dtype)
    return y


def expert_ffn_slabs(xt: np.ndarray, expert_offsets: np.ndarray, sorted_token: np.ndarray, slabs, I: int,
                     dtype=np.float32):
    """Step 6 with the weights addressed through a per-expert slab table (paper Sec. 3.4.2: the expert cache is a set of
    equal-sized slots holding one expert each). slabs[e] is None when expert e is not resident,
    else a flat bf16 array [gate (I x H) | up (I x H) | down (H x I)]. Rows of a non-resident expert are not computed
    (they stay zero); the experts that have rows but no slab are reported, in ascending order.
    Returns (y_sorted [T*k, H], missing list)."""
    H = xt.shape[1]
    y = np.zeros((len(sorted_token), H), dtype=dtype)
    missing = []
    for e in range(len(slabs)):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        if slabs[e] is None:
            missing.append(e)
            continue
        flat = np.asarray(slabs[e])
        wg = flat[: I * H].reshape(I, H)
        wu = flat[I * H: 2 * I * H].reshape(I, H)
        wd = flat[2 * I * H: 3 * I * H].reshape(H, I)
        rows = sorted_token[lo:hi].astype(np.int64)
        y[lo:hi] = swiglu_ffn(xt[rows], wg, wu, wd, dtype)
    return y, missing


def shared_ffn(xt: np.ndarray, ws_gate, ws_up, ws_down, dtype=np.float32) -> Optional[np.ndarray]:
    """Sum of the S always-on experts applied to every token (weight 1 each); None when S == 0."""
    if ws_gate is None or len(ws_gate) == 0:
        return None
    acc = np.zeros((xt.shape[0], ws_down.shape[1]), dtype=dtype)
    for s in range(ws_gate.shape[0]):
        acc += swiglu_ffn(xt, ws_gate[s], ws_up[s], ws_down[s], dtype)
    return acc


def combine(y_sorted: np.ndarray, inv_perm: np.ndarray, w: np.ndarray, ysh: Optional[np.ndarray]) -> np.ndarray:
    """Step 7. out [T, H]."""
    T, k = w.shape
    pos = inv_perm.reshape(T, k).astype(np.int64)
    out = np.zeros((T, y_sorted.shape[1]), dtype=y_sorted.dtype)
    for s in range(k):
        out += w[:, s:s + 1].astype(y_sorted.dtype) * y_sorted[pos[:, s]]
    if ysh is not None:
        out += ysh
    return out


def moe_layer_forward(x, keep_idx, w_router, w_gate, w_up, w_down, k: int, norm_topk: int = 1,
                      ws_gate=None, ws_up=None, ws_down=None, dtype=np.float32) -> dict:
    """Steps 0-7. Returns every intermediate so each C-ABI call can be compared with its own step."""
    E = w_router.shape[0]
    xt = gather_tokens(x, keep_idx, dtype)
    logits = router_logits(xt, w_router, dtype)
    ids = topk_experts(logits, k)
    w = gate_weights(logits, ids, norm_topk)
    offsets, sorted_token, inv_perm = dispatch(ids, E)
    y_sorted = expert_ffn(xt, offsets, sorted_token, w_gate, w_up, w_down, dtype)
    ysh = shared_ffn(xt, ws_gate, ws_up, ws_down, dtype)
    out = combine(y_sorted, inv_perm, w, ysh)
    return dict(xt=xt, logits=logits, topk_ids=ids, topk_w=w, expert_offsets=offsets, sorted_token=sorted_token,
                inv_perm=inv_perm, y_sorted=y_sorted, shared_out=ysh, out=out)


def topk_gap(logits: np.ndarray, k: int) -> np.ndarray:
    """Per token: logit of the k-th selected expert minus the best unselected logit (inf when k == E).
    Tokens whose gap is below the parity threshold are excluded from bit-exact id comparison."""
    srt = -np.sort(-logits, axis=1)
    if k >= logits.shape[1]:
        return np.full(logits.shape[0], np.inf)
    return (srt[:, k - 1] - srt[:, k]).astype(np.float64)
