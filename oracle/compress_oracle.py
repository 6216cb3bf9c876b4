"""CPU oracle for the affinity-aware token compressor -- TEST INFRASTRUCTURE, not part of the product path.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file. It shares no code with the
HIP library and never imports it.

What the compressor does (paper Sec. 3.2, Alg. 1, Eq. 1-5), written here as a data flow over whole arrays:

  1. saliency     one number per visual token: the attention it receives, averaged over the heads, then rescaled
                  so that the smallest value is 0 and the largest 1;
  2. core         the floor(alpha N) most salient tokens; they are always kept;
  3. membership   a boolean matrix M [N, E]: M[i, e] says that token i was routed to expert e in at least one of
                  the pinned-prefix layers; the experts the core touches are the columns with a True in a core row;
  4. novelty      per token, the share of its experts (True entries of its row) that the core does not touch;
  5. score        saliency minus lambda times novelty, for the tokens outside the core;
  6. fill         the floor(beta N) - floor(alpha N) best-scoring outside tokens join the core.

Where the paper is silent this file takes these readings (they are also listed in the design notes):
  * the attention maps arrive as [n_heads, N]: per head, the attention each visual token receives (the reduction
    over the query axis is the vision encoder's business);
  * the rescaling is min-max; all-equal saliency rescales to 0;
  * a selection takes the largest values, ties go to the lower token index;
  * floor(alpha N) and floor(beta N) are taken on the double-precision product;
  * ids outside [0, E) are ignored; a token with no valid id has novelty 0;
  * the kept indices are returned in ascending token order (the paper defines a set).
Scores decide an integer result (which tokens are kept), so the scores are computed in the precision the device
uses, fp32, one rounding per operation and the head sum in head order: the selection is then comparable bit for bit.

Pins (tests/test_compress_oracle_pins.py): a hand-worked example (tests/golden/compress_tiny.json); a brute-force
version over Python sets, token by token, that must give the same indices and scores; the invariants
|kept| = floor(beta N), core inside kept, novelty in [0, 1]; lambda = 0 => plain saliency selection; alpha = beta =>
core only; alpha = 0 => saliency order again (every novelty is 1); huge lambda => tokens that add no expert come
first; invariance under relabelling experts and under rescaling of the saliency by powers of two; planted mistakes
that each break a pin.
"""
from __future__ import annotations

import math
from typing import Dict

import numpy as np

F = np.float32


def head_mean_saliency(A: np.ndarray) -> np.ndarray:
    """Step 1, first half: fp32 sum over heads in head order, then one division."""
    A = np.asarray(A, dtype=F)
    s = np.zeros(A.shape[1], dtype=F)
    for h in range(A.shape[0]):
        s = (s + A[h]).astype(F)
    return (s / F(A.shape[0])).astype(F)


def normalize(s: np.ndarray) -> np.ndarray:
    """Step 1, second half: min-max rescaling to [0, 1]; constant input gives zeros."""
    s = np.asarray(s, dtype=F)
    if s.size == 0:
        return s.copy()
    lo, hi = F(s.min()), F(s.max())
    rng = F(hi - lo)
    if not rng > 0:
        return np.zeros_like(s)
    return ((s - lo).astype(F) / rng).astype(F)


def largest(values: np.ndarray, allowed: np.ndarray, K: int) -> np.ndarray:
    """Indices of the K largest values among the allowed positions, ties to the lower index (a stable sort of the
    negated values keeps equal values in index order)."""
    idx = np.flatnonzero(allowed)
    order = np.argsort(-np.asarray(values, dtype=F)[idx], kind="stable")
    return idx[order[:K]]


def membership(R: np.ndarray, E: int) -> np.ndarray:
    """Step 3: M[i, e] = token i was routed to expert e in some prefix layer. R: [L, N, k] ids."""
    R = np.asarray(R)
    L, N, k = R.shape
    M = np.zeros((N, E), dtype=bool)
    tok = np.broadcast_to(np.arange(N)[None, :, None], R.shape)
    ok = (R >= 0) & (R < E)
    M[tok[ok], R[ok]] = True
    return M


def token_compress(A: np.ndarray, R: np.ndarray, E: int, alpha: float, beta: float, lam: float) -> Dict[str, object]:
    """The whole compressor. A: [n_heads, N] float; R: [L, N, k] int expert ids. Returns the kept indices
    (ascending) under the paper's name I_keep, and the intermediates."""
    A = np.asarray(A, dtype=F)
    N = A.shape[1]
    K_core = int(math.floor(float(alpha) * N))
    K_keep = int(math.floor(float(beta) * N))
    if K_keep < K_core or K_keep > N:
        raise ValueError("need 0 <= alpha <= beta <= 1")
    s_norm = normalize(head_mean_saliency(A))
    in_core = np.zeros(N, dtype=bool)
    in_core[largest(s_norm, np.ones(N, dtype=bool), K_core)] = True
    M = membership(R, E)
    touched = M[in_core].any(axis=0)                          # experts the core brings in anyway
    n_own = M.sum(axis=1)
    n_new = (M & ~touched[None, :]).sum(axis=1)
    delta = np.zeros(N, dtype=F)
    has = (n_own > 0) & ~in_core
    delta[has] = n_new[has].astype(F) / n_own[has].astype(F)
    p = np.zeros(N, dtype=F)
    penalty = (F(lam) * delta).astype(F)
    p[~in_core] = (s_norm - penalty).astype(F)[~in_core]
    extra = largest(p, ~in_core, K_keep - K_core)
    kept = in_core.copy()
    kept[extra] = True
    return {"I_keep": np.flatnonzero(kept).astype(np.int32), "I_core": np.flatnonzero(in_core).astype(np.int32),
            "s_norm": s_norm, "delta": delta, "p": p, "E_target": np.flatnonzero(touched).tolist(), "K_core": K_core,
            "K_keep": K_keep}
