"""Pins of the token-compressor oracle (paper Alg. 1, Eq. 1-5) against things other than itself."""
import json
import os

import numpy as np
import pytest

from oracle import compress_oracle as CO
from paper_2605_05899_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def _tiny():
    with open(os.path.join(HERE, "golden", "compress_tiny.json")) as f:
        g = json.load(f)
    return g, np.array(g["A"], dtype=np.float32), np.array(g["R"], dtype=np.int32)


def test_hand_worked_example():
    g, A, R = _tiny()
    out = CO.token_compress(A, R, g["E"], g["alpha"], g["beta"], g["lambda"])
    e = g["expect"]
    assert out["I_keep"].tolist() == e["I_keep"]
    assert out["I_core"].tolist() == e["I_core"]
    assert out["E_target"] == e["E_target"]
    np.testing.assert_allclose(out["s_norm"], e["s_norm"], atol=2e-7)
    np.testing.assert_allclose(out["delta"], e["delta"], atol=2e-7)
    for i, v in e["p_noncore"].items():
        assert abs(float(out["p"][int(i)]) - v) < 5e-7
    # lambda = 0 on the same instance is the plain saliency top-5 the example names
    assert CO.token_compress(A, R, g["E"], g["alpha"], g["beta"], 0.0)["I_keep"].tolist() == e["saliency_only_top5"]


def _brute_force(A, R, E, alpha, beta, lam):
    """The compressor token by token over Python sets and a full sort (Eq. 1-5 as written), sharing nothing with the
    array formulation of the oracle but the fp32 saliency."""
    N = A.shape[1]
    f = np.float32
    s = CO.normalize(CO.head_mean_saliency(A))
    K_core, K_keep = int(np.floor(alpha * N)), int(np.floor(beta * N))
    ranked = sorted(range(N), key=lambda i: (-float(s[i]), i))
    core = set(ranked[:K_core])
    experts = [{int(e) for e in R[:, i, :].ravel() if 0 <= int(e) < E} for i in range(N)]
    target = set().union(*[experts[j] for j in core]) if core else set()
    score, delta = {}, np.zeros(N, dtype=f)
    for i in range(N):
        if i in core:
            continue
        if experts[i]:
            delta[i] = f(len(experts[i] - target)) / f(len(experts[i]))
        score[i] = f(s[i] - f(f(lam) * delta[i]))
    rest = sorted(score, key=lambda i: (-float(score[i]), i))[:K_keep - K_core]
    return sorted(core | set(rest)), delta, score


@pytest.mark.parametrize("seed", [10, 11, 12, 13])
def test_array_formulation_equals_brute_force_over_sets(seed):
    A, R, E = _random_case(seed, N=211, heads=4, E=40, L=3, k=4)
    R = R.copy()
    R[0, ::17, 0] = -1                  # some ids out of range
    R[1, ::23, 1] = E + 3
    for alpha, beta, lam in [(0.1, 0.25, 2.0), (0.0, 0.4, 2.0), (0.25, 0.6, 0.7), (0.3, 0.3, 2.0)]:
        out = CO.token_compress(A, R, E, alpha, beta, lam)
        keep, delta, score = _brute_force(A, R, E, alpha, beta, lam)
        assert out["I_keep"].tolist() == keep
        np.testing.assert_array_equal(out["delta"].view(np.uint32), delta.view(np.uint32))
        for i, v in score.items():
            assert np.float32(out["p"][i]).view(np.uint32) == np.float32(v).view(np.uint32)


def _random_case(seed, N=157, heads=3, E=24, L=2, k=3):
    c = synth.make_compress_small(seed, N=N, n_heads=heads, E=E, L=L, k=k, n_clusters=4)
    return c.A, c.R, E


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_invariants(seed):
    A, R, E = _random_case(seed)
    N = A.shape[1]
    for alpha, beta, lam in [(0.1, 0.25, 2.0), (0.0, 0.5, 2.0), (0.3, 0.3, 2.0), (0.05, 1.0, 0.5), (0.2, 0.21, 7.0)]:
        out = CO.token_compress(A, R, E, alpha, beta, lam)
        keep, core = out["I_keep"], out["I_core"]
        assert len(keep) == int(np.floor(beta * N)) and len(core) == int(np.floor(alpha * N))
        assert len(set(keep.tolist())) == len(keep) and np.all(np.diff(keep) > 0)
        assert set(core.tolist()) <= set(keep.tolist())
        assert np.all(out["delta"] >= 0) and np.all(out["delta"] <= 1)
        assert out["s_norm"].min() == 0 and out["s_norm"].max() == 1
        if alpha == beta:
            assert keep.tolist() == core.tolist()
        # every core token's experts are in the target set, so a core token would score Delta = 0
        T = set(out["E_target"])
        for j in core:
            assert {int(e) for e in R[:, int(j), :].ravel() if 0 <= e < E} <= T


@pytest.mark.parametrize("seed", [3, 4])
def test_lambda_zero_is_saliency_topk(seed):
    A, R, E = _random_case(seed)
    N = A.shape[1]
    out = CO.token_compress(A, R, E, 0.1, 0.4, 0.0)
    s = A.astype(np.float64).mean(axis=0)                   # plain definition, in double
    order = np.lexsort((np.arange(N), -s))
    want = sorted(order[: int(np.floor(0.4 * N))].tolist())
    # double and fp32 saliency can only disagree on the order of near-ties; the synthetic saliency has none
    assert out["I_keep"].tolist() == want


@pytest.mark.parametrize("seed", [5, 6])
def test_alpha_zero_every_delta_is_one(seed):
    A, R, E = _random_case(seed)
    out = CO.token_compress(A, R, E, 0.0, 0.3, 2.0)
    assert out["E_target"] == [] and np.all(out["delta"] == 1)
    ref = CO.token_compress(A, R, E, 0.0, 0.3, 0.0)          # p = s~ - lambda shifts every score alike
    assert out["I_keep"].tolist() == ref["I_keep"].tolist()


@pytest.mark.parametrize("seed", [7, 8])
def test_huge_lambda_prefers_tokens_that_add_nothing(seed):
    A, R, E = _random_case(seed)
    out = CO.token_compress(A, R, E, 0.2, 0.6, 1e6)
    core = set(out["I_core"].tolist())
    extra = [i for i in out["I_keep"].tolist() if i not in core]
    d = out["delta"]
    dropped = [i for i in range(A.shape[1]) if i not in core and i not in set(extra)]
    # with lambda this large the score is ordered by Delta first: no dropped token has a smaller Delta than a kept one
    assert max(d[extra]) <= min(d[dropped])


def test_eq2_equals_eq3_on_multihot_masks():
    A, R, E = _random_case(9)
    out = CO.token_compress(A, R, E, 0.15, 0.5, 2.0)
    m_target = np.zeros(E)
    m_target[out["E_target"]] = 1
    core = set(out["I_core"].tolist())
    for i in range(A.shape[1]):
        if i in core:
            continue
        m = np.zeros(E)
        m[np.unique(R[:, i, :])] = 1
        eq3 = np.abs(m * (1 - m_target)).sum() / np.abs(m).sum()
        assert abs(eq3 - float(out["delta"][i])) < 1e-6


def test_relabelling_experts_changes_nothing():
    A, R, E = _random_case(10)
    perm = np.random.default_rng(0).permutation(E)
    a = CO.token_compress(A, R, E, 0.1, 0.35, 2.0)
    b = CO.token_compress(A, perm[R].astype(np.int32), E, 0.1, 0.35, 2.0)
    assert a["I_keep"].tolist() == b["I_keep"].tolist()
    np.testing.assert_array_equal(a["delta"], b["delta"])


def test_power_of_two_rescaling_of_saliency_changes_nothing():
    A, R, E = _random_case(11)
    a = CO.token_compress(A, R, E, 0.1, 0.35, 2.0)
    b = CO.token_compress(A * np.float32(8.0), R, E, 0.1, 0.35, 2.0)      # exact in floating point
    assert a["I_keep"].tolist() == b["I_keep"].tolist()
    np.testing.assert_array_equal(a["s_norm"], b["s_norm"])


def test_ties_go_to_the_lower_index_and_constant_saliency_normalises_to_zero():
    A = np.ones((2, 10), dtype=np.float32)
    R = np.zeros((1, 10, 1), dtype=np.int32)
    out = CO.token_compress(A, R, 4, 0.2, 0.5, 2.0)
    assert np.all(out["s_norm"] == 0)
    assert out["I_core"].tolist() == [0, 1] and out["I_keep"].tolist() == [0, 1, 2, 3, 4]


def test_out_of_range_ids_are_ignored():
    g, A, R = _tiny()
    R2 = R.copy()
    R2[0, 2, :] = [-1, 99]            # token 2 keeps {5, 6} from the second layer
    out = CO.token_compress(A, R2, g["E"], g["alpha"], g["beta"], g["lambda"])
    assert float(out["delta"][2]) == 1.0
    R2[1, 2, :] = [8, 1000]           # now no valid id at all
    out = CO.token_compress(A, R2, g["E"], g["alpha"], g["beta"], g["lambda"])
    assert float(out["delta"][2]) == 0.0


# ---- planted mistakes: each plausible slip must break the hand-worked example
def _run_mutant(monkeypatch, **patches):
    g, A, R = _tiny()
    for name, fn in patches.items():
        monkeypatch.setattr(CO, name, fn)
    return CO.token_compress(A, R, g["E"], g["alpha"], g["beta"], g["lambda"]), g["expect"]


def test_mutation_smallest_instead_of_largest(monkeypatch):
    out, e = _run_mutant(monkeypatch, largest=lambda v, ok, K: np.array(
        sorted(np.flatnonzero(ok).tolist(), key=lambda i: (float(v[i]), i))[:K], dtype=np.int64))
    assert out["I_keep"].tolist() != e["I_keep"]


def test_mutation_only_first_prefix_layer(monkeypatch):
    full = CO.membership
    out, e = _run_mutant(monkeypatch, membership=lambda R, E: full(np.asarray(R)[:1], E))
    assert out["I_keep"].tolist() != e["I_keep"] and not np.allclose(out["delta"], e["delta"])


def test_mutation_no_normalisation(monkeypatch):
    out, e = _run_mutant(monkeypatch, normalize=lambda s: np.asarray(s, dtype=np.float32))
    assert not np.allclose(out["s_norm"], e["s_norm"])


def test_mutation_max_over_heads_instead_of_mean(monkeypatch):
    g, A, R = _tiny()
    A2 = A.copy()
    A2[1, 7] = 0.0       # head mean of token 7 drops to 0.3, its head max stays 0.6
    good = CO.token_compress(A2, R, g["E"], g["alpha"], 0.625, 0.0)
    assert good["I_keep"].tolist() == [1, 3, 4, 5, 6]        # means 0.8 0.8 0.5, then the 0.3 tie in index order
    monkeypatch.setattr(CO, "head_mean_saliency", lambda A: np.asarray(A, dtype=np.float32).max(axis=0))
    bad = CO.token_compress(A2, R, g["E"], g["alpha"], 0.625, 0.0)
    assert good["I_keep"].tolist() != bad["I_keep"].tolist()
