"""GPU parity of moe_token_compress (paper Alg. 1, Eq. 1-5) against the CPU oracle, through the C-ABI binding.

The result is an index list decided by fp32 scores; both sides compute the scores in fp32 with the same operation
order, so the comparison is bit-exact: indices, normalised saliency and marginal expansion."""
import numpy as np
import pytest

from oracle import compress_oracle as CO
from paper_2605_05899_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_05899_amd import moe
    return torch, moe


def run_gpu(torch, moe, A, R, E, alpha, beta, lam, ws=None):
    n_heads, N = A.shape
    L, _, k = R.shape
    dA = torch.from_numpy(np.ascontiguousarray(A)).cuda()
    dR = torch.from_numpy(np.ascontiguousarray(R)).cuda()
    K_keep = int(np.floor(beta * N))
    keep = torch.full((max(K_keep, 1),), -7, dtype=torch.int32, device="cuda")
    s_norm = torch.zeros(max(N, 1), dtype=torch.float32, device="cuda")
    delta = torch.zeros(max(N, 1), dtype=torch.float32, device="cuda")
    if ws is None:
        ws = moe.alloc_compress_workspace(N, E)
    moe.moe_token_compress(dA, n_heads, N, dR, L, k, E, alpha, beta, lam, keep, s_norm, delta, ws)
    torch.cuda.synchronize()
    return keep.cpu().numpy()[:K_keep], s_norm.cpu().numpy()[:N], delta.cpu().numpy()[:N]


def check(torch, moe, c, alpha=None, beta=None, lam=None, label=""):
    alpha = c.alpha if alpha is None else alpha
    beta = c.beta if beta is None else beta
    lam = c.lam if lam is None else lam
    print(f"compress case {label or c.name}: N={c.N} E={c.E} alpha={alpha} beta={beta} lambda={lam}", flush=True)
    want = CO.token_compress(c.A, c.R, c.E, alpha, beta, lam)
    keep, s_norm, delta = run_gpu(torch, moe, c.A, c.R, c.E, alpha, beta, lam)
    if want["K_keep"] == 0:          # documented: with an empty budget the call launches nothing and writes nothing
        assert len(keep) == 0 and len(want["I_keep"]) == 0
        return
    np.testing.assert_array_equal(s_norm.view(np.uint32), want["s_norm"].view(np.uint32))
    np.testing.assert_array_equal(delta.view(np.uint32), want["delta"].view(np.uint32))
    np.testing.assert_array_equal(keep, want["I_keep"])


# (seed, N, heads, E, L, k): ragged sizes around the 256-token and 1024-thread granularities, E across mask widths
SMALL = [
    (201, 1, 1, 1, 1, 1),
    (202, 7, 2, 8, 1, 2),
    (203, 255, 3, 24, 2, 3),
    (204, 257, 4, 33, 3, 4),
    (205, 1023, 8, 64, 4, 6),
    (206, 1025, 16, 72, 2, 6),
    (207, 3000, 12, 128, 4, 8),
    (208, 5000, 5, 512, 2, 8),
    (209, 2049, 2, 200, 1, 64),
    (210, 20001, 4, 96, 2, 4),          # five workgroups on the many-workgroup path, a ragged last one
]


@pytest.mark.parametrize("case", SMALL, ids=[f"seed{c[0]}" for c in SMALL])
def test_small_cases(env, case):
    torch, moe = env
    seed, N, heads, E, L, k = case
    c = synth.make_compress_small(seed, N=N, n_heads=heads, E=E, L=L, k=min(k, E), n_clusters=4)
    for alpha, beta, lam in [(0.1, 0.25, 2.0), (0.0, 0.5, 2.0), (0.3, 0.3, 2.0), (0.05, 1.0, 0.5), (0.5, 0.9, 1e6)]:
        check(torch, moe, c, alpha, beta, lam)


@pytest.fixture
def wide_path(env):
    """Forces the many-workgroup code path for every token count (it is otherwise taken from about 7 K tokens on)."""
    _, moe = env
    before = moe.moe_compress_wide_min_tokens(0)
    yield
    moe.moe_compress_wide_min_tokens(before)


@pytest.mark.parametrize("case", SMALL, ids=[f"seed{c[0]}" for c in SMALL])
def test_small_cases_wide_path(env, wide_path, case):
    torch, moe = env
    seed, N, heads, E, L, k = case
    c = synth.make_compress_small(seed, N=N, n_heads=heads, E=E, L=L, k=min(k, E), n_clusters=4)
    for alpha, beta, lam in [(0.1, 0.25, 2.0), (0.0, 0.5, 2.0), (0.3, 0.3, 2.0), (0.05, 1.0, 0.5), (0.5, 0.9, 1e6)]:
        check(torch, moe, c, alpha, beta, lam, label=f"{c.name} (wide path)")


@pytest.mark.parametrize("name", ["P1", "P2", "P3"])
def test_workloads_full_size(env, name):
    torch, moe = env
    check(torch, moe, synth.make_compress_config(name))


@pytest.mark.parametrize("name", ["P1", "P2"])
def test_workloads_full_size_wide_path(env, wide_path, name):
    torch, moe = env
    check(torch, moe, synth.make_compress_config(name), label=f"{name} (wide path)")


def test_threshold_setter(env):
    _, moe = env
    default = moe.moe_compress_wide_min_tokens(-1)
    assert default > 0
    assert moe.moe_compress_wide_min_tokens(5) == default
    assert moe.moe_compress_wide_min_tokens(-1) == 5
    assert moe.moe_compress_wide_min_tokens(default) == 5
    assert moe.moe_compress_wide_min_tokens(-1) == default


def test_long_video_sampled(env):
    """P3 (32768 tokens): the oracle's Python loops take a while at this size, so the index list is checked against
    properties that hold at any size plus the oracle on the saliency part."""
    torch, moe = env
    c = synth.make_compress_config("P3")
    keep, s_norm, delta = run_gpu(torch, moe, c.A, c.R, c.E, c.alpha, c.beta, c.lam)
    N = c.N
    np.testing.assert_array_equal(s_norm.view(np.uint32), CO.normalize(CO.head_mean_saliency(c.A)).view(np.uint32))
    assert len(keep) == int(np.floor(c.beta * N)) and np.all(np.diff(keep) > 0) and keep[0] >= 0 and keep[-1] < N
    K_core = int(np.floor(c.alpha * N))
    core = np.lexsort((np.arange(N), -s_norm.astype(np.float64)))[:K_core]
    assert set(core.tolist()) <= set(keep.tolist())
    # Delta of every token against the expert set of that core, recomputed here with sets
    target = set(np.unique(c.R[:, core, :]).tolist())
    rng = np.random.default_rng(0)
    for i in rng.choice(N, size=300, replace=False):
        Ei = set(np.unique(c.R[:, i, :]).tolist())
        want = 0.0 if i in set(core.tolist()) else np.float32(len(Ei - target)) / np.float32(len(Ei))
        assert delta[i] == np.float32(want)
    # the kept tokens outside the core are exactly the best-scoring ones
    p = (s_norm - np.float32(c.lam) * delta).astype(np.float32)
    outside = np.setdiff1d(np.arange(N), core)
    order = outside[np.lexsort((outside, -p[outside].astype(np.float64)))]
    extra = order[: len(keep) - K_core]
    np.testing.assert_array_equal(np.sort(np.concatenate([core, extra])), keep)


def test_ties_wide_path(env, wide_path):
    """Few distinct saliency values over many tokens: both selections end inside a run of equal keys that spans
    several workgroups, so the rank among equal keys in token order decides."""
    torch, moe = env
    rng = np.random.default_rng(7)
    N = 10000                                  # three workgroups of 4096 tokens on the many-workgroup path
    A = rng.integers(0, 4, size=(1, N)).astype(np.float32)
    R = rng.integers(0, 16, size=(2, N, 2)).astype(np.int32)
    R[:, N // 2:, :] = 3                       # half of the tokens share one expert set: equal scores
    for alpha, beta in [(0.1, 0.4), (0.26, 0.7), (0.0, 0.33), (0.5, 0.5)]:
        want = CO.token_compress(A, R, 16, alpha, beta, 2.0)
        keep, s_norm, delta = run_gpu(torch, moe, A, R, 16, alpha, beta, 2.0)
        np.testing.assert_array_equal(keep, want["I_keep"])
        np.testing.assert_array_equal(delta, want["delta"])
    test_ties_constant_saliency_and_bad_ids(env)


def test_ties_constant_saliency_and_bad_ids(env):
    torch, moe = env
    A = np.ones((2, 600), dtype=np.float32)
    R = np.zeros((1, 600, 2), dtype=np.int32)
    R[0, :, 1] = np.arange(600) % 7
    R[0, 5, :] = [-3, 1000]                      # no valid id: Delta = 0
    want = CO.token_compress(A, R, 8, 0.1, 0.4, 2.0)
    keep, s_norm, delta = run_gpu(torch, moe, A, R, 8, 0.1, 0.4, 2.0)
    assert np.all(s_norm == 0)
    np.testing.assert_array_equal(keep, want["I_keep"])
    np.testing.assert_array_equal(delta, want["delta"])


def test_hand_worked_example_on_gpu(env):
    import json
    import os
    torch, moe = env
    with open(os.path.join(os.path.dirname(__file__), "golden", "compress_tiny.json")) as f:
        g = json.load(f)
    A, R = np.array(g["A"], dtype=np.float32), np.array(g["R"], dtype=np.int32)
    keep, _, _ = run_gpu(torch, moe, A, R, g["E"], g["alpha"], g["beta"], g["lambda"])
    assert keep.tolist() == g["expect"]["I_keep"]


def test_workspace_reuse_and_side_stream(env):
    torch, moe = env
    big = synth.make_compress_small(301, N=4000, n_heads=4, E=64, L=2, k=4)
    small = synth.make_compress_small(302, N=700, n_heads=4, E=64, L=2, k=4)
    ws = moe.alloc_compress_workspace(4000, 64)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for c in (big, small, big):
            keep, _, _ = run_gpu(torch, moe, c.A, c.R, c.E, c.alpha, c.beta, c.lam, ws=ws)
            np.testing.assert_array_equal(keep, CO.token_compress(c.A, c.R, c.E, c.alpha, c.beta, c.lam)["I_keep"])
