"""Lookahead-driven prefetching over a stack of layers (paper Sec. 3.4.2 / 3.4.3): predictor output -> asynchronous
copy to the host -> polled event -> moe_cache_predict on the transfer stream, the compute stream never synchronised
except for the one read of the routing decision. Whatever the prediction, every layer's output must equal the
all-resident computation bit for bit."""
import numpy as np
import pytest

from paper_2605_05899_amd import synth
from tests import helpers as Hp

pytestmark = pytest.mark.gpu

N_LAYERS, T, H, E, K, I = 4, 96, 128, 16, 2, 64


@pytest.fixture(scope="module")
def rig():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_05899_amd import moe, pipeline
    layers = [synth.make_small(800 + l, T, H, E, K, I, 0) for l in range(N_LAYERS)]
    # all-resident reference outputs through the dense entry point
    ref = []
    for Lr in layers:
        d = Hp.DeviceLayer(Lr, torch, moe)
        d.forward(want_routing=False)
        ref.append(d.out.clone())
    return torch, moe, pipeline, layers, ref


@pytest.mark.parametrize("mode,recall", [("demand", 0.0), ("standin", 1.0), ("standin", 0.5), ("mlp", 0.0)])
def test_stack_outputs_equal_all_resident_in_every_mode(rig, mode, recall):
    torch, moe, pipeline, layers, ref = rig
    stack = pipeline.CachedLayerStack(torch, moe, layers, n_slabs=24, budget=6)
    try:
        truth = stack.true_experts()
        if mode == "mlp":
            stack.set_random_mlp(5, D1=64, D2=32)

        def check(l, needed):
            stack.comp.synchronize()
            assert int(stack.missing[0]) == 0, f"layer {l}: an acquired expert was not resident"
            assert torch.equal(stack.out[l].view(torch.int16), ref[l].view(torch.int16)), f"{mode} layer {l}"
            assert needed == truth[l]

        stats = pipeline.StackStats()
        rng = np.random.default_rng(3)
        for p in range(3):
            print(f"[pipeline] mode={mode} recall={recall} pass {p}", flush=True)
            stack.run_pass(mode, stats, truth=truth, recall=recall, rng=rng, check=check)
        s = stats.summary(stack.cache.stats())
        print("[pipeline]", mode, recall, s, flush=True)
        assert s["layers_run"] == 3 * N_LAYERS and s["experts_demanded"] == 3 * sum(len(t) for t in truth)
        assert s["cache_hits"] + s["cache_misses"] == s["experts_demanded"] and s["demand_misses"] == s["cache_misses"]
        if mode == "demand":
            assert s["experts_listed"] == 0 and s["cache_prefetches"] == 0
        else:
            # a stand-in list is shorter than the budget when a layer leaves too few experts untouched to pad it with
            assert 0 < s["experts_listed"] <= 3 * (N_LAYERS - 1) * 6
            assert s["cache_prefetches"] == s["prefetch_copies_started"]
    finally:
        stack.close()


def test_true_predictions_remove_demand_misses(rig):
    """With the next layer's experts listed correctly (recall 1, budget as large as a layer's demand) the only misses
    left are those of the first layer of the first pass; demand-only fetching misses throughout."""
    torch, moe, pipeline, layers, ref = rig
    res = {}
    for mode in ("demand", "standin"):
        stack = pipeline.CachedLayerStack(torch, moe, layers, n_slabs=2 * E, budget=E)
        try:
            truth = stack.true_experts()
            stats = pipeline.StackStats()
            rng = np.random.default_rng(4)
            for p in range(2):
                stack.run_pass(mode, stats, truth=truth, recall=1.0, rng=rng)
            res[mode] = stats.summary(stack.cache.stats())
            if mode == "standin":
                # 2 E slabs hold two layers' experts: layer 0 of each pass misses (its prediction would have to come
                # from the pass before), every other layer is prefetched in full
                assert res[mode]["demand_misses"] == 2 * len(truth[0]), res[mode]
        finally:
            stack.close()
    assert res["standin"]["demand_misses"] < res["demand"]["demand_misses"]
