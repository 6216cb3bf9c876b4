"""The slab-based expert cache with its transfer and compute streams (paper Sec. 3.4.2 / 3.4.3) on the GPU:
the policy against the CPU model call by call, the bytes that land in the slabs, and a stack of layers whose expert
FFNs read their weights through the cache and must equal the all-resident computation bit for bit."""
import json
import os

import numpy as np
import pytest

from oracle import cache_oracle as CO
from oracle import moe_oracle as O
from paper_2605_05899_amd import synth
from tests import helpers as Hp
from tests.test_cache_oracle_pins import random_trace

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2605_05899_amd import moe
    return torch, moe


class Rig:
    """n_layers * E distinct host images in pinned memory, a device pool, a cache and the CPU model beside it."""

    def __init__(self, torch, moe, n_layers, E, slab_bytes, n_slabs, images=None):
        self.torch, self.n_layers, self.E, self.slab_bytes = torch, n_layers, E, slab_bytes
        if images is None:
            rng = np.random.default_rng(n_layers * 100 + E)
            images = rng.integers(0, 256, size=(n_layers * E, slab_bytes), dtype=np.uint8)
        self.host = torch.from_numpy(images).pin_memory()
        self.pool = torch.zeros(n_slabs * slab_bytes + 256, dtype=torch.uint8, device="cuda")
        off = (-self.pool.data_ptr()) % 256
        self.pool = self.pool[off:off + n_slabs * slab_bytes]
        self.cache = moe.ExpertCache(n_layers, E, slab_bytes, n_slabs, self.pool)
        self.model = CO.ExpertCacheModel(n_slabs)
        self.trans, self.comp = torch.cuda.Stream(), torch.cuda.Stream()

    def addr(self, layer, expert):
        return self.host.data_ptr() + (layer * self.E + expert) * self.slab_bytes

    def compare(self, where):
        res = self.model.residents()
        for l in range(self.n_layers):
            for e in range(self.E):
                slab, cls, prio = self.cache.query(l, e)
                if (l, e) in res:
                    ms, mc, mp = res[(l, e)]
                    assert (slab, cls) == (ms, mc) and prio == np.float32(mp), (where, l, e)
                else:
                    assert slab == -1, (where, l, e)
        st = self.cache.stats()
        for k, v in self.model.stats.items():
            assert st[k] == v, (where, k)
        assert st["bytes_copied"] == (self.model.stats["prefetches"] + self.model.stats["misses"]) * self.slab_bytes

    def check_pool_contents(self):
        self.trans.synchronize()
        self.comp.synchronize()
        pool = self.pool.cpu().numpy().reshape(-1, self.slab_bytes)
        host = self.host.numpy()
        for (l, e), (slab, _, _) in self.model.residents().items():
            assert np.array_equal(pool[slab], host[l * self.E + e]), f"slab {slab} does not hold expert ({l},{e})"


def test_policy_golden_trace_and_slab_contents(env):
    torch, moe = env
    with open(os.path.join(os.path.dirname(__file__), "golden", "cache_trace.json")) as f:
        t = json.load(f)
    rig = Rig(torch, moe, n_layers=4, E=8, slab_bytes=4096, n_slabs=t["n_slabs"])
    for i, step in enumerate(t["steps"]):
        print("cache trace step", i, step["op"], flush=True)
        if step["op"] == "predict":
            items = [tuple(x) for x in step["items"]]
            got = rig.cache.predict(items, rig.addr, rig.trans)
            assert got == [tuple(k) for k in rig.model.predict(items)] == [tuple(k) for k in step["started"]]
        elif step["op"] == "acquire":
            table, missed = rig.cache.acquire(step["layer"], step["needed"], rig.addr, rig.trans, rig.comp)
            assert missed == rig.model.acquire(step["layer"], step["needed"]) == step["missed"]
            res = rig.model.residents()
            for e in range(rig.E):
                want = rig.pool.data_ptr() + res[(step["layer"], e)][0] * rig.slab_bytes if e in step["needed"] else 0
                assert table[e] == want
        else:
            rig.cache.layer_done(step["layer"], rig.comp)
            rig.model.layer_done(step["layer"])
        rig.compare(step["why"])
        rig.check_pool_contents()
    assert {k: rig.cache.stats()[k] for k in t["final_stats"]} == t["final_stats"]
    rig.cache.close()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_policy_random_traces(env, seed):
    torch, moe = env
    rig = Rig(torch, moe, n_layers=4, E=12, slab_bytes=1024, n_slabs=16)
    for op in random_trace(seed):
        if op[0] == "predict":
            assert rig.cache.predict(op[1], rig.addr, rig.trans) == rig.model.predict(op[1])
        elif op[0] == "acquire":
            _, missed = rig.cache.acquire(op[1], op[2], rig.addr, rig.trans, rig.comp)
            assert missed == rig.model.acquire(op[1], op[2])
        elif op[0] == "layer_done":
            rig.cache.layer_done(op[1], rig.comp)
            rig.model.layer_done(op[1])
        rig.compare(str(op[0]))
    rig.check_pool_contents()
    rig.cache.close()


def test_demand_that_cannot_be_placed_and_bad_arguments(env):
    torch, moe = env
    rig = Rig(torch, moe, n_layers=2, E=4, slab_bytes=256, n_slabs=2)
    rig.cache.predict([(0, 0, 0.5), (0, 1, 0.4)], rig.addr, rig.trans)
    assert rig.cache.acquire(0, [2], rig.addr, rig.trans, rig.comp, check=False) == moe.MOE_ERR_CACHE_FULL
    assert rig.cache.predict([(0, 0, 0.5), (0, 0, 0.6)], rig.addr, rig.trans, check=False) == moe.MOE_ERR_SHAPE
    assert rig.cache.predict([(2, 0, 0.5)], rig.addr, rig.trans, check=False) == moe.MOE_ERR_SHAPE
    assert rig.cache.acquire(0, [9], rig.addr, rig.trans, rig.comp, check=False) == moe.MOE_ERR_SHAPE
    rig.trans.synchronize()
    rig.cache.close()
    c = moe.ExpertCache(2, 4, 250, 2, rig.pool, check=False)          # slab size not a multiple of 16
    assert c.status == moe.MOE_ERR_SHAPE


def test_layer_stack_through_the_cache_equals_all_resident(env):
    """Three MoE layers whose routed experts live in host memory; 14 slabs for 24 experts; two passes. Every layer's
    expert FFN read through the cache must equal the dense call bit for bit, whatever was evicted in between."""
    torch, moe = env
    n_layers, T, H, E, k, I = 3, 96, 128, 8, 2, 64
    layers = [synth.make_small(600 + l, T, H, E, k, I, 0) for l in range(n_layers)]
    slab_elems = 3 * I * H
    images = np.stack([np.concatenate([L.w_gate[e].ravel(), L.w_up[e].ravel(), L.w_down[e].ravel()])
                       for L in layers for e in range(E)]).view(np.uint8)
    rig = Rig(torch, moe, n_layers, E, slab_elems * 2, 14, images=images)
    devs = [Hp.DeviceLayer(L, torch, moe) for L in layers]
    rng = np.random.default_rng(9)
    demanded = 0
    for p in range(2):
        x = Hp.bf16_dev(synth.make_small(700 + p, T, H, E, k, I, 0).x, torch)
        for l, d in enumerate(devs):
            with torch.cuda.stream(rig.comp):
                ids = torch.empty((T, k), dtype=torch.int32, device="cuda")
                w = torch.empty((T, k), dtype=torch.float32, device="cuda")
                off = torch.empty(E + 1, dtype=torch.int32, device="cuda")
                st = torch.empty(T * k, dtype=torch.int32, device="cuda")
                inv = torch.empty(T * k, dtype=torch.int32, device="cuda")
                moe.moe_route(d.cfg, x, T, None, T, d.w_router, ids, w, d.ws)
                moe.moe_dispatch(d.cfg, ids, T, off, st, inv, d.ws)
            # a (poor) prediction for the next layer goes out while this one is being routed
            if l + 1 < n_layers:
                guess = [(l + 1, int(e), float(np.round(rng.random(), 3))) for e in rng.choice(E, size=4, replace=False)]
                assert rig.cache.predict(guess, rig.addr, rig.trans) == rig.model.predict(guess)
            rig.comp.synchronize()                          # the routing decision is read on the host, as in the paper
            needed = sorted(set(ids.cpu().numpy().ravel().tolist()))
            demanded += len(needed)
            table, missed = rig.cache.acquire(l, needed, rig.addr, rig.trans, rig.comp)
            assert missed == rig.model.acquire(l, needed)
            with torch.cuda.stream(rig.comp):
                d_table = torch.tensor(table, dtype=torch.int64, device="cuda")
                y_c = torch.zeros((T * k, H), dtype=torch.bfloat16, device="cuda")
                missing = torch.zeros(E + 1, dtype=torch.int32, device="cuda")
                moe.moe_expert_ffn_slabs(d.cfg, x, T, None, T, off, st, d_table, y_c, missing, d.ws)
                rig.cache.layer_done(l, rig.comp)
                rig.model.layer_done(l)
                y_d = torch.zeros_like(y_c)
                moe.moe_expert_ffn(d.cfg, x, T, None, T, off, st, d.w_gate, d.w_up, d.w_down, y_d, d.ws)
                out = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
                moe.moe_combine(d.cfg, y_c, inv, w, T, None, out)
            rig.comp.synchronize()
            assert int(missing[0]) == 0, f"pass {p} layer {l}: an acquired expert was not resident"
            assert torch.equal(y_c, y_d), f"pass {p} layer {l}: cache path differs from the all-resident path"
            rig.compare(f"pass {p} layer {l}")
            x = out
    s = rig.cache.stats()
    print("cache stats over two passes:", s, flush=True)
    assert s["hits"] + s["misses"] == demanded and s["evictions"] > 0
    rig.cache.close()
