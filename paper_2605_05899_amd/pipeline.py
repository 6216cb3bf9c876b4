"""Lookahead-driven expert prefetching over a stack of MoE layers (paper Sec. 3.4.2 "lookahead-driven insertion",
Sec. 3.4.3 transfer / compute streams): host-side orchestration of the C-ABI calls, no arithmetic of the method.

The routed experts of every layer live in pinned host memory; the GPU holds a pool of slabs behind the library's
expert cache. Per layer l, on the compute stream:

    route(l) -> async copy of the routing ids to the host          (the one read of the routing decision the paper
    predictor features + MLP for layer l+1 -> top-B list,             itself has: the host must know which experts to
        async copy of the list to the host, its own event             demand)
    dispatch(l)
    host waits for the routing ids, demands the layer's experts from the cache (moe_cache_acquire: hits, or copies
        on the transfer stream that the compute stream waits for, expert by expert)
    expert FFN through the slab table, combine, moe_cache_layer_done(l)
    host polls the predictor's event (never a stream synchronisation) and hands the list to moe_cache_predict: the
        prefetch copies of layer l+1 run on the transfer stream while layer l computes

Where a prediction comes from is a plug-in: the library's predictor MLP on features computed on the GPU (with whatever
weights it is given; trained weights do not exist here), or a stand-in that lists the next layer's true experts with
a chosen recall (the truth is known because the synthetic layers are independent of each other's outputs).
The compute-stream stall of a layer is measured with two events around the waits that moe_cache_acquire enqueues.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Callable, List, Optional

import numpy as np

from . import harness


@dataclass
class StackStats:
    stall_us: List[float] = field(default_factory=list)        # per executed layer: compute-stream wait for its experts
    demanded: int = 0
    missed: int = 0
    predicted: int = 0
    started: int = 0
    poll_spins: int = 0
    wall_ms: float = 0.0

    def summary(self, cache_stats: dict) -> dict:
        s = np.asarray(self.stall_us) if self.stall_us else np.zeros(1)
        return {"layers_run": len(self.stall_us), "stall_us_mean": float(s.mean()), "stall_us_max": float(s.max()),
                "experts_demanded": self.demanded, "demand_misses": self.missed, "experts_listed": self.predicted,
                "prefetch_copies_started": self.started, "poll_spins": self.poll_spins, "wall_ms": self.wall_ms,
                **{f"cache_{k}": v for k, v in cache_stats.items()}}


class CachedLayerStack:
    """L independent synthetic layers (same shape) run one after the other through one slab cache."""

    def __init__(self, torch, moe, layers, n_slabs: int, budget: int):
        self.torch, self.moe, self.layers = torch, moe, layers
        L0 = layers[0]
        self.n_layers, self.E, self.k, self.H, self.I, self.T = len(layers), L0.E, L0.k, L0.H, L0.I, L0.T
        self.budget = budget
        E, H, I = self.E, self.H, self.I
        self.slab_bytes = 3 * I * H * 2
        # host images [gate | up | down] of every (layer, expert), pinned
        self.host = torch.empty((self.n_layers * E, self.slab_bytes), dtype=torch.uint8).pin_memory()
        hv = self.host.numpy()
        for l, Lr in enumerate(layers):
            for e in range(E):
                img = np.concatenate([Lr.w_gate[e].ravel(), Lr.w_up[e].ravel(), Lr.w_down[e].ravel()]).view(np.uint8)
                hv[l * E + e] = img
        pool = torch.zeros(n_slabs * self.slab_bytes + 256, dtype=torch.uint8, device="cuda")
        off = (-pool.data_ptr()) % 256
        self.pool = pool[off:off + n_slabs * self.slab_bytes]
        self.n_slabs = n_slabs
        self.cache = moe.ExpertCache(self.n_layers, E, self.slab_bytes, n_slabs, self.pool)
        self.comp, self.trans = torch.cuda.Stream(), torch.cuda.Stream()
        # per-layer device state (router weights, tokens, workspace); expert weights are NOT uploaded
        self.cfg = moe.MoEConfig(H=H, I=I, E=E, k=self.k, S=0, norm_topk=L0.norm_topk, max_tokens=self.T)
        self.x = [harness.bf16_dev(Lr.x, torch) for Lr in layers]
        self.w_router = [harness.bf16_dev(Lr.w_router, torch) for Lr in layers]
        self.ws = moe.alloc_workspace(self.cfg)
        T, k = self.T, self.k
        dev = lambda shape, dt: torch.empty(shape, dtype=dt, device="cuda")
        self.ids, self.w = dev((T, k), torch.int32), dev((T, k), torch.float32)
        self.off, self.st, self.inv = dev(E + 1, torch.int32), dev(T * k, torch.int32), dev(T * k, torch.int32)
        self.y, self.out = dev((T * k, H), torch.bfloat16), [dev((T, H), torch.bfloat16) for _ in layers]
        self.missing = dev(E + 1, torch.int32)
        self.d_table = dev(E, torch.int64)
        self.h_ids = torch.empty((T, k), dtype=torch.int32).pin_memory()
        self.h_table = [torch.zeros(E, dtype=torch.int64).pin_memory() for _ in layers]   # one per layer: no reuse in a pass
        self.h_top = torch.empty(max(budget, 1), dtype=torch.int32).pin_memory()
        self.h_score = torch.empty(E, dtype=torch.float32).pin_memory()
        self.ev_route, self.ev_pred = torch.cuda.Event(), torch.cuda.Event()
        self.ev_table = [torch.cuda.Event() for _ in layers]
        # predictor state: features [routing histogram (E) ; mean hidden state (H)], a small bottleneck MLP
        self.feat = dev(E + H, torch.float32)
        self.score, self.top = dev(E, torch.float32), dev(max(budget, 1), torch.int32)
        self.pool_ws = torch.empty(moe.moe_mean_pool_workspace_bytes(H), dtype=torch.uint8, device="cuda")
        self.mlp = None

    def addr(self, layer, expert):
        return self.host.data_ptr() + (layer * self.E + expert) * self.slab_bytes

    def close(self):
        self.torch.cuda.synchronize()
        self.cache.close()

    # ------------------------------------------------------------------ predictors
    def set_random_mlp(self, seed: int, D1: int = 256, D2: int = 128):
        """Random weights for the library's predictor MLP (one network per layer would be trained; untrained, one
        random network serves all layers)."""
        torch, moe = self.torch, self.moe
        rng = np.random.default_rng(seed)
        D = self.E + self.H
        rnd = lambda *shape: torch.from_numpy((rng.standard_normal(shape) / np.sqrt(shape[-1])).astype(np.float32)).cuda()
        self.mlp = dict(D=D, D1=D1, D2=D2, W1=rnd(D1, D), s1=rnd(D1) + 1, t1=rnd(D1), W2=rnd(D2, D1), s2=rnd(D2) + 1,
                        t2=rnd(D2), Wo=rnd(self.E, D2),
                        ws=torch.empty(moe.moe_predictor_workspace_bytes(D1, D2), dtype=torch.uint8, device="cuda"))

    def _enqueue_mlp_prediction(self, l: int):
        """Features of layer l and the MLP's top-B list for layer l+1, on the compute stream; the list and the scores
        are copied to pinned host memory and ev_pred marks their arrival."""
        moe, m = self.moe, self.mlp
        T, k, E, H = self.T, self.k, self.E, self.H
        moe.moe_routing_histogram(self.ids, T * k, E, self.feat[:E], stream=self.comp)
        moe.moe_mean_pool(self.x[l], T, H, None, T, self.feat[E:], self.pool_ws, stream=self.comp)
        moe.moe_predictor_forward(self.feat, m["D"], m["W1"], m["s1"], m["t1"], m["D1"], m["W2"], m["s2"], m["t2"],
                                  m["D2"], m["Wo"], E, self.budget, self.score, self.top, m["ws"], stream=self.comp)
        self.h_top.copy_(self.top, non_blocking=True)
        self.h_score.copy_(self.score, non_blocking=True)
        self.ev_pred.record(self.comp)

    # ------------------------------------------------------------------ one pass over the stack
    def run_pass(self, mode: str, stats: StackStats, truth: Optional[List[List[int]]] = None, recall: float = 1.0,
                 rng: Optional[np.random.Generator] = None, check: Optional[Callable] = None):
        """mode: 'demand' (no prediction), 'mlp' (the library's predictor with the weights of set_random_mlp), 'standin'
        (lists `budget` experts of the next layer of which a share `recall` is true, from `truth`)."""
        torch, moe, cache = self.torch, self.moe, self.cache
        T, k, E = self.T, self.k, self.E
        t_wall = time.perf_counter()
        with torch.cuda.stream(self.comp):
            for l in range(self.n_layers):
                x = self.x[l]
                moe.moe_route(self.cfg, x, T, None, T, self.w_router[l], self.ids, self.w, self.ws)
                self.h_ids.copy_(self.ids, non_blocking=True)
                self.ev_route.record(self.comp)
                has_next = l + 1 < self.n_layers
                if mode == "mlp" and has_next:
                    self._enqueue_mlp_prediction(l)
                moe.moe_dispatch(self.cfg, self.ids, T, self.off, self.st, self.inv, self.ws)
                # the one host read of the routing decision
                self.ev_route.synchronize()
                needed = sorted(set(self.h_ids.numpy().ravel().tolist()))
                stats.demanded += len(needed)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(self.comp)
                table, missed = cache.acquire(l, needed, self.addr, self.trans, self.comp)
                e1.record(self.comp)
                stats.missed += len(missed)
                self.ev_table[l].synchronize()       # the previous pass's upload of this buffer (long done: never waits)
                self.h_table[l].numpy()[:] = np.asarray(table, dtype=np.int64)
                self.d_table.copy_(self.h_table[l], non_blocking=True)
                self.ev_table[l].record(self.comp)
                moe.moe_expert_ffn_slabs(self.cfg, x, T, None, T, self.off, self.st, self.d_table, self.y, self.missing,
                                         self.ws)
                moe.moe_combine(self.cfg, self.y, self.inv, self.w, T, None, self.out[l])
                cache.layer_done(l, self.comp)
                # prediction for the next layer: poll its event, never the stream
                if has_next and mode != "demand":
                    if mode == "mlp":
                        while not self.ev_pred.query():
                            stats.poll_spins += 1
                        top = self.h_top.numpy()[:self.budget].tolist()
                        score = self.h_score.numpy()
                        items = [(l + 1, int(e), float(score[e])) for e in top]
                    else:
                        true_next = truth[l + 1]
                        n_true = min(len(true_next), int(round(recall * min(self.budget, len(true_next)))))
                        pick = list(rng.choice(true_next, size=n_true, replace=False)) if n_true else []
                        others = [e for e in range(E) if e not in set(true_next)]
                        n_false = min(self.budget - n_true, len(others))
                        pick += list(rng.choice(others, size=n_false, replace=False)) if n_false else []
                        items = [(l + 1, int(e), 1.0 - i / (len(pick) + 1)) for i, e in enumerate(pick)]
                    stats.predicted += len(items)
                    stats.started += len(cache.predict(items, self.addr, self.trans))
                if check is not None:
                    check(l, needed)
                stats.stall_us.append((e0, e1))
        self.comp.synchronize()
        stats.wall_ms += (time.perf_counter() - t_wall) * 1e3
        stats.stall_us = [ev if isinstance(ev, float) else ev[0].elapsed_time(ev[1]) * 1e3 for ev in stats.stall_us]

    def true_experts(self) -> List[List[int]]:
        """Which experts each layer's routing touches (the layers' inputs are fixed, so this is known up front)."""
        torch, moe = self.torch, self.moe
        out = []
        with torch.cuda.stream(self.comp):
            for l in range(self.n_layers):
                moe.moe_route(self.cfg, self.x[l], self.T, None, self.T, self.w_router[l], self.ids, self.w, self.ws)
                self.comp.synchronize()
                out.append(sorted(set(self.ids.cpu().numpy().ravel().tolist())))
        return out
