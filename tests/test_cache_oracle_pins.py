"""Pins of the expert-cache policy model (paper Sec. 3.4.2 / 3.4.3) against a hand-worked trace and invariants."""
import json
import os

import numpy as np
import pytest

from oracle import cache_oracle as CO

NAMES = {CO.REQUIRED: "required", CO.SPECULATIVE: "speculative", CO.EXPIRED: "expired"}


def load_trace():
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cache_trace.json")) as f:
        return json.load(f)


def key_str(k):
    return f"{k[0]},{k[1]}"


def replay(model, step):
    """Runs one step of the golden trace on a model with the oracle's method names; returns what to compare."""
    n_log = len(model.log)
    got = {}
    if step["op"] == "predict":
        before = model.stats["refused"]
        got["started"] = [list(k) for k in model.predict([tuple(i) for i in step["items"]])]
        got["refused"] = model.stats["refused"] - before
    elif step["op"] == "acquire":
        got["missed"] = model.acquire(step["layer"], step["needed"])
    elif step["op"] == "layer_done":
        model.layer_done(step["layer"])
    got["evicted"] = [list(v) for _, _, v in model.log[n_log:] if v is not None]
    res = model.residents()
    got["classes"] = {key_str(k): NAMES[c] for k, (_, c, _) in res.items()}
    got["residents"] = {key_str(k): [s, NAMES[c], p] for k, (s, c, p) in res.items()}
    return got


def test_hand_worked_trace():
    t = load_trace()
    m = CO.ExpertCacheModel(t["n_slabs"])
    for step in t["steps"]:
        got = replay(m, step)
        for field in ("started", "missed", "evicted", "refused"):
            if field in step:
                assert got[field] == step[field], (step["op"], field, step["why"])
        for k, c in step.get("classes", {}).items():
            assert got["classes"][k] == c, (step["why"], k)
        if "residents" in step:
            assert got["residents"] == step["residents"], step["why"]
    assert m.stats == t["final_stats"]


def random_trace(seed, n_layers=4, E=12, passes=3):
    rng = np.random.default_rng(seed)
    ops = []
    for _ in range(passes):
        ops.append(("begin_pass",))
        for l in range(n_layers):
            nxt = [(int(l2), int(e), float(np.round(rng.random(), 3)))
                   for l2 in range(l, min(n_layers, l + 2)) for e in rng.choice(E, size=3, replace=False)]
            ops.append(("predict", nxt))
            ops.append(("acquire", l, [int(e) for e in rng.choice(E, size=3, replace=False)]))
            ops.append(("layer_done", l))
    return ops


@pytest.mark.parametrize("seed", range(6))
def test_invariants_on_random_traces(seed):
    m = CO.ExpertCacheModel(16)          # 48 experts in all; at most 15 are protected at any time in these traces
    demanded = 0
    for op in random_trace(seed):
        before = m.residents()
        n_log = len(m.log)
        if op[0] == "predict":
            m.predict(op[1])
        elif op[0] == "acquire":
            m.acquire(op[1], op[2])
            demanded += len(set(op[2]))
            for e in op[2]:
                assert (op[1], e) in m.slab_of and m.cls[(op[1], e)] == CO.REQUIRED
        elif op[0] == "layer_done":
            m.layer_done(op[1])
        else:
            m.begin_pass()
        res = m.residents()
        assert len(res) <= m.n_slabs and len({s for s, _, _ in res.values()}) == len(res)      # one expert per slab
        # every eviction of this step took an expert that was Expired when the step began or expired... no: that
        # was Expired at the moment of eviction; with the state before the step that means Expired before it, since
        # no operation both expires and evicts
        for _, _, victim in m.log[n_log:]:
            if victim is None:
                continue
            assert before[victim][1] == CO.EXPIRED
        # the victims of a step are, in order, the lowest-priority experts among those Expired before the step that
        # the step itself did not ask for again (a listed or demanded resident is promoted before anything is evicted)
        victims = [v for _, _, v in m.log[n_log:] if v is not None]
        if victims:
            asked = {(l, e) for l, e, _ in op[1]} if op[0] == "predict" else {(op[1], e) for e in op[2]}
            expired = sorted((p, k) for k, (_, c, p) in before.items() if c == CO.EXPIRED and k not in asked)
            assert [k for _, k in expired[:len(victims)]] == victims
    assert m.stats["hits"] + m.stats["misses"] == demanded


def test_demand_with_nothing_evictable_fails_loudly():
    m = CO.ExpertCacheModel(2)
    m.predict([(0, 0, 0.5), (0, 1, 0.4)])
    with pytest.raises(CO.CacheFull):
        m.acquire(0, [2])                      # both slabs hold Required experts of a layer that has not run


# ------------------------------------------------------------------------------------------------------------------
# Brute force over a flat event log: every eviction the model makes is checked against the classes and priorities
# that follow, expert by expert, from the plain sequence of calls (readings K1-K7), not from the model's own tables.
def _state_at(events, key, upto):
    """(resident, class, priority) of one expert after events[:upto], by replaying only what concerns it."""
    resident, cls, prio = False, None, None
    for ev in events[:upto]:
        kind = ev[0]
        if kind == "fetch" and ev[1] == key:
            resident, cls, prio = True, CO.REQUIRED, ev[2]
        elif kind == "evict" and ev[1] == key:
            resident, cls, prio = False, None, None
        elif not resident:
            continue
        elif kind == "predict" and cls == CO.REQUIRED and key not in ev[1]:
            cls = CO.SPECULATIVE                    # dropped by a newer list before its layer ran: still protected
        elif kind == "listed" and ev[1] == key:
            cls, prio = CO.REQUIRED, ev[2]
        elif kind == "demanded" and ev[1] == key:
            cls = CO.REQUIRED
        elif kind == "done" and ev[1] == key[0]:
            cls = CO.EXPIRED
    return resident, cls, prio


@pytest.mark.parametrize("seed", range(10))
def test_every_eviction_takes_the_least_valuable_expired_expert_brute_force(seed):
    n_slabs, n_layers, E = 16, 4, 12
    m = CO.ExpertCacheModel(n_slabs)
    events, n_evictions, n_refused = [], 0, 0
    all_keys = [(l, e) for l in range(n_layers) for e in range(E)]

    def absorb_fetches(n_log_before, prio_of):
        nonlocal n_evictions
        for what, key, victim in m.log[n_log_before:]:
            states = {k: _state_at(events, k, len(events)) for k in all_keys}
            residents = [k for k, s in states.items() if s[0]]
            assert not states[key][0], "fetched an expert that was resident"
            if victim is None:
                assert len(residents) < n_slabs, "took a free slab when none was free"
            else:
                n_evictions += 1
                assert len(residents) == n_slabs, "evicted although a slab was free"
                assert states[victim][0] and states[victim][1] == CO.EXPIRED, "evicted a protected expert"
                expired = [(states[k][2], k) for k in residents if states[k][1] == CO.EXPIRED]
                assert (states[victim][2], victim) == min(expired), "a less valuable expired expert was resident"
                events.append(("evict", victim))
            events.append(("fetch", key, prio_of(key)))

    for op in random_trace(seed, n_layers=n_layers, E=E, passes=4):
        n_log = len(m.log)
        if op[0] == "predict":
            listed = {(l, e): p for l, e, p in op[1]}
            events.append(("predict", set(listed)))
            for k, p in listed.items():
                events.append(("listed", k, p))
            refused_before = m.stats["refused"]
            m.predict(op[1])
            absorb_fetches(n_log, lambda k: listed[k])
            if m.stats["refused"] > refused_before:
                n_refused += m.stats["refused"] - refused_before
                states = {k: _state_at(events, k, len(events)) for k in all_keys}
                assert sum(s[0] for s in states.values()) == n_slabs
                assert not any(s[0] and s[1] == CO.EXPIRED for s in states.values()), "refused although evictable"
        elif op[0] == "acquire":
            for e in sorted(set(op[2])):
                events.append(("demanded", (op[1], e)))
            m.acquire(op[1], op[2])
            absorb_fetches(n_log, lambda k: 0.0)
        elif op[0] == "layer_done":
            m.layer_done(op[1])
            events.append(("done", op[1]))
        # the model's tables must agree with the flat reconstruction after every call
        for k in all_keys:
            res, cls, prio = _state_at(events, k, len(events))
            assert res == (k in m.slab_of)
            if res:
                assert (cls, prio) == (m.cls[k], m.prio[k]), (op[0], k)
    assert n_evictions > 20          # the traces do exercise eviction
