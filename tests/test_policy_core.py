"""The C++ policy core (include/pbkv_policy.h) against the reference model, operation by
operation on seeded random traces of node insertions, accesses along radix paths, forecasts,
terminations, pins, evictions and prefetch decisions: scores within 1e-12 relative, every
integer decision (retired tag, eviction list, load list, reclaimed list) identical.  Host code:
runs without a GPU."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import policy_oracle as PO
from paper_2605_06472_amd import binding
from paper_2605_06472_amd import policy as PC

HERE = os.path.dirname(os.path.abspath(__file__))


class Both:
    """Drives the two implementations with the same calls and compares what they return."""

    def __init__(self, V, K, gamma, mode):
        self.o = PO.PolicyOracle(V, K, gamma, mode)
        self.c = PC.Policy(V, K, gamma, mode)

    def __getattr__(self, name):
        fo, fc = getattr(self.o, name), getattr(self.c, name)

        def call(*a, **k):
            ro, rc = fo(*a, **k), fc(*a, **k)
            assert ro == rc, "%s%r: model %r, core %r" % (name, a, ro, rc)
            return ro
        return call

    def check_nodes(self):
        for nid, n in self.o.nodes.items():
            so, sc = self.o.score(nid), self.c.score(nid)
            assert sc == pytest.approx(so, rel=1e-12, abs=1e-15), nid
            assert self.c.value(nid) == pytest.approx(self.o.value(nid), rel=1e-12, abs=1e-15), nid
            assert self.c.is_retired(nid) == self.o.is_retired(nid), nid
            assert self.c.node_tier(nid) == n.tier, nid
        assert self.c.retired_pages() == self.o.retired_pages()


def random_forecast(rng, K, V):
    p = rng.random((K, V + 1)) ** 3           # uneven rows, no near-ties between nodes
    return (p / p.sum(1, keepdims=True)).tolist()


def run_trace(seed, mode, steps=400, V=5, K=3, gamma=0.7):
    rng = np.random.default_rng(seed)
    b = Both(V, K, gamma, mode)
    next_node, next_wf = 0, 0
    live_wf = []
    b.node_add(next_node, -1, 2)
    next_node += 1
    for step in range(steps):
        r = rng.random()
        ids = sorted(b.o.nodes)
        if r < 0.18 or len(ids) < 4:                                   # grow the radix tree
            parent = int(rng.choice(ids)) if rng.random() < 0.85 else -1
            if parent >= 0 and b.o.nodes[parent].tier == PO.HOST:
                continue
            b.node_add(next_node, parent, int(rng.integers(1, 5)))
            next_node += 1
        elif r < 0.50:                                                 # an agent invocation touches a path
            if not live_wf or rng.random() < 0.25:
                live_wf.append(next_wf)
                w = next_wf
                next_wf += 1
            else:
                w = int(rng.choice(live_wf))
            leaf = int(rng.choice(ids))
            path = []
            while leaf >= 0:
                path.append(leaf)
                leaf = b.o.nodes[leaf].parent
            path.reverse()
            for nid in path:                                           # a hit on a host node swaps it back in
                if b.o.nodes[nid].tier == PO.HOST:
                    b.node_set_tier(nid, PO.GPU)
            b.access(w, int(rng.integers(V)), path)
            b.forecast(w, random_forecast(rng, K, V))
        elif r < 0.60 and live_wf:                                     # refreshed forecast only
            b.forecast(int(rng.choice(live_wf)), random_forecast(rng, K, V))
        elif r < 0.70 and live_wf:                                     # termination message
            w = live_wf.pop(int(rng.integers(len(live_wf))))
            b.terminate(w)
        elif r < 0.76:                                                 # a running request pins / releases a node
            nid = int(rng.choice(ids))
            if b.o.nodes[nid].pins and rng.random() < 0.7:
                b.node_pin(nid, -1)
            elif b.o.nodes[nid].tier == PO.GPU:
                b.node_pin(nid, 1)
        elif r < 0.90:                                                 # memory pressure
            b.evict(int(rng.integers(1, 9)), to_host=bool(rng.random() < 0.8))
        else:                                                          # a pure-decode batch: prefetch
            b.prefetch(int(rng.integers(0, 6)), int(rng.integers(0, 12)), pure_decode=bool(rng.random() < 0.9),
                       to_host=bool(rng.random() < 0.8))
        if step % 7 == 0:
            b.check_nodes()
    b.check_nodes()
    b.evict(10 ** 9)                                                   # drain what can be drained
    b.check_nodes()
    return b


@pytest.mark.parametrize("mode", [PO.MODE_HE, PO.MODE_LAE, PO.MODE_LRU], ids=["he", "lae", "lru"])
@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_random_traces_match_the_reference_model(seed, mode):
    run_trace(seed, mode)


def test_hand_example_through_the_c_boundary():
    g = json.load(open(os.path.join(HERE, "golden", "policy_score_example.json")))
    c = PC.Policy(g["num_agents"], g["horizon"], float(Fraction(g["gamma"])))
    ids = {name: i for i, name in enumerate(sorted(g["nodes"]))}
    for i in ids.values():
        c.node_add(i, -1, 1)
    for name, nd in g["nodes"].items():
        for w, agents in nd["access"].items():
            for a in agents:
                c.access(int(w), a, [ids[name]])
    for w, rows in g["forecasts"].items():
        c.forecast(int(w), [[float(Fraction(x)) for x in row] for row in rows])
    for w in g["terminated"]:
        c.terminate(w)
    for name, nd in g["nodes"].items():
        assert c.score(ids[name]) == float(Fraction(nd["score"])), name       # exact binary fractions
        assert c.value(ids[name]) == float(Fraction(nd["value"])), name
        assert c.is_retired(ids[name]) == nd["retired"], name


def test_argument_errors_change_nothing():
    with pytest.raises(binding.PbkvError):
        PC.Policy(65, 3, 0.7)
    with pytest.raises(binding.PbkvError):
        PC.Policy(4, 3, 0.0)
    c = PC.Policy(3, 2, 0.7)
    c.node_add(0, -1, 1)
    for bad in (lambda: c.node_add(0, -1, 1), lambda: c.node_add(1, 7, 1), lambda: c.node_add(1, -1, 0),
                lambda: c.access(1, 3, [0]), lambda: c.access(1, 0, [0, 9]),
                lambda: c.forecast(1, [[0.5, 0.5, 0.5, 0.0], [1.0, 0.0, 0.0, 0.0]]),
                lambda: c.forecast(1, [[1.5, -0.5, 0.0, 0.0], [1.0, 0.0, 0.0, 0.0]]),
                lambda: c.terminate(99), lambda: c.node_pin(0, -1), lambda: c.node_set_tier(5, 0)):
        with pytest.raises(binding.PbkvError):
            bad()
    assert c.is_retired(0) and c.score(0) == 0.0 and np.isnan(c.score(123))
    c.access(1, 0, [0])
    c.terminate(1)
    with pytest.raises(binding.PbkvError):
        c.access(1, 0, [0])                       # a terminated workflow cannot come back
    c.node_add(1, 0, 1)
    with pytest.raises(binding.PbkvError):
        c.node_remove(0)                          # has a child
    c.node_remove(1)
    c.node_remove(0)


def test_dropping_a_node_forgets_its_host_descendants():
    for impl in (lambda: PO.PolicyOracle(1, 1, 0.7), lambda: PC.Policy(1, 1, 0.7)):
        p = impl()
        p.node_add(0, -1, 1)
        p.node_add(1, 0, 1)
        p.node_add(2, 1, 1)
        assert p.evict(2, to_host=True) == ([2, 1], 2)
        assert p.evict(1, to_host=False) == ([0], 1)
        p.node_add(0, -1, 1)                      # all three ids are free again
        p.node_add(1, 0, 1)
        p.node_add(2, 1, 1)


# ---- the synthetic workflow driver -------------------------------------------------------------
from paper_2605_06472_amd import policy_sim as SIM      # noqa: E402


def test_forecast_of_the_synthetic_call_graph_is_a_conditional_distribution():
    for a in range(len(SIM.AGENTS)):
        f = SIM.k_step_forecast(a, 4)
        assert f.shape == (4, len(SIM.AGENTS) + 1)
        assert np.allclose(f.sum(1), 1.0) and (f >= 0).all()
        assert np.allclose(f[0], SIM.CALL_GRAPH[a])
    # two steps after the tester: coder/reviewer/END weighted by the surviving mass 0.85
    f = SIM.k_step_forecast(3, 2)
    want = (0.40 * SIM.CALL_GRAPH[2] + 0.45 * SIM.CALL_GRAPH[4]) / 0.85
    assert np.allclose(f[1], want)


@pytest.mark.parametrize("mode,prefetch", [(PO.MODE_LRU, False), (PO.MODE_LAE, False), (PO.MODE_HE, False),
                                           (PO.MODE_HE, True)], ids=["lru", "lae", "he", "full"])
def test_driver_takes_the_same_decisions_with_core_and_model(mode, prefetch):
    """Whole-system parity: the same seeded workflow run through the C++ core and through the
    reference model yields identical eviction / prefetch decisions and identical hit counts."""
    runs = []
    for pol in (PO.PolicyOracle(6, 3, 0.7, mode), PC.Policy(6, 3, 0.7, mode)):
        w = SIM.World(pol, capacity_pages=160, concurrency=8, seed=11, horizon=3, prefetch=prefetch)
        runs.append((w.run(250), w.decisions))
    assert runs[0][0] == runs[1][0]
    assert runs[0][1] == runs[1][1]
    assert any(d[0] == "evict" and d[1] for d in runs[0][1])
    if prefetch:
        assert any(d[0] == "prefetch" and d[1] for d in runs[0][1])


def test_policy_variants_rank_as_in_the_paper():
    """Table 1 orders the variants LRU < LAE < HE < Full in GPU hit rate on every workload; the
    synthetic driver has no claim on the absolute numbers, only on that order."""
    rates = []
    for mode, prefetch in ((PC.MODE_LRU, False), (PC.MODE_LAE, False), (PC.MODE_HE, False), (PC.MODE_HE, True)):
        tot_hit = tot = 0
        for seed in (3, 7, 19):
            w = SIM.World(PC.Policy(6, 3, 0.7, mode), capacity_pages=300, concurrency=24, seed=seed, horizon=3,
                          prefetch=prefetch)
            r = w.run(3000)
            tot_hit += r["gpu_hit_pages"]
            tot += r["gpu_hit_pages"] + r["host_hit_pages"]
        rates.append(tot_hit / tot)
    assert rates[0] < rates[1] < rates[2] < rates[3], rates


def test_prefetch_is_cut_back_when_the_reclaim_list_is_too_short():
    """Two host nodes worth loading, no free page, retired GPU nodes that would make room -- but the
    caller's reclaim list holds only one entry: the core withdraws the loads it cannot place instead
    of leaving its books ahead of the lists it returns."""
    pol = PC.Policy(3, 2, 0.7, PC.MODE_HE)
    pol._b = pol._b[:1]                                # reclaim list of one node
    pol.node_add(0, -1, 1, PC.GPU)                # root, accessed by both workflows
    pol.node_add(1, 0, 2, PC.GPU)                 # will be retired
    pol.node_add(2, 0, 2, PC.GPU)                 # will be retired
    pol.node_add(3, 0, 2, PC.HOST)                # wanted
    pol.node_add(4, 0, 2, PC.HOST)                # wanted
    pol.access(7, 0, [0, 1])
    pol.access(8, 0, [0, 2])
    pol.terminate(7)
    pol.terminate(8)
    pol.access(9, 1, [0, 3])
    pol.access(9, 2, [0, 4])
    pol.forecast(9, [[0.0, 0.6, 0.4, 0.0], [0.0, 0.5, 0.5, 0.0]])
    assert pol.retired_pages() == 4
    loads, reclaimed = pol.prefetch(0, 100)
    assert len(reclaimed) == 1 and len(loads) == 1
    assert loads == [3]                                # the more valuable one stays
    assert pol.node_tier(3) == PC.GPU and pol.node_tier(4) == PC.HOST
    assert pol.node_tier(reclaimed[0]) == PC.HOST
    assert pol.retired_pages() == 2
    # the withdrawn node is still on offer next time
    pol._b = np.zeros(8, np.int64)
    loads, reclaimed = pol.prefetch(0, 100)
    assert loads == [4] and len(reclaimed) == 1
