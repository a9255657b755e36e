"""Pins of the policy reference model (oracle/policy_oracle.py) against what the paper fixes:
a hand-evaluated example of Eq. 1 / Eq. 2, the brute-force expected discounted miss count of
Lemma 1 (App. G.2), the Lipschitz bound of Lemma 2 (App. G.3), the retired / hierarchical rules
of Sec. 4.2.1 and 4.2.3, the budget rule of Sec. 4.3, and a textbook LRU."""
import collections
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import policy_oracle as PO

HERE = os.path.dirname(os.path.abspath(__file__))


def random_forecast(rng, K, V, end_scale=1.0):
    p = rng.random((K, V + 1))
    p[:, V] *= end_scale
    return (p / p.sum(1, keepdims=True)).tolist()


def build_golden():
    g = json.load(open(os.path.join(HERE, "golden", "policy_score_example.json")))
    o = PO.PolicyOracle(g["num_agents"], g["horizon"], float(Fraction(g["gamma"])))
    for i, name in enumerate(sorted(g["nodes"])):
        o.node_add(i, -1, 1)
    ids = {name: i for i, name in enumerate(sorted(g["nodes"]))}
    for name, nd in g["nodes"].items():
        for w, agents in nd["access"].items():
            for a in agents:
                o.access(int(w), a, [ids[name]])
    for w, rows in g["forecasts"].items():
        o.forecast(int(w), [[float(Fraction(x)) for x in row] for row in rows])
    for w in g["terminated"]:
        o.terminate(w)
    return g, o, ids


def test_hand_evaluated_value_and_score():
    g, o, ids = build_golden()
    for w, s in g["survival"].items():
        assert [o.survival(int(w), k) for k in (1, 2, 3)] == [float(Fraction(x)) for x in s]
    for name, nd in g["nodes"].items():
        assert o.score(ids[name]) == float(Fraction(nd["score"])), name
        assert o.value(ids[name]) == float(Fraction(nd["value"])), name
        assert o.is_retired(ids[name]) == nd["retired"], name
        if "score_terms" in nd:
            assert sum(Fraction(x) for x in nd["score_terms"]) == Fraction(nd["score"])


def test_score_equals_expected_discounted_miss_count():
    """Lemma 1 (App. G.2): Score(c) is the expected discounted number of misses attributable to
    evicting c; the right-hand side is enumerated trajectory by trajectory."""
    rng = np.random.default_rng(1)
    V, K, gamma = 3, 4, 0.7
    o = PO.PolicyOracle(V, K, gamma)
    o.node_add(0, -1, 1)
    want = 0.0
    for w in range(4):
        mask = set(int(a) for a in rng.choice(V, size=int(rng.integers(1, V + 1)), replace=False))
        for a in mask:
            o.access(w, a, [0])
        probs = random_forecast(rng, K, V)
        o.forecast(w, probs)
        want += PO.expected_discounted_misses(probs, mask, gamma)
    assert o.score(0) == pytest.approx(want, rel=1e-13)


def test_one_step_horizon_is_the_value():
    rng = np.random.default_rng(2)
    o = PO.PolicyOracle(5, 1, 0.7)
    o.node_add(0, -1, 1)
    for w in range(6):
        o.access(w, int(rng.integers(5)), [0])
        o.forecast(w, random_forecast(rng, 1, 5))
    assert o.score(0) == pytest.approx(o.value(0), rel=1e-15)


def test_lipschitz_bound_of_the_score():
    """Lemma 2 (App. G.3): |Score - Score^| <= (1 - gamma^K) / (2 (1 - gamma)) * eps_c^gamma with
    eps_c^gamma = sum_w sum_k gamma^(k-1) ||P_w^(k) - P^_w^(k)||_1."""
    rng = np.random.default_rng(3)
    V, K, gamma = 6, 3, 0.7
    for trial in range(200):
        a, b = PO.PolicyOracle(V, K, gamma), PO.PolicyOracle(V, K, gamma)
        a.node_add(0, -1, 1)
        b.node_add(0, -1, 1)
        eps = 0.0
        for w in range(int(rng.integers(1, 6))):
            for ag in rng.choice(V, size=int(rng.integers(1, 4)), replace=False):
                a.access(w, int(ag), [0])
                b.access(w, int(ag), [0])
            p = np.array(random_forecast(rng, K, V))
            lam = rng.random() * (0.05 if trial % 2 else 1.0)
            q = (1 - lam) * p + lam * np.array(random_forecast(rng, K, V))
            a.forecast(w, p.tolist())
            b.forecast(w, q.tolist())
            eps += sum(gamma ** k * np.abs(p[k] - q[k]).sum() for k in range(K))
        bound = (1 - gamma ** K) / (2 * (1 - gamma)) * eps
        assert abs(a.score(0) - b.score(0)) <= bound + 1e-12


def test_score_never_grows_along_a_radix_path_and_retired_is_zero():
    rng = np.random.default_rng(4)
    o = PO.PolicyOracle(4, 3, 0.7)
    for i in range(6):
        o.node_add(i, i - 1, 1)
    for w in range(5):
        depth = int(rng.integers(1, 7))
        o.access(w, int(rng.integers(4)), list(range(depth)))      # a request touches a whole prefix
        o.forecast(w, random_forecast(rng, 3, 4))
    s = [o.score(i) for i in range(6)]
    assert all(s[i] >= s[i + 1] - 1e-15 for i in range(5))
    for w in range(5):
        o.terminate(w)
    assert all(o.score(i) == 0.0 and o.is_retired(i) for i in range(6))


def test_hierarchical_eviction_drains_retired_cache_first():
    """Sec. 4.2.1 / 4.2.3: retired nodes go first, the less shared ones before the popular ones;
    only then active nodes, in ascending Score."""
    o = PO.PolicyOracle(2, 2, 0.5)
    for i in range(6):
        o.node_add(i, -1, 1)
    # nodes 0, 1 retired (1 is the more popular); 2..5 active with scores 0.1 .. 0.4 + eps
    for w in (10, 11, 12):
        o.access(w, 0, [1])
    o.access(10, 0, [0])
    for i, p in zip(range(2, 6), (0.4, 0.1, 0.3, 0.2)):
        o.access(20 + i, 0, [i])
        o.forecast(20 + i, [[p, 0.0, 1 - p], [0.0, 0.0, 1.0]])
    for w in (10, 11, 12):
        o.terminate(w)
    order, freed = o.evict(6)
    assert order == [0, 1, 3, 5, 4, 2] and freed == 6


def test_eviction_keeps_the_radix_prefix_structure_and_pins():
    o = PO.PolicyOracle(2, 1, 0.7)
    o.node_add(0, -1, 2)
    o.node_add(1, 0, 3)
    o.node_add(2, 0, 1)
    o.access(1, 0, [0, 1])
    o.access(2, 1, [0, 2])
    o.forecast(1, [[0.5, 0.0, 0.5]])
    o.forecast(2, [[0.0, 0.1, 0.9]])
    o.node_pin(2, 1)                                  # a running request holds node 2
    order, freed = o.evict(100)
    assert order == [1] and freed == 3                # 0 keeps a GPU child, 2 is pinned
    o.node_pin(2, -1)
    order, freed = o.evict(100)
    assert order == [2, 0] and freed == 3
    assert all(n.tier == PO.HOST for n in o.nodes.values())


def test_lru_mode_is_a_textbook_lru():
    rng = np.random.default_rng(5)
    o = PO.PolicyOracle(1, 1, 0.7, mode=PO.MODE_LRU)
    ref = collections.OrderedDict()
    for i in range(20):
        o.node_add(i, -1, 1, PO.HOST)                 # nothing is GPU-resident before its first access
    for step in range(300):
        i = int(rng.integers(20))
        if o.nodes[i].tier == PO.HOST:
            o.node_set_tier(i, PO.GPU)
        o.access(0, 0, [i])
        ref.pop(i, None)
        ref[i] = True
        if len(ref) > 8:
            victim, _ = ref.popitem(last=False)
            got, _ = o.evict(1)
            assert got == [victim]


def test_lifecycle_mode_falls_back_to_lru_once_retired_cache_is_drained():
    o = PO.PolicyOracle(1, 1, 0.7, mode=PO.MODE_LAE)
    for i in range(4):
        o.node_add(i, -1, 1)
    o.access(1, 0, [2])
    o.access(2, 0, [0])
    o.access(3, 0, [3])
    o.access(4, 0, [1])
    o.forecast(2, [[1.0, 0.0]])          # a forecast must not matter in this mode
    o.terminate(3)
    assert o.evict(4)[0] == [3, 2, 0, 1]


def test_prefetch_budget_is_the_smaller_of_space_and_bandwidth():
    """Sec. 4.3: S = min(S_a, S_bw), S_a = free + retired; candidates in descending Value; nothing
    on a batch that is not pure decode; active cache is never displaced."""
    def world():
        o = PO.PolicyOracle(3, 2, 0.7)
        for i in range(5):
            o.node_add(i, -1, 2, PO.HOST)                       # host candidates, 2 pages each
        o.node_add(10, -1, 3)                                   # retired GPU node
        o.node_add(11, -1, 3)                                   # active GPU node
        o.access(9, 0, [10])
        o.terminate(9)
        o.access(1, 1, [11])
        for i, p in enumerate((0.1, 0.5, 0.0, 0.3, 0.2)):
            o.access(100 + i, 0, [i])
            o.forecast(100 + i, [[p, 0.0, 0.0, 1 - p], [0.0, 0.0, 0.0, 1.0]])
        return o
    assert world().prefetch(100, 100, pure_decode=False) == ([], [])
    assert world().prefetch(100, 5) == ([1, 3], [])             # bandwidth-bound: 2 of 2 pages fit 5
    assert world().prefetch(1, 100) == ([1, 3], [10])           # S_a = 1 + 3 = 4 pages, needs the retired node
    assert world().prefetch(0, 100) == ([1], [10])              # S_a = 3
    loads, reclaimed = world().prefetch(100, 100)
    assert loads == [1, 3, 4, 0] and reclaimed == []            # the zero-value node stays on the host
    o = world()
    o.prefetch(0, 100)
    assert o.nodes[11].tier == PO.GPU                           # the active node was not touched


def test_bandwidth_budget_uses_running_means():
    o = PO.PolicyOracle(1, 1, 0.7)
    assert o.bandwidth_budget_pages(65536) == 0
    o.observe_transfer(40e9 * 0.01, 0.01)
    o.observe_transfer(60e9 * 0.02, 0.02)
    o.observe_step(0.010)
    o.observe_step(0.014)
    assert o.bandwidth_budget_pages(65536) == int(50e9 * 0.012 // 65536)


def test_inheritance_rule_extends_the_access_indicator():
    """Sec. 5 (Limitations): if agent j inherits what agent i accessed, A_w(c)[j] = 1 whenever A_w(c)[i] = 1."""
    o = PO.PolicyOracle(3, 1, 0.7)
    o.set_inherit(0, 2)
    o.node_add(0, -1, 1)
    o.access(1, 0, [0])
    o.forecast(1, [[0.2, 0.3, 0.4, 0.1]])
    assert o.value(0) == pytest.approx(0.2 + 0.4)


# ---- the pins must notice a planted mistake ---------------------------------------------------
class _SurvivalIncludesStepK(PO.PolicyOracle):
    def survival(self, workflow, k):
        return super().survival(workflow, k + 1) if k < self.K else super().survival(workflow, k) * (
            1.0 - self.workflows[workflow].probs[k - 1][self.V])


class _DecayOffByOne(PO.PolicyOracle):
    def score(self, nid):
        return self.gamma * super().score(nid)


class _CountsTerminatedWorkflows(PO.PolicyOracle):
    def terminate(self, workflow):
        self.workflows[workflow].active = False        # keeps the forecast and the access masks


class _NoSurvival(PO.PolicyOracle):
    def survival(self, workflow, k):
        return 1.0


def _golden_holds(cls):
    g = json.load(open(os.path.join(HERE, "golden", "policy_score_example.json")))
    o = cls(g["num_agents"], g["horizon"], float(Fraction(g["gamma"])))
    ids = {name: i for i, name in enumerate(sorted(g["nodes"]))}
    for i in ids.values():
        o.node_add(i, -1, 1)
    for name, nd in g["nodes"].items():
        for w, agents in nd["access"].items():
            for a in agents:
                o.access(int(w), a, [ids[name]])
    for w, rows in g["forecasts"].items():
        o.forecast(int(w), [[float(Fraction(x)) for x in row] for row in rows])
    o.forecast(3, [[0.25, 0.25, 0.25, 0.25]] * 3)
    for w in g["terminated"]:
        o.terminate(w)
    return all(o.score(ids[n]) == float(Fraction(nd["score"])) for n, nd in g["nodes"].items())


def test_planted_mistakes_fail_the_hand_example():
    assert _golden_holds(PO.PolicyOracle)
    for mutant in (_SurvivalIncludesStepK, _DecayOffByOne, _CountsTerminatedWorkflows, _NoSurvival):
        assert not _golden_holds(mutant), mutant.__name__
