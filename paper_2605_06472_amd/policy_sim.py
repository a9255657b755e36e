"""Synthetic dynamic-workflow driver for the policy core.

A seeded stand-in for the paper's workloads (Sec. 6.1 runs HoVer / SWE-bench / FinanceBench
traces through agent frameworks; none of that is available here).  It keeps their structure
(Sec. 2): a looped global call graph of agents walked as a Markov chain, a *global* cache
(one system prompt shared by everybody, one description node per agent) and a *private*
cache (per workflow and agent, one node per invocation, re-read when a loop re-invokes the
agent), a GPU tier of fixed capacity and a host tier behind it.  The forecast handed to the
policy is the chain's own K-step distribution, conditioned on survival step by step (the
paper's predictor is replaced by the ground truth, optionally blurred towards uniform).

The driver owns nothing of the method: it calls a policy object (the C++ core through
``policy.Policy`` or the reference model) and counts GPU hits in pages.
"""
import numpy as np

GPU, HOST = 0, 1

AGENTS = ["planner", "analyzer", "coder", "tester", "reviewer", "summarizer"]
# transition probabilities, rows = current agent, columns = next agent ..., END last
CALL_GRAPH = np.array([
    # plan  anal  code  test  rev   sum   END
    [0.00, 0.90, 0.00, 0.00, 0.00, 0.00, 0.10],   # planner
    [0.00, 0.00, 0.85, 0.00, 0.05, 0.00, 0.10],   # analyzer
    [0.00, 0.00, 0.00, 0.95, 0.00, 0.00, 0.05],   # coder
    [0.00, 0.00, 0.40, 0.00, 0.45, 0.00, 0.15],   # tester (retry loop back to the coder)
    [0.15, 0.00, 0.10, 0.00, 0.00, 0.55, 0.20],   # reviewer (may send the work back)
    [0.00, 0.00, 0.00, 0.00, 0.00, 0.00, 1.00],   # summarizer
])


def k_step_forecast(current_agent, K, blur=0.0):
    """P^(k), k = 1..K: distribution of the k-th next invocation (END last) given that the
    workflow is still running at step k (Sec. 4.2.2; App. G.1, probabilistic model)."""
    V = CALL_GRAPH.shape[0]
    rows = []
    state = np.zeros(V)
    state[current_agent] = 1.0
    for _ in range(K):
        d = state @ CALL_GRAPH                      # over V agents + END
        rows.append(d)
        alive = d[:V].sum()
        state = d[:V] / alive if alive > 0 else np.zeros(V)
        if alive == 0:
            state = np.zeros(V)
    out = np.array([r if r.sum() > 0 else np.eye(V + 1)[V] for r in rows])
    if blur:
        out = (1 - blur) * out + blur / (V + 1)
    return out


class World:
    def __init__(self, policy, capacity_pages, concurrency, seed, horizon, prefetch=False,
                 bw_budget_pages=24, sys_pages=8, desc_pages=4, turn_pages=6, blur=0.0):
        self.p, self.cap, self.K = policy, capacity_pages, horizon
        self.prefetch, self.bw = prefetch, bw_budget_pages
        self.turn_pages, self.blur = turn_pages, blur
        self.rng = np.random.default_rng(seed)
        self.tier, self.pages, self.parent = {}, {}, {}
        self.next_id = 0
        self.used = 0
        self.sys = self._new_node(-1, sys_pages)
        self.desc = [self._new_node(self.sys, desc_pages) for _ in AGENTS]
        self.chains = {}                             # (workflow, agent) -> private node ids
        self.cur = {}                                # workflow -> current agent
        self.next_wf = 0
        self.hit_pages = self.host_pages = self.miss_pages = 0
        self.decisions = []                          # everything the policy decided, for comparison
        for _ in range(concurrency):
            self._spawn()

    # ---- residency bookkeeping (mirrors what the policy is told) ----------------------------
    def _new_node(self, parent, pages):
        nid = self.next_id
        self.next_id += 1
        self._make_room(pages)
        self.p.node_add(nid, parent, pages, GPU)
        self.tier[nid], self.pages[nid], self.parent[nid] = GPU, pages, parent
        self.used += pages
        return nid

    def _make_room(self, pages):
        need = self.used + pages - self.cap
        if need > 0:
            ids, freed = self.p.evict(need, True)
            self.decisions.append(("evict", tuple(ids)))
            for i in ids:
                self.tier[i] = HOST
            self.used -= freed
            # pinned paths can make the tier overflow for a moment; the run keeps going

    def _spawn(self):
        w = self.next_wf
        self.next_wf += 1
        self.cur[w] = 0
        self._invoke(w, 0)

    def _invoke(self, w, agent):
        chain = self.chains.setdefault((w, agent), [])
        path = [self.sys, self.desc[agent]] + chain
        for nid in path:
            if self.tier[nid] == GPU:
                self.hit_pages += self.pages[nid]
            else:
                self.host_pages += self.pages[nid]
        for nid in path:
            if self.tier[nid] == GPU:
                self.p.node_pin(nid, 1)
        for nid in path:                             # host hits are swapped back in, prefix first
            if self.tier[nid] == HOST:
                self._make_room(self.pages[nid])
                self.p.node_set_tier(nid, GPU)
                self.tier[nid] = GPU
                self.used += self.pages[nid]
                self.p.node_pin(nid, 1)
        self.p.access(w, agent, path)
        new = self._new_node(path[-1], self.turn_pages)          # the KV this invocation produces
        self.miss_pages += self.turn_pages
        self.p.access(w, agent, [new])
        chain.append(new)
        for nid in path:
            self.p.node_pin(nid, -1)
        self.p.forecast(w, k_step_forecast(agent, self.K, self.blur))

    def step(self):
        live = sorted(self.cur)
        w = live[int(self.rng.integers(len(live)))]
        nxt = int(self.rng.choice(len(AGENTS) + 1, p=CALL_GRAPH[self.cur[w]]))
        if nxt == len(AGENTS):
            self.p.terminate(w)
            del self.cur[w]
            self._spawn()
        else:
            self.cur[w] = nxt
            self._invoke(w, nxt)
        if self.prefetch:                            # every scheduler tick here is a pure-decode batch
            loads, reclaimed = self.p.prefetch(max(self.cap - self.used, 0), self.bw, True, True)
            self.decisions.append(("prefetch", tuple(loads), tuple(reclaimed)))
            for i in reclaimed:
                self.tier[i] = HOST
                self.used -= self.pages[i]
            for i in loads:
                self.tier[i] = GPU
                self.used += self.pages[i]

    def run(self, steps):
        for _ in range(steps):
            self.step()
        reused = self.hit_pages + self.host_pages
        return {"gpu_hit_rate": self.hit_pages / max(reused, 1), "gpu_hit_pages": self.hit_pages,
                "host_hit_pages": self.host_pages, "new_pages": self.miss_pages}
