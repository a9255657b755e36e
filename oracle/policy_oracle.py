"""Reference model of the PBKV cache-management policy (test infrastructure, not a product path).

A plain, slow restatement of the paper's policy layer, used only by the tests, by
``__graft_entry__.smoke()`` and by bench.py's CPU-baseline leg to check the C++ policy core.
Every decision is taken by scanning and sorting all nodes; there is no heap, no cached weight
and no incremental update, so that each function can be checked against the paper by eye.

What it follows:
  * lifecycle tags and retired cache, ranked by the number of workflows that accessed a
    node                                                             (Sec. 4.2.1)
  * access indicators A_w(c), one-step Value(c)                      (Sec. 4.2.2, Eq. 1)
  * survival s_w^(k) and the K-step Score(c) with confidence decay   (Sec. 4.2.2, Eq. 2)
  * hierarchical eviction: retired cache is drained before any active node, active nodes
    leave in ascending Score                                         (Sec. 4.2.2-4.2.3)
  * conservative prefetch: region S_a = free + retired, S = min(S_a, S_bw), only on
    pure-decode batches, host nodes ranked by Value, greedy          (Sec. 4.3)
  * inheritance customisation of A_w(c)                              (Sec. 5, Limitations)

Readings where the paper is silent (the C++ core takes the same ones):
  R1  a node nobody has accessed is retired (all of its zero workflows have terminated);
  R2  eviction respects the radix tree: only nodes without a GPU-resident child leave, and a
      node a running request has pinned never leaves;
  R3  ties: retired nodes by (accessor count, last access, id); active nodes by (Score or, in
      the LRU-based modes, last access; then last access, id), all ascending;
  R4  evicted nodes move to the host tier when `to_host` is set, otherwise they are dropped;
  R5  prefetch considers host nodes whose parent is GPU-resident (or absent), skips nodes of
      Value 0, takes candidates in descending Value (ties: smaller depth, smaller id) and
      stops at the first one that does not fit the remaining budget;
  R6  when the selected nodes need more than the free pages, retired nodes are reclaimed in
      retired order to cover the difference;
  R7  S_bw uses the arithmetic running means of the observed link rate and step duration.
"""
import math

GPU, HOST = 0, 1
MODE_LRU, MODE_LAE, MODE_HE = 0, 1, 2


class Node:
    def __init__(self, nid, parent, pages, tier, depth):
        self.id, self.parent, self.pages, self.tier, self.depth = nid, parent, pages, tier, depth
        self.masks = {}          # active workflow -> set of agents that accessed the node in it
        self.accessors = set()   # every workflow that ever accessed the node
        self.last_access = 0
        self.pins = 0


class Workflow:
    def __init__(self):
        self.active = True
        self.probs = None        # K rows of |V|+1 probabilities, END last


class PolicyOracle:
    def __init__(self, num_agents, horizon, gamma, mode=MODE_HE):
        self.V, self.K, self.gamma, self.mode = num_agents, horizon, gamma, mode
        self.nodes, self.workflows = {}, {}
        self.clock = 0
        self.inherit = {a: {a} for a in range(num_agents)}
        self.step_obs, self.xfer_obs = [], []

    # ---- bookkeeping -------------------------------------------------------------------
    def set_inherit(self, src, dst):
        """Agent dst inherits the cache agent src has accessed (Sec. 5)."""
        self.inherit[src].add(dst)

    def node_add(self, nid, parent, pages, tier=GPU):
        assert nid not in self.nodes and pages > 0
        depth = 0 if parent < 0 else self.nodes[parent].depth + 1
        self.nodes[nid] = Node(nid, parent, pages, tier, depth)

    def node_remove(self, nid):
        assert not any(n.parent == nid for n in self.nodes.values())
        del self.nodes[nid]

    def node_set_tier(self, nid, tier):
        self.nodes[nid].tier = tier

    def node_pin(self, nid, delta):
        self.nodes[nid].pins += delta
        assert self.nodes[nid].pins >= 0

    def access(self, workflow, agent, node_ids):
        wf = self.workflows.setdefault(workflow, Workflow())
        assert wf.active
        for nid in node_ids:
            n = self.nodes[nid]
            self.clock += 1
            n.last_access = self.clock
            n.accessors.add(workflow)
            n.masks.setdefault(workflow, set()).update(self.inherit[agent])

    def forecast(self, workflow, probs):
        wf = self.workflows.setdefault(workflow, Workflow())
        assert wf.active and len(probs) == self.K
        for row in probs:
            assert len(row) == self.V + 1 and all(0.0 <= x <= 1.0 for x in row)
            assert abs(sum(row) - 1.0) <= 1e-6
        wf.probs = [list(map(float, row)) for row in probs]

    def terminate(self, workflow):
        wf = self.workflows[workflow]
        wf.active = False
        wf.probs = None
        for n in self.nodes.values():
            n.masks.pop(workflow, None)

    # ---- Eq. 1 and Eq. 2 ----------------------------------------------------------------
    def survival(self, workflow, k):
        """s_w^(k) = prod_{j<k} (1 - p_END^(j)), k = 1..K  (Sec. 4.2.2)."""
        s = 1.0
        for j in range(1, k):
            s *= 1.0 - self.workflows[workflow].probs[j - 1][self.V]
        return s

    def value(self, nid):
        """Eq. 1: sum over the active workflows of the node of A_w(c) . P_w (next step)."""
        n = self.nodes[nid]
        total = 0.0
        for w in sorted(n.masks):
            p = self.workflows[w].probs
            if p is not None:
                total += sum(p[0][a] for a in sorted(n.masks[w]))
        return total

    def score(self, nid):
        """Eq. 2: sum_k gamma^(k-1) sum_w s_w^(k) A_w(c) . P_w^(k)."""
        n = self.nodes[nid]
        total = 0.0
        for k in range(1, self.K + 1):
            inner = 0.0
            for w in sorted(n.masks):
                p = self.workflows[w].probs
                if p is not None:
                    inner += self.survival(w, k) * sum(p[k - 1][a] for a in sorted(n.masks[w]))
            total += self.gamma ** (k - 1) * inner
        return total

    def is_retired(self, nid):
        return len(self.nodes[nid].masks) == 0

    # ---- eviction -----------------------------------------------------------------------
    def _gpu_children(self, nid):
        return sum(1 for n in self.nodes.values() if n.parent == nid and n.tier == GPU)

    def _evict_key(self, n):
        if self.mode == MODE_LRU:
            return (1, n.last_access, n.last_access, n.id)
        if self.is_retired(n.id):
            return (0, len(n.accessors), n.last_access, n.id)
        if self.mode == MODE_LAE:
            return (1, n.last_access, n.last_access, n.id)
        return (1, self.score(n.id), n.last_access, n.id)

    def _evictable(self, retired_only=False):
        c = [n for n in self.nodes.values()
             if n.tier == GPU and n.pins == 0 and self._gpu_children(n.id) == 0]
        if retired_only:
            c = [n for n in c if self.mode != MODE_LRU and self.is_retired(n.id)]
        return sorted(c, key=self._evict_key)

    def _drop(self, n, to_host):
        if to_host:
            n.tier = HOST
        else:
            for ch in [x for x in self.nodes.values() if x.parent == n.id]:
                self._drop_subtree(ch)
            del self.nodes[n.id]

    def _drop_subtree(self, n):
        for ch in [x for x in self.nodes.values() if x.parent == n.id]:
            self._drop_subtree(ch)
        del self.nodes[n.id]

    def evict(self, pages_needed, to_host=True):
        """Sec. 4.2.2 / 4.2.3: retired cache first, then ascending Score, until the space is freed."""
        out, freed = [], 0
        while freed < pages_needed:
            cand = self._evictable()
            if not cand:
                break
            n = cand[0]
            out.append(n.id)
            freed += n.pages
            self._drop(n, to_host)
        return out, freed

    # ---- prefetch -----------------------------------------------------------------------
    def observe_step(self, seconds):
        self.step_obs.append(float(seconds))

    def observe_transfer(self, nbytes, seconds):
        self.xfer_obs.append(float(nbytes) / float(seconds))

    def bandwidth_budget_pages(self, page_bytes):
        """S_bw = Bandwidth * StepDuration in pages, both running means (Sec. 4.3)."""
        if not self.step_obs or not self.xfer_obs:
            return 0
        bw = sum(self.xfer_obs) / len(self.xfer_obs)
        step = sum(self.step_obs) / len(self.step_obs)
        return int(math.floor(bw * step / page_bytes))

    def retired_pages(self):
        if self.mode == MODE_LRU:
            return 0
        return sum(n.pages for n in self.nodes.values()
                   if n.tier == GPU and n.pins == 0 and self.is_retired(n.id))

    def prefetch(self, free_pages, bw_budget_pages, pure_decode=True, to_host=True):
        """Sec. 4.3.  Returns (nodes to load in order, retired nodes reclaimed to make room)."""
        if not pure_decode:
            return [], []
        budget = min(free_pages + self.retired_pages(), bw_budget_pages)
        loads, used = [], 0
        while True:
            cand = [n for n in self.nodes.values() if n.tier == HOST
                    and (n.parent < 0 or self.nodes[n.parent].tier == GPU) and self.value(n.id) > 0.0]
            if not cand:
                break
            cand.sort(key=lambda n: (-self.value(n.id), n.depth, n.id))
            n = cand[0]
            if used + n.pages > budget:
                break
            used += n.pages
            n.tier = GPU
            n.pins += 1              # a node being loaded cannot be reclaimed in the same decision
            loads.append(n.id)
        reclaimed, freed = [], 0
        while used - freed > free_pages:
            cand = self._evictable(retired_only=True)
            assert cand, "S_a promised retired space that cannot be reclaimed"
            n = cand[0]
            reclaimed.append(n.id)
            freed += n.pages
            self._drop(n, to_host)
        for nid in loads:
            self.nodes[nid].pins -= 1
        return loads, reclaimed


def expected_discounted_misses(probs, mask, gamma):
    """Brute force for Lemma 1 (App. G.2): enumerate every K-step trajectory of one workflow
    (agent or END at each step, nothing after END) and add gamma^(k-1) for every step at which
    the workflow invokes an agent of `mask`, weighted by the trajectory's probability."""
    K, V = len(probs), len(probs[0]) - 1
    total = 0.0

    def walk(k, p):
        nonlocal total
        if k == K or p == 0.0:
            return
        for a in range(V):
            q = p * probs[k][a]
            if a in mask:
                total += q * gamma ** k
            walk(k + 1, q)
        # END: the trajectory stops, no later step counts

    walk(0, 1.0)
    return total
