// Cache-management policy core behind include/pbkv_policy.h: lifecycle tags, access indicators,
// the scores of Eq. 1 / Eq. 2, indexed heaps, hierarchical eviction and conservative prefetch.
// Host code only.
//
// Cost model.  A forecast is folded once into per-agent weights
//     wt_w[a] = sum_k gamma^(k-1) s_w^(k) P_w^(k)[a]        (Eq. 2 with the survival product)
//     v1_w[a] = P_w^(1)[a]                                  (Eq. 1)
// so that a node's score is a sum over its active workflows of the weights its access mask
// selects; a state change of workflow w re-keys only w's nodes, O(log n) each (Sec. 5).
#include "../../include/pbkv.h"
#include "../../include/pbkv_policy.h"
#include "pbkv_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <unordered_map>
#include <vector>

namespace {

using pbkv::set_error;

struct Node;

struct Entry {                      // an active workflow's access mask on a node
    int64_t wf;
    uint64_t mask;
};

struct Key {                        // lexicographic, ascending = leaves / loads first
    double a, b, c, d;
    bool operator<(const Key &o) const {
        if (a != o.a) return a < o.a;
        if (b != o.b) return b < o.b;
        if (c != o.c) return c < o.c;
        return d < o.d;
    }
};

struct Node {
    int64_t id = 0, parent_id = -1;
    Node *parent = nullptr;
    std::vector<Node *> children;
    int32_t pages = 0, tier = PBKV_TIER_GPU, depth = 0, pins = 0, gpu_children = 0;
    int64_t accessors = 0;          // distinct workflows that ever accessed the node
    uint64_t last_access = 0;
    std::vector<Entry> act;         // active workflows, ascending id
    double score = 0.0, value = 0.0;
    int64_t retired_contrib = 0;    // pages this node adds to the reclaimable retired space
    int pos[2] = {-1, -1};          // position in the eviction heap / the load heap
    Key key[2];
};

// Indexed binary min-heap; WHICH selects the position / key slot inside the node.
template <int WHICH>
struct Heap {
    std::vector<Node *> h;
    bool empty() const { return h.empty(); }
    Node *top() const { return h[0]; }
    void place(size_t i, Node *n) { h[i] = n; n->pos[WHICH] = (int)i; }
    void up(size_t i) {
        Node *n = h[i];
        while (i > 0) {
            const size_t p = (i - 1) / 2;
            if (!(n->key[WHICH] < h[p]->key[WHICH])) break;
            place(i, h[p]);
            i = p;
        }
        place(i, n);
    }
    void down(size_t i) {
        Node *n = h[i];
        const size_t sz = h.size();
        for (;;) {
            size_t c = 2 * i + 1;
            if (c >= sz) break;
            if (c + 1 < sz && h[c + 1]->key[WHICH] < h[c]->key[WHICH]) c++;
            if (!(h[c]->key[WHICH] < n->key[WHICH])) break;
            place(i, h[c]);
            i = c;
        }
        place(i, n);
    }
    void set(Node *n, const Key &k) {             // insert or re-key
        n->key[WHICH] = k;
        if (n->pos[WHICH] < 0) {
            h.push_back(n);
            up(h.size() - 1);
        } else {
            const size_t i = (size_t)n->pos[WHICH];
            up(i);
            down((size_t)n->pos[WHICH]);
        }
    }
    void erase(Node *n) {
        const int i = n->pos[WHICH];
        if (i < 0) return;
        n->pos[WHICH] = -1;
        Node *last = h.back();
        h.pop_back();
        if (last != n) {
            place((size_t)i, last);
            up((size_t)i);
            down((size_t)last->pos[WHICH]);
        }
    }
};

struct Workflow {
    bool active = true, has_forecast = false;
    double wt[64], v1[64];
    std::vector<int64_t> nodes;     // ids of the nodes it has accessed (may go stale; checked on use)
};

}  // namespace

struct pbkv_policy {
    int32_t V, K, mode;
    double gamma;
    uint64_t inherit[64];
    uint64_t clock = 0;
    std::unordered_map<int64_t, Node *> nodes;
    std::unordered_map<int64_t, Workflow> workflows;
    Heap<0> evictable;
    Heap<1> loadable;
    int64_t retired_total = 0;
    double step_sum = 0, rate_sum = 0;
    int64_t step_n = 0, rate_n = 0;

    Node *find(int64_t id) const {
        auto it = nodes.find(id);
        return it == nodes.end() ? nullptr : it->second;
    }

    void rescore(Node *n) {
        double s = 0.0, v = 0.0;
        for (const Entry &e : n->act) {
            const Workflow &w = workflows.find(e.wf)->second;
            if (!w.has_forecast) continue;
            double cs = 0.0, cv = 0.0;
            for (uint64_t m = e.mask; m; m &= m - 1) {
                const int a = __builtin_ctzll(m);
                cs += w.wt[a];
                cv += w.v1[a];
            }
            s += cs;
            v += cv;
        }
        n->score = s;
        n->value = v;
    }

    bool retired(const Node *n) const { return n->act.empty(); }

    // bring heap membership, keys and the retired-space total in line with the node's state
    void refresh(Node *n) {
        const int64_t contrib =
            (mode != PBKV_MODE_LRU && n->tier == PBKV_TIER_GPU && n->pins == 0 && retired(n)) ? n->pages : 0;
        retired_total += contrib - n->retired_contrib;
        n->retired_contrib = contrib;

        if (n->tier == PBKV_TIER_GPU && n->gpu_children == 0 && n->pins == 0) {
            Key k;
            const double la = (double)n->last_access, id = (double)n->id;
            if (mode == PBKV_MODE_LRU) k = Key{1.0, la, la, id};
            else if (retired(n)) k = Key{0.0, (double)n->accessors, la, id};
            else if (mode == PBKV_MODE_LAE) k = Key{1.0, la, la, id};
            else k = Key{1.0, n->score, la, id};
            evictable.set(n, k);
        } else {
            evictable.erase(n);
        }
        if (n->tier == PBKV_TIER_HOST && (!n->parent || n->parent->tier == PBKV_TIER_GPU) && n->value > 0.0)
            loadable.set(n, Key{-n->value, (double)n->depth, (double)n->id, 0.0});
        else
            loadable.erase(n);
    }

    void set_tier(Node *n, int32_t tier) {
        if (n->tier == tier) return;
        if (n->parent) n->parent->gpu_children += tier == PBKV_TIER_GPU ? 1 : -1;
        n->tier = tier;
        refresh(n);
        if (n->parent) refresh(n->parent);
        for (Node *c : n->children) refresh(c);
    }

    void unlink(Node *n) {                          // n has no children
        evictable.erase(n);
        loadable.erase(n);
        retired_total -= n->retired_contrib;
        if (n->parent) {
            auto &ch = n->parent->children;
            ch.erase(std::find(ch.begin(), ch.end(), n));
            if (n->tier == PBKV_TIER_GPU) n->parent->gpu_children--;
            refresh(n->parent);
        }
        nodes.erase(n->id);
        delete n;
    }

    void forget_subtree(Node *n) {
        while (!n->children.empty()) forget_subtree(n->children.back());
        unlink(n);
    }

    // the node leaves the GPU: to the host tier, or out of the books with its host descendants
    void leave_gpu(Node *n, bool to_host) {
        if (to_host) set_tier(n, PBKV_TIER_HOST);
        else forget_subtree(n);
    }
};

extern "C" {

pbkv_policy *pbkv_policy_create(int32_t num_agents, int32_t horizon, double gamma, int32_t mode) {
    pbkv::clear_error();
    if (num_agents < 1 || num_agents > 64 || horizon < 1 || horizon > 8 || !(gamma > 0.0 && gamma <= 1.0) ||
        mode < PBKV_MODE_LRU || mode > PBKV_MODE_HE) {
        set_error(PBKV_ERR_SHAPE, "pbkv_policy_create: agents %d (1..64), horizon %d (1..8), gamma %g (0..1], mode %d",
                  num_agents, horizon, gamma, mode);
        return nullptr;
    }
    pbkv_policy *p = new pbkv_policy;
    p->V = num_agents;
    p->K = horizon;
    p->gamma = gamma;
    p->mode = mode;
    for (int a = 0; a < 64; a++) p->inherit[a] = 1ull << a;
    return p;
}

void pbkv_policy_destroy(pbkv_policy *p) {
    if (!p) return;
    for (auto &kv : p->nodes) delete kv.second;
    delete p;
}

int pbkv_policy_set_inherit(pbkv_policy *p, int32_t src, int32_t dst) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    if (src < 0 || src >= p->V || dst < 0 || dst >= p->V) return set_error(PBKV_ERR_RANGE, "agent %d -> %d of %d", src, dst, p->V);
    p->inherit[src] |= 1ull << dst;
    return PBKV_OK;
}

int pbkv_policy_node_add(pbkv_policy *p, int64_t node, int64_t parent, int32_t pages, int32_t tier) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    if (pages <= 0 || (tier != PBKV_TIER_GPU && tier != PBKV_TIER_HOST))
        return set_error(PBKV_ERR_RANGE, "node %lld: pages %d, tier %d", (long long)node, pages, tier);
    if (p->find(node)) return set_error(PBKV_ERR_ALIAS, "node %lld exists", (long long)node);
    Node *par = nullptr;
    if (parent >= 0 && !(par = p->find(parent))) return set_error(PBKV_ERR_RANGE, "parent %lld unknown", (long long)parent);
    Node *n = new Node;
    n->id = node;
    n->parent_id = par ? parent : -1;
    n->parent = par;
    n->pages = pages;
    n->tier = tier;
    n->depth = par ? par->depth + 1 : 0;
    p->nodes.emplace(node, n);
    if (par) {
        par->children.push_back(n);
        if (tier == PBKV_TIER_GPU) par->gpu_children++;
        p->refresh(par);
    }
    p->refresh(n);
    return PBKV_OK;
}

int pbkv_policy_node_remove(pbkv_policy *p, int64_t node) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    Node *n = p->find(node);
    if (!n) return set_error(PBKV_ERR_RANGE, "node %lld unknown", (long long)node);
    if (!n->children.empty()) return set_error(PBKV_ERR_RANGE, "node %lld has children", (long long)node);
    p->unlink(n);
    return PBKV_OK;
}

int pbkv_policy_node_set_tier(pbkv_policy *p, int64_t node, int32_t tier) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    Node *n = p->find(node);
    if (!n || (tier != PBKV_TIER_GPU && tier != PBKV_TIER_HOST))
        return set_error(PBKV_ERR_RANGE, "node %lld unknown or tier %d", (long long)node, tier);
    p->set_tier(n, tier);
    return PBKV_OK;
}

int pbkv_policy_node_pin(pbkv_policy *p, int64_t node, int32_t delta) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    Node *n = p->find(node);
    if (!n || n->pins + delta < 0) return set_error(PBKV_ERR_RANGE, "node %lld unknown or pin count below zero", (long long)node);
    n->pins += delta;
    p->refresh(n);
    return PBKV_OK;
}

int pbkv_policy_access(pbkv_policy *p, int64_t workflow, int32_t agent, const int64_t *nodes, int32_t n_nodes) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    if (agent < 0 || agent >= p->V) return set_error(PBKV_ERR_RANGE, "agent %d of %d", agent, p->V);
    if (n_nodes < 0 || (n_nodes > 0 && !nodes)) return set_error(PBKV_ERR_NULL, "nodes is NULL");
    for (int i = 0; i < n_nodes; i++)
        if (!p->find(nodes[i])) return set_error(PBKV_ERR_RANGE, "node %lld unknown", (long long)nodes[i]);
    auto it = p->workflows.find(workflow);
    if (it == p->workflows.end()) it = p->workflows.emplace(workflow, Workflow()).first;
    Workflow &w = it->second;
    if (!w.active) return set_error(PBKV_ERR_RANGE, "workflow %lld has terminated", (long long)workflow);
    for (int i = 0; i < n_nodes; i++) {
        Node *n = p->find(nodes[i]);
        n->last_access = ++p->clock;
        auto e = std::lower_bound(n->act.begin(), n->act.end(), workflow,
                                  [](const Entry &x, int64_t id) { return x.wf < id; });
        bool changed = false;
        if (e == n->act.end() || e->wf != workflow) {
            e = n->act.insert(e, Entry{workflow, 0});
            n->accessors++;
            w.nodes.push_back(n->id);
            changed = true;
        }
        const uint64_t m = e->mask | p->inherit[agent];
        changed |= m != e->mask;
        e->mask = m;
        if (changed) p->rescore(n);
        p->refresh(n);
    }
    return PBKV_OK;
}

int pbkv_policy_forecast(pbkv_policy *p, int64_t workflow, const double *probs) {
    pbkv::clear_error();
    if (!p || !probs) return set_error(PBKV_ERR_NULL, "pbkv_policy_forecast: NULL argument");
    const int V = p->V, K = p->K;
    for (int k = 0; k < K; k++) {
        double sum = 0.0;
        for (int a = 0; a <= V; a++) {
            const double x = probs[k * (V + 1) + a];
            if (!(x >= 0.0 && x <= 1.0)) return set_error(PBKV_ERR_RANGE, "forecast step %d entry %d = %g", k + 1, a, x);
            sum += x;
        }
        if (std::fabs(sum - 1.0) > 1e-6) return set_error(PBKV_ERR_RANGE, "forecast step %d sums to %.9g", k + 1, sum);
    }
    auto it = p->workflows.find(workflow);
    if (it == p->workflows.end()) it = p->workflows.emplace(workflow, Workflow()).first;
    Workflow &w = it->second;
    if (!w.active) return set_error(PBKV_ERR_RANGE, "workflow %lld has terminated", (long long)workflow);
    for (int a = 0; a < V; a++) { w.wt[a] = 0.0; w.v1[a] = probs[a]; }
    double surv = 1.0, g = 1.0;                       // s^(k), gamma^(k-1)
    for (int k = 0; k < K; k++) {
        for (int a = 0; a < V; a++) w.wt[a] += g * surv * probs[k * (V + 1) + a];
        surv *= 1.0 - probs[k * (V + 1) + V];
        g *= p->gamma;
    }
    w.has_forecast = true;
    for (int64_t id : w.nodes) {
        Node *n = p->find(id);
        if (!n) continue;
        p->rescore(n);
        p->refresh(n);
    }
    return PBKV_OK;
}

int pbkv_policy_terminate(pbkv_policy *p, int64_t workflow) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    auto it = p->workflows.find(workflow);
    if (it == p->workflows.end()) return set_error(PBKV_ERR_RANGE, "workflow %lld unknown", (long long)workflow);
    Workflow &w = it->second;
    if (!w.active) return PBKV_OK;
    w.active = false;
    w.has_forecast = false;
    for (int64_t id : w.nodes) {
        Node *n = p->find(id);
        if (!n) continue;
        auto e = std::lower_bound(n->act.begin(), n->act.end(), workflow,
                                  [](const Entry &x, int64_t wid) { return x.wf < wid; });
        if (e == n->act.end() || e->wf != workflow) continue;
        n->act.erase(e);
        p->rescore(n);
        p->refresh(n);
    }
    std::vector<int64_t>().swap(w.nodes);
    return PBKV_OK;
}

double pbkv_policy_score(const pbkv_policy *p, int64_t node) {
    const Node *n = p ? p->find(node) : nullptr;
    return n ? n->score : std::numeric_limits<double>::quiet_NaN();
}
double pbkv_policy_value(const pbkv_policy *p, int64_t node) {
    const Node *n = p ? p->find(node) : nullptr;
    return n ? n->value : std::numeric_limits<double>::quiet_NaN();
}
int32_t pbkv_policy_is_retired(const pbkv_policy *p, int64_t node) {
    const Node *n = p ? p->find(node) : nullptr;
    return n ? (int32_t)n->act.empty() : -1;
}
int32_t pbkv_policy_node_tier(const pbkv_policy *p, int64_t node) {
    const Node *n = p ? p->find(node) : nullptr;
    return n ? n->tier : -1;
}
int64_t pbkv_policy_retired_pages(const pbkv_policy *p) { return p ? p->retired_total : 0; }

int64_t pbkv_policy_evict(pbkv_policy *p, int64_t pages_needed, int32_t to_host, int64_t *out_nodes,
                          int64_t capacity, int64_t *pages_freed) {
    pbkv::clear_error();
    if (!p || !pages_freed || (capacity > 0 && !out_nodes)) return set_error(PBKV_ERR_NULL, "pbkv_policy_evict: NULL argument");
    int64_t n_out = 0, freed = 0;
    while (freed < pages_needed && !p->evictable.empty() && n_out < capacity) {
        Node *n = p->evictable.top();
        out_nodes[n_out++] = n->id;
        freed += n->pages;
        p->leave_gpu(n, to_host != 0);
    }
    *pages_freed = freed;
    return n_out;
}

int pbkv_policy_observe_step(pbkv_policy *p, double seconds) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    if (!(seconds > 0.0)) return set_error(PBKV_ERR_RANGE, "step duration %g", seconds);
    p->step_sum += seconds;
    p->step_n++;
    return PBKV_OK;
}

int pbkv_policy_observe_transfer(pbkv_policy *p, double bytes, double seconds) {
    pbkv::clear_error();
    if (!p) return set_error(PBKV_ERR_NULL, "policy is NULL");
    if (!(seconds > 0.0) || !(bytes >= 0.0)) return set_error(PBKV_ERR_RANGE, "transfer of %g bytes in %g s", bytes, seconds);
    p->rate_sum += bytes / seconds;
    p->rate_n++;
    return PBKV_OK;
}

int64_t pbkv_policy_bandwidth_budget_pages(const pbkv_policy *p, int64_t page_bytes) {
    if (!p || page_bytes <= 0 || p->step_n == 0 || p->rate_n == 0) return 0;
    const double bw = p->rate_sum / (double)p->rate_n, step = p->step_sum / (double)p->step_n;
    return (int64_t)std::floor(bw * step / (double)page_bytes);
}

int64_t pbkv_policy_prefetch(pbkv_policy *p, int64_t free_pages, int64_t bw_budget_pages, int32_t pure_decode,
                             int32_t to_host, int64_t *out_loads, int64_t load_capacity, int64_t *out_reclaimed,
                             int64_t reclaim_capacity, int64_t *n_reclaimed) {
    pbkv::clear_error();
    if (!p || !n_reclaimed || (load_capacity > 0 && !out_loads) || (reclaim_capacity > 0 && !out_reclaimed))
        return set_error(PBKV_ERR_NULL, "pbkv_policy_prefetch: NULL argument");
    *n_reclaimed = 0;
    if (!pure_decode || free_pages < 0) return 0;
    const int64_t budget = std::min(free_pages + p->retired_total, bw_budget_pages);
    int64_t n_loads = 0, used = 0;
    while (!p->loadable.empty() && n_loads < load_capacity) {
        Node *n = p->loadable.top();
        if (used + n->pages > budget) break;
        used += n->pages;
        n->pins++;                                   // being loaded: not reclaimable in this decision
        p->set_tier(n, PBKV_TIER_GPU);
        out_loads[n_loads++] = n->id;
    }
    int64_t freed = 0, n_rec = 0;
    while (used - freed > free_pages) {
        if (p->evictable.empty() || !p->retired(p->evictable.top()) || n_rec >= reclaim_capacity) break;
        Node *n = p->evictable.top();
        out_reclaimed[n_rec++] = n->id;
        freed += n->pages;
        p->leave_gpu(n, to_host != 0);
    }
    // Retired space that could not be reclaimed after all (the caller's list is full, or what is left
    // of it is held by a pinned or GPU-resident child): the decision is cut back instead of being
    // left half applied -- loads are withdrawn from the end (children before their parents) until
    // the rest fits, so the books always describe what the caller is told to do.
    while (used - freed > free_pages && n_loads > 0) {
        Node *n = p->find(out_loads[--n_loads]);
        n->pins--;
        used -= n->pages;
        p->set_tier(n, PBKV_TIER_HOST);
    }
    for (int64_t i = 0; i < n_loads; i++) {
        Node *n = p->find(out_loads[i]);
        n->pins--;
        p->refresh(n);
    }
    *n_reclaimed = n_rec;
    return n_loads;
}

}  // extern "C"
