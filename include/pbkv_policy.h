/*
 * pbkv_policy.h -- C boundary of the cache-management policy core (host code, no GPU work).
 *
 * The policy layer of PBKV decides WHICH radix-tree nodes leave the GPU pool and WHICH host
 * nodes are loaded ahead of a hit; its outputs (lists of node ids, hence of page ids) are
 * the inputs of pbkv_swap_out_pages / pbkv_swap_in_pages in pbkv.h.  It keeps, per node,
 * the workflows that accessed it and which of their agents did (Sec. 4.2.1, 4.2.2), turns
 * every workflow's K-step forecast into the node scores of Eq. 1 and Eq. 2, holds the
 * candidates in indexed heaps (Sec. 5, Complexity: O(1) peek, O(log n) pop / insert /
 * re-key) and answers eviction (Sec. 4.2.3) and prefetch (Sec. 4.3) requests.
 *
 * All functions are synchronous host functions; none touches the GPU.  A policy object is
 * not thread-safe: one scheduler thread drives it (App. F).  Node and workflow ids are
 * chosen by the caller (any int64, unique among live nodes / workflows).  Every function
 * that returns int returns PBKV_OK (0) or a negative pbkv_status from pbkv.h; the message
 * is available from pbkv_last_error().
 *
 * Readings where the paper is silent:
 *   - a node no workflow has accessed counts as retired;
 *   - only nodes without a GPU-resident child and without pins can leave the GPU (the radix
 *     tree keeps whole prefixes), and only host nodes whose parent is GPU-resident (or that
 *     have no parent) can be loaded;
 *   - ties are broken by last access (older first), then by node id (smaller first); retired
 *     nodes are ranked by the number of workflows that ever accessed them (fewer first);
 *   - prefetch skips nodes of Value 0, takes candidates in descending Value (then smaller
 *     depth, smaller id) and stops at the first one that does not fit the remaining budget.
 */
#ifndef PBKV_POLICY_H
#define PBKV_POLICY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pbkv_policy pbkv_policy;

enum { PBKV_TIER_GPU = 0, PBKV_TIER_HOST = 1 };

/* Eviction order among non-retired nodes; retired nodes are irrelevant to PBKV_MODE_LRU. */
enum {
    PBKV_MODE_LRU = 0,   /* least recently used only (the default policy the paper compares with) */
    PBKV_MODE_LAE = 1,   /* lifecycle-aware: retired cache first, then LRU        (Sec. 4.2.1)    */
    PBKV_MODE_HE = 2     /* hierarchical: retired cache first, then ascending Score (Sec. 4.2.3) */
};

/* num_agents = |V| in [1, 64]; horizon = K in [1, 8]; gamma in (0, 1] (Eq. 2).  NULL on bad
 * arguments (see pbkv_last_error). */
pbkv_policy *pbkv_policy_create(int32_t num_agents, int32_t horizon, double gamma, int32_t mode);
void pbkv_policy_destroy(pbkv_policy *p);

/* Customisation of the access indicator (Sec. 5, Limitations): agent dst inherits the cache
 * agent src accesses, i.e. A_w(c)[dst] is set whenever A_w(c)[src] is.  Affects later accesses. */
int pbkv_policy_set_inherit(pbkv_policy *p, int32_t src_agent, int32_t dst_agent);

/* A radix-tree node of `pages` pool pages (> 0) under `parent` (-1: none) in the given tier. */
int pbkv_policy_node_add(pbkv_policy *p, int64_t node, int64_t parent, int32_t pages, int32_t tier);
/* Forget a node that has no children. */
int pbkv_policy_node_remove(pbkv_policy *p, int64_t node);
/* The caller moved the node's pages (after a swap-in on a hit, say). */
int pbkv_policy_node_set_tier(pbkv_policy *p, int64_t node, int32_t tier);
/* delta = +1 while a running request uses the node, -1 when it is done. */
int pbkv_policy_node_pin(pbkv_policy *p, int64_t node, int32_t delta);

/* Agent `agent` of workflow `workflow` accessed these nodes (normally a whole radix path).
 * Creates the workflow on first use; fails for a terminated workflow. */
int pbkv_policy_access(pbkv_policy *p, int64_t workflow, int32_t agent, const int64_t *nodes,
                       int32_t n_nodes);
/* New forecast of a workflow: probs[k][a], k < K, a < |V| + 1 with END last; every row in
 * [0, 1] and summing to 1 (within 1e-6).  Refreshes the scores of the workflow's nodes. */
int pbkv_policy_forecast(pbkv_policy *p, int64_t workflow, const double *probs);
/* Termination message of a workflow (Sec. 4.2.1): its tags leave every node; nodes whose
 * workflows have all terminated become retired. */
int pbkv_policy_terminate(pbkv_policy *p, int64_t workflow);

/* Eq. 2, Eq. 1, and the retired tag of a node (NaN / -1 for an unknown node). */
double pbkv_policy_score(const pbkv_policy *p, int64_t node);
double pbkv_policy_value(const pbkv_policy *p, int64_t node);
int32_t pbkv_policy_is_retired(const pbkv_policy *p, int64_t node);
int32_t pbkv_policy_node_tier(const pbkv_policy *p, int64_t node);   /* -1: unknown node */
/* Pages of retired, unpinned GPU nodes: the part of S_a beyond the free space (Sec. 4.3). */
int64_t pbkv_policy_retired_pages(const pbkv_policy *p);

/* Eviction (Sec. 4.2.2 "Implementation", Sec. 4.2.3): pops candidates until `pages_needed`
 * pages are freed or none is left.  Evicted nodes move to the host tier if to_host is set,
 * else they (and their host-resident descendants) are forgotten.  Writes at most `capacity`
 * node ids to out_nodes in eviction order and the pages they free to *pages_freed; returns
 * the number of evicted nodes (it stops early when out_nodes is full), or a negative status. */
int64_t pbkv_policy_evict(pbkv_policy *p, int64_t pages_needed, int32_t to_host, int64_t *out_nodes,
                          int64_t capacity, int64_t *pages_freed);

/* Running means for S_bw = Bandwidth * StepDuration (Sec. 4.3). */
int pbkv_policy_observe_step(pbkv_policy *p, double seconds);
int pbkv_policy_observe_transfer(pbkv_policy *p, double bytes, double seconds);
int64_t pbkv_policy_bandwidth_budget_pages(const pbkv_policy *p, int64_t page_bytes);

/* Prefetch decision (Sec. 4.3): budget S = min(free_pages + retired pages, bw_budget_pages);
 * nothing unless the batch is pure decode.  Host nodes are taken in descending Value and
 * become GPU-tier; if they need more than free_pages, retired nodes are reclaimed (as in
 * eviction, honouring to_host) and listed in out_reclaimed.  If the retired space cannot be
 * reclaimed after all (out_reclaimed is full, or a retired node is held by a pinned or
 * GPU-resident child), loads are withdrawn from the end of the list until the rest fits: the
 * books always match the lists returned.  Returns the number of nodes to load (written to
 * out_loads, at most load_capacity), *n_reclaimed the number reclaimed. */
int64_t pbkv_policy_prefetch(pbkv_policy *p, int64_t free_pages, int64_t bw_budget_pages,
                             int32_t pure_decode, int32_t to_host, int64_t *out_loads,
                             int64_t load_capacity, int64_t *out_reclaimed,
                             int64_t reclaim_capacity, int64_t *n_reclaimed);

#ifdef __cplusplus
}
#endif
#endif /* PBKV_POLICY_H */
