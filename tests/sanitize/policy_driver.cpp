// Host-only driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the policy core
// (csrc/policy.cpp): seeded random traces of node insertions and removals, accesses along radix
// paths, forecasts, terminations, pins, evictions (to the host tier and dropped) and prefetch
// decisions with short output lists, in all three modes.  What is checked here is only what needs
// no model: list lengths within capacity, page totals, scores finite and non-negative, retired
// nodes score zero.  (Decision-by-decision equality with the reference model is the Python test.)
#include "../../include/pbkv.h"
#include "../../include/pbkv_policy.h"

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

// the two error hooks the core expects from the library's HIP translation unit
namespace pbkv {
int set_error(int code, const char *, ...) { return code; }
void clear_error() {}
}

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint64_t rnd() { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }
static int rint_(int lo, int hi) { return lo + (int)(rnd() % (uint64_t)(hi - lo)); }
static double runit() { return (double)(rnd() >> 11) / 9007199254740992.0; }

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); exit(1); } } while (0)

static long g_evicted = 0, g_loaded = 0, g_reclaimed = 0;

static void trace(int mode, int steps) {
    const int V = 5, K = 3;
    pbkv_policy *p = pbkv_policy_create(V, K, 0.7, mode);
    CHECK(p);
    CHECK(pbkv_policy_set_inherit(p, 0, 1) == 0);
    std::map<int64_t, int64_t> parent;             // live nodes
    std::vector<int64_t> wfs;
    int64_t next_node = 0, next_wf = 0;
    CHECK(pbkv_policy_node_add(p, next_node, -1, 2, PBKV_TIER_GPU) == 0);
    parent[next_node++] = -1;
    for (int s = 0; s < steps; s++) {
        const double r = runit();
        if (r < 0.25 || parent.empty()) {
            auto it = parent.begin();
            std::advance(it, parent.empty() ? 0 : rint_(0, (int)parent.size()));
            const int64_t par = parent.empty() ? -1 : it->first;
            const int tier = pbkv_policy_node_tier(p, par) == PBKV_TIER_HOST ? PBKV_TIER_HOST : rint_(0, 2) ? PBKV_TIER_GPU : PBKV_TIER_HOST;
            if (pbkv_policy_node_add(p, next_node, par, rint_(1, 5), tier) == 0) parent[next_node] = par;
            next_node++;
        } else if (r < 0.5 && !parent.empty()) {
            auto it = parent.begin();
            std::advance(it, rint_(0, (int)parent.size()));
            std::vector<int64_t> path;
            for (int64_t n = it->first; n >= 0; n = parent.count(n) ? parent[n] : -1) path.insert(path.begin(), n);
            int64_t wf;
            if (wfs.empty() || runit() < 0.3) { wf = next_wf++; wfs.push_back(wf); } else wf = wfs[rint_(0, (int)wfs.size())];
            pbkv_policy_access(p, wf, rint_(0, V), path.data(), (int32_t)path.size());
        } else if (r < 0.65 && !wfs.empty()) {
            double probs[K][V + 1];
            for (int k = 0; k < K; k++) {
                double sum = 0;
                for (int a = 0; a <= V; a++) sum += probs[k][a] = runit() * runit();
                for (int a = 0; a <= V; a++) probs[k][a] /= sum;
            }
            CHECK(pbkv_policy_forecast(p, wfs[rint_(0, (int)wfs.size())], &probs[0][0]) == 0);
        } else if (r < 0.72 && !wfs.empty()) {
            const int i = rint_(0, (int)wfs.size());
            CHECK(pbkv_policy_terminate(p, wfs[i]) == 0);
            wfs.erase(wfs.begin() + i);
        } else if (r < 0.8 && !parent.empty()) {
            auto it = parent.begin();
            std::advance(it, rint_(0, (int)parent.size()));
            if (pbkv_policy_node_pin(p, it->first, +1) == 0 && runit() < 0.8) pbkv_policy_node_pin(p, it->first, -1);
        } else if (r < 0.9) {
            int64_t out[4], freed = 0;
            const int to_host = rint_(0, 2);
            const int64_t n = pbkv_policy_evict(p, rint_(1, 12), to_host, out, rint_(0, 5), &freed);
            CHECK(n >= 0 && n <= 4 && freed >= 0);
            g_evicted += n;
            if (!to_host)                                  // dropped nodes (and their host descendants) are gone
                for (auto it = parent.begin(); it != parent.end();)
                    it = pbkv_policy_node_tier(p, it->first) < 0 ? parent.erase(it) : std::next(it);
        } else {
            int64_t loads[3], rec[2], n_rec = -1;
            const int to_host = rint_(0, 2);
            const int64_t n = pbkv_policy_prefetch(p, rint_(0, 6), rint_(0, 12), runit() < 0.9, to_host, loads, rint_(0, 4), rec, rint_(0, 3), &n_rec);
            CHECK(n >= 0 && n <= 3 && n_rec >= 0 && n_rec <= 2);
            g_loaded += n;
            g_reclaimed += n_rec;
            for (int64_t i = 0; i < n; i++) CHECK(pbkv_policy_node_tier(p, loads[i]) == PBKV_TIER_GPU);
            if (!to_host)
                for (auto it = parent.begin(); it != parent.end();)
                    it = pbkv_policy_node_tier(p, it->first) < 0 ? parent.erase(it) : std::next(it);
        }
        CHECK(pbkv_policy_retired_pages(p) >= 0);
        for (auto &kv : parent) {
            const double sc = pbkv_policy_score(p, kv.first), va = pbkv_policy_value(p, kv.first);
            CHECK(std::isfinite(sc) && sc >= 0.0 && std::isfinite(va) && va >= 0.0);
            if (pbkv_policy_is_retired(p, kv.first) == 1) CHECK(sc == 0.0 && va == 0.0);
        }
    }
    pbkv_policy_observe_step(p, 0.012);
    pbkv_policy_observe_transfer(p, 64e6, 0.001);
    CHECK(pbkv_policy_bandwidth_budget_pages(p, 65536) > 0);
    pbkv_policy_destroy(p);
}

int main() {
    for (int mode = 0; mode < 3; mode++) trace(mode, 3000);
    CHECK(g_evicted > 100 && g_loaded > 20 && g_reclaimed > 0);   // the traces reach every decision
    printf("policy driver: clean (%ld evicted, %ld loaded, %ld reclaimed)\n", g_evicted, g_loaded, g_reclaimed);
    return 0;
}
