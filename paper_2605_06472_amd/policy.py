"""ctypes binding of the policy core in libpbkv.so (include/pbkv_policy.h): same operations,
argument marshalling only -- every decision is taken by the C++ code."""
import ctypes

import numpy as np

from . import binding

GPU, HOST = 0, 1
MODE_LRU, MODE_LAE, MODE_HE = 0, 1, 2

_ready = False


def _lib():
    global _ready
    lib = binding.load()
    if not _ready:
        vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double
        i64p = ctypes.POINTER(ctypes.c_int64)
        sig = {
            "pbkv_policy_create": (vp, [i32, i32, dbl, i32]),
            "pbkv_policy_destroy": (None, [vp]),
            "pbkv_policy_set_inherit": (ctypes.c_int, [vp, i32, i32]),
            "pbkv_policy_node_add": (ctypes.c_int, [vp, i64, i64, i32, i32]),
            "pbkv_policy_node_remove": (ctypes.c_int, [vp, i64]),
            "pbkv_policy_node_set_tier": (ctypes.c_int, [vp, i64, i32]),
            "pbkv_policy_node_pin": (ctypes.c_int, [vp, i64, i32]),
            "pbkv_policy_access": (ctypes.c_int, [vp, i64, i32, vp, i32]),
            "pbkv_policy_forecast": (ctypes.c_int, [vp, i64, vp]),
            "pbkv_policy_terminate": (ctypes.c_int, [vp, i64]),
            "pbkv_policy_score": (dbl, [vp, i64]),
            "pbkv_policy_value": (dbl, [vp, i64]),
            "pbkv_policy_is_retired": (i32, [vp, i64]),
            "pbkv_policy_node_tier": (i32, [vp, i64]),
            "pbkv_policy_retired_pages": (i64, [vp]),
            "pbkv_policy_evict": (i64, [vp, i64, i32, vp, i64, i64p]),
            "pbkv_policy_observe_step": (ctypes.c_int, [vp, dbl]),
            "pbkv_policy_observe_transfer": (ctypes.c_int, [vp, dbl, dbl]),
            "pbkv_policy_bandwidth_budget_pages": (i64, [vp, i64]),
            "pbkv_policy_prefetch": (i64, [vp, i64, i64, i32, i32, vp, i64, vp, i64, i64p]),
        }
        for name, (res, args) in sig.items():
            f = getattr(lib, name)
            f.restype, f.argtypes = res, args
        _ready = True
    return lib


def _check(rc):
    if rc < 0:
        raise binding.PbkvError(int(rc), _lib().pbkv_last_error().decode())
    return rc


class Policy:
    def __init__(self, num_agents, horizon, gamma, mode=MODE_HE, list_capacity=1 << 16):
        self._l = _lib()
        self._p = self._l.pbkv_policy_create(num_agents, horizon, gamma, mode)
        if not self._p:
            raise binding.PbkvError(-2, self._l.pbkv_last_error().decode())
        self.V, self.K = num_agents, horizon
        self._a = np.zeros(list_capacity, np.int64)
        self._b = np.zeros(list_capacity, np.int64)

    def close(self):
        if self._p:
            self._l.pbkv_policy_destroy(self._p)
            self._p = None

    __del__ = close

    def set_inherit(self, src, dst):
        _check(self._l.pbkv_policy_set_inherit(self._p, src, dst))

    def node_add(self, nid, parent, pages, tier=GPU):
        _check(self._l.pbkv_policy_node_add(self._p, nid, parent, pages, tier))

    def node_remove(self, nid):
        _check(self._l.pbkv_policy_node_remove(self._p, nid))

    def node_set_tier(self, nid, tier):
        _check(self._l.pbkv_policy_node_set_tier(self._p, nid, tier))

    def node_pin(self, nid, delta):
        _check(self._l.pbkv_policy_node_pin(self._p, nid, delta))

    def access(self, workflow, agent, node_ids):
        ids = np.ascontiguousarray(node_ids, np.int64)
        _check(self._l.pbkv_policy_access(self._p, workflow, agent, ids.ctypes.data, int(ids.shape[0])))

    def forecast(self, workflow, probs):
        pr = np.ascontiguousarray(probs, np.float64)
        if pr.shape != (self.K, self.V + 1):
            raise ValueError("forecast must be [K][|V|+1]")
        _check(self._l.pbkv_policy_forecast(self._p, workflow, pr.ctypes.data))

    def terminate(self, workflow):
        _check(self._l.pbkv_policy_terminate(self._p, workflow))

    def score(self, nid):
        return self._l.pbkv_policy_score(self._p, nid)

    def value(self, nid):
        return self._l.pbkv_policy_value(self._p, nid)

    def is_retired(self, nid):
        return bool(self._l.pbkv_policy_is_retired(self._p, nid))

    def node_tier(self, nid):
        return int(self._l.pbkv_policy_node_tier(self._p, nid))

    def retired_pages(self):
        return int(self._l.pbkv_policy_retired_pages(self._p))

    def evict(self, pages_needed, to_host=True):
        freed = ctypes.c_int64(0)
        n = _check(self._l.pbkv_policy_evict(self._p, pages_needed, int(to_host), self._a.ctypes.data,
                                             int(self._a.shape[0]), ctypes.byref(freed)))
        return self._a[:n].tolist(), int(freed.value)

    def observe_step(self, seconds):
        _check(self._l.pbkv_policy_observe_step(self._p, seconds))

    def observe_transfer(self, nbytes, seconds):
        _check(self._l.pbkv_policy_observe_transfer(self._p, nbytes, seconds))

    def bandwidth_budget_pages(self, page_bytes):
        return int(self._l.pbkv_policy_bandwidth_budget_pages(self._p, page_bytes))

    def prefetch(self, free_pages, bw_budget_pages, pure_decode=True, to_host=True):
        nrec = ctypes.c_int64(0)
        n = _check(self._l.pbkv_policy_prefetch(self._p, free_pages, bw_budget_pages, int(pure_decode),
                                                int(to_host), self._a.ctypes.data, int(self._a.shape[0]),
                                                self._b.ctypes.data, int(self._b.shape[0]), ctypes.byref(nrec)))
        return self._a[:n].tolist(), self._b[:int(nrec.value)].tolist()
