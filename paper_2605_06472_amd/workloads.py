"""Seeded synthetic agent-workflow batches for prefix-reuse prefill.

This module only *draws inputs*: lengths, radix-tree sharing, page placement
and N(0, sigma) values, rounded once to the storage dtype.  It holds none of
the attention / append / swap-in arithmetic, so the GPU tests and the CPU
oracle can both be fed from it without sharing any of the method's code.

The batches stand in for the paper's workloads (Sec. 6.1: HoVer + LangChain,
SWE-bench + AutoGen, FinanceBench + CrewAI), which are not available here.
They keep the structure the paper describes in Sec. 2: a *global cache* shared
by every request (system prompt, tool / agent descriptions), a *private cache*
accumulated along one workflow, page-granular radix-tree nodes, contexts of
tens of thousands of tokens, partial GPU hit rates and a host tier whose pages
are swapped back on a hit (HiCache) or prefetched (Sec. 4.3).

Storage layouts (row-major):
    q, out        [N, Hq, d]      N = sum(new_lens), requests packed in order
    k_new, v_new  [N, Hkv, d]
    kv_pool       [num_pages, 2, Hkv, P, d]     index 0 = K, 1 = V
    block_table   [B, max_pages] int32          logical page -> physical page
bf16 tensors are numpy ``uint16`` arrays of bit patterns.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional

import numpy as np

PAGE = 16


# ----------------------------------------------------------------------------
# dtype helpers (storage conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (bf16 bits or float32) to float64."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------
# random values: counter-based streams, one per (seed, tag, chunk), so the
# result does not depend on how many threads fill the array
# ----------------------------------------------------------------------------
_CHUNK = 1 << 22


def _normal_chunk(seed: int, tag: int, idx: int, n: int, sigma: float, dtype: str) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, tag, idx])))
    x = rng.standard_normal(n, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def normal_tensor(seed: int, tag: int, shape, sigma: float, dtype: str) -> np.ndarray:
    """N(0, sigma^2) drawn in float32 and rounded once to ``dtype`` ('bf16' | 'f32')."""
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16 if dtype == "bf16" else np.float32)
    spans = [(i, s, min(_CHUNK, n - s)) for i, s in enumerate(range(0, n, _CHUNK))]

    def fill(sp):
        i, s, m = sp
        out[s:s + m] = _normal_chunk(seed, tag, i, m, sigma, dtype)

    if len(spans) <= 2:
        for sp in spans:
            fill(sp)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, spans))
    return out.reshape(shape)


# ----------------------------------------------------------------------------
# batch container
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Batch:
    name: str
    dtype: str                      # 'bf16' | 'f32'
    Hq: int
    Hkv: int
    d: int
    P: int
    num_pages: int
    q: np.ndarray
    k_new: np.ndarray
    v_new: np.ndarray
    kv_pool: np.ndarray             # pool with every *resident* prefix page in place
    block_table: np.ndarray
    prefix_lens: np.ndarray
    new_lens: np.ndarray
    # contiguous per-request K/V (prefix + suffix) kept before paging, for brute force
    logical_k: Optional[List[np.ndarray]] = None
    logical_v: Optional[List[np.ndarray]] = None
    # host tier (mixed hit/miss batches): pages to swap in and their destination slots
    host_pages: Optional[np.ndarray] = None      # [n_swap, 2, Hkv, P, d]
    swap_page_ids: Optional[np.ndarray] = None   # [n_swap] int32
    swap_offsets: Optional[np.ndarray] = None    # [B+1]: request r owns host pages [o[r], o[r+1])

    @property
    def B(self) -> int:
        return int(self.prefix_lens.shape[0])

    @property
    def N(self) -> int:
        return int(self.new_lens.sum())

    @property
    def max_pages(self) -> int:
        return int(self.block_table.shape[1])

    @property
    def elt(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def page_bytes(self) -> int:
        return 2 * self.Hkv * self.P * self.d * self.elt

    def attention_flops(self) -> int:
        """4*d*Hq*sum_r(n*p + n(n+1)/2): QK^T and PV over the visible keys only."""
        p = self.prefix_lens.astype(np.int64)
        n = self.new_lens.astype(np.int64)
        return int(4 * self.d * self.Hq * np.sum(n * p + n * (n + 1) // 2))

    def distinct_prefix_pages(self) -> int:
        used = set()
        for r in range(self.B):
            used.update(self.block_table[r, : -(-int(self.prefix_lens[r]) // self.P)].tolist())
        return len(used)

    def attention_bytes(self) -> int:
        """Bytes that must move once: distinct prefix pages, suffix K/V, Q in, out."""
        tok = self.Hkv * self.d * self.elt * 2
        return (self.distinct_prefix_pages() * self.page_bytes + self.N * tok
                + 2 * self.N * self.Hq * self.d * self.elt)

    def append_bytes(self) -> int:
        """Suffix K/V read once and written once."""
        return 2 * self.N * 2 * self.Hkv * self.d * self.elt


@dataclasses.dataclass
class _Segment:
    """A radix-tree node: a token run stored in whole pages (the last may be partial)."""
    tokens: int
    pages: np.ndarray


def _assemble(name, dtype, Hq, Hkv, d, num_pages, seed, sigma, requests, new_lens,
              q_scale=1.0, keep_logical=False, nonresident=None, page_perm=None) -> Batch:
    """Place segments on pages and draw the values.

    ``requests``: per request, the list of _Segment making up its cached prefix
    (shared segments are the same object).  Every segment but the last of a
    request holds a whole number of pages.  ``nonresident``: per request, how
    many trailing prefix pages live in the host tier instead of the pool.
    """
    P = PAGE
    B = len(requests)
    new_lens = np.asarray(new_lens, np.int32)
    prefix_lens = np.array([sum(s.tokens for s in segs) for segs in requests], np.int32)
    N = int(new_lens.sum())
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 7])))
    perm = rng.permutation(num_pages).astype(np.int32) if page_perm is None else np.asarray(page_perm, np.int32)
    cursor = 0

    def take(n):
        nonlocal cursor
        if cursor + n > num_pages:
            raise ValueError("pool too small for this batch")
        ids = perm[cursor:cursor + n]
        cursor += n
        return ids

    # physical pages of every distinct segment, in first-use order
    seen = {}
    for segs in requests:
        for i, s in enumerate(segs):
            if i + 1 < len(segs):
                assert s.tokens % P == 0, "only a request's last prefix segment may end mid-page"
            if id(s) not in seen:
                s.pages = take(-(-s.tokens // P))
                seen[id(s)] = s
    max_pages = 0
    rows = []
    for r, segs in enumerate(requests):
        ids = [s.pages for s in segs]
        pre = np.concatenate(ids) if ids else np.zeros(0, np.int32)
        total = -(-(int(prefix_lens[r]) + int(new_lens[r])) // P)
        extra = take(total - pre.shape[0])           # pages the suffix will be appended to
        rows.append(np.concatenate([pre, extra]))
        max_pages = max(max_pages, total)
    max_pages = max(max_pages, 1)
    block_table = np.zeros((B, max_pages), np.int32)
    for r, row in enumerate(rows):
        block_table[r, : row.shape[0]] = row

    # pool: every slot random, so a wrong page or slot cannot go unnoticed
    kv_pool = normal_tensor(seed, 1, (num_pages, 2, Hkv, P, d), sigma, dtype)
    q = normal_tensor(seed, 2, (N, Hq, d), sigma * q_scale, dtype)
    k_new = normal_tensor(seed, 3, (N, Hkv, d), sigma, dtype)
    v_new = normal_tensor(seed, 4, (N, Hkv, d), sigma, dtype)

    logical_k = logical_v = None
    if keep_logical:
        # the pre-paging view: per request, K/V of prefix + suffix as contiguous [L, Hkv, d].
        # A page's content *is* its random fill, so read each segment's pages back once.
        logical_k, logical_v = [], []
        off = 0
        for r, segs in enumerate(requests):
            ks, vs = [], []
            for s in segs:
                pg = kv_pool[s.pages]                              # [np, 2, Hkv, P, d]
                kk = pg[:, 0].transpose(0, 2, 1, 3).reshape(-1, Hkv, d)[: s.tokens]
                vv = pg[:, 1].transpose(0, 2, 1, 3).reshape(-1, Hkv, d)[: s.tokens]
                ks.append(kk)
                vs.append(vv)
            n = int(new_lens[r])
            ks.append(k_new[off:off + n])
            vs.append(v_new[off:off + n])
            off += n
            logical_k.append(np.concatenate(ks, axis=0))
            logical_v.append(np.concatenate(vs, axis=0))

    host_pages = swap_ids = swap_off = None
    if nonresident is not None:
        # trailing prefix pages of each request live in the host tier: move their
        # content out of the pool and overwrite the pool slot with other values
        ids, swap_off = [], [0]
        for r in range(B):
            npre = -(-int(prefix_lens[r]) // P)
            k = int(nonresident[r])
            assert 0 <= k <= npre
            ids.append(block_table[r, npre - k:npre])
            swap_off.append(swap_off[-1] + k)
        swap_ids = np.concatenate(ids).astype(np.int32) if ids else np.zeros(0, np.int32)
        swap_off = np.asarray(swap_off, np.int64)
        host_pages = kv_pool[swap_ids].copy()
        stale = normal_tensor(seed, 5, (swap_ids.shape[0], 2, Hkv, P, d), sigma, dtype)
        kv_pool[swap_ids] = stale

    return Batch(name=name, dtype=dtype, Hq=Hq, Hkv=Hkv, d=d, P=P, num_pages=num_pages,
                 q=q, k_new=k_new, v_new=v_new, kv_pool=kv_pool, block_table=block_table,
                 prefix_lens=prefix_lens, new_lens=new_lens, logical_k=logical_k,
                 logical_v=logical_v, host_pages=host_pages, swap_page_ids=swap_ids,
                 swap_offsets=swap_off)


def _seg(tokens: int) -> _Segment:
    return _Segment(tokens=int(tokens), pages=np.zeros(0, np.int32))


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------
def tiny_fp32(seed: int = 1000, keep_logical: bool = True, q_scale: float = 1.0) -> Batch:
    """One request, fp32, 2 query / 1 KV heads, d=64, 256 cached + 64 new tokens, 64-page pool."""
    return _assemble("cfg0_tiny_fp32", "f32", 2, 1, 64, 64, seed, 1.0, [[_seg(256)]], [64],
                     q_scale=q_scale, keep_logical=keep_logical)


def shared_system_prompt(seed: int = 1001, q_scale: float = 1.0, keep_logical: bool = False,
                         batch: int = 4, prefix: int = 2048, new: int = 512,
                         num_pages: int = 1024) -> Batch:
    """Agents of different workflows sharing one system prompt (global cache, Sec. 2):
    every block-table row names the same prefix pages; each request has its own suffix."""
    root = _seg(prefix)
    return _assemble("cfg1_shared_system_prompt", "bf16", 32, 8, 128, num_pages, seed,
                     2 ** -0.5, [[root] for _ in range(batch)], [new] * batch,
                     q_scale=q_scale, keep_logical=keep_logical)


def dynamic_workflow_batch(seed: int = 1002, q_scale: float = 1.0, keep_logical: bool = False) -> Batch:
    """16 requests over a radix tree: a 1024-token root (system prompt + tool descriptions)
    shared by all, three branch histories (512..4096 tokens) each shared by a subset, and a
    private cached tail per request; 128..1024 new tokens."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 11])))
    B = 16
    root = _seg(1024)
    branches = [_seg(int(rng.integers(512 // PAGE, 4096 // PAGE + 1)) * PAGE) for _ in range(3)]
    attach = np.concatenate([np.arange(3), rng.integers(0, 3, B - 3)])
    rng.shuffle(attach)
    reqs, new = [], []
    for r in range(B):
        tail = int(rng.integers(0, 2048 // PAGE + 1)) * PAGE
        segs = [root, branches[int(attach[r])]]
        if tail:
            segs.append(_seg(tail))
        reqs.append(segs)
        new.append(int(rng.integers(128, 1025)))
    return _assemble("cfg2_dynamic_workflow", "bf16", 32, 8, 128, 4096, seed, 2 ** -0.5,
                     reqs, new, q_scale=q_scale, keep_logical=keep_logical)


def long_history(seed: int = 1003, q_scale: float = 1.0, batch: int = 4, prefix: int = 32768,
                 new: int = 2048, num_pages: int = 16384) -> Batch:
    """Long accumulated private history: fully scattered 32768-token prefixes, 2048 new tokens."""
    return _assemble("cfg3_long_history", "bf16", 32, 8, 128, num_pages, seed, 2 ** -0.5,
                     [[_seg(prefix)] for _ in range(batch)], [new] * batch, q_scale=q_scale)


def mixed_hit_miss(seed: int = 1004, q_scale: float = 1.0, batch: int = 32,
                   max_prefix: int = 16384, min_new: int = 64, max_new: int = 2048,
                   num_pages: int = 40960) -> Batch:
    """Mixed GPU hit / host hit: per request a seeded fraction of the prefix pages is
    resident; the trailing pages (radix leaves are evicted before their ancestors) sit in
    the host tier and must be swapped in to the slots the block table names."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 13])))
    reqs, new, nonres = [], [], []
    for _ in range(batch):
        p = int(rng.integers(0, max_prefix + 1))
        n = int(rng.integers(min_new, max_new + 1))
        f = float(rng.random())
        pages = -(-p // PAGE)
        reqs.append([_seg(p)] if p else [])
        new.append(n)
        nonres.append(pages - int(np.floor(f * pages)))
    return _assemble("cfg4_mixed_hit_miss", "bf16", 32, 8, 128, num_pages, seed, 2 ** -0.5,
                     reqs, new, q_scale=q_scale, nonresident=nonres)


def ragged_small(seed: int, dtype: str = "bf16", Hq: int = 8, Hkv: int = 2, d: int = 128,
                 prefix_lens=(0, 5, 16, 37, 130), new_lens=(1, 3, 70, 0, 129), num_pages: int = 64,
                 shared_root: int = 0, q_scale: float = 1.0, sigma: float = 2 ** -0.5,
                 nonresident=None, page_perm=None) -> Batch:
    """Small edge-case batch: unaligned prefixes, empty requests, single rows, optional
    page-aligned root shared by every request.  Keeps the contiguous K/V for brute force."""
    root = _seg(shared_root) if shared_root else None
    reqs = []
    for p in prefix_lens:
        segs = []
        if root is not None:
            segs.append(root)
        if p:
            segs.append(_seg(p))
        reqs.append(segs)
    return _assemble("ragged_small", dtype, Hq, Hkv, d, num_pages, seed, sigma, reqs,
                     list(new_lens), q_scale=q_scale, keep_logical=True,
                     nonresident=nonresident, page_perm=page_perm)


def decode_batch(seed: int = 1005, batch: int = 64, min_ctx: int = 1024, max_ctx: int = 16384,
                 num_pages: int = 40960, q_scale: float = 1.0) -> Batch:
    """A pure-decode batch (the steps behind which prefetch transfers are hidden): every request
    contributes one query row over a private, fully scattered context of U{min_ctx..max_ctx}
    tokens (prefix_lens holds the context lengths; new_lens is all ones and only sizes q)."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 17])))
    ctx = [int(rng.integers(min_ctx, max_ctx + 1)) for _ in range(batch)]
    return _assemble("decode_batch", "bf16", 32, 8, 128, num_pages, seed, 2 ** -0.5,
                     [[_seg(c)] for c in ctx], [1] * batch, q_scale=q_scale)


# ----------------------------------------------------------------------------
# workflow predictor (App. B): random-init model of the stated widths and a batch of workflow states
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class PredictorModel:
    """Weights of the predictor, all float32, row-major, named as in App. B.  The paper gives the
    parameter count (~350 K) and the served model (Qwen3-32B, hidden width 5120) but not the
    widths; V=8, d=64, hidden=64, K=3 with a 5120-wide x give 362 779 parameters."""
    V: int
    d: int
    d_x: int
    hidden: int
    K: int
    emb: np.ndarray        # H^(0)  [V][d]
    trans: np.ndarray      # A      [V][V], rows sum to 1 (or are all zero: an agent never left)
    w1: np.ndarray         # W^(1)  [d][2d]
    w2: np.ndarray         # W^(2)  [d][2d]
    wq: np.ndarray         # W_q    [d][d]
    wt: np.ndarray         # W_t    [d][d_x]
    wa: np.ndarray         # first MLP layer  [hidden][3d]   (input order: h_cur, h_path, h_txt)
    ba: np.ndarray         # [hidden]
    wb: np.ndarray         # second MLP layer [K*(V+1)][hidden], output index = k*(V+1) + agent, END last
    bb: np.ndarray         # [K*(V+1)]

    def num_params(self) -> int:
        return sum(int(getattr(self, n).size) for n in ("emb", "w1", "w2", "wq", "wt", "wa", "ba", "wb", "bb"))


@dataclasses.dataclass
class PredictorBatch:
    B: int
    L: int                 # prefix slots per request
    x: np.ndarray          # [B][d_x] bf16 bit patterns: post-norm hidden state of the last prefill token
    cur_agent: np.ndarray  # [B] int32: v_t
    prefix: np.ndarray     # [B][L] int32: v_1 .. v_{t-1} in the first prefix_len slots (rest: -1)
    prefix_len: np.ndarray  # [B] int32: t - 1 in [0, L]


def predictor_model(seed: int = 2000, V: int = 8, d: int = 64, d_x: int = 5120, hidden: int = 64,
                    K: int = 3, gain: float = 1.0) -> PredictorModel:
    """Random-init weights (N(0, gain^2 / fan_in), embeddings N(0, 1)) and a looped call graph:
    every agent has 1-3 successors with random counts, as a transition matrix estimated from
    traces would look (Sec. 2, App. B)."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 31])))

    def w(rows, cols, fan_in):
        return (rng.standard_normal((rows, cols)) * gain / np.sqrt(fan_in)).astype(np.float32)

    counts = np.zeros((V, V))
    for v in range(V):
        succ = rng.choice(V, size=int(rng.integers(1, min(3, V) + 1)), replace=False)
        counts[v, succ] = rng.integers(1, 20, size=len(succ))
    trans = (counts / counts.sum(1, keepdims=True)).astype(np.float32)
    return PredictorModel(V, d, d_x, hidden, K,
                          emb=rng.standard_normal((V, d)).astype(np.float32), trans=trans,
                          w1=w(d, 2 * d, 2 * d), w2=w(d, 2 * d, 2 * d), wq=w(d, d, d), wt=w(d, d_x, d_x),
                          wa=w(hidden, 3 * d, 3 * d), ba=(rng.standard_normal(hidden) * 0.1).astype(np.float32),
                          wb=w(K * (V + 1), hidden, hidden),
                          bb=(rng.standard_normal(K * (V + 1)) * 0.1).astype(np.float32))


def predictor_batch(model: PredictorModel, seed: int = 2001, B: int = 1024, L: int = 16,
                    sigma_x: float = 1.0) -> PredictorBatch:
    """B workflow states: a walk of U{1..L+1} invocations over the model's call graph (the last
    one is the current agent, the ones before it the prefix) and an N(0, sigma_x^2) hidden state."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 37])))
    cur = np.zeros(B, np.int32)
    prefix = np.full((B, L), -1, np.int32)
    plen = np.zeros(B, np.int32)
    for b in range(B):
        t = int(rng.integers(1, L + 2))
        v = int(rng.integers(model.V))
        walk = [v]
        for _ in range(t - 1):
            row = model.trans[v].astype(np.float64)
            v = int(rng.choice(model.V, p=row / row.sum())) if row.sum() > 0 else int(rng.integers(model.V))
            walk.append(v)
        cur[b] = walk[-1]
        plen[b] = t - 1
        prefix[b, :t - 1] = walk[:-1]
    x = normal_tensor(seed, 41, (B, model.d_x), sigma_x, "bf16")
    return PredictorBatch(B, L, x, cur, prefix, plen)


CONFIGS = {
    "cfg0": tiny_fp32,
    "cfg1": shared_system_prompt,
    "cfg2": dynamic_workflow_batch,
    "cfg3": long_history,
    "cfg4": mixed_hit_miss,
}
