"""Pins for the fp64 oracle: what the mathematics fixes, checked without any GPU.

Each test is chosen so that a plausible mistake in the oracle (a dropped 1/sqrt(d), a
wrong mask edge, a transposed page index, a wrong GQA mapping, K and V swapped, a wrong
slot inside a page) makes at least one of them fail.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2605_06472_amd import workloads as W
from tests import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _run(oracle, b, **kw):
    return oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens,
                          b.new_lens, **kw)


# ---------------------------------------------------------------- hand-derived values
def test_golden_rational_example(oracle):
    g = json.load(open(os.path.join(GOLDEN, "rational_attention.json")))
    d, P, Hkv, Hq = g["d"], g["P"], g["Hkv"], g["Hq"]
    rng = np.random.default_rng(5)
    pool = rng.standard_normal((g["num_pages"], 2, Hkv, P, d)).astype(np.float32)
    keys = np.zeros((4, d), np.float32)
    keys[:, 0] = np.log(np.array(g["a"], np.float64)).astype(np.float32)
    keys[:, 1] = np.log(np.array(g["b"], np.float64)).astype(np.float32)
    V = np.array(g["V"], np.float32)
    p, n = g["prefix_len"], g["new_len"]
    pool[g["prefix_page"], 0, 0, :p] = keys[:p]
    pool[g["prefix_page"], 1, 0, :p] = V[:p]
    bt = np.array([[g["prefix_page"]]], np.int32)
    q = np.array(g["q"], np.float32)                       # [n, Hq, d]
    out, rowsum, lse = _run_raw(oracle, q, keys[p:, None, :], V[p:, None, :], pool, bt, [p], [n])
    exp = np.array([[[float(Fraction(x)) for x in head] for head in row]
                    for row in g["expected_out_fractions"]])
    # inputs are ln(.) rounded to float32, so agreement is to float32 rounding of the logs
    np.testing.assert_allclose(out, exp, rtol=0, atol=2e-6)
    z = np.array([[float(Fraction(x)) for x in row]
                  for row in g["expected_sum_of_weights_before_normalising"]])
    np.testing.assert_allclose(np.exp(lse), z, rtol=1e-6)
    np.testing.assert_allclose(rowsum, 1.0, atol=1e-14)


def _run_raw(oracle, q, k_new, v_new, pool, bt, p, n, **kw):
    return oracle.prefill(np.ascontiguousarray(q), np.ascontiguousarray(k_new),
                          np.ascontiguousarray(v_new), pool, np.asarray(bt, np.int32),
                          np.asarray(p, np.int32), np.asarray(n, np.int32), want_stats=True, **kw)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("make", [
    lambda: W.tiny_fp32(),
    lambda: W.ragged_small(3, "bf16"),
    lambda: W.ragged_small(4, "f32", Hq=6, Hkv=3, d=64),
    lambda: W.ragged_small(5, "bf16", Hq=4, Hkv=4, d=32, shared_root=32),
    lambda: W.ragged_small(6, "bf16", q_scale=8.0),
])
def test_matches_contiguous_bruteforce(oracle, make):
    b = make()
    out, rowsum, lse = _run(oracle, b, want_stats=True)
    ref, ref_lse = bruteforce.attention(b)
    assert out.shape == ref.shape
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-12)
    np.testing.assert_allclose(rowsum, 1.0, rtol=0, atol=1e-13)


def test_row_subset_equals_full(oracle):
    b = W.ragged_small(8, "bf16")
    full = _run(oracle, b)
    rows = np.array([0, 3, 4, 73, b.N - 1], np.int64)
    sub = _run(oracle, b, rows=rows)
    assert np.array_equal(sub, full[rows])


# ---------------------------------------------------------------- invariants
def test_page_permutation_is_bit_identical(oracle):
    a = W.ragged_small(9, "bf16", num_pages=64)
    rng = np.random.default_rng(1)
    perm = rng.permutation(a.num_pages)                 # new physical slot of old page i
    pool2 = np.empty_like(a.kv_pool)
    pool2[perm] = a.kv_pool
    bt2 = perm[a.block_table].astype(np.int32)
    o1 = _run(oracle, a)
    o2 = oracle.prefill(a.q, a.k_new, a.v_new, pool2, bt2, a.prefix_lens, a.new_lens)
    assert np.array_equal(o1, o2)
    assert not np.array_equal(bt2, a.block_table)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_prefix_reuse_equals_from_scratch_prefill(oracle, dtype):
    """Rows of the suffix computed with a cached prefix == the same rows of a full prefill,
    for every split point of the same token sequence."""
    b = W.ragged_small(10, dtype, Hq=4, Hkv=2, d=64, prefix_lens=(37,), new_lens=(27,))
    L = 64
    K, V = b.logical_k[0], b.logical_v[0]
    qfull = W.normal_tensor(77, 0, (L, b.Hq, b.d), 1.0, dtype)
    pool0 = b.kv_pool
    bt0 = np.zeros((1, 1), np.int32)
    scratch = oracle.prefill(qfull, K, V, pool0, bt0, np.array([0], np.int32),
                             np.array([L], np.int32))
    for p in (1, 16, 37, 48, 63):
        n = L - p
        # page the first p tokens at fresh physical slots
        npg = -(-p // b.P)
        slots = np.random.default_rng(p).permutation(b.num_pages)[:npg].astype(np.int32)
        pool = pool0.copy()
        for t in range(p):
            pool[slots[t // b.P], 0, :, t % b.P] = K[t]
            pool[slots[t // b.P], 1, :, t % b.P] = V[t]
        bt = np.zeros((1, 4), np.int32)
        bt[0, :npg] = slots
        part = oracle.prefill(qfull[p:], K[p:], V[p:], pool, bt, np.array([p], np.int32),
                              np.array([n], np.int32))
        assert np.array_equal(part, scratch[p:]), p


def test_weights_sum_to_one(oracle):
    b = W.ragged_small(11, "bf16", q_scale=8.0)
    _, rowsum, _ = _run(oracle, b, want_stats=True)
    L = (np.repeat(b.prefix_lens, b.new_lens) + 1 + b.N)[:, None]
    assert np.all(np.abs(rowsum - 1.0) <= 1e-15 * L)


def test_causality(oracle):
    b = W.ragged_small(12, "f32", Hq=4, Hkv=2, d=64, prefix_lens=(20,), new_lens=(40,))
    base = _run(oracle, b)
    j = 17
    k2, v2 = b.k_new.copy(), b.v_new.copy()
    k2[j] += 3.0
    v2[j] -= 2.0
    pert = oracle.prefill(b.q, k2, v2, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    assert np.array_equal(pert[:j], base[:j])
    assert np.all(np.any(pert[j:] != base[j:], axis=(1, 2)))   # the diagonal is visible


def test_gqa_head_mapping(oracle):
    b = W.ragged_small(13, "f32", Hq=6, Hkv=3, d=64, prefix_lens=(33,), new_lens=(9,))
    q = b.q.copy()
    q[:, 1] = q[:, 0]                # heads 0,1 share KV head 0 -> equal outputs
    q[:, 2] = q[:, 0]                # head 2 reads KV head 1 -> different output
    out = oracle.prefill(q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    assert np.array_equal(out[:, 0], out[:, 1])
    assert not np.array_equal(out[:, 0], out[:, 2])
    # swapping the data of KV heads 0 and 2 (pool and suffix) swaps the groups' outputs
    sw = [2, 1, 0]
    pool2 = b.kv_pool[:, :, sw]
    out2 = oracle.prefill(q[:, [4, 5, 2, 3, 0, 1]], b.k_new[:, sw], b.v_new[:, sw],
                          np.ascontiguousarray(pool2), b.block_table, b.prefix_lens, b.new_lens)
    assert np.array_equal(out2[:, [4, 5, 2, 3, 0, 1]], out)


# ---------------------------------------------------------------- closed forms
def _small_problem(seed, p=37, n=11, Hq=4, Hkv=2, d=64):
    return W.ragged_small(seed, "f32", Hq=Hq, Hkv=Hkv, d=d, prefix_lens=(p,), new_lens=(n,))


def test_equal_keys_give_mean_of_values(oracle):
    b = _small_problem(20)
    pool = b.kv_pool.copy()
    pool[:, 0] = 0.25                                   # every K row identical
    k_new = np.full_like(b.k_new, 0.25)
    out = oracle.prefill(b.q, k_new, b.v_new, pool, b.block_table, b.prefix_lens, b.new_lens)
    p = int(b.prefix_lens[0])
    V = b.logical_v[0].astype(np.float64)
    for i in range(b.N):
        mean = V[: p + i + 1].mean(axis=0)               # [Hkv, d]
        np.testing.assert_allclose(out[i], np.repeat(mean, 2, axis=0), atol=1e-13)


def test_equal_values_are_returned(oracle):
    b = _small_problem(21)
    pool = b.kv_pool.copy()
    c = np.linspace(-1, 1, b.d, dtype=np.float32)
    pool[:, 1] = c
    v_new = np.broadcast_to(c, b.v_new.shape).copy()
    out = oracle.prefill(b.q, b.k_new, v_new, pool, b.block_table, b.prefix_lens, b.new_lens)
    np.testing.assert_allclose(out, np.broadcast_to(c.astype(np.float64), out.shape), atol=1e-14)


def test_dominant_key_selects_its_value(oracle):
    b = _small_problem(22, p=40, n=1)
    pool = b.kv_pool.copy()
    pool[:, 0] = 0.0
    k_new = np.zeros_like(b.k_new)
    t_star = 21                                          # page 1, slot 5 of the prefix
    qv = b.q[0, 0].astype(np.float64)
    qhat = (qv / np.linalg.norm(qv)).astype(np.float32)
    q = np.broadcast_to(qhat * 10, b.q.shape).copy()
    pg = b.block_table[0, t_star // 16]
    pool[pg, 0, :, t_star % 16] = qhat * 50              # score = 500/sqrt(64) = 62.5, others 0
    out = oracle.prefill(q, k_new, b.v_new, pool, b.block_table, b.prefix_lens, b.new_lens)
    Vstar = np.repeat(pool[pg, 1, :, t_star % 16].astype(np.float64), 2, axis=0)
    np.testing.assert_allclose(out[0], Vstar, atol=41 * np.exp(-62.0) * 10)


def test_first_row_of_empty_prefix_is_its_own_value(oracle):
    b = W.ragged_small(23, "bf16", prefix_lens=(0,), new_lens=(5,))
    out = _run(oracle, b)
    G = b.Hq // b.Hkv
    np.testing.assert_array_equal(out[0], np.repeat(W.to_f64(b.v_new[0]), G, axis=0))


def test_oracle_rejects_bad_tables(oracle):
    b = _small_problem(24)
    bt = b.block_table.copy()
    bt[0, 1] = b.num_pages
    with pytest.raises(ValueError):
        oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, bt, b.prefix_lens, b.new_lens)


# ---------------------------------------------------------------- append / swap-in
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_append_matches_indexed_scatter(oracle, dtype):
    b = W.ragged_small(30, dtype, Hq=4, Hkv=2, d=64)
    got = oracle.append_kv(b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    want = b.kv_pool.copy()
    touched = np.zeros(want.shape[:1] + (b.P,), bool)
    off = 0
    for r in range(b.B):
        pos = int(b.prefix_lens[r]) + np.arange(int(b.new_lens[r]))
        pg = b.block_table[r, pos // b.P]
        want[pg, 0, :, pos % b.P] = b.k_new[off:off + len(pos)]
        want[pg, 1, :, pos % b.P] = b.v_new[off:off + len(pos)]
        touched[pg, pos % b.P] = True
        off += len(pos)
    assert np.array_equal(got, want)
    # every untouched slot keeps its bytes
    keep = ~touched
    assert np.array_equal(got.transpose(0, 3, 1, 2, 4)[keep], b.kv_pool.transpose(0, 3, 1, 2, 4)[keep])
    assert touched.sum() == b.N


def test_append_then_attend_equals_longer_prefix(oracle):
    """After the append, the pool alone holds prefix + suffix: a follow-up request whose
    prefix is the whole sequence sees exactly the keys the first one saw plus its own."""
    b = W.ragged_small(31, "bf16", Hq=4, Hkv=2, d=64, prefix_lens=(21,), new_lens=(30,))
    pool2 = oracle.append_kv(b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    last = oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)[-1]
    # one-token request: prefix = first 50 tokens from the pool, suffix = token 50
    again = oracle.prefill(b.q[-1:], b.k_new[-1:], b.v_new[-1:], pool2, b.block_table,
                           np.array([50], np.int32), np.array([1], np.int32))[0]
    assert np.array_equal(last, again)


def test_swap_in_matches_fancy_index(oracle):
    b = W.ragged_small(32, "bf16", Hq=4, Hkv=2, d=64, prefix_lens=(48, 100), new_lens=(3, 9),
                       nonresident=(2, 5))
    assert b.host_pages.shape[0] == 7
    got = oracle.swap_in(b.host_pages, b.swap_page_ids, b.kv_pool)
    want = b.kv_pool.copy()
    want[b.swap_page_ids] = b.host_pages
    assert np.array_equal(got, want)
    assert not np.array_equal(got, b.kv_pool)
    # with the pages back, attention equals the brute force over the pre-paging K/V
    out = oracle.prefill(b.q, b.k_new, b.v_new, got, b.block_table, b.prefix_lens, b.new_lens)
    ref, _ = bruteforce.attention(b)
    np.testing.assert_allclose(out, ref, atol=1e-12)
    stale = oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    assert np.abs(stale - ref).max() > 1e-3


def test_swap_out_matches_fancy_index_and_round_trips(oracle):
    """Swap-out (Sec. 2, host tier) is a page gather: equal to numpy fancy indexing, pool untouched,
    and swap-out followed by swap-in into other slots reproduces the pages there."""
    b = W.ragged_small(33, "bf16", Hq=4, Hkv=2, d=64, prefix_lens=(48, 100), new_lens=(3, 9))
    rng = np.random.default_rng(5)
    ids = rng.permutation(b.num_pages)[:9].astype(np.int32)
    ids[3] = ids[0]                                        # a page may be named twice
    pool0 = b.kv_pool.copy()
    host = oracle.swap_out(b.kv_pool, ids)
    assert np.array_equal(b.kv_pool, pool0)
    assert np.array_equal(host, b.kv_pool[ids])
    assert not np.array_equal(host[0], host[1])
    dst = np.setdiff1d(np.arange(b.num_pages, dtype=np.int32), ids)[:9].astype(np.int32)
    back = oracle.swap_in(host, dst, b.kv_pool)
    assert np.array_equal(back[dst], b.kv_pool[ids])
    with pytest.raises(ValueError):
        oracle.swap_out(b.kv_pool, np.array([b.num_pages], np.int32))


def test_decode_is_a_softmax_weighted_mean_over_the_paged_context(oracle):
    """Decode rows (one query per request over its whole paged context) against a textbook
    softmax-weighted mean over the contiguous K/V that the generator kept before paging."""
    from scipy.special import softmax
    b = W.ragged_small(61, "bf16", Hq=8, Hkv=2, d=64, prefix_lens=(1, 16, 37, 130, 0), new_lens=(1, 1, 1, 1, 1))
    lens = b.prefix_lens.copy()
    q = b.q                                    # one row per request: [5, Hq, d]
    out = oracle.decode(q, b.kv_pool, b.block_table, lens)
    G = b.Hq // b.Hkv
    for r in range(b.B):
        L = int(lens[r])
        if L == 0:
            assert not out[r].any()
            continue
        K, V = W.to_f64(b.logical_k[r][:L]), W.to_f64(b.logical_v[r][:L])
        for h in range(b.Hq):
            w = softmax(W.to_f64(q[r, h]) @ K[:, h // G].T / np.sqrt(b.d))
            np.testing.assert_allclose(out[r, h], w @ V[:, h // G], atol=1e-12)
