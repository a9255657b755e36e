"""GPU parity: the HIP path, called through the C boundary, against the fp64 oracle.

Tolerances: bf16 max abs error 2e-2 and relative L2 error 1e-2; fp32 max abs error 1e-5 and
relative L2 error 1e-5.  Where they come from: bf16 keeps 8 significand bits (2^-9 relative
rounding); the probabilities and the output are each rounded once, the rounding errors of the
probabilities average out over the keys, and rounding the pre-scaled query moves a score by
about 2^-9 |s| / sqrt(d), so the expected relative error is about 2^-9 = 2e-3 (with near-uniform
softmax over thousands of keys the outputs are O(0.01), hence the relative bound beside the
absolute one); fp32 sums 64..128 products per score and takes exp2 of arguments below 30, which
gives about 1e-6 relative.  Append and swap-in are byte moves and must be bit-exact.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2605_06472_amd import binding                      # noqa: E402
from paper_2605_06472_amd import workloads as W               # noqa: E402
from tests import bruteforce                                  # noqa: E402
from tests.gpu_util import PEAKED_ATOL, DeviceBatch, assert_close, attention_unit, sample_rows, to_numpy, to_torch   # noqa: E402


def _oracle(oracle, b, rows=None):
    return oracle.prefill(b.q, b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens,
                          b.new_lens, rows=rows)


def _check_full(oracle, b, what):
    print("case", what, "B", b.B, "N", b.N, flush=True)
    db = DeviceBatch(b)
    db.prefill()
    torch.cuda.synchronize()
    got = db.out_f64()
    want = _oracle(oracle, b)
    return assert_close(got, want, b.dtype, what)


# ------------------------------------------------------------------ small, element by element
def test_cfg0_tiny_fp32(oracle):
    b = W.tiny_fp32()
    _check_full(oracle, b, "cfg0")
    db = DeviceBatch(b)
    db.prefill()
    torch.cuda.synchronize()
    ref, _ = bruteforce.attention(b)
    assert_close(db.out_f64(), ref, "f32", "cfg0 vs contiguous brute force")


RAGGED = {
    "bf16_d128_g4": dict(dtype="bf16"),
    "bf16_d128_g4_peaked": dict(dtype="bf16", q_scale=8.0),
    "bf16_d64_g4": dict(dtype="bf16", d=64),
    "bf16_d128_g1": dict(dtype="bf16", Hq=2, Hkv=2),
    "bf16_d128_g2": dict(dtype="bf16", Hq=4, Hkv=2),
    "bf16_d128_g8": dict(dtype="bf16", Hq=16, Hkv=2),
    "bf16_d64_g16": dict(dtype="bf16", Hq=16, Hkv=1, d=64),
    "bf16_shared_root": dict(dtype="bf16", shared_root=48, num_pages=96),
    "bf16_tiles_and_tail": dict(dtype="bf16", prefix_lens=(300, 77, 1000, 0), new_lens=(200, 65, 130, 257),
                                num_pages=256),
    "f32_d64_g2": dict(dtype="f32", Hq=4, Hkv=2, d=64, sigma=1.0),
    "f32_d128_g3": dict(dtype="f32", Hq=6, Hkv=2, d=128, sigma=1.0),
    "f32_tiles_and_tail": dict(dtype="f32", Hq=2, Hkv=1, d=64, sigma=1.0, prefix_lens=(300, 77, 0),
                               new_lens=(100, 65, 130), num_pages=128),
}


@pytest.mark.parametrize("name", sorted(RAGGED))
def test_ragged_small_batches(oracle, name):
    b = W.ragged_small(40, **RAGGED[name])
    _check_full(oracle, b, name)


@pytest.fixture
def force_waves():
    """Forces the work-group shape of the bf16 attention launches for one test."""
    yield binding.set_attn_waves
    binding.set_attn_waves(0)


@pytest.mark.parametrize("waves", [4, 8, 64])
@pytest.mark.parametrize("name", sorted(n for n in RAGGED if n.startswith("bf16")))
def test_every_work_group_shape_of_the_bf16_kernel(oracle, name, waves, force_waves):
    """The library picks the work-group shape (4 waves of 32 rows or 4 of 64; 8 of 32 on request) from
    the batch; small batches like these would only ever see one of them, so each is forced in turn."""
    force_waves(waves)
    b = W.ragged_small(40, **RAGGED[name])
    _check_full(oracle, b, "%s, %s waves" % (name, waves))


MID = {
    "d64_g4": dict(Hq=8, Hkv=2, d=64),
    "d128_g8": dict(Hq=16, Hkv=2, d=128),
    "d128_g1": dict(Hq=2, Hkv=2, d=128),
    "d64_g16": dict(Hq=16, Hkv=1, d=64),
}


@pytest.mark.parametrize("waves", [4, 8, 64])
@pytest.mark.parametrize("name", sorted(MID))
def test_prefixes_of_several_page_id_blocks_in_every_shape(oracle, name, waves, force_waves):
    """The kernels hold 64 page ids (16 tiles) at a time and load the next block while the current one
    is in use; prefixes of 35 to 52 tiles take every work-group shape through two or three such
    reloads, a partly filled last page and a ragged suffix, for the head shapes the full-size
    configurations do not have."""
    force_waves(waves)
    b = W.ragged_small(43, "bf16", prefix_lens=(3301, 2240, 0, 2900), new_lens=(150, 65, 130, 1), num_pages=640, **MID[name])
    _check_sampled(oracle, b, "%s, %d waves" % (name, waves), per_request=24, max_boundaries=8)


def test_the_work_group_shape_does_not_change_a_bit(force_waves):
    """A row is computed by one wave in the same order of operations whichever shape the launch has."""
    b = W.ragged_small(41, "bf16", prefix_lens=(300, 77, 1000, 0), new_lens=(200, 65, 130, 257), num_pages=256, q_scale=8.0)
    outs = []
    for waves in (4, 8, 64):
        force_waves(waves)
        db = DeviceBatch(b)
        db.prefill()
        torch.cuda.synchronize()
        outs.append(to_numpy(db.out))
    assert np.array_equal(outs[0], outs[1])
    assert np.array_equal(outs[0], outs[2])


def test_repeated_calls_launch_from_the_cached_work_list(oracle):
    """A call that repeats the shape and lengths of an earlier call on its stream takes its work list
    from device memory (written there by the first launch); the result must not depend on that, nor
    on another batch's lists being cached in between, nor on the stream."""
    a = W.ragged_small(61, "bf16", prefix_lens=(300, 77, 1000, 0), new_lens=(200, 65, 130, 257), num_pages=256)
    c = W.ragged_small(62, "bf16", prefix_lens=(5, 130), new_lens=(70, 3))
    da, dc = DeviceBatch(a), DeviceBatch(c)
    want_a, want_c = _oracle(oracle, a), _oracle(oracle, c)
    pool_a = oracle.append_kv(a.k_new, a.v_new, a.kv_pool, a.block_table, a.prefix_lens, a.new_lens)
    da.prefill()
    first = da.out.clone()
    for k in range(3):
        da.out.zero_()
        dc.out.zero_()
        da.prefill()
        dc.prefill()
        da.append()
        torch.cuda.synchronize()
        assert torch.equal(da.out, first), k
        assert_close(dc.out_f64(), want_c, "bf16", "second batch, pass %d" % k)
        assert np.array_equal(to_numpy(da.kv_pool), pool_a)
    assert_close(da.out_f64(), want_a, "bf16", "cached list")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for k in range(2):                       # the side stream has its own cache: miss, then hit
        da.out.zero_()
        da.prefill(stream=side)
        side.synchronize()
        assert torch.equal(da.out, first)
    # many distinct batches in a row: more lists than the cache has slots
    for k in range(20):
        e = W.ragged_small(100 + k, "bf16", prefix_lens=(16 * k, 3), new_lens=(40 + k, 9), num_pages=64)
        de = DeviceBatch(e)
        de.prefill()
        de.prefill()
        torch.cuda.synchronize()
        assert_close(de.out_f64(), _oracle(oracle, e), "bf16", "batch %d" % k)
    da.out.zero_()
    da.prefill()
    torch.cuda.synchronize()
    assert torch.equal(da.out, first)


def test_single_row_and_empty_requests(oracle):
    b = W.ragged_small(41, "bf16", prefix_lens=(0, 0, 17, 64), new_lens=(1, 0, 1, 1))
    _check_full(oracle, b, "single rows")
    out = DeviceBatch(b)
    out.prefill()
    torch.cuda.synchronize()
    # first row of an empty prefix returns its own value exactly (bf16 in, bf16 out)
    G = b.Hq // b.Hkv
    assert np.array_equal(to_numpy(out.out)[0], np.repeat(b.v_new[0], G, axis=0))


def test_rows_of_other_calls_are_untouched(oracle):
    b = W.ragged_small(42, "bf16")
    db = DeviceBatch(b)
    big = torch.full((b.N + 8, b.Hq, b.d), 3.0, dtype=torch.bfloat16, device="cuda")
    db.prefill(out=big[4:4 + b.N])
    torch.cuda.synchronize()
    assert torch.all(big[:4] == 3.0) and torch.all(big[4 + b.N:] == 3.0)
    assert_close(W.to_f64(to_numpy(big[4:4 + b.N])), _oracle(oracle, b), "bf16", "offset out")


def test_more_streams_than_the_library_caches_for(oracle):
    """The library keeps work lists for eight streams per device; calls rotating over twelve make it
    hand the least recently used stream's slots to a new stream (after draining the device).  Every
    call must still give the oracle's result, attention, append and decode alike."""
    a = W.ragged_small(63, "bf16", prefix_lens=(300, 77, 0), new_lens=(130, 65, 70), num_pages=128)
    dec = W.ragged_small(64, "bf16", Hq=8, Hkv=2, prefix_lens=(700, 33, 130), new_lens=(1, 1, 1), num_pages=128)
    want = _oracle(oracle, a)
    want_dec = oracle.decode(dec.q, dec.kv_pool, dec.block_table, dec.prefix_lens)
    want_pool = oracle.append_kv(a.k_new, a.v_new, a.kv_pool, a.block_table, a.prefix_lens, a.new_lens)
    streams = [torch.cuda.Stream() for _ in range(12)]
    torch.cuda.synchronize()
    for rnd in range(2):
        for st in streams:
            da, dd = DeviceBatch(a), DeviceBatch(dec)
            out_dec = torch.full_like(dd.q, 7.0)
            torch.cuda.synchronize()
            da.prefill(stream=st)
            da.append(stream=st)
            binding.paged_decode(dd.shape, dd.q, dd.kv_pool, dd.block_table, dec.prefix_lens, out_dec, st)
            da.prefill(stream=st)                      # the cached list of this stream
            st.synchronize()
            assert_close(da.out_f64(), want, "bf16", "stream rotation")
            assert np.array_equal(to_numpy(da.kv_pool), want_pool)
            assert_close(W.to_f64(to_numpy(out_dec)), want_dec, "bf16", "decode, stream rotation")


# ------------------------------------------------------------------ invariants on the GPU
def test_page_permutation_is_bit_identical_on_gpu():
    a = W.ragged_small(43, "bf16", prefix_lens=(300, 77, 1000, 0), new_lens=(200, 65, 130, 257),
                       num_pages=256)
    perm = np.random.default_rng(2).permutation(a.num_pages)
    da = DeviceBatch(a)
    da.prefill()
    pool2 = np.empty_like(a.kv_pool)
    pool2[perm] = a.kv_pool
    dbb = DeviceBatch(a)
    dbb.kv_pool = to_torch(pool2)
    dbb.block_table = to_torch(perm[a.block_table].astype(np.int32))
    dbb.prefill()
    torch.cuda.synchronize()
    assert torch.equal(da.out, dbb.out)


def test_run_to_run_determinism():
    b = W.shared_system_prompt(batch=2, prefix=512, new=200, num_pages=128)
    db = DeviceBatch(b)
    db.prefill()
    first = db.out.clone()
    for _ in range(3):
        db.out.zero_()
        db.prefill()
        assert torch.equal(first, db.out)


def test_prefix_reuse_equals_from_scratch_on_gpu(oracle):
    """Same token sequence, once with a cached prefix and once as a full prefill."""
    b = W.ragged_small(44, "bf16", prefix_lens=(200,), new_lens=(120,), num_pages=64)
    L = 320
    K, V = b.logical_k[0], b.logical_v[0]
    qfull = W.normal_tensor(78, 0, (L, b.Hq, b.d), 2 ** -0.5, "bf16")
    qfull[200:] = b.q
    scratch = W.Batch(name="scratch", dtype="bf16", Hq=b.Hq, Hkv=b.Hkv, d=b.d, P=b.P,
                      num_pages=b.num_pages, q=qfull, k_new=np.ascontiguousarray(K),
                      v_new=np.ascontiguousarray(V), kv_pool=b.kv_pool,
                      block_table=np.zeros((1, 20), np.int32), prefix_lens=np.array([0], np.int32),
                      new_lens=np.array([L], np.int32))
    d1, d2 = DeviceBatch(b), DeviceBatch(scratch)
    d1.prefill()
    d2.prefill()
    torch.cuda.synchronize()
    want = _oracle(oracle, b)
    assert_close(d1.out_f64(), want, "bf16", "reuse")
    assert_close(d2.out_f64()[200:], want, "bf16", "from scratch")
    # the two GPU results agree with each other far inside the oracle tolerance
    assert np.abs(d1.out_f64() - d2.out_f64()[200:]).max() <= 1e-2


# ------------------------------------------------------------------ append / swap-in: bit-exact
@pytest.mark.parametrize("dtype,kw", [("bf16", {}), ("bf16", dict(d=64, Hq=4, Hkv=4)),
                                      ("f32", dict(d=64, Hq=2, Hkv=1, sigma=1.0))])
def test_append_is_bit_exact(oracle, dtype, kw):
    b = W.ragged_small(50, dtype, **kw)
    db = DeviceBatch(b)
    db.append()
    torch.cuda.synchronize()
    want = oracle.append_kv(b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    assert np.array_equal(to_numpy(db.kv_pool), want)
    assert not np.array_equal(want, b.kv_pool)


def test_swap_in_is_bit_exact_and_restores_attention(oracle):
    b = W.ragged_small(51, "bf16", prefix_lens=(48, 100, 333), new_lens=(3, 9, 40), nonresident=(2, 5, 11),
                       num_pages=96)
    db = DeviceBatch(b)
    db.swap_in()
    torch.cuda.synchronize()
    want_pool = oracle.swap_in(b.host_pages, b.swap_page_ids, b.kv_pool)
    assert np.array_equal(to_numpy(db.kv_pool), want_pool)
    db.prefill()
    torch.cuda.synchronize()
    ref, _ = bruteforce.attention(b)
    assert_close(db.out_f64(), ref, "bf16", "after swap-in")


def test_append_on_side_stream_overlaps_attention(oracle):
    b = W.ragged_small(52, "bf16", prefix_lens=(300, 77, 1000, 5), new_lens=(200, 65, 130, 257), num_pages=256)
    db = DeviceBatch(b)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    db.append(stream=side)
    db.prefill()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert_close(db.out_f64(), _oracle(oracle, b), "bf16", "attention beside append")
    want = oracle.append_kv(b.k_new, b.v_new, b.kv_pool, b.block_table, b.prefix_lens, b.new_lens)
    assert np.array_equal(to_numpy(db.kv_pool), want)


# ------------------------------------------------------------------ full-size configurations
def _check_sampled(oracle, b, what, per_request=4, max_boundaries=24, atol=None):
    db = DeviceBatch(b)
    unit = attention_unit(db)
    print("case", what, "B", b.B, "N", b.N, "unit", unit, "flops %.3g" % b.attention_flops(), flush=True)
    db.prefill()
    torch.cuda.synchronize()
    rows = sample_rows(b, per_request=per_request, unit=unit, max_boundaries=max_boundaries)
    got = db.out_f64()
    assert np.isfinite(got).all()
    want = _oracle(oracle, b, rows=rows)
    err, rel = assert_close(got[rows], want, b.dtype, what, atol=atol)
    print(what, "rows checked", len(rows), "max abs err %.3e rel L2 %.3e max |want| %.3f" % (err, rel, np.abs(want).max()), flush=True)
    return db


@pytest.mark.parametrize("q_scale", [1.0, 8.0])
def test_cfg1_shared_system_prompt(oracle, q_scale):
    b = W.shared_system_prompt(q_scale=q_scale)
    _check_sampled(oracle, b, "cfg1 q_scale=%g" % q_scale, per_request=8, atol=PEAKED_ATOL if q_scale > 1 else None)


@pytest.mark.parametrize("q_scale", [1.0, 8.0])
def test_cfg2_dynamic_workflow(oracle, q_scale):
    b = W.dynamic_workflow_batch(q_scale=q_scale)
    _check_sampled(oracle, b, "cfg2 q_scale=%g" % q_scale, atol=PEAKED_ATOL if q_scale > 1 else None)


@pytest.mark.parametrize("waves", [4, 8, 64])
def test_cfg2_peaked_in_every_work_group_shape(oracle, waves, force_waves):
    force_waves(waves)
    b = W.dynamic_workflow_batch(q_scale=8.0)
    _check_sampled(oracle, b, "cfg2 q_scale=8, %d waves" % waves, atol=PEAKED_ATOL)


@pytest.mark.parametrize("q_scale", [1.0, 8.0])
def test_cfg3_long_history(oracle, q_scale):
    """At least 256 rows per request: every boundary between 64-token units on both sides, the
    sub-block edges of the first and last unit, and 220 random rows."""
    b = W.long_history(q_scale=q_scale)
    _check_sampled(oracle, b, "cfg3 q_scale=%g" % q_scale, per_request=220, max_boundaries=64,
                   atol=PEAKED_ATOL if q_scale > 1 else None)


@pytest.mark.parametrize("slope", [0.0062, -0.0062], ids=["rising", "falling"])
def test_long_context_with_a_moving_reference(oracle, slope):
    """One request of the long-history size (32768 cached + 2048 new tokens, 545 tile steps in the
    64-token units) whose scores climb by about 13 log2 units per 32-key block -- past the
    threshold at which the kernel moves its reference, so the redo path runs at nearly every block
    of every step -- or fall at that rate (the reference stays where the first block put it and the
    later probabilities vanish)."""
    b = _moving_reference_batch(slope)
    db = DeviceBatch(b)
    unit = attention_unit(db)
    assert unit == 64
    db.prefill()
    torch.cuda.synchronize()
    rows = sample_rows(b, per_request=64, unit=unit, max_boundaries=32)
    want = _oracle(oracle, b, rows=rows)
    err, rel = assert_close(db.out_f64()[rows], want, "bf16", "moving reference, slope %g" % slope)
    print("moving reference slope %g: rows %d max abs err %.3e rel L2 %.3e" % (slope, len(rows), err, rel), flush=True)


def _moving_reference_batch(slope):
    b = W.long_history(seed=1013, batch=1, num_pages=4096)
    d, p, n = b.d, int(b.prefix_lens[0]), int(b.new_lens[0])
    u = np.sign(np.random.default_rng(3).standard_normal(d)).astype(np.float32)
    b.q = W.f32_to_bf16_bits(np.broadcast_to(4.0 * u, (n, b.Hq, d)).astype(np.float32))
    t = np.arange(p + n, dtype=np.float32) + 1.0
    keys = W.f32_to_bf16_bits((slope * t)[:, None, None] * np.broadcast_to(u, (p + n, b.Hkv, d)))
    pages = b.block_table[0, :p // b.P]
    b.kv_pool[pages, 0] = keys[:p].reshape(p // b.P, b.P, b.Hkv, d).transpose(0, 2, 1, 3)
    b.k_new[:] = keys[p:]
    return b


@pytest.mark.parametrize("case", ["cfg4_peaked", "moving_reference"])
def test_full_size_outputs_are_the_same_bits_in_every_shape(case, force_waves):
    """The three work-group shapes run the same arithmetic per row in the same order, one of them
    with its matrix and softmax instructions placed and its hazards kept by hand: at full size and
    under full load their outputs must agree bit for bit -- on the mixed batch with peaked scores, and
    on the batch whose reference moves at nearly every block."""
    b = W.mixed_hit_miss(q_scale=8.0) if case == "cfg4_peaked" else _moving_reference_batch(0.0062)
    db = DeviceBatch(b)
    if b.host_pages is not None:
        db.swap_in()
    outs = []
    for waves in (4, 8, 64):
        force_waves(waves)
        db.out.zero_()
        db.prefill()
        torch.cuda.synchronize()
        outs.append(db.out.clone())
    assert torch.isfinite(outs[0].float()).all()
    assert torch.equal(outs[0], outs[1]), "4 against 8 waves"
    assert torch.equal(outs[0], outs[2]), "4 waves against the 64-row form"


@pytest.mark.parametrize("q_scale", [1.0, 8.0])
def test_cfg4_mixed_hit_miss_with_swap_in(oracle, q_scale):
    """Pages of the host tier are swapped in on a side stream, group by group, while the
    main stream attends to the requests whose pages have landed; then the suffix KV is
    appended.  Pool content and attention output are checked against the oracle (at least 64
    rows per request, unit boundaries included)."""
    b = W.mixed_hit_miss(q_scale=q_scale)
    print("case cfg4 B", b.B, "N", b.N, "swap pages", b.host_pages.shape[0], flush=True)
    db = DeviceBatch(b)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    order = np.argsort(np.diff(b.swap_offsets), kind="stable")      # fewest missing pages first
    # the C calls take contiguous request ranges, so each group is a set of single requests
    off = np.concatenate([[0], np.cumsum(b.new_lens)]).astype(np.int64)
    side.wait_stream(main)
    for grp in np.array_split(order, 4):
        for r in grp:
            lo, hi = int(b.swap_offsets[r]), int(b.swap_offsets[r + 1])
            if hi > lo:
                binding.swap_in_pages(db.shape, db.host_pages[lo:hi], b.swap_page_ids[lo:hi], db.kv_pool, side)
        ev = torch.cuda.Event()
        ev.record(side)
        main.wait_event(ev)
        for r in grp:
            sl = slice(int(off[r]), int(off[r + 1]))
            binding.prefix_prefill(db.sub_shape(1), db.q[sl], db.k_new[sl], db.v_new[sl], db.kv_pool,
                                   db.block_table[r:r + 1], b.prefix_lens[r:r + 1], b.new_lens[r:r + 1],
                                   db.out[sl], main)
    done = torch.cuda.Event()
    done.record(main)
    side.wait_event(done)
    db.append(stream=side)
    torch.cuda.synchronize()
    resident = oracle.swap_in(b.host_pages, b.swap_page_ids, b.kv_pool)
    # single-request calls take the 32-row or the 64-row shape request by request: sample around both unit sizes
    rows = np.union1d(sample_rows(b, per_request=40, unit=64, max_boundaries=12),
                      sample_rows(b, per_request=0, unit=32, max_boundaries=12, seed=1))
    want = oracle.prefill(b.q, b.k_new, b.v_new, resident, b.block_table, b.prefix_lens, b.new_lens, rows=rows)
    err, rel = assert_close(db.out_f64()[rows], want, "bf16", "cfg4 q_scale=%g" % q_scale,
                            atol=PEAKED_ATOL if q_scale > 1 else None)
    print("cfg4 q_scale=%g rows checked" % q_scale, len(rows), "max abs err %.3e rel L2 %.3e" % (err, rel), flush=True)
    final = oracle.append_kv(b.k_new, b.v_new, resident, b.block_table, b.prefix_lens, b.new_lens)
    assert np.array_equal(to_numpy(db.kv_pool), final)


def test_pageable_host_memory_is_rejected():
    b = W.ragged_small(53, "bf16", prefix_lens=(48,), new_lens=(3,), nonresident=(2,))
    db = DeviceBatch(b)
    pageable = to_torch(b.host_pages, "cpu", pin=False)
    with pytest.raises(binding.PbkvError) as e:
        binding.swap_in_pages(db.shape, pageable, b.swap_page_ids, db.kv_pool)
    assert e.value.code == -6


def test_swap_out_bit_exact_and_round_trip(oracle):
    """Pool -> pinned host page gather (the host-tier half that swap-in mirrors): equal to the
    oracle byte for byte, pool untouched, and swapped back into other slots it reproduces the pages."""
    b = W.ragged_small(41, "bf16", prefix_lens=(48, 100, 7), new_lens=(3, 9, 20))
    db = DeviceBatch(b)
    rng = np.random.default_rng(11)
    ids = rng.permutation(b.num_pages)[:11].astype(np.int32)
    ids[4] = ids[1]
    want = oracle.swap_out(b.kv_pool, ids)
    host = torch.zeros((len(ids),) + tuple(db.kv_pool.shape[1:]), dtype=db.kv_pool.dtype).pin_memory()
    binding.swap_out_pages(db.shape, db.kv_pool, ids, host)
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(host), want)
    assert np.array_equal(to_numpy(db.kv_pool), b.kv_pool)
    dst = np.setdiff1d(np.arange(b.num_pages, dtype=np.int32), ids)[:len(ids)].astype(np.int32)
    binding.swap_in_pages(db.shape, host, dst, db.kv_pool)
    torch.cuda.synchronize()
    assert np.array_equal(to_numpy(db.kv_pool), oracle.swap_in(want, dst, b.kv_pool))
    with pytest.raises(binding.PbkvError) as e:
        binding.swap_out_pages(db.shape, db.kv_pool, np.array([b.num_pages], np.int32), host)
    assert e.value.code == -4
    # empty list is a no-op
    binding.swap_out_pages(db.shape, db.kv_pool, np.zeros(0, np.int32), host)


@pytest.mark.parametrize("slope", [0.05, -0.05], ids=["rising", "falling"])
def test_scores_that_run_away_along_the_context(oracle, slope):
    """Scores that climb (or fall) by ~100 log2 units per 32-key block: every block overflows the
    reference set by its predecessors (or underflows it), so the kernel's redo path runs at every
    block; the result must still match the exact definition."""
    b = W.ragged_small(95, "bf16", prefix_lens=(300, 37, 0), new_lens=(70, 5, 40), num_pages=64)
    d = b.d
    u = np.sign(np.random.default_rng(3).standard_normal(d)).astype(np.float32)       # |u|^2 = d
    q = np.broadcast_to(4.0 * u, W.to_f64(b.q).shape).astype(np.float32)
    b.q = W.f32_to_bf16_bits(q)
    # key t of a request = u * slope * (t + 1): prefix keys live in the pool, suffix keys in k_new
    off = 0
    for r in range(b.B):
        p, n = int(b.prefix_lens[r]), int(b.new_lens[r])
        t = np.arange(p + n, dtype=np.float32) + 1.0
        keys = W.f32_to_bf16_bits((slope * t)[:, None, None] * np.broadcast_to(u, (p + n, b.Hkv, d)))
        for tok in range(p):
            b.kv_pool[b.block_table[r, tok // b.P], 0, :, tok % b.P] = keys[tok]
        b.k_new[off:off + n] = keys[p:]
        off += n
    db = DeviceBatch(b)
    db.prefill()
    torch.cuda.synchronize()
    want = _oracle(oracle, b)
    assert_close(db.out_f64(), want, "bf16", "runaway scores, slope %g" % slope)
