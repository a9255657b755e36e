"""Paged decode attention against the oracle (the prefill definition with one new token): small
ragged contexts for every supported head shape, element by element; a full-size pure-decode batch
on all of its rows; repeatability; argument errors."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2605_06472_amd import binding, workloads as W          # noqa: E402
from tests.gpu_util import DeviceBatch, assert_close, to_numpy     # noqa: E402


def run_decode(b, lens=None):
    db = DeviceBatch(b)
    lens = b.prefix_lens if lens is None else np.asarray(lens, np.int32)
    out = torch.full_like(db.q, 7.0)
    binding.paged_decode(db.shape, db.q, db.kv_pool, db.block_table, lens, out)
    torch.cuda.synchronize()
    return db, W.to_f64(to_numpy(out))


CONTEXTS = (1, 15, 16, 17, 64, 130, 1000, 0, 4097)


@pytest.mark.parametrize("hq,hkv,d", [(8, 2, 128), (4, 4, 64), (4, 2, 64), (16, 2, 64), (32, 2, 128), (32, 8, 128), (8, 8, 128)],
                         ids=["g4_d128", "g1_d64", "g2_d64", "g8_d64", "g16_d128", "g4x8_d128", "g1_d128"])
def test_decode_small_contexts_match_oracle(oracle, hq, hkv, d):
    b = W.ragged_small(70 + hq + d, "bf16", Hq=hq, Hkv=hkv, d=d, prefix_lens=CONTEXTS, new_lens=(1,) * len(CONTEXTS),
                       num_pages=640)
    db, got = run_decode(b)
    want = oracle.decode(b.q, b.kv_pool, b.block_table, b.prefix_lens)
    assert not got[CONTEXTS.index(0)].any()
    assert_close(got, want, "bf16", "decode %d/%d d=%d" % (hq, hkv, d))


def test_decode_peaked_scores_and_late_maximum(oracle):
    """Scores that grow along the context force the reference to move many times."""
    b = W.ragged_small(90, "bf16", prefix_lens=(700, 33), new_lens=(1, 1), num_pages=64, q_scale=8.0)
    db, got = run_decode(b)
    want = oracle.decode(b.q, b.kv_pool, b.block_table, b.prefix_lens)
    assert_close(got, want, "bf16", "peaked decode")


def test_decode_shorter_context_than_the_table_holds(oracle):
    """context_lens may stop anywhere inside the pages the table names."""
    b = W.ragged_small(91, "bf16", prefix_lens=(300, 300, 300), new_lens=(1, 1, 1), num_pages=64)
    lens = np.array([299, 160, 1], np.int32)
    db, got = run_decode(b, lens)
    assert_close(got, oracle.decode(b.q, b.kv_pool, b.block_table, lens), "bf16", "short contexts")


def test_decode_full_size_batch_all_rows(oracle):
    b = W.decode_batch()
    db, got = run_decode(b)
    want = oracle.decode(b.q, b.kv_pool, b.block_table, b.prefix_lens)
    err, rel = assert_close(got, want, "bf16", "decode batch")
    # run to run bit-identical: fixed slice boundaries, fixed merge order
    _, again = run_decode(b)
    assert np.array_equal(got, again)


def test_decode_calls_on_two_streams_overlap_safely(oracle):
    """Two decode calls in flight at once on different streams, each with its own batch, its own
    cached work list and its own scratch buffer (the second batch needs a larger one than the first
    call left behind on its stream), several rounds: every result equals the oracle's."""
    big = W.decode_batch(seed=1105, batch=24, min_ctx=2000, max_ctx=9000, num_pages=16384)
    small = W.ragged_small(93, "bf16", Hq=32, Hkv=8, prefix_lens=(700, 33, 4097), new_lens=(1, 1, 1), num_pages=512)
    want = {id(x): oracle.decode(x.q, x.kv_pool, x.block_table, x.prefix_lens) for x in (big, small)}
    dbig, dsmall = DeviceBatch(big), DeviceBatch(small)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = []
    for k in range(4):
        (a, sa), (c, sc) = ((dbig, s1), (dsmall, s2)) if k % 2 == 0 else ((dsmall, s1), (dbig, s2))
        oa, oc = torch.full_like(a.q, 7.0), torch.full_like(c.q, 7.0)
        binding.paged_decode(a.shape, a.q, a.kv_pool, a.block_table, a.b.prefix_lens, oa, sa)
        binding.paged_decode(c.shape, c.q, c.kv_pool, c.block_table, c.b.prefix_lens, oc, sc)
        binding.paged_decode(a.shape, a.q, a.kv_pool, a.block_table, a.b.prefix_lens, oa, sa)
        outs.append((a, oa, c, oc))
    torch.cuda.synchronize()
    for a, oa, c, oc in outs:
        assert_close(W.to_f64(to_numpy(oa)), want[id(a.b)], "bf16", "stream 1")
        assert_close(W.to_f64(to_numpy(oc)), want[id(c.b)], "bf16", "stream 2")


def test_decode_argument_errors():
    b = W.ragged_small(92, "bf16", prefix_lens=(40,), new_lens=(1,))
    db = DeviceBatch(b)
    out = torch.zeros_like(db.q)
    for lens, code in ((np.array([-1], np.int32), -4), (np.array([16 * b.max_pages + 1], np.int32), -4)):
        with pytest.raises(binding.PbkvError) as e:
            binding.paged_decode(db.shape, db.q, db.kv_pool, db.block_table, lens, out)
        assert e.value.code == code
    f = W.tiny_fp32()
    df = DeviceBatch(f)
    with pytest.raises(binding.PbkvError) as e:
        binding.paged_decode(df.shape, df.q, df.kv_pool, df.block_table, f.prefix_lens, torch.zeros_like(df.q))
    assert e.value.code == -3
