"""The decode entry point that allocates nothing (for callers that cannot call hipMalloc: graph
capture, serving loops) against the ordinary one: same kernels, so the outputs must agree bit for
bit, and both must match the oracle; two calls in a row on the one static array, the second with a
smaller input; the limits are refused with a clear error."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2605_06472_amd import binding, workloads as W          # noqa: E402
from tests.gpu_util import DeviceBatch, assert_close, to_numpy     # noqa: E402


def test_static_decode_matches_the_allocating_entry_point(oracle):
    big = W.decode_batch(seed=1205, batch=48, min_ctx=1500, max_ctx=12000, num_pages=32768)
    small = W.ragged_small(94, "bf16", Hq=32, Hkv=8, prefix_lens=(700, 33, 0, 4097, 16), new_lens=(1,) * 5, num_pages=512)
    for b in (big, small):                       # second call: smaller input, same static array
        print("case static decode", b.name, "B", b.B, "tokens", int(b.prefix_lens.sum()), flush=True)
        db = DeviceBatch(b)
        ref = torch.full_like(db.q, 7.0)
        got = torch.full_like(db.q, 5.0)
        binding.paged_decode(db.shape, db.q, db.kv_pool, db.block_table, b.prefix_lens, ref)
        torch.cuda.synchronize()
        binding.paged_decode_static(db.shape, db.q, db.kv_pool, db.block_table, b.prefix_lens, got)
        torch.cuda.synchronize()
        assert torch.equal(got, ref)
        want = oracle.decode(b.q, b.kv_pool, b.block_table, b.prefix_lens)
        assert_close(W.to_f64(to_numpy(got)), want, "bf16", "static decode, " + b.name)
    # and the first one again, after the smaller call left its lists and partials behind
    db = DeviceBatch(big)
    got = torch.full_like(db.q, 5.0)
    binding.paged_decode_static(db.shape, db.q, db.kv_pool, db.block_table, big.prefix_lens, got)
    torch.cuda.synchronize()
    assert_close(W.to_f64(to_numpy(got)), oracle.decode(big.q, big.kv_pool, big.block_table, big.prefix_lens),
                 "bf16", "static decode, repeated")


def test_static_decode_refuses_what_does_not_fit():
    b = W.ragged_small(95, "bf16", prefix_lens=(40,), new_lens=(1,))
    db = DeviceBatch(b)
    shape = binding.make_shape(5000, b.Hq, b.Hkv, b.d, b.P, b.num_pages, b.max_pages, "bf16")
    q = torch.zeros((5000, b.Hq, b.d), dtype=torch.bfloat16, device="cuda")
    table = torch.zeros((5000, b.max_pages), dtype=torch.int32, device="cuda")
    with pytest.raises(binding.PbkvError) as e:
        binding.paged_decode_static(shape, q, db.kv_pool, table, np.full(5000, 16, np.int32), torch.zeros_like(q))
    assert e.value.code == -7 and "at most 4096" in str(e.value)
