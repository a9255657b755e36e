"""Gather diagnostic: the words the attention kernel's page gather stages, XORed per work unit,
against the same XOR taken over the contiguous pre-paging K/V (or, for the large batches, over a
plain numpy walk of the block table).  Bit-exact."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2605_06472_amd import binding, workloads as W          # noqa: E402
from tests.gpu_util import DeviceBatch                             # noqa: E402


def _words(a):
    return np.ascontiguousarray(a).view(np.uint32).reshape(-1)


def _logical_kv(b, r):
    """[p + n, Hkv, d] K and V of request r: the kept pre-paging arrays, else a block-table walk."""
    if b.logical_k is not None:
        return b.logical_k[r], b.logical_v[r]
    p, n = int(b.prefix_lens[r]), int(b.new_lens[r])
    off = int(b.new_lens[:r].sum())
    npg = -(-p // b.P)
    pg = b.kv_pool[b.block_table[r, :npg]]
    k = pg[:, 0].transpose(0, 2, 1, 3).reshape(-1, b.Hkv, b.d)[:p]
    v = pg[:, 1].transpose(0, 2, 1, 3).reshape(-1, b.Hkv, b.d)[:p]
    return (np.concatenate([k, b.k_new[off:off + n]], 0), np.concatenate([v, b.v_new[off:off + n]], 0))


def expected_unit_xor(b, unit_tokens):
    G = b.Hq // b.Hkv
    nsplit = G // min(G, 4)
    out = []
    for r in range(b.B):
        p, n = int(b.prefix_lens[r]), int(b.new_lens[r])
        if n == 0:
            continue
        k, v = _logical_kv(b, r)
        for t0 in range(0, n, unit_tokens):
            t1 = min(t0 + unit_tokens, n)
            per_head = [np.bitwise_xor.reduce(_words(k[:p + t1, g])) ^ np.bitwise_xor.reduce(_words(v[:p + t1, g]))
                        for g in range(b.Hkv)]
            for _ in range(nsplit):
                out.extend(per_head)
    return np.array(out, np.uint32)


def run_probe(b):
    db = DeviceBatch(b)
    n_units, T = binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                                      b.prefix_lens, b.new_lens, None)
    assert T > 0 and T % 32 == 0
    buf = torch.full((n_units + 3,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    n2, T2 = binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                                  b.prefix_lens, b.new_lens, buf)
    torch.cuda.synchronize()
    assert (n2, T2) == (n_units, T)
    got = buf.cpu().numpy().view(np.uint32)
    assert (got[n_units:] == 0x5A5A5A5A).all(), "wrote past the units"
    return got[:n_units], T


@pytest.mark.parametrize("maker", [lambda: W.ragged_small(7), lambda: W.ragged_small(8, d=64, Hq=4, Hkv=4), lambda: W.shared_system_prompt(keep_logical=True),
                                   W.dynamic_workflow_batch], ids=["ragged", "ragged_d64_mha", "cfg1", "cfg2"])
def test_gather_probe_matches_logical_kv(maker):
    b = maker()
    got, T = run_probe(b)
    want = expected_unit_xor(b, T)
    assert got.shape == want.shape
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, "%d of %d units differ, first %s" % (bad.size, got.size, bad[:8])


def test_gather_probe_capacity_and_dtype_errors():
    b = W.ragged_small(9)
    db = DeviceBatch(b)
    n_units, _ = binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                                      b.prefix_lens, b.new_lens, None)
    small = torch.zeros(max(n_units - 1, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(binding.PbkvError) as e:
        binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                             b.prefix_lens, b.new_lens, small)
    assert e.value.code == -4
    f = W.tiny_fp32()
    df = DeviceBatch(f)
    with pytest.raises(binding.PbkvError) as e:
        binding.gather_probe(df.shape, df.k_new, df.v_new, df.kv_pool, df.block_table,
                             f.prefix_lens, f.new_lens, None)
    assert e.value.code == -3
