"""Helpers for the GPU parity tests: move a synthetic batch to the device and call the
HIP path through the C boundary.  No arithmetic of the method happens here."""
import numpy as np
import torch

from paper_2605_06472_amd import binding
from paper_2605_06472_amd import workloads as W


def to_torch(a, device="cuda", pin=False):
    """numpy (float32, uint16 bf16 bits, int32) -> torch tensor of the matching dtype."""
    if a.dtype == np.uint16:
        t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(a)
    if device == "cpu":
        return t.pin_memory() if pin else t
    return t.to(device)


def to_numpy(t):
    """device tensor -> numpy (bf16 comes back as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


class DeviceBatch:
    def __init__(self, b: W.Batch):
        self.b = b
        self.shape = binding.make_shape(b.B, b.Hq, b.Hkv, b.d, b.P, b.num_pages, b.max_pages, b.dtype)
        self.q = to_torch(b.q)
        self.k_new = to_torch(b.k_new)
        self.v_new = to_torch(b.v_new)
        self.kv_pool = to_torch(b.kv_pool)
        self.block_table = to_torch(b.block_table)
        self.out = torch.zeros_like(self.q)
        self.host_pages = to_torch(b.host_pages, "cpu", pin=True) if b.host_pages is not None else None

    def sub_shape(self, nreq):
        b = self.b
        return binding.make_shape(nreq, b.Hq, b.Hkv, b.d, b.P, b.num_pages, b.max_pages, b.dtype)

    def prefill(self, stream=None, out=None):
        b = self.b
        binding.prefix_prefill(self.shape, self.q, self.k_new, self.v_new, self.kv_pool,
                               self.block_table, b.prefix_lens, b.new_lens,
                               self.out if out is None else out, stream)

    def append(self, stream=None):
        b = self.b
        binding.append_kv(self.shape, self.k_new, self.v_new, self.kv_pool, self.block_table,
                          b.prefix_lens, b.new_lens, stream)

    def swap_in(self, stream=None):
        binding.swap_in_pages(self.shape, self.host_pages, self.b.swap_page_ids, self.kv_pool, stream)

    def out_f64(self, out=None):
        return W.to_f64(to_numpy(self.out if out is None else out))


def sample_rows(b: W.Batch, per_request=6, tile=64, seed=0):
    """Packed row indices: first, last, tile-boundary and random rows of every request."""
    rng = np.random.default_rng(seed)
    rows, off = [], 0
    for r in range(b.B):
        n = int(b.new_lens[r])
        if n:
            cand = {0, n - 1, min(tile - 1, n - 1), min(tile, n - 1), (n // tile) * tile - 1 if n >= tile else 0,
                    min((n // tile) * tile, n - 1)}
            cand.update(int(x) for x in rng.integers(0, n, per_request))
            rows.extend(off + c for c in sorted(cand))
        off += n
    return np.array(sorted(set(rows)), np.int64)


TOL = {"bf16": (2e-2, 1e-2), "f32": (1e-5, 1e-5)}    # (max abs error, relative L2 error)


def assert_close(got, want, dtype, what=""):
    atol, rtol = TOL[dtype]
    err = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert np.isfinite(got).all(), what
    assert err <= atol, "%s max abs err %.3e > %.1e" % (what, err, atol)
    assert rel <= rtol, "%s rel L2 err %.3e > %.1e" % (what, rel, rtol)
    return err, rel
