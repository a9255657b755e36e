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


def attention_unit(db):
    """Suffix tokens per work unit of the attention launch this batch will get (asked of the
    library through the size query of the gather diagnostic; 0 for fp32 batches)."""
    b = db.b
    if b.dtype != "bf16":
        return 0
    return binding.gather_probe(db.shape, db.k_new, db.v_new, db.kv_pool, db.block_table,
                                b.prefix_lens, b.new_lens, None)[1]


def sample_rows(b: W.Batch, per_request=6, unit=64, seed=0, max_boundaries=24):
    """Packed row indices: first and last row, the rows on both sides of boundaries between work
    units of `unit` suffix tokens (all of them up to max_boundaries, else a seeded choice that
    keeps the first and the last), the rows around the 32-token sub-blocks of the first and last
    unit, and per_request random rows of every request."""
    rng = np.random.default_rng(seed)
    unit = unit or 64
    rows, off = [], 0
    for r in range(b.B):
        n = int(b.new_lens[r])
        if n:
            cand = {0, n - 1}
            bounds = list(range(unit, n, unit))
            if len(bounds) > max_boundaries:
                keep = rng.choice(len(bounds) - 2, max_boundaries - 2, replace=False) + 1
                bounds = [bounds[0], bounds[-1]] + [bounds[int(i)] for i in keep]
            for x in bounds:
                cand.update((x - 1, x))
            for x in (31, 32, (n - 1) // unit * unit + 31, (n - 1) // unit * unit + 32):
                if 0 <= x < n:
                    cand.add(x)
            cand.update(int(x) for x in rng.integers(0, n, per_request))
            rows.extend(off + c for c in sorted(cand))
        off += n
    return np.array(sorted(set(rows)), np.int64)


TOL = {"bf16": (2e-2, 1e-2), "f32": (1e-5, 1e-5)}    # (max abs error, relative L2 error)
# The stress runs with Q scaled x8 (peaked softmax, outputs of order 1) get one and a half times the
# absolute bound.  The kernel folds log2(e)/sqrt(d) into Q and rounds the product once to bf16; that moves a
# score by sigma = 2^-9/sqrt(3) * |c q * k|_2, about 0.0065 log2 units at x8 (0.0008 at x1), and in a
# softmax that two keys dominate an output moves by up to ln2 * |delta_1 - delta_2| * 1/4 * |v_1 - v_2|,
# about 0.03 for a 5-sigma pair and |v_1 - v_2| = 4.  A CPU emulation of the kernel's roundings on
# 96 rows of the long-history batch gives 1.2e-2 with that rounding and 6e-3 without it (then the
# final rounding of outputs near 3 is what is left); over the 3.5 million elements the test compares
# the tail reaches 2.0e-2 - 2.2e-2.  (A build that keeps Q exact and multiplies every score by the
# scale instead is 2.2 % slower on every configuration; by the emulation it would leave 6e-3.  The
# kernel keeps the folded scale.)  The relative L2 bound is the same as for the plain runs.
PEAKED_ATOL = 3e-2


def assert_close(got, want, dtype, what="", atol=None):
    atol0, rtol = TOL[dtype]
    atol = atol0 if atol is None else atol
    err = np.abs(got - want).max()
    rel = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)
    assert np.isfinite(got).all(), what
    assert err <= atol, "%s max abs err %.3e > %.1e" % (what, err, atol)
    assert rel <= rtol, "%s rel L2 err %.3e > %.1e" % (what, rel, rtol)
    return err, rel
