"""Contiguous brute-force attention used to pin the oracle.

Independent of the oracle: it works on the per-request K/V kept *before*
paging (never sees the pool or the block table) and is written with library
routines (numpy matmul, scipy softmax / logsumexp) instead of explicit loops.
"""
import numpy as np
from scipy.special import logsumexp, softmax

from paper_2605_06472_amd.workloads import to_f64


def attention(batch):
    """Returns out [N,Hq,d] float64 and lse [N,Hq] from batch.logical_k / logical_v."""
    G = batch.Hq // batch.Hkv
    q = to_f64(batch.q)
    outs, lses = [], []
    off = 0
    for r in range(batch.B):
        p, n = int(batch.prefix_lens[r]), int(batch.new_lens[r])
        K = to_f64(batch.logical_k[r])            # [p+n, Hkv, d]
        V = to_f64(batch.logical_v[r])
        assert K.shape[0] == p + n
        o = np.zeros((n, batch.Hq, batch.d))
        l = np.zeros((n, batch.Hq))
        visible = np.arange(p + n)[None, :] <= (p + np.arange(n))[:, None]
        for h in range(batch.Hq):
            s = q[off:off + n, h] @ K[:, h // G].T / np.sqrt(batch.d)
            s = np.where(visible, s, -np.inf)
            o[:, h] = softmax(s, axis=1) @ V[:, h // G]
            l[:, h] = logsumexp(s, axis=1)
        outs.append(o)
        lses.append(l)
        off += n
    return np.concatenate(outs), np.concatenate(lses)
