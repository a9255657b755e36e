"""Predictor forward (pbkv_predictor_prepare / pbkv_predictor_forward) against the fp64 reference
of App. B, element by element.

Tolerance (absolute, on probabilities): 1e-5 for unit-scale activations, 1e-4 for the peaked case
(logits of a few tens, where the fp32 rounding of a logit, 2^-24 relative, is ~1e-5 absolute).
Derivation: x is bf16 and enters exactly; W_t is
used as hi + lo (two bf16 numbers, relative error 2^-17 = 7.6e-6 per weight), products are exact
in fp32 and sums of d_x = 5120 terms of size ~|x||w| round with 2^-24 per addition, so a
pre-activation of size ~1 carries ~1e-5; the fp32 head (two layers of <= 192 / 64 terms, expf to
an ulp) adds ~1e-6 and the softmax does not amplify (|dp| <= |dlogit| / 2).  Measured: 1e-7 .. 8e-7, peaked case 2e-5."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import predictor_oracle                                   # noqa: E402
from paper_2605_06472_amd import predictor as PR, workloads as W      # noqa: E402
from tests.gpu_util import to_torch                                   # noqa: E402

TOL = 1e-5          # models with unit-scale activations; the peaked case states its own


class DevicePredictor:
    def __init__(self, model, L, max_batch):
        self.m, self.L, self.max_batch = model, L, max_batch
        self.shape = PR.make_shape(model.V, model.d, model.d_x, model.hidden, model.K, L)
        self.nbytes = PR.predictor_workspace_bytes(self.shape, max_batch)
        self.ws = torch.empty(self.nbytes, dtype=torch.uint8, device="cuda")
        self.weights = {n: to_torch(np.ascontiguousarray(getattr(model, n))) for n in PR.WEIGHT_NAMES}
        PR.predictor_prepare(self.shape, self.weights, self.ws, self.nbytes, max_batch)

    def forward(self, b, batch=None):
        n = b.B if batch is None else batch
        x, cur, plen = to_torch(b.x), to_torch(b.cur_agent), to_torch(b.prefix_len)
        pre = to_torch(b.prefix) if self.L > 0 else None
        probs = torch.full((max(n, 1), self.m.K, self.m.V + 1), -1.0, dtype=torch.float32, device="cuda")
        PR.predictor_forward(self.shape, self.ws, self.nbytes, self.max_batch, x, cur, pre, plen, n, probs)
        torch.cuda.synchronize()
        return probs.cpu().numpy().astype(np.float64)[:n] if n else probs.cpu().numpy()


def _check(model, b, got, what, tol=TOL):
    want = predictor_oracle.forward(model, b.x, b.cur_agent, b.prefix, b.prefix_len)
    err = float(np.abs(got - want).max())
    print("%s: max abs err %.2e over %d probabilities" % (what, err, want.size), flush=True)
    assert np.isfinite(got).all()
    assert err <= tol, (what, err)
    assert np.allclose(got.sum(-1), 1.0, atol=1e-5)
    return err


@pytest.mark.parametrize("V,d,d_x,hidden,K,L,B", [
    (8, 64, 5120, 64, 3, 16, 200),        # the benchmark model, several row blocks and a ragged tail
    (5, 32, 64, 12, 1, 4, 1),             # smallest widths, a single request
    (64, 128, 1040, 256, 8, 64, 77),      # largest everything: 8 x 65 outputs, 64 prefix slots, d_x not a multiple of 64
    (3, 64, 272, 7, 2, 0, 33),            # no prefix slots at all; odd hidden width
    (13, 128, 4096, 100, 4, 9, 513),      # one request past a row-block boundary
])
def test_forward_matches_reference(V, d, d_x, hidden, K, L, B):
    m = W.predictor_model(300 + V, V=V, d=d, d_x=d_x, hidden=hidden, K=K)
    b = W.predictor_batch(m, seed=400 + B, B=B, L=max(L, 1))
    if L == 0:
        b.prefix_len[:] = 0
        b.L = 0
    dp = DevicePredictor(m, L, max_batch=B)
    _check(m, b, dp.forward(b), "V=%d d=%d d_x=%d hidden=%d K=%d L=%d B=%d" % (V, d, d_x, hidden, K, L, B))


def test_benchmark_batch_all_rows():
    """The configuration bench.py times: 1024 requests of the 362 779-parameter model."""
    m = W.predictor_model()
    b = W.predictor_batch(m, B=1024, L=16)
    dp = DevicePredictor(m, 16, max_batch=1024)
    got = dp.forward(b)
    _check(m, b, got, "benchmark batch")
    # run to run bit-identical (fixed reduction order); a smaller batch on the same workspace cuts d_x
    # into more slices, so its sums round differently
    assert np.array_equal(dp.forward(b), got)
    sub = W.PredictorBatch(100, 16, b.x[:100], b.cur_agent[:100], b.prefix[:100], b.prefix_len[:100])
    assert np.abs(dp.forward(sub) - got[:100]).max() < 1e-6


def test_peaked_and_degenerate_inputs():
    m = W.predictor_model(77, V=6, d=64, d_x=512, hidden=32, K=3, gain=3.0)     # logits of a few tens, near one-hot outputs
    b = W.predictor_batch(m, seed=78, B=40, L=8, sigma_x=2.0)
    b.prefix_len[:5] = 0                                                          # first invocations
    b.prefix[5, :8] = b.prefix[5, 0]                                              # a prefix of one agent
    b.prefix_len[5] = 8
    dp = DevicePredictor(m, 8, max_batch=64)
    _check(m, b, dp.forward(b), "peaked", tol=1e-4)
    # out-of-range indices are clamped, entries past prefix_len are never read
    junk = W.PredictorBatch(b.B, b.L, b.x, b.cur_agent.copy(), b.prefix.copy(), b.prefix_len.copy())
    for i in range(b.B):
        junk.prefix[i, b.prefix_len[i]:] = 1000 + i
    assert np.array_equal(dp.forward(junk), dp.forward(b))
    junk.cur_agent[0], junk.cur_agent[1] = 99, -7
    clamped = W.PredictorBatch(b.B, b.L, b.x, junk.cur_agent.copy(), b.prefix, b.prefix_len)
    clamped.cur_agent[0], clamped.cur_agent[1] = m.V - 1, 0
    assert np.array_equal(dp.forward(junk), dp.forward(clamped))
    # batch = 0 writes nothing
    assert (dp.forward(b, batch=0) == -1.0).all()


def test_probabilities_feed_the_policy_core():
    """The forward pass' output is a valid forecast for pbkv_policy_forecast (rows sum to 1 within its 1e-6)."""
    from paper_2605_06472_amd import policy as PC
    m = W.predictor_model(91, V=4, d=32, d_x=128, hidden=16, K=2)
    b = W.predictor_batch(m, seed=92, B=3, L=4)
    probs = DevicePredictor(m, 4, max_batch=4).forward(b)
    pol = PC.Policy(num_agents=4, horizon=2, gamma=0.7)
    pol.node_add(1, -1, 2)
    for wf in range(3):
        pol.access(wf, int(b.cur_agent[wf]), [1])
        pol.forecast(wf, probs[wf])
    want = sum(float(probs[wf, 0, int(b.cur_agent[wf])]) for wf in range(3))     # Eq. 1 with A_w(c) = e_{agent}
    assert abs(pol.value(1) - want) < 1e-9
