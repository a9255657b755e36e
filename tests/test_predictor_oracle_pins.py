"""Pins of the predictor reference (oracle/predictor_oracle.py) against what App. B and the
mathematics fix: a hand-worked example, closed forms, invariants, an independent library
implementation (torch float64, scaled_dot_product_attention for the history stream), and a
set of planted mistakes that these pins must reject."""
import json
import math
import os
import types

import numpy as np
import pytest

from paper_2605_06472_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_SRC = os.path.join(os.path.dirname(HERE), "oracle", "predictor_oracle.py")


def _load(src_text=None):
    """The oracle module, optionally from modified source text (for the planted mistakes)."""
    text = open(ORACLE_SRC).read() if src_text is None else src_text
    mod = types.ModuleType("predictor_oracle_under_test")
    exec(compile(text, ORACLE_SRC, "exec"), mod.__dict__)
    return mod


@pytest.fixture(scope="module")
def orc():
    return _load()


def _bf16(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def _example():
    g = json.load(open(os.path.join(HERE, "golden", "predictor_example.json")))
    f = lambda k: np.array(g[k], np.float32)
    ln2 = math.log(2.0)
    m = W.PredictorModel(g["V"], g["d"], g["d_x"], g["hidden"], g["K"], emb=f("emb"), trans=f("trans"),
                         w1=f("w1"), w2=f("w2"), wq=(f("wq_in_units") * ln2 * math.sqrt(2.0)).astype(np.float32),
                         wt=f("wt"), wa=f("wa"), ba=f("ba"), wb=(f("wb_in_units") * ln2).astype(np.float32),
                         bb=(f("bb_in_units") * ln2).astype(np.float32))
    return g, m


def _small_model(seed=5, **kw):
    args = dict(V=5, d=8, d_x=32, hidden=12, K=3)
    args.update(kw)
    return W.predictor_model(seed, **args)


# ---- the pins, as functions of the oracle module so that the mutants can be run through them ----
def pin_worked_example(orc):
    g, m = _example()
    assert np.allclose(orc.graphsage(m.emb, m.trans, m.w1, m.w2), g["H2"], atol=1e-12)
    H2 = np.array(g["H2"], np.float64)
    assert np.allclose(orc.history_attention(H2, m.wq, 0, [1, 0, 1]), g["h_path_request0"], atol=1e-6)
    got = orc.forward(m, _bf16(g["x"]), g["cur_agent"], g["prefix"], g["prefix_len"])
    want = np.array(g["probs_numerators"], np.float64) / np.array(g["probs_denominators"], np.float64)[:, None]
    assert got.shape == (2, 1, 3)
    assert np.allclose(got[:, 0, :], want, atol=2e-6)      # fp32 storage of ln 2 and sqrt 2


def pin_torch_library(orc):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    m = _small_model()
    b = W.predictor_batch(m, seed=6, B=24, L=7)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    H = t(m.emb)
    for w in (m.w1, m.w2):
        H = F.relu(F.linear(torch.cat([H, t(m.trans) @ H], dim=1), t(w)))
    x = t(W.to_f64(b.x))
    want = np.zeros((b.B, m.K, m.V + 1))
    for i in range(b.B):
        cur, n = int(b.cur_agent[i]), int(b.prefix_len[i])
        h_cur = H[cur]
        if n:
            kv = H[torch.from_numpy(b.prefix[i, :n].astype(np.int64))][None, None]
            q = F.linear(h_cur, t(m.wq))[None, None, None]
            h_path = F.scaled_dot_product_attention(q, kv, kv)[0, 0, 0]
        else:
            h_path = torch.zeros(m.d, dtype=torch.float64)
        h_txt = F.relu(F.linear(x[i], t(m.wt)))
        hid = F.relu(F.linear(torch.cat([h_cur, h_path, h_txt]), t(m.wa), t(m.ba)))
        want[i] = F.softmax(F.linear(hid, t(m.wb), t(m.bb)).view(m.K, m.V + 1), dim=-1).numpy()
    got = orc.forward(m, b.x, b.cur_agent, b.prefix, b.prefix_len)
    assert np.allclose(got, want, atol=1e-12)


def pin_graphsage_closed_forms(orc):
    rng = np.random.default_rng(0)
    V, d = 6, 4
    H0 = np.abs(rng.standard_normal((V, d)))
    A = rng.random((V, V))
    A /= A.sum(1, keepdims=True)
    I, Z = np.eye(d), np.zeros((d, d))
    keep_self = np.concatenate([I, Z], axis=1)      # W = [I || 0]
    keep_nbr = np.concatenate([Z, I], axis=1)       # W = [0 || I]
    assert np.allclose(orc.graphsage(H0, A, keep_self, keep_self), H0, atol=1e-14)
    assert np.allclose(orc.graphsage(H0, A, keep_nbr, keep_nbr), A @ A @ H0, atol=1e-14)
    assert np.allclose(orc.graphsage(H0, A, keep_nbr, keep_self), A @ H0, atol=1e-14)
    # the activation clips: a negated embedding with W = [I || 0] gives zero
    assert np.all(orc.graphsage(-H0, A, keep_self, keep_self) == 0)
    # a map that mixes features: one layer is a plain matrix product of the concatenation
    Wm = rng.standard_normal((d, 2 * d))
    one = np.maximum(np.concatenate([H0, A @ H0], axis=1) @ Wm.T, 0)
    assert np.allclose(orc.graphsage(H0, A, Wm, keep_self), one, atol=1e-13)


def pin_attention_closed_forms(orc):
    rng = np.random.default_rng(1)
    V, d = 5, 6
    H2 = rng.standard_normal((V, d))
    wq = rng.standard_normal((d, d))
    # a zero query map is mean pooling (App. B contrasts the attention with it)
    assert np.allclose(orc.history_attention(H2, 0 * wq, 2, [0, 3, 3, 1]), H2[[0, 3, 3, 1]].mean(0), atol=1e-14)
    # a prefix of one agent, however long, returns that agent's representation
    assert np.allclose(orc.history_attention(H2, wq, 1, [4, 4, 4]), H2[4], atol=1e-14)
    # the order of the prefix does not matter
    assert np.allclose(orc.history_attention(H2, wq, 0, [1, 2, 3, 4]), orc.history_attention(H2, wq, 0, [4, 2, 1, 3]), atol=1e-14)
    # two-agent prefix: weights are a logistic function of the score difference / sqrt(d)
    q = wq @ H2[0]
    p1 = 1.0 / (1.0 + math.exp(-(q @ (H2[1] - H2[2])) / math.sqrt(d)))
    assert np.allclose(orc.history_attention(H2, wq, 0, [1, 2]), p1 * H2[1] + (1 - p1) * H2[2], atol=1e-13)
    # empty prefix
    assert np.all(orc.history_attention(H2, wq, 0, []) == 0)
    # the query is W_q h (not W_q^T h): an asymmetric map that reads feature 0 of h and writes feature 1
    wq2 = np.zeros((d, d))
    wq2[1, 0] = 50.0
    Hs = np.zeros((3, d))
    Hs[0, 0] = 1.0          # current agent
    Hs[1, 1] = 1.0          # matches W_q h_cur
    Hs[2, 0] = 1.0          # would match W_q^T h_cur
    assert np.allclose(orc.history_attention(Hs, wq2, 0, [1, 2]), Hs[1], atol=1e-6)


def pin_head_closed_forms(orc):
    m = _small_model(seed=9)
    b = W.predictor_batch(m, seed=10, B=6, L=5)
    # zero output weights: every step's distribution is softmax(b_b) whatever the request
    target = np.random.default_rng(2).random((m.K, m.V + 1)) + 0.05
    target /= target.sum(1, keepdims=True)
    m0 = W.PredictorModel(**{**m.__dict__, "wb": np.zeros_like(m.wb), "bb": np.log(target).reshape(-1).astype(np.float32)})
    got = orc.forward(m0, b.x, b.cur_agent, b.prefix, b.prefix_len)
    assert np.allclose(got, np.broadcast_to(target, got.shape), atol=1e-6)
    # zero hidden layer and bias: hidden = 0, same statement through the second layer's bias only
    m1 = W.PredictorModel(**{**m.__dict__, "wa": np.zeros_like(m.wa), "ba": -np.ones_like(m.ba)})
    got = orc.forward(m1, b.x, b.cur_agent, b.prefix, b.prefix_len)
    want = np.exp(m.bb.astype(np.float64)).reshape(m.K, m.V + 1)
    want /= want.sum(1, keepdims=True)
    assert np.allclose(got, np.broadcast_to(want, got.shape), atol=1e-12)
    # a first layer that copies one stream at a time: hidden = the chosen slice of z, checked through
    # a second layer that reads it back as logits (K = 1, V + 1 = hidden = d)
    d = 4
    mm = W.predictor_model(11, V=d - 1, d=d, d_x=8, hidden=d, K=1)
    bb = W.predictor_batch(mm, seed=12, B=5, L=4)
    H2 = orc.graphsage(mm.emb, mm.trans, mm.w1, mm.w2)
    for stream in range(3):
        wa = np.zeros((d, 3 * d), np.float32)
        wa[:, stream * d:(stream + 1) * d] = np.eye(d)
        mc = W.PredictorModel(**{**mm.__dict__, "wa": wa, "ba": np.zeros(d, np.float32),
                                 "wb": np.eye(d, dtype=np.float32), "bb": np.zeros(d, np.float32)})
        got = orc.forward(mc, bb.x, bb.cur_agent, bb.prefix, bb.prefix_len)
        for i in range(bb.B):
            cur, n = int(bb.cur_agent[i]), int(bb.prefix_len[i])
            if stream == 0:
                h = H2[cur]
            elif stream == 1:
                h = orc.history_attention(H2, mm.wq, cur, list(bb.prefix[i, :n]))
            else:
                h = np.maximum(mm.wt.astype(np.float64) @ W.to_f64(bb.x[i]), 0)
            e = np.exp(np.maximum(h, 0))
            assert np.allclose(got[i, 0], e / e.sum(), atol=1e-12), (stream, i)


def pin_invariants(orc):
    m = _small_model(seed=13)
    b = W.predictor_batch(m, seed=14, B=20, L=6)
    got = orc.forward(m, b.x, b.cur_agent, b.prefix, b.prefix_len)
    assert np.all(got >= 0) and np.allclose(got.sum(-1), 1.0, atol=1e-14)
    # relabelling the agents permutes the agent outputs (END stays last) and nothing else
    perm = np.random.default_rng(3).permutation(m.V)          # new index of old agent v is perm[v]
    inv = np.argsort(perm)
    out_rows = np.concatenate([(k * (m.V + 1) + np.concatenate([inv, [m.V]])) for k in range(m.K)])
    mp = W.PredictorModel(**{**m.__dict__, "emb": m.emb[inv], "trans": m.trans[inv][:, inv],
                             "wb": m.wb[out_rows], "bb": m.bb[out_rows]})
    pre = np.where(b.prefix >= 0, perm[np.maximum(b.prefix, 0)], -1).astype(np.int32)
    gp = orc.forward(mp, b.x, perm[b.cur_agent].astype(np.int32), pre, b.prefix_len)
    assert np.allclose(gp[:, :, np.concatenate([perm, [m.V]])], got, atol=1e-13)
    # entries of the prefix array past prefix_len are never read
    junk = b.prefix.copy()
    for i in range(b.B):
        junk[i, b.prefix_len[i]:] = (i * 7) % m.V
    assert np.array_equal(orc.forward(m, b.x, b.cur_agent, junk, b.prefix_len), got)
    # requests are independent: a sub-batch gives the same rows
    sub = [3, 11, 17]
    assert np.array_equal(orc.forward(m, b.x[sub], b.cur_agent[sub], b.prefix[sub], b.prefix_len[sub]), got[sub])


PINS = [pin_worked_example, pin_torch_library, pin_graphsage_closed_forms, pin_attention_closed_forms,
        pin_head_closed_forms, pin_invariants]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(orc, pin):
    pin(orc)


def test_parameter_count_of_the_benchmark_model():
    m = W.predictor_model()
    assert (m.V, m.d, m.d_x, m.hidden, m.K) == (8, 64, 5120, 64, 3)
    assert m.num_params() == 362779                           # "roughly 350K parameters" (Sec. 4.1)
    assert np.allclose(m.trans.sum(1), 1.0, atol=1e-6)


MUTANTS = {
    "dropped_scale": ("/ np.sqrt(d))", ")"),
    "transposed_transition": ("A @ H]", "A.T @ H]"),
    "swapped_concat_halves": ("[H, A @ H]", "[A @ H, H]"),
    "one_layer_only": ("(_f64(w1), _f64(w2))", "(_f64(w1),)"),
    "no_graphsage_activation": ("H = relu(np.concatenate", "H = (np.concatenate"),
    "transposed_query_map": ("_f64(wq) @ H2[cur]", "_f64(wq).T @ H2[cur]"),
    "mean_pooling": ("return alpha @ keys", "return keys.mean(axis=0)"),
    "query_is_not_projected": ("q = _f64(wq) @ H2[cur]", "q = H2[cur]"),
    "no_text_activation": ("h_txt = relu(wt @ x[b])", "h_txt = wt @ x[b]"),
    "stream_order": ("[h_cur, h_path, h_txt]", "[h_path, h_cur, h_txt]"),
    "no_hidden_activation": ("hidden = relu(wa @ z + ba)", "hidden = wa @ z + ba"),
    "dropped_hidden_bias": ("relu(wa @ z + ba)", "relu(wa @ z)"),
    "dropped_output_bias": ("(wb @ hidden + bb)", "(wb @ hidden)"),
    "agent_major_logits": (".reshape(K, V + 1)", ".reshape(V + 1, K).T"),
    "softmax_over_all_steps": ("out[b, k] = softmax(logits[k])", "out[b, k] = softmax(logits.reshape(-1)).reshape(K, V + 1)[k]"),
    "current_agent_joins_prefix": ("prefix[b][:int(prefix_len[b])]]", "prefix[b][:int(prefix_len[b])]] + [cur]"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_rejected(name):
    old, new = MUTANTS[name]
    text = open(ORACLE_SRC).read()
    assert text.count(old) == 1, "mutation site not found exactly once: %r" % old
    mutant = _load(text.replace(old, new))
    failed = []
    for pin in PINS:
        try:
            pin(mutant)
        except AssertionError:
            failed.append(pin.__name__)
        except Exception as e:          # a shape error is a rejection too
            failed.append("%s (%s)" % (pin.__name__, type(e).__name__))
    assert failed, "no pin noticed the planted mistake %s" % name
