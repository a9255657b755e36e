"""Reference forward pass of the workflow predictor (App. B), numpy, fp64.

TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and bench.py's CPU baseline leg.
It shares no code with the HIP path and takes the formulas of App. B in the paper's order
and notation, one request at a time, with no precomputed tables and no reordering:

  (i)   H^(l) = ReLU([H^(l-1) || A H^(l-1)] W^(l)T), l = 1, 2            (GraphSAGE equation)
  (ii)  alpha_i = softmax_i((W_q h_cur)^T H2[v_i] / sqrt(d)), i < t,
        h_path = sum_i alpha_i H2[v_i]                                     (history attention equation)
  (iii) h_txt = ReLU(W_t x)                                                (semantic stream)
  head  [h_cur || h_path || h_txt] -> Linear, ReLU, (dropout: identity at inference) -> Linear
        -> K x (|V|+1) logits -> one softmax per step (multi-step head, Sec. 4.1)

Readings where the paper is silent (listed again in the design notes):
  - the two MLP layers have biases, the other maps have none (their formulas show none);
  - the stream order of the concatenation is (h_cur, h_path, h_txt), as the overview lists them;
  - a workflow at its first invocation has an empty prefix: h_path = 0;
  - logit index k*(|V|+1) + a, END last (the convention of the policy core's forecast input).
All pins of this file are in tests/test_predictor_oracle_pins.py.
"""
import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def _bf16_to_f64(bits):
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def relu(a):
    return np.maximum(a, 0.0)


def softmax(z):
    z = z - np.max(z)
    e = np.exp(z)
    return e / np.sum(e)


def graphsage(emb, trans, w1, w2):
    """H^(2): two propagation layers over the row-normalised transition matrix (App. B, stream (i))."""
    H = _f64(emb)
    A = _f64(trans)
    for W in (_f64(w1), _f64(w2)):
        H = relu(np.concatenate([H, A @ H], axis=1) @ W.T)
    return H


def history_attention(H2, wq, cur, prefix_agents):
    """h_path of one workflow: attention of the current agent's representation over the prefix
    agents' representations (App. B, stream (ii)); zero vector for an empty prefix."""
    d = H2.shape[1]
    if len(prefix_agents) == 0:
        return np.zeros(d)
    q = _f64(wq) @ H2[cur]
    keys = H2[np.asarray(prefix_agents, dtype=np.int64)]
    alpha = softmax(keys @ q / np.sqrt(d))
    return alpha @ keys


def forward(model, x_bits, cur_agent, prefix, prefix_len):
    """probs[b][k][a]: distribution of the (k+1)-th next invocation of request b over the |V|
    agents and END (last).  `model` has the attributes of workloads.PredictorModel; x_bits is
    the bf16 hidden state [B][d_x]; prefix[b][:prefix_len[b]] are the agents invoked before the
    current one, oldest first."""
    V, K = model.V, model.K
    H2 = graphsage(model.emb, model.trans, model.w1, model.w2)
    wt, wa, ba, wb, bb = _f64(model.wt), _f64(model.wa), _f64(model.ba), _f64(model.wb), _f64(model.bb)
    x = _bf16_to_f64(x_bits)
    B = x.shape[0]
    out = np.zeros((B, K, V + 1))
    for b in range(B):
        cur = int(cur_agent[b])
        h_cur = H2[cur]
        h_path = history_attention(H2, model.wq, cur, [int(v) for v in prefix[b][:int(prefix_len[b])]])
        h_txt = relu(wt @ x[b])
        z = np.concatenate([h_cur, h_path, h_txt])
        hidden = relu(wa @ z + ba)
        logits = (wb @ hidden + bb).reshape(K, V + 1)
        for k in range(K):
            out[b, k] = softmax(logits[k])
    return out
