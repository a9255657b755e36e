/*
 * pbkv_predictor.h -- C boundary of the workflow predictor's forward pass (GPU work).
 *
 * The predictor of PBKV (Sec. 4.1, App. B of arxiv 2605.06472) turns the state of an
 * active workflow -- the agents invoked so far and the post-norm hidden state x of the
 * last prefill token -- into K distributions over the next invocations, which are the
 * `probs` input of pbkv_policy_forecast (pbkv_policy.h).  Three streams feed a two-layer
 * head (App. B):
 *   (i)   H^(l) = ReLU([H^(l-1) || A H^(l-1)] W^(l)T), l = 1, 2, over the row-normalised
 *         transition matrix A; h_cur = H^(2)[v_t]
 *   (ii)  h_path = sum_i alpha_i H^(2)[v_i], alpha = softmax_i((W_q h_cur)^T H^(2)[v_i] / sqrt(d))
 *         over the prefix agents v_1 .. v_{t-1} (zero vector for an empty prefix)
 *   (iii) h_txt = ReLU(W_t x)
 *   head  [h_cur || h_path || h_txt] -> Linear(+bias), ReLU -> Linear(+bias) -> K x (|V|+1)
 *         logits -> one softmax per step; output index k*(|V|+1) + agent, END last.
 * Dropout is the identity at inference.
 *
 * Two calls.  pbkv_predictor_prepare runs whenever the weights change: everything that does
 * not depend on the request (H^(2), the |V| x |V| table of attention scores between agents,
 * transposed head weights, W_t split into two bf16 parts whose sum carries 16 significand
 * bits) goes into a caller-owned device workspace.  pbkv_predictor_forward runs per batch:
 * the x-projection on the matrix cores (bf16 x, fp32 accumulation, split over the batch and
 * over d_x so that the whole chip takes part), then eight requests per work-group for the history
 * attention, the head and the softmaxes, all in fp32.
 *
 * Conventions as in pbkv.h: plain pointers, every buffer is DEVICE memory owned by the
 * caller, `stream` is a hipStream_t passed as void* (NULL = default stream), calls validate
 * on the host, enqueue and return; return value PBKV_OK or a negative pbkv_status with the
 * text in pbkv_last_error().  The library allocates nothing here.  Indices in cur_agent /
 * prefix live in device memory and cannot be validated by the host: the kernels clamp them
 * to [0, |V|-1] and prefix_len to [0, max_prefix].
 */
#ifndef PBKV_PREDICTOR_H
#define PBKV_PREDICTOR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pbkv_predictor_shape {
    int32_t num_agents;   /* |V| in [1, 64]                                             */
    int32_t d;            /* width of the agent representations: 32, 64 or 128          */
    int32_t d_x;          /* width of x: a multiple of 16, at least 64                  */
    int32_t hidden;       /* width of the head's hidden layer, [1, 256]                 */
    int32_t horizon;      /* K in [1, 8]                                                */
    int32_t max_prefix;   /* prefix slots per request (row pitch of `prefix`), [0, 64]  */
} pbkv_predictor_shape;

/* fp32, row-major, 16-byte aligned device arrays (App. B notation) */
typedef struct pbkv_predictor_weights {
    const float *emb;     /* H^(0) [num_agents][d]                                       */
    const float *trans;   /* A     [num_agents][num_agents]                              */
    const float *w1;      /* W^(1) [d][2d]                                               */
    const float *w2;      /* W^(2) [d][2d]                                               */
    const float *wq;      /* W_q   [d][d]                                                */
    const float *wt;      /* W_t   [d][d_x]                                              */
    const float *wa;      /* head layer 1 [hidden][3d], input order (h_cur, h_path, h_txt) */
    const float *ba;      /* [hidden]                                                    */
    const float *wb;      /* head layer 2 [horizon*(num_agents+1)][hidden]               */
    const float *bb;      /* [horizon*(num_agents+1)]                                    */
} pbkv_predictor_weights;

/* Bytes of device workspace for batches of up to max_batch requests (0 on a bad shape). */
int64_t pbkv_predictor_workspace_bytes(const pbkv_predictor_shape *shape, int32_t max_batch);

/* Fills the workspace from the weights.  `workspace` is 256-byte aligned device memory of at
 * least pbkv_predictor_workspace_bytes(shape, max_batch) bytes; the weights are not needed
 * once the stream has run this call. */
int pbkv_predictor_prepare(const pbkv_predictor_shape *shape, const pbkv_predictor_weights *weights,
                           void *workspace, int64_t workspace_bytes, int32_t max_batch, void *stream);

/* probs[b][k][a] for b < batch (fp32, [batch][horizon][num_agents+1]).
 *   x          [batch][d_x] bf16
 *   cur_agent  [batch] int32              v_t
 *   prefix     [batch][max_prefix] int32  v_1 .. v_{t-1}, oldest first (may be NULL if max_prefix is 0)
 *   prefix_len [batch] int32              t - 1
 * `workspace` must have been prepared with the same shape and a max_batch >= batch; calls
 * that share a workspace must not overlap in time (they share its partial-sum area).
 * batch = 0 is a no-op. */
int pbkv_predictor_forward(const pbkv_predictor_shape *shape, void *workspace, int64_t workspace_bytes,
                           int32_t max_batch, const void *x, const int32_t *cur_agent,
                           const int32_t *prefix, const int32_t *prefix_len, int32_t batch,
                           float *probs, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PBKV_PREDICTOR_H */
