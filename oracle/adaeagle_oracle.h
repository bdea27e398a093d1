/*
 * CPU oracle for the AdaEAGLE speculative decode step (arxiv 2412.18910).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-accumulator fp32
 * implementation of what the paper's step computes: target verify (Eq. 1),
 * EAGLE-style sequential drafting (Eq. 2, Sec. 2.2), LDLP draft-length
 * prediction (Eq. 3), the acceptance rule (Sec. 2.1 for temperature > 0,
 * Sec. 3.1 footnote for greedy) and the loop of Algorithm 1.  It shares no
 * code with the HIP library and must never be reached from the product path;
 * only tests, the smoke check and the CPU-baseline leg of the benchmark load it.
 *
 * Precision: the paper ran in FP32 (Sec. 4.1), so activations and
 * accumulators are float, summed in ascending index order with one
 * accumulator per output and no FMA contraction.  Building with
 * -DORC_ACC_DOUBLE switches every accumulator to double (used by tests to
 * bound the fp32 summation error).  The T>0 acceptance arithmetic (softmax,
 * ratio, residual, prefix sums) is always double.
 *
 * Parity pins (tests/test_oracle_*.py): block verify == sequential one-row
 * forwards (bit-exact), greedy speculative output == autoregressive output,
 * rejection sampling reproduces the target law (chi-square + worked example),
 * Eq. 3 round/clamp table, attention/RoPE/RMSNorm special cases, and a
 * float64 library re-expression of the whole forward at the tiny config.
 * Unpinned: behaviour of trained EAGLE/LDLP checkpoints (none available);
 * the draft layer is a standard pre-norm Llama-style layer with both RMSNorms, an fc with bias
 * over [feature ; embedding] and no norm on its output (the paper does not spell these out).
 */
#ifndef ADAEAGLE_ORACLE_H
#define ADAEAGLE_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_BF16 = 0, ORC_FP32 = 1 };

typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base, rms_eps;
  int32_t wdtype;        /* ORC_BF16: matrices are bf16 bit patterns (uint16) and the KV
                            list holds bf16-rounded values; ORC_FP32: everything float */
  int32_t k_max;         /* upper clamp of Eq. 3 */
  int32_t n_ctx_max;     /* capacity of the KV lists */
  int32_t ldlp_in_mode;  /* 0: input [e ; f] (2d, Sec. 3.2)   1: f only (d) */
  int32_t ldlp_hidden, ldlp_n_res;
  float temperature;     /* 0 => greedy */
  int32_t ddd_enabled;   /* AdaEAGLE-DDD (Sec. 3.4): keep drafting past the predicted length ... */
  float ddd_threshold;   /* ... while the draft sequence's log-probability is >= this value */
  int32_t ldlp_cls;      /* 0: Eq. 3 (scalar, round, clamp)   1: argmax over k_max+1 class scores
                            (classification variant of the Sec. 4.3 ablation) */
} orc_config;

/* One decoder layer: matrices row-major [out, in] in cfg.wdtype, norm gains float[d]. */
typedef struct {
  const float *attn_norm;
  const void *wq, *wk, *wv, *wo;
  const float *ffn_norm;
  const void *w_gate, *w_up, *w_down;
} orc_layer;

typedef struct {
  const void *tok_emb;       /* [V, d] */
  const float *final_norm;   /* [d] */
  const void *lm_head;       /* [V, d] */
  const orc_layer *layers;   /* n_layers entries */
  orc_layer draft_layer;     /* the single EAGLE-style layer */
  const void *draft_fc_w;    /* [d, 2d], columns = [feature ; embedding] */
  const float *draft_fc_b;   /* [d] or NULL */
  const void *ldlp_w_in;     /* [h, 2d] or [h, d] */
  const float *ldlp_b_in;    /* [h] */
  const void *ldlp_w_res;    /* [n_res, h, h] or NULL */
  const float *ldlp_b_res;   /* [n_res, h] or NULL */
  const float *ldlp_w_out;   /* [h]; ldlp_cls: [k_max+1, h] */
  const float *ldlp_b_out;   /* [1]; ldlp_cls: [k_max+1] */
} orc_weights;

typedef struct orc_model orc_model;

/* Weights are borrowed (must outlive the model).  Returns NULL on bad config. */
orc_model *orc_create(const orc_config *cfg, const orc_weights *w);
void orc_destroy(orc_model *m);

/* Alg. 1 first iteration: run the prompt through the target (and the draft head for
 * every slot whose next token is known), leave pending = first generated token. */
int orc_prefill(orc_model *m, const int32_t *ids, int n);

/* Install externally generated K/V rows (float, [n][n_kv_heads*head_dim]) for
 * layer `layer` (n_layers = the draft layer) at slots 0..n-1. */
int orc_kv_import(orc_model *m, int layer, const float *k, const float *v, int n);
/* Declare the state after an accept: n cached tokens, `pending` bonus token,
 * one valid feature row (position n) and the token at position n. */
int orc_set_state(orc_model *m, int kv_len, int32_t last_tok, int32_t pending, const float *feat);

/* Eq. 3.  y_out (nullable) receives the raw scalar before rounding (ldlp_cls: the winning
 * class score; the lowest length wins ties). */
int orc_ldlp(orc_model *m, int *k_out, float *y_out);
/* Eq. 2: catch-up over newly validated slots, then chain to k tokens.  With ddd_enabled
 * (Sec. 3.4, 4.2) the head exits before token s iff s > k AND the log-probability of the
 * s-1 tokens drafted so far is below ddd_threshold, so at least one token is drafted and
 * the longer of the two lengths is kept; never more than k_max tokens.
 * override_ids[i] >= 0 replaces the i-th emitted token (nullable).
 * u_draft[i] in [0,1) drives sampling of the i-th token when temperature > 0. */
int orc_draft(orc_model *m, int k, const int32_t *override_ids, const double *u_draft,
              int32_t *ids_out);
/* Eq. 1, forward part.  block_ids NULL => [pending, current draft]. */
int orc_verify(orc_model *m, const int32_t *block_ids, int n_rows);
/* Acceptance + rollback.  u = NULL for greedy, else n_rows uniforms:
 * u[i] (i < k) tests draft token i+1, u[k] draws the bonus / resample. */
int orc_accept(orc_model *m, const double *u, int *n_accepted, int32_t *bonus);

/* ldlp -> draft -> verify -> accept.  k_force >= 0 bypasses the LDLP result. */
int orc_step(orc_model *m, int k_force, const int32_t *override_ids, const double *u_draft,
             const double *u_accept, int *k_out, int *n_accepted, int32_t *tokens_out /*[k_max+1]*/);

/* Plain autoregressive greedy decoding from the current state (definition of the
 * sequence a lossless greedy speculative run must reproduce). */
int orc_ar_greedy(orc_model *m, int n_tokens, int32_t *out);

int orc_kv_len(const orc_model *m);
int orc_last_draft_len(const orc_model *m);      /* tokens actually drafted by the last orc_draft */
double orc_draft_logprob(const orc_model *m);    /* log-probability of that draft sequence */
int32_t orc_pending(const orc_model *m);
const float *orc_logits(const orc_model *m, int row);        /* [V] of the last verify */
const float *orc_feature(const orc_model *m, int row);       /* [d] */
const float *orc_draft_logits(const orc_model *m, int i);    /* [V] behind draft token i */
const float *orc_kv_row(const orc_model *m, int layer, int which /*0=K,1=V*/, int slot);

/* Stand-alone pieces exposed so tests can pin them individually. */
void orc_rmsnorm(const float *x, const float *g, int d, float eps, float *out);
void orc_rope(float *x, int n_heads, int head_dim, int pos, float base);
void orc_attention_row(const float *q, const float *k, const float *v, int n_keys,
                       int n_heads, int n_kv_heads, int head_dim, int kv_stride, float *out);
int orc_round_clamp(float y, int k_max);
float orc_bf16_round(float x);
int orc_argmax(const float *x, int n);
/* Sec. 2.1 rule on explicit logits; same argument meaning as orc_accept. */
int orc_accept_sample(const float *target_logits, const float *draft_logits, int vocab, int k,
                      const int32_t *draft_ids, double temperature, const double *u,
                      int *n_accepted, int32_t *bonus);
int orc_accept_greedy(const float *target_logits, int vocab, int k, const int32_t *draft_ids,
                      int *n_accepted, int32_t *bonus);
int32_t orc_sample_inverse_cdf(const double *q, int n, double u);
/* LDLP training criterion (Sec. 3.3): mean over n pairs of |pred - truth|, scaled by lambda
 * where pred < truth (predicting too short costs a target forward, too long only draft steps). */
double orc_ldlp_loss(const float *pred, const int32_t *truth, int n, double lambda);

#ifdef __cplusplus
}
#endif
#endif
