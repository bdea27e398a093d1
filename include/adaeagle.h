/*
 * libadaeagle -- C ABI of the AdaEAGLE speculative decode step on one AMD MI355X
 * (gfx950).  The step follows arxiv 2412.18910: a Lightweight Draft Length
 * Predictor chooses the draft length k (Eq. 3), an EAGLE-style draft head chains k
 * cached forwards (Eq. 2, Sec. 2.2), the target verifies the (k+1)-row block in one
 * forward against its KV cache (Eq. 1), the acceptance rule runs (Sec. 2.1; greedy
 * "validated prefix" of Sec. 3.1) and the KV cache is rolled back; Algorithm 1 is the
 * loop over ae_step.
 *
 * Conventions
 *  - All functions return AE_OK (0) or a negative ae_status; nothing throws or aborts.
 *    ae_last_error() gives a human-readable reason (NULL ctx: reason of the last
 *    failed ae_init on this thread).
 *  - One ae_ctx = one sequence on one HIP stream.  A ctx is not thread-safe; calls
 *    on one ctx must not overlap.  Distinct ctxs are independent.
 *  - "host" / "device" below says where a pointer must live.  Weights and the stream
 *    are owned by the caller and must outlive the ctx; with AE_BF16 the ctx keeps its
 *    own re-tiled copy of every matrix (made in ae_init, 2 bytes per parameter), so
 *    the caller's copies are only read during ae_init and by the embedding lookup.
 *    Everything else (KV cache, activations, logits, scratch) is owned by the ctx.
 *  - Output arrays are caller-owned host memory, filled before the call returns
 *    (such calls synchronise the stream).
 *  - Token positions in the paper are 1-based; cache slots and rotary positions
 *    here are 0-based: token t_{s+1} lives in slot s.  kv_len = n = number of tokens
 *    whose K/V are cached; the pending token (last bonus) is t_{n+1}, not yet cached.
 *  - Matrices are row-major [out_features, in_features] in cfg.dtype (bf16 bit
 *    patterns or float); every 1-D vector (norm gains, biases, LDLP output row)
 *    is float.
 *  - Shapes: head_dim in {64, 128}; 1 <= k_max <= 15; with AE_BF16 every matrix
 *    needs out_features % 16 == 0 and in_features % 256 == 0 (else AE_EUNSUPPORTED).
 */
#ifndef ADAEAGLE_H
#define ADAEAGLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ae_ctx ae_ctx;

typedef enum {
  AE_OK = 0,
  AE_EINVAL = -1,       /* argument out of range (k, rows, ids, capacity, NULL) */
  AE_ESTATE = -2,       /* call not allowed in the current state of the sequence */
  AE_ENOMEM = -3,       /* device or host allocation failed */
  AE_EHIP = -4,         /* a HIP runtime call failed; see ae_last_error */
  AE_EUNSUPPORTED = -5  /* shape or option outside what the kernels implement */
} ae_status;

typedef enum { AE_BF16 = 0, AE_FP32 = 1 } ae_dtype;

typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base, rms_eps;
  int32_t dtype;         /* ae_dtype of matrices and of the KV cache */
  int32_t k_max;         /* upper clamp of Eq. 3; verify blocks have <= k_max+1 rows */
  int32_t n_ctx_max;     /* KV capacity in tokens (context + generated + k_max + 1) */
  int32_t ldlp_in_mode;  /* 0: LDLP input [e ; f] (Sec. 3.2)   1: f only */
  int32_t ldlp_hidden;   /* width h of the LDLP hidden layers (<= 1024) */
  int32_t ldlp_n_res;    /* residual h->h blocks between input and output layer */
  float temperature;     /* 0: greedy (Sec. 3.1); > 0: rejection sampling (Sec. 2.1) */
  int32_t ddd_enabled;   /* AdaEAGLE-DDD exit rule (Sec. 3.4, 4.2) */
  float ddd_threshold;   /* log-probability threshold of that rule (the paper picks -0.6) */
  int32_t ldlp_cls;      /* 0: LDLP regresses a scalar, rounded and clamped (Eq. 3)
                            1: classification over the lengths 0..k_max (the "w/ Cls"
                               ablation of Sec. 4.3): k = argmax of k_max+1 scores */
} ae_config;

/* One pre-norm Llama-style decoder layer (device pointers). */
typedef struct {
  const float *attn_norm;                       /* [d] */
  const void *wq, *wk, *wv, *wo;                /* [H*hd,d] [Hkv*hd,d] [Hkv*hd,d] [d,H*hd] */
  const float *ffn_norm;                        /* [d] */
  const void *w_gate, *w_up, *w_down;           /* [f,d] [f,d] [d,f] */
} ae_layer_w;

/* All device pointers.  The draft head reuses tok_emb and lm_head (Sec. 2.2). */
typedef struct {
  const void *tok_emb;        /* [V, d] */
  const float *final_norm;    /* [d] */
  const void *lm_head;        /* [V, d] */
  const ae_layer_w *layers;   /* HOST array of n_layers entries holding device pointers */
  ae_layer_w draft_layer;     /* the one EAGLE-style layer */
  const void *draft_fc_w;     /* [d, 2d]; input columns = [target feature ; token embedding] */
  const float *draft_fc_b;    /* [d] or NULL */
  const void *ldlp_w_in;      /* [h, 2d] (in_mode 0) or [h, d] */
  const float *ldlp_b_in;     /* [h] */
  const void *ldlp_w_res;     /* [n_res, h, h] or NULL */
  const float *ldlp_b_res;    /* [n_res, h] or NULL */
  const float *ldlp_w_out;    /* [h]; with ldlp_cls: [k_max+1, h] */
  const float *ldlp_b_out;    /* [1]; with ldlp_cls: [k_max+1] */
} ae_weights;

/* Validates cfg, re-tiles bf16 matrices, allocates the KV cache and work buffers on the
 * current device, and binds the ctx to `hip_stream` (a hipStream_t; NULL = the default
 * stream).  *out is NULL on failure. */
int ae_init(const ae_config *cfg, const ae_weights *w, void *hip_stream, ae_ctx **out);
void ae_free(ae_ctx *ctx);
const char *ae_last_error(const ae_ctx *ctx);

/* First iteration of Algorithm 1 (k = 0, T = prompt): runs the n prompt tokens (host
 * ids) through the target and through the draft head for every slot whose next token is
 * known; leaves kv_len = n and pending = first new token.  Prompts of up to 16 tokens go through
 * the decode kernels as one block; longer bf16 prompts take the dense pass
 * (matrix-core bound GEMMs over chunks of up to chunk_rows rows, causal attention straight
 * off the cache; the draft head only needs its K/V rows there).  Both give the same state
 * up to rounding order. */
int ae_prefill(ae_ctx *ctx, const int32_t *prompt_ids, int n);

/* How ae_prefill runs.  mode: AE_PREFILL_AUTO (default, rule above), AE_PREFILL_BLOCKS
 * (always the 16-row decode kernels) or AE_PREFILL_DENSE (always the dense pass;
 * AE_EUNSUPPORTED for fp32 weights).  chunk_rows: rows per dense pass, a multiple of 128
 * in [128, 8192], or 0 to keep the current value (default 2048). */
enum { AE_PREFILL_AUTO = 0, AE_PREFILL_BLOCKS = 1, AE_PREFILL_DENSE = 2 };
int ae_set_prefill_mode(ae_ctx *ctx, int mode, int chunk_rows);

/* Test / benchmark set-up: install K and V rows (host float [n][n_kv_heads*head_dim],
 * converted to the cache dtype) for layer `layer` (n_layers = the draft layer) at
 * slots 0..n-1 ...                                                                    */
int ae_kv_import(ae_ctx *ctx, int layer, const float *k, const float *v, int n);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same import as ae_kv_import, staged
 * through a fixed array that lives in the library's device image instead of a temporary
 * allocation.  Calls no hipMalloc / hipFree.  Limit: 2 * n * n_kv_heads * head_dim <=
 * AE_KV_IMPORT_STATIC_MAX_FLOATS (8 MiB of staging per GPU, held until the process ends),
 * else AE_EINVAL; import longer caches with ae_kv_import.  All contexts on one GPU share
 * that array: calls to this function that overlap in time on the same GPU race (calls on
 * one thread, one after the other, are fine: each returns after its kernel has finished). */
#define AE_KV_IMPORT_STATIC_MAX_FLOATS (2 * 1024 * 1024)
int ae_kv_import_static(ae_ctx *ctx, int layer, const float *k, const float *v, int n);
/* ... and declare the state right after an accept: kv_len cached tokens, the token in
 * the last slot, the pending bonus token and the feature row (host float [d]) of the
 * last slot.  The draft cache is taken to be valid for slots 0..kv_len-2. */
int ae_set_state(ae_ctx *ctx, int kv_len, int32_t last_tok, int32_t pending, const float *feat);

/* Eq. 3: k = min(k_max, max(0, Round(MLP(e, f)))), round half to even.  e is the
 * embedding of the last validated token, f its post-final-norm hidden state.
 * y_out (nullable) receives the scalar before rounding.  With cfg.ldlp_cls the MLP's last
 * layer scores the lengths 0..k_max, k is the best-scoring length (the lowest on ties)
 * and y_out its score. */
int ae_ldlp(ae_ctx *ctx, int *k_out, float *y_out);

/* Training criterion of the LDLP (Sec. 3.3, the asymmetric L1 loss) as an evaluation
 * function: mean over the n pairs of lambda*|pred - truth| where pred < truth (a short draft
 * costs a whole target forward) and |pred - truth| otherwise; pred holds raw predictions
 * (regression output before rounding, or chosen lengths), truth the optimal lengths (host
 * arrays).  Computed on the device in float64 with a fixed-shape reduction; *out = 0 for
 * n = 0.  Training itself is not part of this library. */
int ae_ldlp_loss(ae_ctx *ctx, const float *pred, const int32_t *truth, int n, double lambda, double *out);

/* Eq. 2: draft catch-up over the newly validated slots, then a chain of k-1 further
 * one-row forwards; emits k tokens (argmax of the shared LM head, lowest id on ties;
 * with temperature > 0 inverse-CDF samples driven by u_draft[i] in [0,1)).
 * override_ids (host, nullable, k_max entries when ddd_enabled else k): entry i >= 0
 * replaces the i-th emitted token before it is chained.  draft_ids_out (host, nullable,
 * room for k_max ids) receives the tokens.
 * With cfg.ddd_enabled the head exits before token s iff s > k AND the log-probability of
 * the s-1 tokens drafted so far (under softmax(logits / T), T = 1 when greedy) is below
 * cfg.ddd_threshold: at least one token is drafted (for thresholds <= 0), the longer of the
 * two lengths is kept, never more than k_max; override_ids and u_draft then hold k_max
 * entries.  Where the rule is evaluated is chosen with ae_set_ddd_mode.
 * ae_last_draft_len() tells how many tokens were drafted. */
int ae_draft(ae_ctx *ctx, int k, const int32_t *override_ids, const double *u_draft,
             int32_t *draft_ids_out);

/* Where the exit rule of cfg.ddd_enabled is evaluated (Sec. 3.2 worries about CPU<->GPU
 * traffic in the decoding loop; Sec. 3.4 / 4.2 give the rule).
 *  AE_DDD_HOST: the host reads the running log-probability back before every token past k:
 *    one stream synchronisation per such decision, no wasted launches.
 *  AE_DDD_DEVICE (default; measured faster at the 7B shape whether the rule extends drafts
 *    never, sometimes or always): ae_draft enqueues all k_max tokens; the kernels of every token past k
 *    check a device-side flag at entry and return at once after the rule has said stop.
 *    No synchronisation inside ae_draft: a whole ae_step synchronises once, in ae_accept.
 *    The drafted length then lives on the device until ae_accept: the implicit verify block
 *    is padded to k_max + 1 rows (rows past the drafted length hold stale tokens whose
 *    cache rows are dead after the rollback) and u_accept must hold k_max + 1 uniforms.
 *    ae_draft with draft_ids_out != NULL synchronises anyway and un-pads: ae_last_draft_len()
 *    is exact after it, else only after ae_accept.
 * Both modes draft the same tokens. */
enum { AE_DDD_HOST = 0, AE_DDD_DEVICE = 1 };
int ae_set_ddd_mode(ae_ctx *ctx, int mode);

/* Temperature of the next steps (Sec. 2.1: 0 = greedy longest-prefix match, > 0 = rejection
 * sampling with softmax(logits / T) for both models).  Replaces cfg.temperature; nothing is
 * re-allocated and the caches stay valid.  AE_ESTATE between ae_draft and ae_accept (a draft
 * sampled at one temperature must be judged at the same one), AE_EINVAL for a negative or
 * non-finite value, AE_EUNSUPPORTED for T > 0 with a vocabulary above 1048576 tokens. */
int ae_set_temperature(ae_ctx *ctx, float temperature);

/* Eq. 1, forward part: target forward of an n_rows block at slots kv_len.. with causal
 * attention over the cache; row i's logits judge block token i+1.  block_ids (host)
 * NULL => the block is [pending, the k draft tokens] and n_rows must be k+1. */
int ae_verify(ae_ctx *ctx, const int32_t *block_ids, int n_rows);

/* Number of tokens the last ae_draft emitted, and the log-probability of that sequence under
 * the draft head (valid when cfg.ddd_enabled). */
int ae_last_draft_len(const ae_ctx *ctx);
int ae_get_draft_logprob(ae_ctx *ctx, float *out);

/* Acceptance and rollback.  Greedy (Sec. 3.1 footnote, the "validated prefix" of Eq. 1;
 * temperature 0, u ignored): n_accepted = length of the longest draft prefix equal to the
 * target argmax, bonus = target argmax of the next row.  temperature > 0 (the speculative
 * sampling rule of Sec. 2.1): u (host) holds n_rows uniforms in [0,1): u[i], i < k,
 * accepts draft token i+1 iff u[i] < min(1, p/p_hat); the first rejection resamples
 * from norm(max(0, p - p_hat)) over the vocabulary, no rejection samples the bonus
 * from the last row; both draws use u[k] by inverse CDF in token order, in float64.
 * Afterwards kv_len += 1 + n_accepted (rows beyond are dead) and pending = bonus. */
int ae_accept(ae_ctx *ctx, const double *u, int *n_accepted, int32_t *bonus);

typedef struct {
  /* inputs */
  int32_t k_force;              /* >= 0: use this draft length instead of the LDLP's */
  const int32_t *override_ids;  /* host, nullable: see ae_draft */
  const double *u_draft;        /* host, [k_max]  (temperature > 0 only) */
  const double *u_accept;       /* host, [k_max+1] (temperature > 0 only) */
  /* outputs */
  int32_t k;                    /* draft length used */
  int32_t n_accepted;           /* k-circle of Eq. 1 */
  int32_t n_tokens;             /* n_accepted + 1 */
  int32_t tokens[16];           /* accepted draft tokens, then the bonus token */
  float us_total;               /* wall time of the step, host clock */
} ae_step_io;

/* One iteration of Algorithm 1 in the order LDLP -> draft -> verify -> accept+rollback. */
int ae_step(ae_ctx *ctx, ae_step_io *io);

/* Introspection for parity tests (host outputs). */
int ae_kv_len(const ae_ctx *ctx);
int32_t ae_pending(const ae_ctx *ctx);
int ae_get_logits(ae_ctx *ctx, int row, float *out_vocab);       /* last verify */
int ae_get_feature(ae_ctx *ctx, int row, float *out_d);          /* last verify / prefill block */
int ae_get_draft_logits(ae_ctx *ctx, int i, float *out_vocab);   /* behind draft token i */
int ae_get_kv_row(ae_ctx *ctx, int layer, int which /*0=K 1=V*/, int slot, float *out_dkv);

/* Phase timing: when enabled, ae_step brackets its phases with HIP events. */
typedef struct { float us_ldlp, us_draft, us_verify, us_accept; } ae_phase_times;
int ae_set_profiling(ae_ctx *ctx, int enabled);
int ae_get_phase_times(ae_ctx *ctx, ae_phase_times *out);   /* of the last ae_step */

/* Per-kernel timing of the dominant kernel (the fused gate/up SwiGLU GEMM of every decoder
 * layer): while enabled, each of its launches is bracketed by HIP events on the ctx's
 * stream; totals are folded in at every stream synchronisation.  Enabling resets them. */
int ae_set_kernel_timing(ae_ctx *ctx, int enabled);
int ae_get_kernel_timing(ae_ctx *ctx, double *total_us, int64_t *launches);

/* Diagnostic yardstick for the bandwidth figures: runs `launches` plain read-only streaming
 * kernels back to back on `hip_stream` (each reads bytes_per_launch bytes, a multiple of 4096,
 * from device memory it allocates and frees itself; consecutive launches read different
 * buffers), `repeats` times, and returns the mean wall time per launch in microseconds (host
 * pointer).  This is what a dependent chain of kernels that do nothing but stream their operand
 * sustains on the GPU: the decode GEMMs of this library (Eq. 1 / Eq. 2 forwards at batch size 1)
 * are exactly such chains with arithmetic attached. */
int ae_probe_read_stream(void *hip_stream, size_t bytes_per_launch, int launches, int repeats, double *us_per_launch);

const char *ae_version(void);

#ifdef __cplusplus
}
#endif
#endif
