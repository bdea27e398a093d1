/*
 * CPU oracle for the AdaEAGLE decode step -- TEST INFRASTRUCTURE ONLY.
 * See adaeagle_oracle.h for scope, precision and pins.  Every routine below is
 * the textbook definition written out: one accumulator per output, ascending
 * index order, no blocking, no fusion.  OpenMP is used only across independent
 * outputs, which does not change any summation order.
 *
 * Index conventions: token positions in the paper are 1-based (t_1..t_n); cache
 * slots and rotary positions here are 0-based, slot s holds token t_{s+1}.
 */
#include "adaeagle_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORC_ACC_DOUBLE
typedef double acc_t;
#else
typedef float acc_t;
#endif

#define ORC_MAX_ROWS 64 /* rows handled per internal block (prefill chunking only) */

struct orc_model {
  orc_config c;
  orc_weights w;
  orc_layer *layers; /* private copy of the layer table */
  int d_kv;
  float **K, **V;        /* [L+1] lists of [n_ctx_max][d_kv] */
  float *cos_t, *sin_t;  /* [n_ctx_max][head_dim/2] */
  int32_t *hist;         /* token at every slot; hist[kv_len] is the pending bonus token */
  int kv_len;            /* n: tokens held by the target lists */
  int dlen;              /* draft slots computed from true target features */
  int nF;                /* valid feature rows: row i <-> slot kv_len - nF + i */
  float *F;              /* [ORC_MAX_ROWS][d] post-final-norm hidden states */
  float *logits;         /* [k_max+1][V] of the last verify */
  float *dlogits;        /* [k_max][V] draft logits behind each draft token */
  float *fhat;           /* [d] last draft-head output */
  int32_t *draft_ids;    /* [k_max] */
  int32_t *block;        /* [k_max+1] ids of the last verify block */
  int cur_k, block_rows;
  double cum_logp;       /* log-probability of the current draft sequence */
  int have_pending, have_draft, have_verify;
};

/* ---------------------------------------------------------------- scalars */

static inline float bf16_bits_to_float(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* round-to-nearest-even to 8 significant bits, result returned as float */
float orc_bf16_round(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return x; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static inline float wval(const void *W, int wdtype, size_t idx) {
  return wdtype == ORC_BF16 ? bf16_bits_to_float(((const uint16_t *)W)[idx]) : ((const float *)W)[idx];
}

int orc_argmax(const float *x, int n) {
  int best = 0;
  for (int i = 1; i < n; ++i)
    if (x[i] > x[best]) best = i; /* strict: lowest index wins ties */
  return best;
}

/* Eq. 3: round (half to even) then clamp to [0, k_max]. */
int orc_round_clamp(float y, int k_max) {
  if (isnan(y)) return 0;
  double r = nearbyint((double)y);
  if (r < 0.0) r = 0.0;
  if (r > (double)k_max) r = (double)k_max;
  return (int)r;
}

static inline float silu(float x) { return x / (1.0f + expf(-x)); }

/* ---------------------------------------------------------------- pieces */

/* y[r][n] = sum_k x[r][k] * W[n][k]  (+ bias[n]) */
static void matmul(const void *W, int wdtype, int N, int K, const float *x, int rows, int ldx,
                   const float *bias, float *y, int ldy) {
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    acc_t acc[ORC_MAX_ROWS];
    for (int r = 0; r < rows; ++r) acc[r] = 0;
    const size_t base = (size_t)n * (size_t)K;
    for (int k = 0; k < K; ++k) {
      const float wv = wval(W, wdtype, base + (size_t)k);
      for (int r = 0; r < rows; ++r) acc[r] += (acc_t)x[(size_t)r * ldx + k] * (acc_t)wv;
    }
    for (int r = 0; r < rows; ++r) {
      float v = (float)acc[r];
      if (bias) v += bias[n];
      y[(size_t)r * ldy + n] = v;
    }
  }
}

void orc_rmsnorm(const float *x, const float *g, int d, float eps, float *out) {
  acc_t ss = 0;
  for (int i = 0; i < d; ++i) ss += (acc_t)x[i] * (acc_t)x[i];
  const float ms = (float)(ss / (acc_t)d);
  const float r = 1.0f / sqrtf(ms + eps);
  for (int i = 0; i < d; ++i) out[i] = (x[i] * r) * g[i];
}

static void rope_angles(int pos, int i, int head_dim, float base, float *c, float *s) {
  const double inv = pow((double)base, -2.0 * (double)i / (double)head_dim);
  const double ang = (double)pos * inv;
  *c = (float)cos(ang);
  *s = (float)sin(ang);
}

/* rotate-half pairing: element i rotates with element i + head_dim/2 */
static void rope_apply(float *x, int n_heads, int head_dim, const float *c, const float *s) {
  const int half = head_dim / 2;
  for (int h = 0; h < n_heads; ++h) {
    float *p = x + (size_t)h * head_dim;
    for (int i = 0; i < half; ++i) {
      const float a = p[i], b = p[i + half];
      p[i] = a * c[i] - b * s[i];
      p[i + half] = b * c[i] + a * s[i];
    }
  }
}

void orc_rope(float *x, int n_heads, int head_dim, int pos, float base) {
  const int half = head_dim / 2;
  float *c = (float *)malloc(sizeof(float) * half), *s = (float *)malloc(sizeof(float) * half);
  for (int i = 0; i < half; ++i) rope_angles(pos, i, head_dim, base, &c[i], &s[i]);
  rope_apply(x, n_heads, head_dim, c, s);
  free(c);
  free(s);
}

/* softmax(q.k / sqrt(hd)) . v over keys 0..n_keys-1, one query row, all heads.
 * Query head h reads KV head h / (n_heads / n_kv_heads). */
void orc_attention_row(const float *q, const float *k, const float *v, int n_keys, int n_heads,
                       int n_kv_heads, int head_dim, int kv_stride, float *out) {
  const float scale = 1.0f / sqrtf((float)head_dim);
  const int group = n_heads / n_kv_heads;
  float *sc = (float *)malloc(sizeof(float) * (size_t)n_keys);
  for (int h = 0; h < n_heads; ++h) {
    const int kh = h / group;
    const float *qh = q + (size_t)h * head_dim;
    float mx = -INFINITY;
    for (int j = 0; j < n_keys; ++j) {
      const float *kj = k + (size_t)j * kv_stride + (size_t)kh * head_dim;
      acc_t a = 0;
      for (int d = 0; d < head_dim; ++d) a += (acc_t)qh[d] * (acc_t)kj[d];
      sc[j] = (float)a * scale;
      if (sc[j] > mx) mx = sc[j];
    }
    acc_t den = 0;
    for (int j = 0; j < n_keys; ++j) {
      sc[j] = expf(sc[j] - mx);
      den += (acc_t)sc[j];
    }
    for (int d = 0; d < head_dim; ++d) {
      acc_t a = 0;
      for (int j = 0; j < n_keys; ++j)
        a += (acc_t)sc[j] * (acc_t)v[(size_t)j * kv_stride + (size_t)kh * head_dim + d];
      out[(size_t)h * head_dim + d] = (float)(a / den);
    }
  }
  free(sc);
}

/* One pre-norm Llama-style decoder layer over `rows` consecutive slots starting at
 * pos0; appends K/V for those slots to list `li` and updates x in place. */
static void decoder_layer(orc_model *m, const orc_layer *lw, int li, float *x, int rows, int pos0) {
  const orc_config *c = &m->c;
  const int d = c->d_model, H = c->n_heads, Hk = c->n_kv_heads, hd = c->head_dim, f = c->d_ffn;
  const int dq = H * hd, dkv = Hk * hd, half = hd / 2;
  float *h = (float *)malloc(sizeof(float) * (size_t)rows * d);
  float *q = (float *)malloc(sizeof(float) * (size_t)rows * dq);
  float *kk = (float *)malloc(sizeof(float) * (size_t)rows * dkv);
  float *vv = (float *)malloc(sizeof(float) * (size_t)rows * dkv);
  float *a = (float *)malloc(sizeof(float) * (size_t)rows * dq);
  float *o = (float *)malloc(sizeof(float) * (size_t)rows * d);
  float *g = (float *)malloc(sizeof(float) * (size_t)rows * f);
  float *u = (float *)malloc(sizeof(float) * (size_t)rows * f);

  for (int r = 0; r < rows; ++r) orc_rmsnorm(x + (size_t)r * d, lw->attn_norm, d, c->rms_eps, h + (size_t)r * d);
  matmul(lw->wq, c->wdtype, dq, d, h, rows, d, NULL, q, dq);
  matmul(lw->wk, c->wdtype, dkv, d, h, rows, d, NULL, kk, dkv);
  matmul(lw->wv, c->wdtype, dkv, d, h, rows, d, NULL, vv, dkv);
  for (int r = 0; r < rows; ++r) {
    const int pos = pos0 + r;
    const float *cs = m->cos_t + (size_t)pos * half, *sn = m->sin_t + (size_t)pos * half;
    rope_apply(q + (size_t)r * dq, H, hd, cs, sn);
    rope_apply(kk + (size_t)r * dkv, Hk, hd, cs, sn);
    float *Kd = m->K[li] + (size_t)pos * dkv, *Vd = m->V[li] + (size_t)pos * dkv;
    for (int i = 0; i < dkv; ++i) {
      /* a bf16 cache stores 8 significant bits; fp32 mode stores the value as is */
      Kd[i] = c->wdtype == ORC_BF16 ? orc_bf16_round(kk[(size_t)r * dkv + i]) : kk[(size_t)r * dkv + i];
      Vd[i] = c->wdtype == ORC_BF16 ? orc_bf16_round(vv[(size_t)r * dkv + i]) : vv[(size_t)r * dkv + i];
    }
  }
#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < rows; ++r) /* row r sees keys 0 .. pos0 + r (causal) */
    orc_attention_row(q + (size_t)r * dq, m->K[li], m->V[li], pos0 + r + 1, H, Hk, hd, dkv, a + (size_t)r * dq);
  matmul(lw->wo, c->wdtype, d, dq, a, rows, dq, NULL, o, d);
  for (size_t i = 0; i < (size_t)rows * d; ++i) x[i] += o[i];

  for (int r = 0; r < rows; ++r) orc_rmsnorm(x + (size_t)r * d, lw->ffn_norm, d, c->rms_eps, h + (size_t)r * d);
  matmul(lw->w_gate, c->wdtype, f, d, h, rows, d, NULL, g, f);
  matmul(lw->w_up, c->wdtype, f, d, h, rows, d, NULL, u, f);
  for (size_t i = 0; i < (size_t)rows * f; ++i) g[i] = silu(g[i]) * u[i];
  matmul(lw->w_down, c->wdtype, d, f, g, rows, f, NULL, o, d);
  for (size_t i = 0; i < (size_t)rows * d; ++i) x[i] += o[i];

  free(h); free(q); free(kk); free(vv); free(a); free(o); free(g); free(u);
}

static void embed(const orc_model *m, int32_t id, float *out) {
  const int d = m->c.d_model;
  for (int i = 0; i < d; ++i) out[i] = wval(m->w.tok_emb, m->c.wdtype, (size_t)id * d + i);
}

/* Target forward over a block of rows at slots pos0.. : features (post final norm)
 * into feat[rows][d]; logits for rows >= logit_from into m->logits[row - logit_from]. */
static void target_block(orc_model *m, const int32_t *ids, int rows, int pos0, float *feat,
                         int logit_from) {
  const orc_config *c = &m->c;
  const int d = c->d_model;
  float *x = (float *)malloc(sizeof(float) * (size_t)rows * d);
  for (int r = 0; r < rows; ++r) embed(m, ids[r], x + (size_t)r * d);
  for (int l = 0; l < c->n_layers; ++l) decoder_layer(m, &m->layers[l], l, x, rows, pos0);
  for (int r = 0; r < rows; ++r) orc_rmsnorm(x + (size_t)r * d, m->w.final_norm, d, c->rms_eps, feat + (size_t)r * d);
  if (logit_from < rows)
    matmul(m->w.lm_head, c->wdtype, c->vocab, d, feat + (size_t)logit_from * d, rows - logit_from, d, NULL,
           m->logits, c->vocab);
  free(x);
}

/* Draft head over `rows` slots starting at slot0: input of a slot is
 * fc([feature of that slot ; embedding of the NEXT token]); output of the last row
 * (no final norm) is left in m->fhat. */
static void draft_rows(orc_model *m, const float *feats, const int32_t *next_tok, int rows, int slot0) {
  const orc_config *c = &m->c;
  const int d = c->d_model;
  float *cat = (float *)malloc(sizeof(float) * (size_t)rows * 2 * d);
  float *x = (float *)malloc(sizeof(float) * (size_t)rows * d);
  for (int r = 0; r < rows; ++r) {
    memcpy(cat + (size_t)r * 2 * d, feats + (size_t)r * d, sizeof(float) * d);
    embed(m, next_tok[r], cat + (size_t)r * 2 * d + d);
  }
  matmul(m->w.draft_fc_w, c->wdtype, d, 2 * d, cat, rows, 2 * d, m->w.draft_fc_b, x, d);
  decoder_layer(m, &m->w.draft_layer, c->n_layers, x, rows, slot0);
  memcpy(m->fhat, x + (size_t)(rows - 1) * d, sizeof(float) * d);
  free(cat);
  free(x);
}

/* ---------------------------------------------------------------- sampling */

static void softmax_T(const float *logits, int n, double T, double *p) {
  double mx = -INFINITY;
  for (int i = 0; i < n; ++i)
    if ((double)logits[i] > mx) mx = (double)logits[i];
  double s = 0.0;
  for (int i = 0; i < n; ++i) {
    p[i] = exp(((double)logits[i] - mx) / T);
    s += p[i];
  }
  for (int i = 0; i < n; ++i) p[i] /= s;
}

/* smallest x with q[0] + .. + q[x] > u * sum(q); q need not be normalised */
int32_t orc_sample_inverse_cdf(const double *q, int n, double u) {
  double tot = 0.0;
  for (int i = 0; i < n; ++i) tot += q[i];
  const double thr = u * tot;
  double c = 0.0;
  int last = 0;
  for (int i = 0; i < n; ++i) {
    if (q[i] > 0.0) last = i;
    c += q[i];
    if (c > thr) return i;
  }
  return last;
}

int orc_accept_greedy(const float *target_logits, int vocab, int k, const int32_t *draft_ids,
                      int *n_accepted, int32_t *bonus) {
  int acc = 0;
  while (acc < k && draft_ids[acc] == orc_argmax(target_logits + (size_t)acc * vocab, vocab)) ++acc;
  *n_accepted = acc;
  *bonus = orc_argmax(target_logits + (size_t)acc * vocab, vocab);
  return 0;
}

/* Sec. 2.1: accept draft token i with probability min(1, p/p_hat); at the first
 * rejection resample from the normalised positive part of (p - p_hat) taken over the
 * whole vocabulary; if nothing is rejected the bonus comes from the target law of
 * the row after the last draft token. */
int orc_accept_sample(const float *target_logits, const float *draft_logits, int vocab, int k,
                      const int32_t *draft_ids, double temperature, const double *u,
                      int *n_accepted, int32_t *bonus) {
  double *p = (double *)malloc(sizeof(double) * vocab), *ph = (double *)malloc(sizeof(double) * vocab);
  int acc = 0;
  for (; acc < k; ++acc) {
    softmax_T(target_logits + (size_t)acc * vocab, vocab, temperature, p);
    softmax_T(draft_logits + (size_t)acc * vocab, vocab, temperature, ph);
    const int32_t t = draft_ids[acc];
    double ratio = ph[t] > 0.0 ? p[t] / ph[t] : 1.0;
    if (ratio > 1.0) ratio = 1.0;
    if (u[acc] < ratio) continue;
    double tot = 0.0;
    for (int i = 0; i < vocab; ++i) {
      ph[i] = p[i] - ph[i] > 0.0 ? p[i] - ph[i] : 0.0;
      tot += ph[i];
    }
    *bonus = orc_sample_inverse_cdf(tot > 0.0 ? ph : p, vocab, u[k]);
    *n_accepted = acc;
    free(p); free(ph);
    return 0;
  }
  softmax_T(target_logits + (size_t)k * vocab, vocab, temperature, p);
  *bonus = orc_sample_inverse_cdf(p, vocab, u[k]);
  *n_accepted = k;
  free(p); free(ph);
  return 0;
}

/* ---------------------------------------------------------------- model */

orc_model *orc_create(const orc_config *cfg, const orc_weights *w) {
  if (!cfg || !w) return NULL;
  if (cfg->n_layers < 1 || cfg->d_model < 1 || cfg->n_heads < 1 || cfg->n_kv_heads < 1 ||
      cfg->n_heads % cfg->n_kv_heads || cfg->head_dim < 2 || cfg->head_dim % 2 || cfg->k_max < 0 ||
      cfg->k_max + 1 > ORC_MAX_ROWS || cfg->n_ctx_max < 1 || cfg->vocab < 1)
    return NULL;
  orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
  m->c = *cfg;
  m->w = *w;
  m->layers = (orc_layer *)malloc(sizeof(orc_layer) * cfg->n_layers);
  memcpy(m->layers, w->layers, sizeof(orc_layer) * cfg->n_layers);
  m->d_kv = cfg->n_kv_heads * cfg->head_dim;
  const int L1 = cfg->n_layers + 1, half = cfg->head_dim / 2;
  m->K = (float **)malloc(sizeof(float *) * L1);
  m->V = (float **)malloc(sizeof(float *) * L1);
  for (int l = 0; l < L1; ++l) {
    m->K[l] = (float *)calloc((size_t)cfg->n_ctx_max * m->d_kv, sizeof(float));
    m->V[l] = (float *)calloc((size_t)cfg->n_ctx_max * m->d_kv, sizeof(float));
  }
  m->cos_t = (float *)malloc(sizeof(float) * (size_t)cfg->n_ctx_max * half);
  m->sin_t = (float *)malloc(sizeof(float) * (size_t)cfg->n_ctx_max * half);
  for (int p = 0; p < cfg->n_ctx_max; ++p)
    for (int i = 0; i < half; ++i)
      rope_angles(p, i, cfg->head_dim, cfg->rope_base, &m->cos_t[(size_t)p * half + i], &m->sin_t[(size_t)p * half + i]);
  m->hist = (int32_t *)calloc((size_t)cfg->n_ctx_max + 2, sizeof(int32_t));
  m->F = (float *)calloc((size_t)ORC_MAX_ROWS * cfg->d_model, sizeof(float));
  m->logits = (float *)calloc((size_t)(cfg->k_max + 1) * cfg->vocab, sizeof(float));
  m->dlogits = (float *)calloc((size_t)(cfg->k_max > 0 ? cfg->k_max : 1) * cfg->vocab, sizeof(float));
  m->fhat = (float *)calloc(cfg->d_model, sizeof(float));
  m->draft_ids = (int32_t *)calloc(cfg->k_max + 1, sizeof(int32_t));
  m->block = (int32_t *)calloc(cfg->k_max + 1, sizeof(int32_t));
  return m;
}

void orc_destroy(orc_model *m) {
  if (!m) return;
  for (int l = 0; l <= m->c.n_layers; ++l) { free(m->K[l]); free(m->V[l]); }
  free(m->K); free(m->V); free(m->cos_t); free(m->sin_t); free(m->hist); free(m->F);
  free(m->logits); free(m->dlogits); free(m->fhat); free(m->draft_ids); free(m->block);
  free(m->layers); free(m);
}

static int ids_ok(const orc_model *m, const int32_t *ids, int n) {
  for (int i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= m->c.vocab) return 0;
  return 1;
}

int orc_prefill(orc_model *m, const int32_t *ids, int n) {
  if (!ids || n < 1 || n + m->c.k_max + 1 > m->c.n_ctx_max || !ids_ok(m, ids, n)) return -1;
  const int chunk = m->c.k_max + 1;
  memcpy(m->hist, ids, sizeof(int32_t) * n);
  m->kv_len = 0; m->dlen = 0; m->nF = 0;
  for (int p0 = 0; p0 < n; p0 += chunk) {
    const int rows = n - p0 < chunk ? n - p0 : chunk;
    const int last = p0 + rows == n;
    /* only the very last prompt row needs logits: it yields the first new token */
    target_block(m, ids + p0, rows, p0, m->F, last ? rows - 1 : rows);
    /* draft slots whose next token is already known from the prompt */
    const int drows = last ? rows - 1 : rows;
    if (drows > 0) draft_rows(m, m->F, ids + p0 + 1, drows, p0);
    m->nF = rows;
  }
  m->kv_len = n;
  m->dlen = n - 1;
  m->hist[n] = orc_argmax(m->logits, m->c.vocab);
  m->have_pending = 1; m->have_draft = 0; m->have_verify = 0; m->cur_k = 0;
  return 0;
}

int orc_kv_import(orc_model *m, int layer, const float *k, const float *v, int n) {
  if (layer < 0 || layer > m->c.n_layers || n < 0 || n > m->c.n_ctx_max || !k || !v) return -1;
  const size_t cnt = (size_t)n * m->d_kv;
  for (size_t i = 0; i < cnt; ++i) {
    m->K[layer][i] = m->c.wdtype == ORC_BF16 ? orc_bf16_round(k[i]) : k[i];
    m->V[layer][i] = m->c.wdtype == ORC_BF16 ? orc_bf16_round(v[i]) : v[i];
  }
  return 0;
}

int orc_set_state(orc_model *m, int kv_len, int32_t last_tok, int32_t pending, const float *feat) {
  if (kv_len < 1 || kv_len + m->c.k_max + 1 > m->c.n_ctx_max || !feat) return -1;
  if (!ids_ok(m, &last_tok, 1) || !ids_ok(m, &pending, 1)) return -1;
  m->kv_len = kv_len;
  m->dlen = kv_len - 1;
  m->nF = 1;
  memcpy(m->F, feat, sizeof(float) * m->c.d_model);
  m->hist[kv_len - 1] = last_tok;
  m->hist[kv_len] = pending;
  m->have_pending = 1; m->have_draft = 0; m->have_verify = 0; m->cur_k = 0;
  return 0;
}

/* Eq. 3 with the MLP body: z = W_in u + b_in; z += silu(W_r z + b_r) per residual
 * block; y = w_out . silu(z) + b_out.  u = [e ; f] where e embeds the last validated
 * token (slot n-1) and f is its post-norm hidden state. */
int orc_ldlp(orc_model *m, int *k_out, float *y_out) {
  if (!m->have_pending || m->nF < 1) return -2;
  const orc_config *c = &m->c;
  const int d = c->d_model, h = c->ldlp_hidden;
  const int in = c->ldlp_in_mode == 0 ? 2 * d : d;
  float *u = (float *)malloc(sizeof(float) * in);
  const float *f = m->F + (size_t)(m->nF - 1) * d;
  if (c->ldlp_in_mode == 0) {
    embed(m, m->hist[m->kv_len - 1], u);
    memcpy(u + d, f, sizeof(float) * d);
  } else {
    memcpy(u, f, sizeof(float) * d);
  }
  float *z = (float *)malloc(sizeof(float) * h), *t = (float *)malloc(sizeof(float) * h);
  matmul(m->w.ldlp_w_in, c->wdtype, h, in, u, 1, in, m->w.ldlp_b_in, z, h);
  for (int r = 0; r < c->ldlp_n_res; ++r) {
    const void *Wr = c->wdtype == ORC_BF16 ? (const void *)((const uint16_t *)m->w.ldlp_w_res + (size_t)r * h * h)
                                           : (const void *)((const float *)m->w.ldlp_w_res + (size_t)r * h * h);
    matmul(Wr, c->wdtype, h, h, z, 1, h, m->w.ldlp_b_res + (size_t)r * h, t, h);
    for (int i = 0; i < h; ++i) z[i] += silu(t[i]);
  }
  if (c->ldlp_cls) {
    /* one score per candidate length 0..k_max; the best score names the length */
    int best = 0;
    float best_y = 0.0f;
    for (int cl = 0; cl <= c->k_max; ++cl) {
      acc_t a = 0;
      for (int i = 0; i < h; ++i) a += (acc_t)silu(z[i]) * (acc_t)m->w.ldlp_w_out[(size_t)cl * h + i];
      const float y = (float)a + m->w.ldlp_b_out[cl];
      if (cl == 0 || y > best_y) { best = cl; best_y = y; }
    }
    if (y_out) *y_out = best_y;
    *k_out = best;
  } else {
    acc_t a = 0;
    for (int i = 0; i < h; ++i) a += (acc_t)silu(z[i]) * (acc_t)m->w.ldlp_w_out[i];
    const float y = (float)a + m->w.ldlp_b_out[0];
    if (y_out) *y_out = y;
    *k_out = orc_round_clamp(y, c->k_max);
  }
  free(u); free(z); free(t);
  return 0;
}

static int32_t pick_draft_token(orc_model *m, int i, const double *u_draft) {
  const int V = m->c.vocab;
  const float *lg = m->dlogits + (size_t)i * V;
  if (m->c.temperature <= 0.0f || !u_draft) return orc_argmax(lg, V);
  double *p = (double *)malloc(sizeof(double) * V);
  softmax_T(lg, V, (double)m->c.temperature, p);
  const int32_t t = orc_sample_inverse_cdf(p, V, u_draft[i]);
  free(p);
  return t;
}

int orc_draft(orc_model *m, int k, const int32_t *override_ids, const double *u_draft, int32_t *ids_out) {
  const orc_config *c = &m->c;
  if (!m->have_pending) return -2;
  if (k < 0 || k > c->k_max || m->kv_len + c->k_max + 1 > c->n_ctx_max) return -1;
  if (c->temperature > 0.0f && (k > 0 || c->ddd_enabled) && !u_draft) return -1;
  const int n = m->kv_len, d = c->d_model, V = c->vocab;
  const int catch_rows = n - m->dlen;
  if (catch_rows < 1 || catch_rows > m->nF) return -2;
  /* catch-up: slots dlen..n-1 pair the true feature of the slot with the next token */
  draft_rows(m, m->F + (size_t)(m->nF - catch_rows) * d, m->hist + m->dlen + 1, catch_rows, m->dlen);
  m->dlen = n;
  float *feat = (float *)malloc(sizeof(float) * d);
  const double T = c->temperature > 0.0f ? (double)c->temperature : 1.0;
  m->cum_logp = 0.0;
  int i = 0;
  for (; i < c->k_max; ++i) {
    /* exit rule: past the predicted length, stop unless DDD says the sequence is still likely */
    if (i >= k && !(c->ddd_enabled && m->cum_logp >= (double)c->ddd_threshold)) break;
    if (i > 0) { /* chain: the head's own previous output stands in for the feature */
      memcpy(feat, m->fhat, sizeof(float) * d);
      draft_rows(m, feat, &m->draft_ids[i - 1], 1, n - 1 + i);
    }
    matmul(m->w.lm_head, c->wdtype, V, d, m->fhat, 1, d, NULL, m->dlogits + (size_t)i * V, V);
    int32_t t = pick_draft_token(m, i, u_draft);
    if (override_ids && override_ids[i] >= 0) {
      if (override_ids[i] >= V) { free(feat); return -1; }
      t = override_ids[i];
    }
    m->draft_ids[i] = t;
    if (ids_out) ids_out[i] = t;
    { /* log p_hat(t) under softmax(logits / T) */
      const float *lg = m->dlogits + (size_t)i * V;
      double mx = -INFINITY, se = 0.0;
      for (int x = 0; x < V; ++x) if ((double)lg[x] > mx) mx = (double)lg[x];
      for (int x = 0; x < V; ++x) se += exp(((double)lg[x] - mx) / T);
      m->cum_logp += ((double)lg[t] - mx) / T - log(se);
    }
  }
  k = i;
  free(feat);
  m->cur_k = k;
  m->have_draft = 1;
  return 0;
}

int orc_verify(orc_model *m, const int32_t *block_ids, int n_rows) {
  const orc_config *c = &m->c;
  if (!m->have_pending) return -2;
  if (n_rows < 1 || n_rows > c->k_max + 1 || m->kv_len + n_rows > c->n_ctx_max) return -1;
  if (block_ids) {
    if (!ids_ok(m, block_ids, n_rows)) return -1;
    memcpy(m->block, block_ids, sizeof(int32_t) * n_rows);
  } else {
    if (!m->have_draft || n_rows != m->cur_k + 1) return -2;
    m->block[0] = m->hist[m->kv_len];
    for (int i = 0; i < m->cur_k; ++i) m->block[1 + i] = m->draft_ids[i];
  }
  target_block(m, m->block, n_rows, m->kv_len, m->F, 0);
  m->block_rows = n_rows;
  m->have_verify = 1;
  return 0;
}

int orc_accept(orc_model *m, const double *u, int *n_accepted, int32_t *bonus) {
  const orc_config *c = &m->c;
  if (!m->have_verify) return -2;
  const int k = m->block_rows - 1;
  int acc = 0;
  int32_t b = 0;
  if (c->temperature > 0.0f) {
    if (!u) return -1;
    orc_accept_sample(m->logits, m->dlogits, c->vocab, k, m->block + 1, (double)c->temperature, u, &acc, &b);
  } else {
    orc_accept_greedy(m->logits, c->vocab, k, m->block + 1, &acc, &b);
  }
  /* rollback: the accepted prefix is already in place, everything after it is dead */
  const int n = m->kv_len;
  for (int i = 0; i <= acc; ++i) m->hist[n + i] = m->block[i];
  m->kv_len = n + 1 + acc;
  m->hist[m->kv_len] = b;
  m->nF = acc + 1;
  m->have_verify = 0; m->have_draft = 0; m->cur_k = 0;
  if (n_accepted) *n_accepted = acc;
  if (bonus) *bonus = b;
  return 0;
}

int orc_step(orc_model *m, int k_force, const int32_t *override_ids, const double *u_draft,
             const double *u_accept, int *k_out, int *n_accepted, int32_t *tokens_out) {
  int k = 0, rc;
  if ((rc = orc_ldlp(m, &k, NULL))) return rc;
  if (k_force >= 0) k = k_force;
  if ((rc = orc_draft(m, k, override_ids, u_draft, NULL))) return rc;
  k = m->cur_k; /* DDD may have extended the draft */
  if ((rc = orc_verify(m, NULL, k + 1))) return rc;
  int acc = 0;
  int32_t b = 0;
  if ((rc = orc_accept(m, u_accept, &acc, &b))) return rc;
  if (tokens_out) {
    for (int i = 0; i < acc; ++i) tokens_out[i] = m->block[1 + i];
    tokens_out[acc] = b;
  }
  if (k_out) *k_out = k;
  if (n_accepted) *n_accepted = acc;
  return 0;
}

int orc_ar_greedy(orc_model *m, int n_tokens, int32_t *out) {
  if (!m->have_pending) return -2;
  if (m->kv_len + n_tokens > m->c.n_ctx_max) return -1;
  for (int i = 0; i < n_tokens; ++i) {
    int32_t id = m->hist[m->kv_len];
    target_block(m, &id, 1, m->kv_len, m->F, 0);
    m->kv_len += 1;
    m->hist[m->kv_len] = orc_argmax(m->logits, m->c.vocab);
    m->nF = 1;
    out[i] = m->hist[m->kv_len];
  }
  return 0;
}

int orc_kv_len(const orc_model *m) { return m->kv_len; }
int orc_last_draft_len(const orc_model *m) { return m->cur_k; }
double orc_draft_logprob(const orc_model *m) { return m->cum_logp; }
int32_t orc_pending(const orc_model *m) { return m->hist[m->kv_len]; }
const float *orc_logits(const orc_model *m, int row) { return m->logits + (size_t)row * m->c.vocab; }
const float *orc_feature(const orc_model *m, int row) { return m->F + (size_t)row * m->c.d_model; }
const float *orc_draft_logits(const orc_model *m, int i) { return m->dlogits + (size_t)i * m->c.vocab; }
const float *orc_kv_row(const orc_model *m, int layer, int which, int slot) {
  return (which ? m->V[layer] : m->K[layer]) + (size_t)slot * m->d_kv;
}

/* Sec. 3.3, optimisation criterion: L1 distance, times lambda when the prediction is short. */
double orc_ldlp_loss(const float *pred, const int32_t *truth, int n, double lambda) {
  double tot = 0.0;
  for (int i = 0; i < n; ++i) {
    const double diff = (double)pred[i] - (double)truth[i];
    tot += diff < 0.0 ? lambda * -diff : diff;
  }
  return n > 0 ? tot / n : 0.0;
}
