// C ABI of libadaeagle: context set-up, the state machine of one sequence, and the
// host-side sequencing of the kernels of one decode step (LDLP -> draft -> verify ->
// accept + rollback, i.e. one iteration of Algorithm 1 of arxiv 2412.18910).
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "ae_internal.h"

using namespace ae;

// Staging area of ae_kv_import_static: device memory that exists from the moment the library
// is loaded, so that entry point never allocates.  Every GPU holds its own copy at its own
// address; host code only ever uses the per-device address looked up in static_stage().
constexpr size_t kStageFloats = (size_t)AE_KV_IMPORT_STATIC_MAX_FLOATS;
static __device__ __align__(256) float g_kv_stage[kStageFloats];

namespace {

thread_local std::string g_init_error;

constexpr int kMaxDevices = 64;
std::mutex g_stage_mu;
float *g_stage_ptr[kMaxDevices] = {};

// Address of g_kv_stage on device `dev`, which must be the current device.
hipError_t static_stage(int dev, float **out) {
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_stage_mu);
  if (!g_stage_ptr[dev]) {
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_kv_stage));
    if (e != hipSuccess) return e;
    g_stage_ptr[dev] = (float *)p;
  }
  *out = g_stage_ptr[dev];
  return hipSuccess;
}

int fail(ae_ctx *c, int code, const std::string &msg) {
  if (c) c->err = msg; else g_init_error = msg;
  return code;
}

#define HIPCHK(c, call)                                                                          \
  do {                                                                                           \
    hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess)                                                                        \
      return fail((c), e_ == hipErrorOutOfMemory ? AE_ENOMEM : AE_EHIP,                          \
                  std::string(#call) + ": " + hipGetErrorString(e_));                            \
  } while (0)

template <typename T>
int dev_alloc(ae_ctx *c, T **p, size_t count) {
  void *q = nullptr;
  hipError_t e = hipMalloc(&q, count * sizeof(T) + 256);
  if (e != hipSuccess) return fail(c, AE_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e));
  c->owned.push_back(q);
  *p = (T *)q;
  return AE_OK;
}

Mat make_mat(const void *p, int N, int K) {
  Mat m;
  m.rowmajor = p; m.N = N; m.K = K;
  return m;
}

// generic path: Y[r][n] (+)= X[r][:] . W[n][:] + bias[n]
void gemm(ae_ctx *c, const Mat &W, const float *X, int ldx, int rows, const float *bias, float *Y, int ldy,
          int accumulate) {
  launch_gemm_generic(W.rowmajor, c->cfg.dtype, W.N, W.K, X, ldx, rows, bias, Y, ldy, accumulate, c->stream, c->gate);
}

bool tileable(const Mat &m) { return m.N % 16 == 0 && m.K % 256 == 0; }

// Allocate a fused k-major tiled matrix and fill it from up to three row-major sources.
// stride 1: sources stacked ([q;k;v]); stride 2 (two sources): row-blocks interleaved (gate, up).
int retile_fused(ae_ctx *c, Mat &dst, const Mat *const *src, int nsrc, bool interleave, int rope_srcs = 0) {
  int N = 0;
  for (int i = 0; i < nsrc; ++i) N += src[i]->N;
  const int K = src[0]->K, NBtot = N / 16;
  char *p = nullptr;
  int rc = dev_alloc(c, &p, (size_t)N * K * 2);
  if (rc) return rc;
  dst.tiled = p; dst.rowmajor = nullptr; dst.N = N; dst.K = K;
  int off = 0;
  for (int i = 0; i < nsrc; ++i) {
    const int perm = i < rope_srcs ? c->cfg.head_dim : 0;   // q / k rows in rotary-pair order
    if (interleave) launch_retile(src[i]->rowmajor, src[i]->N, K, p, NBtot, i, nsrc, perm, c->stream);
    else launch_retile(src[i]->rowmajor, src[i]->N, K, p, NBtot, off, 1, perm, c->stream);
    off += src[i]->N / 16;
  }
  return AE_OK;
}

void *kv_layer_ptr(ae_ctx *c, int li) { return (char *)c->kv + (size_t)li * c->kv_layer_stride; }

// One pre-norm decoder layer over `rows` slots starting at pos0; x is updated in place.
// next_gain (fast path): RMSNorm gain applied to this layer's output for its consumer (the
// next layer, the final norm, or nullptr when the consumer takes the raw output).
void run_layer(ae_ctx *c, int li, float *x, int rows, int pos0, const float *next_gain) {
  const ae_config &g = c->cfg;
  const LayerW &w = c->layers[li];
  const int d = g.d_model, dq = g.n_heads * g.head_dim, dkv = g.n_kv_heads * g.head_dim, f = g.d_ffn;
  hipStream_t s = c->stream;
  if (c->fast) {
    // Activations stay in packed (MFMA B-operand) form between kernels.  RMSNorm is split
    // between producer (x*gain, partial sums of x^2) and consumer (1/rms on accumulators);
    // SwiGLU and both residual adds are GEMM epilogues.
    const int Pd = d / 16;
    GemmLaunch qkv;
    qkv.W = &w.f_qkv; qkv.Xp = c->xp_a; qkv.rows = rows; qkv.ssq_in = c->ssq_a; qkv.P_in = c->Pa; qkv.eps = g.rms_eps;
    qkv.epi = EPI_QKV; qkv.nseg = 3;   // rotary embedding + KV append happen in the epilogue
    qkv.Y[0] = c->q; qkv.ldy[0] = dq;
    qkv.seg_N[0] = dq; qkv.seg_N[1] = dkv; qkv.seg_N[2] = dkv;
    qkv.rope_tab = c->rope_tab; qkv.Kc = kv_layer_ptr(c, li); qkv.Vc = (char *)kv_layer_ptr(c, li) + c->kv_v_offset;
    qkv.pos0 = pos0; qkv.n_ctx = kv_capacity(g); qkv.hd = g.head_dim;
    qkv.gate = c->gate;
    launch_gemm_mfma(qkv, s);
    launch_attention_mfma(c->q, rows, pos0, g, kv_layer_ptr(c, li), c->kv_v_offset, c->attn_part, c->xp_att, s, c->gate);
    GemmLaunch o;
    o.W = &w.wo; o.Xp = c->xp_att; o.rows = rows; o.epi = EPI_RESID; o.Y[0] = x; o.ldy[0] = d; o.seg_N[0] = d;
    o.Xp_out = c->xp_f; o.gain_out = w.ffn_norm; o.ssq_out = c->ssq_f;
    o.gate = c->gate;
    launch_gemm_mfma(o, s);
    GemmLaunch gu;
    gu.W = &w.f_gu; gu.Xp = c->xp_f; gu.rows = rows; gu.ssq_in = c->ssq_f; gu.P_in = Pd; gu.eps = g.rms_eps;
    gu.epi = EPI_SWIGLU; gu.Xp_out = c->xp_h; gu.seg_N[0] = 2 * f;
    gu.gate = c->gate;
    const bool timed = c->ktime && c->kt_used + 2 <= (int)c->kt_ev.size();
    if (timed) hipEventRecord(c->kt_ev[c->kt_used], s);
    launch_gemm_mfma(gu, s);
    if (timed) { hipEventRecord(c->kt_ev[c->kt_used + 1], s); c->kt_used += 2; }
    GemmLaunch dn;
    dn.W = &w.w_down; dn.Xp = c->xp_h; dn.rows = rows; dn.epi = EPI_RESID; dn.Y[0] = x; dn.ldy[0] = d; dn.seg_N[0] = d;
    // the draft layer's raw output is the first half of the next chained token's input [feature ;
    // embedding] and the LM head's operand: it goes straight into that packed buffer
    const bool draft_layer = li == g.n_layers;
    dn.Xp_out = draft_layer ? c->xp_cat : c->xp_a; dn.gain_out = next_gain; dn.ssq_out = c->ssq_a;
    dn.gate = c->gate;
    launch_gemm_mfma(dn, s);
    c->Pa = Pd;
    return;
  }
  launch_rmsnorm(x, w.attn_norm, rows, d, g.rms_eps, c->xn, s, c->gate);
  gemm(c, w.wq, c->xn, d, rows, nullptr, c->q, dq, 0);
  gemm(c, w.wk, c->xn, d, rows, nullptr, c->kbuf, dkv, 0);
  gemm(c, w.wv, c->xn, d, rows, nullptr, c->vbuf, dkv, 0);
  launch_rope_append(c->q, c->kbuf, c->vbuf, rows, pos0, g, c->rope_tab, kv_layer_ptr(c, li), c->kv_v_offset, false, s,
                     c->gate);
  launch_attention(c->q, rows, pos0, g, kv_layer_ptr(c, li), c->kv_v_offset, c->attn_part, c->att, s, c->gate);
  gemm(c, w.wo, c->att, dq, rows, nullptr, x, d, 1);
  launch_rmsnorm(x, w.ffn_norm, rows, d, g.rms_eps, c->xn, s, c->gate);
  gemm(c, w.w_gate, c->xn, d, rows, nullptr, c->gate_proj, f, 0);
  gemm(c, w.w_up, c->xn, d, rows, nullptr, c->up, f, 0);
  launch_silu_mul(c->gate_proj, c->up, rows, f, c->hmid, s, c->gate);
  gemm(c, w.w_down, c->hmid, f, rows, nullptr, x, d, 1);
}

// Target forward of `rows` tokens (device ids) at slots pos0..; features -> F rows 0..rows-1;
// logits (+ per-row argmax into st->argmax) for rows >= logit_from.
void target_forward(ae_ctx *c, const int32_t *ids_dev, int rows, int pos0, int logit_from) {
  const ae_config &g = c->cfg;
  hipStream_t s = c->stream;
  const int nr = rows - logit_from;
  if (c->fast) {
    launch_embed_packed(c->tok_emb, ids_dev, rows, g.d_model, c->layers[0].attn_norm, c->x, c->xp_a, c->ssq_a, s);
    c->Pa = 1;
    for (int l = 0; l < g.n_layers; ++l)
      run_layer(c, l, c->x, rows, pos0, l + 1 < g.n_layers ? c->layers[l + 1].attn_norm : c->final_norm);
    launch_rmsnorm(c->x, c->final_norm, rows, g.d_model, g.rms_eps, c->F, s);   // feature rows (LDLP, draft head)
    if (nr > 0) {
      GemmLaunch lm;   // final RMSNorm folded into the LM head
      lm.W = &c->lm_head; lm.Xp = c->xp_a; lm.rows = nr; lm.row0 = logit_from; lm.ssq_in = c->ssq_a; lm.P_in = c->Pa;
      lm.eps = g.rms_eps; lm.epi = EPI_STORE; lm.Y[0] = c->logits; lm.ldy[0] = g.vocab; lm.seg_N[0] = g.vocab;
      lm.amax_val = c->amax_val; lm.amax_idx = c->amax_idx;   // per-row argmax rides on the epilogue
      launch_gemm_mfma(lm, s);
      launch_argmax_finish(c->amax_val, c->amax_idx, g.vocab / 16, nr, c->st, -1, s);
    }
    return;
  }
  launch_embed(c->tok_emb, g.dtype, ids_dev, rows, g.d_model, c->x, s);
  for (int l = 0; l < g.n_layers; ++l) run_layer(c, l, c->x, rows, pos0, nullptr);
  launch_rmsnorm(c->x, c->final_norm, rows, g.d_model, g.rms_eps, c->F, s);
  if (nr > 0) {
    gemm(c, c->lm_head, c->F + (size_t)logit_from * g.d_model, g.d_model, nr, nullptr, c->logits, g.vocab, 0);
    launch_argmax(c->logits, nr, g.vocab, c->st->argmax, s);
  }
}

// Draft head over `rows` slots from slot0: slot input = fc([feature ; emb(next token)]).
// Leaves the head's outputs in x rows 0..rows-1 (bf16 path: also packed in xp_cat, first half).
// chained_row >= 0 (bf16 path, one row): the input is already in row chained_row of xp_cat, the
// head's previous output (left there by its down projection) and the embedding of the token
// picked from it (left there by the kernel that picked it).
void draft_rows(ae_ctx *c, const float *feat, int feat_ld, const int32_t *next_ids_dev, int rows, int slot0,
                int chained_row = -1) {
  const ae_config &g = c->cfg;
  hipStream_t s = c->stream;
  const LayerW &dl = c->layers[g.n_layers];
  if (c->fast) {
    if (chained_row < 0)
      launch_draft_cat_packed(feat, feat_ld, c->tok_emb, next_ids_dev, rows, g.d_model, c->xp_cat, s, c->gate);
    GemmLaunch fc;
    fc.W = &c->draft_fc; fc.Xp = c->xp_cat; fc.rows = rows; fc.epi = EPI_STORE; fc.bias = c->draft_fc_b;
    fc.row0 = chained_row < 0 ? 0 : chained_row;
    fc.Y[0] = c->x; fc.ldy[0] = g.d_model; fc.seg_N[0] = g.d_model;
    fc.Xp_out = c->xp_a; fc.gain_out = dl.attn_norm; fc.ssq_out = c->ssq_a;
    fc.gate = c->gate;
    launch_gemm_mfma(fc, s);
    c->Pa = g.d_model / 16;
    run_layer(c, g.n_layers, c->x, rows, slot0, nullptr);   // leaves packed(raw output) in xp_a
    return;
  }
  launch_draft_cat(feat, feat_ld, c->tok_emb, g.dtype, next_ids_dev, rows, g.d_model, c->cat, s, c->gate);
  gemm(c, c->draft_fc, c->cat, 2 * g.d_model, rows, c->draft_fc_b, c->x, g.d_model, 0);
  run_layer(c, g.n_layers, c->x, rows, slot0, nullptr);
}

// LM head (shared with the target) on draft-head output row `row` -> dlogits[i], then the
// head's token i: argmax (greedy) or an inverse-CDF sample driven by u_draft[i] (temperature
// > 0); the caller's override table is applied last.
void draft_lm_head(ae_ctx *c, int row, int i, int k) {
  const ae_config &g = c->cfg;
  hipStream_t s = c->stream;
  float *dl = c->dlogits + (size_t)i * g.vocab;
  const bool greedy = !(g.temperature > 0.f);
  if (c->fast) {
    GemmLaunch lm;
    lm.W = &c->lm_head; lm.Xp = c->xp_cat; lm.rows = 1; lm.row0 = row; lm.epi = EPI_STORE;
    lm.Y[0] = dl; lm.ldy[0] = g.vocab; lm.seg_N[0] = g.vocab;
    DddFinish ddd;   // the DDD rule's statistic rides on the LM-head epilogue and on the kernel that fixes the token
    if (g.ddd_enabled) {
      ddd.val = c->amax_val; ddd.lse_sum = c->lse_sum; ddd.logits = dl; ddd.NB = g.vocab / 16; ddd.k = k;
      ddd.inv_t = greedy ? 1.f : 1.f / g.temperature; ddd.theta = g.ddd_threshold;
      lm.lse_sum = c->lse_sum; lm.lse_inv_t = ddd.inv_t;
    }
    if (greedy || g.ddd_enabled) { lm.amax_val = c->amax_val; lm.amax_idx = c->amax_idx; }
    lm.gate = c->gate;
    launch_gemm_mfma(lm, s);
    DraftCat cat;   // the picked token's embedding joins the head's output in its packed input row
    cat.emb = c->tok_emb; cat.Xp = c->xp_cat; cat.d = g.d_model; cat.row = row;
    if (greedy) {
      launch_argmax_finish(c->amax_val, c->amax_idx, g.vocab / 16, 1, c->st, i, s, c->gate, cat, ddd);   // argmax + override
    } else {
      launch_sample_draft(dl, g.vocab, g.temperature, c->st, i, c->prob, s, c->gate);
      launch_pick_draft_packed(c->st, i, s, c->gate, cat, ddd);
    }
    return;
  }
  gemm(c, c->lm_head, c->x + (size_t)row * g.d_model, g.d_model, 1, nullptr, dl, g.vocab, 0);
  if (greedy) launch_argmax(dl, 1, g.vocab, c->st->argmax, s, c->gate);
  else launch_sample_draft(dl, g.vocab, g.temperature, c->st, i, c->prob, s, c->gate);
  launch_pick_draft(c->st, i, s, c->gate);
  if (g.ddd_enabled) launch_draft_logprob(dl, g.vocab, g.temperature, c->st, i, k, g.ddd_threshold, s, c->gate);
}

void enqueue_ldlp(ae_ctx *c, int slot, int f_row, bool relative_to_accept) {
  const ae_config &g = c->cfg;
  hipStream_t s = c->stream;
  launch_ldlp_in(c->ldlp_in.rowmajor, c->ldlp_b_in, c->tok_emb, g.dtype, c->hist, c->F, g.d_model, g.ldlp_in_mode,
                 g.ldlp_hidden, slot, f_row, relative_to_accept ? c->st : nullptr, c->ldlp_z, s);
  launch_ldlp_tail(c->ldlp_z, c->ldlp_w_res, g.dtype, c->ldlp_b_res, c->ldlp_w_out, c->ldlp_b_out, g.ldlp_hidden,
                   g.ldlp_n_res, g.k_max, g.ldlp_cls, c->st, c->h_st_dev, s);
}

// after a stream synchronisation: fold the finished event pairs into the totals
void drain_kernel_timing(ae_ctx *c) {
  for (int i = 0; i + 1 < c->kt_used; i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->kt_ev[i], c->kt_ev[i + 1]) == hipSuccess) {
      c->kt_total_us += (double)ms * 1e3;
      c->kt_count += 1;
    }
  }
  c->kt_used = 0;
}

// Bring the host's mirror of the device state up to date and wait for it.  The mirror is pinned
// host memory that the device writes itself; `published`: the last kernel enqueued (the LDLP
// tail) has already done so.
int read_state(ae_ctx *c, bool published = false) {
  if (!published) launch_publish_state(c->st, c->h_st_dev, c->stream);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipGetLastError());
  if (c->kt_used) drain_kernel_timing(c);
  return AE_OK;
}

// ---- dense prompt pass --------------------------------------------------------------
// the dense GEMM's workgroup tile spans 256 output rows
bool dense_ok(const ae_ctx *c) {
  const ae_config &g = c->cfg;
  return c->fast && g.d_model >= 256 && 2 * g.d_ffn >= 256 && (g.n_heads + 2 * g.n_kv_heads) * g.head_dim >= 256;
}

// Chunk buffers for `cap` rows (a multiple of 128): float residual stream and queries, the
// packed inputs of the five GEMMs, RMSNorm partial sums and 1/rms.  Zero-filled so that the
// padding rows of a chunk are finite.
int ensure_dense(ae_ctx *c, int n) {
  const ae_config &g = c->cfg;
  const int want = ((n < c->dense_chunk ? n : c->dense_chunk) + 127) / 128 * 128;
  if (want <= c->dense_cap) return AE_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (void *p : c->dense_owned) hipFree(p);
  c->dense_owned.clear();
  c->dense_cap = 0;
  const size_t cap = want, d = g.d_model, dq = (size_t)g.n_heads * g.head_dim, f = g.d_ffn;
  struct { void **p; size_t bytes; } bufs[] = {
      {(void **)&c->px, cap * d * 4},      {(void **)&c->pq, cap * dq * 4},   {(void **)&c->prinv, cap * 4},
      {(void **)&c->pssq_a, cap * d * 4 / 16 * 1 + cap * 4}, {(void **)&c->pssq_f, cap * d * 4 / 16 + cap * 4},
      {&c->pxa, cap * d * 4},              {&c->pxf, cap * d * 4},            {&c->pxatt, cap * dq * 4},
      {&c->pxh, cap * f * 4},              {&c->pxcat, cap * 2 * d * 4}};
  for (auto &b : bufs) {
    void *q = nullptr;
    const size_t bytes = (b.bytes + 255) / 256 * 256;
    hipError_t e = hipMalloc(&q, bytes);
    if (e != hipSuccess) return fail(c, AE_ENOMEM, std::string("dense prefill buffers: ") + hipGetErrorString(e));
    c->dense_owned.push_back(q);
    *b.p = q;
    launch_fill_zero(q, bytes, c->stream);
  }
  c->dense_cap = want;
  return AE_OK;
}

// Target layers over chunk rows [p0, p0+rows) and the draft head's K/V rows for the first
// `drows` of them (the slots whose next token is in the prompt).
void dense_chunk(ae_ctx *c, int p0, int rows, int drows) {
  const ae_config &g = c->cfg;
  hipStream_t s = c->stream;
  const int d = g.d_model, dq = g.n_heads * g.head_dim, dkv = g.n_kv_heads * g.head_dim, f = g.d_ffn;
  const int RB = c->dense_cap / 16, RBu = (rows + 15) / 16, Pd = d / 16, cap = kv_capacity(g);
  launch_embed_dense(c->tok_emb, c->hist + p0, rows, d, c->layers[0].attn_norm, c->px, c->pxa, RB, c->pssq_a, s);
  int Pa = 1;
  auto qkv_pass = [&](int li, int nrows) {
    const LayerW &w = c->layers[li];
    launch_rinv_finalize(c->pssq_a, (nrows + 15) / 16, Pa, d, g.rms_eps, c->prinv, s);
    GemmLaunch qkv;
    qkv.W = &w.f_qkv; qkv.Xp = c->pxa; qkv.rows = nrows; qkv.epi = EPI_QKV; qkv.nseg = 3;
    qkv.Y[0] = c->pq; qkv.ldy[0] = dq;
    qkv.seg_N[0] = dq; qkv.seg_N[1] = dkv; qkv.seg_N[2] = dkv;
    qkv.rope_tab = c->rope_tab; qkv.Kc = kv_layer_ptr(c, li); qkv.Vc = (char *)kv_layer_ptr(c, li) + c->kv_v_offset;
    qkv.pos0 = p0; qkv.n_ctx = cap; qkv.hd = g.head_dim;
    launch_gemm_dense(qkv, RB, c->prinv, s);
  };
  for (int l = 0; l < g.n_layers; ++l) {
    const LayerW &w = c->layers[l];
    qkv_pass(l, rows);
    launch_attention_prefill(c->pq, rows, p0, g, kv_layer_ptr(c, l), c->kv_v_offset, c->pxatt, RB, s);
    GemmLaunch o;
    o.W = &w.wo; o.Xp = c->pxatt; o.rows = rows; o.epi = EPI_RESID; o.Y[0] = c->px; o.ldy[0] = d; o.seg_N[0] = d;
    o.Xp_out = c->pxf; o.gain_out = w.ffn_norm; o.ssq_out = c->pssq_f;
    launch_gemm_dense(o, RB, nullptr, s);
    launch_rinv_finalize(c->pssq_f, RBu, Pd, d, g.rms_eps, c->prinv, s);
    GemmLaunch gu;
    gu.W = &w.f_gu; gu.Xp = c->pxf; gu.rows = rows; gu.epi = EPI_SWIGLU; gu.Xp_out = c->pxh; gu.seg_N[0] = 2 * f;
    launch_gemm_dense(gu, RB, c->prinv, s);
    GemmLaunch dn;
    dn.W = &w.w_down; dn.Xp = c->pxh; dn.rows = rows; dn.epi = EPI_RESID; dn.Y[0] = c->px; dn.ldy[0] = d; dn.seg_N[0] = d;
    dn.Xp_out = c->pxa; dn.gain_out = l + 1 < g.n_layers ? c->layers[l + 1].attn_norm : c->final_norm;
    dn.ssq_out = c->pssq_a;
    launch_gemm_dense(dn, RB, nullptr, s);
    Pa = Pd;
  }
  if (drows > 0) {
    // Eq. 2 catch-up of prompt slots: only the head's K/V rows are ever read again
    const LayerW &dl = c->layers[g.n_layers];
    launch_draft_cat_dense(c->px, drows, d, c->final_norm, g.rms_eps, c->tok_emb, c->hist + p0 + 1, c->pxcat, RB, s);
    GemmLaunch fc;
    fc.W = &c->draft_fc; fc.Xp = c->pxcat; fc.rows = drows; fc.epi = EPI_STORE; fc.bias = c->draft_fc_b;
    fc.seg_N[0] = d; fc.ldy[0] = d;
    fc.Xp_out = c->pxa; fc.gain_out = dl.attn_norm; fc.ssq_out = c->pssq_a;
    launch_gemm_dense(fc, RB, nullptr, s);
    Pa = Pd;
    qkv_pass(g.n_layers, drows);
  }
}

// Whole prompt through the dense pass; leaves the last position's feature in F row
// (n-1) % 16 (where the 16-row path leaves it) and its logits / argmax in row 0.
int prefill_dense(ae_ctx *c, int n) {
  const ae_config &g = c->cfg;
  hipStream_t s = c->stream;
  int rc = ensure_dense(c, n);
  if (rc) return rc;
  int last_rows = 0;
  for (int p0 = 0; p0 < n; p0 += c->dense_cap) {
    const int rows = n - p0 < c->dense_cap ? n - p0 : c->dense_cap;
    const bool last = p0 + rows == n;
    dense_chunk(c, p0, rows, last ? rows - 1 : rows);
    last_rows = rows;
  }
  const int frow = (n - 1) % kMaxRows;
  float *F = c->F + (size_t)frow * g.d_model;
  launch_rmsnorm(c->px + (size_t)(last_rows - 1) * g.d_model, c->final_norm, 1, g.d_model, g.rms_eps, F, s);
  launch_pack_rows(F, g.d_model, 1, g.d_model, nullptr, c->xp_a, s);
  GemmLaunch lm;
  lm.W = &c->lm_head; lm.Xp = c->xp_a; lm.rows = 1; lm.epi = EPI_STORE;
  lm.Y[0] = c->logits; lm.ldy[0] = g.vocab; lm.seg_N[0] = g.vocab;
  lm.amax_val = c->amax_val; lm.amax_idx = c->amax_idx;
  launch_gemm_mfma(lm, s);
  launch_argmax_finish(c->amax_val, c->amax_idx, g.vocab / 16, 1, c->st, -1, s);
  c->nF = frow + 1;
  return AE_OK;
}

__global__ void finish_prefill_kernel(DevState *st, int32_t *hist, int n) {
  hist[n] = st->argmax[0];
  st->bonus = st->argmax[0];
  st->n_acc = 0;
}

// Asymmetric L1 criterion of the LDLP (Sec. 3.3): per pair lambda*|p - t| where the prediction
// is short of the optimal length, |p - t| otherwise; float64, one workgroup, fixed-shape tree.
__global__ __launch_bounds__(256) void ldlp_loss_kernel(const float *pred, const int32_t *truth, int n, double lambda,
                                                        double *out) {
  __shared__ double sh[256];
  double tot = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) {
    const double diff = (double)pred[i] - (double)truth[i];
    tot += diff < 0.0 ? lambda * -diff : diff;
  }
  sh[threadIdx.x] = tot;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = n > 0 ? sh[0] / (double)n : 0.0;
}

// The matrix-core attention multiplies the V rows of masked keys by an exact zero, so every
// cache row, live or dead, has to hold finite values.
bool all_finite(const float *p, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (!(p[i] - p[i] == 0.0f)) return false;
  return true;
}

bool ids_ok(const ae_ctx *c, const int32_t *ids, int n) {
  for (int i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= c->cfg.vocab) return false;
  return true;
}

}  // namespace

extern "C" {

const char *ae_version(void) { return "adaeagle-gfx950 0.1"; }

const char *ae_last_error(const ae_ctx *ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

int ae_init(const ae_config *cfg, const ae_weights *w, void *hip_stream, ae_ctx **out) {
  if (out) *out = nullptr;
  if (!cfg || !w || !out) return fail(nullptr, AE_EINVAL, "ae_init: NULL argument");
  const ae_config &g = *cfg;
  if (g.n_layers < 1 || g.d_model < 8 || g.n_heads < 1 || g.n_kv_heads < 1 || g.d_ffn < 8 || g.vocab < 1 ||
      g.n_heads % g.n_kv_heads != 0 || g.k_max < 0 || g.n_ctx_max < 1 || g.ldlp_hidden < 1 || g.ldlp_n_res < 0 ||
      (g.dtype != AE_BF16 && g.dtype != AE_FP32) || (g.ldlp_in_mode != 0 && g.ldlp_in_mode != 1) ||
      !(g.temperature >= 0.f) || !(g.rms_eps >= 0.f) || !(g.rope_base > 0.f) ||
      (g.ddd_enabled != 0 && g.ddd_enabled != 1) || (g.ddd_enabled && !(g.ddd_threshold == g.ddd_threshold)) ||
      (g.ldlp_cls != 0 && g.ldlp_cls != 1))
    return fail(nullptr, AE_EINVAL, "ae_init: configuration field out of range");
  if (g.head_dim != 64 && g.head_dim != 128) return fail(nullptr, AE_EUNSUPPORTED, "head_dim must be 64 or 128");
  if (g.k_max + 1 > kMaxRows) return fail(nullptr, AE_EUNSUPPORTED, "k_max must be <= 15");
  if (g.d_model % 8 || g.d_ffn % 8 || g.ldlp_hidden % 8 || g.ldlp_hidden > kMaxLdlpHidden)
    return fail(nullptr, AE_EUNSUPPORTED, "d_model, d_ffn, ldlp_hidden must be multiples of 8 (ldlp_hidden <= 1024)");
  if ((g.n_heads / g.n_kv_heads) * kMaxRows > 64)
    return fail(nullptr, AE_EUNSUPPORTED, "n_heads / n_kv_heads must be <= 4");
  if (g.temperature > 0.f && g.vocab > 1024 * 1024)
    return fail(nullptr, AE_EUNSUPPORTED, "temperature > 0 supports vocabularies of up to 1048576 tokens");
  if (g.n_ctx_max > kMaxSplits * kAttnChunk) return fail(nullptr, AE_EUNSUPPORTED, "n_ctx_max too large (<= 16384)");
  if (!w->tok_emb || !w->final_norm || !w->lm_head || !w->layers || !w->draft_fc_w || !w->ldlp_w_in ||
      !w->ldlp_b_in || !w->ldlp_w_out || !w->ldlp_b_out || (g.ldlp_n_res > 0 && (!w->ldlp_w_res || !w->ldlp_b_res)))
    return fail(nullptr, AE_EINVAL, "ae_init: NULL weight pointer");

  ae_ctx *c = new (std::nothrow) ae_ctx();
  if (!c) return fail(nullptr, AE_ENOMEM, "out of host memory");
  c->cfg = g;
  c->stream = (hipStream_t)hip_stream;
  int rc = AE_OK;
  auto bail = [&](int code) { g_init_error = c->err; ae_free(c); return code; };
  if (hipGetDevice(&c->device) != hipSuccess) { c->err = "hipGetDevice failed (no GPU?)"; return bail(AE_EHIP); }
  {
    hipError_t e = static_stage(c->device, &c->kv_stage);
    if (e != hipSuccess) { c->err = std::string("hipGetSymbolAddress(kv stage): ") + hipGetErrorString(e); return bail(AE_EHIP); }
  }

  const int d = g.d_model, dq = g.n_heads * g.head_dim, dkv = g.n_kv_heads * g.head_dim, f = g.d_ffn, V = g.vocab;
  auto conv_layer = [&](const ae_layer_w &s, LayerW &o) -> bool {
    if (!s.attn_norm || !s.wq || !s.wk || !s.wv || !s.wo || !s.ffn_norm || !s.w_gate || !s.w_up || !s.w_down) return false;
    o.attn_norm = s.attn_norm; o.ffn_norm = s.ffn_norm;
    o.wq = make_mat(s.wq, dq, d); o.wk = make_mat(s.wk, dkv, d); o.wv = make_mat(s.wv, dkv, d);
    o.wo = make_mat(s.wo, d, dq); o.w_gate = make_mat(s.w_gate, f, d); o.w_up = make_mat(s.w_up, f, d);
    o.w_down = make_mat(s.w_down, d, f);
    return true;
  };
  c->layers.resize(g.n_layers + 1);
  for (int l = 0; l < g.n_layers; ++l)
    if (!conv_layer(w->layers[l], c->layers[l])) { c->err = "ae_init: NULL layer weight"; return bail(AE_EINVAL); }
  if (!conv_layer(w->draft_layer, c->layers[g.n_layers])) { c->err = "ae_init: NULL draft layer weight"; return bail(AE_EINVAL); }
  c->tok_emb = w->tok_emb; c->final_norm = w->final_norm;
  c->lm_head = make_mat(w->lm_head, V, d);
  c->draft_fc = make_mat(w->draft_fc_w, d, 2 * d);
  c->draft_fc_b = w->draft_fc_b;
  c->ldlp_in = make_mat(w->ldlp_w_in, g.ldlp_hidden, g.ldlp_in_mode == 0 ? 2 * d : d);
  c->ldlp_b_in = w->ldlp_b_in; c->ldlp_w_res = w->ldlp_w_res; c->ldlp_b_res = w->ldlp_b_res;
  c->ldlp_w_out = w->ldlp_w_out; c->ldlp_b_out = w->ldlp_b_out;

  // bf16: re-tile every streamed matrix into the MFMA operand layout (see kernels_mfma.hip)
  c->fast = g.dtype == AE_BF16;
  if (c->fast) {
    attention_mfma_setup();
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess) gemm_mfma_setup(cus);
    bool ok = tileable(c->lm_head) && tileable(c->draft_fc) && g.head_dim % 32 == 0;
    for (auto &l : c->layers)
      ok = ok && tileable(l.wq) && tileable(l.wk) && tileable(l.wv) && tileable(l.wo) && tileable(l.w_gate) &&
           tileable(l.w_up) && tileable(l.w_down);
    if (!ok) {
      c->err = "bf16 matrices need out_features % 16 == 0 and in_features % 256 == 0";
      return bail(AE_EUNSUPPORTED);
    }
    const Mat *one[1];
    one[0] = &c->lm_head;
    Mat lm = c->lm_head;
    if ((rc = retile_fused(c, lm, one, 1, false))) return bail(rc);
    c->lm_head.tiled = lm.tiled;
    one[0] = &c->draft_fc;
    Mat fc = c->draft_fc;
    if ((rc = retile_fused(c, fc, one, 1, false))) return bail(rc);
    c->draft_fc.tiled = fc.tiled;
    for (auto &l : c->layers) {
      const Mat *qkv[3] = {&l.wq, &l.wk, &l.wv};
      const Mat *gu[2] = {&l.w_gate, &l.w_up};
      Mat t;
      if ((rc = retile_fused(c, l.f_qkv, qkv, 3, false, 2)) || (rc = retile_fused(c, l.f_gu, gu, 2, true))) return bail(rc);
      one[0] = &l.wo; t = l.wo;
      if ((rc = retile_fused(c, t, one, 1, false))) return bail(rc);
      l.wo.tiled = t.tiled;
      one[0] = &l.w_down; t = l.w_down;
      if ((rc = retile_fused(c, t, one, 1, false))) return bail(rc);
      l.w_down.tiled = t.tiled;
    }
    // packed activation buffers: K * 64 bytes each (hi + lo, 16 row slots)
    const size_t dqq = (size_t)g.n_heads * g.head_dim;
    char *pa = nullptr, *pf = nullptr, *pt = nullptr, *ph = nullptr, *pc = nullptr;
    if ((rc = dev_alloc(c, &pa, (size_t)g.d_model * 64)) || (rc = dev_alloc(c, &pf, (size_t)g.d_model * 64)) ||
        (rc = dev_alloc(c, &pt, dqq * 64)) || (rc = dev_alloc(c, &ph, (size_t)g.d_ffn * 64)) ||
        (rc = dev_alloc(c, &pc, (size_t)2 * g.d_model * 64)) ||
        (rc = dev_alloc(c, &c->ssq_a, (size_t)g.d_model)) || (rc = dev_alloc(c, &c->ssq_f, (size_t)g.d_model)) ||
        (rc = dev_alloc(c, &c->amax_val, (size_t)g.vocab)) || (rc = dev_alloc(c, &c->amax_idx, (size_t)g.vocab)) ||
        (rc = dev_alloc(c, &c->lse_sum, (size_t)g.vocab)))
      return bail(rc);
    c->xp_a = pa; c->xp_f = pf; c->xp_att = pt; c->xp_h = ph; c->xp_cat = pc;
    launch_fill_zero(pa, (size_t)g.d_model * 64, c->stream);
    launch_fill_zero(pf, (size_t)g.d_model * 64, c->stream);
    launch_fill_zero(pt, dqq * 64, c->stream);
    launch_fill_zero(ph, (size_t)g.d_ffn * 64, c->stream);
    launch_fill_zero(pc, (size_t)2 * g.d_model * 64, c->stream);
    launch_fill_zero(c->ssq_a, (size_t)g.d_model * 4, c->stream);
    launch_fill_zero(c->ssq_f, (size_t)g.d_model * 4, c->stream);
  }

  // KV cache for n_layers target layers + the draft layer, zero-filled so that slots that
  // were never written hold finite values
  c->kv_layer_stride = kv_layer_bytes(g);
  c->kv_v_offset = kv_v_offset_bytes(g);
  const size_t kv_bytes = c->kv_layer_stride * (size_t)(g.n_layers + 1);
  char *kvp = nullptr;
  if ((rc = dev_alloc(c, &kvp, kv_bytes))) return bail(rc);
  c->kv = kvp;
  launch_fill_zero(c->kv, (kv_bytes + 15) / 16 * 16, c->stream);

  const size_t R = kMaxRows;
  const int dmax = dq > d ? dq : d;
  if ((rc = dev_alloc(c, &c->rope_tab, (size_t)g.n_ctx_max * (g.head_dim / 2))) ||
      (rc = dev_alloc(c, &c->x, R * d)) || (rc = dev_alloc(c, &c->xn, R * d)) ||
      (rc = dev_alloc(c, &c->q, R * dq)) || (rc = dev_alloc(c, &c->kbuf, R * dkv)) ||
      (rc = dev_alloc(c, &c->vbuf, R * dkv)) || (rc = dev_alloc(c, &c->att, R * dmax)) ||
      (rc = dev_alloc(c, &c->gate_proj, R * f)) || (rc = dev_alloc(c, &c->up, R * f)) ||
      (rc = dev_alloc(c, &c->hmid, R * f)) || (rc = dev_alloc(c, &c->F, R * d)) ||
      (rc = dev_alloc(c, &c->cat, R * 2 * d)) || (rc = dev_alloc(c, &c->logits, (size_t)(g.k_max + 1) * V)) ||
      (rc = dev_alloc(c, &c->dlogits, (size_t)(g.k_max > 0 ? g.k_max : 1) * V)) ||
      (rc = dev_alloc(c, &c->attn_part, attn_part_floats(g))) ||
      (rc = dev_alloc(c, &c->ldlp_z, (size_t)kMaxLdlpHidden)) ||
      (rc = dev_alloc(c, &c->hist, (size_t)g.n_ctx_max + 2)) || (rc = dev_alloc(c, &c->st, 1)) ||
      (rc = dev_alloc(c, &c->prob, sample_scratch_doubles(g.vocab))))
    return bail(rc);
  launch_rope_table(c->rope_tab, g.n_ctx_max, g.head_dim, g.rope_base, c->stream);
  launch_fill_zero(c->st, (sizeof(DevState) + 15) / 16 * 16, c->stream);
  launch_fill_zero(c->hist, ((size_t)(g.n_ctx_max + 2) * 4 + 15) / 16 * 16, c->stream);
  if (hipHostMalloc((void **)&c->h_st, sizeof(DevState), hipHostMallocMapped) != hipSuccess) {
    c->err = "hipHostMalloc failed";
    return bail(AE_ENOMEM);
  }
  memset(c->h_st, 0, sizeof(DevState));
  if (hipHostGetDevicePointer((void **)&c->h_st_dev, c->h_st, 0) != hipSuccess) {
    c->err = "hipHostGetDevicePointer failed";
    return bail(AE_EHIP);
  }
  for (auto &e : c->ev)
    if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) { c->err = "hipEventCreate failed"; return bail(AE_EHIP); }
  c->h_hist.assign((size_t)g.n_ctx_max + 2, 0);
  c->h_block.assign(kMaxRows, 0);
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) { c->err = std::string("ae_init: ") + hipGetErrorString(e); return bail(AE_EHIP); }
  *out = c;
  return AE_OK;
}

void ae_free(ae_ctx *c) {
  if (!c) return;
  hipStreamSynchronize(c->stream);
  for (void *p : c->owned) hipFree(p);
  for (void *p : c->dense_owned) hipFree(p);
  if (c->h_st) hipHostFree(c->h_st);
  for (auto &e : c->ev)
    if (e) hipEventDestroy(e);
  for (auto &e : c->kt_ev) hipEventDestroy(e);
  delete c;
}

int ae_prefill(ae_ctx *c, const int32_t *ids, int n) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (!ids || n < 1) return fail(c, AE_EINVAL, "ae_prefill: empty prompt");
  if (n + g.k_max + 1 > g.n_ctx_max) return fail(c, AE_EINVAL, "ae_prefill: prompt does not fit n_ctx_max");
  if (!ids_ok(c, ids, n)) return fail(c, AE_EINVAL, "ae_prefill: token id out of range");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(c->hist, ids, sizeof(int32_t) * n, hipMemcpyHostToDevice));
  memcpy(c->h_hist.data(), ids, sizeof(int32_t) * n);
  c->kv_len = 0; c->dlen = 0; c->nF = 0;
  c->have_pending = c->have_draft = c->have_verify = c->k_next_valid = false;
  const bool dense = c->prefill_mode == AE_PREFILL_DENSE || (c->prefill_mode == AE_PREFILL_AUTO && dense_ok(c) && n >= kDenseMinPrompt);
  if (dense) {
    int rc = prefill_dense(c, n);
    if (rc) return rc;
  } else {
    for (int p0 = 0; p0 < n; p0 += kMaxRows) {
      const int rows = n - p0 < kMaxRows ? n - p0 : kMaxRows;
      const bool last = p0 + rows == n;
      // keep the number of launches in flight bounded (a block is ~200 launches): tools that
      // keep a record per outstanding dispatch have been seen to fail on tens of thousands
      if (p0 > 0 && (p0 / kMaxRows) % 16 == 0) HIPCHK(c, hipStreamSynchronize(c->stream));
      target_forward(c, c->hist + p0, rows, p0, last ? rows - 1 : rows);
      const int drows = last ? rows - 1 : rows;  // slots whose next token is in the prompt
      if (drows > 0) draft_rows(c, c->F, g.d_model, c->hist + p0 + 1, drows, p0);
      c->nF = rows;
    }
  }
  finish_prefill_kernel<<<1, 1, 0, c->stream>>>(c->st, c->hist, n);
  c->kv_len = n;
  c->dlen = n - 1;
  enqueue_ldlp(c, n - 1, c->nF - 1, false);
  int rc = read_state(c, true);
  if (rc) return rc;
  c->pending = c->h_st->bonus;
  c->h_hist[n] = c->pending;
  c->k_next = c->h_st->k_next; c->y_next = c->h_st->y_next; c->k_next_valid = true;
  c->have_pending = true;
  c->cur_k = 0;
  return AE_OK;
}

int ae_set_prefill_mode(ae_ctx *c, int mode, int chunk_rows) {
  if (!c) return AE_EINVAL;
  if (mode != AE_PREFILL_AUTO && mode != AE_PREFILL_BLOCKS && mode != AE_PREFILL_DENSE)
    return fail(c, AE_EINVAL, "ae_set_prefill_mode: unknown mode");
  if (chunk_rows != 0 && (chunk_rows < 128 || chunk_rows > 8192 || chunk_rows % 128))
    return fail(c, AE_EINVAL, "ae_set_prefill_mode: chunk_rows must be a multiple of 128 in [128, 8192]");
  if (mode == AE_PREFILL_DENSE && !dense_ok(c))
    return fail(c, AE_EUNSUPPORTED, "the dense prompt pass needs bf16 weights and d_model >= 256");
  c->prefill_mode = mode;
  if (chunk_rows && chunk_rows != c->dense_chunk) {
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (void *p : c->dense_owned) hipFree(p);
    c->dense_owned.clear();
    c->dense_cap = 0;
    c->dense_chunk = chunk_rows;
  }
  return AE_OK;
}

int ae_kv_import(ae_ctx *c, int layer, const float *k, const float *v, int n) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (layer < 0 || layer > g.n_layers || n < 0 || n > g.n_ctx_max || !k || !v)
    return fail(c, AE_EINVAL, "ae_kv_import: argument out of range");
  if (n == 0) return AE_OK;
  const size_t cnt = (size_t)n * g.n_kv_heads * g.head_dim;
  if (!all_finite(k, cnt) || !all_finite(v, cnt)) return fail(c, AE_EINVAL, "ae_kv_import: non-finite value");
  float *tmp = nullptr;
  HIPCHK(c, hipMalloc((void **)&tmp, 2 * cnt * sizeof(float)));
  hipError_t e = hipMemcpy(tmp, k, cnt * sizeof(float), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(tmp + cnt, v, cnt * sizeof(float), hipMemcpyHostToDevice);
  if (e == hipSuccess) {
    launch_kv_import(kv_layer_ptr(c, layer), c->kv_v_offset, g, tmp, tmp + cnt, n, c->fast, c->stream);
    e = hipStreamSynchronize(c->stream);
  }
  hipFree(tmp);
  if (e != hipSuccess) return fail(c, AE_EHIP, std::string("ae_kv_import: ") + hipGetErrorString(e));
  return AE_OK;
}

int ae_kv_import_static(ae_ctx *c, int layer, const float *k, const float *v, int n) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (layer < 0 || layer > g.n_layers || n < 0 || n > g.n_ctx_max || !k || !v)
    return fail(c, AE_EINVAL, "ae_kv_import_static: argument out of range");
  if (n == 0) return AE_OK;
  const size_t cnt = (size_t)n * g.n_kv_heads * g.head_dim;
  if (2 * cnt > kStageFloats)
    return fail(c, AE_EINVAL, "ae_kv_import_static: 2 * n * n_kv_heads * head_dim exceeds the " +
                                  std::to_string(kStageFloats) + "-float staging area (use fewer rows or ae_kv_import)");
  if (!all_finite(k, cnt) || !all_finite(v, cnt)) return fail(c, AE_EINVAL, "ae_kv_import_static: non-finite value");
  float *stage = c->kv_stage;   // this device's copy of the staging array
  // the previous user of the staging area (any ctx on this device) has finished: every call
  // returns only after its import kernel has completed
  HIPCHK(c, hipMemcpy(stage, k, cnt * sizeof(float), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(stage + cnt, v, cnt * sizeof(float), hipMemcpyHostToDevice));
  launch_kv_import(kv_layer_ptr(c, layer), c->kv_v_offset, g, stage, stage + cnt, n, c->fast, c->stream);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipGetLastError());
  return AE_OK;
}

int ae_set_state(ae_ctx *c, int kv_len, int32_t last_tok, int32_t pending, const float *feat) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (kv_len < 1 || kv_len + g.k_max + 1 > g.n_ctx_max || !feat) return fail(c, AE_EINVAL, "ae_set_state: bad kv_len");
  if (!ids_ok(c, &last_tok, 1) || !ids_ok(c, &pending, 1)) return fail(c, AE_EINVAL, "ae_set_state: id out of range");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(c->F, feat, sizeof(float) * g.d_model, hipMemcpyHostToDevice));
  const int32_t two[2] = {last_tok, pending};
  HIPCHK(c, hipMemcpy(c->hist + kv_len - 1, two, sizeof(two), hipMemcpyHostToDevice));
  c->h_hist[kv_len - 1] = last_tok; c->h_hist[kv_len] = pending;
  c->kv_len = kv_len; c->dlen = kv_len - 1; c->nF = 1; c->pending = pending;
  c->have_pending = true; c->have_draft = c->have_verify = false; c->k_next_valid = false; c->cur_k = 0;
  return AE_OK;
}

int ae_ldlp(ae_ctx *c, int *k_out, float *y_out) {
  if (!c) return AE_EINVAL;
  if (!k_out) return fail(c, AE_EINVAL, "ae_ldlp: NULL output");
  if (!c->have_pending || c->nF < 1) return fail(c, AE_ESTATE, "ae_ldlp: no validated token yet (prefill first)");
  if (!c->k_next_valid) {
    enqueue_ldlp(c, c->kv_len - 1, c->nF - 1, false);
    int rc = read_state(c, true);
    if (rc) return rc;
    c->k_next = c->h_st->k_next; c->y_next = c->h_st->y_next; c->k_next_valid = true;
  }
  *k_out = c->k_next;
  if (y_out) *y_out = c->y_next;
  return AE_OK;
}

int ae_draft(ae_ctx *c, int k, const int32_t *override_ids, const double *u_draft, int32_t *out) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (!c->have_pending) return fail(c, AE_ESTATE, "ae_draft: no pending token (prefill first)");
  if (k < 0 || k > g.k_max) return fail(c, AE_EINVAL, "ae_draft: k outside [0, k_max]");
  if (c->kv_len + g.k_max + 1 > g.n_ctx_max) return fail(c, AE_EINVAL, "ae_draft: KV capacity exceeded");
  const int n = c->kv_len, catch_rows = n - c->dlen;
  if (catch_rows < 1 || catch_rows > c->nF)
    return fail(c, AE_ESTATE, "ae_draft: draft cache is stale (target advanced without the draft head)");
  const int n_ov = g.ddd_enabled ? g.k_max : k;   // DDD may extend the draft up to k_max tokens
  if (override_ids)
    for (int i = 0; i < n_ov; ++i)
      if (override_ids[i] >= g.vocab) return fail(c, AE_EINVAL, "ae_draft: override id out of range");
  const bool sampling = g.temperature > 0.f;
  if (sampling && n_ov > 0 && !u_draft) return fail(c, AE_EINVAL, "ae_draft: temperature > 0 needs u_draft");
  if (sampling)
    for (int i = 0; i < n_ov; ++i)
      if (!(u_draft[i] >= 0.0 && u_draft[i] < 1.0)) return fail(c, AE_EINVAL, "ae_draft: u_draft outside [0,1)");
  hipStream_t s = c->stream;
  // override table (-1 = keep the head's own token), chain gate reset and the sampling uniforms
  launch_set_draft_inputs(c->st, override_ids, n_ov, sampling ? u_draft : nullptr, n_ov, s);
  // catch-up over the slots validated by the last accept: true feature + following token
  draft_rows(c, c->F + (size_t)(c->nF - catch_rows) * g.d_model, g.d_model, c->hist + c->dlen + 1, catch_rows, c->dlen);
  c->dlen = n;
  const float *fh = c->x + (size_t)(catch_rows - 1) * g.d_model;
  int fh_row = catch_rows - 1;
  // AdaEAGLE-DDD (Sec. 3.4, 4.2): past the predicted length the head exits unless the
  // log-probability of the tokens drafted so far is still at least the threshold.  Host mode
  // reads the running sum back before every such token; device mode enqueues all k_max tokens
  // and lets the kernels of the tokens past k return at entry once the device-side rule says
  // stop (the verify block is then padded to k_max + 1 rows and ae_accept takes the drafted
  // length from the device).
  const bool dev_rule = g.ddd_enabled && c->ddd_mode == AE_DDD_DEVICE;
  bool gated = false;
  int i = 0;
  for (; i < g.k_max; ++i) {
    if (i >= k) {
      if (!g.ddd_enabled) break;
      if (i == 0) {
        if (!(0.f >= g.ddd_threshold)) break;   // the empty sequence has log-probability 0
      } else if (dev_rule) {
        c->gate = &c->st->draft_live;
        gated = true;
      } else {
        c->gate = nullptr;
        int rc = read_state(c);
        if (rc) return rc;
        if (!(c->h_st->cum_logp >= g.ddd_threshold)) break;
      }
    }
    if (i > 0) {  // chain: the head's previous output replaces the feature
      draft_rows(c, fh, g.d_model, c->st->draft_ids + (i - 1), 1, n - 1 + i, c->fast ? fh_row : -1);
      fh = c->x;
      fh_row = 0;
    }
    draft_lm_head(c, fh_row, i, k);
  }
  c->gate = nullptr;
  k = i;   // tokens enqueued; with a gated tail the number drafted is st->draft_len <= k
  c->cur_k = k;
  c->cur_k_last = k;
  c->k_on_device = gated;
  c->have_draft = true;
  c->have_verify = false;
  if (out && k > 0) {
    int rc = read_state(c);
    if (rc) return rc;
    if (gated) {   // the caller synchronised anyway: from here on the host knows the length
      k = c->h_st->draft_len;
      c->cur_k = c->cur_k_last = k;
      c->k_on_device = false;
    }
    memcpy(out, c->h_st->draft_ids, sizeof(int32_t) * k);
  }
  return AE_OK;
}

int ae_verify(ae_ctx *c, const int32_t *block_ids, int rows) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (!c->have_pending) return fail(c, AE_ESTATE, "ae_verify: no pending token (prefill first)");
  if (rows < 1 || rows > g.k_max + 1) return fail(c, AE_EINVAL, "ae_verify: rows outside [1, k_max+1]");
  if (c->kv_len + rows > g.n_ctx_max) return fail(c, AE_EINVAL, "ae_verify: KV capacity exceeded");
  hipStream_t s = c->stream;
  if (block_ids) {
    if (!ids_ok(c, block_ids, rows)) return fail(c, AE_EINVAL, "ae_verify: token id out of range");
    launch_set_block(c->st, block_ids, rows, s);
  } else {
    if (!c->have_draft || rows != c->cur_k + 1)
      return fail(c, AE_ESTATE, "ae_verify: implicit block needs a draft of rows-1 tokens");
    launch_build_block(c->st, c->hist, c->kv_len, c->cur_k, s);
  }
  target_forward(c, c->st->block, rows, c->kv_len, 0);
  c->block_rows = rows;
  c->have_verify = true;
  return AE_OK;
}

int ae_accept(ae_ctx *c, const double *u, int *n_accepted, int32_t *bonus) {
  if (!c) return AE_EINVAL;
  if (!c->have_verify) return fail(c, AE_ESTATE, "ae_accept: nothing verified");
  const ae_config &g = c->cfg;
  const int n = c->kv_len, rows = c->block_rows;
  if (g.temperature > 0.f) {
    if (!u) return fail(c, AE_EINVAL, "ae_accept: temperature > 0 needs the uniforms u");
    if (rows > 1 && !c->have_draft) return fail(c, AE_ESTATE, "ae_accept: rejection sampling needs the draft's own logits");
    for (int i = 0; i < rows; ++i)
      if (!(u[i] >= 0.0 && u[i] < 1.0)) return fail(c, AE_EINVAL, "ae_accept: u outside [0,1)");
    launch_set_u_accept(c->st, u, rows, c->stream);
    launch_accept_sample(c->logits, c->dlogits, g.vocab, rows - 1, c->k_on_device, g.temperature, c->st, c->hist, n,
                         c->prob, c->stream);
  } else {
    launch_accept_greedy(c->st, c->hist, n, rows, c->k_on_device, c->stream);
  }
  // Alg. 1 predicts the next draft length right after the verification
  const bool spec = c->have_draft;
  if (spec) enqueue_ldlp(c, n, 0, true);
  int rc = read_state(c, spec);
  if (rc) return rc;
  const int acc = c->h_st->n_acc;
  for (int i = 0; i <= acc; ++i) c->h_hist[n + i] = c->h_st->block[i];
  c->kv_len = n + 1 + acc;   // rollback: rows beyond the accepted prefix are dead
  c->pending = c->h_st->bonus;
  c->h_hist[c->kv_len] = c->pending;
  memcpy(c->h_block.data(), c->h_st->block, sizeof(int32_t) * kMaxRows);
  c->nF = acc + 1;
  if (c->k_on_device) c->cur_k_last = c->h_st->draft_len;   // padded block: the drafted length arrives here
  c->k_on_device = false;
  c->have_verify = c->have_draft = false;
  c->cur_k = 0;
  c->k_next_valid = spec;
  if (spec) { c->k_next = c->h_st->k_next; c->y_next = c->h_st->y_next; }
  if (n_accepted) *n_accepted = acc;
  if (bonus) *bonus = c->pending;
  return AE_OK;
}

int ae_step(ae_ctx *c, ae_step_io *io) {
  if (!c) return AE_EINVAL;
  if (!io) return fail(c, AE_EINVAL, "ae_step: NULL io");
  const auto t0 = std::chrono::steady_clock::now();
  const bool prof = c->profiling;
  hipStream_t s = c->stream;
  int rc, k = 0;
  if (prof) hipEventRecord(c->ev[0], s);
  if (io->k_force >= 0) {
    k = io->k_force;
  } else if ((rc = ae_ldlp(c, &k, nullptr))) {
    return rc;
  }
  if (prof) hipEventRecord(c->ev[1], s);
  if ((rc = ae_draft(c, k, io->override_ids, io->u_draft, nullptr))) return rc;
  k = c->cur_k;   // the DDD rule may have extended the draft (device rule: padded to k_max)
  if (prof) hipEventRecord(c->ev[2], s);
  if ((rc = ae_verify(c, nullptr, k + 1))) return rc;
  if (prof) hipEventRecord(c->ev[3], s);
  int acc = 0;
  int32_t b = 0;
  if ((rc = ae_accept(c, io->u_accept, &acc, &b))) return rc;
  if (prof) {
    hipEventRecord(c->ev[4], s);
    hipEventSynchronize(c->ev[4]);
    float ms[4] = {0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) hipEventElapsedTime(&ms[i], c->ev[i], c->ev[i + 1]);
    c->last_times = {ms[0] * 1e3f, ms[1] * 1e3f, ms[2] * 1e3f, ms[3] * 1e3f};
  }
  io->k = c->cur_k_last;
  io->n_accepted = acc;
  io->n_tokens = acc + 1;
  for (int i = 0; i < acc; ++i) io->tokens[i] = c->h_block[1 + i];
  io->tokens[acc] = b;
  io->us_total = std::chrono::duration<float, std::micro>(std::chrono::steady_clock::now() - t0).count();
  return AE_OK;
}

int ae_ldlp_loss(ae_ctx *c, const float *pred, const int32_t *truth, int n, double lambda, double *out) {
  if (!c) return AE_EINVAL;
  if (n < 0 || (n > 0 && (!pred || !truth)) || !out || !(lambda >= 0.0))
    return fail(c, AE_EINVAL, "ae_ldlp_loss: argument out of range");
  if (n == 0) { *out = 0.0; return AE_OK; }
  char *buf = nullptr;
  const size_t off_t = ((size_t)n * 4 + 15) / 16 * 16, off_o = 2 * off_t;
  HIPCHK(c, hipMalloc((void **)&buf, off_o + 16));
  hipError_t e = hipMemcpy(buf, pred, (size_t)n * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(buf + off_t, truth, (size_t)n * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) {
    ldlp_loss_kernel<<<1, 256, 0, c->stream>>>((const float *)buf, (const int32_t *)(buf + off_t), n, lambda,
                                               (double *)(buf + off_o));
    e = hipStreamSynchronize(c->stream);
  }
  if (e == hipSuccess) e = hipMemcpy(out, buf + off_o, sizeof(double), hipMemcpyDeviceToHost);
  hipFree(buf);
  if (e != hipSuccess) return fail(c, AE_EHIP, std::string("ae_ldlp_loss: ") + hipGetErrorString(e));
  return AE_OK;
}

int ae_set_ddd_mode(ae_ctx *c, int mode) {
  if (!c) return AE_EINVAL;
  if (mode != AE_DDD_HOST && mode != AE_DDD_DEVICE) return fail(c, AE_EINVAL, "ae_set_ddd_mode: unknown mode");
  if (c->have_draft) return fail(c, AE_ESTATE, "ae_set_ddd_mode: a draft is pending (accept first)");
  c->ddd_mode = mode;
  return AE_OK;
}

int ae_set_temperature(ae_ctx *c, float temperature) {
  if (!c) return AE_EINVAL;
  if (!(temperature >= 0.f) || temperature > 3.0e38f) return fail(c, AE_EINVAL, "ae_set_temperature: negative or non-finite");
  if (temperature > 0.f && c->cfg.vocab > 1024 * 1024)
    return fail(c, AE_EUNSUPPORTED, "temperature > 0 supports vocabularies of up to 1048576 tokens");
  if (c->have_draft || c->have_verify) return fail(c, AE_ESTATE, "ae_set_temperature: a step is in flight (accept first)");
  c->cfg.temperature = temperature;
  return AE_OK;
}

int ae_kv_len(const ae_ctx *c) { return c ? c->kv_len : AE_EINVAL; }
int ae_last_draft_len(const ae_ctx *c) { return c ? c->cur_k_last : AE_EINVAL; }

int ae_get_draft_logprob(ae_ctx *c, float *out) {
  if (!c) return AE_EINVAL;
  if (!out) return fail(c, AE_EINVAL, "ae_get_draft_logprob: NULL output");
  int rc = read_state(c);
  if (rc) return rc;
  *out = c->h_st->cum_logp;
  return AE_OK;
}
int32_t ae_pending(const ae_ctx *c) { return c && c->have_pending ? c->pending : -1; }

static int copy_out(ae_ctx *c, const float *src, size_t n, float *dst) {
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(dst, src, n * sizeof(float), hipMemcpyDeviceToHost));
  return AE_OK;
}

int ae_get_logits(ae_ctx *c, int row, float *out) {
  if (!c) return AE_EINVAL;
  if (!out || row < 0 || row > c->cfg.k_max) return fail(c, AE_EINVAL, "ae_get_logits: bad row");
  return copy_out(c, c->logits + (size_t)row * c->cfg.vocab, c->cfg.vocab, out);
}

int ae_get_feature(ae_ctx *c, int row, float *out) {
  if (!c) return AE_EINVAL;
  if (!out || row < 0 || row >= kMaxRows) return fail(c, AE_EINVAL, "ae_get_feature: bad row");
  return copy_out(c, c->F + (size_t)row * c->cfg.d_model, c->cfg.d_model, out);
}

int ae_get_draft_logits(ae_ctx *c, int i, float *out) {
  if (!c) return AE_EINVAL;
  if (!out || i < 0 || i >= c->cfg.k_max) return fail(c, AE_EINVAL, "ae_get_draft_logits: bad index");
  return copy_out(c, c->dlogits + (size_t)i * c->cfg.vocab, c->cfg.vocab, out);
}

int ae_get_kv_row(ae_ctx *c, int layer, int which, int slot, float *out) {
  if (!c) return AE_EINVAL;
  const ae_config &g = c->cfg;
  if (!out || layer < 0 || layer > g.n_layers || (which != 0 && which != 1) || slot < 0 || slot >= g.n_ctx_max)
    return fail(c, AE_EINVAL, "ae_get_kv_row: argument out of range");
  launch_kv_export(kv_layer_ptr(c, layer), c->kv_v_offset, g, which, slot, c->attn_part, c->fast, c->stream);
  return copy_out(c, c->attn_part, (size_t)g.n_kv_heads * g.head_dim, out);
}

int ae_set_kernel_timing(ae_ctx *c, int enabled) {
  if (!c) return AE_EINVAL;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  if (enabled && c->kt_ev.empty()) {
    // enough pairs for every decoder layer of one step (k_max+1 draft forwards + verify)
    const int pairs = (c->cfg.n_layers + c->cfg.k_max + 2) * 2;
    for (int i = 0; i < 2 * pairs; ++i) {
      hipEvent_t e;
      HIPCHK(c, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
      c->kt_ev.push_back(e);
    }
  }
  drain_kernel_timing(c);
  c->ktime = enabled != 0;
  c->kt_total_us = 0.0;
  c->kt_count = 0;
  return AE_OK;
}

int ae_get_kernel_timing(ae_ctx *c, double *total_us, int64_t *launches) {
  if (!c) return AE_EINVAL;
  if (!total_us || !launches) return fail(c, AE_EINVAL, "ae_get_kernel_timing: NULL output");
  *total_us = c->kt_total_us;
  *launches = c->kt_count;
  return AE_OK;
}

int ae_set_profiling(ae_ctx *c, int enabled) {
  if (!c) return AE_EINVAL;
  c->profiling = enabled != 0;
  return AE_OK;
}

int ae_get_phase_times(ae_ctx *c, ae_phase_times *out) {
  if (!c) return AE_EINVAL;
  if (!out) return fail(c, AE_EINVAL, "ae_get_phase_times: NULL output");
  *out = c->last_times;
  return AE_OK;
}

}  // extern "C"
