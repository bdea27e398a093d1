// Internal declarations of libadaeagle (gfx950).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "adaeagle.h"

namespace ae {

constexpr int kMaxRows = 16;       // rows of one verify / prefill block (one MFMA tile)
constexpr int kAttnChunk = 256;    // keys per split-KV workgroup (fixed by absolute slot)
constexpr int kMaxSplits = 64;     // n_ctx_max / kAttnChunk upper bound
constexpr int kMfmaKeysPerWave = 64;                     // bf16 matrix-core attention: keys per wave,
constexpr int kMfmaAttnChunk = 4 * kMfmaKeysPerWave;     // keys per workgroup (4 waves)
constexpr int kMaxLdlpHidden = 1024;
constexpr int kDenseRB = 8;        // activation row-blocks per workgroup of the dense prompt GEMM (128 rows)
constexpr int kDenseMinPrompt = 17;   // prompts of one 16-row block go through the decode kernels

// Device-resident step state.  The host mirrors kv_len (it learns it at every accept).
struct DevState {
  int32_t n_acc;            // result of the last accept
  int32_t bonus;
  int32_t k_next;           // Eq. 3 result for the next step
  float y_next;             // LDLP scalar before rounding
  int32_t draft_ids[kMaxRows];
  int32_t override_ids[kMaxRows];
  // Device-gated DDD chain (reset together with override_ids): every kernel of a draft token
  // past the predicted length reads draft_live at entry and returns when it is 0; draft_len
  // counts the tokens drafted.
  int32_t draft_live;
  int32_t draft_len;
  int32_t block[kMaxRows];  // ids of the verify block
  int32_t argmax[kMaxRows]; // per-row argmax of the last LM-head call
  double u_draft[kMaxRows];
  double u_accept[kMaxRows];
  float cum_logp;           // log-probability of the current draft sequence (DDD exit rule)
  float draft_lp[kMaxRows]; // per-token log-probabilities
};
static_assert(offsetof(DevState, u_draft) % 8 == 0, "doubles must stay aligned");

// A kernel launched with a non-null gate pointer does nothing when *gate == 0.
#define AE_GATE(gate)                          \
  do {                                         \
    if ((gate) != nullptr && *(gate) == 0) return; \
  } while (0)

// Weight matrix handle: row-major source plus (bf16 fast path) the re-tiled copy.
struct Mat {
  const void *rowmajor = nullptr;  // caller's [N,K]
  void *tiled = nullptr;           // ctx-owned MFMA-tile layout, bf16 only
  int N = 0, K = 0;
};

struct LayerW {
  const float *attn_norm = nullptr, *ffn_norm = nullptr;
  Mat wq, wk, wv, wo, w_gate, w_up, w_down;
  Mat f_qkv, f_gu;   // bf16 fast path: fused tiled [q;k;v] and row-block-interleaved [gate,up]
};

}  // namespace ae

struct ae_ctx {
  ae_config cfg{};
  hipStream_t stream = nullptr;
  int device = 0;
  bool fast = false;            // bf16 MFMA path (else generic kernels)
  std::string err;

  // weights
  const void *tok_emb = nullptr;
  const float *final_norm = nullptr;
  ae::Mat lm_head, draft_fc, ldlp_in;
  const float *draft_fc_b = nullptr, *ldlp_b_in = nullptr, *ldlp_b_res = nullptr;
  const void *ldlp_w_res = nullptr;
  const float *ldlp_w_out = nullptr, *ldlp_b_out = nullptr;
  std::vector<ae::LayerW> layers;  // n_layers target layers + the draft layer last
  std::vector<void *> owned;       // device allocations to free

  // KV cache: per layer K in d-group-major layout, V row-major (see kernels_attn.hip)
  void *kv = nullptr;
  size_t kv_layer_stride = 0;      // bytes between layers
  size_t kv_v_offset = 0;          // bytes from a layer's K to its V
  float2 *rope_tab = nullptr;      // [n_ctx_max][head_dim/2] (cos, sin)
  float *kv_stage = nullptr;       // this device's address of the library's static staging array

  // activations (float, kMaxRows rows each)
  float *x = nullptr, *xn = nullptr, *q = nullptr, *kbuf = nullptr, *vbuf = nullptr, *att = nullptr;
  float *gate_proj = nullptr, *up = nullptr, *hmid = nullptr;
  float *F = nullptr;              // feature rows (post final norm)
  float *cat = nullptr;            // [rows][2d] draft fc input
  float *logits = nullptr;         // [k_max+1][V]
  float *dlogits = nullptr;        // [k_max][V]
  float *attn_part = nullptr;      // split-KV partials
  float *ldlp_z = nullptr;         // LDLP hidden vector
  // bf16 fast path: packed activations (GEMM B operands) and RMSNorm partial sums
  void *xp_a = nullptr, *xp_f = nullptr, *xp_att = nullptr, *xp_h = nullptr, *xp_cat = nullptr;
  float *ssq_a = nullptr, *ssq_f = nullptr;
  float *amax_val = nullptr;       // LM-head argmax partials [16][vocab/16]
  int32_t *amax_idx = nullptr;
  float *lse_sum = nullptr;        // LM-head softmax partials [16][vocab/16] (DDD rule)
  int Pa = 0;                      // number of valid partial-sum rows in ssq_a
  double *prob = nullptr;          // T>0 scratch: segment / row statistics of the sampling kernels
  int32_t *hist = nullptr;         // device token history by slot
  ae::DevState *st = nullptr;      // device state
  ae::DevState *h_st = nullptr;    // pinned host mirror of *st, written by the device (publish_state)
  ae::DevState *h_st_dev = nullptr;   // the device's address of that mirror

  // dense prompt pass (bf16 only): chunk buffers, allocated at the first long prompt
  int prefill_mode = 0;            // AE_PREFILL_AUTO / _BLOCKS / _DENSE
  int dense_chunk = 2048;          // rows per dense pass (multiple of 128)
  int dense_cap = 0;               // rows the buffers below hold
  std::vector<void *> dense_owned;
  float *px = nullptr, *pq = nullptr, *prinv = nullptr, *pssq_a = nullptr, *pssq_f = nullptr;
  void *pxa = nullptr, *pxf = nullptr, *pxatt = nullptr, *pxh = nullptr, *pxcat = nullptr;

  // host-side state machine
  int kv_len = 0, dlen = 0, nF = 0;
  int cur_k = 0, cur_k_last = 0, block_rows = 0;
  int ddd_mode = AE_DDD_DEVICE;    // AE_DDD_HOST / AE_DDD_DEVICE
  bool k_on_device = false;        // the last draft's length is only known on the device (st->draft_len)
  const int32_t *gate = nullptr;   // gate of the kernels being enqueued (device-gated DDD chain), else nullptr
  int32_t pending = 0;
  bool have_pending = false, have_draft = false, have_verify = false, k_next_valid = false;
  int k_next = 0;
  float y_next = 0.f;
  std::vector<int32_t> h_hist;     // host mirror of the token history
  std::vector<int32_t> h_block;

  // per-kernel event timing of the gate/up GEMM launches (see ae_set_kernel_timing)
  bool ktime = false;
  std::vector<hipEvent_t> kt_ev;   // pairs (begin, end)
  int kt_used = 0;
  double kt_total_us = 0.0;
  long long kt_count = 0;

  // profiling
  bool profiling = false;
  hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
  ae_phase_times last_times{};
};

namespace ae {

// ---- generic kernels (kernels_generic.hip); all launches are asynchronous on `s` ----
void launch_embed(const void *emb, int dtype, const int32_t *ids_dev, int rows, int d, float *out, hipStream_t s);
void launch_rmsnorm(const float *x, const float *g, int rows, int d, float eps, float *out, hipStream_t s,
                    const int32_t *gate = nullptr);
// Y[r][n] (+)= sum_k X[r][k] W[n][k] + bias[n];  accumulate != 0 adds into Y (residual)
void launch_gemm_generic(const void *W, int dtype, int N, int K, const float *X, int ldx, int rows,
                         const float *bias, float *Y, int ldy, int accumulate, hipStream_t s,
                         const int32_t *gate = nullptr);
void launch_silu_mul(const float *gate_proj, const float *up, int rows, int f, float *out, hipStream_t s,
                     const int32_t *gate = nullptr);
void launch_argmax(const float *logits, int rows, int V, int32_t *out_ids, hipStream_t s, const int32_t *gate = nullptr);
void launch_draft_cat(const float *feat, int feat_ld, const void *emb, int dtype, const int32_t *next_ids,
                      int rows, int d, float *cat, hipStream_t s, const int32_t *gate = nullptr);
void launch_pick_draft(DevState *st, int i, hipStream_t s, const int32_t *gate = nullptr);
// DDD bookkeeping behind draft token i: log softmax(logits / T)[token i] -> st->draft_lp[i], added
// to st->cum_logp (reset when i == 0); st->draft_len = i + 1; and the exit rule for the NEXT
// token: st->draft_live = 0 when i + 1 >= k and the sequence log-probability is below theta.
void launch_draft_logprob(const float *logits, int V, float T, DevState *st, int i, int k, float theta, hipStream_t s,
                          const int32_t *gate = nullptr);
// Host arrays (override ids: -1 keeps the head's own token; uniforms; explicit block ids) are
// passed by value inside the launch; the pointers are read before the call returns.
void launch_set_draft_inputs(DevState *st, const int32_t *override_ids, int n_ov, const double *u_draft, int n_u,
                             hipStream_t s);
void launch_set_block(DevState *st, const int32_t *ids, int rows, hipStream_t s);
void launch_set_u_accept(DevState *st, const double *u, int rows, hipStream_t s);
void launch_build_block(DevState *st, const int32_t *hist, int kv_len, int k, hipStream_t s);
// k_on_device: the draft length is st->draft_len (the block is padded to `rows` rows)
void launch_accept_greedy(DevState *st, int32_t *hist, int kv_len, int rows, bool k_on_device, hipStream_t s);
// z0 = W_in [e ; f] + b_in (Eq. 3 input layer), e and f read in place; st_nacc != nullptr: slot and
// row relative to the acceptance result in *st_nacc
void launch_ldlp_in(const void *W, const float *bias, const void *emb, int dtype, const int32_t *hist, const float *F, int d,
                    int in_mode, int h, int slot, int f_row, const DevState *st_nacc, float *z0, hipStream_t s);
// also copies the whole device state to `mirror` (device-visible pinned host memory)
void launch_ldlp_tail(const float *z0, const void *w_res, int dtype, const float *b_res, const float *w_out,
                      const float *b_out, int h, int n_res, int k_max, int cls, DevState *st, DevState *mirror,
                      hipStream_t s);
// *mirror = *st, written by the device itself
void launch_publish_state(const DevState *st, DevState *mirror, hipStream_t s);
void launch_rope_table(float2 *tab, int n_pos, int head_dim, float base, hipStream_t s);
void launch_fill_zero(void *p, size_t bytes, hipStream_t s);

// ---- attention (kernels_attn.hip) ----
size_t kv_layer_bytes(const ae_config &c);
size_t kv_v_offset_bytes(const ae_config &c);
int kv_capacity(const ae_config &c);   // n_ctx_max rounded up to a whole attention chunk
void launch_rope_append(float *q, const float *k, const float *v, int rows, int pos0, const ae_config &c,
                        const float2 *rope_tab, void *kv_layer, size_t v_off, bool tiled, hipStream_t s,
                        const int32_t *gate = nullptr);
// bf16 MFMA attention over the tiled cache layout (kernels_attn_mfma.hip)
void attention_mfma_setup();   // once per context set-up: dynamic LDS limit of the kernels
void launch_attention_mfma(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                           float *part, void *Xp_out, hipStream_t s, const int32_t *gate = nullptr);
void launch_attention(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                      float *part, float *out, hipStream_t s, const int32_t *gate = nullptr);
void launch_kv_import(void *kv_layer, size_t v_off, const ae_config &c, const float *k_dev, const float *v_dev, int n,
                      bool tiled, hipStream_t s);
void launch_kv_export(const void *kv_layer, size_t v_off, const ae_config &c, int which, int slot, float *out_dev,
                      bool tiled, hipStream_t s);
size_t attn_part_floats(const ae_config &c);

// ---- T > 0 sampling (kernels_sample.hip) ----
size_t sample_scratch_doubles(int V);   // size of the scratch both launches below take
void launch_sample_draft(const float *logits, int V, float T, DevState *st, int i, double *scratch, hipStream_t s,
                         const int32_t *gate = nullptr);
// k = draft tokens the block holds room for (rows - 1); k_on_device: only the first
// st->draft_len of them were drafted (padded block of the device-gated DDD chain)
void launch_accept_sample(const float *tl, const float *dl, int V, int k, bool k_on_device, float T, DevState *st,
                          int32_t *hist, int kv_len, double *prob, hipStream_t s);

// ---- bf16 MFMA path (kernels_mfma.hip) ----
// Row-block nb of a row-major [N,K] matrix -> row-block nb_off + nb*nb_stride of a fused
// k-major tiled matrix with NBtot row-blocks.
void launch_retile(const void *rowmajor, int N, int K, void *tiled, int NBtot, int nb_off, int nb_stride, int perm_hd,
                   hipStream_t s);
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_QKV = 3 };
struct GemmLaunch {
  const Mat *W = nullptr;         // fused tiled matrix: N = all output rows, K
  const void *Xp = nullptr;       // packed activations
  int rows = 0, row0 = 0;         // output row m reads packed row row0 + m
  const float *ssq_in = nullptr;  // != nullptr: fused RMSNorm, [P_in][16] partial sums of x^2
  int P_in = 0;
  float eps = 0.f;
  const float *bias = nullptr;
  int epi = EPI_STORE;
  int nseg = 1;                   // output segments (q | k | v)
  float *Y[3] = {nullptr, nullptr, nullptr};
  int ldy[3] = {0, 0, 0};
  int seg_N[3] = {0, 0, 0};
  void *Xp_out = nullptr;         // packed output for the next GEMM
  const float *gain_out = nullptr;
  float *ssq_out = nullptr;
  float *amax_val = nullptr;      // LM head: argmax partials per row and row-block [16][N/16]
  int32_t *amax_idx = nullptr;
  float *lse_sum = nullptr;       // with amax_val: sum of exp((x - block max) * lse_inv_t) per row and row-block
  float lse_inv_t = 1.f;
  // EPI_QKV: rotary embedding + KV append fused into the epilogue
  const float2 *rope_tab = nullptr;
  void *Kc = nullptr, *Vc = nullptr;
  int pos0 = 0, n_ctx = 0, hd = 0;
  const int32_t *gate = nullptr;  // see AE_GATE
};
void launch_gemm_mfma(const GemmLaunch &L, hipStream_t s);
void gemm_mfma_setup(int num_cus);   // once per context set-up: compute-unit count for the shape table
// Where the kernel that fixes a draft token leaves that token's embedding: row `row`, second
// half (k = d .. 2d-1) of the draft head's packed input.  Xp == nullptr: nowhere.
struct DraftCat {
  const void *emb = nullptr;   // bf16 embedding table [V][d]
  void *Xp = nullptr;
  int d = 0, row = 0;
};
// DDD bookkeeping folded into the kernel that fixes draft token i (bf16 path): the token's
// log-probability under softmax(logits / T) from the LM-head epilogue's row-block statistics
// (block maxima `val`, block sums `lse_sum`), the running sum, the drafted length and the exit
// rule for the next token (see launch_draft_logprob).  lse_sum == nullptr: rule off.
struct DddFinish {
  const float *val = nullptr, *lse_sum = nullptr;
  const float *logits = nullptr;   // the token's logit row
  int NB = 0, k = 0;
  float inv_t = 1.f, theta = 0.f;
};
void launch_argmax_finish(const float *val, const int32_t *idx, int NB, int rows, DevState *st, int pick_i, hipStream_t s,
                          const int32_t *gate = nullptr, DraftCat cat = DraftCat(), DddFinish ddd = DddFinish());
void launch_pick_draft_packed(DevState *st, int i, hipStream_t s, const int32_t *gate, DraftCat cat, DddFinish ddd);
void launch_embed_packed(const void *emb, const int32_t *ids_dev, int rows, int d, const float *gain, float *x,
                         void *Xp, float *ssq, hipStream_t s);
void launch_pack_rows(const float *src, int ld, int rows, int K, const float *gain, void *Xp, hipStream_t s);
void launch_draft_cat_packed(const float *feat, int feat_ld, const void *emb, const int32_t *next_ids, int rows, int d,
                             void *Xp, hipStream_t s, const int32_t *gate = nullptr);

// ---- dense prompt pass (kernels_dense.hip); packed buffers hold RB row-blocks ----
// Same GemmLaunch as the decode GEMM (rows = rows of the chunk, row0 unused); rinv != nullptr
// folds RMSNorm in (1/rms per row from launch_rinv_finalize).
void launch_gemm_dense(const GemmLaunch &L, int RB, const float *rinv, hipStream_t s);
void launch_rinv_finalize(const float *ssq, int RBused, int P, int K, float eps, float *rinv, hipStream_t s);
void launch_embed_dense(const void *emb, const int32_t *ids_dev, int rows, int d, const float *gain, float *x, void *Xp,
                        int RB, float *ssq, hipStream_t s);
void launch_draft_cat_dense(const float *x, int rows, int d, const float *gain, float eps, const void *emb,
                            const int32_t *next_ids, void *Xp, int RB, hipStream_t s);
void launch_attention_prefill(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                              void *Xp_out, int RB, hipStream_t s);

}  // namespace ae
