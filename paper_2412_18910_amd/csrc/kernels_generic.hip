// Dtype-generic kernels of the decode step (gfx950, wave64).  They serve the fp32
// configuration and every small op of the bf16 configuration; the bandwidth-critical
// bf16 GEMMs have their own MFMA kernels in kernels_mfma.hip.
#include "ae_internal.h"

namespace ae {

using bf16_t = uint16_t;

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <typename T>
__device__ __forceinline__ float ld1(const T *p);
template <>
__device__ __forceinline__ float ld1<float>(const float *p) { return *p; }
template <>
__device__ __forceinline__ float ld1<bf16_t>(const bf16_t *p) { return bf2f(*p); }

// 8 consecutive weights -> float[8] with 128-bit loads
__device__ __forceinline__ void ld8(const float *p, float *w) {
  const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
  w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
}
__device__ __forceinline__ void ld8(const bf16_t *p, float *w) {
  const uint4 a = *reinterpret_cast<const uint4 *>(p);
  w[0] = __uint_as_float(a.x << 16); w[1] = __uint_as_float(a.x & 0xffff0000u);
  w[2] = __uint_as_float(a.y << 16); w[3] = __uint_as_float(a.y & 0xffff0000u);
  w[4] = __uint_as_float(a.z << 16); w[5] = __uint_as_float(a.z & 0xffff0000u);
  w[6] = __uint_as_float(a.w << 16); w[7] = __uint_as_float(a.w & 0xffff0000u);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ void embed_kernel(const T *emb, const int32_t *ids, int d, float *out) {
  const int r = blockIdx.x;
  const T *src = emb + (size_t)ids[r] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) out[(size_t)r * d + i] = ld1(src + i);
}

void launch_embed(const void *emb, int dtype, const int32_t *ids_dev, int rows, int d, float *out, hipStream_t s) {
  if (dtype == AE_BF16)
    embed_kernel<bf16_t><<<rows, 256, 0, s>>>((const bf16_t *)emb, ids_dev, d, out);
  else
    embed_kernel<float><<<rows, 256, 0, s>>>((const float *)emb, ids_dev, d, out);
}

// ------------------------------------------------------------------ RMSNorm
// out = (x / sqrt(mean(x^2) + eps)) * g, one workgroup per row
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float *x, const float *g, int d, float eps, float *out,
                                                      const int32_t *gate) {
  __shared__ float red[4];
  AE_GATE(gate);
  const float *xr = x + (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int i = threadIdx.x * 4; i < d; i += 1024) {   // d is a multiple of 8
    const float4 v = *reinterpret_cast<const float4 *>(xr + i);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int i = threadIdx.x * 4; i < d; i += 1024) {
    const float4 v = *reinterpret_cast<const float4 *>(xr + i), gn = *reinterpret_cast<const float4 *>(g + i);
    *reinterpret_cast<float4 *>(out + (size_t)blockIdx.x * d + i) =
        make_float4((v.x * r) * gn.x, (v.y * r) * gn.y, (v.z * r) * gn.z, (v.w * r) * gn.w);
  }
}

void launch_rmsnorm(const float *x, const float *g, int rows, int d, float eps, float *out, hipStream_t s,
                    const int32_t *gate) {
  rmsnorm_kernel<<<rows, 256, 0, s>>>(x, g, d, eps, out, gate);
}

// ------------------------------------------------------------------ generic skinny GEMM
// One wave per output column n, all rows at once; lanes stride over K in 8-element
// pieces.  The per-output summation order does not depend on the number of rows.
template <typename WT, int MT>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const WT *W, int N, int K, const float *X, int ldx, int rows,
                                                           const float *bias, float *Y, int ldy, int accumulate,
                                                           const int32_t *gate) {
  AE_GATE(gate);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + wave;
  if (n >= N) return;
  float acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = 0.f;
  const WT *wrow = W + (size_t)n * K;
  for (int k0 = lane * 8; k0 < K; k0 += 512) {
    float w[8];
    ld8(wrow + k0, w);
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      if (m < rows) {
        float xv[8];
        ld8(X + (size_t)m * ldx + k0, xv);
        float a = acc[m];
#pragma unroll
        for (int j = 0; j < 8; ++j) a = fmaf(xv[j], w[j], a);
        acc[m] = a;
      }
    }
  }
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    if (m < rows) {
      float v = wave_sum(acc[m]);
      if (lane == 0) {
        if (bias) v += bias[n];
        float *y = Y + (size_t)m * ldy + n;
        *y = accumulate ? *y + v : v;
      }
    }
  }
}

template <typename WT>
static void gemm_generic_dispatch(const WT *W, int N, int K, const float *X, int ldx, int rows, const float *bias,
                                  float *Y, int ldy, int acc, hipStream_t s, const int32_t *gate) {
  const dim3 grid((N + 3) / 4);
  if (rows <= 1)
    gemm_generic_kernel<WT, 1><<<grid, 256, 0, s>>>(W, N, K, X, ldx, rows, bias, Y, ldy, acc, gate);
  else if (rows <= 4)
    gemm_generic_kernel<WT, 4><<<grid, 256, 0, s>>>(W, N, K, X, ldx, rows, bias, Y, ldy, acc, gate);
  else
    gemm_generic_kernel<WT, 16><<<grid, 256, 0, s>>>(W, N, K, X, ldx, rows, bias, Y, ldy, acc, gate);
}

void launch_gemm_generic(const void *W, int dtype, int N, int K, const float *X, int ldx, int rows,
                         const float *bias, float *Y, int ldy, int accumulate, hipStream_t s, const int32_t *gate) {
  if (dtype == AE_BF16)
    gemm_generic_dispatch<bf16_t>((const bf16_t *)W, N, K, X, ldx, rows, bias, Y, ldy, accumulate, s, gate);
  else
    gemm_generic_dispatch<float>((const float *)W, N, K, X, ldx, rows, bias, Y, ldy, accumulate, s, gate);
}

// ------------------------------------------------------------------ SwiGLU elementwise
__global__ void silu_mul_kernel(const float *gate_proj, const float *up, size_t n, float *out, const int32_t *gate) {
  AE_GATE(gate);
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    out[i] = silu_f(gate_proj[i]) * up[i];
}

void launch_silu_mul(const float *gate_proj, const float *up, int rows, int f, float *out, hipStream_t s,
                     const int32_t *gate) {
  const size_t n = (size_t)rows * f;
  const int blocks = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
  silu_mul_kernel<<<blocks, 256, 0, s>>>(gate_proj, up, n, out, gate);
}

// ------------------------------------------------------------------ argmax (lowest id wins ties)
__global__ __launch_bounds__(1024) void argmax_kernel(const float *logits, int V, int32_t *out, const int32_t *gate) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  AE_GATE(gate);
  const float *x = logits + (size_t)blockIdx.x * V;
  float best = -INFINITY;
  int idx = 0x7fffffff;
  for (int i = threadIdx.x; i < V; i += 1024) {
    const float v = x[i];
    if (v > best) { best = v; idx = i; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(idx, o, 64);
    if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
    out[blockIdx.x] = idx == 0x7fffffff ? 0 : idx;
  }
}

void launch_argmax(const float *logits, int rows, int V, int32_t *out_ids, hipStream_t s, const int32_t *gate) {
  argmax_kernel<<<rows, 1024, 0, s>>>(logits, V, out_ids, gate);
}

// ------------------------------------------------------------------ draft head input
// cat[r] = [feature row r ; embedding of the token that FOLLOWS slot r]  (Sec. 2.2)
template <typename T>
__global__ void draft_cat_kernel(const float *feat, int feat_ld, const T *emb, const int32_t *next_ids, int d,
                                 float *cat, const int32_t *gate) {
  AE_GATE(gate);
  const int r = blockIdx.x;
  const T *e = emb + (size_t)next_ids[r] * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    cat[(size_t)r * 2 * d + i] = feat[(size_t)r * feat_ld + i];
    cat[(size_t)r * 2 * d + d + i] = ld1(e + i);
  }
}

void launch_draft_cat(const float *feat, int feat_ld, const void *emb, int dtype, const int32_t *next_ids, int rows,
                      int d, float *cat, hipStream_t s, const int32_t *gate) {
  if (dtype == AE_BF16)
    draft_cat_kernel<bf16_t><<<rows, 256, 0, s>>>(feat, feat_ld, (const bf16_t *)emb, next_ids, d, cat, gate);
  else
    draft_cat_kernel<float><<<rows, 256, 0, s>>>(feat, feat_ld, (const float *)emb, next_ids, d, cat, gate);
}

// ------------------------------------------------------------------ tiny control kernels
__global__ void pick_draft_kernel(DevState *st, int i, const int32_t *gate) {
  AE_GATE(gate);
  int32_t t = st->argmax[0];
  if (st->override_ids[i] >= 0) t = st->override_ids[i];
  st->draft_ids[i] = t;
}
void launch_pick_draft(DevState *st, int i, hipStream_t s, const int32_t *gate) {
  pick_draft_kernel<<<1, 1, 0, s>>>(st, i, gate);
}

// AdaEAGLE-DDD bookkeeping behind draft token i (Sec. 3.4, 4.2): its log-probability under
// softmax(logits / T) joins the running sum, the drafted length becomes i + 1, and the exit
// rule for the next token is evaluated on the device: past the predicted length k the chain
// goes on only while the sequence log-probability is at least theta (draft_live gates the
// kernels of the tokens that follow).  One workgroup, fixed-shape reductions.
__global__ __launch_bounds__(1024) void draft_logprob_kernel(const float *logits, int V, float inv_T, DevState *st, int i,
                                                             int k, float theta, const int32_t *gate) {
  __shared__ float sh[1024];
  AE_GATE(gate);
  const int t = threadIdx.x;
  float mx = -INFINITY;
  for (int x = t; x < V; x += 1024) mx = fmaxf(mx, logits[x]);
  sh[t] = mx;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (t < o) sh[t] = fmaxf(sh[t], sh[t + o]);
    __syncthreads();
  }
  mx = sh[0];
  __syncthreads();
  float se = 0.f;
  for (int x = t; x < V; x += 1024) se += expf((logits[x] - mx) * inv_T);
  sh[t] = se;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (t < o) sh[t] += sh[t + o];
    __syncthreads();
  }
  if (t == 0) {
    const float lp = (logits[st->draft_ids[i]] - mx) * inv_T - logf(sh[0]);
    const float cum = (i == 0 ? 0.f : st->cum_logp) + lp;
    st->draft_lp[i] = lp;
    st->cum_logp = cum;
    st->draft_len = i + 1;
    if (i + 1 >= k && !(cum >= theta)) st->draft_live = 0;
  }
}
void launch_draft_logprob(const float *logits, int V, float T, DevState *st, int i, int k, float theta, hipStream_t s,
                          const int32_t *gate) {
  draft_logprob_kernel<<<1, 1024, 0, s>>>(logits, V, T > 0.f ? 1.0f / T : 1.0f, st, i, k, theta, gate);
}

// Small host values reach the device state as kernel arguments: the launch carries them, so no
// staging buffer has to outlive the call and no copy engine is involved.
struct HostIds { int32_t v[kMaxRows]; };
struct HostUniforms { double v[kMaxRows]; };

__global__ void set_draft_inputs_kernel(DevState *st, HostIds ov, HostUniforms u, int n_u) {
  const int t = threadIdx.x;
  if (t < kMaxRows) {
    st->override_ids[t] = ov.v[t];
    if (t < n_u) st->u_draft[t] = u.v[t];
  }
  if (t == 0) {
    st->draft_live = 1;
    st->draft_len = 0;
  }
}
void launch_set_draft_inputs(DevState *st, const int32_t *override_ids, int n_ov, const double *u_draft, int n_u,
                             hipStream_t s) {
  HostIds ov;
  HostUniforms u;
  for (int i = 0; i < kMaxRows; ++i) {
    ov.v[i] = (override_ids && i < n_ov) ? override_ids[i] : -1;
    u.v[i] = (u_draft && i < n_u) ? u_draft[i] : 0.0;
  }
  set_draft_inputs_kernel<<<1, 64, 0, s>>>(st, ov, u, u_draft ? n_u : 0);
}

__global__ void set_block_kernel(DevState *st, HostIds ids, int rows) {
  if ((int)threadIdx.x < rows) st->block[threadIdx.x] = ids.v[threadIdx.x];
}
void launch_set_block(DevState *st, const int32_t *ids, int rows, hipStream_t s) {
  HostIds h;
  for (int i = 0; i < kMaxRows; ++i) h.v[i] = i < rows ? ids[i] : 0;
  set_block_kernel<<<1, 64, 0, s>>>(st, h, rows);
}

__global__ void set_u_accept_kernel(DevState *st, HostUniforms u, int rows) {
  if ((int)threadIdx.x < rows) st->u_accept[threadIdx.x] = u.v[threadIdx.x];
}
void launch_set_u_accept(DevState *st, const double *u, int rows, hipStream_t s) {
  HostUniforms h;
  for (int i = 0; i < kMaxRows; ++i) h.v[i] = i < rows ? u[i] : 0.0;
  set_u_accept_kernel<<<1, 64, 0, s>>>(st, h, rows);
}

__global__ void build_block_kernel(DevState *st, const int32_t *hist, int kv_len, int k) {
  if (threadIdx.x == 0) st->block[0] = hist[kv_len];
  if ((int)threadIdx.x < k) st->block[1 + threadIdx.x] = st->draft_ids[threadIdx.x];
}
void launch_build_block(DevState *st, const int32_t *hist, int kv_len, int k, hipStream_t s) {
  build_block_kernel<<<1, 64, 0, s>>>(st, hist, kv_len, k);
}

// Greedy acceptance (longest draft prefix equal to the target argmax, then the target's
// own token) and the token-history side of the rollback.
__global__ void accept_greedy_kernel(DevState *st, int32_t *hist, int kv_len, int rows, int k_on_device) {
  const int k = k_on_device ? min(st->draft_len, rows - 1) : rows - 1;
  int acc = 0;
  while (acc < k && st->block[1 + acc] == st->argmax[acc]) ++acc;
  const int32_t bonus = st->argmax[acc];
  for (int i = 0; i <= acc; ++i) hist[kv_len + i] = st->block[i];
  hist[kv_len + 1 + acc] = bonus;
  st->n_acc = acc;
  st->bonus = bonus;
}
void launch_accept_greedy(DevState *st, int32_t *hist, int kv_len, int rows, bool k_on_device, hipStream_t s) {
  accept_greedy_kernel<<<1, 1, 0, s>>>(st, hist, kv_len, rows, k_on_device ? 1 : 0);
}

// The host reads the device state through a mirror in pinned host memory that the device
// writes itself (no copy engine, no blit kernel): all threads of a workgroup call this behind
// a barrier that follows the last write to *st; the words in [skip0, skip1) are left to the caller.
__device__ __forceinline__ void publish_state(const DevState *st, DevState *mirror, int skip0 = 0, int skip1 = 0) {
  const uint32_t *src = reinterpret_cast<const uint32_t *>(st);
  uint32_t *dst = reinterpret_cast<uint32_t *>(mirror);
  for (int i = threadIdx.x; i < (int)(sizeof(DevState) / 4); i += blockDim.x)
    if (i < skip0 || i >= skip1) dst[i] = src[i];
}
__global__ void publish_state_kernel(const DevState *st, DevState *mirror) { publish_state(st, mirror); }
void launch_publish_state(const DevState *st, DevState *mirror, hipStream_t s) {
  publish_state_kernel<<<1, 128, 0, s>>>(st, mirror);
}

// ------------------------------------------------------------------ LDLP (Eq. 3)
// Input layer z0 = W_in u + b_in with u = [e ; f] (in_mode 0) or f (in_mode 1) read in place:
// e = embedding of the last validated token (hist[slot]), f = its feature row F[f_row].  When
// use_nacc is set, slot and row are taken relative to the acceptance result that an earlier
// kernel left in *st.  One wave per output, lanes stride over the input in 8-element pieces
// (the summation order of the generic GEMM).
template <typename T>
__global__ __launch_bounds__(256) void ldlp_in_kernel(const T *W, const float *bias, const T *emb, const int32_t *hist,
                                                      const float *F, int d, int in_mode, int h, int slot, int f_row,
                                                      int use_nacc, const DevState *st, float *z0) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + wave;
  if (n >= h) return;
  const int add = use_nacc ? st->n_acc : 0;
  const float *f = F + (size_t)(f_row + add) * d;
  const T *e = emb + (size_t)hist[slot + add] * d;
  const int K = in_mode == 0 ? 2 * d : d;
  const T *wrow = W + (size_t)n * K;
  float acc = 0.f;
  // unrolled so that several iterations' loads are in flight; the products still join acc in index order
#pragma unroll 4
  for (int k0 = lane * 8; k0 < K; k0 += 512) {
    float w[8], x[8];
    ld8(wrow + k0, w);
    if (in_mode == 0 && k0 < d) ld8(e + k0, x);
    else ld8(f + (in_mode == 0 ? k0 - d : k0), x);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = fmaf(x[j], w[j], acc);
  }
  acc = wave_sum(acc);
  if (lane == 0) z0[n] = acc + bias[n];
}

void launch_ldlp_in(const void *W, const float *bias, const void *emb, int dtype, const int32_t *hist, const float *F, int d,
                    int in_mode, int h, int slot, int f_row, const DevState *st_nacc, float *z0, hipStream_t s) {
  const int use = st_nacc != nullptr;
  const dim3 grid((h + 3) / 4);
  if (dtype == AE_BF16)
    ldlp_in_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)W, bias, (const bf16_t *)emb, hist, F, d, in_mode, h, slot,
                                                f_row, use, st_nacc, z0);
  else
    ldlp_in_kernel<float><<<grid, 256, 0, s>>>((const float *)W, bias, (const float *)emb, hist, F, d, in_mode, h, slot,
                                               f_row, use, st_nacc, z0);
}

// z0 = W_in u + b_in comes from the GEMM; here: residual blocks z += silu(W_r z + b_r),
// y = w_out . silu(z) + b_out, k = clamp(round_half_even(y), 0, k_max)  (Eq. 3).
// cls != 0: the classification variant (Sec. 4.3 ablation), one score per length 0..k_max,
// k = argmax (lowest length on ties), y_next = the winning score.
template <typename T>
__global__ __launch_bounds__(1024) void ldlp_tail_kernel(const float *z0, const T *w_res, const float *b_res,
                                                         const float *w_out, const float *b_out, int h, int n_res,
                                                         int k_max, int cls, DevState *st, DevState *mirror) {
  __shared__ float z[kMaxLdlpHidden];
  __shared__ float t[kMaxLdlpHidden];
  const int i = threadIdx.x;
  if (i < h) z[i] = z0[i];
  __syncthreads();
  for (int r = 0; r < n_res; ++r) {
    if (i < h) {
      const T *row = w_res + ((size_t)r * h + i) * h;
      float a = 0.f;
      for (int j = 0; j < h; ++j) a = fmaf(z[j], ld1(row + j), a);
      t[i] = silu_f(a + b_res[(size_t)r * h + i]);
    }
    __syncthreads();
    if (i < h) z[i] += t[i];
    __syncthreads();
  }
  const float a = i < h ? silu_f(z[i]) : 0.f;
  int best = 0;
  float best_y = 0.f;
  for (int c = 0; c < (cls ? k_max + 1 : 1); ++c) {
    t[i] = i < h ? a * w_out[(size_t)c * h + i] : 0.f;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {  // fixed-shape tree: deterministic
      if (i < o) t[i] += t[i + o];
      __syncthreads();
    }
    const float y = t[0] + b_out[c];
    if (c == 0 || y > best_y) { best = c; best_y = y; }
    __syncthreads();
  }
  if (i == 0) {
    int k = best;
    if (!cls) {
      float r = rintf(best_y);  // round half to even
      if (!(r >= 0.f)) r = 0.f;
      if (r > (float)k_max) r = (float)k_max;
      k = (int)r;
    }
    st->y_next = best_y;
    st->k_next = k;
    mirror->y_next = best_y;
    mirror->k_next = k;
  }
  // the rest of the state (acceptance result, block ids, draft bookkeeping) was written by earlier kernels
  static_assert(offsetof(DevState, y_next) == offsetof(DevState, k_next) + 4, "k_next and y_next are adjacent words");
  publish_state(st, mirror, offsetof(DevState, k_next) / 4, offsetof(DevState, y_next) / 4 + 1);
}

void launch_ldlp_tail(const float *z0, const void *w_res, int dtype, const float *b_res, const float *w_out,
                      const float *b_out, int h, int n_res, int k_max, int cls, DevState *st, DevState *mirror,
                      hipStream_t s) {
  if (dtype == AE_BF16)
    ldlp_tail_kernel<bf16_t><<<1, 1024, 0, s>>>(z0, (const bf16_t *)w_res, b_res, w_out, b_out, h, n_res, k_max, cls, st,
                                                mirror);
  else
    ldlp_tail_kernel<float><<<1, 1024, 0, s>>>(z0, (const float *)w_res, b_res, w_out, b_out, h, n_res, k_max, cls, st,
                                               mirror);
}

// ------------------------------------------------------------------ set-up helpers
// (cos, sin) of pos * base^(-2i/hd), evaluated in double and rounded once to float
__global__ void rope_table_kernel(float2 *tab, int n_pos, int half, int head_dim, double base) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_pos * half) return;
  const int p = idx / half, i = idx % half;
  const double inv = pow(base, -2.0 * (double)i / (double)head_dim);
  const double ang = (double)p * inv;
  tab[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

void launch_rope_table(float2 *tab, int n_pos, int head_dim, float base, hipStream_t s) {
  const int half = head_dim / 2, n = n_pos * half;
  rope_table_kernel<<<(n + 255) / 256, 256, 0, s>>>(tab, n_pos, half, head_dim, (double)base);
}

__global__ void fill_zero_kernel(uint4 *p, size_t n16) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
}

void launch_fill_zero(void *p, size_t bytes, hipStream_t s) {  // bytes must be a multiple of 16
  fill_zero_kernel<<<2048, 256, 0, s>>>((uint4 *)p, bytes / 16);
}

}  // namespace ae
