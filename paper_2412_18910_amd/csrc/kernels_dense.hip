// Dense prompt pass (first iteration of Algorithm 1 of arxiv 2412.18910 on a long prompt):
// the only place of the method where the matrix cores, not HBM, are the limit.
//
// The prompt is processed in chunks of up to a few thousand rows.  Activations of a chunk
// live in the packed bf16 hi/lo form of the decode step, extended to many row-blocks
// (Xp[kt][rb][h][64], see packed.h); weights are the same k-major MFMA tiles the decode
// GEMMs stream.  Kernels:
//  * gemm_dense_kernel: workgroup tile = 256 weight rows x 128 (or 64) activation rows.  Each
//    of the 4 waves owns 4 weight row-blocks (A operands: buffer loads straight from the tiled
//    matrix into registers, one coalesced 1 KB burst per tile, double-buffered) and all 8 (4)
//    activation row-blocks, which the workgroup stages through double-buffered LDS (32 KB per
//    stage of 2 k-tiles).  64 MFMAs per wave and k-tile against 16 LDS reads, which are issued
//    one step ahead of the MFMAs that use them; two workgroups per CU (<= 256 registers) so
//    that two waves feed every matrix pipe; tiles are handed out XCD-aware; epilogues are
//    those of the decode GEMM.
//  * attn_prefill_kernel: causal flash attention straight off the tiled KV cache; a wave owns
//    32 (row, head) pairs of one KV head and walks the visible keys 32 at a time with an
//    online softmax in the log2 domain; no partials, no merge, packed output.
//  * embedding, 1/rms finalisation and the draft head's [feature ; embedding] input.
#include "ae_internal.h"
#include "gemm_epilogue.h"
#include "packed.h"

namespace ae {

constexpr int DN = 4;    // weight row-blocks per wave
constexpr int DKS = 2;   // k-tiles per pipeline stage

// DM = activation row-blocks per workgroup: 8 (128 rows), or 4 when the wide tile would leave
// compute units without two resident workgroups.
template <int EPI, bool NORM, int DM>
__global__ __launch_bounds__(256, 2) void gemm_dense_kernel(const GemmArgs a) {
  extern __shared__ u32x4 bs[];   // [2][DKS][DM][2][64]
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 4, m = lane & 15;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps operand bases in scalar registers
  // Workgroup -> tile.  Workgroups are handed to the 8 XCDs round-robin (id % 8) and each XCD
  // has its own L2, so XCD x takes a contiguous share of the tile list, and the list runs
  // through panels of 8 weight tiles with the activation tile advancing every 8 entries: the
  // ~64 workgroups resident on an XCD then cover about 8 x 8 tiles and share their operands in
  // that L2 (7B gate/up GEMM over 2048 rows: 1.4 GB fetched from HBM instead of 3.3 GB with
  // the plain row-major order).
  const int NT = (a.NBtot + 4 * DN - 1) / (4 * DN), MT = (a.rows + DM * 16 - 1) / (DM * 16);
  const int per = (NT * MT + 7) >> 3;
  const int v = ((int)blockIdx.x & 7) * per + ((int)blockIdx.x >> 3);
  if (v >= NT * MT) return;
  constexpr int PN = 8;
  const int full = (NT / PN) * PN * MT;
  int tn, tm;
  if (v < full) {
    const int r = v % (PN * MT);
    tn = (v / (PN * MT)) * PN + r % PN;
    tm = r / PN;
  } else {
    const int r = v - full, pn = NT % PN;
    tn = (NT / PN) * PN + r % pn;
    tm = r / pn;
  }
  const int rb0 = tm * DM;
  // a workgroup hanging over the end of the matrix slides back (recomputes, stores nothing new)
  const int nbw = min(tn * (4 * DN), a.NBtot - 4 * DN) + w * DN;
  const size_t kts = (size_t)a.RB * 128;
  // Operands come through buffer loads: resource descriptor and per-stage byte offset in
  // scalar registers, one fixed per-lane offset register each (out-of-range reads return 0).
  // The DM row-blocks of one k-tile are 1024 contiguous pieces (16 tiles of 64); a thread
  // fetches the piece its MFMA lane position needs (packed slot m*4+g of tile w + 4i), so LDS
  // holds the tiles in lane order and its accesses are conflict-free.
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)a.W, 0, a.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)a.Xp, 0, a.xp_bytes, 0x00020000);
  const unsigned wl = lane * 16, xl = (m * 4 + g) * 16;                  // per-lane byte offsets
  const unsigned kstride_b = a.NBtot * 1024u, kts_b = a.RB * 2048u;      // bytes per k-tile
  unsigned wq = nbw * 1024u, xq = (rb0 * 128u + w * 64u) * 16u;           // stage to load next (uniform)
  constexpr int STAGE = DKS * DM * 128;                 // pieces per LDS stage

  f32x4 acc[DN][DM];
#pragma unroll
  for (int i = 0; i < DN; ++i)
#pragma unroll
    for (int j = 0; j < DM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Two register sets of A tiles (wa, wb) alternate between "being multiplied" and "being
  // loaded"; B tiles go global -> registers (xs) -> the other LDS stage.  The loads of stage
  // s+1 are issued before the MFMAs of stage s (sched_barrier keeps them there) and are
  // parked in LDS half-way through them, so nothing but the barrier separates two stages.
  u32x4 wa[DKS][DN], wb[DKS][DN], xs[DKS][DM / 2];
  auto issue = [&](u32x4 (&wr)[DKS][DN]) {
    // B first: the LDS write only has to wait for these (the counter retires loads in order)
#pragma unroll
    for (int ks = 0; ks < DKS; ++ks)
#pragma unroll
      for (int i = 0; i < DM / 2; ++i) xs[ks][i] = __builtin_amdgcn_raw_buffer_load_b128(rx, xl, xq + ks * kts_b + i * 4096, 0);
#pragma unroll
    for (int ks = 0; ks < DKS; ++ks)
#pragma unroll
      for (int i = 0; i < DN; ++i) wr[ks][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, wl + i * 1024, wq + ks * kstride_b, 0);
  };
  auto stash = [&](int buf) {
    u32x4 *dst = bs + buf * STAGE + tid;
#pragma unroll
    for (int ks = 0; ks < DKS; ++ks)
#pragma unroll
      for (int i = 0; i < DM / 2; ++i) dst[ks * (DM * 128) + i * 256] = xs[ks][i];
  };
  // MFMAs of one stage.  The B tiles of step t+1 are read from LDS while the 2*DN MFMAs of
  // step t run, and the next stage's B tiles are written to the other LDS stage after half of
  // the steps; the sched_group_barrier sequence pins that interleaving.
  auto multiply = [&](const u32x4 (&wr)[DKS][DN], int buf) {
    const u32x4 *bcur = bs + buf * STAGE + lane;
    constexpr int T = DKS * DM, STASH_AT = T - 2;
    u32x4 f[2][2];
    f[0][0] = bcur[0];
    f[0][1] = bcur[64];
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const int ks = t / DM, j = t % DM;
      if (t + 1 < T) {
        f[(t + 1) & 1][0] = bcur[(t + 1) * 128];
        f[(t + 1) & 1][1] = bcur[(t + 1) * 128 + 64];
      }
#pragma unroll
      for (int i = 0; i < DN; ++i) acc[i][j] = mfma_bf16(wr[ks][i], f[t & 1][0], acc[i][j]);
#pragma unroll
      for (int i = 0; i < DN; ++i) acc[i][j] = mfma_bf16(wr[ks][i], f[t & 1][1], acc[i][j]);
      if (t == STASH_AT) stash(buf ^ 1);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);        // DS reads of step 0
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (t + 1 < T) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // DS reads of step t+1
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * DN, 0);            // MFMAs of step t
      if (t == STASH_AT) __builtin_amdgcn_sched_group_barrier(0x200, DKS * DM / 2, 0);   // DS writes
    }
  };
  const int NS = a.KT / DKS;   // even: K is a multiple of 256
  const unsigned wstep = DKS * kstride_b, xstep = DKS * kts_b;
  issue(wa);
  stash(0);
  wq += wstep; xq += xstep;
  __syncthreads();
  for (int st = 0; st < NS; st += 2) {
    issue(wb);                       // stage st+1
    if (st + 2 < NS) { wq += wstep; xq += xstep; }   // the last stage re-issues its own loads (ignored)
    __builtin_amdgcn_sched_barrier(0);
    multiply(wa, 0);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    issue(wa);                       // stage st+2
    if (st + 2 < NS) { wq += wstep; xq += xstep; }
    __builtin_amdgcn_sched_barrier(0);
    multiply(wb, 1);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  }

  constexpr int STEP = EPI == EPI_SWIGLU ? 2 : 1;
#pragma unroll
  for (int i = 0; i < DN; i += STEP) {
    const int nb = nbw + i;
    if (nb < tn * (4 * DN)) continue;   // slid-back duplicate of a neighbour's row-block
#pragma unroll
    for (int j = 0; j < DM; ++j) {
      const int rb = rb0 + j, row = rb * 16 + m;
      const bool row_ok = row < a.rows;
      const float rinv = NORM ? a.rinv[row] : 1.f;
      epi_tile<EPI>(a, acc[i][j], acc[i + STEP - 1][j], nb, g, m, rb, row_ok, rinv, kts);
    }
  }
}

template <int EPI, bool NORM, int DM>
static void launch_dense_tile(const GemmArgs &a, hipStream_t s) {
  constexpr int sm = 2 * DKS * DM * 128 * 16;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void *)gemm_dense_kernel<EPI, NORM, DM>, hipFuncAttributeMaxDynamicSharedMemorySize, sm);
    attr_set = true;
  }
  const int tiles = ((a.NBtot + 4 * DN - 1) / (4 * DN)) * ((a.rows + DM * 16 - 1) / (DM * 16));
  gemm_dense_kernel<EPI, NORM, DM><<<(tiles + 7) / 8 * 8, 256, sm, s>>>(a);
}

template <int EPI, bool NORM>
static void launch_dense_cfg(const GemmArgs &a, hipStream_t s) {
  // 256 compute units x 2 resident workgroups: estimate both tilings in rounds of 512
  // workgroups; a 64-row tile costs about 0.55 of a 128-row one.
  const long nt = (a.NBtot + 4 * DN - 1) / (4 * DN);
  const long t8 = nt * ((a.rows + 127) / 128), t4 = nt * ((a.rows + 63) / 64);
  const double c8 = (double)((t8 + 511) / 512), c4 = 0.55 * (double)((t4 + 511) / 512);
  if (c4 < c8) launch_dense_tile<EPI, NORM, 4>(a, s);
  else launch_dense_tile<EPI, NORM, 8>(a, s);
}

void launch_gemm_dense(const GemmLaunch &L, int RB, const float *rinv, hipStream_t s) {
  GemmArgs a{};
  a.W = (const u32x4 *)L.W->tiled;
  a.NBtot = L.W->N / 16;
  a.KT = L.W->K / 32;
  a.Xp = (const u32x4 *)L.Xp;
  a.rows = L.rows;
  a.RB = RB;
  a.w_bytes = (int)((size_t)L.W->N * L.W->K * 2);
  a.xp_bytes = (int)((size_t)L.W->K * RB * 64);
  a.rinv = rinv;
  a.bias = L.bias;
  a.Xp_out = (u32x4 *)L.Xp_out; a.gain_out = L.gain_out; a.ssq_out = L.ssq_out;
  int end = 0;
  for (int i = 0; i < 3; ++i) {
    if (i < L.nseg) end += L.seg_N[i] / 16;
    a.seg[i] = GemmSeg{i < L.nseg ? L.Y[i] : nullptr, i < L.nseg ? L.ldy[i] : 0, i < L.nseg ? end : 0x7fffffff};
  }
  a.rope_tab = L.rope_tab; a.Kc = (uint16_t *)L.Kc; a.Vc = (uint16_t *)L.Vc;
  a.pos0 = L.pos0; a.n_ctx = L.n_ctx; a.hd = L.hd;
  const bool norm = rinv != nullptr;
  if (L.epi == EPI_QKV) launch_dense_cfg<EPI_QKV, true>(a, s);
  else if (L.epi == EPI_SWIGLU) launch_dense_cfg<EPI_SWIGLU, true>(a, s);
  else if (L.epi == EPI_RESID) launch_dense_cfg<EPI_RESID, false>(a, s);
  else if (norm) launch_dense_cfg<EPI_STORE, true>(a, s);
  else launch_dense_cfg<EPI_STORE, false>(a, s);
}

// ------------------------------------------------------------------ 1/rms of every row
// ssq: [RB][P][16] partial sums of x^2 -> rinv[rb*16 + m]; one workgroup per row-block,
// 16 threads per row, fixed summation order.
__global__ __launch_bounds__(256) void rinv_finalize_kernel(const float *ssq, int P, int K, float eps, float *rinv) {
  __shared__ float sh[256];
  const int rb = blockIdx.x, m = threadIdx.x & 15, pg = threadIdx.x >> 4;
  float t = 0.f;
  for (int p = pg; p < P; p += 16) t += ssq[((size_t)rb * P + p) * 16 + m];
  sh[threadIdx.x] = t;
  __syncthreads();
  if (threadIdx.x < 16) {
    float tot = 0.f;
    for (int i = 0; i < 16; ++i) tot += sh[i * 16 + threadIdx.x];
    rinv[rb * 16 + threadIdx.x] = 1.0f / sqrtf(tot / (float)K + eps);
  }
}

void launch_rinv_finalize(const float *ssq, int RBused, int P, int K, float eps, float *rinv, hipStream_t s) {
  rinv_finalize_kernel<<<RBused, 256, 0, s>>>(ssq, P, K, eps, rinv);
}

// ------------------------------------------------------------------ packed-form producers
// Embedding rows -> float residual stream, packed(x * gain) and the row's sum of x^2 ([rb][1][16]).
__global__ __launch_bounds__(256) void embed_dense_kernel(const uint16_t *emb, const int32_t *ids, int d, const float *gain,
                                                          float *x, u32x4 *Xp, size_t kts, float *ssq) {
  __shared__ float red[4];
  const int r = blockIdx.x, rb = r >> 4, m = r & 15;
  const uint16_t *src = emb + (size_t)ids[r] * d;
  u32x4 *xp = Xp + (size_t)rb * 128;
  float ss = 0.f;
  for (int k0 = threadIdx.x * 4; k0 < d; k0 += 1024) {
    const uint2 raw = *reinterpret_cast<const uint2 *>(src + k0);
    const float v0 = __uint_as_float(raw.x << 16), v1 = __uint_as_float(raw.x & 0xffff0000u);
    const float v2 = __uint_as_float(raw.y << 16), v3 = __uint_as_float(raw.y & 0xffff0000u);
    *reinterpret_cast<float4 *>(x + (size_t)r * d + k0) = make_float4(v0, v1, v2, v3);
    ss += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3;
    const float4 gn = *reinterpret_cast<const float4 *>(gain + k0);
    packed_store4(xp, m, k0, v0 * gn.x, v1 * gn.y, v2 * gn.z, v3 * gn.w, kts);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssq[r] = (red[0] + red[1]) + (red[2] + red[3]);
}

void launch_embed_dense(const void *emb, const int32_t *ids_dev, int rows, int d, const float *gain, float *x, void *Xp,
                        int RB, float *ssq, hipStream_t s) {
  embed_dense_kernel<<<rows, 256, 0, s>>>((const uint16_t *)emb, ids_dev, d, gain, x, (u32x4 *)Xp, (size_t)RB * 128, ssq);
}

// Draft head input of every slot of the chunk whose next token is known (Eq. 2):
// [RMSNorm(x_r) * gain ; embedding of the following token] -> packed, K = 2d.
__global__ __launch_bounds__(256) void draft_cat_dense_kernel(const float *x, int d, const float *gain, float eps,
                                                              const uint16_t *emb, const int32_t *next_ids, u32x4 *Xp,
                                                              size_t kts) {
  __shared__ float red[4];
  const int r = blockIdx.x, rb = r >> 4, m = r & 15;
  const float *xr = x + (size_t)r * d;
  float ss = 0.f;
  for (int k0 = threadIdx.x * 4; k0 < d; k0 += 1024) {
    const float4 v = *reinterpret_cast<const float4 *>(xr + k0);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float rinv = 1.0f / sqrtf(((red[0] + red[1]) + (red[2] + red[3])) / (float)d + eps);
  u32x4 *xp = Xp + (size_t)rb * 128;
  const uint16_t *e = emb + (size_t)next_ids[r] * d;
  for (int k0 = threadIdx.x * 4; k0 < d; k0 += 1024) {
    const float4 v = *reinterpret_cast<const float4 *>(xr + k0);
    const float4 gn = *reinterpret_cast<const float4 *>(gain + k0);
    packed_store4(xp, m, k0, v.x * rinv * gn.x, v.y * rinv * gn.y, v.z * rinv * gn.z, v.w * rinv * gn.w, kts);
    const uint2 raw = *reinterpret_cast<const uint2 *>(e + k0);
    packed_store4(xp, m, d + k0, __uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                  __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u), kts);
  }
}

void launch_draft_cat_dense(const float *x, int rows, int d, const float *gain, float eps, const void *emb,
                            const int32_t *next_ids, void *Xp, int RB, hipStream_t s) {
  draft_cat_dense_kernel<<<rows, 256, 0, s>>>(x, d, gain, eps, (const uint16_t *)emb, next_ids, (u32x4 *)Xp, (size_t)RB * 128);
}

// ------------------------------------------------------------------ causal attention of a prompt chunk
// q: float [rows][H*HD] of the chunk (already rotated); chunk row i sits at slot pos0 + i and
// sees slots 0..pos0+i of the tiled cache (which already holds the chunk's own K and V).
// Pairs (row, query head of the KV head's group) are numbered r = row*G + head%G; a wave owns
// MT tiles of 16 consecutive pairs and walks the visible keys 32 at a time: the K and V tiles
// of a step (16 KB at head_dim 128) are loaded once and multiplied against all MT tiles, which
// halves the cache traffic per MFMA against one tile per wave.  Late (long) tiles are
// scheduled first.  No barriers, no LDS: every wave is independent.
template <int HD, int MT>
__global__ __launch_bounds__(256) void attn_prefill_kernel(const float *q, int rows, int pos0, int H, int Hkv, int n_ctx,
                                                           const u32x4 *Kc, const u32x4 *Vc, u32x4 *Xp_out, size_t kts,
                                                           float scale_log2e) {
  constexpr int DT = HD / 32, VT = HD / 16;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, g = lane >> 4, m = lane & 15;
  const int kh = blockIdx.x, G = H / Hkv, R = rows * G;
  const int r0 = (((int)gridDim.y - 1 - (int)blockIdx.y) * 4 + w) * (16 * MT);
  if (r0 >= R) return;   // wave-uniform
  int row[MT], head[MT], limit[MT];
  bool rok[MT];
  u32x4 qh[MT][DT], ql[MT][DT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int r = r0 + t * 16 + m;
    rok[t] = r < R;
    const int rr = rok[t] ? r : R - 1;
    row[t] = rr / G;
    head[t] = kh * G + rr % G;
    limit[t] = pos0 + row[t];   // last slot this lane's row may see
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const float *src = q + ((size_t)row[t] * H + head[t]) * HD + dt * 32 + g * 8;
      const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
      uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
      split2(a.x * scale_log2e, a.y * scale_log2e, h0, l0);
      split2(a.z * scale_log2e, a.w * scale_log2e, h1, l1);
      split2(b.x * scale_log2e, b.y * scale_log2e, h2, l2);
      split2(b.z * scale_log2e, b.w * scale_log2e, h3, l3);
      qh[t][dt] = u32x4{h0, h1, h2, h3};
      ql[t][dt] = u32x4{l0, l1, l2, l3};
    }
  }
  const int last_key = pos0 + min(r0 + 16 * MT - 1, R - 1) / G;   // last slot any row of the wave sees

  float mx[MT], lsum[MT];
  f32x4 O[MT][VT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    mx[t] = -INFINITY;
    lsum[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < VT; ++dt) O[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // K and V tiles of a step live in registers; the K tiles of the next step are requested as soon as
  // this step's scores are done and the V tiles as soon as its P.V products are issued, so the loads
  // fly behind the softmax / MFMA work instead of in front of it (no extra registers).
  u32x4 kreg[2][DT], vreg[VT];
  auto load_k = [&](int kb) {
    const u32x4 *kp = Kc + (((size_t)kh * (n_ctx / 16) + (kb >> 4)) * DT) * 64 + lane;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) kreg[kt][dt] = kp[(kt * DT + dt) * 64];
  };
  auto load_v = [&](int kb) {
    const u32x4 *vp = Vc + (((size_t)kh * (n_ctx / 32) + (kb >> 5)) * VT) * 64 + lane;
#pragma unroll
    for (int dt = 0; dt < VT; ++dt) vreg[dt] = vp[dt * 64];
  };
  load_k(0);
  load_v(0);
  const int last_kb = last_key & ~31;
  for (int kb = 0; kb <= last_key; kb += 32) {
    const int kb_next = min(kb + 32, last_kb);   // the last step re-requests its own tiles (ignored)
    f32x4 S[MT][2];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      S[t][0] = f32x4{0.f, 0.f, 0.f, 0.f};
      S[t][1] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        S[t][0] = mfma_bf16(kreg[0][dt], qh[t][dt], S[t][0]);
        S[t][1] = mfma_bf16(kreg[1][dt], qh[t][dt], S[t][1]);
        S[t][0] = mfma_bf16(kreg[0][dt], ql[t][dt], S[t][0]);
        S[t][1] = mfma_bf16(kreg[1][dt], ql[t][dt], S[t][1]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    load_k(kb_next);
    __builtin_amdgcn_sched_barrier(0);
    u32x4 ph[MT], pl[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      float bmax = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int key = kb + kt * 16 + 4 * g + e;
          S[t][kt][e] = key <= limit[t] ? S[t][kt][e] : -INFINITY;
          bmax = fmaxf(bmax, S[t][kt][e]);
        }
      bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
      bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
      const float mnew = fmaxf(mx[t], bmax);   // finite from the first block on: slot 0 is visible to every row
      const float alpha = __builtin_amdgcn_exp2f(mx[t] - mnew);
      float bsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          S[t][kt][e] = __builtin_amdgcn_exp2f(S[t][kt][e] - mnew);
          bsum += S[t][kt][e];
        }
      bsum += __shfl_xor(bsum, 16, 64);
      bsum += __shfl_xor(bsum, 32, 64);
      lsum[t] = lsum[t] * alpha + bsum;
      mx[t] = mnew;
#pragma unroll
      for (int dt = 0; dt < VT; ++dt) O[t][dt] *= alpha;
      // P^T as B operand: k-slot e of lane group g = key 16*(e/4) + 4g + e%4 of the 32-key block
      uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
      split2(S[t][0][0], S[t][0][1], h0, l0);
      split2(S[t][0][2], S[t][0][3], h1, l1);
      split2(S[t][1][0], S[t][1][1], h2, l2);
      split2(S[t][1][2], S[t][1][3], h3, l3);
      ph[t] = u32x4{h0, h1, h2, h3};
      pl[t] = u32x4{l0, l1, l2, l3};
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
#pragma unroll
      for (int dt = 0; dt < VT; ++dt) O[t][dt] = mfma_bf16(vreg[dt], ph[t], O[t][dt]);
#pragma unroll
      for (int dt = 0; dt < VT; ++dt) O[t][dt] = mfma_bf16(vreg[dt], pl[t], O[t][dt]);
    }
    __builtin_amdgcn_sched_barrier(0);
    load_v(kb_next);
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    if (rok[t]) {
      const float inv = 1.0f / lsum[t];
      u32x4 *xp = Xp_out + (size_t)(row[t] >> 4) * 128;
#pragma unroll
      for (int dt = 0; dt < VT; ++dt)
        packed_store4(xp, row[t] & 15, head[t] * HD + dt * 16 + 4 * g, O[t][dt][0] * inv, O[t][dt][1] * inv,
                      O[t][dt][2] * inv, O[t][dt][3] * inv, kts);
    }
  }
}

void launch_attention_prefill(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                              void *Xp_out, int RB, hipStream_t s) {
  constexpr int MT = 2;
  const int G = c.n_heads / c.n_kv_heads, R = rows * G, HD = c.head_dim;
  const dim3 grid(c.n_kv_heads, (R + 64 * MT - 1) / (64 * MT));
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
  const u32x4 *Kc = (const u32x4 *)kv_layer, *Vc = (const u32x4 *)((const char *)kv_layer + v_off);
  const int cap = kv_capacity(c);
  if (HD == 128)
    attn_prefill_kernel<128, MT><<<grid, 256, 0, s>>>(q, rows, pos0, c.n_heads, c.n_kv_heads, cap, Kc, Vc, (u32x4 *)Xp_out,
                                                     (size_t)RB * 128, scale_log2e);
  else
    attn_prefill_kernel<64, MT><<<grid, 256, 0, s>>>(q, rows, pos0, c.n_heads, c.n_kv_heads, cap, Kc, Vc, (u32x4 *)Xp_out,
                                                    (size_t)RB * 128, scale_log2e);
}

}  // namespace ae
