// Skinny bf16 GEMMs of the decode step on the gfx950 matrix cores.
//
//   Y[m][n] = epilogue( sum_k X[m][k] * W[n][k] ),  m < rows <= 16,  W bf16.
//
// These GEMMs are HBM-bound: every weight byte is read exactly once per call and the
// whole job is to keep the memory system saturated.  Design:
//  * Weights are re-tiled once (ae_init) into the A-operand layout of
//    v_mfma_f32_16x16x32_bf16: a tile = 16 output rows x 32 k = 1 KB whose 16-byte piece
//    `lane` is what lane (lane%16 = row, lane/16 = k-octet) feeds to the instruction, so a
//    wave-wide 128-bit load is one coalesced 1 KB burst with no LDS staging.  Tiles are
//    stored k-major, tile (nb, kt) at index kt*NB + nb: the row-blocks a workgroup owns
//    are contiguous for every kt and neighbouring workgroups read neighbouring memory,
//    which measured ~25% faster than strip-major storage on MI355X.
//  * Activations travel between kernels already in B-operand form ("packed"): for every
//    k-tile two 1 KB tiles (bf16 hi, bf16 lo; x ~= hi + lo keeps 16 significant bits),
//    slot = row*4 + k-octet (rows contiguous).  Producers (embedding, GEMM epilogues, attention merge)
//    write this form, so the GEMM hot loop is only loads and MFMAs (two per weight tile).
//  * A workgroup owns NACC adjacent row-blocks and splits K over its NW waves; every wave
//    runs a register ring of D k-tiles (loads for tile t+D are issued when tile t is
//    consumed), then the waves' partial tiles are summed through LDS in a fixed order.
//    No atomics; column m of a tile never mixes with another column, so a row's result
//    is independent of the number of rows in the block.
//  * RMSNorm is folded in: the producer stores x*gain (packed) and per-row-block partial
//    sums of x^2; the consumer sums the partials in a fixed order and scales its
//    accumulators by 1/rms.  Epilogues: store(+bias), residual add, SwiGLU (gate and up
//    tiles interleaved in the matrix), each optionally emitting the packed form (and the
//    x^2 partials) for the next GEMM.
#include "ae_internal.h"
#include "gemm_epilogue.h"
#include "packed.h"

namespace ae {

// ------------------------------------------------------------------ re-tiling (set-up)
// Row-block nb of a row-major [N,K] bf16 matrix goes to row-block (nb_off + nb*nb_stride)
// of a fused k-major tiled matrix with NBtot row-blocks.  perm_hd != 0 (q and k
// projections, perm_hd = head_dim) reorders the rows of every head so that tile j of a head
// holds rows 8j..8j+7 followed by their rotary partners hd/2+8j..hd/2+8j+7: a rotary
// pair then sits in lanes l and l^32 of the same accumulator (see the EPI_QKV epilogue).
__global__ void retile_kernel(const uint4 *src, uint4 *dst, int NB, int KT, int NBtot, int nb_off, int nb_stride,
                              int perm_hd) {
  const size_t total = (size_t)NB * KT * 64;
  for (size_t o = blockIdx.x * (size_t)blockDim.x + threadIdx.x; o < total; o += (size_t)gridDim.x * blockDim.x) {
    const int lane = o & 63;
    const size_t tile = o >> 6;
    const int nb = tile % NB;
    const size_t kt = tile / NB;
    size_t row = (size_t)nb * 16 + (lane & 15);
    if (perm_hd) {
      const int bph = perm_hd / 16, head = nb / bph, j = nb % bph, rho = lane & 15;
      row = (size_t)head * perm_hd + (rho < 8 ? 8 * j + rho : perm_hd / 2 + 8 * j + rho - 8);
    }
    dst[(kt * NBtot + nb_off + (size_t)nb * nb_stride) * 64 + lane] = src[row * (size_t)(KT * 4) + kt * 4 + (lane >> 4)];
  }
}

void launch_retile(const void *rowmajor, int N, int K, void *tiled, int NBtot, int nb_off, int nb_stride, int perm_hd,
                   hipStream_t s) {
  retile_kernel<<<2048, 256, 0, s>>>((const uint4 *)rowmajor, (uint4 *)tiled, N / 16, K / 32, NBtot, nb_off, nb_stride,
                                     perm_hd);
}

// ------------------------------------------------------------------ GEMM
// GATED instantiations (draft tokens whose existence a device-side rule decides) check
// a.gate at entry; the check is compiled out of the others: even with a null pointer it
// measured 0.3-0.8 us per launch.
template <int EPI, bool NORM, int NACC, int NW, int D, bool GATED>
__global__ __launch_bounds__(NW * 64) void gemm_mfma_kernel(const GemmArgs a) {
  __shared__ f32x4 red[NW][NACC][64];
  if constexpr (GATED) AE_GATE(a.gate);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int g = lane >> 4, m = lane & 15;
  // a workgroup hanging over the end of the matrix slides back (recomputes, stores nothing new)
  const int nb0 = min((int)blockIdx.x * NACC, a.NBtot - NACC);
  const bool row_ok = m < a.rows;
  const int xrow = a.row0 + (row_ok ? m : a.rows - 1);    // rows beyond the block re-read the last row
  const int xlane = xrow * 4 + g;   // packed slot of (row, k-octet)

  const u32x4 *wp = a.W + (size_t)nb0 * 64 + lane;
  const size_t kstride = (size_t)a.NBtot * 64;
  const u32x4 *xp = a.Xp + xlane;
  // K is cut into chunks of D k-tiles dealt round-robin to the waves: at any time the whole
  // grid reads one narrow band of the matrix (neighbouring k-tiles are neighbours in memory)
  const int NC = a.KT / D;

  f32x4 acc[NACC];
#pragma unroll
  for (int i = 0; i < NACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

  // what the epilogue of this wave's row-blocks will read (old residual, gain, bias, rotary
  // table): requested now, consumed behind the main loop
  constexpr int STEP = EPI == EPI_SWIGLU ? 2 : 1;
  constexpr int NE = NACC / STEP >= NW ? (NACC / STEP + NW - 1) / NW : 1;   // row-blocks per wave in the epilogue
  EpiPre pre[NE];
  if (EPI != EPI_SWIGLU) {
#pragma unroll
    for (int e = 0; e < NE; ++e) {
      const int rb = (w + e * NW) * STEP;
      if (rb < NACC) pre[e] = epi_prefetch<EPI>(a, nb0 + rb, g, m, row_ok);
    }
  }

  u32x4 xb[D][2], wb[D][NACC];
  if (w < NC) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      const size_t t = (size_t)w * D + j;
      xb[j][0] = xp[t * 128];
      xb[j][1] = xp[t * 128 + 64];
#pragma unroll
      for (int i = 0; i < NACC; ++i) wb[j][i] = wp[t * kstride + i * 64];
    }
  }

  // 1/rms of every row from the producer's partial sums of x^2 ([P_in][16] floats): wave 0
  // sums them with wide independent loads while its weight loads are in flight and
  // publishes the 16 values through LDS (read after the barrier below).  Fixed order.
  __shared__ float rinv_s[16];
  if (NORM && w == 0) {
    const float4 *pp = reinterpret_cast<const float4 *>(a.ssq_in);
    const int n4 = a.P_in * 4;   // float4 count; lane l covers rows 4*(l%4)..+3 of partial (i*64+l)/4
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = lane; i < n4; i += 64) {
      const float4 v = pp[i];
      t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
    }
#pragma unroll
    for (int o = 4; o < 64; o <<= 1) {
      t.x += __shfl_xor(t.x, o, 64); t.y += __shfl_xor(t.y, o, 64);
      t.z += __shfl_xor(t.z, o, 64); t.w += __shfl_xor(t.w, o, 64);
    }
    if (lane < 4) {
      const float kk = (float)(a.KT * 32);
      rinv_s[lane * 4 + 0] = 1.0f / sqrtf(t.x / kk + a.eps);
      rinv_s[lane * 4 + 1] = 1.0f / sqrtf(t.y / kk + a.eps);
      rinv_s[lane * 4 + 2] = 1.0f / sqrtf(t.z / kk + a.eps);
      rinv_s[lane * 4 + 3] = 1.0f / sqrtf(t.w / kk + a.eps);
    }
  }

  for (int c = w; c < NC; c += NW) {
    const int cn = c + NW < NC ? c + NW : c;   // the last chunk re-issues its own loads (ignored)
#pragma unroll
    for (int j = 0; j < D; ++j) {
#pragma unroll
      for (int i = 0; i < NACC; ++i) {
        const bf16x8 wa = __builtin_bit_cast(bf16x8, wb[j][i]);
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, xb[j][0]), acc[i], 0, 0, 0);
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, xb[j][1]), acc[i], 0, 0, 0);
      }
      // Refill slot j at once (a rolling ring: D k-tiles stay in flight).  With one row-block per
      // workgroup the scheduler would otherwise sink all D refills below the last MFMA of the
      // chunk, so that the ring drains to empty once per chunk (o-proj + down-proj of a 7B layer:
      // 30.4 -> 28.3 us with the barriers; the wider shapes interleave by themselves).
      if (NACC == 1) __builtin_amdgcn_sched_barrier(0);
      const size_t t = (size_t)cn * D + j;
      xb[j][0] = xp[t * 128];
      xb[j][1] = xp[t * 128 + 64];
#pragma unroll
      for (int i = 0; i < NACC; ++i) wb[j][i] = wp[t * kstride + i * 64];
      if (NACC == 1) __builtin_amdgcn_sched_barrier(0);
    }
  }

  // cross-wave (split-K) reduction through LDS, fixed order
#pragma unroll
  for (int i = 0; i < NACC; ++i) red[w][i][lane] = acc[i];
  __syncthreads();
  const float rinv = NORM ? rinv_s[xrow] : 1.f;

#pragma unroll
  for (int e = 0; e < NE; ++e) {
    const int rb = (w + e * NW) * STEP;
    if (rb >= NACC) break;
    const int nb = nb0 + rb;
    if (nb < (int)blockIdx.x * NACC) continue;   // slid-back duplicate of a neighbour's row-block
    f32x4 s = red[0][rb][lane];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) s += red[ww][rb][lane];
    f32x4 u = s;
    if (EPI == EPI_SWIGLU) {
      u = red[0][rb + 1][lane];
#pragma unroll
      for (int ww = 1; ww < NW; ++ww) u += red[ww][rb + 1][lane];
    }
    epi_tile<EPI>(a, s, u, nb, g, m, 0, row_ok, rinv, 128, EPI != EPI_SWIGLU ? &pre[e] : nullptr);
  }
}

template <int EPI, bool NORM, int NACC, int NW, int D>
static void launch_cfg(const GemmArgs &a, hipStream_t s) {
  const int grid = (a.NBtot + NACC - 1) / NACC;
  if (a.gate) gemm_mfma_kernel<EPI, NORM, NACC, NW, D, true><<<grid, NW * 64, 0, s>>>(a);
  else gemm_mfma_kernel<EPI, NORM, NACC, NW, D, false><<<grid, NW * 64, 0, s>>>(a);
}

// Shape -> (row-blocks per workgroup, waves, ring depth), tuned on MI355X at the 7B shape: wide
// matrices amortise the activation loads over 8 row-blocks, narrow ones need every CU.  With
// the K chunks dealt round-robin to the waves a shallow ring (2 k-tiles per wave) keeps the
// band of the matrix that is being read narrow, which the wide shapes prefer (gate/up 31.2 ->
// 30.8 us, QKV 19.6 -> 19.2 us, LM head 46.2 -> 43.4 us against the deeper rings).
static int g_num_cus = 256;   // compute units of the device (gemm_mfma_setup)

void gemm_mfma_setup(int num_cus) {
  if (num_cus > 0) g_num_cus = num_cus;
}

template <int EPI, bool NORM>
static void launch_shape(const GemmArgs &a, hipStream_t s) {
  if (EPI == EPI_SWIGLU) {
    // 6 row-blocks per workgroup while that still gives at most one workgroup per compute unit
    // (7B gate/up: 230 workgroups, 30.4 us against 30.7 with 8 row-blocks and 172 workgroups)
    if (a.NBtot >= 1024 && (a.NBtot + 5) / 6 <= g_num_cus) launch_cfg<EPI, NORM, 6, 8, 2>(a, s);
    else if (a.NBtot >= 1024) launch_cfg<EPI, NORM, 8, 4, 2>(a, s);
    else if (a.NBtot >= 512) launch_cfg<EPI, NORM, 4, 4, 4>(a, s);
    else launch_cfg<EPI, NORM, 2, 4, 4>(a, s);
  } else {
    if (a.NBtot >= 1536) launch_cfg<EPI, NORM, 8, 8, 2>(a, s);
    else if (a.NBtot >= 640) launch_cfg<EPI, NORM, 4, 8, 2>(a, s);
    // 8B-GQA QKV (384 row-blocks): (2,8,4) 12.6 us against (2,4,8) 15.6, (2,8,2) 13.5, (2,16,2) 13.0, (1,4,4) 15.2
    else if (a.NBtot >= 384) launch_cfg<EPI, NORM, 2, 8, 4>(a, s);
    // more row-blocks than compute units (13B o / down, 320): two per workgroup and 16 waves, 21.1 us
    // for the pair's average against 26.9 with (1,4,4), 24.1 (2,8,4), 22.2 (2,16,4), 28.7 (1,16,2)
    else if (a.NBtot > g_num_cus) launch_cfg<EPI, NORM, 2, 16, 2>(a, s);
    // at most one row-block per compute unit (7B o / down, 256): (1,4,8) 14.1, (1,8,4) 13.0, (1,16,1) 13.3,
    // (1,2,8) 13.0, (2,16,2) 16.3 us against 12.7
    else launch_cfg<EPI, NORM, 1, 4, 4>(a, s);
  }
}

void launch_gemm_mfma(const GemmLaunch &L, hipStream_t s) {
  GemmArgs a{};
  a.W = (const u32x4 *)L.W->tiled;
  a.NBtot = L.W->N / 16;
  a.KT = L.W->K / 32;
  a.Xp = (const u32x4 *)L.Xp;
  a.rows = L.rows;
  a.row0 = L.row0;
  a.RB = 1;
  a.ssq_in = L.ssq_in; a.P_in = L.P_in; a.eps = L.eps;
  a.bias = L.bias;
  a.Xp_out = (u32x4 *)L.Xp_out; a.gain_out = L.gain_out; a.ssq_out = L.ssq_out;
  int end = 0;
  for (int i = 0; i < 3; ++i) {
    if (i < L.nseg) end += L.seg_N[i] / 16;
    a.seg[i] = GemmSeg{i < L.nseg ? L.Y[i] : nullptr, i < L.nseg ? L.ldy[i] : 0, i < L.nseg ? end : 0x7fffffff};
  }
  const bool norm = L.ssq_in != nullptr;
  a.amax_val = L.amax_val; a.amax_idx = L.amax_idx;
  a.lse_sum = L.amax_val ? L.lse_sum : nullptr; a.lse_inv_t = L.lse_inv_t;
  a.rope_tab = L.rope_tab; a.Kc = (uint16_t *)L.Kc; a.Vc = (uint16_t *)L.Vc;
  a.pos0 = L.pos0; a.n_ctx = L.n_ctx; a.hd = L.hd;
  a.gate = L.gate;
  if (L.epi == EPI_QKV) {
    launch_shape<EPI_QKV, true>(a, s);
  } else if (L.epi == EPI_SWIGLU) {
    if (norm) launch_shape<EPI_SWIGLU, true>(a, s); else launch_shape<EPI_SWIGLU, false>(a, s);
  } else if (L.epi == EPI_RESID) {
    launch_shape<EPI_RESID, false>(a, s);
  } else {
    if (norm) launch_shape<EPI_STORE, true>(a, s); else launch_shape<EPI_STORE, false>(a, s);
  }
}

// Embedding of token t -> packed row `row`, k = k_off .. k_off + d - 1 (the second half of the
// draft head's input [feature ; embedding of the next token]); all threads of the workgroup.
__device__ __forceinline__ void pack_embedding(const uint16_t *emb, int32_t t, int d, u32x4 *Xp, int row, int k_off) {
  const uint16_t *e = emb + (size_t)t * d;
  for (int k0 = threadIdx.x * 4; k0 < d; k0 += blockDim.x * 4) {
    const uint2 raw = *reinterpret_cast<const uint2 *>(e + k0);
    packed_store4(Xp, row, k_off + k0, __uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                  __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u));
  }
}

// AdaEAGLE-DDD bookkeeping behind draft token i = tok (Sec. 3.4, 4.2) from the LM-head epilogue's
// row-block statistics of row 0; all 256 threads call.  Fixed-shape reductions.
__device__ void ddd_finish(const DddFinish &d, int32_t tok, int i, DevState *st) {
  __shared__ float red_s[4];
  const int t = threadIdx.x;
  float mx = -INFINITY;
  for (int p = t; p < d.NB; p += 256) mx = fmaxf(mx, d.val[p]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  if ((t & 63) == 0) red_s[t >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red_s[0], red_s[1]), fmaxf(red_s[2], red_s[3]));
  __syncthreads();
  float se = 0.f;
  for (int p = t; p < d.NB; p += 256) se += d.lse_sum[p] * expf((d.val[p] - mx) * d.inv_t);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
  if ((t & 63) == 0) red_s[t >> 6] = se;
  __syncthreads();
  if (t == 0) {
    se = (red_s[0] + red_s[1]) + (red_s[2] + red_s[3]);
    const float lp = (d.logits[tok] - mx) * d.inv_t - logf(se);
    const float cum = (i == 0 ? 0.f : st->cum_logp) + lp;
    st->draft_lp[i] = lp;
    st->cum_logp = cum;
    st->draft_len = i + 1;
    if (i + 1 >= d.k && !(cum >= d.theta)) st->draft_live = 0;
  }
}

// Final argmax over the LM head's row-block partials (lowest token id wins ties), one
// workgroup per row.  pick_i >= 0 (draft head, one row): also applies the caller's override
// table, records draft token pick_i and, when cat.Xp is set, writes that token's embedding into
// the draft head's packed input row for the next chained forward.
__global__ __launch_bounds__(256) void argmax_finish_kernel(const float *val, const int32_t *idx, int NB, DevState *st,
                                                            int pick_i, const int32_t *gate, DraftCat cat, DddFinish ddd) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  __shared__ int32_t tok_s;
  AE_GATE(gate);
  const int row = blockIdx.x;
  float best = -INFINITY;
  int best_i = 0x7fffffff;
  const float *vr = val + (size_t)row * NB;
  const int32_t *ir = idx + (size_t)row * NB;
  for (int p0 = threadIdx.x; p0 < NB; p0 += 256 * 8) {   // 8 independent coalesced loads in flight
    float v[8];
    int i[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int p = p0 + j * 256;
      v[j] = p < NB ? vr[p] : -INFINITY;
      i[j] = p < NB ? ir[p] : 0x7fffffff;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (v[j] > best || (v[j] == best && i[j] < best_i)) { best = v[j]; best_i = i[j]; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(best_i, o, 64);
    if (ov > best || (ov == best && oi < best_i)) { best = ov; best_i = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = best_i; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < best_i)) { best = bv[w]; best_i = bi[w]; }
    int32_t t = best_i == 0x7fffffff ? 0 : best_i;
    st->argmax[row] = t;
    if (pick_i >= 0) {
      if (st->override_ids[pick_i] >= 0) t = st->override_ids[pick_i];
      st->draft_ids[pick_i] = t;
    }
    tok_s = t;
  }
  if (pick_i >= 0 && (cat.Xp || ddd.lse_sum)) {
    __syncthreads();
    if (cat.Xp) pack_embedding((const uint16_t *)cat.emb, tok_s, cat.d, (u32x4 *)cat.Xp, cat.row, cat.d);
    if (ddd.lse_sum) ddd_finish(ddd, tok_s, pick_i, st);
  }
}

void launch_argmax_finish(const float *val, const int32_t *idx, int NB, int rows, DevState *st, int pick_i, hipStream_t s,
                          const int32_t *gate, DraftCat cat, DddFinish ddd) {
  argmax_finish_kernel<<<rows, 256, 0, s>>>(val, idx, NB, st, pick_i, gate, cat, ddd);
}

// temperature > 0: the sampled token (st->argmax[0]) with the override table applied becomes draft
// token i; its embedding goes into the draft head's packed input row like above
__global__ __launch_bounds__(256) void pick_draft_packed_kernel(DevState *st, int i, const int32_t *gate, DraftCat cat,
                                                                DddFinish ddd) {
  AE_GATE(gate);
  int32_t t = st->argmax[0];
  if (st->override_ids[i] >= 0) t = st->override_ids[i];
  if (threadIdx.x == 0) st->draft_ids[i] = t;
  pack_embedding((const uint16_t *)cat.emb, t, cat.d, (u32x4 *)cat.Xp, cat.row, cat.d);
  if (ddd.lse_sum) ddd_finish(ddd, t, i, st);
}

void launch_pick_draft_packed(DevState *st, int i, hipStream_t s, const int32_t *gate, DraftCat cat, DddFinish ddd) {
  pick_draft_packed_kernel<<<1, 256, 0, s>>>(st, i, gate, cat, ddd);
}

// ------------------------------------------------------------------ packed-form producers
// Embedding rows -> float residual stream, packed(x * gain) and the full-row sum of x^2.
__global__ __launch_bounds__(256) void embed_packed_kernel(const uint16_t *emb, const int32_t *ids, int d,
                                                           const float *gain, float *x, u32x4 *Xp, float *ssq) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const uint16_t *src = emb + (size_t)ids[r] * d;
  float ss = 0.f;
  for (int k0 = threadIdx.x * 4; k0 < d; k0 += 1024) {
    const uint2 raw = *reinterpret_cast<const uint2 *>(src + k0);
    const float v0 = __uint_as_float(raw.x << 16), v1 = __uint_as_float(raw.x & 0xffff0000u);
    const float v2 = __uint_as_float(raw.y << 16), v3 = __uint_as_float(raw.y & 0xffff0000u);
    *reinterpret_cast<float4 *>(x + (size_t)r * d + k0) = make_float4(v0, v1, v2, v3);
    ss += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3;
    const float4 gn = *reinterpret_cast<const float4 *>(gain + k0);
    packed_store4(Xp, r, k0, v0 * gn.x, v1 * gn.y, v2 * gn.z, v3 * gn.w);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) ssq[r] = (red[0] + red[1]) + (red[2] + red[3]);
}

void launch_embed_packed(const void *emb, const int32_t *ids_dev, int rows, int d, const float *gain, float *x,
                         void *Xp, float *ssq, hipStream_t s) {
  embed_packed_kernel<<<rows, 256, 0, s>>>((const uint16_t *)emb, ids_dev, d, gain, x, (u32x4 *)Xp, ssq);
}

// float rows [rows][ld] (* gain) -> packed; one workgroup per row
__global__ void pack_rows_kernel(const float *src, int ld, int K, const float *gain, u32x4 *Xp) {
  const int r = blockIdx.x;
  for (int k0 = threadIdx.x * 4; k0 < K; k0 += blockDim.x * 4) {
    float4 v = *reinterpret_cast<const float4 *>(src + (size_t)r * ld + k0);
    if (gain) {
      const float4 gn = *reinterpret_cast<const float4 *>(gain + k0);
      v.x *= gn.x; v.y *= gn.y; v.z *= gn.z; v.w *= gn.w;
    }
    packed_store4(Xp, r, k0, v.x, v.y, v.z, v.w);
  }
}

void launch_pack_rows(const float *src, int ld, int rows, int K, const float *gain, void *Xp, hipStream_t s) {
  pack_rows_kernel<<<rows, 256, 0, s>>>(src, ld, K, gain, (u32x4 *)Xp);
}

// draft head input [feature ; embedding of the following token] -> packed, K = 2d
__global__ void draft_cat_packed_kernel(const float *feat, int feat_ld, const uint16_t *emb, const int32_t *next_ids,
                                        int d, u32x4 *Xp, const int32_t *gate) {
  AE_GATE(gate);
  const int r = blockIdx.x;
  const uint16_t *e = emb + (size_t)next_ids[r] * d;
  for (int k0 = threadIdx.x * 4; k0 < d; k0 += blockDim.x * 4) {
    const float4 f = *reinterpret_cast<const float4 *>(feat + (size_t)r * feat_ld + k0);
    packed_store4(Xp, r, k0, f.x, f.y, f.z, f.w);
    const uint2 raw = *reinterpret_cast<const uint2 *>(e + k0);
    packed_store4(Xp, r, d + k0, __uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u),
                  __uint_as_float(raw.y << 16), __uint_as_float(raw.y & 0xffff0000u));
  }
}

void launch_draft_cat_packed(const float *feat, int feat_ld, const void *emb, const int32_t *next_ids, int rows, int d,
                             void *Xp, hipStream_t s, const int32_t *gate) {
  draft_cat_packed_kernel<<<rows, 256, 0, s>>>(feat, feat_ld, (const uint16_t *)emb, next_ids, d, (u32x4 *)Xp, gate);
}

}  // namespace ae
