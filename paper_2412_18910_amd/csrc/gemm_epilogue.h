// Epilogues shared by the two bf16 MFMA GEMMs (the skinny decode GEMM of kernels_mfma.hip
// and the dense prompt GEMM of kernels_dense.hip).  Both hold a 16x16 output tile as the
// accumulator of v_mfma_f32_16x16x32_bf16: lane (g = lane/16, m = lane%16) owns output
// columns 16*nb + 4g .. +3 of activation row m of the tile's row-block.
#pragma once
#include "ae_internal.h"
#include "packed.h"

namespace ae {

__device__ __forceinline__ float silu_dev(float x) { return x / (1.0f + expf(-x)); }

struct GemmSeg {
  float *Y;     // float destination of this range of row-blocks (nullable: nothing stored)
  int ldy;
  int nb_end;   // exclusive end of the range in fused row-block indices
};

struct GemmArgs {
  const u32x4 *W;       // fused k-major tiled matrix
  const u32x4 *Xp;      // packed activations [KT][RB][2][64]
  const float *ssq_in;  // decode, NORM: [P_in][16] partial sums of x^2
  const float *rinv;    // dense, NORM: 1/rms of every row (nullable)
  const float *bias;    // [N] or nullptr (EPI_STORE, segment 0)
  u32x4 *Xp_out;        // packed output for the next GEMM (nullable)
  const float *gain_out;  // gain folded into Xp_out (nullable = 1)
  float *ssq_out;       // [RB][NBtot][16] partial sums of the new x^2 (nullable)
  GemmSeg seg[3];
  int NBtot, KT, rows, row0, P_in;   // output row m reads packed row row0 + m (decode)
  int RB;               // row-blocks held by the packed buffers (decode: 1)
  int w_bytes, xp_bytes;  // dense: sizes of W and Xp (buffer-load range checks)
  float eps;
  float *amax_val;      // EPI_STORE, LM head: per row, per row-block maximum of the outputs ...
  int32_t *amax_idx;    // ... and the lowest column index attaining it ([16][NBtot] each)
  float *lse_sum;       // with amax_val (nullable): per row, per row-block sum of exp((x - block max) * lse_inv_t)
  float lse_inv_t;
  // EPI_QKV: rotary embedding + KV-cache append in the epilogue
  const float2 *rope_tab;   // [slot][hd/2] (cos, sin)
  uint16_t *Kc, *Vc;        // this layer's tiled bf16 cache (layouts of kernels_attn_mfma.hip)
  int pos0, n_ctx, hd;
  const int32_t *gate;      // nullable: the kernel does nothing when *gate == 0
};

__device__ __forceinline__ uint16_t f2bf_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7f800000u) == 0x7f800000u) return (uint16_t)(u >> 16);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Values an epilogue reads from memory (old residual, gain, bias, rotary table).  The decode
// GEMM requests them before its main loop (epi_prefetch) so that their latency hides behind the
// weight stream instead of sitting at the very end of the kernel; the dense GEMM lets the
// epilogue load them itself (pre == nullptr).
struct EpiPre {
  float4 a, b;
};

// Which segment (q | k | v, or the single output) row-block nb falls in, and its index there.
__device__ __forceinline__ void epi_segment(const GemmArgs &a, int nb, int &si, int &nbs) {
  si = 0; nbs = nb;
  if (nb >= a.seg[0].nb_end) { si = 1; nbs = nb - a.seg[0].nb_end; }
  if (nb >= a.seg[1].nb_end) { si = 2; nbs = nb - a.seg[1].nb_end; }
}

template <int EPI>
__device__ __forceinline__ EpiPre epi_prefetch(const GemmArgs &a, int nb, int g, int m, bool row_ok) {
  EpiPre p;
  p.a = make_float4(0.f, 0.f, 0.f, 0.f);
  p.b = make_float4(1.f, 1.f, 1.f, 1.f);
  int si, nbs;
  epi_segment(a, nb, si, nbs);
  if (EPI == EPI_QKV) {
    if (si < 2) {   // (cos, sin) of the lane's two rotary pairs at the row's slot
      const int hd = a.hd, bph = hd >> 4, j = nbs % bph, slot = a.pos0 + (row_ok ? m : 0);
      const int i0 = 8 * j + 4 * (g & 1);
      p.a = *reinterpret_cast<const float4 *>(a.rope_tab + (size_t)slot * (hd >> 1) + i0);
      p.b = *reinterpret_cast<const float4 *>(a.rope_tab + (size_t)slot * (hd >> 1) + i0 + 2);
    }
  } else if (EPI == EPI_RESID || EPI == EPI_STORE) {
    const int n = nbs * 16 + g * 4;
    if (row_ok) {
      if (EPI == EPI_RESID) p.a = *reinterpret_cast<const float4 *>(a.seg[si].Y + (size_t)m * a.seg[si].ldy + n);
      else if (a.bias && si == 0) p.a = *reinterpret_cast<const float4 *>(a.bias + n);
      if (a.Xp_out && a.gain_out) p.b = *reinterpret_cast<const float4 *>(a.gain_out + n);
    }
  }
  return p;
}

// s = accumulator of row-block nb (EPI_SWIGLU: the gate block, u = the up block nb + 1).
// rb = row-block of the activations, the lane's row is rb*16 + m; kts = k-tile stride of the
// packed output (pieces).  Every lane of the wave must call this (it shuffles).
template <int EPI>
__device__ __forceinline__ void epi_tile(const GemmArgs &a, f32x4 s, f32x4 u, int nb, int g, int m, int rb, bool row_ok,
                                         float rinv, size_t kts, const EpiPre *pre = nullptr) {
  const int row = rb * 16 + m;
  u32x4 *xpo = a.Xp_out + (size_t)rb * 128;
  if (EPI == EPI_SWIGLU) {
    // fused matrix interleaves gate (even row-blocks) and up (odd): h = silu(gate) * up
    if (row_ok) {
      const int n = (nb >> 1) * 16 + g * 4;
      packed_store4(xpo, m, n, silu_dev(s[0] * rinv) * (u[0] * rinv), silu_dev(s[1] * rinv) * (u[1] * rinv),
                    silu_dev(s[2] * rinv) * (u[2] * rinv), silu_dev(s[3] * rinv) * (u[3] * rinv), kts);
    }
  } else if (EPI == EPI_QKV) {
    // Row-blocks [0, seg0) = q, [seg0, seg1) = k (both with the rotary row order of
    // retile_kernel), [seg1, ..) = v.  q: rotate, store float in natural column order.
    // k: rotate, round to bf16, append to the tiled K cache.  v: round, append.
    int si, nbs;
    epi_segment(a, nb, si, nbs);
    const int hd = a.hd, bph = hd >> 4, head = nbs / bph, j = nbs % bph;
    const int slot = a.pos0 + (row_ok ? row : 0);
    float4 o = make_float4(s[0] * rinv, s[1] * rinv, s[2] * rinv, s[3] * rinv);
    if (si < 2) {
      const int i0 = 8 * j + 4 * (g & 1);   // rotary index of the pair, first-half coordinates
      const float4 cs01 = pre ? pre->a : *reinterpret_cast<const float4 *>(a.rope_tab + (size_t)slot * (hd >> 1) + i0);
      const float4 cs23 = pre ? pre->b : *reinterpret_cast<const float4 *>(a.rope_tab + (size_t)slot * (hd >> 1) + i0 + 2);
      const float sgn = g < 2 ? -1.f : 1.f;   // first half: a*c - b*s; second half: b*c + a*s
      const float p0 = __shfl_xor(o.x, 32, 64), p1 = __shfl_xor(o.y, 32, 64);
      const float p2 = __shfl_xor(o.z, 32, 64), p3 = __shfl_xor(o.w, 32, 64);
      o.x = o.x * cs01.x + sgn * p0 * cs01.y;
      o.y = o.y * cs01.z + sgn * p1 * cs01.w;
      o.z = o.z * cs23.x + sgn * p2 * cs23.y;
      o.w = o.w * cs23.z + sgn * p3 * cs23.w;
      const int dcol = (g < 2 ? 0 : hd >> 1) + i0;   // natural head-dim index of o.x
      if (row_ok) {
        if (si == 0) {
          *reinterpret_cast<float4 *>(a.seg[0].Y + (size_t)row * a.seg[0].ldy + head * hd + dcol) = o;
        } else {
          // K tile layout: [kh][slot/16][d/32][lane = ((d%32)/8)*16 + slot%16][d%8]
          const size_t idx = ((((size_t)head * (a.n_ctx >> 4) + (slot >> 4)) * (hd >> 5) + (dcol >> 5)) * 64 +
                              ((dcol & 31) >> 3) * 16 + (slot & 15)) * 8 + (dcol & 7);
          u32x2 pk;
          pk[0] = (uint32_t)f2bf_rne(o.x) | ((uint32_t)f2bf_rne(o.y) << 16);
          pk[1] = (uint32_t)f2bf_rne(o.z) | ((uint32_t)f2bf_rne(o.w) << 16);
          *reinterpret_cast<u32x2 *>(a.Kc + idx) = pk;
        }
      }
    } else if (row_ok) {
      // V tile layout: [kh][slot/32][d/16][lane = ((slot%16)/4)*16 + d%16][e = slot%4 + 4*((slot%32)/16)]
      const int w16 = slot & 15, e = (w16 & 3) + 4 * ((slot & 31) >> 4);
      const size_t base = ((((size_t)head * (a.n_ctx >> 5) + (slot >> 5)) * bph + j) * 64 + (w16 >> 2) * 16 + g * 4) * 8 + e;
      a.Vc[base] = f2bf_rne(o.x);
      a.Vc[base + 8] = f2bf_rne(o.y);
      a.Vc[base + 16] = f2bf_rne(o.z);
      a.Vc[base + 24] = f2bf_rne(o.w);
    }
  } else {
    int si, nbs;
    epi_segment(a, nb, si, nbs);
    const int n = nbs * 16 + g * 4;   // this lane holds columns n..n+3 of its row
    float4 o = make_float4(s[0] * rinv, s[1] * rinv, s[2] * rinv, s[3] * rinv);
    float ssq = 0.f;
    if (row_ok) {
      float *yp = a.seg[si].Y + (size_t)row * a.seg[si].ldy + n;
      if (a.bias && si == 0) {
        const float4 b = (pre && EPI == EPI_STORE) ? pre->a : *reinterpret_cast<const float4 *>(a.bias + n);
        o.x += b.x; o.y += b.y; o.z += b.z; o.w += b.w;
      }
      if (EPI == EPI_RESID) {
        const float4 old = pre ? pre->a : *reinterpret_cast<const float4 *>(yp);
        o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
      }
      if (EPI == EPI_RESID || a.seg[si].Y) *reinterpret_cast<float4 *>(yp) = o;
      if (EPI == EPI_STORE && a.amax_val) {
        // argmax partial of this row-block: columns ascend with (g, component), ties keep the lowest
        float bv = o.x; int bi = n;
        if (o.y > bv) { bv = o.y; bi = n + 1; }
        if (o.z > bv) { bv = o.z; bi = n + 2; }
        if (o.w > bv) { bv = o.w; bi = n + 3; }
        ssq = bv;               // reuse the two registers for the cross-lane step below
        nbs = bi;
      }
      if (a.Xp_out) {
        ssq = o.x * o.x + o.y * o.y + o.z * o.z + o.w * o.w;
        float4 gn = make_float4(1.f, 1.f, 1.f, 1.f);
        if (a.gain_out) gn = pre ? pre->b : *reinterpret_cast<const float4 *>(a.gain_out + n);
        packed_store4(xpo, m, n, o.x * gn.x, o.y * gn.y, o.z * gn.z, o.w * gn.w, kts);
      }
    }
    if (EPI == EPI_STORE && a.amax_val) {
      float bv = row_ok ? ssq : -INFINITY;
      int bi = row_ok ? nbs : 0x7fffffff;
#pragma unroll
      for (int o2 = 16; o2 < 64; o2 <<= 1) {
        const float ov = __shfl_xor(bv, o2, 64);
        const int oi = __shfl_xor(bi, o2, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      // row-major by activation row ([16][NBtot]) so that the finishing kernel reads a row's partials contiguously
      if (g == 0) { a.amax_val[(size_t)m * a.NBtot + nb] = bv; a.amax_idx[(size_t)m * a.NBtot + nb] = bi; }
      if (a.lse_sum) {   // softmax statistics of the row-block (log-probability of a draft token, DDD rule)
        float e = 0.f;
        if (row_ok)
          e = (expf((o.x - bv) * a.lse_inv_t) + expf((o.y - bv) * a.lse_inv_t)) +
              (expf((o.z - bv) * a.lse_inv_t) + expf((o.w - bv) * a.lse_inv_t));
        e += __shfl_xor(e, 16, 64);
        e += __shfl_xor(e, 32, 64);
        if (g == 0) a.lse_sum[(size_t)m * a.NBtot + nb] = e;
      }
    } else if (a.ssq_out) {   // partial sum of x^2 over this row-block's 16 columns
      ssq += __shfl_xor(ssq, 16, 64);
      ssq += __shfl_xor(ssq, 32, 64);
      if (g == 0) a.ssq_out[((size_t)rb * a.NBtot + nb) * 16 + m] = ssq;
    }
  }
}

}  // namespace ae
