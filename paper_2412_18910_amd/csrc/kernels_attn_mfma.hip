// Variable-length causal attention over the bf16 KV cache on the gfx950 matrix cores.
//
// One workgroup = one KV head x one chunk of kAttnChunk (256) keys fixed by absolute slot;
// its 4 waves take 64 keys each.  All query rows that share the KV head (rows x group
// size, <= 64) are processed in tiles of 16.  HBM-bound: a wave issues its whole K and V
// working set (32 KB) as 1 KB coalesced loads up front, everything else hides behind it.
//
// Cache layouts (bf16, one 1 KB tile = one wave-wide 128-bit load = one MFMA operand):
//   K tile (16 keys x 32 d):   [kh][slot/16][d/32][lane = ((d%32)/8)*16 + slot%16][d%8]
//       -> A operand of S^T = K . Q^T  (rows = keys, contraction over d)
//   V tile (16 d x 32 keys):   [kh][slot/32][d/16][lane = ((slot%16)/4)*16 + d%16][e],
//       e = slot%4 + 4*((slot%32)/16)
//       -> A operand of O^T = V^T . P^T (rows = d, contraction over keys), with the keys
//       of a tile permuted so that the P values a lane already holds after the S MFMAs
//       (keys 4g..4g+3 of two 16-key tiles) are exactly its B operand: no shuffles.
// Scores are kept in the log2 domain (q is pre-scaled by log2(e)/sqrt(hd)); q and P are
// split into bf16 hi + lo so the products carry ~16 significant bits.  Masked keys give
// exact zeros and every reduction has a fixed order, so a row's result does not depend on
// the number of rows in the block.
#include "ae_internal.h"
#include "packed.h"

namespace ae {

#define split2a split2

template <int HD>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const float *q, int rows, int pos0, int H, int Hkv, int n_ctx,
                                                        const u32x4 *Kc, const u32x4 *Vc, float *part,
                                                        float scale_log2e, const int32_t *gate) {
  constexpr int DT = HD / 32, VT = HD / 16;
  extern __shared__ u32x4 smem[];
  AE_GATE(gate);
  const int kh = blockIdx.x, chunk = blockIdx.y, n_chunks = gridDim.y;
  const int G = H / Hkv, R = rows * G, MT = (R + 15) / 16;
  u32x4 *Qs = smem;                                           // [MT][DT][2][64]
  float *red = reinterpret_cast<float *>(smem + MT * DT * 128); // [4][16][HD]
  float *wm = red + 4 * 16 * HD;                              // [4][16]
  float *wl = wm + 64;                                        // [4][16]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, m = lane & 15;
  const int kbase = chunk * kAttnChunk + w * 64;
  const bool active = kbase < pos0 + rows;   // does this wave own any visible key?

  // the wave's whole K / V working set, issued before anything else
  u32x4 kreg[4][DT], vreg[2][VT];
  if (active) {
    const u32x4 *kp = Kc + (((size_t)kh * (n_ctx / 16) + (kbase >> 4)) * DT) * 64 + lane;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) kreg[kt][dt] = kp[(kt * DT + dt) * 64];
    const u32x4 *vp = Vc + (((size_t)kh * (n_ctx / 32) + (kbase >> 5)) * VT) * 64 + lane;
#pragma unroll
    for (int vb = 0; vb < 2; ++vb)
#pragma unroll
      for (int dt = 0; dt < VT; ++dt) vreg[vb][dt] = vp[(vb * VT + dt) * 64];
  }

  // queries -> bf16 hi/lo B-operand tiles in LDS, pre-scaled into the log2 domain
  for (int idx = tid; idx < MT * DT * 64; idx += 256) {
    const int l = idx & 63, dt = (idx >> 6) % DT, mt = idx / (DT * 64);
    const int row = mt * 16 + (l & 15), gg = l >> 4;
    u32x4 hi = {0, 0, 0, 0}, lo = {0, 0, 0, 0};
    if (row < R) {
      const float *src = q + ((size_t)(row / G) * H + kh * G + row % G) * HD + dt * 32 + gg * 8;
      const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
      uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
      split2a(a.x * scale_log2e, a.y * scale_log2e, h0, l0);
      split2a(a.z * scale_log2e, a.w * scale_log2e, h1, l1);
      split2a(b.x * scale_log2e, b.y * scale_log2e, h2, l2);
      split2a(b.z * scale_log2e, b.w * scale_log2e, h3, l3);
      hi = u32x4{h0, h1, h2, h3};
      lo = u32x4{l0, l1, l2, l3};
    }
    Qs[((mt * DT + dt) * 2 + 0) * 64 + l] = hi;
    Qs[((mt * DT + dt) * 2 + 1) * 64 + l] = lo;
  }
  __syncthreads();

  for (int mt = 0; mt < MT; ++mt) {
    const int row = mt * 16 + m;
    float mx = -INFINITY, lsum = 0.f;
    f32x4 O[VT];
#pragma unroll
    for (int dt = 0; dt < VT; ++dt) O[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (active) {
      f32x4 S[4];
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) S[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const u32x4 qh = Qs[((mt * DT + dt) * 2 + 0) * 64 + lane], ql = Qs[((mt * DT + dt) * 2 + 1) * 64 + lane];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
          S[kt] = mfma_bf16(kreg[kt][dt], qh, S[kt]);
          S[kt] = mfma_bf16(kreg[kt][dt], ql, S[kt]);
        }
      }
      // causal mask: row (query row = row / G) sees slots <= pos0 + row / G
      const int limit = row < R ? pos0 + row / G : -1;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = kbase + kt * 16 + 4 * g + r;
          S[kt][r] = key <= limit ? S[kt][r] : -INFINITY;
          mx = fmaxf(mx, S[kt][r]);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (mx > -INFINITY) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            S[kt][r] = __builtin_amdgcn_exp2f(S[kt][r] - mx);
            lsum += S[kt][r];
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) S[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      lsum += __shfl_xor(lsum, 16, 64);
      lsum += __shfl_xor(lsum, 32, 64);
      // P^T as B operand: k-slot e of lane group g = key 16*(e/4) + 4g + e%4 of a 32-key block
#pragma unroll
      for (int vb = 0; vb < 2; ++vb) {
        uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
        split2a(S[2 * vb][0], S[2 * vb][1], h0, l0);
        split2a(S[2 * vb][2], S[2 * vb][3], h1, l1);
        split2a(S[2 * vb + 1][0], S[2 * vb + 1][1], h2, l2);
        split2a(S[2 * vb + 1][2], S[2 * vb + 1][3], h3, l3);
        const u32x4 ph = {h0, h1, h2, h3}, pl = {l0, l1, l2, l3};
#pragma unroll
        for (int dt = 0; dt < VT; ++dt) {
          O[dt] = mfma_bf16(vreg[vb][dt], ph, O[dt]);
          O[dt] = mfma_bf16(vreg[vb][dt], pl, O[dt]);
        }
      }
    }
    // combine the four waves (fixed order) with the usual max-rescaling
#pragma unroll
    for (int dt = 0; dt < VT; ++dt)
      *reinterpret_cast<f32x4 *>(red + ((size_t)w * 16 + m) * HD + dt * 16 + 4 * g) = O[dt];
    if (g == 0) { wm[w * 16 + m] = mx; wl[w * 16 + m] = lsum; }
    __syncthreads();
    {
      const int m2 = tid >> 4, seg = tid & 15, row2 = mt * 16 + m2;
      if (row2 < R) {
        float ms = fmaxf(fmaxf(wm[m2], wm[16 + m2]), fmaxf(wm[32 + m2], wm[48 + m2]));
        float wgt[4], l = 0.f;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) {
          const float mw = wm[ww * 16 + m2];
          wgt[ww] = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - ms) : 0.f;
          l = fmaf(wgt[ww], wl[ww * 16 + m2], l);
        }
        float *dst = part + (((size_t)kh * n_chunks + chunk) * R + row2) * (HD + 2);
#pragma unroll
        for (int i = 0; i < HD / 16; ++i) {
          const int d = seg * (HD / 16) + i;
          float o = 0.f;
#pragma unroll
          for (int ww = 0; ww < 4; ++ww) o = fmaf(wgt[ww], red[((size_t)ww * 16 + m2) * HD + d], o);
          dst[d] = o;
        }
        if (seg == 0) { dst[HD] = ms; dst[HD + 1] = l; }
      }
    }
    __syncthreads();
  }
}

// Merge of the chunk partials (log2-domain maxima); one workgroup of 256 threads per (row,
// head): HD/4 threads across the head dimension (four elements each) times 1024/HD chunk
// lanes, so the partials of many chunks are in flight at once.  Chunk lane cl sums chunks cl,
// cl+CL, ... in ascending order and the lanes are combined in ascending order: a fixed order
// that does not depend on the number of rows.  The result is written in packed form as the
// input of the output projection (k index = h*HD + d).
template <int HD>
__global__ __launch_bounds__(256) void attn_merge_log2_kernel(const float *part, int rows, int H, int Hkv, int n_chunks,
                                                              u32x4 *Xp_out, const int32_t *gate) {
  constexpr int DQ = HD / 4, CL = 256 / DQ;
  __shared__ float ms[kMaxSplits];
  __shared__ float4 nums[CL][DQ];
  __shared__ float dens[CL];
  AE_GATE(gate);
  const int mrow = blockIdx.x / H, h = blockIdx.x % H, dq = threadIdx.x % DQ, cl = threadIdx.x / DQ;
  const int G = H / Hkv, kh = h / G, r = mrow * G + (h % G), R = rows * G;
  const float *base = part + ((size_t)kh * n_chunks * R + r) * (HD + 2);
  const size_t cstride = (size_t)R * (HD + 2);
  for (int c = threadIdx.x; c < n_chunks; c += 256) ms[c] = base[c * cstride + HD];
  __syncthreads();
  float mx = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) mx = fmaxf(mx, ms[c]);
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
#pragma unroll 2
  for (int c = cl; c < n_chunks; c += CL) {
    const float mc = ms[c];
    const float *p = base + c * cstride;
    const float2 a = *reinterpret_cast<const float2 *>(p + dq * 4), b = *reinterpret_cast<const float2 *>(p + dq * 4 + 2);
    const float lc = p[HD + 1];
    if (mc > -INFINITY) {
      const float wgt = __builtin_amdgcn_exp2f(mc - mx);
      num.x = fmaf(wgt, a.x, num.x); num.y = fmaf(wgt, a.y, num.y);
      num.z = fmaf(wgt, b.x, num.z); num.w = fmaf(wgt, b.y, num.w);
      den = fmaf(wgt, lc, den);
    }
  }
  nums[cl][dq] = num;
  if (dq == 0) dens[cl] = den;
  __syncthreads();
  if (cl == 0) {
#pragma unroll
    for (int i = 1; i < CL; ++i) {
      const float4 o = nums[i][dq];
      num.x += o.x; num.y += o.y; num.z += o.z; num.w += o.w;
      den += dens[i];
    }
    packed_store4(Xp_out, mrow, h * HD + dq * 4, num.x / den, num.y / den, num.z / den, num.w / den);
  }
}

void launch_attention_mfma(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                           float *part, void *Xp_out, hipStream_t s, const int32_t *gate) {
  const int n_chunks = (pos0 + rows + kAttnChunk - 1) / kAttnChunk;
  const int G = c.n_heads / c.n_kv_heads, R = rows * G, MT = (R + 15) / 16;
  const int HD = c.head_dim;
  const size_t sm = (size_t)MT * (HD / 32) * 128 * 16 + (size_t)4 * 16 * HD * 4 + 128 * 4;
  const dim3 grid(c.n_kv_heads, n_chunks);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
  const u32x4 *Kc = (const u32x4 *)kv_layer, *Vc = (const u32x4 *)((const char *)kv_layer + v_off);
  const int cap = kv_capacity(c);
  if (HD == 128) {
    if (sm > 48 * 1024)
      (void)hipFuncSetAttribute((const void *)attn_mfma_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    attn_mfma_kernel<128><<<grid, 256, sm, s>>>(q, rows, pos0, c.n_heads, c.n_kv_heads, cap, Kc, Vc, part, scale_log2e, gate);
    attn_merge_log2_kernel<128><<<rows * c.n_heads, 256, 0, s>>>(part, rows, c.n_heads, c.n_kv_heads, n_chunks, (u32x4 *)Xp_out, gate);
  } else {
    if (sm > 48 * 1024)
      (void)hipFuncSetAttribute((const void *)attn_mfma_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    attn_mfma_kernel<64><<<grid, 256, sm, s>>>(q, rows, pos0, c.n_heads, c.n_kv_heads, cap, Kc, Vc, part, scale_log2e, gate);
    attn_merge_log2_kernel<64><<<rows * c.n_heads, 256, 0, s>>>(part, rows, c.n_heads, c.n_kv_heads, n_chunks, (u32x4 *)Xp_out, gate);
  }
}

}  // namespace ae
