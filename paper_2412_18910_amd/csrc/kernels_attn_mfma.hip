// Variable-length causal attention over the bf16 KV cache on the gfx950 matrix cores.
//
// One workgroup = one KV head x one chunk of 4 * KPW keys fixed by absolute slot; its 4 waves
// take KPW = 64 keys each.  (32 keys per wave, twice the workgroups, measured per layer at the 7B
// shape 8.2 against 7.7 us at 1024 cached tokens and 11.1 against 11.6 us at 2100, but it lost
// 80-120 us per verify forward at the 13B / 4096-token and 8B-GQA / 8192-token shapes: every
// workgroup repeats the query staging and the combine.)  About 5 us of the kernel are its chain
// of latencies, launch -> operand fetch -> combine -> store.  All
// query rows that share the KV head (rows x group size, <= 64) are processed in tiles of 16.
// A wave issues its whole K and V working set as 1 KB coalesced loads up front, everything
// else hides behind it.
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

// KPW = keys per wave (32 or 64); a workgroup covers kMfmaAttnChunk = 4 * KPW keys.
template <int HD, int KPW, bool GATED>
__global__ __launch_bounds__(256) void attn_mfma_kernel(const float *q, int rows, int pos0, int H, int Hkv, int n_ctx,
                                                        const u32x4 *Kc, const u32x4 *Vc, float *part,
                                                        float scale_log2e, const int32_t *gate) {
  constexpr int DT = HD / 32, VT = HD / 16, KT = KPW / 16, VB = KPW / 32;
  extern __shared__ u32x4 smem[];
  if constexpr (GATED) AE_GATE(gate);
  const int kh = blockIdx.x, chunk = blockIdx.y, n_chunks = gridDim.y;
  const int G = H / Hkv, R = rows * G, MT = (R + 15) / 16;
  u32x4 *Qs = smem;                                           // [MT][DT][2][64]
  float *red = reinterpret_cast<float *>(smem + MT * DT * 128); // [4][16][HD]
  float *wm = red + 4 * 16 * HD;                              // [4][16]
  float *wl = wm + 64;                                        // [4][16]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, g = lane >> 4, m = lane & 15;
  const int kbase = chunk * (4 * KPW) + w * KPW;
  const bool active = kbase < pos0 + rows;   // does this wave own any visible key?

  // the wave's whole K / V working set, issued before anything else
  u32x4 kreg[KT][DT], vreg[VB][VT];
  if (active) {
    const u32x4 *kp = Kc + (((size_t)kh * (n_ctx / 16) + (kbase >> 4)) * DT) * 64 + lane;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) kreg[kt][dt] = kp[(kt * DT + dt) * 64];
    const u32x4 *vp = Vc + (((size_t)kh * (n_ctx / 32) + (kbase >> 5)) * VT) * 64 + lane;
#pragma unroll
    for (int vb = 0; vb < VB; ++vb)
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
      f32x4 S[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) S[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const u32x4 qh = Qs[((mt * DT + dt) * 2 + 0) * 64 + lane], ql = Qs[((mt * DT + dt) * 2 + 1) * 64 + lane];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          S[kt] = mfma_bf16(kreg[kt][dt], qh, S[kt]);
          S[kt] = mfma_bf16(kreg[kt][dt], ql, S[kt]);
        }
      }
      // causal mask: row (query row = row / G) sees slots <= pos0 + row / G
      const int limit = row < R ? pos0 + row / G : -1;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
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
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            S[kt][r] = __builtin_amdgcn_exp2f(S[kt][r] - mx);
            lsum += S[kt][r];
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) S[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      lsum += __shfl_xor(lsum, 16, 64);
      lsum += __shfl_xor(lsum, 32, 64);
      // P^T as B operand: k-slot e of lane group g = key 16*(e/4) + 4g + e%4 of a 32-key block
#pragma unroll
      for (int vb = 0; vb < VB; ++vb) {
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
// lanes, so the partials of many chunks are in flight at once and every value is fetched in a
// single round trip.  Chunk lane cl folds chunks cl, cl+CL, ... in ascending order with a
// running maximum (rescaling its sums when the maximum grows) and the lanes are then combined
// in ascending order against the overall maximum: a fixed order that does not depend on the
// number of rows.  The result is written in packed form as the input of the output
// projection (k index = h*HD + d).
template <int HD, bool GATED>
__global__ __launch_bounds__(256) void attn_merge_log2_kernel(const float *part, int rows, int H, int Hkv, int n_chunks,
                                                              u32x4 *Xp_out, const int32_t *gate) {
  constexpr int DQ = HD / 4, CL = 256 / DQ;
  __shared__ float4 nums[CL][DQ];
  __shared__ float dens[CL], maxs[CL];
  if constexpr (GATED) AE_GATE(gate);
  const int mrow = blockIdx.x / H, h = blockIdx.x % H, dq = threadIdx.x % DQ, cl = threadIdx.x / DQ;
  const int G = H / Hkv, kh = h / G, r = mrow * G + (h % G), R = rows * G;
  const float *base = part + ((size_t)kh * n_chunks * R + r) * (HD + 2);
  const size_t cstride = (size_t)R * (HD + 2);
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f, mx = -INFINITY;
#pragma unroll 2
  for (int c = cl; c < n_chunks; c += CL) {
    const float *p = base + c * cstride;
    const float2 a = *reinterpret_cast<const float2 *>(p + dq * 4), b = *reinterpret_cast<const float2 *>(p + dq * 4 + 2);
    const float2 ml = *reinterpret_cast<const float2 *>(p + HD);   // (chunk maximum, chunk sum)
    if (ml.x > -INFINITY) {
      const float mn = fmaxf(mx, ml.x);
      const float so = __builtin_amdgcn_exp2f(mx - mn), sn = __builtin_amdgcn_exp2f(ml.x - mn);   // exp2(-inf) = 0 the first time
      num.x = fmaf(sn, a.x, num.x * so); num.y = fmaf(sn, a.y, num.y * so);
      num.z = fmaf(sn, b.x, num.z * so); num.w = fmaf(sn, b.y, num.w * so);
      den = fmaf(sn, ml.y, den * so);
      mx = mn;
    }
  }
  nums[cl][dq] = num;
  if (dq == 0) { dens[cl] = den; maxs[cl] = mx; }
  __syncthreads();
  if (cl == 0) {
    float mall = maxs[0];
#pragma unroll
    for (int i = 1; i < CL; ++i) mall = fmaxf(mall, maxs[i]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float dall = 0.f;
#pragma unroll
    for (int i = 0; i < CL; ++i) {
      const float mi = maxs[i];
      if (mi > -INFINITY) {
        const float wgt = __builtin_amdgcn_exp2f(mi - mall);
        const float4 o = nums[i][dq];
        acc.x = fmaf(wgt, o.x, acc.x); acc.y = fmaf(wgt, o.y, acc.y);
        acc.z = fmaf(wgt, o.z, acc.z); acc.w = fmaf(wgt, o.w, acc.w);
        dall = fmaf(wgt, dens[i], dall);
      }
    }
    packed_store4(Xp_out, mrow, h * HD + dq * 4, acc.x / dall, acc.y / dall, acc.z / dall, acc.w / dall);
  }
}

size_t attn_mfma_smem_bytes(int MT, int HD) {
  return (size_t)MT * (HD / 32) * 128 * 16 + (size_t)4 * 16 * HD * 4 + 128 * 4;
}

// The widest block (4 query tiles: 16 rows x group size 4) needs more dynamic LDS than the
// default limit; raised once per context set-up instead of before every launch.
void attention_mfma_setup() {
  const int sm128 = (int)attn_mfma_smem_bytes(4, 128), sm64 = (int)attn_mfma_smem_bytes(4, 64);
  constexpr int KPW = kMfmaKeysPerWave;
  const auto raise = [](const void *f, int bytes) { (void)hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); };
  raise((const void *)attn_mfma_kernel<128, KPW, false>, sm128);
  raise((const void *)attn_mfma_kernel<128, KPW, true>, sm128);
  raise((const void *)attn_mfma_kernel<64, KPW, false>, sm64);
  raise((const void *)attn_mfma_kernel<64, KPW, true>, sm64);
}

template <int HD, bool GATED>
static void launch_attention_cfg(const float *q, int rows, int pos0, const ae_config &c, const u32x4 *Kc, const u32x4 *Vc,
                                 size_t sm, float *part, void *Xp_out, hipStream_t s, const int32_t *gate) {
  const int n_chunks = (pos0 + rows + kMfmaAttnChunk - 1) / kMfmaAttnChunk;
  const dim3 grid(c.n_kv_heads, n_chunks);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
  attn_mfma_kernel<HD, kMfmaKeysPerWave, GATED><<<grid, 256, sm, s>>>(q, rows, pos0, c.n_heads, c.n_kv_heads, kv_capacity(c),
                                                                      Kc, Vc, part, scale_log2e, gate);
  attn_merge_log2_kernel<HD, GATED><<<rows * c.n_heads, 256, 0, s>>>(part, rows, c.n_heads, c.n_kv_heads, n_chunks,
                                                                     (u32x4 *)Xp_out, gate);
}

void launch_attention_mfma(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                           float *part, void *Xp_out, hipStream_t s, const int32_t *gate) {
  const int G = c.n_heads / c.n_kv_heads, R = rows * G, MT = (R + 15) / 16;
  const size_t sm = attn_mfma_smem_bytes(MT, c.head_dim);
  const u32x4 *Kc = (const u32x4 *)kv_layer, *Vc = (const u32x4 *)((const char *)kv_layer + v_off);
  if (c.head_dim == 128) {
    if (gate) launch_attention_cfg<128, true>(q, rows, pos0, c, Kc, Vc, sm, part, Xp_out, s, gate);
    else launch_attention_cfg<128, false>(q, rows, pos0, c, Kc, Vc, sm, part, Xp_out, s, gate);
  } else {
    if (gate) launch_attention_cfg<64, true>(q, rows, pos0, c, Kc, Vc, sm, part, Xp_out, s, gate);
    else launch_attention_cfg<64, false>(q, rows, pos0, c, Kc, Vc, sm, part, Xp_out, s, gate);
  }
}

}  // namespace ae
