// KV cache layout, RoPE + append, and variable-length causal attention (split-KV).
//
// Cache of one layer (element type bf16 bits or float):
//   K: [n_kv_heads][head_dim/8][n_ctx_max][8]   -- "d-group major": for a fixed group of 8
//      head-dim elements, consecutive slots are contiguous, so 64 lanes that each own one
//      key load one contiguous 1 KB (bf16) line set per instruction;
//   V: [n_kv_heads][n_ctx_max][head_dim]        -- row-major: lanes own head-dim elements.
// A verify block first appends its K/V rows at slots pos0.., then every row attends the
// cache causally (row i sees slots 0..pos0+i).  Split-KV chunks are fixed by absolute
// slot (kAttnChunk keys each), masked keys contribute exact zeros, and all reductions
// have a fixed shape, so a row's result does not depend on how many rows share the block.
#include "ae_internal.h"

namespace ae {

using bf16_t = uint16_t;

__device__ __forceinline__ float bf2f_(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
// round-to-nearest-even float -> bf16 bits
__device__ __forceinline__ bf16_t f2bf_(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7f800000u) == 0x7f800000u) return (bf16_t)(u >> 16);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float cvt_in(T v);
template <> __device__ __forceinline__ float cvt_in<float>(float v) { return v; }
template <> __device__ __forceinline__ float cvt_in<bf16_t>(bf16_t v) { return bf2f_(v); }
template <typename T> __device__ __forceinline__ T cvt_out(float v);
template <> __device__ __forceinline__ float cvt_out<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t cvt_out<bf16_t>(float v) { return f2bf_(v); }

static size_t esize(const ae_config &c) { return c.dtype == AE_BF16 ? 2 : 4; }
int kv_capacity(const ae_config &c) { return (c.n_ctx_max + kAttnChunk - 1) / kAttnChunk * kAttnChunk; }
size_t kv_v_offset_bytes(const ae_config &c) {
  return (size_t)c.n_kv_heads * c.head_dim * kv_capacity(c) * esize(c);
}
size_t kv_layer_bytes(const ae_config &c) { return 2 * kv_v_offset_bytes(c); }

// Element index of K[kh][slot][d] / V[kh][slot][d] in the cache of one layer.  n_ctx is
// the capacity (a multiple of kAttnChunk).  `tiled` selects the MFMA operand layout
// of kernels_attn_mfma.hip, else the layout described at the top of this file.
template <typename T>
__device__ __forceinline__ size_t k_index(int kh, int d, int slot, int hd, int n_ctx, bool tiled) {
  if (tiled)  // [kh][slot/16][d/32][lane = ((d%32)/8)*16 + slot%16][d%8]
    return ((((size_t)kh * (n_ctx / 16) + (slot >> 4)) * (hd / 32) + (d >> 5)) * 64 + ((d & 31) >> 3) * 16 + (slot & 15)) * 8 + (d & 7);
  return (((size_t)kh * (hd / 8) + (d >> 3)) * n_ctx + slot) * 8 + (d & 7);
}
__device__ __forceinline__ size_t v_index(int kh, int d, int slot, int hd, int n_ctx, bool tiled) {
  if (tiled) {  // [kh][slot/32][d/16][lane = ((slot%16)/4)*16 + d%16][e = slot%4 + 4*((slot%32)/16)]
    const int w16 = slot & 15, half = (slot & 31) >> 4;
    return ((((size_t)kh * (n_ctx / 32) + (slot >> 5)) * (hd / 16) + (d >> 4)) * 64 + (w16 >> 2) * 16 + (d & 15)) * 8 + (w16 & 3) + 4 * half;
  }
  return ((size_t)kh * n_ctx + slot) * hd + d;
}

// ------------------------------------------------------------------ RoPE + append
// grid (rows, H + 2*Hkv), block hd/2.  Rotate-half pairing (i, i + hd/2).
template <typename T>
__global__ void rope_append_kernel(float *q, const float *k, const float *v, int pos0, int H, int Hkv, int hd,
                                   int n_ctx, bool tiled, const float2 *tab, T *Kc, T *Vc, const int32_t *gate) {
  AE_GATE(gate);
  const int r = blockIdx.x, hs = blockIdx.y, i = threadIdx.x, half = hd / 2;
  const int slot = pos0 + r;
  const float2 cs = tab[(size_t)slot * half + i];
  if (hs < H) {
    float *p = q + ((size_t)r * H + hs) * hd;
    const float a = p[i], b = p[i + half];
    p[i] = a * cs.x - b * cs.y;
    p[i + half] = b * cs.x + a * cs.y;
  } else if (hs < H + Hkv) {
    const int kh = hs - H;
    const float *p = k + ((size_t)r * Hkv + kh) * hd;
    const float a = p[i], b = p[i + half];
    Kc[k_index<T>(kh, i, slot, hd, n_ctx, tiled)] = cvt_out<T>(a * cs.x - b * cs.y);
    Kc[k_index<T>(kh, i + half, slot, hd, n_ctx, tiled)] = cvt_out<T>(b * cs.x + a * cs.y);
  } else {
    const int kh = hs - H - Hkv;
    const float *p = v + ((size_t)r * Hkv + kh) * hd;
    Vc[v_index(kh, i, slot, hd, n_ctx, tiled)] = cvt_out<T>(p[i]);
    Vc[v_index(kh, i + half, slot, hd, n_ctx, tiled)] = cvt_out<T>(p[i + half]);
  }
}

void launch_rope_append(float *q, const float *k, const float *v, int rows, int pos0, const ae_config &c,
                        const float2 *rope_tab, void *kv_layer, size_t v_off, bool tiled, hipStream_t s,
                        const int32_t *gate) {
  const dim3 grid(rows, c.n_heads + 2 * c.n_kv_heads);
  void *vc = (char *)kv_layer + v_off;
  if (c.dtype == AE_BF16)
    rope_append_kernel<bf16_t><<<grid, c.head_dim / 2, 0, s>>>(q, k, v, pos0, c.n_heads, c.n_kv_heads, c.head_dim,
                                                               kv_capacity(c), tiled, rope_tab, (bf16_t *)kv_layer, (bf16_t *)vc, gate);
  else
    rope_append_kernel<float><<<grid, c.head_dim / 2, 0, s>>>(q, k, v, pos0, c.n_heads, c.n_kv_heads, c.head_dim,
                                                              kv_capacity(c), tiled, rope_tab, (float *)kv_layer, (float *)vc, gate);
}

// ------------------------------------------------------------------ attention, split-KV partials
// grid (Hkv, n_chunks), block 256.  Rows of the workgroup: r = m*G + g  (query row m,
// query head kh*G + g), R = rows*G <= 64.  part[(kh*n_chunks + chunk)][r][HD + 2] holds the
// unnormalised output, the chunk max and the chunk sum of exponentials.
template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t *p) { raw = *reinterpret_cast<const uint4 *>(p); }
  __device__ __forceinline__ void get(float *w) const {
    w[0] = __uint_as_float(raw.x << 16); w[1] = __uint_as_float(raw.x & 0xffff0000u);
    w[2] = __uint_as_float(raw.y << 16); w[3] = __uint_as_float(raw.y & 0xffff0000u);
    w[4] = __uint_as_float(raw.z << 16); w[5] = __uint_as_float(raw.z & 0xffff0000u);
    w[6] = __uint_as_float(raw.w << 16); w[7] = __uint_as_float(raw.w & 0xffff0000u);
  }
};
template <> struct Vec8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float *p) {
    a = *reinterpret_cast<const float4 *>(p);
    b = *reinterpret_cast<const float4 *>(p + 4);
  }
  __device__ __forceinline__ void get(float *w) const {
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
  }
};

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(const float *q, int rows, int pos0, int H, int Hkv,
                                                           int n_ctx, const T *Kc, const T *Vc, float *part,
                                                           float scale, const int32_t *gate) {
  extern __shared__ float smem[];
  AE_GATE(gate);
  const int kh = blockIdx.x, chunk = blockIdx.y, n_chunks = gridDim.y;
  const int G = H / Hkv, R = rows * G;
  const int c0 = chunk * kAttnChunk;
  float *qs = smem;                 // [R][HD]
  float *S = smem + (size_t)R * HD; // [R][kAttnChunk]
  float *rmax = S + (size_t)R * kAttnChunk;  // [R]
  float *rsum = rmax + R;                    // [R]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;

  for (int i = t; i < R * HD; i += 256) {
    const int r = i / HD, d = i % HD, m = r / G, g = r % G;
    qs[i] = q[((size_t)m * H + kh * G + g) * HD + d];
  }
  __syncthreads();

  // scores: thread t owns key c0 + t
  const int key = c0 + t;
  const bool key_in = key < n_ctx;
  for (int r0 = 0; r0 < R; r0 += 16) {
    float sc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) sc[i] = 0.f;
    if (key_in) {
#pragma unroll 4
      for (int c = 0; c < HD / 8; ++c) {
        Vec8<T> kv8;
        kv8.load(Kc + (((size_t)kh * (HD / 8) + c) * n_ctx + key) * 8);
        float kf[8];
        kv8.get(kf);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          if (r0 + i < R) {
            const float4 qa = *reinterpret_cast<const float4 *>(qs + (size_t)(r0 + i) * HD + c * 8);
            const float4 qb = *reinterpret_cast<const float4 *>(qs + (size_t)(r0 + i) * HD + c * 8 + 4);
            float a = sc[i];
            a = fmaf(qa.x, kf[0], a); a = fmaf(qa.y, kf[1], a); a = fmaf(qa.z, kf[2], a); a = fmaf(qa.w, kf[3], a);
            a = fmaf(qb.x, kf[4], a); a = fmaf(qb.y, kf[5], a); a = fmaf(qb.z, kf[6], a); a = fmaf(qb.w, kf[7], a);
            sc[i] = a;
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (r0 + i < R) {
        const int m = (r0 + i) / G;
        S[(size_t)(r0 + i) * kAttnChunk + t] = (key <= pos0 + m) ? sc[i] * scale : -INFINITY;
      }
    }
  }
  __syncthreads();

  // per-row max and exponentials: wave w owns rows w, w+4, ...
  for (int r = wave; r < R; r += 4) {
    float *row = S + (size_t)r * kAttnChunk;
    float v0 = row[lane], v1 = row[lane + 64], v2 = row[lane + 128], v3 = row[lane + 192];
    float mx = fmaxf(fmaxf(v0, v1), fmaxf(v2, v3));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
    if (mx > -INFINITY) {
      p0 = expf(v0 - mx); p1 = expf(v1 - mx); p2 = expf(v2 - mx); p3 = expf(v3 - mx);
    }
    row[lane] = p0; row[lane + 64] = p1; row[lane + 128] = p2; row[lane + 192] = p3;
    float sum = (p0 + p1) + (p2 + p3);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (lane == 0) { rmax[r] = mx; rsum[r] = sum; }
  }
  __syncthreads();

  // P.V: wave w owns rows w, w+4, ...; lanes own EPL consecutive head-dim elements
  constexpr int EPL = HD / 64;
  const int n_keys = min(kAttnChunk, pos0 + rows - c0);  // keys past the block are masked anyway
  float *pbase = part + ((size_t)kh * n_chunks + chunk) * (size_t)R * (HD + 2);
  for (int rt = wave; rt < R; rt += 32) {  // tiles of 8 rows: rt, rt+4, ..., rt+28
    float acc[8][EPL];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[i][e] = 0.f;
    for (int j = 0; j < n_keys; ++j) {
      float vf[EPL];
      const T *vp = Vc + ((size_t)kh * n_ctx + c0 + j) * HD + lane * EPL;
#pragma unroll
      for (int e = 0; e < EPL; ++e) vf[e] = cvt_in<T>(vp[e]);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = rt + 4 * i;
        if (r < R) {
          const float p = S[(size_t)r * kAttnChunk + j];
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[i][e] = fmaf(p, vf[e], acc[i][e]);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rt + 4 * i;
      if (r < R) {
        float *o = pbase + (size_t)r * (HD + 2);
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[lane * EPL + e] = acc[i][e];
        if (lane == 0) { o[HD] = rmax[r]; o[HD + 1] = rsum[r]; }
      }
    }
  }
}

// merge of the chunk partials, grid (rows*H), block HD; fixed chunk order
template <int HD>
__global__ void attn_merge_kernel(const float *part, int rows, int H, int Hkv, int n_chunks, float *out,
                                  const int32_t *gate) {
  AE_GATE(gate);
  const int m = blockIdx.x / H, h = blockIdx.x % H, d = threadIdx.x;
  const int G = H / Hkv, kh = h / G, r = m * G + (h % G), R = rows * G;
  float mx = -INFINITY;
  for (int c = 0; c < n_chunks; ++c)
    mx = fmaxf(mx, part[(((size_t)kh * n_chunks + c) * R + r) * (HD + 2) + HD]);
  float num = 0.f, den = 0.f;
  for (int c = 0; c < n_chunks; ++c) {
    const float *p = part + (((size_t)kh * n_chunks + c) * R + r) * (HD + 2);
    const float mc = p[HD];
    if (mc > -INFINITY) {
      const float w = expf(mc - mx);
      num = fmaf(w, p[d], num);
      den = fmaf(w, p[HD + 1], den);
    }
  }
  out[((size_t)m * H + h) * HD + d] = num / den;
}

size_t attn_part_floats(const ae_config &c) {
  const int max_chunks = kv_capacity(c) / (kMfmaAttnChunk < kAttnChunk ? kMfmaAttnChunk : kAttnChunk);
  return (size_t)c.n_heads * max_chunks * kMaxRows * (c.head_dim + 2);
}

void launch_attention(const float *q, int rows, int pos0, const ae_config &c, const void *kv_layer, size_t v_off,
                      float *part, float *out, hipStream_t s, const int32_t *gate) {
  const int n_chunks = (pos0 + rows + kAttnChunk - 1) / kAttnChunk;
  const int G = c.n_heads / c.n_kv_heads, R = rows * G;
  const size_t sm = ((size_t)R * c.head_dim + (size_t)R * kAttnChunk + 2 * R) * sizeof(float);
  const dim3 grid(c.n_kv_heads, n_chunks);
  const float scale = 1.0f / sqrtf((float)c.head_dim);
  const void *vc = (const char *)kv_layer + v_off;
#define AE_ATTN(T, HD)                                                                                         \
  if (sm > 48 * 1024)                                                                                          \
    (void)hipFuncSetAttribute((const void *)attn_partial_kernel<T, HD>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                              (int)sm);                                                                        \
  attn_partial_kernel<T, HD><<<grid, 256, sm, s>>>(q, rows, pos0, c.n_heads, c.n_kv_heads, kv_capacity(c),      \
                                                   (const T *)kv_layer, (const T *)vc, part, scale, gate);      \
  attn_merge_kernel<HD><<<rows * c.n_heads, HD, 0, s>>>(part, rows, c.n_heads, c.n_kv_heads, n_chunks, out, gate);
  if (c.dtype == AE_BF16) {
    if (c.head_dim == 128) { AE_ATTN(bf16_t, 128) } else { AE_ATTN(bf16_t, 64) }
  } else {
    if (c.head_dim == 128) { AE_ATTN(float, 128) } else { AE_ATTN(float, 64) }
  }
#undef AE_ATTN
}

// ------------------------------------------------------------------ import / export (tests, set-up)
template <typename T>
__global__ void kv_import_kernel(T *Kc, T *Vc, const float *k, const float *v, int n, int Hkv, int hd, int n_ctx,
                                 bool tiled) {
  const size_t total = (size_t)n * Hkv * hd;
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int d = i % hd, kh = (i / hd) % Hkv, slot = i / ((size_t)hd * Hkv);
    Kc[k_index<T>(kh, d, slot, hd, n_ctx, tiled)] = cvt_out<T>(k[i]);
    Vc[v_index(kh, d, slot, hd, n_ctx, tiled)] = cvt_out<T>(v[i]);
  }
}

void launch_kv_import(void *kv_layer, size_t v_off, const ae_config &c, const float *k_dev, const float *v_dev, int n,
                      bool tiled, hipStream_t s) {
  void *vc = (char *)kv_layer + v_off;
  if (c.dtype == AE_BF16)
    kv_import_kernel<bf16_t><<<1024, 256, 0, s>>>((bf16_t *)kv_layer, (bf16_t *)vc, k_dev, v_dev, n, c.n_kv_heads,
                                                  c.head_dim, kv_capacity(c), tiled);
  else
    kv_import_kernel<float><<<1024, 256, 0, s>>>((float *)kv_layer, (float *)vc, k_dev, v_dev, n, c.n_kv_heads,
                                                 c.head_dim, kv_capacity(c), tiled);
}

template <typename T>
__global__ void kv_export_kernel(const T *Kc, const T *Vc, int which, int slot, int Hkv, int hd, int n_ctx, bool tiled,
                                 float *out) {
  for (int i = threadIdx.x; i < Hkv * hd; i += blockDim.x) {
    const int d = i % hd, kh = i / hd;
    out[i] = which ? cvt_in<T>(Vc[v_index(kh, d, slot, hd, n_ctx, tiled)]) : cvt_in<T>(Kc[k_index<T>(kh, d, slot, hd, n_ctx, tiled)]);
  }
}

void launch_kv_export(const void *kv_layer, size_t v_off, const ae_config &c, int which, int slot, float *out_dev,
                      bool tiled, hipStream_t s) {
  const void *vc = (const char *)kv_layer + v_off;
  if (c.dtype == AE_BF16)
    kv_export_kernel<bf16_t><<<1, 256, 0, s>>>((const bf16_t *)kv_layer, (const bf16_t *)vc, which, slot, c.n_kv_heads,
                                               c.head_dim, kv_capacity(c), tiled, out_dev);
  else
    kv_export_kernel<float><<<1, 256, 0, s>>>((const float *)kv_layer, (const float *)vc, which, slot, c.n_kv_heads,
                                              c.head_dim, kv_capacity(c), tiled, out_dev);
}

}  // namespace ae
