// Temperature > 0: draft sampling and the lossless rejection-sampling rule of speculative
// decoding (arxiv 2412.18910, Sec. 2.1):  draft token t is accepted with probability
// min(1, p(t)/p_hat(t)); the first rejection resamples from norm(max(0, p - p_hat)) over the
// whole vocabulary; with no rejection the bonus token comes from the target law of the row
// after the last draft token.  Every draw is an inverse CDF in token-id order driven by a
// caller-supplied uniform.  Softmax, ratio, residual and prefix sums are float64: in float32
// a prefix sum over ~128k tokens would let rounding noise decide a visible share of draws.
//
// The vocabulary is cut into segments of 1024 tokens handled by one workgroup each:
//   seg_stats_kernel   (max, sum exp((l - max)/T)) of every segment of every row involved;
//   a one-workgroup kernel combines them per row (fixed-shape trees), takes the accept
//   decisions and finds the segment that holds u * total;
//   seg_total_kernel   (rejection only) sums max(0, p - p_hat) per segment;
//   the final one-workgroup kernel scans the owning segment (one token per thread).
// All reductions have a fixed shape, so a draw does not depend on launch geometry.
#include "ae_internal.h"

namespace ae {

constexpr int kSeg = 1024;        // tokens per segment = threads of the one-workgroup kernels
constexpr int kSegThreads = 256;  // threads of the per-segment kernels (4 tokens each)

// ---- reductions of fixed shape: a butterfly inside every wave (all lanes end with the same
// value: each step adds the same two operands on both sides), then the N/64 wave results are
// combined in wave order by every thread.  sh needs N/64 entries. ----
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_max_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}

template <int N>
__device__ __forceinline__ double block_sum(double v, double *sh) {
  v = wave_sum_d(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = sh[0];
#pragma unroll
  for (int w = 1; w < N / 64; ++w) r += sh[w];
  __syncthreads();
  return r;
}

template <int N>
__device__ __forceinline__ double block_max(double v, double *sh) {
  v = wave_max_d(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  double r = sh[0];
#pragma unroll
  for (int w = 1; w < N / 64; ++w) r = fmax(r, sh[w]);
  __syncthreads();
  return r;
}

// Inclusive prefix over the values of the kSeg threads, left in out[0..kSeg) (LDS): a
// Kogge-Stone scan inside every wave, then the totals of the waves in front are added in wave
// order.  Fixed shape.  wsum needs kSeg/64 entries; ends with a barrier.
__device__ __forceinline__ void block_scan_inclusive(double v, double *out, double *wsum) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double up = __shfl_up(v, o, 64);
    if (lane >= o) v += up;
  }
  if (lane == 63) wsum[w] = v;
  __syncthreads();
  double off = 0.0;
  for (int i = 0; i < w; ++i) off += wsum[i];
  out[threadIdx.x] = off + v;
  __syncthreads();
}

// rows 0..n_target-1 are target rows, the rest draft rows
__device__ __forceinline__ const float *row_ptr(const float *tl, const float *dl, int V, int n_target, int row) {
  return row < n_target ? tl + (size_t)row * V : dl + (size_t)(row - n_target) * V;
}

// segstats[(row*S + seg)*2 + {0,1}] = (max, sum exp((l - max)/T)) of the segment; grid (S, rows)
__global__ __launch_bounds__(kSegThreads) void seg_stats_kernel(const float *tl, const float *dl, int V, int n_target,
                                                                double T, double *segstats, const int32_t *gate) {
  __shared__ double sh[kSegThreads];
  AE_GATE(gate);
  const int seg = blockIdx.x, row = blockIdx.y, S = gridDim.x;
  const float *x = row_ptr(tl, dl, V, n_target, row);
  const int lo = seg * kSeg;
  double v[kSeg / kSegThreads];
  double mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < kSeg / kSegThreads; ++i) {
    const int idx = lo + threadIdx.x + i * kSegThreads;
    v[i] = idx < V ? (double)x[idx] : -INFINITY;
    mx = fmax(mx, v[i]);
  }
  mx = block_max<kSegThreads>(mx, sh);
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < kSeg / kSegThreads; ++i) s += v[i] > -INFINITY ? exp((v[i] - mx) / T) : 0.0;
  s = block_sum<kSegThreads>(s, sh);
  if (threadIdx.x == 0) {
    segstats[((size_t)row * S + seg) * 2] = mx;
    segstats[((size_t)row * S + seg) * 2 + 1] = s;
  }
}

// (max, sum exp((l - max)/T)) of a whole row from its segment statistics, computed by one wave
// (lane l takes segments l, l + 64, ... in order, then a butterfly): every lane gets the result
__device__ void combine_row_wave(const double *segstats, int S, int row, double T, double &mx, double &sum) {
  const int lane = threadIdx.x & 63;
  const double *rs = segstats + (size_t)row * S * 2;
  double m = -INFINITY;
  for (int sg = lane; sg < S; sg += 64) m = fmax(m, rs[(size_t)sg * 2]);
  m = wave_max_d(m);
  double acc = 0.0;
  for (int sg = lane; sg < S; sg += 64) acc += rs[(size_t)sg * 2 + 1] * exp((rs[(size_t)sg * 2] - m) / T);
  mx = m;
  sum = wave_sum_d(acc);
}

// mode 0: q(x) = p(x);  mode 1: q(x) = max(0, p(x) - p_hat(x)).  p, p_hat normalised softmaxes.
__device__ __forceinline__ double qval(const float *trow, const float *drow, int x, int mode, double T, double mt, double st,
                                       double md, double sd) {
  const double p = exp(((double)trow[x] - mt) / T) / st;
  if (mode == 0) return p;
  const double ph = exp(((double)drow[x] - md) / T) / sd;
  return p - ph > 0.0 ? p - ph : 0.0;
}

// Inverse CDF, last step.  segv = total of q over segment threadIdx.x (0 beyond the S segments).
// Finds the smallest x with q(0)+..+q(x) > u * sum(q): an inclusive prefix over the segment
// totals names the owning segment, which is then scanned with one token per thread (same scan).  If rounding pushes the threshold past the total, the last token with
// q > 0 is returned.  *total_out receives sum(q).  All kSeg threads call; sh holds kSeg + 16 doubles.
__device__ int inverse_cdf_final(double segv, int S, const float *trow, const float *drow, int V, int mode, double T,
                                 double mt, double st, double md, double sd, double u, double *sh, double *total_out) {
  __shared__ int owner_s, lastseg_s, res_s, lastq_s;
  const int t = threadIdx.x;
  if (t == 0) { owner_s = 0x7fffffff; lastseg_s = 0; res_s = 0x7fffffff; lastq_s = -1; }
  double *a = sh, *wsum = sh + kSeg;
  block_scan_inclusive(segv, a, wsum);
  const double tot = a[S - 1];
  const double thr = u * tot;
  if (t < S && segv > 0.0) {
    atomicMax(&lastseg_s, t);
    if (a[t] > thr) atomicMin(&owner_s, t);
  }
  __syncthreads();
  int owner = owner_s;
  double before;
  if (owner == 0x7fffffff) { owner = lastseg_s; before = -1.0; }   // threshold beyond the total
  else before = owner > 0 ? a[owner - 1] : 0.0;
  __syncthreads();   // the prefix buffer is reused below
  const int x = owner * kSeg + t;
  const double q = x < V ? qval(trow, drow, x, mode, T, mt, st, md, sd) : 0.0;
  block_scan_inclusive(q, a, wsum);
  if (q > 0.0) atomicMax(&lastq_s, x);
  if (before >= 0.0 && q > 0.0 && before + a[t] > thr) atomicMin(&res_s, x);
  __syncthreads();
  if (total_out) *total_out = tot;
  int res = res_s;
  if (res == 0x7fffffff) res = lastq_s >= 0 ? lastq_s : owner * kSeg;   // rounding: last token with mass
  __syncthreads();
  return res;
}

// ------------------------------------------------------------------ draft sampling
// Draft token i ~ softmax(logits / T) by inverse CDF with st->u_draft[i]; result in st->argmax[0].
// Segment totals of p follow from the segment statistics, no second pass over the logits.
__global__ __launch_bounds__(kSeg) void sample_draft_final_kernel(const float *logits, int V, int S, double T,
                                                                  const double *segstats, DevState *st, int i,
                                                                  const int32_t *gate) {
  __shared__ double sh[kSeg + kSeg / 64];
  AE_GATE(gate);
  double mx, sum;
  combine_row_wave(segstats, S, 0, T, mx, sum);   // every wave computes the same pair
  const int t = threadIdx.x;
  // segment totals of p follow from the segment statistics
  const double segv = t < S ? segstats[(size_t)t * 2 + 1] * exp((segstats[(size_t)t * 2] - mx) / T) / sum : 0.0;
  const int tok = inverse_cdf_final(segv, S, logits, nullptr, V, 0, T, mx, sum, 0.0, 1.0, st->u_draft[i], sh, nullptr);
  if (t == 0) st->argmax[0] = tok;
}

// scratch layout (doubles): segstats [rows][S][2] | rowstats [rows][2] | segtot [S]
size_t sample_scratch_doubles(int V) {
  const size_t S = (V + kSeg - 1) / kSeg;
  return (size_t)2 * kMaxRows * S * 2 + 2 * kMaxRows * 2 + 2 * S + 16;
}

void launch_sample_draft(const float *logits, int V, float T, DevState *st, int i, double *scratch, hipStream_t s,
                         const int32_t *gate) {
  const int S = (V + kSeg - 1) / kSeg;
  double *segstats = scratch;
  seg_stats_kernel<<<dim3(S, 1), kSegThreads, 0, s>>>(logits, nullptr, V, 1, (double)T, segstats, gate);
  sample_draft_final_kernel<<<1, kSeg, 0, s>>>(logits, V, S, (double)T, segstats, st, i, gate);
}

// ------------------------------------------------------------------ acceptance + rollback bookkeeping
// Rows: kp+1 target rows then kp draft rows, kp = the draft tokens the block has room for; the
// number actually drafted is k = kp, or st->draft_len when the block was padded (k_on_device).
__device__ __forceinline__ int drafted(const DevState *st, int kp, int k_on_device) {
  return k_on_device ? min(st->draft_len, kp) : kp;
}

// Combines the row statistics, runs the accept tests (thread 0, in order) and records the
// outcome: st->n_acc, and the (max, sum) pairs of target row n_acc and, on a rejection, of
// draft row n_acc in rowstats[0..3].
__global__ __launch_bounds__(kSeg) void accept_decide_kernel(const float *tl, const float *dl, int V, int S, int kp,
                                                             int k_on_device, double T, const double *segstats,
                                                             double *rowstats, DevState *st) {
  __shared__ double rs[2 * kMaxRows][2];
  const int k = drafted(st, kp, k_on_device);
  const int wave = threadIdx.x >> 6;
  for (int row = wave; row < 2 * kp + 1; row += kSeg / 64) {   // one wave per row
    if ((row > k && row <= kp) || row > kp + k) continue;      // rows of tokens that were not drafted
    double mx, sum;
    combine_row_wave(segstats, S, row, T, mx, sum);
    if ((threadIdx.x & 63) == 0) { rs[row][0] = mx; rs[row][1] = sum; }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int acc = 0;
    for (; acc < k; ++acc) {
      const int t = st->block[1 + acc];
      const double p = exp(((double)tl[(size_t)acc * V + t] - rs[acc][0]) / T) / rs[acc][1];
      const double ph = exp(((double)dl[(size_t)acc * V + t] - rs[kp + 1 + acc][0]) / T) / rs[kp + 1 + acc][1];
      double ratio = ph > 0.0 ? p / ph : 1.0;
      if (ratio > 1.0) ratio = 1.0;
      if (!(st->u_accept[acc] < ratio)) break;
    }
    st->n_acc = acc;
    rowstats[0] = rs[acc][0]; rowstats[1] = rs[acc][1];
    rowstats[2] = acc < k ? rs[kp + 1 + acc][0] : 0.0;
    rowstats[3] = acc < k ? rs[kp + 1 + acc][1] : 1.0;
  }
}

// segtot[s] = sum over segment s of q for the row the accept tests stopped at (grid S)
__global__ __launch_bounds__(kSegThreads) void seg_total_kernel(const float *tl, const float *dl, int V, int kp,
                                                                int k_on_device, double T, const double *rowstats,
                                                                const DevState *st, double *segtot) {
  __shared__ double sh[kSegThreads];
  const int k = drafted(st, kp, k_on_device);
  const int acc = st->n_acc, mode = acc < k ? 1 : 0;
  const float *trow = tl + (size_t)acc * V, *drow = dl + (size_t)(acc < k ? acc : 0) * V;
  const double mt = rowstats[0], stt = rowstats[1], md = rowstats[2], sd = rowstats[3];
  double s = 0.0;
#pragma unroll
  for (int i = 0; i < kSeg / kSegThreads; ++i) {
    const int x = blockIdx.x * kSeg + threadIdx.x + i * kSegThreads;
    if (x < V) s += qval(trow, drow, x, mode, T, mt, stt, md, sd);
  }
  s = block_sum<kSegThreads>(s, sh);
  if (threadIdx.x == 0) segtot[blockIdx.x] = s;
}

// Draw of the bonus / resampled token and the rollback bookkeeping (one workgroup).
__global__ __launch_bounds__(kSeg) void accept_final_kernel(const float *tl, const float *dl, int V, int S, int kp,
                                                            int k_on_device, double T, const double *segstats,
                                                            const double *rowstats, const double *segtot, DevState *st,
                                                            int32_t *hist, int kv_len) {
  __shared__ double sh[kSeg + kSeg / 64];
  const int k = drafted(st, kp, k_on_device);
  const int acc = st->n_acc, mode = acc < k ? 1 : 0;
  const float *trow = tl + (size_t)acc * V, *drow = dl + (size_t)(acc < k ? acc : 0) * V;
  const double mt = rowstats[0], stt = rowstats[1], md = rowstats[2], sd = rowstats[3];
  const double u = st->u_accept[k];
  double tot = 0.0;
  const int t = threadIdx.x;
  int bonus = inverse_cdf_final(t < S ? segtot[t] : 0.0, S, trow, drow, V, mode, T, mt, stt, md, sd, u, sh, &tot);
  if (mode == 1 && !(tot > 0.0)) {
    // p == p_hat: the residual is empty, draw from the target law (segment totals from the statistics)
    const double segv = t < S ? segstats[((size_t)acc * S + t) * 2 + 1] * exp((segstats[((size_t)acc * S + t) * 2] - mt) / T) / stt
                              : 0.0;
    bonus = inverse_cdf_final(segv, S, trow, nullptr, V, 0, T, mt, stt, 0.0, 1.0, u, sh, nullptr);
  }
  if (threadIdx.x == 0) {
    for (int i = 0; i <= acc; ++i) hist[kv_len + i] = st->block[i];
    hist[kv_len + 1 + acc] = bonus;
    st->bonus = bonus;
  }
}

void launch_accept_sample(const float *tl, const float *dl, int V, int k, bool k_on_device, float T, DevState *st,
                          int32_t *hist, int kv_len, double *scratch, hipStream_t s) {
  const int kd = k_on_device ? 1 : 0;
  const int S = (V + kSeg - 1) / kSeg;
  double *segstats = scratch;
  double *rowstats = scratch + (size_t)2 * kMaxRows * S * 2;
  double *segtot = rowstats + 2 * kMaxRows * 2;
  seg_stats_kernel<<<dim3(S, 2 * k + 1), kSegThreads, 0, s>>>(tl, dl, V, k + 1, (double)T, segstats, nullptr);
  accept_decide_kernel<<<1, kSeg, 0, s>>>(tl, dl, V, S, k, kd, (double)T, segstats, rowstats, st);
  seg_total_kernel<<<S, kSegThreads, 0, s>>>(tl, dl, V, k, kd, (double)T, rowstats, st, segtot);
  accept_final_kernel<<<1, kSeg, 0, s>>>(tl, dl, V, S, k, kd, (double)T, segstats, rowstats, segtot, st, hist, kv_len);
}

}  // namespace ae
