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

// ---- block-wide helpers (fixed-shape trees over N = blockDim.x values in LDS) ----
template <int N>
__device__ __forceinline__ double block_sum(double v, double *sh) {
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
#pragma unroll
  for (int o = N / 2; o > 0; o >>= 1) {
    if (t < o) sh[t] += sh[t + o];
    __syncthreads();
  }
  const double r = sh[0];
  __syncthreads();
  return r;
}

template <int N>
__device__ __forceinline__ double block_max(double v, double *sh) {
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
#pragma unroll
  for (int o = N / 2; o > 0; o >>= 1) {
    if (t < o) sh[t] = fmax(sh[t], sh[t + o]);
    __syncthreads();
  }
  const double r = sh[0];
  __syncthreads();
  return r;
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

// (max, sum exp((l - max)/T)) of a whole row from its segment statistics; all kSeg threads call
__device__ void combine_row(const double *segstats, int S, int row, double T, double *sh, double &mx, double &sum) {
  const int t = threadIdx.x;
  const double ms = t < S ? segstats[((size_t)row * S + t) * 2] : -INFINITY;
  mx = block_max<kSeg>(ms, sh);
  const double term = t < S ? segstats[((size_t)row * S + t) * 2 + 1] * exp((ms - mx) / T) : 0.0;
  sum = block_sum<kSeg>(term, sh);
}

// mode 0: q(x) = p(x);  mode 1: q(x) = max(0, p(x) - p_hat(x)).  p, p_hat normalised softmaxes.
__device__ __forceinline__ double qval(const float *trow, const float *drow, int x, int mode, double T, double mt, double st,
                                       double md, double sd) {
  const double p = exp(((double)trow[x] - mt) / T) / st;
  if (mode == 0) return p;
  const double ph = exp(((double)drow[x] - md) / T) / sd;
  return p - ph > 0.0 ? p - ph : 0.0;
}

// Inverse CDF, last step.  segtot[s] = total of q over segment s (all threads may read it).
// Finds the smallest x with q(0)+..+q(x) > u * sum(q): thread 0 walks the segment totals, then
// the owning segment is scanned with one token per thread (Hillis-Steele prefix in LDS).  If
// rounding pushes the threshold past the total, the last token with q > 0 is returned.
// *total_out receives sum(q).  All kSeg threads call.
__device__ int inverse_cdf_final(const double *segtot, int S, const float *trow, const float *drow, int V, int mode, double T,
                                 double mt, double st, double md, double sd, double u, double *sh, double *total_out) {
  __shared__ double thr_s, before_s, tot_s;
  __shared__ int owner_s, res_s, lastq_s;
  const int t = threadIdx.x;
  if (t == 0) {
    double tot = 0.0;
    for (int s = 0; s < S; ++s) tot += segtot[s];
    const double thr = u * tot;
    double c = 0.0;
    int owner = -1, lastseg = 0;
    for (int s = 0; s < S; ++s) {
      const double v = segtot[s];
      if (v > 0.0) lastseg = s;
      if (owner < 0 && c + v > thr) { owner = s; before_s = c; }
      if (owner < 0) c += v;
    }
    tot_s = tot; thr_s = thr;
    if (owner < 0) { owner = lastseg; before_s = -1.0; }   // threshold beyond the total
    owner_s = owner;
    res_s = 0x7fffffff; lastq_s = -1;
  }
  __syncthreads();
  const int x = owner_s * kSeg + t;
  const double q = x < V ? qval(trow, drow, x, mode, T, mt, st, md, sd) : 0.0;
  // inclusive prefix over the segment (double buffer in sh[0..2*kSeg))
  double *a = sh, *b = sh + kSeg;
  a[t] = q;
  __syncthreads();
#pragma unroll
  for (int o = 1; o < kSeg; o <<= 1) {
    b[t] = t >= o ? a[t] + a[t - o] : a[t];
    __syncthreads();
    double *tmp = a; a = b; b = tmp;
  }
  const double incl = a[t];
  if (q > 0.0) atomicMax(&lastq_s, x);
  if (before_s >= 0.0 && q > 0.0 && before_s + incl > thr_s) atomicMin(&res_s, x);
  __syncthreads();
  if (total_out) *total_out = tot_s;
  int res = res_s;
  if (res == 0x7fffffff) res = lastq_s >= 0 ? lastq_s : owner_s * kSeg;   // rounding: last token with mass
  __syncthreads();
  return res;
}

// ------------------------------------------------------------------ draft sampling
// Draft token i ~ softmax(logits / T) by inverse CDF with st->u_draft[i]; result in st->argmax[0].
// Segment totals of p follow from the segment statistics, no second pass over the logits.
__global__ __launch_bounds__(kSeg) void sample_draft_final_kernel(const float *logits, int V, int S, double T,
                                                                  const double *segstats, double *segtot, DevState *st, int i,
                                                                  const int32_t *gate) {
  __shared__ double sh[2 * kSeg];
  AE_GATE(gate);
  double mx, sum;
  combine_row(segstats, S, 0, T, sh, mx, sum);
  const int t = threadIdx.x;
  if (t < S) segtot[t] = segstats[(size_t)t * 2 + 1] * exp((segstats[(size_t)t * 2] - mx) / T) / sum;
  __syncthreads();
  const int tok = inverse_cdf_final(segtot, S, logits, nullptr, V, 0, T, mx, sum, 0.0, 1.0, st->u_draft[i], sh, nullptr);
  if (t == 0) st->argmax[0] = tok;
}

// scratch layout (doubles): segstats [rows][S][2] | rowstats [rows][2] | segtot [S] | segtot2 [S]
size_t sample_scratch_doubles(int V) {
  const size_t S = (V + kSeg - 1) / kSeg;
  return (size_t)2 * kMaxRows * S * 2 + 2 * kMaxRows * 2 + 2 * S + 16;
}

void launch_sample_draft(const float *logits, int V, float T, DevState *st, int i, double *scratch, hipStream_t s,
                         const int32_t *gate) {
  const int S = (V + kSeg - 1) / kSeg;
  double *segstats = scratch, *segtot = scratch + (size_t)2 * kMaxRows * S * 2 + 2 * kMaxRows * 2;
  seg_stats_kernel<<<dim3(S, 1), kSegThreads, 0, s>>>(logits, nullptr, V, 1, (double)T, segstats, gate);
  sample_draft_final_kernel<<<1, kSeg, 0, s>>>(logits, V, S, (double)T, segstats, segtot, st, i, gate);
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
  __shared__ double sh[kSeg];
  __shared__ double rs[2 * kMaxRows][2];
  const int k = drafted(st, kp, k_on_device);
  for (int row = 0; row < 2 * kp + 1; ++row) {
    if ((row > k && row <= kp) || row > kp + k) continue;   // rows of tokens that were not drafted (uniform branch)
    double mx, sum;
    combine_row(segstats, S, row, T, sh, mx, sum);
    if (threadIdx.x == 0) { rs[row][0] = mx; rs[row][1] = sum; }
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
                                                            const double *rowstats, double *segtot, double *segtot2,
                                                            DevState *st, int32_t *hist, int kv_len) {
  __shared__ double sh[2 * kSeg];
  const int k = drafted(st, kp, k_on_device);
  const int acc = st->n_acc, mode = acc < k ? 1 : 0;
  const float *trow = tl + (size_t)acc * V, *drow = dl + (size_t)(acc < k ? acc : 0) * V;
  const double mt = rowstats[0], stt = rowstats[1], md = rowstats[2], sd = rowstats[3];
  const double u = st->u_accept[k];
  double tot = 0.0;
  int bonus = inverse_cdf_final(segtot, S, trow, drow, V, mode, T, mt, stt, md, sd, u, sh, &tot);
  if (mode == 1 && !(tot > 0.0)) {
    // p == p_hat: the residual is empty, draw from the target law (segment totals from the statistics)
    if (threadIdx.x < S)
      segtot2[threadIdx.x] = segstats[((size_t)acc * S + threadIdx.x) * 2 + 1] *
                             exp((segstats[((size_t)acc * S + threadIdx.x) * 2] - mt) / T) / stt;
    __syncthreads();
    bonus = inverse_cdf_final(segtot2, S, trow, nullptr, V, 0, T, mt, stt, 0.0, 1.0, u, sh, nullptr);
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
  double *segtot = rowstats + 2 * kMaxRows * 2, *segtot2 = segtot + S;
  seg_stats_kernel<<<dim3(S, 2 * k + 1), kSegThreads, 0, s>>>(tl, dl, V, k + 1, (double)T, segstats, nullptr);
  accept_decide_kernel<<<1, kSeg, 0, s>>>(tl, dl, V, S, k, kd, (double)T, segstats, rowstats, st);
  seg_total_kernel<<<S, kSegThreads, 0, s>>>(tl, dl, V, k, kd, (double)T, rowstats, st, segtot);
  accept_final_kernel<<<1, kSeg, 0, s>>>(tl, dl, V, S, k, kd, (double)T, segstats, rowstats, segtot, segtot2, st, hist, kv_len);
}

}  // namespace ae
