// Temperature > 0: draft sampling and the lossless rejection-sampling rule of speculative
// decoding (arxiv 2412.18910, Sec. 2.1):  draft token t is accepted with probability
// min(1, p(t)/p_hat(t)); the first rejection resamples from norm(max(0, p - p_hat)) over the
// whole vocabulary; with no rejection the bonus token comes from the target law of the row
// after the last draft token.  Every draw is an inverse CDF in token-id order driven by a
// caller-supplied uniform.  Softmax, ratio, residual and prefix sums are float64: in float32
// a prefix sum over ~128k tokens would let rounding noise decide a visible share of draws.
#include "ae_internal.h"

namespace ae {

constexpr int kSampThreads = 1024;

__device__ __forceinline__ double block_reduce(double v, double *sh, bool is_max) {
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
  for (int o = kSampThreads / 2; o > 0; o >>= 1) {   // fixed-shape tree: deterministic
    if (t < o) sh[t] = is_max ? fmax(sh[t], sh[t + o]) : sh[t] + sh[t + o];
    __syncthreads();
  }
  const double r = sh[0];
  __syncthreads();
  return r;
}

// (max, sum exp((l - max)/T)) of one logits row per workgroup
__global__ __launch_bounds__(kSampThreads) void row_stats_kernel(const float *tl, const float *dl, int V, int n_target,
                                                                  double T, double *stats) {
  __shared__ double sh[kSampThreads];
  const int row = blockIdx.x;
  const float *x = row < n_target ? tl + (size_t)row * V : dl + (size_t)(row - n_target) * V;
  double mx = -INFINITY;
  for (int i = threadIdx.x; i < V; i += kSampThreads) mx = fmax(mx, (double)x[i]);
  mx = block_reduce(mx, sh, true);
  double s = 0.0;
  for (int i = threadIdx.x; i < V; i += kSampThreads) s += exp(((double)x[i] - mx) / T);
  s = block_reduce(s, sh, false);
  if (threadIdx.x == 0) { stats[2 * row] = mx; stats[2 * row + 1] = s; }
}

// mode 0: q(x) = p(x);  mode 1: q(x) = max(0, p(x) - p_hat(x)).  p, p_hat normalised softmaxes.
__device__ __forceinline__ double qval(const float *tl, const float *dl, int x, int mode, double T, double mt, double st,
                                       double md, double sd) {
  const double p = exp(((double)tl[x] - mt) / T) / st;
  if (mode == 0) return p;
  const double ph = exp(((double)dl[x] - md) / T) / sd;
  return p - ph > 0.0 ? p - ph : 0.0;
}

// Inverse CDF over token ids: smallest x with q(0)+..+q(x) > u * sum(q).  Each thread owns a
// contiguous slice; slice totals are scanned, then the slice holding the threshold is walked.
__device__ int inverse_cdf(const float *tl, const float *dl, int V, int mode, double T, double mt, double st, double md,
                           double sd, double u, double *sh, double *total_out) {
  const int t = threadIdx.x;
  const int per = (V + kSampThreads - 1) / kSampThreads;
  const int lo = t * per, hi = min(V, lo + per);
  double loc = 0.0;
  for (int x = lo; x < hi; ++x) loc += qval(tl, dl, x, mode, T, mt, st, md, sd);
  sh[t] = loc;
  __syncthreads();
  __shared__ double tot_s, before_s;
  __shared__ int owner_s, last_pos_s;
  if (t == 0) {
    double tot = 0.0;
    for (int i = 0; i < kSampThreads; ++i) tot += sh[i];
    tot_s = tot;
    const double thr = u * tot;
    double c = 0.0;
    int owner = -1, lastpos = 0;
    for (int i = 0; i < kSampThreads; ++i) {
      if (sh[i] > 0.0) lastpos = i;
      if (owner < 0 && c + sh[i] > thr) { owner = i; before_s = c; }
      if (owner < 0) c += sh[i];
    }
    if (owner < 0) { owner = lastpos; before_s = -1.0; }   // rounding pushed thr past the total
    owner_s = owner;
    last_pos_s = lastpos;
  }
  __syncthreads();
  __shared__ int result_s;
  if (t == owner_s) {
    const double thr = u * tot_s;
    int res = -1, lastq = lo;
    double c = before_s < 0.0 ? 0.0 : before_s;
    for (int x = lo; x < hi; ++x) {
      const double q = qval(tl, dl, x, mode, T, mt, st, md, sd);
      if (q > 0.0) lastq = x;
      c += q;
      if (before_s >= 0.0 && c > thr) { res = x; break; }
    }
    result_s = res >= 0 ? res : lastq;
  }
  __syncthreads();
  if (total_out) *total_out = tot_s;
  return result_s;
}

// Draft token i ~ softmax(logits / T) by inverse CDF with st->u_draft[i]; result in st->argmax[0]
__global__ __launch_bounds__(kSampThreads) void sample_draft_kernel(const float *logits, int V, double T, DevState *st,
                                                                     int i) {
  __shared__ double sh[kSampThreads];
  double mx = -INFINITY;
  for (int x = threadIdx.x; x < V; x += kSampThreads) mx = fmax(mx, (double)logits[x]);
  mx = block_reduce(mx, sh, true);
  double s = 0.0;
  for (int x = threadIdx.x; x < V; x += kSampThreads) s += exp(((double)logits[x] - mx) / T);
  s = block_reduce(s, sh, false);
  const int tok = inverse_cdf(logits, nullptr, V, 0, T, mx, s, 0.0, 1.0, st->u_draft[i], sh, nullptr);
  if (threadIdx.x == 0) st->argmax[0] = tok;
}

void launch_sample_draft(const float *logits, int V, float T, DevState *st, int i, double *, hipStream_t s) {
  sample_draft_kernel<<<1, kSampThreads, 0, s>>>(logits, V, (double)T, st, i);
}

// Acceptance + rollback bookkeeping, one workgroup.  stats = row_stats of the k+1 target rows
// followed by the k draft rows.
__global__ __launch_bounds__(kSampThreads) void accept_sample_kernel(const float *tl, const float *dl, int V, int k,
                                                                      double T, const double *stats, DevState *st,
                                                                      int32_t *hist, int kv_len) {
  __shared__ double sh[kSampThreads];
  __shared__ int n_acc_s;
  if (threadIdx.x == 0) {
    int acc = 0;
    for (; acc < k; ++acc) {
      const int t = st->block[1 + acc];
      const double p = exp(((double)tl[(size_t)acc * V + t] - stats[2 * acc]) / T) / stats[2 * acc + 1];
      const double ph = exp(((double)dl[(size_t)acc * V + t] - stats[2 * (k + 1 + acc)]) / T) / stats[2 * (k + 1 + acc) + 1];
      double ratio = ph > 0.0 ? p / ph : 1.0;
      if (ratio > 1.0) ratio = 1.0;
      if (!(st->u_accept[acc] < ratio)) break;
    }
    n_acc_s = acc;
  }
  __syncthreads();
  const int acc = n_acc_s;
  const float *trow = tl + (size_t)acc * V;
  const double mt = stats[2 * acc], stt = stats[2 * acc + 1];
  const double u = st->u_accept[k];
  int bonus;
  if (acc < k) {
    const float *drow = dl + (size_t)acc * V;
    const double md = stats[2 * (k + 1 + acc)], sd = stats[2 * (k + 1 + acc) + 1];
    double tot = 0.0;
    bonus = inverse_cdf(trow, drow, V, 1, T, mt, stt, md, sd, u, sh, &tot);
    if (!(tot > 0.0)) bonus = inverse_cdf(trow, nullptr, V, 0, T, mt, stt, 0.0, 1.0, u, sh, nullptr);   // p == p_hat
  } else {
    bonus = inverse_cdf(trow, nullptr, V, 0, T, mt, stt, 0.0, 1.0, u, sh, nullptr);
  }
  if (threadIdx.x == 0) {
    for (int i = 0; i <= acc; ++i) hist[kv_len + i] = st->block[i];
    hist[kv_len + 1 + acc] = bonus;
    st->n_acc = acc;
    st->bonus = bonus;
  }
}

void launch_accept_sample(const float *tl, const float *dl, int V, int k, float T, DevState *st, int32_t *hist, int kv_len,
                          double *stats, hipStream_t s) {
  row_stats_kernel<<<2 * k + 1, kSampThreads, 0, s>>>(tl, dl, V, k + 1, (double)T, stats);
  accept_sample_kernel<<<1, kSampThreads, 0, s>>>(tl, dl, V, k, (double)T, stats, st, hist, kv_len);
}

}  // namespace ae
