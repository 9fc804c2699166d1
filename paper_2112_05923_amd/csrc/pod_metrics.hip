// Trading performance of recorded rollouts (Sec. 5.3 "Performance metrics";
// what the evaluator of Sec. 4.2 reports next to the episodic reward):
// cumulative return, annual return and volatility, maximum drawdown, Sharpe
// and Calmar ratio of the account-value curve of the first episode of every
// env in an observation buffer.
//
// The value V_t = cash_t + sum_d h_{t,d} p_{t,d} is decoded from the
// observation (Table 1 state; the power-of-two scales divide out exactly) in
// binary64, stock order.  A workgroup owns 64 envs (one per lane) and its 16
// wavefronts split the time axis into chunks; each reduces its chunk to a
// small summary (Welford moments of the per-period returns, running peak,
// lowest value, lowest value-to-running-peak ratio) and the first wavefront
// merges the 16 summaries in time order:
//   moments:   Chan's pairwise update;
//   drawdown:  min over t of V_t / max_{s<=t} V_s over two consecutive spans
//              a, b is min(ratio_a, ratio_b, lowest_b / peak_a).
// Bound by HBM: 4 (1 + 2 D) bytes per (t, env) out of every S-float row.
#include "pod_internal.h"

namespace pod {
namespace {

constexpr int ME = 64;   // envs per workgroup
constexpr int MW = 16;   // wavefronts = time chunks

struct Chunk {
  double mean, m2;      // of the returns r_t = V_{t+1} / V_t - 1 inside the chunk
  double peak, low;     // highest and lowest value
  double ratio;         // lowest V_t / (running peak within the chunk)
  double v_last;        // value at point L when it falls into the chunk
  int32_t n_ret, n_pts;
};

__device__ inline double value_at(const float *__restrict__ o, int D, double inv_cash, double inv_price,
                                  double inv_hold) {
  double v = (double)o[0] * inv_cash;
  for (int d = 0; d < D; ++d) v += ((double)o[1 + D + d] * inv_hold) * ((double)o[1 + d] * inv_price);
  return v;
}

__global__ __launch_bounds__(ME * MW) void metrics_kernel(int T, int N, int D, int S, const float *__restrict__ obs,
                                                          const uint8_t *__restrict__ done, double inv_cash,
                                                          double inv_price, double inv_hold, double periods, double rf,
                                                          double *__restrict__ metrics, int32_t *__restrict__ length) {
  __shared__ int32_t s_first[MW][ME];
  __shared__ Chunk s_chunk[MW][ME];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n = blockIdx.x * ME + lane;
  const bool live = n < N;
  const int span = (T + 1 + MW - 1) / MW;          // points per chunk
  const int c0 = w * span, c1 = min(c0 + span, T + 1);

  // ---- length of the first episode: first step whose done flag is set, else T
  int first = T;
  if (live)
    for (int t = min(c1, T) - 1; t >= c0; --t)
      if (done[(size_t)t * N + n]) first = t;
  s_first[w][lane] = first;
  __syncthreads();
  int L = T;
  for (int c = 0; c < MW; ++c) L = min(L, s_first[c][lane]);

  // ---- summary of this chunk: points c0 .. min(c1 - 1, L), returns for t with t + 1 <= L
  Chunk ck;
  ck.mean = 0.0;
  ck.m2 = 0.0;
  ck.peak = 0.0;
  ck.low = 0.0;
  ck.ratio = 1.0;
  double v_first = 0.0;  // (only the first chunk's is used, by the lanes that merge)
  ck.v_last = 0.0;
  ck.n_ret = 0;
  ck.n_pts = 0;
  if (live && c0 <= L) {
    const int last = min(c1 - 1, L);
    double v = value_at(obs + ((size_t)c0 * N + n) * S, D, inv_cash, inv_price, inv_hold);
    v_first = v;
    ck.peak = v;
    ck.low = v;
    ck.n_pts = 1;
    if (c0 == L) ck.v_last = v;
    for (int t = c0; t <= last; ++t) {
      if (t + 1 > L) break;
      // the return of step t needs the next point, which may be the first point of the next chunk
      const double vn = value_at(obs + ((size_t)(t + 1) * N + n) * S, D, inv_cash, inv_price, inv_hold);
      const double r = vn / v - 1.0;
      ck.n_ret += 1;
      const double dlt = r - ck.mean;
      ck.mean += dlt / (double)ck.n_ret;
      ck.m2 += dlt * (r - ck.mean);
      if (t + 1 <= last) {  // the next point belongs to this chunk
        ck.peak = fmax(ck.peak, vn);
        ck.low = fmin(ck.low, vn);
        ck.ratio = fmin(ck.ratio, vn / ck.peak);
        ck.n_pts += 1;
        if (t + 1 == L) ck.v_last = vn;
      }
      v = vn;
    }
  }
  s_chunk[w][lane] = ck;
  __syncthreads();

  // ---- merge in time order, one lane per env
  if (w == 0 && live) {
    double mean = 0.0, m2 = 0.0, peak = 0.0, ratio = 1.0, v0 = 0.0, vl = 0.0;
    int64_t cnt = 0;
    for (int c = 0; c < MW; ++c) {
      const Chunk &b = s_chunk[c][lane];
      if (b.n_pts > 0) {
        if (c == 0) v0 = v_first;
        if (peak > 0.0) ratio = fmin(ratio, b.low / peak);
        ratio = fmin(ratio, b.ratio);
        peak = fmax(peak, b.peak);
        const int cl = c * span, ch = min(cl + span, T + 1) - 1;
        if (L >= cl && L <= ch) vl = b.v_last;
      }
      if (b.n_ret > 0) {
        const double nb = (double)b.n_ret, na = (double)cnt, nt = na + nb;
        const double dlt = b.mean - mean;
        mean += dlt * (nb / nt);
        m2 += b.m2 + dlt * dlt * (na * nb / nt);
        cnt += b.n_ret;
      }
    }
    double out[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    if (L >= 1) {
      const double sd = L >= 2 ? sqrt(m2 / (double)(L - 1)) : 0.0;
      const double mdd = 1.0 - ratio;
      out[0] = (vl - v0) / v0;
      out[1] = pow(vl / v0, periods / (double)L) - 1.0;
      out[2] = sqrt(periods) * sd;
      out[3] = mdd;
      out[4] = sd > 0.0 ? sqrt(periods) * (mean - rf / periods) / sd : 0.0;
      out[5] = mdd > 0.0 ? out[1] / mdd : 0.0;
    }
    for (int i = 0; i < 6; ++i) metrics[(size_t)i * N + n] = out[i];
    if (length) length[n] = L;
  }
}

}  // namespace

hipError_t launch_trading_metrics(hipStream_t st, int32_t T, int32_t N, int32_t D, int32_t S, const float *obs,
                                  const uint8_t *done, const float *obs_scale, double periods, double rf,
                                  double *metrics, int32_t *length) {
  const unsigned blocks = (unsigned)((N + ME - 1) / ME);
  hipLaunchKernelGGL(metrics_kernel, dim3(blocks), dim3(ME * MW), 0, st, T, N, D, S, obs, done,
                     1.0 / (double)obs_scale[0], 1.0 / (double)obs_scale[1], 1.0 / (double)obs_scale[2], periods, rf,
                     metrics, length);
  return hipGetLastError();
}

}  // namespace pod
