// Trading performance of recorded rollouts (Sec. 5.3 "Performance metrics";
// what the evaluator of Sec. 4.2 reports next to the episodic reward):
// cumulative return, annual return and volatility, maximum drawdown, Sharpe
// and Calmar ratio of the account-value curve of the first episode of every
// env in an observation buffer.
//
// The value V_t = cash_t + sum_d h_{t,d} p_{t,d} is decoded from the
// observation (Table 1 state; the power-of-two scales divide out exactly) in
// binary64, stock order.  A workgroup owns 64 envs and its 8 wavefronts split
// the time axis into chunks.  For every point of its chunk a wavefront stages
// the price and holdings runs of the 64 rows in LDS with coalesced loads (a few
// rows per load instruction), then each lane walks its own env's row there;
// the chunk is reduced to a small summary (Welford moments of the per-period
// returns, running peak, lowest value, lowest value-to-running-peak ratio) and
// the first wavefront merges the 8 summaries in time order:
//   moments:   Chan's pairwise update;
//   drawdown:  min over t of V_t / max_{s<=t} V_s over two consecutive spans
//              a, b is min(ratio_a, ratio_b, lowest_b / peak_a).
// Bound by HBM: 4 (1 + 2 D) bytes per (t, env) out of every S-float row.
#include "pod_internal.h"

namespace pod {
namespace {

constexpr int ME = 64;           // envs per workgroup
constexpr int MW = 8;            // wavefronts = time chunks
constexpr int MB = 32;           // stocks staged at a time
constexpr int MP = 2 * MB + 1;   // floats per staged row (odd: lanes reading their own row hit distinct banks)

struct Chunk {
  double mean, m2;      // of the returns r_t = V_{t+1} / V_t - 1 inside the chunk
  double peak, low;     // highest and lowest value
  double ratio;         // lowest V_t / (running peak within the chunk)
  double v_last;        // value at point L when it falls into the chunk
  int32_t n_ret, n_pts;
};

struct MetricArgs {
  int32_t T, N, D, S;
  const float *obs;
  const uint8_t *done;
  double inv_cash, inv_price, inv_hold, periods, rf;
  double *metrics;
  int32_t *length;
};

__global__ __launch_bounds__(ME * MW) void metrics_kernel(MetricArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  // [MW][ME][MP] staging floats; the chunk summaries reuse the space once the chunks are done
  float *stage_all = reinterpret_cast<float *>(lds);
  int32_t *s_first = reinterpret_cast<int32_t *>(stage_all + (size_t)MW * ME * MP);  // [MW][ME]
  Chunk *s_chunk = reinterpret_cast<Chunk *>(lds);                                  // [MW][ME]
  const int T = a.T, N = a.N, D = a.D, S = a.S;
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n0 = blockIdx.x * ME;
  const int n = n0 + lane;
  const bool live = n < N;
  const int span = (T + 1 + MW - 1) / MW;  // points per chunk
  const int c0 = w * span, c1 = min(c0 + span, T + 1);
  float *stage = stage_all + (size_t)w * ME * MP;

  // ---- length of the first episode: first step whose done flag is set, else T
  int first = T;
  if (live)
    for (int t = min(c1, T) - 1; t >= c0; --t)
      if (a.done[(size_t)t * N + n]) first = t;
  s_first[w * ME + lane] = first;
  __syncthreads();
  int L = T;
  for (int c = 0; c < MW; ++c) L = min(L, s_first[c * ME + lane]);
  // the wavefront works on point t as long as any of its lanes needs it
  int Lmax = L;
  for (int off = 32; off > 0; off >>= 1) Lmax = max(Lmax, __shfl_xor(Lmax, off));

  // Value of point t for this lane's env (every lane of the wavefront takes part in the staging).
  auto value_at = [&](int t) -> double {
    const float *base = a.obs + (size_t)t * N * S;
    double v = live ? (double)base[(size_t)n * S] * a.inv_cash : 0.0;
    constexpr int RPI = 64 / MB;  // rows per load instruction
    const int sub = lane / MB, c = lane % MB;
    for (int d0 = 0; d0 < D; d0 += MB) {
      const int bw = min(MB, D - d0);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the previous block's reads are done
      // all of the block's loads are issued before the first of them is stored (one round trip per block, not one
      // per pair of rows)
      float pr[ME / RPI], ho[ME / RPI];
#pragma unroll
      for (int rr = 0; rr < ME / RPI; ++rr) {
        const int row = RPI * rr + sub;
        const bool ok = c < bw && n0 + row < N;
        const float *o = base + (size_t)(n0 + (ok ? row : 0)) * S;
        pr[rr] = ok ? __builtin_nontemporal_load(o + 1 + d0 + c) : 0.0f;
        ho[rr] = ok ? __builtin_nontemporal_load(o + 1 + D + d0 + c) : 0.0f;
      }
#pragma unroll
      for (int rr = 0; rr < ME / RPI; ++rr) {
        const int row = RPI * rr + sub;
        if (c < bw && n0 + row < N) {
          stage[row * MP + c] = pr[rr];
          stage[row * MP + MB + c] = ho[rr];
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // LDS executes a wavefront's accesses in order
      if (live)
        for (int j = 0; j < bw; ++j)
          v += ((double)stage[lane * MP + MB + j] * a.inv_hold) * ((double)stage[lane * MP + j] * a.inv_price);
    }
    return v;
  };

  // ---- summary of this chunk: points c0 .. min(c1 - 1, L), returns for t with t + 1 <= L
  Chunk ck;
  ck.mean = 0.0;
  ck.m2 = 0.0;
  ck.peak = 0.0;
  ck.low = 0.0;
  ck.ratio = 1.0;
  ck.v_last = 0.0;
  ck.n_ret = 0;
  ck.n_pts = 0;
  double v_first = 0.0;  // (only the first chunk's is used, by the lanes that merge)
  if (c0 <= Lmax) {      // wavefront-uniform
    const int last_w = min(c1 - 1, Lmax);
    const int last = min(c1 - 1, L);
    double v = value_at(c0);
    if (c0 <= L) {
      v_first = v;
      ck.peak = v;
      ck.low = v;
      ck.n_pts = 1;
      if (c0 == L) ck.v_last = v;
    }
    for (int t = c0; t <= last_w && t + 1 <= Lmax; ++t) {
      // the return of step t needs the next point, which may be the first point of the next chunk
      const double vn = value_at(t + 1);
      if (t <= last && t + 1 <= L) {
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
      }
      v = vn;
    }
  }
  __syncthreads();  // staging buffers are dead: the summaries go over them
  s_chunk[w * ME + lane] = ck;
  __syncthreads();

  // ---- merge in time order, one lane per env
  if (w == 0 && live) {
    double mean = 0.0, m2 = 0.0, peak = 0.0, ratio = 1.0, vl = 0.0;
    const double v0 = v_first;
    int64_t cnt = 0;
    for (int c = 0; c < MW; ++c) {
      const Chunk b = s_chunk[c * ME + lane];
      if (b.n_pts > 0) {
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
      out[1] = pow(vl / v0, a.periods / (double)L) - 1.0;
      out[2] = sqrt(a.periods) * sd;
      out[3] = mdd;
      out[4] = sd > 0.0 ? sqrt(a.periods) * (mean - a.rf / a.periods) / sd : 0.0;
      out[5] = mdd > 0.0 ? out[1] / mdd : 0.0;
    }
    for (int i = 0; i < 6; ++i) a.metrics[(size_t)i * N + n] = out[i];
    if (a.length) a.length[n] = L;
  }
}

}  // namespace

hipError_t launch_trading_metrics(hipStream_t st, int32_t T, int32_t N, int32_t D, int32_t S, const float *obs,
                                  const uint8_t *done, const float *obs_scale, double periods, double rf,
                                  double *metrics, int32_t *length) {
  MetricArgs a;
  a.T = T;
  a.N = N;
  a.D = D;
  a.S = S;
  a.obs = obs;
  a.done = done;
  a.inv_cash = 1.0 / (double)obs_scale[0];
  a.inv_price = 1.0 / (double)obs_scale[1];
  a.inv_hold = 1.0 / (double)obs_scale[2];
  a.periods = periods;
  a.rf = rf;
  a.metrics = metrics;
  a.length = length;
  size_t lds = (size_t)MW * ME * MP * 4;
  if (lds < (size_t)MW * ME * sizeof(Chunk)) lds = (size_t)MW * ME * sizeof(Chunk);
  lds += (size_t)MW * ME * 4;
  const hipError_t e = allow_full_lds<metrics_kernel>();
  if (e != hipSuccess) return e;
  const unsigned blocks = (unsigned)((N + ME - 1) / ME);
  hipLaunchKernelGGL(metrics_kernel, dim3(blocks), dim3(ME * MW), lds, st, a);
  return hipGetLastError();
}

}  // namespace pod
