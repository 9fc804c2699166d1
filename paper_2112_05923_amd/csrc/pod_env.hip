// Vectorised stock-trading environment: observation assembly, Gaussian action
// sampling, trade execution, reward, episode end and reset (Table 1 and
// Sec. 5.3 of the paper; the worker of Sec. 4.2 steps N such envs at once),
// plus the per-env state plumbing and the leaderboard reduction (Sec. 4.1).
//
// This translation unit is compiled with floating-point contraction off: the
// share counts are decided by a fixed sequence of binary32 operations with one
// rounding each, and a fused multiply-add would change which integer a
// quotient lands on.
#include "pod_internal.h"

namespace pod {

namespace {

constexpr int kThreads = 256;

struct RowInfo {
  int32_t row_now;   // market row the trades execute at
  int32_t row_val;   // market row the portfolio is valued at (cursor + 1)
  int32_t row_obs;   // market row of the next observation (0 after a reset)
  int32_t done;
};

__device__ inline RowInfo rows_of(const EnvDims &d, int32_t tau, int32_t n) {
  const int32_t m = d.M == 1 ? 0 : n;
  RowInfo r;
  r.row_now = tau * d.M + m;
  r.row_val = (tau + 1) * d.M + m;
  r.done = (tau + 1 == d.H);
  r.row_obs = r.done ? m : r.row_val;
  return r;
}

// ------------------------------------------------------------------ observe
// obs[n] = [cash s0, price s1, holdings s2, indicators s3] at the current cursor.
__global__ __launch_bounds__(kThreads) void observe_kernel(EnvDims d, EnvState s, const float *__restrict__ price,
                                                          const float *__restrict__ ind, float *__restrict__ obs) {
  // one wavefront per env row, lanes across the row
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
  if (n >= d.N) return;
  const int32_t tau = s.tau[n];
  const int32_t m = d.M == 1 ? 0 : n;
  const size_t row = (size_t)tau * d.M + m;
  float *o = obs + (size_t)n * d.S;
  const int DK = d.D * d.K;
  for (int j = lane; j < d.S; j += 64) {
    float v;
    if (j == 0) {
      v = s.cash[n] * d.s_cash;
    } else if (j <= d.D) {
      v = price[row * d.D + (j - 1)] * d.s_price;
    } else if (j <= 2 * d.D) {
      v = (float)s.h[(size_t)(j - 1 - d.D) * d.N + n] * d.s_hold;
    } else {
      v = ind[row * DK + (j - 1 - 2 * d.D)] * d.s_ind;
    }
    o[j] = v;
  }
}

// ----------------------------------------------------------------- env step
// One workgroup steps E consecutive envs.  LDS holds five [E][Dp] arrays
// (Dp odd so that the per-env serial loops of the trade pass hit distinct
// banks): clamped action, eps^2 (later the executed shares), execution prices,
// valuation prices, holdings.
template <int E>
__global__ __launch_bounds__(kThreads) void env_step_kernel(EnvDims d, EnvState s, const float *__restrict__ price,
                                                           const float *__restrict__ ind, StepIO io) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int D = d.D, Dp = D | 1;
  float *s_a = reinterpret_cast<float *>(lds_raw);
  float *s_e2 = s_a + E * Dp;
  int32_t *s_q = reinterpret_cast<int32_t *>(s_e2);
  float *s_p = s_e2 + E * Dp;
  float *s_pv = s_p + E * Dp;
  int32_t *s_h = reinterpret_cast<int32_t *>(s_pv + E * Dp);
  RowInfo *s_row = reinterpret_cast<RowInfo *>(s_h + E * Dp);
  float *s_cash = reinterpret_cast<float *>(s_row + E);

  const int tid = threadIdx.x;
  const int n0 = blockIdx.x * E;
  const int ne = min(E, d.N - n0);  // live envs of this tile

  if (tid < ne) s_row[tid] = rows_of(d, s.tau[n0 + tid], n0 + tid);
  __syncthreads();

  // -- stage the tile: sample the action, fetch prices and holdings
  const int tile_elems = ne * D;
  const size_t g0 = (size_t)n0 * D;
  for (int idx = tid; idx < tile_elems; idx += kThreads) {
    const int e = idx / D, dd = idx - e * D;
    const float mu = io.mu[g0 + idx];
    const float eps = io.noise[g0 + idx];
    const float a_raw = mu + d.sigma * eps;  // two roundings (contraction is off)
    io.act_raw[g0 + idx] = a_raw;
    s_a[e * Dp + dd] = fminf(1.0f, fmaxf(-1.0f, a_raw));
    s_e2[e * Dp + dd] = eps * eps;
    s_p[e * Dp + dd] = price[(size_t)s_row[e].row_now * D + dd];
    s_pv[e * Dp + dd] = price[(size_t)s_row[e].row_val * D + dd];
  }
  for (int idx = tid; idx < E * D; idx += kThreads) {
    const int dd = idx / E, e = idx - dd * E;
    if (e < ne) s_h[e * Dp + dd] = s.h[(size_t)dd * d.N + n0 + e];
  }
  __syncthreads();

  if (tid < E) {
    // -- one lane per env: the serial part (Table 1 actions: sell / buy / hold)
    if (tid < ne) {
      const int e = tid, n = n0 + e;
      float *a = s_a + e * Dp;
      float *p = s_p + e * Dp;
      float *pv = s_pv + e * Dp;
      int32_t *h = s_h + e * Dp;
      int32_t *q_out = s_q + e * Dp;
      float cash = s.cash[n];
      float e2 = 0.0f;
      double asset0 = (double)cash;
      for (int dd = 0; dd < D; ++dd) {
        asset0 += (double)h[dd] * (double)p[dd];
        e2 += s_e2[e * Dp + dd];
      }
      // wanted shares, then all sales in stock order
      for (int dd = 0; dd < D; ++dd) {
        const int32_t k = (int32_t)truncf(a[dd] * d.hmax);
        int32_t q = 0;
        if (k < 0) {
          q = min(-k, h[dd]);
          h[dd] -= q;
          const float gross = p[dd] * (float)q;
          const float net = gross * d.one_minus_c;
          cash = cash + net;
          q = -q;
        }
        a[dd] = __int_as_float(k);
        q_out[dd] = q;
      }
      // all purchases in stock order, each limited by the cash left
      for (int dd = 0; dd < D; ++dd) {
        const int32_t k = __float_as_int(a[dd]);
        if (k > 0) {
          const float u = p[dd] * d.one_plus_c;
          const float ratio = cash / u;
          int32_t m = (int32_t)floorf(ratio);
          m = max(m, 0);
          int32_t q = min(k, m);
          float outlay = (float)q * u;
          if (outlay > cash) {
            q -= 1;
            outlay = (float)q * u;
          }
          h[dd] += q;
          cash = cash - outlay;
          q_out[dd] = q;
        }
      }
      double asset1 = (double)cash;
      for (int dd = 0; dd < D; ++dd) asset1 += (double)h[dd] * (double)pv[dd];
      const double r = (asset1 - asset0) * (double)d.rho;
      const RowInfo ri = s_row[e];
      double ep = s.ep_ret[n] + r;
      if (ri.done) {
        s.ep_sum[n] += ep;
        s.ep_sqsum[n] += ep * ep;
        s.ep_cnt[n] += 1;
        ep = 0.0;
        cash = d.cash0;
        for (int dd = 0; dd < D; ++dd) h[dd] = 0;
      }
      s.ep_ret[n] = ep;
      s.cash[n] = cash;
      s.tau[n] = ri.done ? 0 : s.tau[n] + 1;
      s_cash[e] = cash;
      io.reward[n] = (float)r;
      io.done[n] = (uint8_t)ri.done;
      if (io.logp) io.logp[n] = fmaf(-0.5f, e2, d.logp_const);
    }
  } else {
    // -- the other wavefronts stream the market part of the next observation
    const int DK = D * d.K;
    const int per_row = D + DK;  // prices then indicators, both at row_obs
    const int nthr = kThreads - E;
    const int t2 = tid - E;
    if (nthr > 0) {
      for (int idx = t2; idx < ne * per_row; idx += nthr) {
        const int e = idx / per_row, j = idx - e * per_row;
        const size_t row = (size_t)s_row[e].row_obs;
        float *o = io.obs_next + (size_t)(n0 + e) * d.S;
        if (j < D)
          o[1 + j] = price[row * D + j] * d.s_price;
        else
          o[1 + 2 * D + (j - D)] = ind[row * DK + (j - D)] * d.s_ind;
      }
    }
  }
  __syncthreads();

  // -- write back what the trade pass produced
  if (tid < ne) io.obs_next[(size_t)(n0 + tid) * d.S] = s_cash[tid] * d.s_cash;
  for (int idx = tid; idx < tile_elems; idx += kThreads) {
    const int e = idx / D, dd = idx - e * D;
    io.obs_next[(size_t)(n0 + e) * d.S + 1 + D + dd] = (float)s_h[e * Dp + dd] * d.s_hold;
    if (io.shares) io.shares[g0 + idx] = s_q[e * Dp + dd];
  }
  for (int idx = tid; idx < E * D; idx += kThreads) {
    const int dd = idx / E, e = idx - dd * E;
    if (e < ne) s.h[(size_t)dd * d.N + n0 + e] = s_h[e * Dp + dd];
  }
}

size_t env_lds(int E, int D) {
  const int Dp = D | 1;
  return (size_t)5 * E * Dp * 4 + (size_t)E * (sizeof(RowInfo) + sizeof(float));
}

// ------------------------------------------------------------ state plumbing
__global__ void state_reset_kernel(EnvDims d, EnvState s) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (size_t)d.N) {
    s.cash[i] = d.cash0;
    s.tau[i] = 0;
    s.ep_ret[i] = 0.0;
    s.ep_sum[i] = 0.0;
    s.ep_sqsum[i] = 0.0;
    s.ep_cnt[i] = 0;
  }
  if (i < (size_t)d.N * d.D) s.h[i] = 0;
}

// user layout (env-major holdings [N, D]) <-> structure of arrays ([D][N])
__global__ void state_copy_kernel(EnvDims d, EnvState s, pr_state u, int to_user) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (size_t)d.N) {
    if (to_user) {
      if (u.cash) u.cash[i] = s.cash[i];
      if (u.cursor) u.cursor[i] = s.tau[i];
      if (u.ep_return) u.ep_return[i] = s.ep_ret[i];
      if (u.ep_sum) u.ep_sum[i] = s.ep_sum[i];
      if (u.ep_sqsum) u.ep_sqsum[i] = s.ep_sqsum[i];
      if (u.ep_count) u.ep_count[i] = s.ep_cnt[i];
    } else {
      if (u.cash) s.cash[i] = u.cash[i];
      if (u.cursor) s.tau[i] = u.cursor[i];
      if (u.ep_return) s.ep_ret[i] = u.ep_return[i];
      if (u.ep_sum) s.ep_sum[i] = u.ep_sum[i];
      if (u.ep_sqsum) s.ep_sqsum[i] = u.ep_sqsum[i];
      if (u.ep_count) s.ep_cnt[i] = u.ep_count[i];
    }
  }
  if (u.holdings && i < (size_t)d.N * d.D) {
    const size_t n = i / d.D, dd = i - n * d.D;  // i indexes the user layout
    if (to_user)
      u.holdings[i] = s.h[dd * d.N + n];
    else
      s.h[dd * d.N + n] = u.holdings[i];
  }
}

// -------------------------------------------------------------- leaderboard
// One workgroup per agent: fixed-shape tree reduction (deterministic) of the
// episode statistics of its envs, in binary64.
__global__ __launch_bounds__(256) void leaderboard_reduce_kernel(int32_t envs_per_agent, EnvState s,
                                                                double *__restrict__ mean, double *__restrict__ var) {
  __shared__ double s1[256], s2[256];
  __shared__ long long sc[256];
  const int g = blockIdx.x, tid = threadIdx.x;
  double a = 0.0, b = 0.0;
  long long c = 0;
  for (int i = tid; i < envs_per_agent; i += 256) {
    const size_t n = (size_t)g * envs_per_agent + i;
    a += s.ep_sum[n];
    b += s.ep_sqsum[n];
    c += s.ep_cnt[n];
  }
  s1[tid] = a;
  s2[tid] = b;
  sc[tid] = c;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if (tid < off) {
      s1[tid] += s1[tid + off];
      s2[tid] += s2[tid + off];
      sc[tid] += sc[tid + off];
    }
    __syncthreads();
  }
  if (tid == 0) {
    if (sc[0] > 0) {
      const double m = s1[0] / (double)sc[0];
      mean[g] = m;
      var[g] = s2[0] / (double)sc[0] - m * m;
    } else {
      mean[g] = -INFINITY;
      var[g] = 0.0;
    }
  }
}

// rank[place] = agent id, best mean first, equal means by lower id.
__global__ void leaderboard_rank_kernel(int32_t P, const double *__restrict__ mean, int32_t *__restrict__ rank) {
  const int g = blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= P) return;
  const double mg = mean[g];
  int place = 0;
  for (int j = 0; j < P; ++j) {
    const double mj = mean[j];
    place += (mj > mg) || (mj == mg && j < g);
  }
  rank[place] = g;
}

}  // namespace

// ------------------------------------------------------------------ launchers

size_t env_step_lds_bytes(const EnvDims &d, int *envs_per_block) {
  const int choices[4] = {64, 16, 4, 1};
  for (int E : choices) {
    if (env_lds(E, d.D) <= 64 * 1024 || E == 1) {
      if (envs_per_block) *envs_per_block = E;
      return env_lds(E, d.D);
    }
  }
  return 0;
}

hipError_t launch_observe(hipStream_t st, const EnvDims &d, const EnvState &s, const float *price, const float *ind,
                          float *obs) {
  const int per_block = kThreads / 64;
  hipLaunchKernelGGL(observe_kernel, dim3((d.N + per_block - 1) / per_block), dim3(kThreads), 0, st, d, s, price, ind,
                     obs);
  return hipGetLastError();
}

hipError_t launch_env_step(hipStream_t st, const EnvDims &d, const EnvState &s, const float *price, const float *ind,
                           const StepIO &io) {
  int E = 0;
  const size_t lds = env_step_lds_bytes(d, &E);
  const dim3 grid((d.N + E - 1) / E), block(kThreads);
  switch (E) {
    case 64: hipLaunchKernelGGL(env_step_kernel<64>, grid, block, lds, st, d, s, price, ind, io); break;
    case 16: hipLaunchKernelGGL(env_step_kernel<16>, grid, block, lds, st, d, s, price, ind, io); break;
    case 4: hipLaunchKernelGGL(env_step_kernel<4>, grid, block, lds, st, d, s, price, ind, io); break;
    default: hipLaunchKernelGGL(env_step_kernel<1>, grid, block, lds, st, d, s, price, ind, io); break;
  }
  return hipGetLastError();
}

hipError_t launch_state_reset(hipStream_t st, const EnvDims &d, const EnvState &s) {
  const size_t n = (size_t)d.N * (size_t)(d.D > 1 ? d.D : 1);
  hipLaunchKernelGGL(state_reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d, s);
  return hipGetLastError();
}

hipError_t launch_state_copy(hipStream_t st, const EnvDims &d, const EnvState &s, const pr_state &user, bool to_user) {
  const size_t n = (size_t)d.N * (size_t)(d.D > 1 ? d.D : 1);
  hipLaunchKernelGGL(state_copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d, s, user,
                     (int)to_user);
  return hipGetLastError();
}

hipError_t launch_leaderboard(hipStream_t st, int32_t N, int32_t P, const EnvState &s, double *scratch_mean,
                              double *score_mean, double *score_var, int32_t *rank) {
  (void)scratch_mean;
  hipLaunchKernelGGL(leaderboard_reduce_kernel, dim3(P), dim3(256), 0, st, N / P, s, score_mean, score_var);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(leaderboard_rank_kernel, dim3((P + 255) / 256), dim3(256), 0, st, P, score_mean, rank);
  return hipGetLastError();
}

}  // namespace pod
