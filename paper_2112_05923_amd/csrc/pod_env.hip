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

__device__ inline RowInfo rows_of(const EnvDims &d, int32_t tau, int32_t start, int32_t n) {
  const int32_t m = d.M == 1 ? 0 : n;
  RowInfo r;
  r.row_now = tau * d.M + m;
  r.row_val = (tau + 1) * d.M + m;
  r.done = (tau + 1 - start == d.H);
  r.row_obs = r.done ? start * d.M + m : r.row_val;
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
// One workgroup of 8 wavefronts steps E consecutive envs.  LDS holds [E][Dp]
// arrays (Dp odd so that the per-env serial loops of the trade pass hit
// distinct banks): wanted shares, eps^2, unit value of the trade (sale proceeds
// or purchase cost per share), executed shares, valuation prices, holdings.
// The kernel is a chain of memory round trips, so each phase requests everything it needs at once:
//  0. cursors, holdings (from their [D][N] layout, lanes across envs), means and noise;
//  1. prices at the cursor and at the valuation row; sample and clamp the action, size the orders (a group of
//     32 or 64 lanes per env row, no index divisions);
//  2. wavefront 0, one lane per env: the serial trade pass in branch-free code (a lane's branch costs all 64
//     a round trip through the scalar unit; what bounds the pass is the dependent chain on the running cash)
//     -- meanwhile wavefront 1 sums the account value before the trades and all others stream the market part
//     of the next observation, several env rows in flight per wavefront, 16 bytes per lane where the rows allow;
//  3. wavefront 0: reward and episode bookkeeping in binary64;
//  4. all lanes: holdings / cash part of the next observation, executed shares, state write-back.
constexpr int kEnvThreads = 512;
typedef float env_f32x4 __attribute__((ext_vector_type(4)));

template <int E>
__global__ __launch_bounds__(kEnvThreads) void env_step_kernel(EnvDims d, EnvState s, const float *__restrict__ price,
                                                              const float *__restrict__ ind, StepIO io) {
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int D = d.D, Dp = D | 1;
  double *s_a0 = reinterpret_cast<double *>(lds_raw);  // [E] account value before the trades
  double *s_a1 = s_a0 + E;                             // [E] account value after them, at the valuation prices
  double *s_rcp = s_a1 + E;                            // [E][Dp] 1 / unit cost of a purchase in binary64, else 0
  int32_t *s_k = reinterpret_cast<int32_t *>(s_rcp + E * Dp);
  float *s_e2 = reinterpret_cast<float *>(s_k + E * Dp);
  float *s_val = s_e2 + E * Dp;
  int32_t *s_q = reinterpret_cast<int32_t *>(s_val + E * Dp);
  float *s_pv = reinterpret_cast<float *>(s_q + E * Dp);
  int32_t *s_h = reinterpret_cast<int32_t *>(s_pv + E * Dp);
  float *s_pn = reinterpret_cast<float *>(s_h + E * Dp);  // prices the trades execute at
  RowInfo *s_row = reinterpret_cast<RowInfo *>(s_pn + E * Dp);
  float *s_cash = reinterpret_cast<float *>(s_row + E);   // cash after the trades, then after the reset
  float *s_e2sum = s_cash + E;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int NWV = kEnvThreads / 64;
  const int n0 = blockIdx.x * E;
  const int ne = min(E, d.N - n0);  // live envs of this tile

  // order slots: a group of GW lanes per env row, G rows per pass, U passes in flight
  constexpr int U = 4;
  const int GW = D <= 32 ? 32 : 64, G = kEnvThreads / GW;
  const int gl = tid & (GW - 1), grp = tid / GW;  // (GW is 32 or 64)

  // -- 0. everything that does not depend on the cursor
  int32_t tau_in = 0, start_in = 0;
  if (tid < ne) {
    tau_in = s.tau[n0 + tid], start_in = s.start[n0 + tid];
    s_row[tid] = rows_of(d, tau_in, start_in, n0 + tid);
  }
  {
    // holdings: up to 8 stocks per wavefront in flight (E <= 64: one env per lane), the rest (D > 64) in a plain loop
    int32_t hreg[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int dd = wave + NWV * i;
      hreg[i] = (dd < D && lane < ne) ? s.h[(size_t)dd * d.N + n0 + lane] : 0;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int dd = wave + NWV * i;
      if (dd < D && lane < ne) s_h[lane * Dp + dd] = hreg[i];
    }
    for (int dd = wave + NWV * 8; dd < D; dd += NWV)
      if (lane < ne) s_h[lane * Dp + dd] = s.h[(size_t)dd * d.N + n0 + lane];
  }
  float mu0[U], eps0[U];  // first column chunk of the first U passes (the whole tile when D <= 64 and E <= U G)
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int e = u * G + grp;
    const bool ok = e < ne && gl < D;
    const size_t g = (size_t)(n0 + (ok ? e : 0)) * D + (ok ? gl : 0);
    mu0[u] = ok ? io.mu[g] : 0.0f;
    eps0[u] = ok ? io.noise[g] : 0.0f;
  }
  // wavefront 0, lane e: the env's scalars, held in registers until the bookkeeping of phase 3 (E <= 64)
  float cash_in = 0.0f;
  double ep_ret = 0.0, ep_sum = 0.0, ep_sqsum = 0.0;
  int32_t ep_cnt = 0;
  if (tid < ne) {
    const int n = n0 + tid;
    cash_in = s.cash[n], ep_ret = s.ep_ret[n], ep_sum = s.ep_sum[n], ep_sqsum = s.ep_sqsum[n], ep_cnt = s.ep_cnt[n];
    s_cash[tid] = cash_in;
  }
  __syncthreads();

  // -- 1a. request the market part of the next observation (it only depends on the cursor): one wavefront per env
  // row, all of a wavefront's rows in flight; stored after the orders are sized
  const int DK = D * d.K;
  const bool vec = (DK & 3) == 0 && (reinterpret_cast<uintptr_t>(ind) & 15u) == 0;
  constexpr int UE = (E + NWV - 1) / NWV;  // env rows per wavefront
  const bool one_pass = D <= 64 && DK <= 256 && vec;
  float m_pr[UE];
  env_f32x4 m_ind[UE];
  if (one_pass) {
#pragma unroll
    for (int u = 0; u < UE; ++u) {
      const int e = wave + u * NWV;
      m_pr[u] = 0.0f;
      m_ind[u] = env_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      if (e < ne) {
        const size_t row = (size_t)s_row[e].row_obs;
        if (lane < D) m_pr[u] = price[row * D + lane];
        if (4 * lane < DK) m_ind[u] = *reinterpret_cast<const env_f32x4 *>(ind + row * DK + 4 * lane);
      }
    }
  }

  // -- 1. prices, then sample and size the orders
  for (int eb = 0; eb < ne; eb += U * G) {
    for (int d0 = 0; d0 < D; d0 += GW) {
      const int dd = d0 + gl;
      float mu[U], eps[U], pn[U], pv[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int e = eb + u * G + grp;
        const bool ok = e < ne && dd < D;
        const RowInfo ri = s_row[ok ? e : 0];
        if (eb == 0 && d0 == 0) {
          mu[u] = mu0[u], eps[u] = eps0[u];
        } else {
          const size_t g = (size_t)(n0 + (ok ? e : 0)) * D + (ok ? dd : 0);
          mu[u] = ok ? io.mu[g] : 0.0f;
          eps[u] = ok ? io.noise[g] : 0.0f;
        }
        pn[u] = ok ? price[(size_t)ri.row_now * D + dd] : 1.0f;
        pv[u] = ok ? price[(size_t)ri.row_val * D + dd] : 1.0f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int e = eb + u * G + grp;
        if (e < ne && dd < D) {
          const int o = e * Dp + dd;
          const float a_raw = mu[u] + d.sigma * eps[u];  // two roundings (contraction is off)
          io.act_raw[(size_t)(n0 + e) * D + dd] = a_raw;
          const float ac = fminf(1.0f, fmaxf(-1.0f, a_raw));
          const int32_t k = (int32_t)truncf(ac * d.hmax);
          const float p = pn[u];
          const int32_t h = s_h[o];
          int32_t q = 0;
          float val = 0.0f;
          double rcp = 0.0;
          if (k < 0) {
            q = min(-k, h);
            s_h[o] = h - q;
            const float gross = p * (float)q;
            val = gross * d.one_minus_c;
            q = -q;
          } else if (k > 0) {
            val = p * d.one_plus_c;
            rcp = 1.0 / (double)val;
          }
          s_rcp[o] = rcp;
          s_k[o] = k;
          s_e2[o] = eps[u] * eps[u];
          s_val[o] = val;
          s_q[o] = q;
          s_pv[o] = pv[u];
          s_pn[o] = p;
        }
      }
    }
  }
  if (one_pass) {
#pragma unroll
    for (int u = 0; u < UE; ++u) {
      const int e = wave + u * NWV;
      if (e < ne) {
        float *o = io.obs_next + (size_t)(n0 + e) * d.S;
        if (lane < D) o[1 + lane] = m_pr[u] * d.s_price;
        if (4 * lane < DK) {
          env_f32x4 t = m_ind[u];
          t[0] *= d.s_ind;
          t[1] *= d.s_ind;
          t[2] *= d.s_ind;
          t[3] *= d.s_ind;
          *reinterpret_cast<env_f32x4 *>(o + 1 + 2 * D + 4 * lane) = t;  // (4-byte aligned is enough for a global store)
        }
      }
    }
  }
  __syncthreads();

  if (wave == 0) {
    // -- 2a. one lane per env: the serial part (Table 1 actions: sell / buy / hold)
    for (int e = lane; e < ne; e += 64) {
      const int o0 = e * Dp;
      float cash = cash_in;  // (e == lane: E <= 64)
      float e2 = 0.0f;
      // Each pass stages a chunk of the lane's row in registers first, so that the LDS reads of a chunk are all in
      // flight together and the dependent chain on `cash` runs on registers only (slots beyond D read as holds).
      // (whole chunks run without bounds checks; the last D % 8 slots one by one)
      constexpr int CH = 8;
      const int Dfull = D & ~(CH - 1);
      auto sell = [&](int32_t k, float v, float sq) {
        e2 += sq;
        cash = k < 0 ? cash + v : cash;  // all sales in stock order
      };
      for (int c0 = 0; c0 < Dfull; c0 += CH) {
        int32_t kk[CH];
        float vv[CH], ee[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) kk[j] = s_k[o0 + c0 + j], vv[j] = s_val[o0 + c0 + j], ee[j] = s_e2[o0 + c0 + j];
#pragma unroll
        for (int j = 0; j < CH; ++j) sell(kk[j], vv[j], ee[j]);
      }
      for (int dd = Dfull; dd < D; ++dd) sell(s_k[o0 + dd], s_val[o0 + dd], s_e2[o0 + dd]);
      // all purchases in stock order, each limited by the cash left:
      //   m = floor(cash / u); q = min(k, max(m, 0)); if (q u > cash) q -= 1; cash -= q u        (binary32)
      // The binary32 quotient comes from one binary64 product with the reciprocal of u prepared by the other lanes:
      // the product is within 2^-52 of cash / u, and a quotient of two binary32 numbers is at least 2^-49 (relative)
      // away from every binary32 rounding boundary it does not hit exactly, so the product rounded to binary32 is
      // the correctly rounded cash / u.  The quotient is never negative (cash is not), so truncation is the floor
      // and needs no clamp at 0; the outlay of one share less, (q - 1) u rounded once, is the fused q u - u (the
      // same real number, one rounding); both candidate balances are formed before the comparison is known.
      // Sales and holds have k = 0 and reciprocal 0: q = 0, outlay 0.
      // (A purchase slot of s_q held 0, any other slot is rewritten with what it held: wavefront 1 reads the sale
      // slots meanwhile.)  s_h keeps the holdings after the sales; purchases are added on the way out.
      auto buy = [&](int32_t k, float u, double r, int32_t q_in, int o) {
        const float kf = (float)max(k, 0);
        const float ratio = (float)((double)cash * r);
        const float q0 = fminf(kf, truncf(ratio));
        const float out_q = q0 * u, out_q1 = fmaf(q0, u, -u);
        const float bal0 = cash - out_q, bal1 = cash - out_q1;
        const bool over = out_q > cash;
        cash = over ? bal1 : bal0;
        s_q[o] = q_in + (int32_t)(over ? q0 - 1.0f : q0);
      };
      for (int c0 = 0; c0 < Dfull; c0 += CH) {
        int32_t kk[CH], qq[CH];
        float uu[CH];
        double rr[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j)
          kk[j] = s_k[o0 + c0 + j], uu[j] = s_val[o0 + c0 + j], rr[j] = s_rcp[o0 + c0 + j], qq[j] = s_q[o0 + c0 + j];
#pragma unroll
        for (int j = 0; j < CH; ++j) buy(kk[j], uu[j], rr[j], qq[j], o0 + c0 + j);
      }
      for (int dd = Dfull; dd < D; ++dd) buy(s_k[o0 + dd], s_val[o0 + dd], s_rcp[o0 + dd], s_q[o0 + dd], o0 + dd);
      double asset1 = (double)cash;
      for (int c0 = 0; c0 < Dfull; c0 += CH) {
        int32_t hh[CH];
        float pp[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) hh[j] = s_h[o0 + c0 + j] + max(s_q[o0 + c0 + j], 0), pp[j] = s_pv[o0 + c0 + j];
#pragma unroll
        for (int j = 0; j < CH; ++j) asset1 += (double)hh[j] * (double)pp[j];
      }
      for (int dd = Dfull; dd < D; ++dd) asset1 += (double)(s_h[o0 + dd] + max(s_q[o0 + dd], 0)) * (double)s_pv[o0 + dd];
      s_a1[e] = asset1;
      cash_in = cash;  // now: cash after the trades
      s_e2sum[e] = e2;
    }
  } else {
    if (wave == 1) {
      // account value before the trades: cash + sum h p in stock order, binary64 (lane per env)
      for (int e = lane; e < ne; e += 64) {
        double v = (double)s_cash[e];
        for (int dd = 0; dd < D; ++dd) {
          // holdings before the sales = holdings after them + what the sale pass took (the slots of sales are
          // stable while wavefront 0 books the purchases)
          const int32_t k = s_k[e * Dp + dd];
          const int32_t h0 = s_h[e * Dp + dd] + (k < 0 ? -s_q[e * Dp + dd] : 0);
          v += (double)h0 * (double)s_pn[e * Dp + dd];
        }
        s_a0[e] = v;
      }
    }
    // -- 2b. wide rows: stream the market part of the next observation here, UB env rows in flight per wavefront
    constexpr int UB = 5;
    for (int eb = wave - 1; eb < ne && !one_pass; eb += UB * (NWV - 1)) {
      for (int j0 = 0; j0 < D; j0 += 64) {
        float pr[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int e = eb + u * (NWV - 1);
          const bool ok = e < ne && j0 + lane < D;
          pr[u] = ok ? price[(size_t)s_row[e].row_obs * D + j0 + lane] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int e = eb + u * (NWV - 1);
          if (e < ne && j0 + lane < D) io.obs_next[(size_t)(n0 + e) * d.S + 1 + j0 + lane] = pr[u] * d.s_price;
        }
      }
      if (vec) {
        for (int j0 = 0; j0 < DK; j0 += 256) {
          const int j = j0 + 4 * lane;
          env_f32x4 v[UB];
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int e = eb + u * (NWV - 1);
            if (e < ne && j < DK)
              v[u] = *reinterpret_cast<const env_f32x4 *>(ind + (size_t)s_row[e].row_obs * DK + j);
          }
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int e = eb + u * (NWV - 1);
            if (e < ne && j < DK) {
              env_f32x4 t = v[u];
              t[0] *= d.s_ind;
              t[1] *= d.s_ind;
              t[2] *= d.s_ind;
              t[3] *= d.s_ind;
              // (4-byte aligned is enough for a global store)
              *reinterpret_cast<env_f32x4 *>(io.obs_next + (size_t)(n0 + e) * d.S + 1 + 2 * D + j) = t;
            }
          }
        }
      } else {
        for (int j0 = 0; j0 < DK; j0 += 64) {
          const int j = j0 + lane;
          float v[UB];
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int e = eb + u * (NWV - 1);
            v[u] = (e < ne && j < DK) ? ind[(size_t)s_row[e].row_obs * DK + j] : 0.0f;
          }
#pragma unroll
          for (int u = 0; u < UB; ++u) {
            const int e = eb + u * (NWV - 1);
            if (e < ne && j < DK) io.obs_next[(size_t)(n0 + e) * d.S + 1 + 2 * D + j] = v[u] * d.s_ind;
          }
        }
      }
    }
  }
  __syncthreads();

  // -- 3. reward and episode bookkeeping (binary64), reset of the envs whose episode ended
  if (tid < ne) {
    const int e = tid, n = n0 + e;
    const double r = (s_a1[e] - s_a0[e]) * (double)d.rho;
    const RowInfo ri = s_row[e];
    float cash = cash_in;
    double ep = ep_ret + r;
    if (ri.done) {
      s.ep_sum[n] = ep_sum + ep;
      s.ep_sqsum[n] = ep_sqsum + ep * ep;
      s.ep_cnt[n] = ep_cnt + 1;
      ep = 0.0;
      cash = d.cash0;
    }
    s.ep_ret[n] = ep;
    s.cash[n] = cash;
    s.tau[n] = ri.done ? start_in : tau_in + 1;
    io.obs_next[(size_t)n * d.S] = cash * d.s_cash;
    io.reward[n] = (float)r;
    io.done[n] = (uint8_t)ri.done;
    if (io.logp) io.logp[n] = fmaf(-0.5f, s_e2sum[e], d.logp_const);
  }

  // -- 4. write back what the trade pass produced
  // holdings after the step: after the sales + purchases, none after a reset
  for (int e = wave; e < ne; e += NWV) {
    const size_t g0 = (size_t)(n0 + e) * D;
    const bool dn = s_row[e].done;
    for (int dd = lane; dd < D; dd += 64) {
      const int32_t q = s_q[e * Dp + dd];
      const int32_t h = dn ? 0 : s_h[e * Dp + dd] + max(q, 0);
      io.obs_next[(size_t)(n0 + e) * d.S + 1 + D + dd] = (float)h * d.s_hold;
      if (io.shares) io.shares[g0 + dd] = q;
    }
  }
  for (int dd = wave; dd < D; dd += NWV)
    for (int e = lane; e < ne; e += 64) {
      const int o = e * Dp + dd;
      s.h[(size_t)dd * d.N + n0 + e] = s_row[e].done ? 0 : s_h[o] + max(s_q[o], 0);
    }
}

size_t env_lds(int E, int D) {
  const int Dp = D | 1;
  return (size_t)9 * E * Dp * 4 + (size_t)E * (sizeof(RowInfo) + 2 * sizeof(float) + 2 * sizeof(double));
}

// ------------------------------------------------------------ state plumbing
// *bad = 1 unless every env's episode rows start .. start + H lie inside a table of `rows` rows.
__global__ __launch_bounds__(256) void check_starts_kernel(int32_t N, int32_t H, int32_t rows,
                                                           const int32_t *__restrict__ start, int32_t *bad) {
  int flag = 0;
  for (int i = threadIdx.x; i < N; i += 256) {
    const int32_t s = start[i];
    flag |= (s < 0 || s > rows - 1 - H);
  }
  flag = __syncthreads_or(flag);
  if (threadIdx.x == 0) *bad = flag;
}

__global__ void state_reset_kernel(EnvDims d, EnvState s) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (size_t)d.N) {
    s.cash[i] = d.cash0;
    s.tau[i] = s.start[i];
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

// LDS per workgroup up to which a tile size is taken: two workgroups per compute unit still fit.
constexpr size_t kEnvLdsBudget = 78 * 1024;

size_t env_step_lds_bytes(const EnvDims &d, int *envs_per_block) {
  const int choices[4] = {32, 16, 4, 1};  // (32-env tiles: two workgroups per compute unit overlap their round trips; measured 3 % ahead of 64)
  for (int E : choices) {
    if (env_lds(E, d.D) <= kEnvLdsBudget || E == 1) {
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
  const dim3 grid((d.N + E - 1) / E), block(kEnvThreads);
  if (lds > kMaxLdsBytes) return hipErrorInvalidValue;
  hipError_t e = hipSuccess;
  switch (E) {
    case 32:
      if ((e = allow_full_lds<env_step_kernel<32>>()) != hipSuccess) return e;
      hipLaunchKernelGGL(env_step_kernel<32>, grid, block, lds, st, d, s, price, ind, io);
      break;
    case 16:
      if ((e = allow_full_lds<env_step_kernel<16>>()) != hipSuccess) return e;
      hipLaunchKernelGGL(env_step_kernel<16>, grid, block, lds, st, d, s, price, ind, io);
      break;
    case 4:
      if ((e = allow_full_lds<env_step_kernel<4>>()) != hipSuccess) return e;
      hipLaunchKernelGGL(env_step_kernel<4>, grid, block, lds, st, d, s, price, ind, io);
      break;
    default:
      if ((e = allow_full_lds<env_step_kernel<1>>()) != hipSuccess) return e;
      hipLaunchKernelGGL(env_step_kernel<1>, grid, block, lds, st, d, s, price, ind, io);
      break;
  }
  return hipGetLastError();
}

hipError_t launch_check_starts(hipStream_t st, int32_t N, int32_t H, int32_t rows, const int32_t *start, int32_t *bad) {
  hipLaunchKernelGGL(check_starts_kernel, dim3(1), dim3(256), 0, st, N, H, rows, start, bad);
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
