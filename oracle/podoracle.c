/*
 * podoracle.c -- plain, slow CPU statement of what the pod rollout computes.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or
 * import this file; it exists so that tests, the smoke check and the bench's
 * CPU-baseline leg have an independent result to compare the HIP kernels with.
 * It shares no code, header, table or helper with the HIP sources.
 *
 * What it follows.  The paper states the computation only in words: a worker
 * produces batches of transitions from an actor acting in a batched
 * environment of independent sub-environments (Sec. 4.2 "Worker"), the data are
 * tensors in contiguous GPU memory (Sec. 4.3 "Cloud-oriented optimizations"),
 * and the stock-trading task has state {balance, shares, close prices,
 * technical indicators}, actions {buy, sell, hold} and reward "change of
 * account value" (Table 1, Sec. 5.3; initial capital 1e6 and a proportional
 * transaction cost in the caption of Fig. 6).  All experiments use PPO
 * (Sec. 5.2), which implies a Gaussian policy and generalised advantage
 * estimation.  Every concrete rule below (trade order, truncation, execution
 * and valuation price, reset, GAE termination handling) is a reading of those
 * passages; the readings are listed in the design notes of the repository.
 *
 * Arithmetic.  Decisions that produce integers (share counts, cursors) are
 * taken in IEEE binary32 with one rounding per operation in a fixed order, so
 * another implementation can reproduce them bit for bit.  Everything that is a
 * real-valued result (network outputs, asset value, reward, log-probability,
 * GAE, leaderboard moments) is evaluated in binary64.
 *
 * Pins (tests/test_oracle_*.py): zero-action and forced-liquidation closed
 * forms, self-financing identity, cash/holdings non-negativity, order-of-trade
 * cases, exact-rational brute force on a 1-env 2-stock 3-step grid; numpy
 * matmul + tanh for the MLP; library bf16 rounding and hand-built ties for
 * the bf16 emulation; closed forms and the O(T^2) direct sum for GAE; numpy
 * mean/var/stable argsort for the leaderboard; a hand-computed curve, geometric
 * closed forms, numpy std / maximum.accumulate / prod and the rollout's own
 * rewards for the trading metrics of Sec. 5.3 (whose annualisation period,
 * risk-free rate and deviation estimator the paper leaves open: parameters and
 * the sample estimator here); the per-agent network selection of a free-running
 * population by equality with one single-agent run per agent and the numpy
 * matmul chain on that agent's weights.  The whole free-running rollout
 * has no printed trajectory in the paper to compare with: parity unpinned for
 * the composition, pinned stage by stage.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Constants of the trading task (Table 1 / Fig. 6 caption) and of the
 * observation scaling.  Plain data, filled by the caller. */
typedef struct orc_cfg {
  int32_t n_stocks;     /* D */
  int32_t n_ind;        /* K indicators per stock */
  int32_t horizon;      /* H: an episode ends H steps after its start row */
  float cash0;          /* initial capital */
  float hmax;           /* largest trade per stock and step, in shares */
  float cost;           /* proportional transaction cost c */
  float sigma;          /* fixed standard deviation of the Gaussian policy */
  float reward_scale;   /* rho */
  float obs_scale[4];   /* cash, price, holdings, indicator */
} orc_cfg;

/* flag bits reported per (t, env, stock) */
#define ORC_FLAG_TRUNC 1u /* a*hmax within a few ulp of an integer */
#define ORC_FLAG_FLOOR 2u /* cash/u within a few ulp of an integer */
#define ORC_FLAG_GUARD 4u /* the q -= 1 guard of the buy rule fired */

static int state_dim(const orc_cfg *c) { return 1 + 2 * c->n_stocks + c->n_stocks * c->n_ind; }

/* ------------------------------------------------------------------ bf16 -- */

/* Round a binary32 value to the nearest bfloat16 (8 significand bits), ties
 * to even, returned as binary32.  NaN stays NaN. */
float orc_bf16_round(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu)) {
    u |= 0x00400000u; /* quiet NaN, keep sign */
    u &= 0xffff0000u;
  } else {
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
  }
  memcpy(&x, &u, 4);
  return x;
}

void orc_bf16_round_array(const float *in, float *out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_round(in[i]);
}

/* ------------------------------------------------------------------- MLP -- */

/* One affine layer for one row: out[j] = b[j] + sum_i in[i] * W[i][j], inputs
 * taken in ascending order of i, accumulated in binary64. */
static void affine(int n_in, int n_out, const double *in, const float *W, const float *b, double *out) {
  for (int j = 0; j < n_out; ++j) out[j] = 0.0;
  for (int i = 0; i < n_in; ++i) {
    const double xi = in[i];
    const float *w = W + (int64_t)i * n_out;
    for (int j = 0; j < n_out; ++j) out[j] += xi * (double)w[j];
  }
  for (int j = 0; j < n_out; ++j) out[j] += (double)b[j];
}

/* Three-layer perceptron on `rows` input rows (actor: tanh on the output too;
 * critic: linear scalar output).  X is [rows, ldx] with the first S entries of
 * each row used; W1 [S,Hd], W2 [Hd,Hd], W3 [Hd,O] row-major, biases [out].
 * bf16 != 0: inputs and hidden activations are rounded to bfloat16 before each
 * layer; the weights passed in must then already be bfloat16-valued (see
 * orc_bf16_round_array) -- products of two bfloat16 values are exact in
 * binary64, so the result is the true value of the rounded-operand network.
 * out is [rows, O] in binary64. */
void orc_mlp(int64_t rows, int S, int Hd, int O, const float *X, int64_t ldx, const float *W1, const float *b1,
             const float *W2, const float *b2, const float *W3, const float *b3, int out_tanh, int bf16, double *out) {
  int widest = S > Hd ? S : Hd;
  double *a = (double *)malloc(sizeof(double) * (size_t)widest);
  double *z = (double *)malloc(sizeof(double) * (size_t)(Hd > O ? Hd : O));
  for (int64_t r = 0; r < rows; ++r) {
    const float *x = X + r * ldx;
    for (int i = 0; i < S; ++i) a[i] = bf16 ? (double)orc_bf16_round(x[i]) : (double)x[i];
    affine(S, Hd, a, W1, b1, z);
    for (int j = 0; j < Hd; ++j) {
      double h = tanh(z[j]);
      a[j] = bf16 ? (double)orc_bf16_round((float)h) : h;
    }
    affine(Hd, Hd, a, W2, b2, z);
    for (int j = 0; j < Hd; ++j) {
      double h = tanh(z[j]);
      a[j] = bf16 ? (double)orc_bf16_round((float)h) : h;
    }
    affine(Hd, O, a, W3, b3, z);
    for (int j = 0; j < O; ++j) out[r * O + j] = out_tanh ? tanh(z[j]) : z[j];
  }
  free(a);
  free(z);
}

/* ----------------------------------------------------------- environment -- */

/* Observation of one env (Table 1 state space): [cash, prices, holdings,
 * indicators (stock-major)], each block scaled by its power-of-two factor. */
void orc_observe(const orc_cfg *c, float cash, const int32_t *h, const float *p, const float *ind, float *obs) {
  const int D = c->n_stocks, K = c->n_ind;
  obs[0] = cash * c->obs_scale[0];
  for (int d = 0; d < D; ++d) obs[1 + d] = p[d] * c->obs_scale[1];
  for (int d = 0; d < D; ++d) obs[1 + D + d] = (float)h[d] * c->obs_scale[2];
  for (int i = 0; i < D * K; ++i) obs[1 + 2 * D + i] = ind[i] * c->obs_scale[3];
}

/* Gaussian policy sample with externally drawn standard-normal noise:
 * a_raw = mu + sigma * eps (two binary32 roundings), and the log-density of
 * a_raw under N(mu, sigma^2 I), which depends on eps only. */
void orc_sample(int D, float sigma, const float *mu, const float *eps, float *a_raw, double *logp) {
  const double half_log_2pi = 0.91893853320467274178;
  double lp = 0.0;
  for (int d = 0; d < D; ++d) {
    volatile float se = sigma * eps[d];
    volatile float a = mu[d] + se;
    a_raw[d] = a;
    lp += -0.5 * (double)eps[d] * (double)eps[d] - log((double)sigma) - half_log_2pi;
  }
  *logp = lp;
}

/* x lies within a few binary32 ulp of an integer without being one. */
static int near_integer(double x) {
  double ax = fabs(x);
  double tol = 8.0 * ldexp(1.0, -24) * (ax > 1.0 ? ax : 1.0);
  double gap = fabs(x - nearbyint(x));
  return gap != 0.0 && gap <= tol;
}

/* Trade execution of one env at prices p (buy / sell / hold of Table 1):
 * wanted shares k_d = trunc(clamp(a_d) * hmax); first every sale in ascending
 * stock order (limited by the holding), then every purchase in ascending stock
 * order (limited by the cash left, cost included).  binary32 throughout, one
 * rounding per operation.  shares[d] receives the signed executed quantity,
 * flags[d] (optional) the ORC_FLAG_* bits. */
void orc_trade(const orc_cfg *c, float *cash_io, int32_t *h, const float *a_raw, const float *p, int32_t *shares,
               uint8_t *flags) {
  const int D = c->n_stocks;
  volatile float cash = *cash_io;
  volatile float one_minus_c = 1.0f - c->cost;
  volatile float one_plus_c = 1.0f + c->cost;
  int32_t *k = (int32_t *)malloc(sizeof(int32_t) * (size_t)D);
  for (int d = 0; d < D; ++d) {
    float a = a_raw[d];
    a = a < -1.0f ? -1.0f : a;
    a = a > 1.0f ? 1.0f : a;
    volatile float x = a * c->hmax;
    k[d] = (int32_t)truncf(x);
    shares[d] = 0;
    if (flags) flags[d] = near_integer((double)a * (double)c->hmax) ? ORC_FLAG_TRUNC : 0;
  }
  for (int d = 0; d < D; ++d) {
    if (k[d] >= 0) continue;
    int32_t q = -k[d] < h[d] ? -k[d] : h[d];
    h[d] -= q;
    volatile float gross = p[d] * (float)q;
    volatile float net = gross * one_minus_c;
    cash = cash + net;
    shares[d] = -q;
  }
  for (int d = 0; d < D; ++d) {
    if (k[d] <= 0) continue;
    volatile float u = p[d] * one_plus_c;
    volatile float ratio = cash / u;
    int32_t m = (int32_t)floorf(ratio);
    if (m < 0) m = 0;
    int32_t q = k[d] < m ? k[d] : m;
    volatile float outlay = (float)q * u;
    if (flags && near_integer((double)cash / (double)u) && m <= k[d] + 1) flags[d] |= ORC_FLAG_FLOOR;
    if (outlay > cash) {
      q -= 1;
      outlay = (float)q * u;
      if (flags) flags[d] |= ORC_FLAG_GUARD;
    }
    h[d] += q;
    cash = cash - outlay;
    shares[d] = q;
  }
  free(k);
  *cash_io = cash;
}

/* Account value in binary64: cash + sum_d h_d * p_d. */
double orc_asset(int D, float cash, const int32_t *h, const float *p) {
  double v = (double)cash;
  for (int d = 0; d < D; ++d) v += (double)h[d] * (double)p[d];
  return v;
}

/* Per-env persistent state.  Arrays of length N (h: [N, D]). */
typedef struct orc_state {
  float *cash;
  int32_t *h;
  int32_t *tau;
  double *asset;
  double *ep_ret, *ep_sum, *ep_sqsum;
  int32_t *ep_cnt;
  int32_t *start; /* table row every episode of the env begins at (replay of one historical table from per-env
                     offsets, Sec. 5.3 data; 0 everywhere is the plain case).  Set by the caller before
                     orc_reset_state and kept by it. */
} orc_state;

void orc_reset_state(const orc_cfg *c, int64_t N, orc_state *s) {
  for (int64_t n = 0; n < N; ++n) {
    s->cash[n] = c->cash0;
    s->tau[n] = s->start[n];
    s->asset[n] = (double)c->cash0;
    s->ep_ret[n] = s->ep_sum[n] = s->ep_sqsum[n] = 0.0;
    s->ep_cnt[n] = 0;
    for (int d = 0; d < c->n_stocks; ++d) s->h[n * c->n_stocks + d] = 0;
  }
}

/* One transition of env n given its raw action: trade at the prices of the
 * current cursor, advance the cursor, value the portfolio at the new prices,
 * reward = rho * (change of account value) (Table 1), episode end after H
 * steps from the env's start row, then bookkeeping of the finished episode's
 * return and reset to the initial capital with no shares at the start row.  p_now / p_next are the market
 * rows at the cursor before / after the advance.  Returns the reward. */
double orc_env_step(const orc_cfg *c, int64_t n, orc_state *s, const float *a_raw, const float *p_now,
                    const float *p_next, int32_t *shares, uint8_t *flags, uint8_t *done_out) {
  const int D = c->n_stocks;
  int32_t *h = s->h + n * D;
  orc_trade(c, &s->cash[n], h, a_raw, p_now, shares, flags);
  s->tau[n] += 1;
  double asset_new = orc_asset(D, s->cash[n], h, p_next);
  double r = (asset_new - s->asset[n]) * (double)c->reward_scale;
  s->asset[n] = asset_new;
  s->ep_ret[n] += r;
  uint8_t done = (uint8_t)(s->tau[n] - s->start[n] == c->horizon);
  if (done) {
    s->ep_sum[n] += s->ep_ret[n];
    s->ep_sqsum[n] += s->ep_ret[n] * s->ep_ret[n];
    s->ep_cnt[n] += 1;
    s->ep_ret[n] = 0.0;
    s->cash[n] = c->cash0;
    for (int d = 0; d < D; ++d) h[d] = 0;
    s->tau[n] = s->start[n];
    s->asset[n] = (double)c->cash0;
  }
  *done_out = done;
  return r;
}

/* The worker's rollout (Sec. 4.2): N independent sub-environments, T steps.
 *
 *   market:  price [H+1, M, D], ind [H+1, M, D*K]; env n reads path market_of[n]
 *   nets:    per-agent weights, agent_of[n] selects the agent of env n;
 *            layouts as in orc_mlp with a leading agent axis; critic pointers
 *            may be NULL (then value is not written)
 *   noise:   [T, N, D] standard normal
 *   mu_forced: NULL, or [T, N, D] policy means to use instead of the actor
 *   outputs (any may be NULL): obs [T+1,N,S] f32, mu [T,N,D] f64, act_raw
 *            [T,N,D] f32, logp [T,N] f64, reward [T,N] f64, done [T,N] u8,
 *            value [T+1,N] f64, shares [T,N,D] i32, flags [T,N,D] u8
 * State is read and updated in place, so consecutive calls continue episodes. */
int orc_rollout(const orc_cfg *c, int64_t N, int M, int Hd, int bf16, int T, const int32_t *agent_of,
                const int32_t *market_of, const float *price, const float *ind, const float *const *actor,
                const float *const *critic, const float *noise, const float *mu_forced, orc_state *s, float *obs_out,
                double *mu_out, float *act_out, double *logp_out, double *reward_out, uint8_t *done_out,
                double *value_out, int32_t *shares_out, uint8_t *flags_out) {
  const int D = c->n_stocks, K = c->n_ind, S = state_dim(c);
  const int64_t w1 = (int64_t)S * Hd, w2 = (int64_t)Hd * Hd, w3a = (int64_t)Hd * D, w3c = Hd;
  float *obs = (float *)malloc(sizeof(float) * (size_t)S);
  float *mu32 = (float *)malloc(sizeof(float) * (size_t)D);
  float *a_raw = (float *)malloc(sizeof(float) * (size_t)D);
  double *mu = (double *)malloc(sizeof(double) * (size_t)D);
  int32_t *shares = (int32_t *)malloc(sizeof(int32_t) * (size_t)D);
  uint8_t *flags = (uint8_t *)malloc((size_t)D);
  if (!obs || !mu32 || !a_raw || !mu || !shares || !flags) return -1;
  for (int64_t n = 0; n < N; ++n) {
    const int g = agent_of[n];
    const int64_t m = market_of[n];
    for (int t = 0; t <= T; ++t) {
      const int32_t tau = s->tau[n];
      const float *p_now = price + ((int64_t)tau * M + m) * D;
      const float *i_now = ind + ((int64_t)tau * M + m) * D * K;
      orc_observe(c, s->cash[n], s->h + n * D, p_now, i_now, obs);
      if (obs_out) memcpy(obs_out + ((int64_t)t * N + n) * S, obs, sizeof(float) * (size_t)S);
      if (critic && value_out) {
        double v;
        orc_mlp(1, S, Hd, 1, obs, S, critic[0] + g * w1, critic[1] + (int64_t)g * Hd, critic[2] + g * w2,
                critic[3] + (int64_t)g * Hd, critic[4] + g * w3c, critic[5] + g, 0, bf16, &v);
        value_out[(int64_t)t * N + n] = v;
      }
      if (t == T) break;
      const int64_t tn = (int64_t)t * N + n;
      if (mu_forced) {
        for (int d = 0; d < D; ++d) mu[d] = (double)mu_forced[tn * D + d];
      } else {
        orc_mlp(1, S, Hd, D, obs, S, actor[0] + g * w1, actor[1] + (int64_t)g * Hd, actor[2] + g * w2,
                actor[3] + (int64_t)g * Hd, actor[4] + g * w3a, actor[5] + (int64_t)g * D, 1, bf16, mu);
      }
      for (int d = 0; d < D; ++d) mu32[d] = (float)mu[d];
      double lp;
      orc_sample(D, c->sigma, mu32, noise + tn * D, a_raw, &lp);
      const float *p_next = price + ((int64_t)(tau + 1) * M + m) * D;
      uint8_t done;
      double r = orc_env_step(c, n, s, a_raw, p_now, p_next, shares, flags, &done);
      if (mu_out) memcpy(mu_out + tn * D, mu, sizeof(double) * (size_t)D);
      if (act_out) memcpy(act_out + tn * D, a_raw, sizeof(float) * (size_t)D);
      if (logp_out) logp_out[tn] = lp;
      if (reward_out) reward_out[tn] = r;
      if (done_out) done_out[tn] = done;
      if (shares_out) memcpy(shares_out + tn * D, shares, sizeof(int32_t) * (size_t)D);
      if (flags_out) memcpy(flags_out + tn * D, flags, (size_t)D);
    }
  }
  free(obs);
  free(mu32);
  free(a_raw);
  free(mu);
  free(shares);
  free(flags);
  return 0;
}

/* ------------------------------------------------------------------- GAE -- */

/* Generalised advantage estimation per env, backwards in time (implied by the
 * use of PPO, Sec. 5.2): with nd_t = 1 - done_t,
 *   delta_t = r_t + gamma nd_t V_{t+1} - V_t,
 *   A_t = delta_t + gamma lambda nd_t A_{t+1},  A_T = 0,   R_t = A_t + V_t.
 * An episode end is a termination: nothing is bootstrapped through it.
 * reward [T,N], value [T+1,N], done [T,N]; adv, ret [T,N]. */
void orc_gae(int T, int64_t N, const double *reward, const double *value, const uint8_t *done, double gamma,
             double lambda, double *adv, double *ret) {
  for (int64_t n = 0; n < N; ++n) {
    double a_next = 0.0;
    for (int t = T - 1; t >= 0; --t) {
      const int64_t i = (int64_t)t * N + n;
      const double nd = 1.0 - (double)(done[i] != 0);
      const double delta = reward[i] + gamma * nd * value[i + N] - value[i];
      const double a = delta + gamma * lambda * nd * a_next;
      adv[i] = a;
      ret[i] = a + value[i];
      a_next = a;
    }
  }
}

/* ----------------------------------------------------------- leaderboard -- */

/* Score of each agent = mean (and population variance) of the returns of the
 * episodes its envs completed (Sec. 4.1 leaderboard; Sec. 4.2 evaluator: mean
 * and variance of the episodic reward).  Agents with no finished episode score
 * -inf with variance 0.  rank[i] = id of the agent in place i, best first,
 * equal means ordered by lower agent id.  Env n belongs to agent_of[n]. */
void orc_leaderboard(int P, int64_t N, const int32_t *agent_of, const double *ep_sum, const double *ep_sqsum,
                     const int32_t *ep_cnt, double *mean, double *var, int32_t *rank) {
  double *s1 = (double *)calloc((size_t)P, sizeof(double));
  double *s2 = (double *)calloc((size_t)P, sizeof(double));
  int64_t *cnt = (int64_t *)calloc((size_t)P, sizeof(int64_t));
  for (int64_t n = 0; n < N; ++n) {
    s1[agent_of[n]] += ep_sum[n];
    s2[agent_of[n]] += ep_sqsum[n];
    cnt[agent_of[n]] += ep_cnt[n];
  }
  for (int g = 0; g < P; ++g) {
    if (cnt[g] > 0) {
      mean[g] = s1[g] / (double)cnt[g];
      var[g] = s2[g] / (double)cnt[g] - mean[g] * mean[g];
    } else {
      mean[g] = -INFINITY;
      var[g] = 0.0;
    }
    rank[g] = g;
  }
  /* stable insertion sort, descending mean */
  for (int i = 1; i < P; ++i) {
    int32_t id = rank[i];
    int j = i - 1;
    while (j >= 0 && mean[rank[j]] < mean[id]) {
      rank[j + 1] = rank[j];
      --j;
    }
    rank[j + 1] = id;
  }
  free(s1);
  free(s2);
  free(cnt);
}

/* ------------------------------------------------------- trading metrics -- */

/* Account-value curve of each env decoded from a recorded observation buffer
 * (state layout of Table 1: [cash, prices, holdings, indicators] times the
 * power-of-two observation scales, which divide out exactly):
 *   V_t = cash_t + sum_d h_{t,d} p_{t,d},  summed in stock order, binary64.
 * The curve of env n covers the first episode in the buffer: t = 0 .. L_n with
 * L_n = the first t whose done flag is set (obs[t+1] is then a reset
 * observation and not part of the episode), or T when none is.
 * obs [T+1, N, S], done [T, N]; value [T+1, N] (entries beyond L_n are 0), len [N]. */
void orc_asset_curve(int T, int64_t N, int D, int S, const float *obs, const uint8_t *done, const float *obs_scale,
                     double *value, int32_t *len) {
  for (int64_t n = 0; n < N; ++n) {
    int L = T;
    for (int t = 0; t < T; ++t)
      if (done[(int64_t)t * N + n]) {
        L = t;
        break;
      }
    len[n] = L;
    for (int t = 0; t <= T; ++t) {
      double v = 0.0;
      if (t <= L) {
        const float *o = obs + ((int64_t)t * N + n) * S;
        v = (double)o[0] / (double)obs_scale[0];
        for (int d = 0; d < D; ++d)
          v += ((double)o[1 + D + d] / (double)obs_scale[2]) * ((double)o[1 + d] / (double)obs_scale[1]);
      }
      value[(int64_t)t * N + n] = v;
    }
  }
}

/* The five trading-performance figures of Sec. 5.3 ("Performance metrics") for one value curve V_0 .. V_L,
 * with P periods per year and an annual risk-free rate rf; per-period simple returns r_t = V_{t+1} / V_t - 1:
 *   out[0] cumulative return   (V_L - V_0) / V_0
 *   out[1] annual return       (V_L / V_0)^(P / L) - 1                      (geometric average, yearly)
 *   out[2] annual volatility   sqrt(P) * sample standard deviation of r     (0 when L < 2)
 *   out[3] maximum drawdown    max_t (1 - V_t / max_{s <= t} V_s)           (>= 0)
 *   out[4] Sharpe ratio        sqrt(P) * (mean(r) - rf / P) / std(r)        (0 when std(r) = 0)
 *   out[5] Calmar ratio        annual return / maximum drawdown             (0 when the drawdown is 0)
 * L = 0 (no step observed) gives all zeros. */
void orc_metrics_curve(int L, const double *V, double periods_per_year, double rf, double *out) {
  for (int i = 0; i < 6; ++i) out[i] = 0.0;
  if (L < 1) return;
  out[0] = (V[L] - V[0]) / V[0];
  out[1] = pow(V[L] / V[0], periods_per_year / (double)L) - 1.0;
  double mean = 0.0;
  for (int t = 0; t < L; ++t) mean += V[t + 1] / V[t] - 1.0;
  mean /= (double)L;
  double sd = 0.0;
  if (L >= 2) {
    double ss = 0.0;
    for (int t = 0; t < L; ++t) {
      const double dv = (V[t + 1] / V[t] - 1.0) - mean;
      ss += dv * dv;
    }
    sd = sqrt(ss / (double)(L - 1));
  }
  out[2] = sqrt(periods_per_year) * sd;
  double peak = V[0], mdd = 0.0;
  for (int t = 0; t <= L; ++t) {
    if (V[t] > peak) peak = V[t];
    const double dd = 1.0 - V[t] / peak;
    if (dd > mdd) mdd = dd;
  }
  out[3] = mdd;
  out[4] = sd > 0.0 ? sqrt(periods_per_year) * (mean - rf / periods_per_year) / sd : 0.0;
  out[5] = mdd > 0.0 ? out[1] / mdd : 0.0;
}

/* All envs: metrics [6, N] from value [T+1, N] and len [N] (as written by orc_asset_curve). */
void orc_metrics(int T, int64_t N, const double *value, const int32_t *len, double periods_per_year, double rf,
                 double *metrics) {
  double *V = (double *)malloc((size_t)(T + 1) * sizeof(double));
  for (int64_t n = 0; n < N; ++n) {
    for (int t = 0; t <= T; ++t) V[t] = value[(int64_t)t * N + n];
    double out[6];
    orc_metrics_curve(len[n], V, periods_per_year, rf, out);
    for (int i = 0; i < 6; ++i) metrics[(int64_t)i * N + n] = out[i];
  }
  free(V);
}

/* ------------------------------------------------- population generator -- */

/* Generator / updater step on a population held in one parameter block
 * (Sec. 4.1: the leaderboard records the candidate agents with high
 * performance; the generator produces the training files of a new pod from a
 * candidate and "may perform a mutation" to increase diversity).
 * params [P, count]: one row per agent.  rank [P]: agent ids, best first.
 * The first `keep` agents of rank are the candidates and stay as they are;
 * agent rank[j], j >= keep, becomes candidate rank[(j - keep) % keep] plus
 * sigma * noise[rank[j]], each operation rounded to binary32:
 *   child = fl32(parent + fl32(sigma * z)). */
void orc_population_refill(int P, int64_t count, const int32_t *rank, int keep, float sigma, const float *noise,
                           float *params) {
  for (int j = keep; j < P; ++j) {
    const float *parent = params + (int64_t)rank[(j - keep) % keep] * count;
    float *child = params + (int64_t)rank[j] * count;
    const float *z = noise ? noise + (int64_t)rank[j] * count : NULL;
    for (int64_t i = 0; i < count; ++i) {
      volatile float step = z ? sigma * z[i] : 0.0f;
      volatile float v = parent[i] + step;
      child[i] = v;
    }
  }
}

/* ------------------------------------------------------ PPO learner step -- */

/* One minibatch of the learner (Sec. 4.2 "Learner": fetch a batch of transitions, train the networks; Sec. 5.2:
 * PPO, batch size 1024, learning rate 1e-3).  The paper points to PPO without writing it out; this is the
 * clipped-surrogate objective with a fixed-deviation Gaussian policy, everything in binary64:
 *   mu = actor(obs) (tanh after every layer), V = critic(obs) (linear output)
 *   logp = sum_d -(a_d - mu_d)^2 / (2 sigma^2) - D ln sigma - D/2 ln(2 pi),   ratio = exp(logp - logp_old)
 *   L_pi = -(1/B) sum_b min(ratio A, clip(ratio, 1 - eps, 1 + eps) A)
 *   L_v  = (1/B) sum_b (V - R)^2 / 2,          L = L_pi + c_v L_v
 * A sample's surrogate passes gradient when ratio A <= clip(ratio) A (inside the clip range, or outside it on
 * the side the minimum does not cut).
 * Weights [in, out] row-major, fp32 inputs; gradients of L w.r.t. the 6 + 6 tensors in binary64, same layouts.
 * stats[0..3] = L_pi, L_v, fraction of samples whose surrogate is cut, mean ratio.
 * margin[b] (optional) = distance of ratio from the nearer clip bound, for harnesses that want to tell a flipped
 * min() from an error. */
static void orc_dense_fwd(int in, int out, const double *x, const float *W, const float *b, int act, double *y) {
  for (int o = 0; o < out; ++o) {
    double acc = (double)b[o];
    for (int i = 0; i < in; ++i) acc += x[i] * (double)W[(size_t)i * out + o];
    y[o] = act ? tanh(acc) : acc;
  }
}

/* dz [out] -> accumulates gW [in,out], gb [out]; writes dx [in] (if not NULL) */
static void orc_dense_bwd(int in, int out, const double *x, const float *W, const double *dz, double *gW, double *gb,
                          double *dx) {
  for (int o = 0; o < out; ++o) gb[o] += dz[o];
  for (int i = 0; i < in; ++i) {
    double acc = 0.0;
    for (int o = 0; o < out; ++o) {
      gW[(size_t)i * out + o] += x[i] * dz[o];
      acc += dz[o] * (double)W[(size_t)i * out + o];
    }
    if (dx) dx[i] = acc;
  }
}

void orc_ppo_grads(int B, int S, int Hd, int D, const float *obs, const float *act, const float *logp_old,
                   const float *adv, const float *ret, const float *aW1, const float *ab1, const float *aW2,
                   const float *ab2, const float *aW3, const float *ab3, const float *cW1, const float *cb1,
                   const float *cW2, const float *cb2, const float *cW3, const float *cb3, double sigma, double clip,
                   double value_coef, double *gaW1, double *gab1, double *gaW2, double *gab2, double *gaW3,
                   double *gab3, double *gcW1, double *gcb1, double *gcW2, double *gcb2, double *gcW3, double *gcb3,
                   double *stats, double *margin) {
  double *x = (double *)malloc((size_t)S * sizeof(double));
  double *h1 = (double *)malloc((size_t)Hd * sizeof(double)), *h2 = (double *)malloc((size_t)Hd * sizeof(double));
  double *d1 = (double *)malloc((size_t)Hd * sizeof(double)), *d2 = (double *)malloc((size_t)Hd * sizeof(double));
  double *mu = (double *)malloc((size_t)D * sizeof(double)), *dz = (double *)malloc((size_t)D * sizeof(double));
  memset(gaW1, 0, sizeof(double) * (size_t)S * Hd), memset(gab1, 0, sizeof(double) * Hd);
  memset(gaW2, 0, sizeof(double) * (size_t)Hd * Hd), memset(gab2, 0, sizeof(double) * Hd);
  memset(gaW3, 0, sizeof(double) * (size_t)Hd * D), memset(gab3, 0, sizeof(double) * D);
  memset(gcW1, 0, sizeof(double) * (size_t)S * Hd), memset(gcb1, 0, sizeof(double) * Hd);
  memset(gcW2, 0, sizeof(double) * (size_t)Hd * Hd), memset(gcb2, 0, sizeof(double) * Hd);
  memset(gcW3, 0, sizeof(double) * (size_t)Hd), memset(gcb3, 0, sizeof(double));
  double l_pi = 0.0, l_v = 0.0, n_cut = 0.0, r_sum = 0.0;
  const double log_norm = -(double)D * log(sigma) - 0.5 * (double)D * log(2.0 * 3.14159265358979323846);
  for (int b = 0; b < B; ++b) {
    for (int i = 0; i < S; ++i) x[i] = (double)obs[(size_t)b * S + i];
    /* ---- actor */
    orc_dense_fwd(S, Hd, x, aW1, ab1, 1, h1);
    orc_dense_fwd(Hd, Hd, h1, aW2, ab2, 1, h2);
    orc_dense_fwd(Hd, D, h2, aW3, ab3, 1, mu);
    double logp = log_norm;
    for (int d = 0; d < D; ++d) {
      const double e = (double)act[(size_t)b * D + d] - mu[d];
      logp -= e * e / (2.0 * sigma * sigma);
    }
    const double ratio = exp(logp - (double)logp_old[b]);
    const double A = (double)adv[b];
    const double rc = ratio < 1.0 - clip ? 1.0 - clip : (ratio > 1.0 + clip ? 1.0 + clip : ratio);
    const double s1 = ratio * A, s2 = rc * A;
    const int active = s1 <= s2;
    l_pi -= (active ? s1 : s2) / (double)B;
    n_cut += active ? 0.0 : 1.0;
    r_sum += ratio;
    if (margin) {
      const double lo = fabs(ratio - (1.0 - clip)), hi = fabs(ratio - (1.0 + clip));
      margin[b] = lo < hi ? lo : hi;
    }
    /* dL/dmu_d = -(1/B) active ratio A (a_d - mu_d) / sigma^2, through the output tanh */
    for (int d = 0; d < D; ++d) {
      const double e = (double)act[(size_t)b * D + d] - mu[d];
      const double dmu = active ? -(ratio * A * e / (sigma * sigma)) / (double)B : 0.0;
      dz[d] = dmu * (1.0 - mu[d] * mu[d]);
    }
    orc_dense_bwd(Hd, D, h2, aW3, dz, gaW3, gab3, d2);
    for (int i = 0; i < Hd; ++i) d2[i] *= 1.0 - h2[i] * h2[i];
    orc_dense_bwd(Hd, Hd, h1, aW2, d2, gaW2, gab2, d1);
    for (int i = 0; i < Hd; ++i) d1[i] *= 1.0 - h1[i] * h1[i];
    orc_dense_bwd(S, Hd, x, aW1, d1, gaW1, gab1, NULL);
    /* ---- critic */
    double v;
    orc_dense_fwd(S, Hd, x, cW1, cb1, 1, h1);
    orc_dense_fwd(Hd, Hd, h1, cW2, cb2, 1, h2);
    orc_dense_fwd(Hd, 1, h2, cW3, cb3, 0, &v);
    const double err = v - (double)ret[b];
    l_v += 0.5 * err * err / (double)B;
    double dv = value_coef * err / (double)B;
    orc_dense_bwd(Hd, 1, h2, cW3, &dv, gcW3, gcb3, d2);
    for (int i = 0; i < Hd; ++i) d2[i] *= 1.0 - h2[i] * h2[i];
    orc_dense_bwd(Hd, Hd, h1, cW2, d2, gcW2, gcb2, d1);
    for (int i = 0; i < Hd; ++i) d1[i] *= 1.0 - h1[i] * h1[i];
    orc_dense_bwd(S, Hd, x, cW1, d1, gcW1, gcb1, NULL);
  }
  stats[0] = l_pi;
  stats[1] = l_v;
  stats[2] = n_cut / (double)B;
  stats[3] = r_sum / (double)B;
  free(x), free(h1), free(h2), free(d1), free(d2), free(mu), free(dz);
}

/* Adam (the optimiser of the PPO implementation the paper uses; Kingma & Ba's update with bias correction):
 *   m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;  theta -= lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps). */
void orc_adam(int64_t n, double *theta, const double *g, double *m, double *v, double lr, double b1, double b2,
              double eps, int t) {
  const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
  for (int64_t i = 0; i < n; ++i) {
    m[i] = b1 * m[i] + (1.0 - b1) * g[i];
    v[i] = b2 * v[i] + (1.0 - b2) * g[i] * g[i];
    theta[i] -= lr * (m[i] / c1) / (sqrt(v[i] / c2) + eps);
  }
}
