/*
 * Runs every entry point of the CPU checker (oracle/podoracle.c) on small inputs that include the awkward
 * shapes -- one env, one stock, no indicators, resets inside the rollout, several agents and markets, an
 * episode that never ends, keep = P in the refill -- so that a build with -fsanitize=address,undefined
 * reports any out-of-bounds access, use of uninitialised heap or undefined arithmetic in it.
 * Test infrastructure only; built and run by tests/test_oracle_sanitized.py.
 */
#include "../oracle/podoracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x243f6a8885a308d3ull;
static double unif(void) { /* splitmix64 -> [0, 1) */
  uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
  z ^= z >> 31;
  return (double)(z >> 11) / 9007199254740992.0;
}
static float *fvec(size_t n, double lo, double hi) {
  float *v = (float *)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) v[i] = (float)(lo + (hi - lo) * unif());
  return v;
}
static double checksum = 0.0;
static void eat_d(const double *v, size_t n) {
  for (size_t i = 0; i < n; ++i) checksum += v[i] * (double)(1 + i % 7);
}
static void eat_f(const float *v, size_t n) {
  for (size_t i = 0; i < n; ++i) checksum += (double)v[i];
}

static void run_rollout(int N, int D, int K, int M, int P, int Hd, int bf16, int T, int H, int forced, float cash0) {
  orc_cfg c;
  c.n_stocks = D, c.n_ind = K, c.horizon = H, c.cash0 = cash0, c.hmax = 100.0f, c.cost = 0.001f, c.sigma = 0.5f;
  c.reward_scale = 1e-4f;
  c.obs_scale[0] = 1e-6f, c.obs_scale[1] = 0.01f, c.obs_scale[2] = 0.01f, c.obs_scale[3] = 1.0f;
  const int S = 1 + 2 * D + D * K;
  const int rows = H + T + 2; /* start rows are 0: the cursor never passes H + 1 */
  float *price = fvec((size_t)rows * M * D, 10.0, 100.0), *ind = fvec((size_t)rows * M * D * K, -1.0, 1.0);
  float *noise = fvec((size_t)T * N * D, -2.0, 2.0), *mu_forced = forced ? fvec((size_t)T * N * D, -1.0, 1.0) : NULL;
  const size_t sizes_a[6] = {(size_t)S * Hd, (size_t)Hd, (size_t)Hd * Hd, (size_t)Hd, (size_t)Hd * D, (size_t)D};
  const size_t sizes_c[6] = {(size_t)S * Hd, (size_t)Hd, (size_t)Hd * Hd, (size_t)Hd, (size_t)Hd, 1};
  const float *actor[6], *critic[6];
  for (int i = 0; i < 6; ++i) actor[i] = fvec(sizes_a[i] * P, -0.3, 0.3), critic[i] = fvec(sizes_c[i] * P, -0.3, 0.3);
  int32_t *agent_of = (int32_t *)malloc(sizeof(int32_t) * N), *market_of = (int32_t *)malloc(sizeof(int32_t) * N);
  for (int n = 0; n < N; ++n) agent_of[n] = n * P / N, market_of[n] = n % M;
  orc_state s;
  s.cash = (float *)malloc(sizeof(float) * N), s.h = (int32_t *)malloc(sizeof(int32_t) * N * D);
  s.tau = (int32_t *)malloc(sizeof(int32_t) * N), s.asset = (double *)malloc(sizeof(double) * N);
  s.ep_ret = (double *)malloc(sizeof(double) * N), s.ep_sum = (double *)malloc(sizeof(double) * N);
  s.ep_sqsum = (double *)malloc(sizeof(double) * N), s.ep_cnt = (int32_t *)malloc(sizeof(int32_t) * N);
  s.start = (int32_t *)calloc(N, sizeof(int32_t));
  orc_reset_state(&c, N, &s);
  float *obs = (float *)malloc(sizeof(float) * (size_t)(T + 1) * N * S), *act = (float *)malloc(sizeof(float) * (size_t)T * N * D);
  double *mu = (double *)malloc(sizeof(double) * (size_t)T * N * D), *logp = (double *)malloc(sizeof(double) * (size_t)T * N);
  double *reward = (double *)malloc(sizeof(double) * (size_t)T * N), *value = (double *)malloc(sizeof(double) * (size_t)(T + 1) * N);
  uint8_t *done = (uint8_t *)malloc((size_t)T * N), *flags = (uint8_t *)malloc((size_t)T * N * D);
  int32_t *shares = (int32_t *)malloc(sizeof(int32_t) * (size_t)T * N * D);
  /* two calls in a row: the second continues the episodes of the first */
  for (int call = 0; call < 2; ++call) {
    if (orc_rollout(&c, N, M, Hd, bf16, T, agent_of, market_of, price, ind, actor, critic, noise, mu_forced, &s, obs, mu,
                    act, logp, reward, done, value, shares, flags) != 0) {
      fprintf(stderr, "orc_rollout failed\n");
      exit(2);
    }
    eat_f(obs, (size_t)(T + 1) * N * S), eat_d(mu, (size_t)T * N * D), eat_f(act, (size_t)T * N * D);
    eat_d(logp, (size_t)T * N), eat_d(reward, (size_t)T * N), eat_d(value, (size_t)(T + 1) * N);
    for (size_t i = 0; i < (size_t)T * N * D; ++i) checksum += shares[i] + flags[i];
    for (size_t i = 0; i < (size_t)T * N; ++i) checksum += done[i];
  }
  /* outputs are optional */
  orc_rollout(&c, N, M, Hd, bf16, 1, agent_of, market_of, price, ind, actor, NULL, noise, mu_forced, &s, NULL, NULL, NULL,
              NULL, NULL, NULL, NULL, NULL, NULL);
  /* GAE, asset curves and metrics of the last recorded call */
  double *adv = (double *)malloc(sizeof(double) * (size_t)T * N), *ret = (double *)malloc(sizeof(double) * (size_t)T * N);
  orc_gae(T, N, reward, value, done, 0.99, 0.95, adv, ret);
  eat_d(adv, (size_t)T * N), eat_d(ret, (size_t)T * N);
  double *curve = (double *)malloc(sizeof(double) * (size_t)(T + 1) * N), *met = (double *)malloc(sizeof(double) * 6 * N);
  int32_t *len = (int32_t *)malloc(sizeof(int32_t) * N);
  orc_asset_curve(T, N, D, S, obs, done, c.obs_scale, curve, len);
  orc_metrics(T, N, curve, len, 252.0, 0.02, met);
  eat_d(curve, (size_t)(T + 1) * N), eat_d(met, (size_t)6 * N);
  /* leaderboard over the agents */
  double *mean = (double *)malloc(sizeof(double) * P), *var = (double *)malloc(sizeof(double) * P);
  int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * P);
  orc_leaderboard(P, N, agent_of, s.ep_sum, s.ep_sqsum, s.ep_cnt, mean, var, rank);
  for (int i = 0; i < P; ++i) checksum += rank[i] + (mean[i] == mean[i] ? mean[i] : 0.0);
  /* refill of the first actor tensor from the ranking, with and without noise, keep = 1 and keep = P */
  float *params = fvec(sizes_a[0] * P, -0.3, 0.3), *z = fvec(sizes_a[0] * P, -1.0, 1.0);
  orc_population_refill(P, (int64_t)sizes_a[0], rank, 1, 0.02f, z, params);
  orc_population_refill(P, (int64_t)sizes_a[0], rank, P, 0.02f, NULL, params);
  eat_f(params, sizes_a[0] * P);
  /* one learner minibatch on the recorded transitions of agent 0's envs, then an Adam step on one tensor */
  {
    int B = T * (N / P);
    if (B > 48) B = 48;
    float *o = (float *)malloc(sizeof(float) * (size_t)B * S), *a = (float *)malloc(sizeof(float) * (size_t)B * D);
    float *lp = (float *)malloc(sizeof(float) * B), *ad = (float *)malloc(sizeof(float) * B), *rt = (float *)malloc(sizeof(float) * B);
    for (int b = 0; b < B; ++b) {
      const int t = b % T, n = (b / T) % (N / P);
      memcpy(o + (size_t)b * S, obs + ((size_t)t * N + n) * S, sizeof(float) * S);
      memcpy(a + (size_t)b * D, act + ((size_t)t * N + n) * D, sizeof(float) * D);
      lp[b] = (float)logp[(size_t)t * N + n] + (float)(0.4 * unif() - 0.2);
      ad[b] = (float)adv[(size_t)t * N + n], rt[b] = (float)ret[(size_t)t * N + n];
    }
    double *g[12];
    for (int i = 0; i < 6; ++i) g[i] = (double *)malloc(sizeof(double) * sizes_a[i]), g[6 + i] = (double *)malloc(sizeof(double) * sizes_c[i]);
    double stats[4], *margin = (double *)malloc(sizeof(double) * B);
    orc_ppo_grads(B, S, Hd, D, o, a, lp, ad, rt, actor[0], actor[1], actor[2], actor[3], actor[4], actor[5], critic[0],
                  critic[1], critic[2], critic[3], critic[4], critic[5], 0.5, 0.2, 0.5, g[0], g[1], g[2], g[3], g[4], g[5],
                  g[6], g[7], g[8], g[9], g[10], g[11], stats, margin);
    for (int i = 0; i < 6; ++i) eat_d(g[i], sizes_a[i]), eat_d(g[6 + i], sizes_c[i]);
    eat_d(stats, 4), eat_d(margin, B);
    double *theta = (double *)malloc(sizeof(double) * sizes_a[0]), *m1 = (double *)calloc(sizes_a[0], sizeof(double));
    double *m2 = (double *)calloc(sizes_a[0], sizeof(double));
    for (size_t i = 0; i < sizes_a[0]; ++i) theta[i] = (double)actor[0][i];
    for (int t = 1; t <= 3; ++t) orc_adam((int64_t)sizes_a[0], theta, g[0], m1, m2, 1e-3, 0.9, 0.999, 1e-8, t);
    eat_d(theta, sizes_a[0]);
    for (int i = 0; i < 12; ++i) free(g[i]);
    free(o), free(a), free(lp), free(ad), free(rt), free(margin), free(theta), free(m1), free(m2);
  }
  for (int i = 0; i < 6; ++i) free((void *)actor[i]), free((void *)critic[i]);
  free(price), free(ind), free(noise), free(mu_forced), free(agent_of), free(market_of);
  free(s.cash), free(s.h), free(s.tau), free(s.asset), free(s.ep_ret), free(s.ep_sum), free(s.ep_sqsum), free(s.ep_cnt), free(s.start);
  free(obs), free(act), free(mu), free(logp), free(reward), free(value), free(done), free(flags), free(shares);
  free(adv), free(ret), free(curve), free(met), free(len), free(mean), free(var), free(rank), free(params), free(z);
}

int main(void) {
  /* bf16 rounding over specials and ties */
  {
    const float xs[] = {0.0f, -0.0f, 1.0f, 1.00390625f, 1.01171875f, 3.3895314e38f, -3.4028235e38f, 1e-45f, INFINITY, NAN};
    float out[10];
    orc_bf16_round_array(xs, out, 10);
    for (int i = 0; i < 9; ++i) checksum += isfinite(out[i]) ? (double)out[i] * 1e-30 : 1.0;
  }
  /*          N   D  K  M  P  Hd  bf16 T   H  forced cash0 */
  run_rollout(1,  1, 0, 1, 1, 4,  0,   3,  3, 0, 1e4f);      /* smallest everything, no indicators, reset at the end */
  run_rollout(5,  2, 1, 2, 1, 8,  1,   7,  3, 0, 5e3f);      /* resets inside the rollout, two markets, bf16 emulation */
  run_rollout(12, 5, 2, 3, 3, 16, 0,   9,  64, 1, 2e3f);     /* three agents, forced means, cash-starved, no episode end */
  run_rollout(6,  30, 8, 1, 2, 32, 1,  4,  2, 0, 1e6f);      /* the Dow-30 observation width */
  /* a strided input with a linear output head */
  {
    const int rows = 3, S = 5, ldx = 9, Hd = 6, O = 2;
    float *X = fvec((size_t)rows * ldx, -1, 1), *W1 = fvec((size_t)S * Hd, -1, 1), *b1 = fvec(Hd, -1, 1);
    float *W2 = fvec((size_t)Hd * Hd, -1, 1), *b2 = fvec(Hd, -1, 1), *W3 = fvec((size_t)Hd * O, -1, 1), *b3 = fvec(O, -1, 1);
    double out[6];
    orc_mlp(rows, S, Hd, O, X, ldx, W1, b1, W2, b2, W3, b3, 0, 1, out);
    eat_d(out, 6);
    free(X), free(W1), free(b1), free(W2), free(b2), free(W3), free(b3);
  }
  /* metrics of degenerate curves: no step, one step, a flat curve, a total loss */
  {
    const double flat[4] = {5.0, 5.0, 5.0, 5.0}, ruin[3] = {4.0, 2.0, 0.0};
    double out[6];
    orc_metrics_curve(0, flat, 252.0, 0.0, out), eat_d(out, 6);
    orc_metrics_curve(1, flat, 252.0, 0.0, out), eat_d(out, 6);
    orc_metrics_curve(3, flat, 252.0, 0.02, out), eat_d(out, 6);
    orc_metrics_curve(2, ruin, 252.0, 0.0, out);
    for (int i = 0; i < 6; ++i) checksum += isfinite(out[i]) ? out[i] : 1.0;
  }
  printf("sanitized checker run complete, checksum %.17g\n", checksum);
  return 0;
}
