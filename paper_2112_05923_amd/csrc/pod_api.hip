// C ABI of libpodrollout: argument validation, workspace layout and the
// sequencing of kernel launches.  No arithmetic of the method lives here.
#include <math.h>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "pod_internal.h"

using namespace pod;

struct pr_handle {
  pr_config cfg;
  hipStream_t stream;
  EnvDims dims;
  EnvState st;
  pr_market market;
  PackedNet actor, critic;
  PackedNet actor_fused;  // the actor with layer 1 packed in the input order of the persistent rollout kernel
  void *w1_fused;
  void *w_packed[2][3];   // device, per net and layer
  float *b_packed[2][3];
  float *mu_scratch;      // [N, D]
  int32_t *start;         // [N] episode start rows (zeros unless a replay table is set)
  float *split;           // activations between the launches of the layer-per-launch actor (small batches), or null
  int32_t S;
};

namespace {

thread_local int g_last_hip = 0;

int hip_fail(hipError_t e) {
  g_last_hip = (int)e;
  return PR_EHIP;
}

#define POD_HIP(call)                       \
  do {                                      \
    hipError_t e__ = (call);                \
    if (e__ != hipSuccess) return hip_fail(e__); \
  } while (0)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool is_pow2_float(float x) {
  if (!(x > 0.0f) || isinf(x)) return false;
  int e;
  return frexpf(x, &e) == 0.5f;
}

struct Layout {
  size_t w[2][3], b[2][3];
  size_t w1_fused;
  size_t cash, tau, h, ep_ret, ep_sum, ep_sqsum, ep_cnt, mu, start, split;
  size_t total;
};

int state_dim(const pr_config &c) { return 1 + 2 * c.n_stocks + c.n_stocks * c.n_ind; }

int validate_config(const pr_config *c) {
  if (!c) return PR_EINVAL;
  if (c->n_envs < 1 || c->n_agents < 1 || c->n_envs % c->n_agents != 0) return PR_EINVAL;
  if (c->n_stocks < 1 || c->n_ind < 0 || c->hidden < 1 || c->horizon < 1) return PR_EINVAL;
  if (c->n_market != 1 && c->n_market != c->n_envs) return PR_EINVAL;
  if (c->mlp_dtype != PR_MLP_F32 && c->mlp_dtype != PR_MLP_BF16) return PR_EINVAL;
  if (c->schedule != PR_SCHED_STEPWISE && c->schedule != PR_SCHED_FUSED) return PR_EINVAL;
  if (!(c->cash0 > 0.0f) || !(c->hmax > 0.0f) || !(c->cost >= 0.0f) || !(c->cost < 1.0f)) return PR_EINVAL;
  if (!(c->sigma > 0.0f) || !isfinite(c->reward_scale) || !isfinite(c->cash0) || !isfinite(c->hmax)) return PR_EINVAL;
  for (int i = 0; i < 4; ++i)
    if (!is_pow2_float(c->obs_scale[i])) return PR_EINVAL;
  // index arithmetic inside the kernels is 32-bit per step and per market row
  const double nd = (double)c->n_envs * c->n_stocks * (c->n_ind > 1 ? c->n_ind : 1);
  const double rows = ((double)c->horizon + 1.0) * c->n_market;
  if (nd >= 2147483647.0 || rows >= 2147483647.0 || (double)c->n_envs * state_dim(*c) >= 2147483647.0)
    return PR_EINVAL;
  // shapes the kernels cover
  const int S = state_dim(*c);
  if (!mlp_supported(S, c->hidden, c->n_stocks, c->mlp_dtype) || !mlp_supported(S, c->hidden, 1, c->mlp_dtype))
    return PR_EUNSUPPORTED;
  if (c->n_agents > 1 && (c->n_envs / c->n_agents) % 64 != 0) return PR_EUNSUPPORTED;
  if (c->schedule == PR_SCHED_FUSED && !fused_supported(*c)) return PR_EUNSUPPORTED;
  return PR_OK;
}

Layout make_layout(const pr_config &c) {
  Layout L;
  const int S = state_dim(c), Hd = c.hidden, D = c.n_stocks, P = c.n_agents, bf = c.mlp_dtype;
  const size_t N = (size_t)c.n_envs;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes, 256);
    return o;
  };
  const int in_dim[3] = {S, Hd, Hd};
  for (int net = 0; net < 2; ++net) {
    const int out_dim[3] = {Hd, Hd, net == 0 ? D : 1};
    for (int l = 0; l < 3; ++l) {
      L.w[net][l] = take(packed_weight_bytes(in_dim[l], out_dim[l], bf) * P);
      L.b[net][l] = take((size_t)padded_out(out_dim[l]) * 4 * P);
    }
  }
  L.w1_fused = c.schedule == PR_SCHED_FUSED ? take(packed_weight_bytes(S, Hd, bf) * P) : 0;
  L.cash = take(N * 4);
  L.tau = take(N * 4);
  L.h = take(N * D * 4);
  L.ep_ret = take(N * 8);
  L.ep_sum = take(N * 8);
  L.ep_sqsum = take(N * 8);
  L.ep_cnt = take(N * 4);
  L.mu = take(N * D * 4);
  L.start = take(N * 4);
  L.split = take((size_t)split_scratch_rows(c.n_envs, Hd) * Hd * 4 * 2);
  L.total = off;
  return L;
}

void fill_net(PackedNet &pn, const pr_handle *h, int net) {
  const pr_config &c = h->cfg;
  const int S = h->S, Hd = c.hidden, D = c.n_stocks, bf = c.mlp_dtype;
  const int KB = bf ? 16 : 8;
  const int in_dim[3] = {S, Hd, Hd};
  const int out_dim[3] = {Hd, Hd, net == 0 ? D : 1};
  for (int l = 0; l < 3; ++l) {
    pn.W[l] = h->w_packed[net][l];
    pn.b[l] = h->b_packed[net][l];
    pn.w_stride[l] = (int64_t)packed_weight_bytes(in_dim[l], out_dim[l], bf);
    pn.b_stride[l] = padded_out(out_dim[l]);
    pn.in_dim[l] = in_dim[l];
    pn.out_dim[l] = out_dim[l];
    pn.nkb[l] = (in_dim[l] + KB - 1) / KB;
    pn.nct[l] = (out_dim[l] + 31) / 32;
  }
  pn.bf16 = bf;
  pn.out_tanh = net == 0 ? 1 : 0;
  pn.split_rows = split_scratch_rows(c.n_envs, Hd);
  pn.split_h[0] = pn.split_rows ? h->split : nullptr;
  pn.split_h[1] = pn.split_rows ? h->split + (size_t)pn.split_rows * Hd : nullptr;
}

bool weights_ok(const pr_weights *w) { return w && w->W1 && w->b1 && w->W2 && w->b2 && w->W3 && w->b3; }

int pack_nets(pr_handle *h, const pr_weights *actor, const pr_weights *critic) {
  const pr_config &c = h->cfg;
  const int S = h->S, Hd = c.hidden, D = c.n_stocks, P = c.n_agents, bf = c.mlp_dtype;
  const pr_weights *ws[2] = {actor, critic};
  for (int net = 0; net < 2; ++net) {
    const float *W[3] = {ws[net]->W1, ws[net]->W2, ws[net]->W3};
    const float *b[3] = {ws[net]->b1, ws[net]->b2, ws[net]->b3};
    const int in_dim[3] = {S, Hd, Hd};
    const int out_dim[3] = {Hd, Hd, net == 0 ? D : 1};
    for (int l = 0; l < 3; ++l)
      POD_HIP(launch_pack_layer(h->stream, W[l], b[l], P, in_dim[l], out_dim[l], bf, 0, h->w_packed[net][l],
                                h->b_packed[net][l]));
  }
  // The persistent rollout kernel keeps its observation tile as [indicators | cash | prices | holdings]:
  // the same layer-1 weights with their rows rotated by the D K indicator columns (biases are shared).
  if (c.schedule == PR_SCHED_FUSED)
    POD_HIP(launch_pack_layer(h->stream, actor->W1, actor->b1, P, S, Hd, bf, D * c.n_ind, h->w1_fused,
                              h->b_packed[0][0]));
  return PR_OK;
}

int check_buffers(const pr_buffers *o) {
  if (!o || !o->obs || !o->act_raw || !o->reward || !o->done) return PR_EINVAL;
  return PR_OK;
}

StepIO step_io(const pr_handle *h, const pr_buffers *o, int t, const float *mu, const float *noise) {
  const size_t N = (size_t)h->cfg.n_envs, D = (size_t)h->cfg.n_stocks, S = (size_t)h->S;
  StepIO io;
  io.mu = mu;
  io.noise = noise + (size_t)t * N * D;
  io.obs_next = o->obs + (size_t)(t + 1) * N * S;
  io.act_raw = o->act_raw + (size_t)t * N * D;
  io.reward = o->reward + (size_t)t * N;
  io.done = o->done + (size_t)t * N;
  io.logp = o->logp ? o->logp + (size_t)t * N : nullptr;
  io.shares = o->shares ? o->shares + (size_t)t * N * D : nullptr;
  return io;
}

}  // namespace

extern "C" {

int rollout_workspace_bytes(const pr_config *cfg, size_t *out) {
  if (!out) return PR_EINVAL;
  const int rc = validate_config(cfg);
  if (rc != PR_OK) return rc;
  *out = make_layout(*cfg).total;
  return PR_OK;
}

int rollout_kernel_lds_bytes(const pr_config *cfg, int32_t with_actor, size_t *out) {
  if (!out || !cfg) return PR_EINVAL;
  pr_config c = *cfg;
  c.schedule = PR_SCHED_STEPWISE;  // (validate the shape itself; whether the persistent kernel covers it is asked below)
  const int rc = validate_config(&c);
  if (rc != PR_OK) return rc;
  if (!fused_supported(*cfg)) return PR_EUNSUPPORTED;
  *out = fused_lds_bytes(*cfg, with_actor != 0);
  return PR_OK;
}

int rollout_init(const pr_config *cfg, const pr_market *market, const pr_weights *actor, const pr_weights *critic,
                 void *workspace, size_t workspace_bytes, void *hip_stream, pr_handle **out) {
  if (!out) return PR_EINVAL;
  *out = nullptr;
  const int rc = validate_config(cfg);
  if (rc != PR_OK) return rc;
  if (!market || !market->price || (cfg->n_ind > 0 && !market->ind)) return PR_EINVAL;
  if (!weights_ok(actor) || !weights_ok(critic)) return PR_EINVAL;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PR_EINVAL;
  // the persistent kernel moves indicator rows in 16-byte groups
  if (cfg->schedule == PR_SCHED_FUSED && (reinterpret_cast<uintptr_t>(market->ind) & 15u)) return PR_EINVAL;
  const Layout L = make_layout(*cfg);
  if (workspace_bytes < L.total) return PR_ENOMEM;

  pr_handle *h = new (std::nothrow) pr_handle;
  if (!h) return PR_ENOMEM;
  memset(h, 0, sizeof(*h));
  h->cfg = *cfg;
  h->stream = static_cast<hipStream_t>(hip_stream);
  h->market = *market;
  h->S = state_dim(*cfg);
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  for (int net = 0; net < 2; ++net)
    for (int l = 0; l < 3; ++l) {
      h->w_packed[net][l] = ws + L.w[net][l];
      h->b_packed[net][l] = reinterpret_cast<float *>(ws + L.b[net][l]);
    }
  h->st.cash = reinterpret_cast<float *>(ws + L.cash);
  h->st.tau = reinterpret_cast<int32_t *>(ws + L.tau);
  h->st.h = reinterpret_cast<int32_t *>(ws + L.h);
  h->st.ep_ret = reinterpret_cast<double *>(ws + L.ep_ret);
  h->st.ep_sum = reinterpret_cast<double *>(ws + L.ep_sum);
  h->st.ep_sqsum = reinterpret_cast<double *>(ws + L.ep_sqsum);
  h->st.ep_cnt = reinterpret_cast<int32_t *>(ws + L.ep_cnt);
  h->mu_scratch = reinterpret_cast<float *>(ws + L.mu);
  h->start = reinterpret_cast<int32_t *>(ws + L.start);
  h->split = reinterpret_cast<float *>(ws + L.split);
  h->st.start = h->start;

  EnvDims &d = h->dims;
  d.N = cfg->n_envs;
  d.D = cfg->n_stocks;
  d.K = cfg->n_ind;
  d.S = h->S;
  d.H = cfg->horizon;
  d.M = cfg->n_market;
  d.cash0 = cfg->cash0;
  d.hmax = cfg->hmax;
  d.one_minus_c = 1.0f - cfg->cost;
  d.one_plus_c = 1.0f + cfg->cost;
  d.sigma = cfg->sigma;
  d.rho = cfg->reward_scale;
  d.logp_const = (float)(-(double)cfg->n_stocks * (log((double)cfg->sigma) + 0.91893853320467274178));
  d.s_cash = cfg->obs_scale[0];
  d.s_price = cfg->obs_scale[1];
  d.s_hold = cfg->obs_scale[2];
  d.s_ind = cfg->obs_scale[3];

  fill_net(h->actor, h, 0);
  h->w1_fused = cfg->schedule == PR_SCHED_FUSED ? static_cast<void *>(ws + L.w1_fused) : nullptr;
  h->actor_fused = h->actor;
  h->actor_fused.W[0] = h->w1_fused;
  fill_net(h->critic, h, 1);
  int prc = pack_nets(h, actor, critic);
  if (prc == PR_OK) {
    hipError_t e = hipMemsetAsync(h->start, 0, (size_t)cfg->n_envs * 4, h->stream);
    if (e == hipSuccess) e = launch_state_reset(h->stream, h->dims, h->st);
    if (e != hipSuccess) prc = hip_fail(e);
  }
  if (prc != PR_OK) {
    delete h;
    return prc;
  }
  *out = h;
  return PR_OK;
}

int rollout_set_weights(pr_handle *h, const pr_weights *actor, const pr_weights *critic) {
  if (!h || !weights_ok(actor) || !weights_ok(critic)) return PR_EINVAL;
  return pack_nets(h, actor, critic);
}

int rollout_reset(pr_handle *h) {
  if (!h) return PR_EINVAL;
  POD_HIP(launch_state_reset(h->stream, h->dims, h->st));
  return PR_OK;
}

int rollout_set_replay(pr_handle *h, const pr_market *table, int32_t table_rows, const int32_t *start) {
  if (!h || !table || !table->price || (h->cfg.n_ind > 0 && !table->ind) || !start) return PR_EINVAL;
  if (table_rows < h->cfg.horizon + 1 || (double)table_rows * h->cfg.n_market >= 2147483647.0) return PR_EINVAL;
  if (h->cfg.schedule == PR_SCHED_FUSED && (reinterpret_cast<uintptr_t>(table->ind) & 15u)) return PR_EINVAL;
  // every episode must stay inside the table: checked on the device, read back here (this call synchronises)
  int32_t *flag = reinterpret_cast<int32_t *>(h->mu_scratch), bad = 1;
  POD_HIP(launch_check_starts(h->stream, h->cfg.n_envs, h->cfg.horizon, table_rows, start, flag));
  POD_HIP(hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, h->stream));
  POD_HIP(hipStreamSynchronize(h->stream));
  if (bad) return PR_EINVAL;
  POD_HIP(hipMemcpyAsync(h->start, start, (size_t)h->cfg.n_envs * 4, hipMemcpyDeviceToDevice, h->stream));
  h->market = *table;
  POD_HIP(launch_state_reset(h->stream, h->dims, h->st));
  return PR_OK;
}

int rollout_step_T(pr_handle *h, int32_t T, const float *noise, const pr_buffers *out) {
  if (!h || T < 1 || !noise) return PR_EINVAL;
  int rc = check_buffers(out);
  if (rc != PR_OK) return rc;
  const size_t N = (size_t)h->cfg.n_envs, D = (size_t)h->cfg.n_stocks, S = (size_t)h->S;
  const int32_t per_agent = h->cfg.n_envs / h->cfg.n_agents;
  if (h->cfg.schedule == PR_SCHED_FUSED) {
    POD_HIP(launch_rollout_fused(h->stream, h->cfg, h->dims, h->st, h->market.price, h->market.ind, h->actor_fused,
                                 per_agent, T, noise, nullptr, *out));
  } else {
    POD_HIP(launch_observe(h->stream, h->dims, h->st, h->market.price, h->market.ind, out->obs));
    for (int t = 0; t < T; ++t) {
      float *mu = out->mu ? out->mu + (size_t)t * N * D : h->mu_scratch;
      POD_HIP(launch_mlp(h->stream, h->actor, (int64_t)N, out->obs + (size_t)t * N * S, (int64_t)S, mu, (int32_t)N,
                         per_agent));
      POD_HIP(launch_env_step(h->stream, h->dims, h->st, h->market.price, h->market.ind,
                              step_io(h, out, t, mu, noise)));
    }
  }
  if (out->value)
    POD_HIP(launch_mlp(h->stream, h->critic, (int64_t)(T + 1) * (int64_t)N, out->obs, (int64_t)S, out->value,
                       (int32_t)N, per_agent));
  return PR_OK;
}

int rollout_step_forced(pr_handle *h, int32_t T, const float *mu, const float *noise, const pr_buffers *out) {
  if (!h || T < 1 || !noise || !mu) return PR_EINVAL;
  int rc = check_buffers(out);
  if (rc != PR_OK) return rc;
  const size_t N = (size_t)h->cfg.n_envs, D = (size_t)h->cfg.n_stocks;
  if (h->cfg.schedule == PR_SCHED_FUSED) {
    POD_HIP(launch_rollout_fused(h->stream, h->cfg, h->dims, h->st, h->market.price, h->market.ind,
                                 h->actor_fused, h->cfg.n_envs / h->cfg.n_agents, T, noise, mu, *out));
    return PR_OK;
  }
  POD_HIP(launch_observe(h->stream, h->dims, h->st, h->market.price, h->market.ind, out->obs));
  for (int t = 0; t < T; ++t)
    POD_HIP(launch_env_step(h->stream, h->dims, h->st, h->market.price, h->market.ind,
                            step_io(h, out, t, mu + (size_t)t * N * D, noise)));
  return PR_OK;
}

int rollout_mlp_forward(pr_handle *h, int32_t net, int64_t rows, const float *X, int64_t ldx, float *Y) {
  if (!h || (net != PR_NET_ACTOR && net != PR_NET_CRITIC) || rows < 1 || !X || !Y || ldx < h->S) return PR_EINVAL;
  if ((rows + 63) / 64 > 2147483647LL) return PR_EINVAL;
  POD_HIP(launch_mlp(h->stream, net == PR_NET_ACTOR ? h->actor : h->critic, rows, X, ldx, Y, h->cfg.n_envs,
                     h->cfg.n_envs / h->cfg.n_agents));
  return PR_OK;
}

int rollout_get_state(pr_handle *h, const pr_state *out) {
  if (!h || !out) return PR_EINVAL;
  POD_HIP(launch_state_copy(h->stream, h->dims, h->st, *out, true));
  return PR_OK;
}

int rollout_set_state(pr_handle *h, const pr_state *in) {
  if (!h || !in) return PR_EINVAL;
  POD_HIP(launch_state_copy(h->stream, h->dims, h->st, *in, false));
  return PR_OK;
}

int compute_gae(void *hip_stream, int32_t T, int32_t N, const float *reward, const float *value, const uint8_t *done,
                float gamma, float lambda, float *adv, float *ret) {
  if (T < 1 || N < 1 || !reward || !value || !done || !adv || !ret) return PR_EINVAL;
  if (!isfinite(gamma) || !isfinite(lambda)) return PR_EINVAL;
  if ((double)(T + 1) * (double)N >= 9.0e18) return PR_EINVAL;
  POD_HIP(launch_gae(static_cast<hipStream_t>(hip_stream), T, N, reward, value, done, gamma, lambda, adv, ret));
  return PR_OK;
}

int trading_metrics(void *hip_stream, int32_t T, int32_t N, int32_t n_stocks, int32_t state_dim, const float *obs,
                    const uint8_t *done, const float *obs_scale, double periods_per_year, double risk_free,
                    double *metrics, int32_t *length) {
  if (T < 1 || N < 1 || n_stocks < 1 || !obs || !done || !obs_scale || !metrics) return PR_EINVAL;
  if (state_dim < 1 + 2 * n_stocks) return PR_EINVAL;
  if (!(periods_per_year > 0.0) || !isfinite(periods_per_year) || !isfinite(risk_free)) return PR_EINVAL;
  for (int i = 0; i < 3; ++i)
    if (!is_pow2_float(obs_scale[i])) return PR_EINVAL;
  if (((double)T + 1.0) * (double)N * (double)state_dim >= 9.0e18) return PR_EINVAL;
  POD_HIP(launch_trading_metrics(static_cast<hipStream_t>(hip_stream), T, N, n_stocks, state_dim, obs, done, obs_scale,
                                 periods_per_year, risk_free, metrics, length));
  return PR_OK;
}

int population_refill(void *hip_stream, int32_t P, int64_t count, const int32_t *rank, int32_t keep, float sigma,
                      const float *noise, float *params) {
  if (P < 1 || count < 1 || !rank || !params || keep < 1 || keep > P || P > 65535) return PR_EINVAL;
  if (!isfinite(sigma) || (sigma != 0.0f && !noise)) return PR_EINVAL;
  if ((double)P * (double)count >= 9.0e18) return PR_EINVAL;
  POD_HIP(launch_population_refill(static_cast<hipStream_t>(hip_stream), P, count, rank, keep, sigma,
                                   sigma != 0.0f ? noise : nullptr, params));
  return PR_OK;
}

namespace {

bool net_ok(const pr_net_params *p) { return p && p->W1 && p->b1 && p->W2 && p->b2 && p->W3 && p->b3; }

int ppo_config_ok(const pr_ppo_config *c) {
  if (!c || c->batch < 1 || c->n_stocks < 1 || c->n_ind < 0 || c->hidden < 32 || c->hidden % 32 != 0) return PR_EINVAL;
  if (!(c->sigma > 0.0f) || !(c->clip > 0.0f) || !(c->clip < 1.0f) || !(c->value_coef >= 0.0f)) return PR_EINVAL;
  if (!isfinite(c->sigma) || !isfinite(c->value_coef)) return PR_EINVAL;
  if ((double)c->batch * (double)(1 + 2 * c->n_stocks + c->n_stocks * c->n_ind) >= 2147483647.0) return PR_EINVAL;
  return PR_OK;
}

// sizes of the six tensors of a network with O outputs
void net_sizes(const pr_ppo_config &c, int O, int64_t n[6]) {
  const int64_t S = 1 + 2 * c.n_stocks + c.n_stocks * c.n_ind, Hd = c.hidden;
  n[0] = S * Hd, n[1] = Hd, n[2] = Hd * Hd, n[3] = Hd, n[4] = Hd * O, n[5] = O;
}

size_t grads_bytes(const pr_ppo_config &c) {
  int64_t a[6], b[6];
  net_sizes(c, c.n_stocks, a);
  net_sizes(c, 1, b);
  size_t t = 0;
  for (int i = 0; i < 6; ++i) t += align_up((size_t)a[i] * 4, 256) + align_up((size_t)b[i] * 4, 256);
  return t;
}

}  // namespace

int ppo_workspace_bytes(const pr_ppo_config *cfg, size_t *out) {
  if (!out) return PR_EINVAL;
  const int rc = ppo_config_ok(cfg);
  if (rc != PR_OK) return rc;
  *out = ppo_scratch_bytes(cfg->batch, cfg->hidden, cfg->n_stocks, 1 + cfg->n_stocks * (2 + cfg->n_ind)) + grads_bytes(*cfg);
  return PR_OK;
}

int ppo_minibatch_grads(void *hip_stream, const pr_ppo_config *cfg, const float *obs, const float *act_raw,
                        const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                        const pr_net_params *actor, const pr_net_params *critic, const pr_net_params *grad_actor,
                        const pr_net_params *grad_critic, void *workspace, size_t workspace_bytes, float *stats) {
  const int rc = ppo_config_ok(cfg);
  if (rc != PR_OK) return rc;
  if (!obs || !act_raw || !logp_old || !adv || !ret || !workspace) return PR_EINVAL;
  if (!net_ok(actor) || !net_ok(critic) || !net_ok(grad_actor) || !net_ok(grad_critic)) return PR_EINVAL;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) ||
      workspace_bytes < ppo_scratch_bytes(cfg->batch, cfg->hidden, cfg->n_stocks, 1 + cfg->n_stocks * (2 + cfg->n_ind)))
    return PR_EINVAL;
  POD_HIP(launch_ppo_grads(static_cast<hipStream_t>(hip_stream), *cfg, obs, act_raw, logp_old, adv, ret, rows, *actor,
                           *critic, *grad_actor, *grad_critic, workspace, stats));
  return PR_OK;
}

int ppo_minibatch_grads_noalloc(void *hip_stream, const pr_ppo_config *cfg, const float *obs, const float *act_raw,
                                const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                                const pr_net_params *actor, const pr_net_params *critic,
                                const pr_net_params *grad_actor, const pr_net_params *grad_critic, float *stats) {
  const int rc = ppo_config_ok(cfg);
  if (rc != PR_OK) return rc;
  if (!obs || !act_raw || !logp_old || !adv || !ret) return PR_EINVAL;
  if (!net_ok(actor) || !net_ok(critic) || !net_ok(grad_actor) || !net_ok(grad_critic)) return PR_EINVAL;
  static_assert(PR_STATIC_SCRATCH_BYTES == (size_t)24 << 20, "header and library disagree on the scratch size");
  if (ppo_static_scratch_bytes() != PR_STATIC_SCRATCH_BYTES ||
      ppo_scratch_bytes(cfg->batch, cfg->hidden, cfg->n_stocks, 1 + cfg->n_stocks * (2 + cfg->n_ind)) >
          PR_STATIC_SCRATCH_BYTES)
    return PR_ETOOBIG;
  POD_HIP(launch_ppo_grads_static(static_cast<hipStream_t>(hip_stream), *cfg, obs, act_raw, logp_old, adv, ret, rows,
                                  *actor, *critic, *grad_actor, *grad_critic, stats));
  return PR_OK;
}

int adam_update(void *hip_stream, int64_t n, float *theta, const float *grad, float *m, float *v, float lr, float beta1,
                float beta2, float eps, int32_t t) {
  if (n < 1 || !theta || !grad || !m || !v || t < 1) return PR_EINVAL;
  if (!(beta1 >= 0.0f) || !(beta1 < 1.0f) || !(beta2 >= 0.0f) || !(beta2 < 1.0f) || !(eps > 0.0f) || !isfinite(lr))
    return PR_EINVAL;
  POD_HIP(launch_adam(static_cast<hipStream_t>(hip_stream), n, theta, grad, m, v, lr, beta1, beta2, eps, t));
  return PR_OK;
}

int ppo_learner_step(void *hip_stream, const pr_ppo_config *cfg, const float *obs, const float *act_raw,
                     const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                     const pr_net_params *actor, const pr_net_params *critic, const pr_net_params *m_actor,
                     const pr_net_params *v_actor, const pr_net_params *m_critic, const pr_net_params *v_critic,
                     void *workspace, size_t workspace_bytes, float *stats) {
  const int rc = ppo_config_ok(cfg);
  if (rc != PR_OK) return rc;
  if (!net_ok(m_actor) || !net_ok(v_actor) || !net_ok(m_critic) || !net_ok(v_critic) || !net_ok(actor) ||
      !net_ok(critic) || !workspace)
    return PR_EINVAL;
  if (cfg->adam_step < 1 || !(cfg->beta1 >= 0.0f) || !(cfg->beta1 < 1.0f) || !(cfg->beta2 >= 0.0f) ||
      !(cfg->beta2 < 1.0f) || !(cfg->adam_eps > 0.0f) || !isfinite(cfg->lr))
    return PR_EINVAL;
  const size_t scratch = ppo_scratch_bytes(cfg->batch, cfg->hidden, cfg->n_stocks, 1 + cfg->n_stocks * (2 + cfg->n_ind));
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < scratch + grads_bytes(*cfg)) return PR_EINVAL;
  // gradients behind the scratch, tensor by tensor
  unsigned char *p = static_cast<unsigned char *>(workspace) + scratch;
  int64_t na[6], nc[6];
  net_sizes(*cfg, cfg->n_stocks, na);
  net_sizes(*cfg, 1, nc);
  float *ga[6], *gc[6];
  for (int i = 0; i < 6; ++i) {
    ga[i] = reinterpret_cast<float *>(p);
    p += align_up((size_t)na[i] * 4, 256);
  }
  for (int i = 0; i < 6; ++i) {
    gc[i] = reinterpret_cast<float *>(p);
    p += align_up((size_t)nc[i] * 4, 256);
  }
  const pr_net_params gpa = {ga[0], ga[1], ga[2], ga[3], ga[4], ga[5]}, gpc = {gc[0], gc[1], gc[2], gc[3], gc[4], gc[5]};
  int r2 = ppo_minibatch_grads(hip_stream, cfg, obs, act_raw, logp_old, adv, ret, rows, actor, critic, &gpa, &gpc,
                               workspace, workspace_bytes, stats);
  if (r2 != PR_OK) return r2;
  // one launch for the twelve tensors
  int64_t n12[12];
  float *th[12], *gg[12], *mm[12], *vv[12];
  float *const *ta = &actor->W1, *const *tc = &critic->W1;
  float *const *ma = &m_actor->W1, *const *va = &v_actor->W1, *const *mc = &m_critic->W1, *const *vc = &v_critic->W1;
  for (int i = 0; i < 6; ++i) {
    n12[i] = na[i], th[i] = ta[i], gg[i] = ga[i], mm[i] = ma[i], vv[i] = va[i];
    n12[6 + i] = nc[i], th[6 + i] = tc[i], gg[6 + i] = gc[i], mm[6 + i] = mc[i], vv[6 + i] = vc[i];
  }
  POD_HIP(launch_adam12(static_cast<hipStream_t>(hip_stream), n12, th, gg, mm, vv, cfg->lr, cfg->beta1, cfg->beta2,
                        cfg->adam_eps, cfg->adam_step));
  return PR_OK;
}

int rollout_leaderboard(pr_handle *h, double *score_mean, double *score_var, int32_t *rank) {
  if (!h || !score_mean || !score_var || !rank) return PR_EINVAL;
  POD_HIP(launch_leaderboard(h->stream, h->cfg.n_envs, h->cfg.n_agents, h->st, nullptr, score_mean, score_var, rank));
  return PR_OK;
}

int rollout_calibrate(void *hip_stream, int32_t kind, int64_t n, const int32_t *params, void *buf_a, void *buf_b) {
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (!buf_a || !buf_b || n < 1) return PR_EINVAL;
  if (kind == PR_CAL_COPY || kind == PR_CAL_READ) {
    if (n % 16 != 0 || (reinterpret_cast<uintptr_t>(buf_a) & 15u) || (kind == PR_CAL_COPY && (reinterpret_cast<uintptr_t>(buf_b) & 15u)))
      return PR_EINVAL;
    const int blocks = 256 * 16;  // sixteen 256-thread workgroups per compute unit, grid-stride over the buffer
    POD_HIP(kind == PR_CAL_COPY ? launch_calib_copy(st, buf_a, buf_b, n, blocks) : launch_calib_read(st, buf_a, buf_b, n, blocks));
    return PR_OK;
  }
  if (kind != PR_CAL_PROBE || !params || n > 65535) return PR_EINVAL;
  bool any = false;
  for (int w = 0; w < 8; ++w) {
    if (params[w] < 0 || params[w] > 4) return PR_EINVAL;
    any = any || params[w] != 0;
  }
  if (!any || params[8] < 0 || params[9] < 0 || params[8] > (1 << 24) || params[9] > (1 << 24)) return PR_EINVAL;
  if (params[10] != 0 && params[10] != 2 && params[10] != 4 && params[10] != 6 && params[10] != 8) return PR_EINVAL;
  if (reinterpret_cast<uintptr_t>(buf_a) & 7u) return PR_EINVAL;
  POD_HIP(launch_calib_probe(st, params, params[8], params[9], params[10], params[11] != 0, (int)n,
                             static_cast<int64_t *>(buf_a), static_cast<float *>(buf_b)));
  return PR_OK;
}

int rollout_destroy(pr_handle *h) {
  if (!h) return PR_EINVAL;
  delete h;
  return PR_OK;
}

const char *rollout_strerror(int code) {
  switch (code) {
    case PR_OK: return "ok";
    case PR_EINVAL: return "invalid argument";
    case PR_ENOMEM: return "workspace too small or out of host memory";
    case PR_EHIP: return "HIP call failed";
    case PR_EUNSUPPORTED: return "shape or schedule not covered by the kernels";
    case PR_ETOOBIG: return "request needs more than the fixed scratch of this no-allocation entry point";
    default: return "unknown status";
  }
}

int rollout_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
