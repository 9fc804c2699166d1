/*
 * podrollout.h -- C ABI of the single-GPU rollout hot path of one pod.
 *
 * The paper describes a pod's worker as an actor interacting with a batched
 * environment of independent sub-environments to produce batches of
 * transitions (Sec. 4.2 "Worker"), with all data kept as tensors in contiguous
 * GPU memory (Sec. 4.3 "Cloud-oriented optimizations").  This library is that
 * worker for the stock-trading task of Table 1 / Sec. 5.3 (state: balance,
 * shares, close prices, technical indicators; actions: buy / sell / hold;
 * reward: change of account value; initial capital and proportional
 * transaction cost as in the caption of Fig. 6), plus the critic forward and
 * the advantage estimation that the PPO learner of Sec. 5.2 consumes, and the
 * leaderboard score of Sec. 4.1 (mean / variance of episodic reward).
 *
 * General rules
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - The caller owns every device buffer, including the workspace; the library
 *    borrows them: market and workspace for the life of the handle, all others
 *    until the work enqueued by the call has finished.  The library allocates
 *    only the small host-side handle.
 *  - Every call enqueues its work on the HIP stream given at init (or passed
 *    in, for compute_gae) and returns without synchronising.
 *  - Return value: PR_OK (0) or a negative pr_status.  Arguments are validated
 *    before any device work is enqueued, so a failed call changes nothing.
 *    No exceptions, no abort().
 *  - Row-major layouts; "[T, N, D]" means D is the fastest axis.
 *
 * Notation: N envs, P agents (env n belongs to agent n / (N/P)), D stocks,
 * K indicators per stock, S = 1 + 2D + DK state width, Hd hidden width,
 * H episode horizon (market has H+1 rows), M market paths, T rollout steps.
 */
#ifndef PODROLLOUT_H
#define PODROLLOUT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pr_status {
  PR_OK = 0,
  PR_EINVAL = -1,       /* bad shape, null pointer, scale not a power of two, ... */
  PR_ENOMEM = -2,       /* workspace too small / host handle allocation failed    */
  PR_EHIP = -3,         /* a HIP call failed; see rollout_last_hip_error()        */
  PR_EUNSUPPORTED = -4, /* valid request outside the shapes the kernels cover     */
  PR_ETOOBIG = -5       /* request needs more than the fixed scratch of a no-allocation entry point */
} pr_status;

enum { PR_MLP_F32 = 0, PR_MLP_BF16 = 1 };        /* pr_config.mlp_dtype */
enum { PR_SCHED_STEPWISE = 0, PR_SCHED_FUSED = 1 }; /* pr_config.schedule  */
enum { PR_NET_ACTOR = 0, PR_NET_CRITIC = 1 };

/* Plain data, copied at init. */
typedef struct pr_config {
  int32_t n_envs;       /* N >= 1 */
  int32_t n_agents;     /* P >= 1, N % P == 0 */
  int32_t n_stocks;     /* D >= 1 */
  int32_t n_ind;        /* K >= 0 */
  int32_t hidden;       /* Hd, multiple of 32 */
  int32_t horizon;      /* H >= 1 */
  int32_t n_market;     /* M in {1, N}: env n reads market path n % M */
  int32_t mlp_dtype;    /* PR_MLP_F32: fp32 operands on fp32 matrix cores;
                           PR_MLP_BF16: observations, weights and hidden
                           activations rounded to bf16 (nearest-even),
                           fp32 accumulate, fp32 bias / tanh / outputs */
  int32_t schedule;     /* PR_SCHED_STEPWISE: one actor launch and one env launch
                           per step; PR_SCHED_FUSED: one persistent launch that
                           keeps each env tile on one compute unit for all T
                           steps (bf16 networks with 256 or 512 hidden units,
                           fp32 networks with 256; D <= 32, D K <= 252 and a
                           multiple of 4; else PR_EUNSUPPORTED at init).  Given the
                           same policy means, the same results bit for bit. */
  float cash0;          /* initial capital (> 0) */
  float hmax;           /* largest trade per stock and step, in shares */
  float cost;           /* proportional transaction cost c, 0 <= c < 1 */
  float sigma;          /* fixed std of the Gaussian policy (> 0) */
  float reward_scale;   /* rho: reward = rho * change of account value */
  float obs_scale[4];   /* cash, price, holdings, indicator; positive powers of two */
} pr_config;

/* Market paths (Table 1: close prices, technical indicators). */
typedef struct pr_market {
  const float *price;   /* [H+1, M, D]   > 0 */
  const float *ind;     /* [H+1, M, D*K] stock-major; may be NULL when K == 0 */
} pr_market;

/* One network 3-layer perceptron per agent, fp32, weights [in, out] row-major:
 * W1 [P, S, Hd], b1 [P, Hd], W2 [P, Hd, Hd], b2 [P, Hd], W3 [P, Hd, O],
 * b3 [P, O]; O = D for the actor (tanh after every layer, output included),
 * O = 1 for the critic (tanh on the hidden layers, linear output). */
typedef struct pr_weights {
  const float *W1, *b1, *W2, *b2, *W3, *b3;
} pr_weights;

/* The rollout buffer: what the worker hands to the learner.  "opt" pointers
 * may be NULL and are then not written. */
typedef struct pr_buffers {
  float *obs;        /* [T+1, N, S] observation before each step, and the last one:
                        [cash*s0, price_d*s1, holdings_d*s2, ind_{d,k}*s3]         */
  float *act_raw;    /* [T, N, D]   sampled action mu + sigma*eps, before clamping */
  float *reward;     /* [T, N]                                                     */
  uint8_t *done;     /* [T, N]      1 where the step ended an episode              */
  float *value;      /* opt [T+1, N] critic value of every observation             */
  float *logp;       /* opt [T, N]  log-density of act_raw under the policy        */
  float *mu;         /* opt [T, N, D] policy mean                                  */
  int32_t *shares;   /* opt [T, N, D] executed trades, signed (+ buy, - sell)      */
} pr_buffers;

/* Per-env state, env-major user layout, for inspection and for planting a
 * state in tests.  Any pointer may be NULL (skipped). */
typedef struct pr_state {
  float *cash;       /* [N]    */
  int32_t *holdings; /* [N, D] */
  int32_t *cursor;   /* [N]    market row of the current observation, start_n <= tau < start_n + H
                                (start_n = 0 unless rollout_set_replay gave start rows)      */
  double *ep_return; /* [N]    return accumulated in the running episode           */
  double *ep_sum;    /* [N]    sum of the returns of finished episodes             */
  double *ep_sqsum;  /* [N]    sum of their squares                                */
  int32_t *ep_count; /* [N]    number of finished episodes                         */
} pr_state;

typedef struct pr_handle pr_handle;

/* Device bytes rollout_init needs in `workspace` for this config (packed
 * weights, env state, per-step scratch).  out: host pointer. */
int rollout_workspace_bytes(const pr_config *cfg, size_t *out);

/* LDS bytes per workgroup the persistent rollout kernel (Sec. 4.2 worker, the
 * PR_SCHED_FUSED schedule) is launched with for this config: with_actor != 0
 * for rollout_step_T, 0 for rollout_step_forced.  The launch reads the same
 * carve-up, so this IS the launch size; it never exceeds 160 KiB for a config
 * the schedule accepts.  out: host pointer.  PR_EUNSUPPORTED when the schedule
 * does not cover the shape (no device work either way). */
int rollout_kernel_lds_bytes(const pr_config *cfg, int32_t with_actor, size_t *out);

/* Create a rollout worker (Sec. 4.2).  Packs both networks into the layout the
 * matrix-core kernels read, puts every env at (cash0, no shares, cursor 0).
 * cfg, market, actor, critic: host structs holding device pointers.
 * workspace: device, 256-byte aligned, >= rollout_workspace_bytes.
 * hip_stream: a hipStream_t (NULL = default stream); all later calls on the
 * handle enqueue there.  out: host pointer receiving the handle.
 * PR_EUNSUPPORTED when Hd, D or the schedule is outside what the kernels cover
 * (Hd % 32 != 0, Hd > 1024, P > 1 with N/P not a multiple of 64, fused
 * schedule with a shape it does not implement). */
int rollout_init(const pr_config *cfg, const pr_market *market, const pr_weights *actor, const pr_weights *critic,
                 void *workspace, size_t workspace_bytes, void *hip_stream, pr_handle **out);

/* Replace both networks (a new policy for the same envs); env state is kept. */
int rollout_set_weights(pr_handle *h, const pr_weights *actor, const pr_weights *critic);

/* All envs back to cash0, no shares, cursor at their start row (0 unless
 * rollout_set_replay gave others); episode statistics cleared. */
int rollout_reset(pr_handle *h);

/* Replay of one long historical table from per-env start rows (Sec. 5.3: every
 * env trades the same minute-level data set; Sec. 4.2 vectorised sub-environments).
 * table: price [table_rows, M, D], ind [table_rows, M, D*K] (device; same M, D, K as
 * the config; M = 1 is the shared-table case).  start: device [N], copied.  From now
 * on env n's episodes run over rows start_n .. start_n + H: done after H steps, then
 * back to cash0, no shares, cursor start_n.  Requires table_rows >= H + 1 and
 * 0 <= start_n <= table_rows - 1 - H for every env (checked on the device; the call
 * synchronises the stream), else PR_EINVAL and nothing changes.  Resets all envs
 * like rollout_reset.  Do not call during stream capture. */
int rollout_set_replay(pr_handle *h, const pr_market *table, int32_t table_rows, const int32_t *start);

/* T steps of agent-environment interaction for all N envs (Sec. 4.2 worker;
 * Table 1 stock trading):
 *   obs_t -> actor -> mu_t;  a = mu_t + sigma * noise_t;  k_d = trunc(clamp(a_d,-1,1) * hmax);
 *   every sale in ascending stock order (at most the holding, proceeds * (1-c)),
 *   then every purchase in ascending stock order (at most what the cash left pays for at price * (1+c));
 *   cursor += 1; reward = rho * (account value at the new prices - account value before);
 *   done when the cursor reaches H, then the env restarts from cash0 with no shares at cursor 0.
 * Then, if out->value is given, the critic on all T+1 observations.
 * noise: [T, N, D] standard-normal draws supplied by the caller.
 * Env state persists in the handle: obs row 0 of a call is the last
 * observation of the previous call.  T >= 1. */
int rollout_step_T(pr_handle *h, int32_t T, const float *noise, const pr_buffers *out);

/* The same T steps with the policy mean supplied by the caller instead of the
 * actor (mu: [T, N, D]); the critic is not run and out->value, out->mu are
 * ignored.  This is the environment + sampling stage on its own. */
int rollout_step_forced(pr_handle *h, int32_t T, const float *mu, const float *noise, const pr_buffers *out);

/* One network on its own: rows of X ([rows, S], row stride ldx floats) through
 * the actor (Y [rows, D]) or the critic (Y [rows]) of the agent that owns env
 * (row % N).  This is the kernel rollout_step_T uses for the critic and, in the
 * stepwise schedule, for the actor. */
int rollout_mlp_forward(pr_handle *h, int32_t net, int64_t rows, const float *X, int64_t ldx, float *Y);

/* Copy the per-env state out of / into the handle (device buffers). */
int rollout_get_state(pr_handle *h, const pr_state *out);
int rollout_set_state(pr_handle *h, const pr_state *in);

/* Generalised advantage estimation (implied by PPO, Sec. 5.2), per env,
 * backwards over t, with nd_t = 1 - done_t:
 *   delta_t = r_t + gamma nd_t V_{t+1} - V_t;  A_t = delta_t + gamma lambda nd_t A_{t+1}, A_T = 0;  R_t = A_t + V_t.
 * Stateless.  reward, done: [T, N]; value: [T+1, N]; adv, ret: [T, N] outputs.
 * hip_stream: hipStream_t to enqueue on.  T >= 1, N >= 1. */
int compute_gae(void *hip_stream, int32_t T, int32_t N, const float *reward, const float *value, const uint8_t *done,
                float gamma, float lambda, float *adv, float *ret);

/* Trading performance of a recorded rollout (Sec. 5.3 "Performance metrics"; the evaluator of Sec. 4.2 reports
 * it next to the episodic reward), per env, over the FIRST episode in the buffer: points t = 0 .. L with L the
 * first step whose done flag is set (the observation after it is a reset observation), else T.  The account value
 *   V_t = cash_t + sum_d holdings_{t,d} price_{t,d}
 * is decoded from obs (layout and scales as rollout_step_T writes them) in binary64; r_t = V_{t+1} / V_t - 1.
 *   metrics[0][n] cumulative return  (V_L - V_0) / V_0
 *   metrics[1][n] annual return      (V_L / V_0)^(periods_per_year / L) - 1
 *   metrics[2][n] annual volatility  sqrt(periods_per_year) * sample standard deviation of r   (0 when L < 2)
 *   metrics[3][n] maximum drawdown   max_t (1 - V_t / max_{s <= t} V_s)
 *   metrics[4][n] Sharpe ratio       sqrt(periods_per_year) (mean(r) - risk_free / periods_per_year) / std(r), 0 if std = 0
 *   metrics[5][n] Calmar ratio       annual return / maximum drawdown, 0 if the drawdown is 0
 * (the paper names the five figures in words; periods per year, the risk-free rate and the sample estimator are
 * this library's parameters / reading).  L = 0 gives zeros.
 * Stateless.  Device pointers: obs [T+1, N, state_dim], done [T, N], metrics [6, N] (binary64, output),
 * length [N] (output L, may be NULL).  obs_scale: HOST pointer to the 4 scales of pr_config (powers of two).
 * state_dim >= 1 + 2 n_stocks.  Only enqueues on hip_stream; PR_EINVAL on bad arguments. */
int trading_metrics(void *hip_stream, int32_t T, int32_t N, int32_t n_stocks, int32_t state_dim, const float *obs,
                    const uint8_t *done, const float *obs_scale, double periods_per_year, double risk_free,
                    double *metrics, int32_t *length);

/* Generator / updater step on a population held on this GPU (Sec. 4.1: the leaderboard records the candidate
 * agents with high performance, the generator produces the training files of a new pod from a candidate and may
 * mutate them).  params [P, count]: one row per agent -- any tensor of pr_weights viewed as [P, count]; call once
 * per tensor with the same rank.  rank [P]: agent ids, best first, a permutation of 0..P-1 (what
 * rollout_leaderboard writes).  The first `keep` agents of rank are left as they are; agent rank[j], j >= keep,
 * is overwritten in place with
 *     fl32( params[rank[(j - keep) % keep]] + fl32(sigma * noise[rank[j]]) )      (element-wise, binary32).
 * noise [P, count] (rows of kept agents are not read); may be NULL when sigma == 0 (plain copies).  The random
 * numbers are the caller's.  Entries of rank outside 0..P-1 leave that agent untouched.
 * Stateless; device pointers; only enqueues on hip_stream.  1 <= keep <= P <= 65535, count >= 1.
 * Follow with rollout_set_weights to let the rollout use the new population. */
int population_refill(void *hip_stream, int32_t P, int64_t count, const int32_t *rank, int32_t keep, float sigma,
                      const float *noise, float *params);

/* ---- the learner's minibatch (Sec. 4.2 "Learner": fetch a batch of transitions from the buffer and train the
 * networks; Sec. 5.2: PPO with batch size 1024 and learning rate 1e-3).  The paper names PPO and stops there; this
 * is its clipped-surrogate objective for the fixed-deviation Gaussian policy of the rollout, one agent:
 *   mu = actor(obs), V = critic(obs)                    (same networks as pr_weights with P = 1)
 *   logp = sum_d -(a_d - mu_d)^2 / (2 sigma^2) - D ln sigma - D/2 ln(2 pi),    ratio = exp(logp - logp_old)
 *   L = -(1/B) sum_b min(ratio A, clip(ratio, 1 - clip, 1 + clip) A)  +  value_coef (1/B) sum_b (V - R)^2 / 2
 * (a sample passes policy gradient when ratio A <= clip(ratio) A).  Advantages are used as given. */
typedef struct pr_ppo_config {
  int32_t batch;                 /* B >= 1 rows in the minibatch                          */
  int32_t n_stocks, n_ind, hidden;  /* D, K, Hd: S = 1 + 2 D + D K inputs, Hd % 32 == 0      */
  float sigma, clip, value_coef;
  float lr, beta1, beta2, adam_eps; /* Adam (used by ppo_learner_step only)                 */
  int32_t adam_step;             /* t >= 1: number of this update, for the bias correction */
} pr_ppo_config;

/* One network's tensors, fp32, device, layouts of pr_weights without the agent axis; mutable. */
typedef struct pr_net_params {
  float *W1, *b1, *W2, *b2, *W3, *b3;
} pr_net_params;

/* Bytes of device scratch the two calls below need (256-byte aligned, caller-owned). */
int ppo_workspace_bytes(const pr_ppo_config *cfg, size_t *out);

/* Gradients of L for one minibatch.  obs [R, S], act_raw [R, D], logp_old, adv, ret [R]: the rollout buffers
 * flattened over (t, n); rows [B]: which of the R rows form the minibatch (NULL: rows 0 .. B-1).
 * actor, critic: parameters (read); grad_actor, grad_critic: outputs, same shapes.
 * stats (device, 4 floats, may be NULL): policy loss, value loss (unweighted), fraction of samples whose
 * surrogate is cut by the min(), mean ratio.  Only enqueues on hip_stream; no allocation. */
int ppo_minibatch_grads(void *hip_stream, const pr_ppo_config *cfg, const float *obs, const float *act_raw,
                        const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                        const pr_net_params *actor, const pr_net_params *critic, const pr_net_params *grad_actor,
                        const pr_net_params *grad_critic, void *workspace, size_t workspace_bytes, float *stats);

/* ppo_minibatch_grads for callers that cannot allocate device memory and own no workspace: code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * results bit for bit, but the scratch lives in a fixed device array inside the library:
 * PR_STATIC_SCRATCH_BYTES (24 MiB) per GPU the library is used on, held until the process ends -- enough for the
 * paper's minibatch of 1024 with 512 hidden units and 30 stocks x 8 indicators (22.5 MB); ppo_workspace_bytes minus
 * the gradient tensors is what a shape needs.  A shape that needs more is refused with PR_ETOOBIG before any device
 * work.  The call allocates nothing (no hipMalloc / hipFree, no allocating library routine) and only enqueues on
 * hip_stream.  All calls on one GPU share that GPU's array, which keeps the previous call's contents (nothing in
 * it has to start at zero): calls whose device work overlaps on one GPU -- two streams, two host threads -- race;
 * serialise them.  The first call on a device looks up the array's address there (not a stream operation, so make
 * that first call outside graph capture). */
#define PR_STATIC_SCRATCH_BYTES ((size_t)24 << 20)
int ppo_minibatch_grads_noalloc(void *hip_stream, const pr_ppo_config *cfg, const float *obs, const float *act_raw,
                                const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                                const pr_net_params *actor, const pr_net_params *critic,
                                const pr_net_params *grad_actor, const pr_net_params *grad_critic, float *stats);

/* Adam on one tensor of n elements:  m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;
 *   theta -= lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps).  All device, fp32, in place. */
int adam_update(void *hip_stream, int64_t n, float *theta, const float *grad, float *m, float *v, float lr, float beta1,
                float beta2, float eps, int32_t t);

/* ppo_minibatch_grads followed by adam_update on all twelve tensors (gradients live in the workspace).
 * m_*, v_*: Adam moments, same shapes as the parameters, zero before the first step. */
int ppo_learner_step(void *hip_stream, const pr_ppo_config *cfg, const float *obs, const float *act_raw,
                     const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                     const pr_net_params *actor, const pr_net_params *critic, const pr_net_params *m_actor,
                     const pr_net_params *v_actor, const pr_net_params *m_critic, const pr_net_params *v_critic,
                     void *workspace, size_t workspace_bytes, float *stats);

/* Leaderboard score of every agent (Sec. 4.1; Sec. 4.2 evaluator): mean and
 * population variance of the returns of the episodes its envs have finished
 * since the last reset, and the agents ordered best first (equal means: lower
 * id first; agents without a finished episode score -inf and come last).
 * score_mean, score_var: [P] f64; rank: [P] agent ids. */
int rollout_leaderboard(pr_handle *h, double *score_mean, double *score_var, int32_t *rank);

/* Machine calibration for the roofline figures reported beside the worker's throughput (the paper names data
 * collection as the bottleneck, Sec. 1 and Sec. 4.2, and prints no kernel-level figure; the kernels of this library
 * are therefore measured against what this chip delivers).  Enqueues ONE launch on hip_stream; timing it (events)
 * is the caller's business.  Stateless, allocates nothing.
 *   kind PR_CAL_COPY:  streams n bytes from buf_a to buf_b (device, 16-byte aligned, n % 16 == 0).
 *   kind PR_CAL_READ:  streams n bytes from buf_a; buf_b: device, >= 4 bytes (never written in practice).
 *   kind PR_CAL_PROBE: n workgroups of up to 8 wavefronts, each wavefront playing the role params[w]
 *        (0 none, 1 matrix: params[8] trips of 8 independent bf16 32x32x16 matrix instructions, 2 vector:
 *        params[9] trips of 32 tanh-epilogue activations per lane, 3 both in one wavefront: params[10] in
 *        {0, 2, 4, 6, 8} activations issued behind every 8 matrix instructions, 4 plain: as 2 with full-rate
 *        instructions only); params[11] != 0: the matrix role also reads its operand from LDS, 16 bytes per
 *        instruction.  buf_a: device int64 [n, 8], receives each wavefront's elapsed time in 10 ns ticks (entries of
 *        wavefronts without a role are left alone); buf_b: device, >= 4 bytes.
 * params: HOST pointer to 12 int32 (PR_CAL_PROBE only, else may be NULL).  PR_EINVAL on bad arguments. */
enum { PR_CAL_COPY = 0, PR_CAL_READ = 1, PR_CAL_PROBE = 2 };
int rollout_calibrate(void *hip_stream, int32_t kind, int64_t n, const int32_t *params, void *buf_a, void *buf_b);

/* Free the host handle.  Device memory stays with the caller. */
int rollout_destroy(pr_handle *h);

/* Static text for a pr_status (host string, never NULL). */
const char *rollout_strerror(int code);

/* hipError_t value of the last failed HIP call on this thread (0 if none). */
int rollout_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PODROLLOUT_H */
