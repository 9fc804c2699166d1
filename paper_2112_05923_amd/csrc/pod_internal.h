// Internal declarations shared by the HIP translation units of libpodrollout.
// Host-side launchers only; every kernel lives in the .hip file that defines
// its launcher.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "podrollout.h"

namespace pod {

// Kernels that use more than the default 64 KiB of dynamic LDS need the limit raised once per device (the
// attribute belongs to that device's copy of the code object).  One bit per device ordinal and kernel; safe to
// call from several host threads (a second call on a device is harmless).
constexpr int kMaxLdsBytes = 160 * 1024;
template <auto Kern>
inline hipError_t allow_full_lds() {
  static std::atomic<uint64_t> done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          kMaxLdsBytes);
  if (e != hipSuccess) return e;
  if (dev < 64) done.fetch_or(bit, std::memory_order_release);
  return hipSuccess;
}

// ---------------------------------------------------------------- env state
// Structure-of-arrays env state in the workspace; n is the fastest axis of
// every array so that a tile of consecutive envs is one contiguous segment.
struct EnvState {
  float *cash;       // [N]
  int32_t *tau;      // [N]
  int32_t *h;        // [D][N]
  double *ep_ret;    // [N]
  double *ep_sum;    // [N]
  double *ep_sqsum;  // [N]
  int32_t *ep_cnt;   // [N]
  const int32_t *start;  // [N] table row every episode of the env begins at (0 unless a replay table is set)
};

struct EnvDims {
  int32_t N, D, K, S, H, M;
  float cash0, hmax, one_minus_c, one_plus_c, sigma, rho;
  float logp_const;  // -D * (ln sigma + 0.5 ln 2 pi)
  float s_cash, s_price, s_hold, s_ind;
};

struct StepIO {
  const float *mu;     // [N, D] policy mean of this step
  const float *noise;  // [N, D]
  float *obs_next;     // [N, S] observation after the step
  float *act_raw;      // [N, D]
  float *reward;       // [N]
  uint8_t *done;       // [N]
  float *logp;         // [N] or null
  int32_t *shares;     // [N, D] or null
};

hipError_t launch_observe(hipStream_t st, const EnvDims &d, const EnvState &s, const float *price, const float *ind,
                          float *obs);
hipError_t launch_env_step(hipStream_t st, const EnvDims &d, const EnvState &s, const float *price, const float *ind,
                           const StepIO &io);
hipError_t launch_state_reset(hipStream_t st, const EnvDims &d, const EnvState &s);
hipError_t launch_check_starts(hipStream_t st, int32_t N, int32_t H, int32_t rows, const int32_t *start, int32_t *bad);
hipError_t launch_state_copy(hipStream_t st, const EnvDims &d, const EnvState &s, const pr_state &user, bool to_user);
hipError_t launch_leaderboard(hipStream_t st, int32_t N, int32_t P, const EnvState &s, double *scratch_mean,
                              double *score_mean, double *score_var, int32_t *rank);
size_t env_step_lds_bytes(const EnvDims &d, int *envs_per_block);

// ---------------------------------------------------------------------- GAE
// obs_scale: host pointer to the four observation scales.
hipError_t launch_trading_metrics(hipStream_t st, int32_t T, int32_t N, int32_t D, int32_t S, const float *obs,
                                  const uint8_t *done, const float *obs_scale, double periods, double rf,
                                  double *metrics, int32_t *length);
hipError_t launch_population_refill(hipStream_t st, int32_t P, int64_t count, const int32_t *rank, int32_t keep,
                                    float sigma, const float *noise, float *params);
size_t ppo_scratch_bytes(int B, int Hd, int D, int S);
hipError_t launch_ppo_grads(hipStream_t st, const pr_ppo_config &c, const float *obs, const float *act,
                            const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                            const pr_net_params &actor, const pr_net_params &critic, const pr_net_params &ga,
                            const pr_net_params &gc, void *scratch, float *stats);
// The same with the scratch in a fixed device array of ppo_static_scratch_bytes() (no workspace, no allocation);
// hipErrorInvalidValue when the shape needs more.
size_t ppo_static_scratch_bytes();
hipError_t launch_ppo_grads_static(hipStream_t st, const pr_ppo_config &c, const float *obs, const float *act,
                                   const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                                   const pr_net_params &actor, const pr_net_params &critic, const pr_net_params &ga,
                                   const pr_net_params &gc, float *stats);
hipError_t launch_adam12(hipStream_t st, const int64_t *n, float *const *theta, float *const *g, float *const *m,
                         float *const *v, float lr, float b1, float b2, float eps, int32_t t);
hipError_t launch_adam(hipStream_t st, int64_t n, float *theta, const float *g, float *m, float *v, float lr, float b1,
                       float b2, float eps, int32_t t);
hipError_t launch_gae(hipStream_t st, int32_t T, int32_t N, const float *reward, const float *value,
                      const uint8_t *done, float gamma, float lambda, float *adv, float *ret);

// -------------------------------------------------------------- calibration
hipError_t launch_calib_copy(hipStream_t st, const void *src, void *dst, int64_t bytes, int blocks);
hipError_t launch_calib_read(hipStream_t st, const void *src, void *sink, int64_t bytes, int blocks);
hipError_t launch_calib_probe(hipStream_t st, const int32_t role_of_wave[8], int32_t iters_matrix,
                              int32_t iters_vector, int32_t acts_per_group, int32_t lds_reads, int blocks,
                              int64_t *ticks, float *sink);

// ---------------------------------------------------------------------- MLP
// Packed network of one agent set.  Weight blocks are stored in the register
// layout of the matrix-core instruction: block (kb, ct) holds, for the 64 lanes
// of a wavefront, the 16 bytes lane l feeds as operand for output features
// [32 ct, 32 ct + 32) and inputs [KB kb, KB kb + KB); KB = 16 (bf16) or 8 (fp32).
// Blocks are ordered k-major: [kb][ct][lane].
struct PackedNet {
  const void *W[3];       // packed weights per layer, agent-major
  const float *b[3];      // biases padded to a multiple of 32, agent-major
  int64_t w_stride[3];    // bytes between agents
  int32_t b_stride[3];    // floats between agents
  int32_t in_dim[3], out_dim[3];  // logical sizes
  int32_t nkb[3], nct[3];         // k-blocks and column tiles per layer
  int32_t bf16;                   // operand type
  int32_t out_tanh;               // tanh on the last layer
  float *split_h[2];              // scratch for the layer-per-launch path: two [split_rows, hidden] fp32 buffers, or null
  int64_t split_rows;
};
// Rows up to which the layer-per-launch path is worth its scratch (fewer 64-row tiles than half the compute units
// of the largest part), 0 if never for this batch size.
int64_t split_scratch_rows(int64_t n_envs, int hidden);

size_t packed_weight_bytes(int in_dim, int out_dim, int bf16);
int padded_out(int out_dim);
// k_rot > 0: packed k row k' holds input row (k' < k_rot ? in_dim - k_rot + k' : k' - k_rot), i.e. the last k_rot
// inputs come first.
hipError_t launch_pack_layer(hipStream_t st, const float *W, const float *b, int P, int in_dim, int out_dim, int bf16,
                             int k_rot, void *Wp, float *bp);
// rows of X [rows, ldx] -> Y [rows, out_dim[2]]; row r uses agent ((r % N) / envs_per_agent).
hipError_t launch_mlp(hipStream_t st, const PackedNet &net, int64_t rows, const float *X, int64_t ldx, float *Y,
                      int32_t N, int32_t envs_per_agent);
bool mlp_supported(int S, int Hd, int O, int bf16);

// ------------------------------------------------------- persistent rollout
// One launch for T steps: each workgroup keeps 64 envs on its compute unit (actor forward, sampling, trading
// step, observation assembly).  mu_forced != null replaces the actor by caller-supplied means.
bool fused_supported(const pr_config &c);
size_t fused_lds_bytes(const pr_config &c, bool with_actor);
hipError_t launch_rollout_fused(hipStream_t st, const pr_config &c, const EnvDims &d, const EnvState &s,
                                const float *price, const float *ind, const PackedNet &actor, int32_t envs_per_agent,
                                int32_t T, const float *noise, const float *mu_forced, const pr_buffers &out);

}  // namespace pod
