// Generalised advantage estimation as a chunked reverse scan (implied by the
// paper's use of PPO, Sec. 5.2; see compute_gae in podrollout.h).
//
// The recurrence A_t = delta_t + c_t A_{t+1} is first-order linear, so a run of
// steps can be summarised by the pair (a, p) with A_first = a + p * A_after.
// One workgroup owns 64 consecutive envs (one per lane, so every load of a row
// is a contiguous 256-byte segment); each of its wavefronts owns a chunk of
// GAE_L consecutive steps, loads the whole chunk into registers (all loads in
// flight at once), scans it locally, publishes its (a, p) through LDS, composes
// the summaries of the later chunks to get its incoming A, and patches its
// results.  Segments of NW * GAE_L steps are walked from the end of the rollout
// to the start with the boundary advantage carried in a register; the rows of the
// next segment are requested before the current one is patched and stored.
#include "pod_internal.h"

namespace pod {

constexpr int GAE_L = 16;    // steps per wavefront chunk (register resident)
constexpr int GAE_NW = 16;   // wavefronts per workgroup

__global__ __launch_bounds__(GAE_NW * 64) void gae_kernel(int T, int N, const float *__restrict__ reward,
                                                         const float *__restrict__ value,
                                                         const uint8_t *__restrict__ done, float gamma, float gl,
                                                         float *__restrict__ adv, float *__restrict__ ret) {
  __shared__ float s_a[GAE_NW][64];
  __shared__ float s_p[GAE_NW][64];
  const int lane = threadIdx.x & 63;
  const int w = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  const bool live = n < N;
  const int seg = GAE_NW * GAE_L;
  float carry = 0.0f;  // advantage at the first step of the segment handled before (later in time)

  // chunks are numbered from the end of a segment: chunk w of the segment ending at hi covers [c_lo, c_lo + GAE_L)
  float r[GAE_L], v[GAE_L], v_after;
  uint8_t dn[GAE_L];
  auto load = [&](int hi, bool en, float (&r_)[GAE_L], float (&v_)[GAE_L], uint8_t (&dn_)[GAE_L], float &va_) {
    const int c_lo = hi - (w + 1) * GAE_L;
#pragma unroll
    for (int i = 0; i < GAE_L; ++i) {
      const int t = c_lo + i;
      const bool ok = en && live && t >= 0;
      const size_t idx = (size_t)(ok ? t : 0) * N + (live ? n : 0);
      r_[i] = ok ? __builtin_nontemporal_load(reward + idx) : 0.0f;
      v_[i] = ok ? __builtin_nontemporal_load(value + idx) : 0.0f;
      dn_[i] = ok ? __builtin_nontemporal_load(done + idx) : (uint8_t)1;
    }
    const int t = c_lo + GAE_L;  // <= T: value has T+1 rows
    va_ = (en && live && t >= 0) ? __builtin_nontemporal_load(value + (size_t)t * N + n) : 0.0f;
  };
  load(T, true, r, v, dn, v_after);

  for (int hi = T; hi > 0; hi -= seg) {
    const int c_lo = hi - (w + 1) * GAE_L;
    float a[GAE_L], p[GAE_L];
    // local scan, newest step first
    float a_next = 0.0f, p_next = 1.0f, v_next = v_after;
#pragma unroll
    for (int i = GAE_L - 1; i >= 0; --i) {
      const bool skip = (c_lo + i) < 0;  // before the start of the rollout: identity
      const float g = dn[i] ? 0.0f : gamma;
      const float c = dn[i] ? 0.0f : gl;
      const float delta = fmaf(g, v_next, r[i]) - v[i];
      const float ai = skip ? a_next : fmaf(c, a_next, delta);
      const float pi = skip ? p_next : c * p_next;
      a[i] = ai;
      p[i] = pi;
      a_next = ai;
      p_next = pi;
      v_next = v[i];
    }
    s_a[w][lane] = a_next;
    s_p[w][lane] = p_next;
    // the next (earlier) segment's rows are requested now, so that they travel while this segment's summaries
    // meet in LDS and its results are written
    float rn[GAE_L], vn[GAE_L], vn_after = 0.0f;
    uint8_t dnn[GAE_L];
    load(hi - seg, hi - seg > 0, rn, vn, dnn, vn_after);
    __syncthreads();
    // advantage just after this chunk = later chunks of the segment applied to the carry
    float a_in = carry;
    for (int c = 0; c < w; ++c) a_in = fmaf(s_p[c][lane], a_in, s_a[c][lane]);
    float seg_first = a_in;
    for (int c = w; c < GAE_NW; ++c) seg_first = fmaf(s_p[c][lane], seg_first, s_a[c][lane]);
    carry = seg_first;
#pragma unroll
    for (int i = 0; i < GAE_L; ++i) {
      const int t = c_lo + i;
      if (live && t >= 0) {
        const float A = fmaf(p[i], a_in, a[i]);
        const size_t idx = (size_t)t * N + n;
        __builtin_nontemporal_store(A, adv + idx);
        __builtin_nontemporal_store(A + v[i], ret + idx);
      }
    }
#pragma unroll
    for (int i = 0; i < GAE_L; ++i) r[i] = rn[i], v[i] = vn[i], dn[i] = dnn[i];
    v_after = vn_after;
    __syncthreads();  // summaries are rewritten by the next segment
  }
}

hipError_t launch_gae(hipStream_t st, int32_t T, int32_t N, const float *reward, const float *value,
                      const uint8_t *done, float gamma, float lambda, float *adv, float *ret) {
  const int blocks = (N + 63) / 64;
  hipLaunchKernelGGL(gae_kernel, dim3(blocks), dim3(GAE_NW * 64), 0, st, (int)T, (int)N, reward, value, done, gamma,
                     gamma * lambda, adv, ret);
  return hipGetLastError();
}

}  // namespace pod
