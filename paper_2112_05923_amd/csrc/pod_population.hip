// Generator / updater step for a population that lives on one GPU (Sec. 4.1:
// the leaderboard keeps the candidate agents with high performance; the
// generator produces the training files of a new pod from a candidate and may
// mutate them).  One parameter block [P, count], one row per agent: the first
// `keep` agents of the ranking stay, agent rank[j] (j >= keep) becomes
// candidate rank[(j - keep) % keep] plus sigma * noise[rank[j]].
//
// Pure streaming: 12 bytes per rewritten parameter (parent and noise in, child
// out).  Candidates are only read and losers only written, so the update is
// safe in place.  Compiled without contraction: child = fl32(parent +
// fl32(sigma z)), the same two roundings on every implementation.
#include "pod_internal.h"

namespace pod {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool VEC>
__global__ __launch_bounds__(256) void population_refill_kernel(int P, int64_t count, const int32_t *__restrict__ rank,
                                                                 int keep, float sigma, const float *noise,
                                                                 float *params) {
  const int j = keep + blockIdx.y;  // position in the ranking of the agent this block row rewrites
  const int64_t child = rank[j], parent = rank[(j - keep) % keep];
  if (child < 0 || child >= P || parent < 0 || parent >= P || child == parent) return;  // not a ranking: leave it
  const float *src = params + parent * count;
  const float *z = noise ? noise + child * count : nullptr;
  float *dst = params + child * count;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (VEC) {
    const int64_t n4 = count >> 2;
    for (; i < n4; i += stride) {
      f32x4 v = reinterpret_cast<const f32x4 *>(src)[i];
      if (z) {
        const f32x4 e = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(z) + i);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float step = sigma * e[q];
          v[q] = v[q] + step;
        }
      }
      reinterpret_cast<f32x4 *>(dst)[i] = v;
    }
  } else {
    for (; i < count; i += stride) {
      float v = src[i];
      if (z) {
        const float step = sigma * z[i];
        v = v + step;
      }
      dst[i] = v;
    }
  }
}

}  // namespace

hipError_t launch_population_refill(hipStream_t st, int32_t P, int64_t count, const int32_t *rank, int32_t keep,
                                    float sigma, const float *noise, float *params) {
  if (keep >= P) return hipSuccess;
  // 16-byte accesses when every row starts on a 16-byte boundary
  const bool vec = count % 4 == 0 && (reinterpret_cast<uintptr_t>(params) & 15u) == 0 &&
                   (!noise || (reinterpret_cast<uintptr_t>(noise) & 15u) == 0);
  const int64_t work = vec ? count / 4 : count;
  int64_t bx = (work + 255) / 256;
  if (bx > 4096) bx = 4096;
  if (bx < 1) bx = 1;
  const dim3 grid((unsigned)bx, (unsigned)(P - keep));
  if (vec)
    hipLaunchKernelGGL(population_refill_kernel<true>, grid, dim3(256), 0, st, P, count, rank, keep, sigma, noise, params);
  else
    hipLaunchKernelGGL(population_refill_kernel<false>, grid, dim3(256), 0, st, P, count, rank, keep, sigma, noise,
                       params);
  return hipGetLastError();
}

}  // namespace pod
