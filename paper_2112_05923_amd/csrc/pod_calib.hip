// Machine calibration for the roofline figures that are reported next to the
// worker's throughput (Sec. 4.2: the rollout is the data-collection bottleneck
// the paper sets out to remove, so its kernels are measured against what the
// chip can deliver): a streaming copy, a streaming read, a matrix-core-only
// loop, and a family of small probes that show how matrix instructions and the
// vector / transcendental instructions of a tanh epilogue share one SIMD --
// issued by different wavefronts of the SIMD, or interleaved in one wavefront.
// None of the method's arithmetic lives here.
#include "pod_internal.h"

namespace pod {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------ memory streams
__global__ __launch_bounds__(256) void calib_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                         int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(256) void calib_read_kernel(const u32x4 *__restrict__ src, uint32_t *__restrict__ sink,
                                                         int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // (practically never: keeps the loads alive)
}

// ------------------------------------------------- matrix / vector co-issue
// Roles of a wavefront inside one probe launch.
enum Role { ROLE_NONE = 0, ROLE_MATRIX = 1, ROLE_VECTOR = 2, ROLE_BOTH = 3, ROLE_PLAIN = 4 };

constexpr int kMfmaPerIter = 8;   // independent accumulators: no dependent matrix instruction within 8 issues
constexpr int kActsPerIter = 32;  // independent tanh chains per lane in the vector role

// One activation of the bf16 networks' hidden-layer epilogue: scale-and-bias, exp2, add, rcp, fma.
__device__ inline float act_step(float x, float b) {
  const float t = fmaf(x, 2.8853900817779268f, b);
  const float e = __builtin_amdgcn_exp2f(t);
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
}

// The same number of plain full-rate instructions without the two transcendentals.
__device__ inline float plain_step(float x, float b) {
  float t = fmaf(x, 0.999f, b);
  t = fmaf(t, 0.5f, b);
  t = t + 1.0f;
  t = fmaf(t, 0.25f, b);
  return fmaf(-0.125f, t, 1.0f);
}

struct ProbeArgs {
  int32_t role_of_wave[8];   // Role per wavefront index of the workgroup
  int32_t iters_matrix;      // loop trips of the matrix role (8 matrix instructions each)
  int32_t iters_vector;      // loop trips of the vector role (32 activations per lane each)
  int32_t acts_per_group;    // ROLE_BOTH: activations issued behind every matrix instruction group of 8
  int32_t lds_reads;         // matrix role: one 16-byte LDS read per matrix instruction (operand fetch), 0 / 1
  int64_t *ticks;            // [blocks][8] elapsed 100 MHz ticks per wavefront
  float *sink;
};

template <int ACTS>
__device__ inline void both_loop(f32x16 (&acc)[kMfmaPerIter], float (&x)[kActsPerIter], const bf16x8 &a,
                                 const bf16x8 &b, int iters, float bias) {
  // (four trips per loop body so that the activation slots are compile-time register indices)
  for (int it = 0; it < iters; it += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int m = 0; m < kMfmaPerIter; ++m) {
        acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m], 0, 0, 0);
        // ACTS activations spread over the 8 matrix instructions of the group, in program order behind them
#pragma unroll
        for (int j = 0; j < ACTS; ++j)
          if (j % kMfmaPerIter == m) {
            constexpr int dummy = 0;
            (void)dummy;
            const int s = (u * ACTS + j) % kActsPerIter;
            x[s] = act_step(x[s], bias);
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
}

__global__ __launch_bounds__(512) void calib_probe_kernel(ProbeArgs p) {
  __shared__ __align__(16) unsigned char lds[32 * 1040];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int role = p.role_of_wave[wave];
  // operands and state from the lane index, so nothing folds away
  const float seed = (float)(lane + 1) * (1.0f / 64.0f);
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)(seed + 0.01f * i);
    b[i] = (__bf16)(0.5f - 0.003f * i * seed);
  }
  f32x16 acc[kMfmaPerIter];
#pragma unroll
  for (int m = 0; m < kMfmaPerIter; ++m)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[m][i] = 0.0f;
  float x[kActsPerIter];
#pragma unroll
  for (int j = 0; j < kActsPerIter; ++j) x[j] = seed * (0.1f + 0.01f * j);
  for (int i = threadIdx.x; i < 32 * 1040 / 4; i += blockDim.x) reinterpret_cast<uint32_t *>(lds)[i] = 0x3c003c00u;
  __syncthreads();
  const float bias = 0.01f * seed;
  const unsigned char *xrow = lds + (size_t)(lane & 31) * 1040 + 16 * (lane >> 5);

  const int64_t t0 = wall_clock64();
  if (role == ROLE_MATRIX) {
    if (p.lds_reads) {
      for (int it = 0; it < p.iters_matrix; ++it) {
        u32x4 xv[kMfmaPerIter];
#pragma unroll
        for (int m = 0; m < kMfmaPerIter; ++m) xv[m] = *reinterpret_cast<const u32x4 *>(xrow + ((it * 8 + m) & 31) * 32);
#pragma unroll
        for (int m = 0; m < kMfmaPerIter; ++m)
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, xv[m]), acc[m], 0, 0, 0);
      }
    } else {
      for (int it = 0; it < p.iters_matrix; ++it) {
#pragma unroll
        for (int m = 0; m < kMfmaPerIter; ++m) acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m], 0, 0, 0);
      }
    }
  } else if (role == ROLE_VECTOR) {
    for (int it = 0; it < p.iters_vector; ++it) {
#pragma unroll
      for (int j = 0; j < kActsPerIter; ++j) x[j] = act_step(x[j], bias);
    }
  } else if (role == ROLE_PLAIN) {
    for (int it = 0; it < p.iters_vector; ++it) {
#pragma unroll
      for (int j = 0; j < kActsPerIter; ++j) x[j] = plain_step(x[j], bias);
    }
  } else if (role == ROLE_BOTH) {
    switch (p.acts_per_group) {
      case 2: both_loop<2>(acc, x, a, b, p.iters_matrix, bias); break;
      case 4: both_loop<4>(acc, x, a, b, p.iters_matrix, bias); break;
      case 6: both_loop<6>(acc, x, a, b, p.iters_matrix, bias); break;
      case 8: both_loop<8>(acc, x, a, b, p.iters_matrix, bias); break;
      default: both_loop<0>(acc, x, a, b, p.iters_matrix, bias); break;
    }
  }
  const int64_t t1 = wall_clock64();

  float s = 0.0f;
#pragma unroll
  for (int m = 0; m < kMfmaPerIter; ++m)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[m][i];
#pragma unroll
  for (int j = 0; j < kActsPerIter; ++j) s += x[j];
  if (s == 12345.678f) p.sink[0] = s;  // (practically never: keeps the arithmetic alive)
  if (lane == 0) p.ticks[(size_t)blockIdx.x * 8 + wave] = t1 - t0;
}

}  // namespace

hipError_t launch_calib_copy(hipStream_t st, const void *src, void *dst, int64_t bytes, int blocks) {
  hipLaunchKernelGGL(calib_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const u32x4 *>(src),
                     static_cast<u32x4 *>(dst), bytes / 16);
  return hipGetLastError();
}

hipError_t launch_calib_read(hipStream_t st, const void *src, void *sink, int64_t bytes, int blocks) {
  hipLaunchKernelGGL(calib_read_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const u32x4 *>(src),
                     static_cast<uint32_t *>(sink), bytes / 16);
  return hipGetLastError();
}

hipError_t launch_calib_probe(hipStream_t st, const int32_t role_of_wave[8], int32_t iters_matrix,
                              int32_t iters_vector, int32_t acts_per_group, int32_t lds_reads, int blocks,
                              int64_t *ticks, float *sink) {
  ProbeArgs p;
  int last = -1;
  for (int w = 0; w < 8; ++w) {
    p.role_of_wave[w] = role_of_wave[w];
    if (role_of_wave[w] != ROLE_NONE) last = w;
  }
  if (last < 0) return hipErrorInvalidValue;
  p.iters_matrix = iters_matrix;
  p.iters_vector = iters_vector;
  p.acts_per_group = acts_per_group;
  p.lds_reads = lds_reads;
  p.ticks = ticks;
  p.sink = sink;
  // wavefronts behind the last one with a role are not launched (they would still occupy a SIMD slot)
  hipLaunchKernelGGL(calib_probe_kernel, dim3((unsigned)blocks), dim3((unsigned)(last + 1) * 64), 0, st, p);
  return hipGetLastError();
}

}  // namespace pod
