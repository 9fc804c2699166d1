// One PPO minibatch of the learner (Sec. 4.2 "Learner": fetch a batch of
// transitions from the buffer, train the networks; Sec. 5.2: PPO, batch size
// 1024, learning rate 1e-3): forward of actor and critic with the activations
// kept, clipped-surrogate and value loss, backward through both 3-layer
// perceptrons, Adam.  fp32 master weights, fp32 matrix-core arithmetic
// (v_mfma_f32_32x32x2_f32), fp32 accumulation.
//
// Every dense product -- forward, input gradient, weight gradient -- goes
// through ONE tiled kernel that reads its operands through (row stride, column
// stride[, row gather]) views, so transposes and the gather of the minibatch
// rows out of the rollout buffer cost no extra pass; bias + tanh, and the tanh
// derivative of the backward pass, are fused into its epilogue.  At the
// paper's batch of 1024 the products are small (<= 0.54 GFLOP): the step is a
// chain of ~30 short launches, bound by launch latency and tile count rather
// than by the matrix pipe; it is built to be correct and allocation-free (it
// can sit in a captured graph), not yet to be fast.
#include "pod_internal.h"

namespace pod {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));


enum Epi { EPI_NONE = 0, EPI_BIAS_TANH = 1, EPI_BIAS = 2, EPI_DTANH = 3 };

struct GemmArgs {
  const float *A;        // A'[m][k] = A[gm * a_rs + gk * a_cs]
  int64_t a_rs, a_cs;
  const int32_t *gather; // row indices of the minibatch (or NULL)
  int32_t gather_dim;    // 0: none, 1: gm = gather[m], 2: gk = gather[k]
  const float *B;        // B'[k][n] = B[k * b_rs + n * b_cs]
  int64_t b_rs, b_cs;
  float *C;              // row-major [M, N]; with k_splits > 1: [k_splits][M, N] partial products
  int32_t M, N, K;
  int32_t k_splits, k_chunk;  // blockIdx.z takes k in [z k_chunk, (z + 1) k_chunk)
  const float *bias;     // [N]   (EPI_BIAS_TANH, EPI_BIAS)
  const float *aux;      // [M, N] saved activation h: C = acc * (1 - h^2)   (EPI_DTANH)
  int32_t epi;           // (EPI_NONE when k_splits > 1)
};

// C = A' B' on the fp32 matrix cores.  A workgroup of 4 wavefronts owns a TM x TM tile of C (each wavefront a
// TM/2 x TM/2 quadrant = (TM/64)^2 accumulators of 32 x 32); the k range is walked in slices of 16 that are staged
// in LDS k-major, so that the two operands of v_mfma_f32_32x32x2_f32 are conflict-free row reads.  The next
// slice's global loads are issued into registers before the matrix instructions of the current one.
// GK: k extent per slice.  Small problems (few workgroups, nothing else on the compute unit to hide a load's
// latency behind) take long slices: 16 loads per thread and operand in flight, a quarter of the iterations.
template <int TM, int GK>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  constexpr int TP = TM + 4;         // LDS row pitch
  constexpr int NE = TM * GK / 256;  // elements per thread, operand and slice
  constexpr int Q = TM / 64;         // 32 x 32 accumulators per wavefront and dimension
  __shared__ float As[GK][TP];
  __shared__ float Bs[GK][TP];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TM;
  const int mi = (w & 1) * (TM / 2), ni = (w >> 1) * (TM / 2);
  const int kbeg = blockIdx.z * g.k_chunk, kend = min(g.K, kbeg + g.k_chunk);
  f32x16 acc[Q][Q];
#pragma unroll
  for (int x = 0; x < Q; ++x)
#pragma unroll
    for (int y = 0; y < Q; ++y)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.0f;
  // staging maps: lanes run along the operand's contiguous dimension
  const bool a_k_contig = g.a_cs == 1, b_n_contig = g.b_cs == 1;
  int am[NE], ak[NE], bn[NE], bk[NE];
#pragma unroll
  for (int j = 0; j < NE; ++j) {
    if (a_k_contig) {
      ak[j] = tid % GK;
      am[j] = tid / GK + (256 / GK) * j;
    } else {
      am[j] = (tid & 63) + 64 * (j % (TM / 64));
      ak[j] = (tid >> 6) + 4 * (j / (TM / 64));
    }
    if (b_n_contig) {
      bn[j] = (tid & 63) + 64 * (j % (TM / 64));
      bk[j] = (tid >> 6) + 4 * (j / (TM / 64));
    } else {
      bk[j] = tid % GK;
      bn[j] = tid / GK + (256 / GK) * j;
    }
  }
  float ra[NE], rb[NE];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int j = 0; j < NE; ++j) {
      float v = 0.0f;
      if (m0 + am[j] < g.M && k0 + ak[j] < kend) {
        int64_t gm = m0 + am[j], gk = k0 + ak[j];
        if (g.gather_dim == 1) gm = g.gather[gm];
        if (g.gather_dim == 2) gk = g.gather[gk];
        v = g.A[gm * g.a_rs + gk * g.a_cs];
      }
      ra[j] = v;
      float u = 0.0f;
      if (n0 + bn[j] < g.N && k0 + bk[j] < kend)
        u = g.B[(int64_t)(k0 + bk[j]) * g.b_rs + (int64_t)(n0 + bn[j]) * g.b_cs];
      rb[j] = u;
    }
  };
  fetch(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += GK) {
#pragma unroll
    for (int j = 0; j < NE; ++j) {
      As[ak[j]][am[j]] = ra[j];
      Bs[bk[j]][bn[j]] = rb[j];
    }
    __syncthreads();
    if (k0 + GK < kend) fetch(k0 + GK);
#pragma unroll
    for (int kk = 0; kk < GK; kk += 2) {
      float a[Q], b[Q];
#pragma unroll
      for (int x = 0; x < Q; ++x) a[x] = As[kk + (lane >> 5)][mi + 32 * x + (lane & 31)];
#pragma unroll
      for (int y = 0; y < Q; ++y) b[y] = Bs[kk + (lane >> 5)][ni + 32 * y + (lane & 31)];
#pragma unroll
      for (int x = 0; x < Q; ++x)
#pragma unroll
        for (int y = 0; y < Q; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
    }
    __syncthreads();
  }
  // accumulator register i of lane l: row 8 (i / 4) + 4 (l / 32) + i % 4, column l % 32
  float *C = g.C + (g.k_splits > 1 ? (int64_t)blockIdx.z * g.M * g.N : 0);
#pragma unroll
  for (int y = 0; y < Q; ++y) {
    const int col = n0 + ni + 32 * y + (lane & 31);
    if (col < g.N) {
      const float bv = (g.epi == EPI_BIAS_TANH || g.epi == EPI_BIAS) ? g.bias[col] : 0.0f;
#pragma unroll
      for (int x = 0; x < Q; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = m0 + mi + 32 * x + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
          if (row < g.M) {
            float v = acc[x][y][i] + bv;
            if (g.epi == EPI_BIAS_TANH) v = tanhf(v);
            if (g.epi == EPI_DTANH) {
              const float h = g.aux[(int64_t)row * g.N + col];
              v = v * (1.0f - h * h);
            }
            C[(int64_t)row * g.N + col] = v;
          }
        }
    }
  }
}

// out[i] = sum_z part[z][i], z ascending
__global__ __launch_bounds__(256) void reduce_splits_kernel(int64_t n, int splits, const float *__restrict__ part,
                                                            float *__restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    float s = part[i];
    for (int z = 1; z < splits; ++z) s += part[(int64_t)z * n + i];
    out[i] = s;
  }
}

// Column sums (bias gradients) gb[n] = sum_b dZ[b][n].  Grid (column blocks of 64, row chunks): a workgroup's
// 4 wavefronts split the rows of its chunk, lanes run along the columns; chunk results go to part[chunk][n] and
// are added up in chunk order by reduce_splits_kernel (or straight to gb when there is one chunk).
constexpr int CS_ROWS = 512;
__global__ __launch_bounds__(256) void colsum_kernel(int B, int N, const float *__restrict__ dZ, float *__restrict__ out) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  const int b0 = blockIdx.y * CS_ROWS, b1 = min(B, b0 + CS_ROWS);
  float s = 0.0f;
  if (n < N)
    for (int b = b0 + w; b < b1; b += 4) s += dZ[(int64_t)b * N + n];
  part[w][lane] = s;
  __syncthreads();
  if (w == 0 && n < N) out[(int64_t)blockIdx.y * N + n] = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

struct LossArgs {
  int32_t B, D;
  const float *mu;        // [B, D] actor output (after tanh)
  const float *v;         // [B]
  const float *act, *logp_old, *adv, *ret;  // rollout buffers, indexed through rows
  const int32_t *rows;
  float sigma, clip, value_coef;
  float *dz_actor;        // [B, D] d L / d (pre-tanh output)
  float *dz_critic;       // [B]
  float *partial;         // [blocks][4]
};

// One lane per sample: log-prob, ratio, which branch of the min() is live, the two loss terms and the gradients
// w.r.t. the networks' last pre-activations.  Per-block partial sums of the statistics in a fixed order.
__global__ __launch_bounds__(256) void ppo_loss_kernel(LossArgs a) {
  __shared__ float red[4][256];
  const int b = blockIdx.x * 256 + threadIdx.x;
  float st[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (b < a.B) {
    const int64_t r = a.rows ? a.rows[b] : b;
    const float inv_b = 1.0f / (float)a.B, inv_s2 = 1.0f / (a.sigma * a.sigma);
    float logp = -(float)a.D * logf(a.sigma) - 0.5f * (float)a.D * 1.8378770664093453f;  // ln(2 pi)
    for (int d = 0; d < a.D; ++d) {
      const float e = a.act[r * a.D + d] - a.mu[(int64_t)b * a.D + d];
      logp -= 0.5f * e * e * inv_s2;
    }
    const float ratio = expf(logp - a.logp_old[r]);
    const float A = a.adv[r];
    const float rc = fminf(fmaxf(ratio, 1.0f - a.clip), 1.0f + a.clip);
    const float s1 = ratio * A, s2 = rc * A;
    const bool live = s1 <= s2;
    st[0] = -(live ? s1 : s2) * inv_b;
    st[2] = live ? 0.0f : inv_b;
    st[3] = ratio * inv_b;
    for (int d = 0; d < a.D; ++d) {
      const float m = a.mu[(int64_t)b * a.D + d];
      const float e = a.act[r * a.D + d] - m;
      const float dmu = live ? -(ratio * A * e * inv_s2) * inv_b : 0.0f;
      a.dz_actor[(int64_t)b * a.D + d] = dmu * (1.0f - m * m);
    }
    const float err = a.v[b] - a.ret[r];
    st[1] = 0.5f * err * err * inv_b;
    a.dz_critic[b] = a.value_coef * err * inv_b;
  }
  for (int i = 0; i < 4; ++i) red[i][threadIdx.x] = st[i];
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s)
      for (int i = 0; i < 4; ++i) red[i][threadIdx.x] += red[i][threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x < 4) a.partial[(int64_t)blockIdx.x * 4 + threadIdx.x] = red[threadIdx.x][0];
}

__global__ void ppo_stats_kernel(int blocks, const float *__restrict__ partial, float *__restrict__ stats) {
  if (threadIdx.x < 4) {
    float s = 0.0f;
    for (int i = 0; i < blocks; ++i) s += partial[(int64_t)i * 4 + threadIdx.x];
    stats[threadIdx.x] = s;
  }
}

struct AdamSeg {
  float *theta, *m, *v;
  const float *g;
  int64_t n;
};
struct AdamBatch {
  AdamSeg seg[12];
};

// blockIdx.y = tensor
__global__ __launch_bounds__(256) void adam_batch_kernel(AdamBatch t, float lr, float b1, float b2, float eps,
                                                         float inv_c1, float inv_c2) {
  const AdamSeg s = t.seg[blockIdx.y];
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < s.n; i += (int64_t)gridDim.x * 256) {
    const float gi = s.g[i];
    const float mi = b1 * s.m[i] + (1.0f - b1) * gi;
    const float vi = b2 * s.v[i] + (1.0f - b2) * gi * gi;
    s.m[i] = mi;
    s.v[i] = vi;
    s.theta[i] -= lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
  }
}

__global__ __launch_bounds__(256) void adam_kernel(int64_t n, float *__restrict__ theta, const float *__restrict__ g,
                                                   float *__restrict__ m, float *__restrict__ v, float lr, float b1,
                                                   float b2, float eps, float inv_c1, float inv_c2) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    const float gi = g[i];
    const float mi = b1 * m[i] + (1.0f - b1) * gi;
    const float vi = b2 * v[i] + (1.0f - b2) * gi * gi;
    m[i] = mi;
    v[i] = vi;
    theta[i] -= lr * (mi * inv_c1) / (sqrtf(vi * inv_c2) + eps);
  }
}

// splitk: scratch for partial products when the k range is split (weight gradients: k is the batch, the output
// is small), NULL to forbid splitting.  Tiles of 128 when they still fill the chip, else 64.
hipError_t gemm(hipStream_t st, GemmArgs g, float *splitk = nullptr, size_t splitk_floats = 0) {
  const int64_t tiles128 = (int64_t)((g.M + 127) / 128) * ((g.N + 127) / 128);
  const int TM = tiles128 >= 256 ? 128 : 64;
  const int64_t tiles = (int64_t)((g.M + TM - 1) / TM) * ((g.N + TM - 1) / TM);
  int splits = 1;
  if (splitk && g.epi == EPI_NONE && tiles < 256 && g.K >= 512) {
    splits = (int)((512 + tiles - 1) / tiles);
    if (splits > 32) splits = 32;
    while (splits > 1 && (g.K / splits < 128 || (size_t)splits * g.M * g.N > splitk_floats)) --splits;
  }
  float *out = g.C;
  g.k_splits = splits;
  g.k_chunk = splits > 1 ? ((g.K + splits - 1) / splits + 63) / 64 * 64 : g.K;
  if (splits > 1) g.C = splitk;
  const dim3 grid((unsigned)((g.N + TM - 1) / TM), (unsigned)((g.M + TM - 1) / TM), (unsigned)splits);
  if (TM == 128)
    hipLaunchKernelGGL((gemm_f32_kernel<128, 16>), grid, dim3(256), 0, st, g);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<64, 64>), grid, dim3(256), 0, st, g);
  if (splits > 1) {
    const int64_t n = (int64_t)g.M * g.N;
    hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, splits, splitk, out);
  }
  return hipGetLastError();
}

hipError_t colsum(hipStream_t st, int B, int N, const float *dZ, float *gb, float *scratch, size_t scratch_floats) {
  int chunks = (B + CS_ROWS - 1) / CS_ROWS;
  if ((size_t)chunks * N > scratch_floats) return hipErrorInvalidValue;
  float *dst = chunks > 1 ? scratch : gb;
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)chunks), dim3(256), 0, st, B, N, dZ, dst);
  if (chunks > 1)
    hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, (int64_t)N, chunks,
                       scratch, gb);
  return hipGetLastError();
}

#define LRN(x)                      \
  do {                              \
    hipError_t e_ = (x);            \
    if (e_ != hipSuccess) return e_; \
  } while (0)

struct Scratch {
  float *h1, *h2, *out, *dz3, *dz2, *dz1, *v, *dzc, *partial, *splitk;
  size_t splitk_floats;
};

// forward with kept activations, then (after the caller's loss kernel filled dz3) the backward pass
hipError_t net_forward(hipStream_t st, int B, int S, int Hd, int O, bool out_tanh, const float *obs,
                       const int32_t *rows, const pr_net_params &p, const Scratch &w, float *out) {
  GemmArgs g{};
  g.A = obs, g.a_rs = S, g.a_cs = 1, g.gather = rows, g.gather_dim = rows ? 1 : 0;
  g.B = p.W1, g.b_rs = Hd, g.b_cs = 1, g.C = w.h1, g.M = B, g.N = Hd, g.K = S, g.bias = p.b1, g.epi = EPI_BIAS_TANH;
  LRN(gemm(st, g));
  g = GemmArgs{};
  g.A = w.h1, g.a_rs = Hd, g.a_cs = 1, g.B = p.W2, g.b_rs = Hd, g.b_cs = 1, g.C = w.h2, g.M = B, g.N = Hd, g.K = Hd;
  g.bias = p.b2, g.epi = EPI_BIAS_TANH;
  LRN(gemm(st, g));
  g = GemmArgs{};
  g.A = w.h2, g.a_rs = Hd, g.a_cs = 1, g.B = p.W3, g.b_rs = O, g.b_cs = 1, g.C = out, g.M = B, g.N = O, g.K = Hd;
  g.bias = p.b3, g.epi = out_tanh ? EPI_BIAS_TANH : EPI_BIAS;
  return gemm(st, g);
}

hipError_t net_backward(hipStream_t st, int B, int S, int Hd, int O, const float *obs, const int32_t *rows,
                        const pr_net_params &p, const Scratch &w, const float *dz3, const pr_net_params &grad) {
  GemmArgs g{};
  // gW3 = H2^T dZ3, gb3
  g.A = w.h2, g.a_rs = 1, g.a_cs = Hd, g.B = dz3, g.b_rs = O, g.b_cs = 1, g.C = grad.W3, g.M = Hd, g.N = O, g.K = B;
  LRN(gemm(st, g, w.splitk, w.splitk_floats));
  LRN(colsum(st, B, O, dz3, grad.b3, w.splitk, w.splitk_floats));
  // dZ2 = (dZ3 W3^T) (1 - H2^2)
  g = GemmArgs{};
  g.A = dz3, g.a_rs = O, g.a_cs = 1, g.B = p.W3, g.b_rs = 1, g.b_cs = O, g.C = w.dz2, g.M = B, g.N = Hd, g.K = O;
  g.aux = w.h2, g.epi = EPI_DTANH;
  LRN(gemm(st, g));
  // gW2 = H1^T dZ2, gb2
  g = GemmArgs{};
  g.A = w.h1, g.a_rs = 1, g.a_cs = Hd, g.B = w.dz2, g.b_rs = Hd, g.b_cs = 1, g.C = grad.W2, g.M = Hd, g.N = Hd, g.K = B;
  LRN(gemm(st, g, w.splitk, w.splitk_floats));
  LRN(colsum(st, B, Hd, w.dz2, grad.b2, w.splitk, w.splitk_floats));
  // dZ1 = (dZ2 W2^T) (1 - H1^2)
  g = GemmArgs{};
  g.A = w.dz2, g.a_rs = Hd, g.a_cs = 1, g.B = p.W2, g.b_rs = 1, g.b_cs = Hd, g.C = w.dz1, g.M = B, g.N = Hd, g.K = Hd;
  g.aux = w.h1, g.epi = EPI_DTANH;
  LRN(gemm(st, g));
  // gW1 = X^T dZ1 (minibatch rows gathered along k), gb1
  g = GemmArgs{};
  g.A = obs, g.a_rs = 1, g.a_cs = S, g.gather = rows, g.gather_dim = rows ? 2 : 0;
  g.B = w.dz1, g.b_rs = Hd, g.b_cs = 1, g.C = grad.W1, g.M = S, g.N = Hd, g.K = B;
  LRN(gemm(st, g, w.splitk, w.splitk_floats));
  LRN(colsum(st, B, Hd, w.dz1, grad.b1, w.splitk, w.splitk_floats));
  return hipGetLastError();
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

// partial products of a split weight gradient: up to 8 copies of the largest (Hd x Hd; S <= 2 Hd assumed else fewer splits)
static size_t splitk_floats(int B, int Hd) {
  const size_t a = (size_t)8 * Hd * Hd, b = (size_t)((B + CS_ROWS - 1) / CS_ROWS) * Hd;  // split products / column-sum chunks
  return a > b ? a : b;
}

size_t ppo_scratch_bytes(int B, int Hd, int D) {
  const size_t f = 4;
  return 2 * align256((size_t)B * Hd * f) + 2 * align256((size_t)B * D * f) + 2 * align256((size_t)B * Hd * f) +
         2 * align256((size_t)B * f) + align256((size_t)((B + 255) / 256) * 4 * f) + align256(splitk_floats(B, Hd) * f);
}

hipError_t launch_ppo_grads(hipStream_t st, const pr_ppo_config &c, const float *obs, const float *act,
                            const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                            const pr_net_params &actor, const pr_net_params &critic, const pr_net_params &ga,
                            const pr_net_params &gc, void *scratch, float *stats) {
  const int B = c.batch, D = c.n_stocks, Hd = c.hidden, S = 1 + 2 * D + D * c.n_ind;
  unsigned char *p = static_cast<unsigned char *>(scratch);
  auto take = [&](size_t bytes) {
    float *r = reinterpret_cast<float *>(p);
    p += align256(bytes);
    return r;
  };
  Scratch w;
  w.h1 = take((size_t)B * Hd * 4);
  w.h2 = take((size_t)B * Hd * 4);
  w.out = take((size_t)B * D * 4);
  w.dz3 = take((size_t)B * D * 4);
  w.dz2 = take((size_t)B * Hd * 4);
  w.dz1 = take((size_t)B * Hd * 4);
  w.v = take((size_t)B * 4);
  w.dzc = take((size_t)B * 4);
  const int blocks = (B + 255) / 256;
  w.partial = take((size_t)blocks * 4 * 4);
  w.splitk_floats = splitk_floats(B, Hd);
  w.splitk = take(w.splitk_floats * 4);
  // critic forward first (its value goes into the loss kernel), then the actor forward, loss, actor backward
  // while its activations are still in place, and the critic forward again for its own backward pass: the
  // scratch holds one network's activations at a time.
  LRN(net_forward(st, B, S, Hd, 1, false, obs, rows, critic, w, w.v));
  LRN(net_forward(st, B, S, Hd, D, true, obs, rows, actor, w, w.out));
  LossArgs l;
  l.B = B, l.D = D, l.mu = w.out, l.v = w.v, l.act = act, l.logp_old = logp_old, l.adv = adv, l.ret = ret, l.rows = rows;
  l.sigma = c.sigma, l.clip = c.clip, l.value_coef = c.value_coef, l.dz_actor = w.dz3, l.dz_critic = w.dzc;
  l.partial = w.partial;
  hipLaunchKernelGGL(ppo_loss_kernel, dim3(blocks), dim3(256), 0, st, l);
  if (stats) hipLaunchKernelGGL(ppo_stats_kernel, dim3(1), dim3(64), 0, st, blocks, w.partial, stats);
  LRN(net_backward(st, B, S, Hd, D, obs, rows, actor, w, w.dz3, ga));
  LRN(net_forward(st, B, S, Hd, 1, false, obs, rows, critic, w, w.v));
  LRN(net_backward(st, B, S, Hd, 1, obs, rows, critic, w, w.dzc, gc));
  return hipGetLastError();
}

hipError_t launch_adam12(hipStream_t st, const int64_t *n, float *const *theta, float *const *g, float *const *m,
                         float *const *v, float lr, float b1, float b2, float eps, int32_t t) {
  AdamBatch bt;
  int64_t nmax = 1;
  for (int i = 0; i < 12; ++i) {
    bt.seg[i].theta = theta[i], bt.seg[i].g = g[i], bt.seg[i].m = m[i], bt.seg[i].v = v[i], bt.seg[i].n = n[i];
    if (n[i] > nmax) nmax = n[i];
  }
  const double c1 = 1.0 - pow((double)b1, (double)t), c2 = 1.0 - pow((double)b2, (double)t);
  int64_t bx = (nmax + 255) / 256;
  if (bx > 1024) bx = 1024;
  hipLaunchKernelGGL(adam_batch_kernel, dim3((unsigned)bx, 12), dim3(256), 0, st, bt, lr, b1, b2, eps, (float)(1.0 / c1),
                     (float)(1.0 / c2));
  return hipGetLastError();
}

hipError_t launch_adam(hipStream_t st, int64_t n, float *theta, const float *g, float *m, float *v, float lr, float b1,
                       float b2, float eps, int32_t t) {
  const double c1 = 1.0 - pow((double)b1, (double)t), c2 = 1.0 - pow((double)b2, (double)t);
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, theta, g, m, v, lr, b1, b2,
                     eps, (float)(1.0 / c1), (float)(1.0 / c2));
  return hipGetLastError();
}

}  // namespace pod
