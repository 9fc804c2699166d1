// One PPO minibatch of the learner (Sec. 4.2 "Learner": fetch a batch of
// transitions from the buffer, train the networks; Sec. 5.2: PPO, batch size
// 1024, learning rate 1e-3): forward of actor and critic with the activations
// kept, clipped-surrogate and value loss, backward through both 3-layer
// perceptrons, Adam.  fp32 master weights, fp32 matrix-core arithmetic
// (v_mfma_f32_32x32x2_f32), fp32 accumulation.
//
// Every dense product -- forward, input gradient, weight gradient -- goes
// through ONE tiled kernel that reads its operands through (row stride, column
// stride) views, so no transposed copy of a weight or an activation is made;
// bias + tanh, and the tanh derivative of the backward pass, are fused into its
// epilogue.  The minibatch rows are gathered once into a zero-padded, aligned
// copy that both networks' first layers read.  Nothing here allocates,
// memsets or synchronises: a step is ~38 kernel launches on the caller's
// stream and can sit in a captured graph (at the paper's batch of 1024 the
// launches are short, so that is how it should be run).
#include "pod_internal.h"

namespace pod {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));


enum Epi { EPI_NONE = 0, EPI_BIAS_TANH = 1, EPI_BIAS = 2, EPI_DTANH = 3 };

struct GemmArgs {
  const float *A;        // A'[m][k] = A[m * a_rs + k * a_cs]
  int64_t a_rs, a_cs;
  const float *B;        // B'[k][n] = B[k * b_rs + n * b_cs]
  int64_t b_rs, b_cs;
  float *C;              // row-major [M, N]; with k_splits > 1: [k_splits][M, N] partial products
  int32_t M, N, K;
  int32_t a_m_phys;      // rows of A' that may be read (>= M: zero padding behind the logical rows); 0 = M
  int32_t b_k_valid;     // rows of B' that exist (<= K: A' is zero beyond); 0 = K
  int32_t k_splits, k_chunk;  // blockIdx.z takes k in [z k_chunk, (z + 1) k_chunk)
  const float *bias;     // [N]   (EPI_BIAS_TANH, EPI_BIAS)
  const float *aux;      // [M, N] saved activation h: C = acc * (1 - h^2)   (EPI_DTANH)
  int32_t epi;           // (EPI_NONE when k_splits > 1)
};

// One operand's staging of a [TM x GK] slice into the k-major LDS tile S[k][mn].
//   VEC: 16-byte global loads along the operand's contiguous dimension (pointers and guards set up once, advanced by
//        a uniform stride per slice).  Needs a 16-byte aligned base, the other stride a multiple of 4 elements and
//        the extent along the contiguous dimension a multiple of 4 (the host checks).  Loads along k are scattered
//        into 4 LDS rows (lanes 4 apart in k, so the 64 stores of a wavefront hit distinct banks), loads along
//        m/n are one 16-byte LDS store.
//   else: 4-byte loads through the general (row stride, column stride) view, for the few skinny or unaligned
//        operands (30-column output layer, scalar value head).
template <int TM, int GK, bool VEC>
struct Stage {
  static constexpr int TP = TM + 4;
  static constexpr int NV = VEC ? TM * GK / 1024 : TM * GK / 256;
  const float *ptr[NV];
  int kof[NV], sof[NV];  // k offset inside the slice; LDS offset of the first element
  bool along_k;
  int64_t kstep;
  float4 v4[VEC ? NV : 1];
  float v1[VEC ? 1 : NV];
  int mn_ok[VEC ? 1 : NV];

  // base: the operand; ks / ms: element strides along k and along m (or n); mn0: first row/column of the tile;
  // mn_lim: rows/columns that may be read
  __device__ void init(const float *base, int64_t ks, int64_t ms, int mn0, int mn_lim, int kbeg, int tid) {
    along_k = (ks == 1);
    kstep = (int64_t)GK * ks;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int idx = tid + 256 * j;
      int k, mn;
      if (VEC) {
        if (along_k) {
          k = 4 * (idx % (GK / 4)), mn = idx / (GK / 4);
        } else {
          mn = 4 * (idx % (TM / 4)), k = idx / (TM / 4);
        }
        // rows/columns past the edge are clamped: they only feed rows/columns of C that are never stored
        int gmn = mn0 + mn;
        const int last = along_k ? mn_lim - 1 : mn_lim - 4;
        gmn = gmn < last ? gmn : last;
        ptr[j] = base + (int64_t)gmn * ms + (int64_t)(kbeg + k) * ks;
      } else {
        if (along_k) {
          k = idx % GK, mn = idx / GK;
        } else {
          mn = idx % TM, k = idx / TM;
        }
        mn_ok[j] = mn0 + mn < mn_lim;
        ptr[j] = base + (int64_t)(mn_ok[j] ? mn0 + mn : 0) * ms + (int64_t)(kbeg + k) * ks;
      }
      kof[j] = k;
      sof[j] = k * TP + mn;
    }
  }
  // k0: first k of the slice, klim: first k that must read as zero
  __device__ void fetch(int k0, int klim) {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (VEC) {
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (k0 + kof[j] < klim) v = *reinterpret_cast<const float4 *>(ptr[j]);
        v4[j] = v;
      } else {
        float v = 0.0f;
        if (mn_ok[j] && k0 + kof[j] < klim) v = *ptr[j];
        v1[j] = v;
      }
      ptr[j] += kstep;
    }
  }
  __device__ void store(float *S) const {
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (VEC) {
        if (along_k) {
          S[sof[j]] = v4[j].x, S[sof[j] + TP] = v4[j].y, S[sof[j] + 2 * TP] = v4[j].z, S[sof[j] + 3 * TP] = v4[j].w;
        } else {
          *reinterpret_cast<float4 *>(S + sof[j]) = v4[j];
        }
      } else {
        S[sof[j]] = v1[j];
      }
    }
  }
};

// C = A' B' on the fp32 matrix cores.  A workgroup of 4 wavefronts owns a TM x TM tile of C (each wavefront a
// TM/2 x TM/2 quadrant = (TM/64)^2 accumulators of 32 x 32); the k range is walked in slices of GK that are staged
// in LDS k-major, so that the two operands of v_mfma_f32_32x32x2_f32 are conflict-free row reads.  The next
// slice's global loads are issued into registers before the matrix instructions of the current one.
template <int TM, int GK, bool VA, bool VB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
  constexpr int TP = TM + 4;         // LDS row pitch
  constexpr int Q = TM / 64;         // 32 x 32 accumulators per wavefront and dimension
  __shared__ __align__(16) float As[GK * TP];
  __shared__ __align__(16) float Bs[GK * TP];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TM;
  const int mi = (w & 1) * (TM / 2), ni = (w >> 1) * (TM / 2);
  const int kbeg = blockIdx.z * g.k_chunk, kend = min(g.K, kbeg + g.k_chunk);
  const int kend_b = min(kend, g.b_k_valid);
  f32x16 acc[Q][Q];
#pragma unroll
  for (int x = 0; x < Q; ++x)
#pragma unroll
    for (int y = 0; y < Q; ++y)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.0f;
  Stage<TM, GK, VA> sa;
  Stage<TM, GK, VB> sb;
  sa.init(g.A, g.a_cs, g.a_rs, m0, g.a_m_phys, kbeg, tid);
  sb.init(g.B, g.b_rs, g.b_cs, n0, g.N, kbeg, tid);
  sa.fetch(kbeg, kend);
  sb.fetch(kbeg, kend_b);
  for (int k0 = kbeg; k0 < kend; k0 += GK) {
    sa.store(As);
    sb.store(Bs);
    __syncthreads();
    if (k0 + GK < kend) {
      sa.fetch(k0 + GK, kend);
      sb.fetch(k0 + GK, kend_b);
    }
#pragma unroll
    for (int kk = 0; kk < GK; kk += 2) {
      float a[Q], b[Q];
#pragma unroll
      for (int x = 0; x < Q; ++x) a[x] = As[(kk + (lane >> 5)) * TP + mi + 32 * x + (lane & 31)];
#pragma unroll
      for (int y = 0; y < Q; ++y) b[y] = Bs[(kk + (lane >> 5)) * TP + ni + 32 * y + (lane & 31)];
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

// Minibatch rows of the buffer, zero-padded to a multiple of 4 columns: the aligned A operand of the first layer's
// forward and weight-gradient products of both networks.  One wavefront per row.
__global__ __launch_bounds__(256) void gather_pad_kernel(int B, int S, int Sp, const float *__restrict__ obs,
                                                         const int32_t *__restrict__ rows, float *__restrict__ xp) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (b >= B) return;
  const float *src = obs + (int64_t)(rows ? rows[b] : b) * S;
  for (int j = lane; j < Sp; j += 64) xp[(int64_t)b * Sp + j] = j < S ? src[j] : 0.0f;
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
constexpr int CS_MAX_CHUNKS = 64;
inline int colsum_chunks(int B) { return B >= 128 * CS_MAX_CHUNKS ? CS_MAX_CHUNKS : (B + 127) / 128; }

__global__ __launch_bounds__(256) void colsum_kernel(int B, int N, int rows_per_chunk, const float *__restrict__ dZ,
                                                     float *__restrict__ out) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  const int b0 = blockIdx.y * rows_per_chunk, b1 = min(B, b0 + rows_per_chunk);
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

// 32 lanes per sample (lanes over the action components): log-prob, ratio, which branch of the min() is live, the
// two loss terms and the gradients w.r.t. the networks' last pre-activations.  Per-block partial sums of the
// statistics in a fixed order.
__global__ __launch_bounds__(256) void ppo_loss_kernel(LossArgs a) {
  __shared__ float red[8][4];
  const int sub = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int b = blockIdx.x * 8 + grp;
  float st[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (b < a.B) {  // uniform over the 32 lanes of a sample
    const int64_t r = a.rows ? a.rows[b] : b;
    const float inv_b = 1.0f / (float)a.B, inv_s2 = 1.0f / (a.sigma * a.sigma);
    float q = 0.0f;
    for (int d = sub; d < a.D; d += 32) {
      const float e = a.act[r * a.D + d] - a.mu[(int64_t)b * a.D + d];
      q += e * e;
    }
    for (int o = 16; o > 0; o >>= 1) q += __shfl_xor(q, o, 32);
    const float logp = -(float)a.D * logf(a.sigma) - 0.5f * (float)a.D * 1.8378770664093453f - 0.5f * q * inv_s2;  // ln(2 pi)
    const float ratio = expf(logp - a.logp_old[r]);
    const float A = a.adv[r];
    const float rc = fminf(fmaxf(ratio, 1.0f - a.clip), 1.0f + a.clip);
    const float s1 = ratio * A, s2 = rc * A;
    const bool live = s1 <= s2;
    for (int d = sub; d < a.D; d += 32) {
      const float m = a.mu[(int64_t)b * a.D + d];
      const float e = a.act[r * a.D + d] - m;
      const float dmu = live ? -(ratio * A * e * inv_s2) * inv_b : 0.0f;
      a.dz_actor[(int64_t)b * a.D + d] = dmu * (1.0f - m * m);
    }
    const float err = a.v[b] - a.ret[r];
    if (sub == 0) {
      st[0] = -(live ? s1 : s2) * inv_b;
      st[1] = 0.5f * err * err * inv_b;
      st[2] = live ? 0.0f : inv_b;
      st[3] = ratio * inv_b;
      a.dz_critic[b] = a.value_coef * err * inv_b;
    }
  }
  if (sub == 0)
    for (int i = 0; i < 4; ++i) red[grp][i] = st[i];
  __syncthreads();
  if (threadIdx.x < 4) {
    float t = 0.0f;
    for (int g = 0; g < 8; ++g) t += red[g][threadIdx.x];
    a.partial[(int64_t)blockIdx.x * 4 + threadIdx.x] = t;
  }
}

// stats[i] = sum over blocks of partial[block][i]: 64 lanes stride the blocks, then a fixed-shape tree
__global__ __launch_bounds__(256) void ppo_stats_kernel(int blocks, const float *__restrict__ partial,
                                                        float *__restrict__ stats) {
  __shared__ float red[4][64];
  const int i = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float s = 0.0f;
  for (int k = lane; k < blocks; k += 64) s += partial[(int64_t)k * 4 + i];
  red[i][lane] = s;
  __syncthreads();
  for (int o = 32; o > 0; o >>= 1) {
    if (lane < o) red[i][lane] += red[i][lane + o];
    __syncthreads();
  }
  if (lane == 0) stats[i] = red[i][0];
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

template <int TM, int GK>
void launch_gemm(hipStream_t st, const dim3 &grid, const GemmArgs &g, bool va, bool vb) {
  if (va && vb)
    hipLaunchKernelGGL((gemm_f32_kernel<TM, GK, true, true>), grid, dim3(256), 0, st, g);
  else if (va)
    hipLaunchKernelGGL((gemm_f32_kernel<TM, GK, true, false>), grid, dim3(256), 0, st, g);
  else if (vb)
    hipLaunchKernelGGL((gemm_f32_kernel<TM, GK, false, true>), grid, dim3(256), 0, st, g);
  else
    hipLaunchKernelGGL((gemm_f32_kernel<TM, GK, false, false>), grid, dim3(256), 0, st, g);
}

// may an operand be staged with 16-byte loads?  ks / ms: strides along k and along m (or n); mn_lim, K: extents
bool vec_ok(const float *p, int64_t ks, int64_t ms, int mn_lim, int K, int k_valid, int k_chunk) {
  if (reinterpret_cast<uintptr_t>(p) & 15u) return false;
  if (ks == 1) return ms % 4 == 0 && K % 4 == 0 && k_valid % 4 == 0 && k_chunk % 4 == 0;
  if (ms == 1) return ks % 4 == 0 && mn_lim % 4 == 0 && mn_lim >= 4;
  return false;
}

// splitk: scratch for partial products when the k range is split (weight gradients: k is the batch, the output
// is small), NULL to forbid splitting.  Tiles of 128 when they still fill the chip, else 64.
hipError_t gemm(hipStream_t st, GemmArgs g, float *splitk = nullptr, size_t splitk_floats = 0) {
  if (!g.a_m_phys) g.a_m_phys = g.M;
  if (!g.b_k_valid) g.b_k_valid = g.K;
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
  const bool va = vec_ok(g.A, g.a_cs, g.a_rs, g.a_m_phys, g.K, g.K, g.k_chunk);
  const bool vb = vec_ok(g.B, g.b_rs, g.b_cs, g.N, g.K, g.b_k_valid, g.k_chunk);
  const dim3 grid((unsigned)((g.N + TM - 1) / TM), (unsigned)((g.M + TM - 1) / TM), (unsigned)splits);
  if (TM == 128)
    launch_gemm<128, 16>(st, grid, g, va, vb);
  else
    launch_gemm<64, 32>(st, grid, g, va, vb);
  if (splits > 1) {
    const int64_t n = (int64_t)g.M * g.N;
    hipLaunchKernelGGL(reduce_splits_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, splits, splitk, out);
  }
  return hipGetLastError();
}

hipError_t colsum(hipStream_t st, int B, int N, const float *dZ, float *gb, float *scratch, size_t scratch_floats) {
  const int chunks = colsum_chunks(B), per = (B + chunks - 1) / chunks;
  if ((size_t)chunks * N > scratch_floats) return hipErrorInvalidValue;
  float *dst = chunks > 1 ? scratch : gb;
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((N + 63) / 64), (unsigned)chunks), dim3(256), 0, st, B, N, per, dZ,
                     dst);
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
  float *xp;               // [B, Sp] gathered minibatch observations, zero-padded to Sp = 4 ceil(S / 4) columns
  float *h1[2], *h2[2];    // hidden activations of the actor [0] and the critic [1]
  float *out, *dz3, *dz2, *dz1, *v, *dzc, *partial, *splitk;
  size_t splitk_floats;
};

// forward of network `net` (0 actor, 1 critic) with kept activations
hipError_t net_forward(hipStream_t st, int B, int S, int Sp, int Hd, int O, bool out_tanh, int net,
                       const pr_net_params &p, const Scratch &w, float *out) {
  GemmArgs g{};
  g.A = w.xp, g.a_rs = Sp, g.a_cs = 1, g.B = p.W1, g.b_rs = Hd, g.b_cs = 1, g.C = w.h1[net], g.M = B, g.N = Hd;
  g.K = Sp, g.b_k_valid = S, g.bias = p.b1, g.epi = EPI_BIAS_TANH;
  LRN(gemm(st, g));
  g = GemmArgs{};
  g.A = w.h1[net], g.a_rs = Hd, g.a_cs = 1, g.B = p.W2, g.b_rs = Hd, g.b_cs = 1, g.C = w.h2[net], g.M = B, g.N = Hd;
  g.K = Hd, g.bias = p.b2, g.epi = EPI_BIAS_TANH;
  LRN(gemm(st, g));
  g = GemmArgs{};
  g.A = w.h2[net], g.a_rs = Hd, g.a_cs = 1, g.B = p.W3, g.b_rs = O, g.b_cs = 1, g.C = out, g.M = B, g.N = O, g.K = Hd;
  g.bias = p.b3, g.epi = out_tanh ? EPI_BIAS_TANH : EPI_BIAS;
  return gemm(st, g);
}

// backward from dz3 = d loss / d (last pre-activation) to the six gradient tensors
hipError_t net_backward(hipStream_t st, int B, int S, int Sp, int Hd, int O, int net, const pr_net_params &p,
                        const Scratch &w, const float *dz3, const pr_net_params &grad) {
  const float *h1 = w.h1[net], *h2 = w.h2[net];
  GemmArgs g{};
  // gW3 = H2^T dZ3, gb3
  g.A = h2, g.a_rs = 1, g.a_cs = Hd, g.B = dz3, g.b_rs = O, g.b_cs = 1, g.C = grad.W3, g.M = Hd, g.N = O, g.K = B;
  LRN(gemm(st, g, w.splitk, w.splitk_floats));
  LRN(colsum(st, B, O, dz3, grad.b3, w.splitk, w.splitk_floats));
  // dZ2 = (dZ3 W3^T) (1 - H2^2)
  g = GemmArgs{};
  g.A = dz3, g.a_rs = O, g.a_cs = 1, g.B = p.W3, g.b_rs = 1, g.b_cs = O, g.C = w.dz2, g.M = B, g.N = Hd, g.K = O;
  g.aux = h2, g.epi = EPI_DTANH;
  LRN(gemm(st, g));
  // gW2 = H1^T dZ2, gb2
  g = GemmArgs{};
  g.A = h1, g.a_rs = 1, g.a_cs = Hd, g.B = w.dz2, g.b_rs = Hd, g.b_cs = 1, g.C = grad.W2, g.M = Hd, g.N = Hd, g.K = B;
  LRN(gemm(st, g, w.splitk, w.splitk_floats));
  LRN(colsum(st, B, Hd, w.dz2, grad.b2, w.splitk, w.splitk_floats));
  // dZ1 = (dZ2 W2^T) (1 - H1^2)
  g = GemmArgs{};
  g.A = w.dz2, g.a_rs = Hd, g.a_cs = 1, g.B = p.W2, g.b_rs = 1, g.b_cs = Hd, g.C = w.dz1, g.M = B, g.N = Hd, g.K = Hd;
  g.aux = h1, g.epi = EPI_DTANH;
  LRN(gemm(st, g));
  // gW1 = X^T dZ1 (the padded rows of X^T are read, their products are never stored), gb1
  g = GemmArgs{};
  g.A = w.xp, g.a_rs = 1, g.a_cs = Sp, g.a_m_phys = Sp, g.B = w.dz1, g.b_rs = Hd, g.b_cs = 1, g.C = grad.W1, g.M = S;
  g.N = Hd, g.K = B;
  LRN(gemm(st, g, w.splitk, w.splitk_floats));
  LRN(colsum(st, B, Hd, w.dz1, grad.b1, w.splitk, w.splitk_floats));
  return hipGetLastError();
}

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

// partial products of a split weight gradient: up to 8 copies of the largest (Hd x Hd; S <= 2 Hd assumed else fewer splits)
static size_t splitk_floats(int Hd) {
  const size_t a = (size_t)8 * Hd * Hd, b = (size_t)CS_MAX_CHUNKS * Hd;  // split products / column-sum chunks
  return a > b ? a : b;
}

size_t ppo_scratch_bytes(int B, int Hd, int D, int S) {
  const size_t f = 4, Sp = (size_t)(S + 3) / 4 * 4;
  return align256((size_t)B * Sp * f) + 4 * align256((size_t)B * Hd * f) + 2 * align256((size_t)B * D * f) +
         2 * align256((size_t)B * Hd * f) + 2 * align256((size_t)B * f) + align256((size_t)((B + 7) / 8) * 4 * f) +
         align256(splitk_floats(Hd) * f);
}

hipError_t launch_ppo_grads(hipStream_t st, const pr_ppo_config &c, const float *obs, const float *act,
                            const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                            const pr_net_params &actor, const pr_net_params &critic, const pr_net_params &ga,
                            const pr_net_params &gc, void *scratch, float *stats) {
  const int B = c.batch, D = c.n_stocks, Hd = c.hidden, S = 1 + 2 * D + D * c.n_ind, Sp = (S + 3) / 4 * 4;
  unsigned char *p = static_cast<unsigned char *>(scratch);
  auto take = [&](size_t bytes) {
    float *r = reinterpret_cast<float *>(p);
    p += align256(bytes);
    return r;
  };
  Scratch w;
  w.xp = take((size_t)B * Sp * 4);
  for (int net = 0; net < 2; ++net) {
    w.h1[net] = take((size_t)B * Hd * 4);
    w.h2[net] = take((size_t)B * Hd * 4);
  }
  w.out = take((size_t)B * D * 4);
  w.dz3 = take((size_t)B * D * 4);
  w.dz2 = take((size_t)B * Hd * 4);
  w.dz1 = take((size_t)B * Hd * 4);
  w.v = take((size_t)B * 4);
  w.dzc = take((size_t)B * 4);
  const int blocks = (B + 7) / 8;
  w.partial = take((size_t)blocks * 4 * 4);
  w.splitk_floats = splitk_floats(Hd);
  w.splitk = take(w.splitk_floats * 4);
  // gather once, both forwards (each network keeps its own activations), the loss, both backward passes
  hipLaunchKernelGGL(gather_pad_kernel, dim3((unsigned)((B + 3) / 4)), dim3(256), 0, st, B, S, Sp, obs, rows, w.xp);
  LRN(net_forward(st, B, S, Sp, Hd, 1, false, 1, critic, w, w.v));
  LRN(net_forward(st, B, S, Sp, Hd, D, true, 0, actor, w, w.out));
  LossArgs l;
  l.B = B, l.D = D, l.mu = w.out, l.v = w.v, l.act = act, l.logp_old = logp_old, l.adv = adv, l.ret = ret, l.rows = rows;
  l.sigma = c.sigma, l.clip = c.clip, l.value_coef = c.value_coef, l.dz_actor = w.dz3, l.dz_critic = w.dzc;
  l.partial = w.partial;
  hipLaunchKernelGGL(ppo_loss_kernel, dim3(blocks), dim3(256), 0, st, l);
  if (stats) hipLaunchKernelGGL(ppo_stats_kernel, dim3(1), dim3(256), 0, st, blocks, w.partial, stats);
  LRN(net_backward(st, B, S, Sp, Hd, D, 0, actor, w, w.dz3, ga));
  LRN(net_backward(st, B, S, Sp, Hd, 1, 1, critic, w, w.dzc, gc));
  return hipGetLastError();
}

// ---- the same minibatch for callers that cannot allocate or own a workspace: scratch in a fixed device array
// (one copy per GPU the library runs on, held until the process ends).  In host code the array's name is only a
// stand-in for the symbol: its device address is looked up once per device and that pointer is what kernels get.
constexpr size_t kStaticScratchBytes = (size_t)24 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
}  // namespace

size_t ppo_static_scratch_bytes() { return kStaticScratchBytes; }

hipError_t launch_ppo_grads_static(hipStream_t st, const pr_ppo_config &c, const float *obs, const float *act,
                                   const float *logp_old, const float *adv, const float *ret, const int32_t *rows,
                                   const pr_net_params &actor, const pr_net_params &critic, const pr_net_params &ga,
                                   const pr_net_params &gc, float *stats) {
  const int S = 1 + 2 * c.n_stocks + c.n_stocks * c.n_ind;
  if (ppo_scratch_bytes(c.batch, c.hidden, c.n_stocks, S) > kStaticScratchBytes) return hipErrorInvalidValue;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    // first call on this device (with it current): every GPU holds its own copy of the array at its own address
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  // nothing in the scratch has to start at zero: every region is written by this call before it is read
  return launch_ppo_grads(st, c, obs, act, logp_old, adv, ret, rows, actor, critic, ga, gc, ptr, stats);
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
