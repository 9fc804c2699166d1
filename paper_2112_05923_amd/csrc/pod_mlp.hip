// Three-layer perceptron forward (actor / critic networks of a pod, Sec. 4.1
// "training files" and Sec. 4.2 worker) on the matrix cores of gfx950.
//
// One workgroup (4 wavefronts) owns a tile of BM = 32 RT rows and carries it
// through all three layers without leaving the compute unit:
//   layer 1: A = rows of X, staged from global memory into LDS in k-chunks
//            (converted to the operand type on the way), B = packed weights;
//   layer 2: A = hidden tile in LDS;   layer 3: A = hidden tile in LDS.
// The four wavefronts split the OUTPUT COLUMNS of a layer, so the activation
// tile is the shared operand (LDS) and every weight block is fetched by
// exactly one wavefront, straight from global/L2 into the registers it is
// consumed from: weights are pre-packed in the B-operand register layout, so a
// block is one 1-KiB fully coalesced load.  Accumulators (fp32) stay in
// registers for a whole layer; bias + tanh are applied once, on the way to LDS.
//
// Operand types: bf16 (v_mfma_f32_32x32x16_bf16, k-block 16) or fp32
// (v_mfma_f32_32x32x2_f32 x 4, k-block 8).  In both, lane l of a wavefront
// feeds row/column (l % 32) and the k-half (l / 32) of a k-block: 16 bytes per
// lane and operand.
#include "pod_internal.h"
#include <type_traits>

#include "pod_tile.h"

namespace pod {

namespace {

using tile::f32x16;
using tile::f32x4;
using tile::u32x4;
using tile::Op;  // operand types: k-block size, element size, the matrix instruction, LDS stores
using tile::tanh_accurate;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

struct MlpArgs {
  const float *X;
  int64_t ldx;
  int64_t rows;
  float *Y;
  PackedNet net;
  int32_t N, envs_per_agent;
  int64_t row_offset;  // global index of row 0 of X (agent lookup when a tail is launched on its own)
  int32_t xpitch;   // bytes per row of one staged X chunk
  int32_t hpitch;   // bytes per row of the hidden tile
};

// B-operand block (ct, kb) of a packed layer for this lane.
__device__ inline u32x4 load_b(const u32x4 *Wp, int nct, int ct, int kb, int lane) {
  return Wp[((size_t)kb * nct + ct) * 64 + lane];
}

// acc += A(tile in LDS, all k-blocks) * B.  Wavefront-uniform control flow.
template <bool BF16, int RT, int CT, int PD>
__device__ inline void layer_from_lds(f32x16 (&acc)[RT][CT], const unsigned char *ldsA, int pitch, int nkb,
                                      const u32x4 *Wp, int ct0, int nct, int lane) {
  using O = Op<BF16>;
  const int arow = lane & 31, g = lane >> 5;
  int cts[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) cts[c] = min(ct0 + c, nct - 1);
  u32x4 ring[PD][CT];
#pragma unroll
  for (int s = 0; s < PD; ++s)
    if (s < nkb) {
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = load_b(Wp, nct, cts[c], s, lane);
    }
  for (int kb0 = 0; kb0 < nkb; kb0 += PD) {
#pragma unroll
    for (int s = 0; s < PD; ++s) {
      const int kb = kb0 + s;
      if (kb < nkb) {
        u32x4 a[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r)
          a[r] = *reinterpret_cast<const u32x4 *>(ldsA + (size_t)(r * 32 + arow) * pitch + kb * 32 + 16 * g);
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
          for (int c = 0; c < CT; ++c) O::mma(a[r], ring[s][c], acc[r][c]);
        if (kb + PD < nkb) {
#pragma unroll
          for (int c = 0; c < CT; ++c) ring[s][c] = load_b(Wp, nct, cts[c], kb + PD, lane);
        }
      }
    }
  }
}

// acc += A(rows of X in global memory, staged through two LDS chunk buffers) * B.
// Every wavefront of the workgroup must call this (staging and barriers are
// collective); `active` says whether this wavefront owns any output column.
template <bool BF16, int RT, int CT, int PD>
__device__ inline void layer_from_global(f32x16 (&acc)[RT][CT], unsigned char *ldsX, int xpitch, const float *X,
                                         int64_t ldx, int64_t row0, int nrows, int S, int nkb, const u32x4 *Wp,
                                         int ct0, int nct, bool active, int tid) {
  using O = Op<BF16>;
  constexpr int BM = 32 * RT;
  constexpr int KC = PD * O::KB;             // inputs per staged chunk (power of two)
  constexpr int NPRE = BM * KC / 4 / kThreads;  // groups of four columns each thread stages per chunk
  const int lane = tid & 63;
  const int arow = lane & 31, g = lane >> 5;
  const int nch = (nkb + PD - 1) / PD;
  const size_t xbuf = (size_t)BM * xpitch;

  int cts[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) cts[c] = min(ct0 + c, nct - 1);
  u32x4 ring[PD][CT];
  if (active) {
#pragma unroll
    for (int s = 0; s < PD; ++s)
      if (s < nkb) {
#pragma unroll
        for (int c = 0; c < CT; ++c) ring[s][c] = load_b(Wp, nct, cts[c], s, lane);
      }
  }

  // a thread moves groups of four consecutive columns of one row: one 16-byte load (rows are only 4-byte
  // aligned, which a global load allows) and one 8- or 16-byte LDS store; the group that straddles the end of
  // the row is read element by element
  f32x4 pre[NPRE];
  auto gload = [&](int ch) {
#pragma unroll
    for (int i = 0; i < NPRE; ++i) {
      const int idx = tid + kThreads * i;
      const int row = idx / (KC / 4), col = ch * KC + 4 * (idx % (KC / 4));
      f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
      if (row < nrows) {
        const float *src = X + (row0 + row) * ldx + col;
        if (col + 3 < S) {
          v = *reinterpret_cast<const f32x4 *>(src);
        } else {
          if (col < S) v[0] = src[0];
          if (col + 1 < S) v[1] = src[1];
          if (col + 2 < S) v[2] = src[2];
        }
      }
      pre[i] = v;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NPRE; ++i) {
      const int idx = tid + kThreads * i;
      const int row = idx / (KC / 4), col = 4 * (idx % (KC / 4));
      O::store4(ldsX + buf * xbuf + (size_t)row * xpitch + col * O::ESZ, pre[i][0], pre[i][1], pre[i][2], pre[i][3]);
    }
  };

  gload(0);
  sstore(0);
  __syncthreads();
  for (int ch = 0; ch < nch; ++ch) {
    const bool more = ch + 1 < nch;
    if (more) gload(ch + 1);
    if (active) {
      const unsigned char *buf = ldsX + (ch & 1) * xbuf;
#pragma unroll
      for (int s = 0; s < PD; ++s) {
        const int kb = ch * PD + s;
        if (kb < nkb) {
          u32x4 a[RT];
#pragma unroll
          for (int r = 0; r < RT; ++r)
            a[r] = *reinterpret_cast<const u32x4 *>(buf + (size_t)(r * 32 + arow) * xpitch + s * 32 + 16 * g);
#pragma unroll
          for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int c = 0; c < CT; ++c) O::mma(a[r], ring[s][c], acc[r][c]);
          if (kb + PD < nkb) {
#pragma unroll
            for (int c = 0; c < CT; ++c) ring[s][c] = load_b(Wp, nct, cts[c], kb + PD, lane);
          }
        }
      }
    }
    if (more) sstore((ch + 1) & 1);
    __syncthreads();
  }
}

template <int RT, int CT>
__device__ inline void zero_acc(f32x16 (&acc)[RT][CT]) {
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[r][c][i] = 0.0f;
}

// hidden = tanh(acc + bias) -> LDS tile in the operand type.
// Accumulator register i of lane l holds row 8 (i / 4) + 4 (l / 32) + i % 4, column l % 32 of a 32x32 tile.
template <bool BF16, int RT, int CT>
__device__ inline void epilogue_to_lds(const f32x16 (&acc)[RT][CT], const float *bias, unsigned char *ldsH, int hpitch,
                                       int ct0, int nct, int lane) {
  using O = Op<BF16>;
  const int g = lane >> 5, cl = lane & 31;
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    if (ct0 + c < nct) {
      const int col = (ct0 + c) * 32 + cl;
      const float bv = bias[col];
#pragma unroll
      for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = r * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          const float z = acc[r][c][i] + bv;
          const float hval = BF16 ? tile::tanh_from_scaled(z * tile::kTwoLog2e) : tanh_accurate(z);
          O::store1(ldsH + (size_t)row * hpitch + col * O::ESZ, hval);
        }
    }
  }
}

template <int RT, int CT>
__device__ inline void epilogue_to_global(const f32x16 (&acc)[RT][CT], const float *bias, float *Y, int64_t row0,
                                          int nrows, int O_dim, int out_tanh, int ct0, int nct, int lane) {
  const int g = lane >> 5, cl = lane & 31;
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    if (ct0 + c < nct) {
      const int col = (ct0 + c) * 32 + cl;
      const float bv = bias[col];
#pragma unroll
      for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = r * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          const float z = acc[r][c][i] + bv;
          const float y = out_tanh ? tanh_accurate(z) : z;
          if (row < nrows && col < O_dim) Y[(row0 + row) * O_dim + col] = y;
        }
    }
  }
}

// TAG only separates the symbol of the per-step launches (0) from that of the
// whole-buffer launches (1) so that a profiler reports them as two kernels.
template <bool BF16, int RT, int CTH, int CTO, int TAG>
__global__ __launch_bounds__(kThreads) void mlp3_kernel(MlpArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int BM = 32 * RT;
  constexpr int PDH = CTH >= 8 ? 2 : 4;
  constexpr int PDO = CTO >= 8 ? 2 : 4;
  unsigned char *ldsH = lds;
  unsigned char *ldsX = lds + (size_t)BM * a.hpitch;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t row0 = (int64_t)blockIdx.x * BM;
  const int nrows = (int)min((int64_t)BM, a.rows - row0);
  const int agent = (int)(((row0 + a.row_offset) % a.N) / a.envs_per_agent);
  const PackedNet &net = a.net;
  const u32x4 *W1 = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(net.W[0]) +
                                                    (size_t)agent * net.w_stride[0]);
  const u32x4 *W2 = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(net.W[1]) +
                                                    (size_t)agent * net.w_stride[1]);
  const u32x4 *W3 = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(net.W[2]) +
                                                    (size_t)agent * net.w_stride[2]);
  const float *b1 = net.b[0] + (size_t)agent * net.b_stride[0];
  const float *b2 = net.b[1] + (size_t)agent * net.b_stride[1];
  const float *b3 = net.b[2] + (size_t)agent * net.b_stride[2];

  const int cth0 = w * CTH;
  const bool act_h = cth0 < net.nct[0];
  {
    f32x16 acc[RT][CTH];
    zero_acc<RT, CTH>(acc);
    layer_from_global<BF16, RT, CTH, PDH>(acc, ldsX, a.xpitch, a.X, a.ldx, row0, nrows, net.in_dim[0], net.nkb[0], W1,
                                          cth0, net.nct[0], act_h, tid);
    if (act_h) epilogue_to_lds<BF16, RT, CTH>(acc, b1, ldsH, a.hpitch, cth0, net.nct[0], lane);
    __syncthreads();
    zero_acc<RT, CTH>(acc);
    if (act_h) layer_from_lds<BF16, RT, CTH, PDH>(acc, ldsH, a.hpitch, net.nkb[1], W2, cth0, net.nct[1], lane);
    __syncthreads();  // every wavefront has read the whole layer-1 tile
    if (act_h) epilogue_to_lds<BF16, RT, CTH>(acc, b2, ldsH, a.hpitch, cth0, net.nct[1], lane);
    __syncthreads();
  }
  {
    const int cto0 = w * CTO;
    if (cto0 < net.nct[2]) {
      f32x16 acc[RT][CTO];
      zero_acc<RT, CTO>(acc);
      layer_from_lds<BF16, RT, CTO, PDO>(acc, ldsH, a.hpitch, net.nkb[2], W3, cto0, net.nct[2], lane);
      epilogue_to_global<RT, CTO>(acc, b3, a.Y, row0, nrows, net.out_dim[2], net.out_tanh, cto0, net.nct[2], lane);
    }
  }
}


// ------------------------------------------------ one layer per launch, for few rows
// A step of a small batch (a few thousand envs) has fewer 64-row tiles than the chip has compute units, and a
// kernel that carries a row tile through all three layers leaves the rest idle.  Here a launch computes ONE
// layer, tiled over rows x output features: workgroup (x, y) owns rows [32 x, 32 x + 32) and the four feature
// tiles [4 y, 4 y + 4), one per wavefront, so rows / 32 x features / 128 workgroups run (512 for 2048 rows and
// 1024 hidden units); the input rows are staged 16 k-blocks at a time, because with so little arithmetic per
// workgroup the time goes to the memory round trips, one per staged chunk.  Activations travel between the launches as fp32 rows in global memory (they stay in L2)
// and are rounded to the operand type when they are staged, exactly where the whole-network kernels round them.
constexpr int kSplitPD = 16;  // k-blocks per staged chunk of the layer-per-launch kernel
struct LayerArgs {
  const float *X;      // [rows, ldx]
  int64_t ldx, rows;
  int64_t row_offset;  // index of X's first row in the caller's buffer (selects the agent)
  float *Y;            // [rows, ldy]
  int64_t ldy;
  const void *W;       // packed weights of the layer, agent-major
  const float *b;      // padded biases, agent-major
  int64_t w_stride;    // bytes between agents
  int32_t b_stride;    // floats between agents
  int32_t in_dim, out_dim, nkb, nct;
  int32_t act;         // 0: linear, 1: tanh of a hidden layer, 2: tanh of an output layer (full accuracy)
  int32_t N, envs_per_agent;
  int32_t xpitch;
};

template <bool BF16, int RT, int PD>
__global__ __launch_bounds__(kThreads) void dense_layer_kernel(LayerArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int BM = 32 * RT;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t row0 = (int64_t)blockIdx.x * BM;
  const int nrows = (int)min((int64_t)BM, a.rows - row0);
  const int agent = (int)(((row0 + a.row_offset) % a.N) / a.envs_per_agent);
  const u32x4 *Wp = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(a.W) + (size_t)agent * a.w_stride);
  const float *bias = a.b + (size_t)agent * a.b_stride;
  const int ct0 = blockIdx.y * kWaves + w;
  const bool active = ct0 < a.nct;
  f32x16 acc[RT][1];
  zero_acc<RT, 1>(acc);
  layer_from_global<BF16, RT, 1, PD>(acc, lds, a.xpitch, a.X, a.ldx, row0, nrows, a.in_dim, a.nkb, Wp, ct0, a.nct, active,
                                     tid);
  if (!active) return;
  const int g = lane >> 5, col = ct0 * 32 + (lane & 31);
  const float bv = bias[col];
#pragma unroll
  for (int r = 0; r < RT; ++r)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = r * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
      const float z = acc[r][0][i] + bv;
      float y = z;
      if (a.act == 1) y = BF16 ? tile::tanh_from_scaled(z * tile::kTwoLog2e) : tanh_accurate(z);
      if (a.act == 2) y = tanh_accurate(z);
      if (row < nrows && col < a.out_dim) a.Y[(row0 + row) * a.ldy + col] = y;
    }
}

// ------------------------------------------------ persistent whole-tile kernel
// Used when the rows of X are dense (ldx == S) and a whole 64 x S tile fits in
// LDS next to the hidden tile.  Each workgroup walks tiles blockIdx.x,
// blockIdx.x + gridDim.x, ...; the next tile's rows are fetched into registers
// (16-byte loads, four columns of one row each) while the current tile is in
// the matrix cores, and dropped into the LDS input tile, converted to the
// operand type, once layer 1 has finished reading it.
constexpr int XPRE_MAX = 10;  // 16-byte loads per thread and tile

struct TileArgs {
  const float *X;
  int64_t rows;       // multiple of 64
  int64_t row_base;   // index of X's first row in the caller's buffer (selects the agent)
  float *Y;
  PackedNet net;
  int32_t N, envs_per_agent;
  int32_t S;
  int32_t groups;     // ceil(S / 4): 16-byte groups per row
  int32_t g_magic;    // ceil(2^32 / groups): i / groups == umulhi(i, g_magic) for the small i used here
  int32_t xpitch, hpitch;
};

template <bool BF16, int NW, int CTH, int NKB1, int NKB2, int TAG>
__global__ __launch_bounds__(NW * 64) void mlp_tiles_kernel(TileArgs a) {
  using namespace tile;
  using O = tile::Op<BF16>;
  constexpr int NT = NW * 64;
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char *ldsH = lds;
  unsigned char *ldsX = lds + (size_t)BM * a.hpitch;
  u32x4 *ldsW3 = reinterpret_cast<u32x4 *>(ldsX + (size_t)BM * a.xpitch);
  float *ldsBias = reinterpret_cast<float *>(ldsW3 + (size_t)a.net.nkb[2] * 64);
  const int tid = threadIdx.x;
  const int S = a.S, G = a.groups;
  const int64_t ntiles = a.rows / BM;
  const int ngroups = BM * G;
  const int nx = (ngroups + NT - 1) / NT;

  // Branch-free fetch: every thread issues nx unconditional 16-byte loads (threads past the last group
  // re-read the last group).  The group that straddles the end of a row is read as the four floats that
  // END at the row end and is shifted into place, with zeros behind, when it is stored.
  f32x4 pre[XPRE_MAX];
  auto fetch = [&](int64_t t) {
    const float *src = a.X + t * BM * S;
#pragma unroll
    for (int i = 0; i < XPRE_MAX; ++i) {
      if (i < nx) {
        const int idx = min(tid + NT * i, ngroups - 1);
        const int row = (int)__umulhi((unsigned)idx, (unsigned)a.g_magic);
        const int c4 = 4 * (idx - row * G);
        const int shift = max(0, c4 + 4 - S);
        pre[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src + (size_t)row * S + c4 - shift));  // 4-byte aligned
      }
    }
  };
  auto stash = [&]() {
    // the LDS addresses are loop invariant; recompute them per call instead of letting the compiler keep
    // them in registers across the matrix-core loops
    int tid_opaque = tid;
    asm volatile("" : "+v"(tid_opaque));
#pragma unroll
    for (int i = 0; i < XPRE_MAX; ++i) {
      if (i < nx) {
        const int idx = tid_opaque + NT * i;
        const int idc = min(idx, ngroups - 1);
        const int row = (int)__umulhi((unsigned)idc, (unsigned)a.g_magic);
        const int c4 = 4 * (idc - row * G);
        const int shift = max(0, c4 + 4 - S);
        const f32x4 v = pre[i];
        const float o0 = shift == 0 ? v[0] : shift == 1 ? v[1] : shift == 2 ? v[2] : v[3];
        const float o1 = shift == 0 ? v[1] : shift == 1 ? v[2] : shift == 2 ? v[3] : 0.0f;
        const float o2 = shift == 0 ? v[2] : shift == 1 ? v[3] : 0.0f;
        const float o3 = shift == 0 ? v[3] : 0.0f;
        // the group that straddles S also writes the zero padding of the k columns
        if (idx < ngroups) O::store4(ldsX + (size_t)row * a.xpitch + c4 * O::ESZ, o0, o1, o2, o3);
      }
    }
  };

  // The first tile's rows are requested before anything else, so that they travel while the tile is cleared and
  // the first network's biases and output weights are staged; every tile's first weight blocks are requested
  // before the barrier that completes its inputs.
  int64_t t = blockIdx.x;
  int staged_agent = -1;
  if (t < ntiles) fetch(t);
  // k columns beyond the last group (when Kp > 4 * groups) are never written by stash: clear the tile once
  for (int i = tid; i < BM * a.xpitch / 4; i += NT) reinterpret_cast<uint32_t *>(ldsX)[i] = 0u;
  __syncthreads();
  if (t < ntiles) {
    const int agent = (int)(((a.row_base + t * BM) % a.N) / a.envs_per_agent);
    stage_net<NT>(net_of(a.net, agent), ldsBias, ldsW3, tid);
    staged_agent = agent;
    stash();
  }
  const int lane_p = tid & 63, ct0_p = __builtin_amdgcn_readfirstlane(tid >> 6) * CTH;
  u32x4 ring[ring_depth(CTH)][CTH];
  for (; t < ntiles; t += gridDim.x) {
    const int64_t row0 = t * BM;
    const int64_t tn = t + gridDim.x;
    const bool more = tn < ntiles;
    const int agent = (int)(((a.row_base + row0) % a.N) / a.envs_per_agent);
    const Net net = net_of(a.net, agent);
    if (ct0_p < net.nct[0]) prime<CTH, ring_depth(CTH)>(ring, net.W[0], net.nkb[0], net.nct[0], ct0_p, lane_p);
    if (agent != staged_agent) {
      __syncthreads();  // the previous tile's output layer may still read its weights and biases
      stage_net<NT>(net, ldsBias, ldsW3, tid);
      staged_agent = agent;
    }
    __syncthreads();  // input tile, biases and W3 complete; previous tile's output layer is done with ldsH
    const int O_dim = net.out_dim;
    float *Y = a.Y + row0 * O_dim;
    mlp_tile<BF16, NW, CTH, false, NKB1, NKB2, true, false>(
        net, ring, ldsX, a.xpitch, ldsH, a.hpitch, ldsBias, ldsW3, tid,
        [&]() {
          if (more) fetch(tn);
        },
        [&]() {
          if (more) stash();
        },
        [&](int b, int f, float y) { __builtin_nontemporal_store(y, &Y[(size_t)b * O_dim + f]); });
  }
}


// ------------------------------------------------ whole-tile kernel for wide inputs
// Observation rows that do not fit in LDS next to the hidden tile (S > 320: a hundred and more stocks) or an
// output layer with several feature tiles: the same tile engine, but layer 1's activations arrive in chunks of
// CC input columns through two LDS buffers.  A chunk is fetched into registers (16-byte loads; rows need only be
// 4-byte aligned) behind the matrix work of the chunk before it, converted and dropped into the other buffer;
// one barrier per chunk; the weight ring runs on across the chunks.  Rows past `rows` (ragged last tile) are
// read as zeros and not stored.
struct WideArgs {
  const float *X;
  int64_t ldx, rows;
  int64_t row_base;
  float *Y;
  PackedNet net;
  int32_t N, envs_per_agent;
  int32_t S;
  int32_t cpitch, hpitch;
};

template <int NW, int CTH, bool WIDE_OUT, int CC>
__global__ __launch_bounds__(NW * 64) void mlp_wide_kernel(WideArgs a) {
  using namespace tile;
  using O = tile::Op<true>;
  constexpr int NT = NW * 64;
  constexpr int NG = BM * CC / 4 / NT;  // 16-byte groups per thread and chunk
  constexpr int CKB = CC / O::KB;       // k-blocks per chunk
  constexpr int PD = ring_depth(CTH);
  static_assert(NG >= 1 && CKB % PD == 0, "chunk geometry");
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char *ldsH = lds;
  unsigned char *ldsC = lds + (size_t)BM * a.hpitch;  // two chunk buffers
  const size_t cbuf = (size_t)BM * a.cpitch;
  u32x4 *ldsW3 = reinterpret_cast<u32x4 *>(ldsC + 2 * cbuf);
  float *ldsBias = reinterpret_cast<float *>(ldsW3 + (WIDE_OUT ? 0 : (size_t)a.net.nkb[2] * 64));
  const int tid = threadIdx.x, lane = tid & 63;
  const int ct0 = __builtin_amdgcn_readfirstlane(tid >> 6) * CTH;
  const int S = a.S;
  const int64_t ntiles = (a.rows + BM - 1) / BM;
  int staged_agent = -1;

  for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int64_t row0 = t * BM;
    const int nrows = (int)min((int64_t)BM, a.rows - row0);
    const int agent = (int)(((a.row_base + row0) % a.N) / a.envs_per_agent);
    const Net net = net_of(a.net, agent);
    const int nkb = net.nkb[0], nch = (nkb + CKB - 1) / CKB;

    f32x4 pre[NG];
    auto fetch = [&](int ch) {
#pragma unroll
      for (int i = 0; i < NG; ++i) {
        const int idx = tid + NT * i;
        const int row = idx / (CC / 4), col = ch * CC + 4 * (idx % (CC / 4));
        f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (row < nrows) {
          const float *src = a.X + (row0 + row) * a.ldx + col;
          if (col + 3 < S) {
            v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src));
          } else {
            if (col < S) v[0] = src[0];
            if (col + 1 < S) v[1] = src[1];
            if (col + 2 < S) v[2] = src[2];
          }
        }
        pre[i] = v;
      }
    };
    auto stash = [&](int buf) {
#pragma unroll
      for (int i = 0; i < NG; ++i) {
        const int idx = tid + NT * i;
        const int row = idx / (CC / 4), c4 = 4 * (idx % (CC / 4));
        O::store4(ldsC + buf * cbuf + (size_t)row * a.cpitch + c4 * O::ESZ, pre[i][0], pre[i][1], pre[i][2], pre[i][3]);
      }
    };

    fetch(0);
    if (agent != staged_agent) {
      __syncthreads();  // the previous tile's output layer may still read its weights and biases
      stage_net<NT>(net, ldsBias, WIDE_OUT ? nullptr : ldsW3, tid);
      staged_agent = agent;
    }
    float *Y = a.Y + row0 * net.out_dim;
    const int O_dim = net.out_dim;
    u32x4 ring[PD][CTH];
    mlp_tile<true, NW, CTH, WIDE_OUT, 0, 0, true, false>(
        net, ring, nullptr, 0, ldsH, a.hpitch, ldsBias, ldsW3, tid, [] {}, [] {},
        [&](int b, int f, float y) {
          if (b < nrows) Y[(size_t)b * O_dim + f] = y;
        },
        [&](f32x16 (&acc)[CTH][2], u32x4 (&rg)[PD][CTH], bool act) {
          if (act) prime<CTH, PD>(rg, net.W[0], nkb, net.nct[0], ct0, lane);
          for (int ch = 0; ch < nch; ++ch) {
            stash(ch & 1);
            __syncthreads();  // chunk ch complete; everybody is done with the buffer chunk ch + 1 goes into
            if (ch + 1 < nch) fetch(ch + 1);
            if (act)
              mma_layer_range<true, CTH, 2, PD>(acc, rg, ldsC + (ch & 1) * cbuf, a.cpitch, ch * CKB,
                                                min(nkb, (ch + 1) * CKB), nkb, net.W[0], net.nct[0], ct0, 0, lane);
          }
        });
    __syncthreads();  // the hidden tile and the chunk buffers are free again
  }
}

// ------------------------------------------------ 128-row value-head kernel
// The critic (one output feature, Sec. 4.1) over a long buffer of observations.
// A 128-row tile halves the weight traffic per row of the 64-row kernel above:
// every weight block a wavefront streams from L2 feeds four 32-row batch tiles,
// which makes the two hidden layers matrix-core bound instead of L2 bound.
//
// Matrix instructions and the vector / transcendental instructions of the tanh
// epilogues co-issue on a SIMD when they come from DIFFERENT wavefronts, so the
// eight wavefronts work as two groups that are half a layer out of step: group
// A (wavefronts 0-3, hidden features 0-255) and group B (wavefronts 4-7,
// features 256-511), one wavefront of each per SIMD.  Per tile, with a
// workgroup barrier between the phases:
//
//   phase   group A                                group B
//   1       layer 1 (matrix)                       epilogue 2 + output dot of the PREVIOUS tile
//   2       epilogue 1 -> hidden half A            layer 1 (matrix)
//   3       layer 2 over k in half A (matrix)      epilogue 1 -> hidden half B
//   4       layer 2 over k in half B (matrix)      layer 2 over k in half B (matrix)
//   5       epilogue 2 + output dot                layer 2 over k in half A (matrix)
//
// so in four of the five phases one wavefront of every SIMD feeds the matrix
// pipe while the other runs an epilogue.  LDS: hidden half A; one region that
// holds the input tile (phases 1-2), then hidden half B (phases 3-4), then the
// next input tile (written in phase 5, behind loads issued in phase 4).
//  - The output layer is folded into layer 2's epilogue: each lane multiplies
//    its bf16-rounded activations by the output weights of its features and the
//    16 partial sums per row (8 wavefronts x 2 lane halves) meet in LDS; they
//    are added up one phase after group B has delivered its share.
//  - Every wavefront's weight ring runs on across the phases: the last blocks of
//    a range are replaced by the first blocks of the wavefront's next range, so
//    no matrix phase starts with a round trip to L2.
#ifndef POD_VK_PRIO
#define POD_VK_PRIO 3
#endif
constexpr int kMatrixPrio = POD_VK_PRIO;  // wavefront priority of the matrix steps (epilogue steps run at 0)
constexpr int VBM = 128;
constexpr int VPRE_MAX = 19;  // 16-byte loads per thread and tile: k-blocks of layer 1
constexpr int VHALF = 256;    // hidden features per group
constexpr int VHPITCH = VHALF * 2 + 16;  // bytes per row of a hidden half

struct ValueArgs {
  const float *X;
  int64_t rows;      // multiple of the tile height
  float *Y;          // [rows]
  PackedNet net;
  int32_t N, envs_per_agent;
  int32_t S;
  int32_t groups;    // 16-byte groups per LDS row: padded k columns / 4
  uint32_t g_magic;  // ceil(2^32 / groups)
  int32_t xpitch;
  int32_t off_xb, off_bias, off_w3, off_part;  // LDS byte offsets: input tile / hidden half B, b1 | b2, output weights, partial sums
};

template <int NKB1, int SS>
__global__ __launch_bounds__(512) void value_kernel(ValueArgs a) {
  using namespace tile;
  using O = tile::Op<true>;
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  constexpr int NW = 8, NBT = 4, NT = NW * 64, CTH = 16 / NW, PD = 4, NKBH = VHALF / 16;
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char *ldsHA = lds;                 // hidden features 0..255, [VBM][VHPITCH]
  unsigned char *ldsXB = lds + a.off_xb;      // input tile [VBM][xpitch], later hidden features 256..511 [VBM][VHPITCH]
  float *ldsBias = reinterpret_cast<float *>(lds + a.off_bias);  // b1 | b2
  __bf16 *ldsW3 = reinterpret_cast<__bf16 *>(lds + a.off_w3);    // output weights, one per hidden feature
  float *ldsPart = reinterpret_cast<float *>(lds + a.off_part);  // [2 NW][VBM] partial sums of the output layer
  const int nct = a.net.nct[0];               // 16 feature tiles in both hidden layers
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool grpB = w >= NW / 2;
  const int ct0 = w * CTH;
  const int S = SS > 0 ? SS : a.S;           // (compile-time for the named workloads: the index
  const int G = NKB1 > 0 ? 4 * NKB1 : a.groups;  //  arithmetic of fetch and stash folds into constants)
  auto row_of_group = [&](int idx) { return NKB1 > 0 ? idx / (4 * (NKB1 > 0 ? NKB1 : 1)) : (int)__umulhi((unsigned)idx, a.g_magic); };
  const int last_c4 = 4 * ((S + 3) / 4 - 1);  // first column of the last group that holds data
  const int64_t ntiles = a.rows / VBM;

  // The next input tiles travel through registers, 16-byte groups of four columns (76 per row at most), 19 per
  // thread.  Two rules shape this.  (1) A wavefront's loads return in order, so a row request in flight during one
  // of its matrix steps would hold up the weight blocks (L2 hits) behind it: rows are requested and received
  // only inside the epilogue steps (b) and (e), and carried across matrix steps packed in the operand type.
  // (2) All compute units walk their tiles in step, so a whole tile per compute unit requested at once would be a
  // 39 MB burst: the requests are spread over four of the five phases.
  //   chunk 0 (NX0 groups): requested at the start of step (b), packed at its end, carried to phase 5 (group A:
  //            start of its step (e); group B: start of its step (d)) and written to the input region there.
  //   chunk 1 (NX1 groups): requested at the start of step (e).  Group A is in phase 5 then: written at the end of
  //            the step.  Group B is already in phase 1 of the next tile, whose input must not be touched: it
  //            requests the rows of the tile AFTER the next one, packs them and carries them to its next step (d).
  constexpr int NX0 = 10, NX1 = 9;
  static_assert(NT * (NX0 + NX1) >= VBM * 4 * VPRE_MAX, "every group of the input tile has an owner");
  const int sh = 4 * ((S + 3) / 4) - S;            // floats the row-end group is shifted by (0..3), uniform
  f32x4 pre[NX0 > NX1 ? NX0 : NX1];                // requests in flight
  u32x2 held0[NX0], held1[NX1];                    // chunks in the operand type
  // Every thread issues its loads unconditionally.  The group that straddles the end of a row is read as the four
  // floats that END at the row end; groups that lie wholly in the k padding, or past the tile, re-read a valid one.
  // Which 16-byte group a thread moves with its i-th request of a chunk.
  //  - Rows wider than 64 groups with the width known at compile time (the named workloads: 76 groups): every
  //    wavefront owns 16 rows of the tile; a request of the "main" kind covers groups 0..63 of one row (lane =
  //    group: 1 KiB contiguous, and the LDS address is the lane's base plus a constant), the remaining TG groups of
  //    the 16 rows are covered by 64-lane "tail" requests in row-major order.  Chunk 0 = main rows 0..9, chunk 1 =
  //    main rows 10..15 and the tail.  Only tail groups can hold a row end.
  //  - Otherwise: groups dealt out to the threads in order (index arithmetic per group).
  constexpr bool ROWS = NKB1 > 16 && SS > 0;
  constexpr int GC = ROWS ? 4 * NKB1 : 65, TG = GC - 64, NTAIL = (16 * TG + 63) / 64;
  static_assert(!ROWS || (NX0 == 10 && 6 + NTAIL <= NX1), "chunk sizes of the row-owning scheme");
  auto group_index = [&](int tid_g, int i, auto part) { return (decltype(part)::value ? NX0 * NT : 0) + tid_g + NT * i; };
  // float offset of the group inside the tile, as requested (the row-end group is read shifted)
  auto src_offset_general = [&](int idx) {
    const int idc = min(idx, VBM * G - 1);
    const int row = row_of_group(idc);
    const int c4 = min(4 * (idc - row * G), last_c4);
    return row * S + (c4 == last_c4 ? c4 - sh : c4);
  };
  auto tail_group = [&](int lane_t, int j, int *row, int *g) {  // ROWS: tail request j of a lane
    const int q = min(lane_t + 64 * j, 16 * TG - 1);
    *row = q / TG;
    *g = 64 + q - *row * TG;
  };
  auto fetch = [&](int64_t t, auto part) {
    constexpr bool P1 = decltype(part)::value;
    constexpr int CNT = P1 ? NX1 : NX0;
    int tid_f = threadIdx.x;
    asm volatile("" : "+v"(tid_f));
    if constexpr (ROWS) {
      const int lane_f = tid_f & 63;
      const float *src = a.X + (t * VBM + 16 * w) * S;
      constexpr int R0 = P1 ? NX0 : 0, NR = P1 ? 16 - NX0 : NX0;
#pragma unroll
      for (int r = 0; r < NR; ++r)
        pre[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src + (R0 + r) * S + 4 * lane_f));
      if constexpr (P1) {
#pragma unroll
        for (int j = 0; j < NTAIL; ++j) {
          int row, g;
          tail_group(lane_f, j, &row, &g);
          const int c4 = 4 * g;
          pre[NR + j] = __builtin_nontemporal_load(
              reinterpret_cast<const f32x4 *>(src + row * S + (c4 == last_c4 ? c4 - sh : c4)));
        }
      }
    } else {
      const float *src = a.X + t * VBM * S;
#pragma unroll
      for (int i = 0; i < CNT; ++i)
        pre[i] = __builtin_nontemporal_load(
            reinterpret_cast<const f32x4 *>(src + src_offset_general(group_index(tid_f, i, part))));
    }
  };
  // a received group as four operand-type values; `end`: it is the row-end group (shifted down, zeros behind),
  // `pad`: it lies wholly in the k padding
  auto pack4 = [&](const f32x4 &v, bool end, bool pad) {
    f32x4 e;  // (selects on the uniform sh, no branches)
    e[0] = sh == 0 ? v[0] : sh == 1 ? v[1] : sh == 2 ? v[2] : v[3];
    e[1] = sh == 0 ? v[1] : sh == 1 ? v[2] : sh == 2 ? v[3] : 0.0f;
    e[2] = sh == 0 ? v[2] : sh == 1 ? v[3] : 0.0f;
    e[3] = sh == 0 ? v[3] : 0.0f;
    f32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = pad ? 0.0f : end ? e[q] : v[q];
    const bf16x4 b = {(__bf16)o[0], (__bf16)o[1], (__bf16)o[2], (__bf16)o[3]};
    return __builtin_bit_cast(u32x2, b);
  };
  auto pack_plain = [&](const f32x4 &v) {
    const bf16x4 b = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
    return __builtin_bit_cast(u32x2, b);
  };
  auto hold = [&](auto part) {  // the chunk in flight -> held0 / held1
    constexpr bool P1 = decltype(part)::value;
    int tid_s = threadIdx.x;
    asm volatile("" : "+v"(tid_s));
    if constexpr (ROWS) {
      if constexpr (P1) {
#pragma unroll
        for (int r = 0; r < 16 - NX0; ++r) held1[r] = pack_plain(pre[r]);
#pragma unroll
        for (int j = 0; j < NTAIL; ++j) {
          int row, g;
          tail_group(tid_s & 63, j, &row, &g);
          held1[16 - NX0 + j] = pack4(pre[16 - NX0 + j], 4 * g == last_c4, 4 * g > last_c4);
        }
      } else {
#pragma unroll
        for (int r = 0; r < NX0; ++r) held0[r] = pack_plain(pre[r]);
      }
    } else {
      constexpr int CNT = P1 ? NX1 : NX0;
#pragma unroll
      for (int i = 0; i < CNT; ++i) {
        const int idc = min(group_index(tid_s, i, part), VBM * G - 1);
        const int c4 = 4 * (idc - row_of_group(idc) * G);
        const u32x2 v = pack4(pre[i], c4 == last_c4, c4 > last_c4);
        if constexpr (P1) held1[i] = v;
        else held0[i] = v;
      }
    }
  };
  auto stash = [&](auto part) {  // held0 / held1 -> the input region
    constexpr bool P1 = decltype(part)::value;
    int tid_s = threadIdx.x;
    asm volatile("" : "+v"(tid_s));  // keeps the LDS addresses out of registers across the matrix-core loops
    if constexpr (ROWS) {
      const int lane_s = tid_s & 63;
      unsigned char *dst = ldsXB + (size_t)(16 * w) * a.xpitch;
      constexpr int R0 = P1 ? NX0 : 0, NR = P1 ? 16 - NX0 : NX0;
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        u32x2 v;
        if constexpr (P1) v = held1[r];
        else v = held0[r];
        *reinterpret_cast<u32x2 *>(dst + (size_t)(R0 + r) * a.xpitch + lane_s * 8) = v;
      }
      if constexpr (P1) {
#pragma unroll
        for (int j = 0; j < NTAIL; ++j) {
          int row, g;
          tail_group(lane_s, j, &row, &g);
          if (lane_s + 64 * j < 16 * TG) *reinterpret_cast<u32x2 *>(dst + (size_t)row * a.xpitch + g * 8) = held1[NR + j];
        }
      }
    } else {
      constexpr int CNT = P1 ? NX1 : NX0;
#pragma unroll
      for (int i = 0; i < CNT; ++i) {
        const int idx = group_index(tid_s, i, part);
        const int idc = min(idx, VBM * G - 1);
        const int row = row_of_group(idc);
        u32x2 v;
        if constexpr (P1) v = held1[i];
        else v = held0[i];
        if (idx < VBM * G) *reinterpret_cast<u32x2 *>(ldsXB + (size_t)row * a.xpitch + (idc - row * G) * 8) = v;
      }
    }
  };
  auto agent_of_tile = [&](int64_t t) { return (int)(((t * VBM) % a.N) / a.envs_per_agent); };
  // both hidden biases of one agent / the output weights of one agent into LDS (any subset of threads, strided by n)
  auto stage_biases = [&](const Net &net, int i0, int n) {
    for (int i = i0; i < nct * 32; i += n) {
      ldsBias[i] = net.b[0][i];
      ldsBias[nct * 32 + i] = net.b[1][i];
    }
  };
  auto stage_w3 = [&](const Net &net, int i0, int n) {
    for (int i = i0; i < nct * 32; i += n) {
      // output weights of feature 0 out of the packed blocks: k = 16 kb + 8 g + e sits in lane 32 g
      const int kb = i >> 4, gg = (i >> 3) & 1, e = i & 7;
      ldsW3[i] = reinterpret_cast<const __bf16 *>(net.W[2])[((size_t)kb * 64 + 32 * gg) * 8 + e];
    }
  };
  // Layer 2's epilogue with the output layer folded in: partial sums of this wavefront's 64 features, per row.
  // Layer 2's epilogue with the output layer folded in (the accumulators started from the bias): partial sums of
  // this wavefront's 64 features, per row.  Overwrites acc.
  auto epilogue_out_dot = [&](f32x16 (&acc)[CTH][NBT]) {
    int lane_e = threadIdx.x & 63;
    asm volatile("" : "+v"(lane_e));
    const int ge = lane_e >> 5;
    float part[NBT][4];  // (one running sum per batch tile and feature group: four-deep dependent chains only)
#pragma unroll
    for (int q = 0; q < NBT; ++q)
#pragma unroll
      for (int j = 0; j < 4; ++j) part[q][j] = 0.0f;
#pragma unroll
    for (int c = 0; c < CTH; ++c) {
      tanh_in_place<NBT>(acc[c]);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int f0 = (ct0 + c) * 32 + 8 * j + 4 * ge;
        const u32x2 wv = *reinterpret_cast<const u32x2 *>(ldsW3 + f0);  // four bf16 weights
        const uint32_t wlo = wv[0], whi = wv[1];  // (scalars first: a bit cast straight from a vector element reads element 0)
        const bf16x2 w01 = __builtin_bit_cast(bf16x2, wlo), w23 = __builtin_bit_cast(bf16x2, whi);
#pragma unroll
        for (int q = 0; q < NBT; ++q) {
          // activations rounded to bf16 as the hidden tile would hold them; products summed in fp32
          const bf16x2 h01 = {(__bf16)acc[c][q][4 * j], (__bf16)acc[c][q][4 * j + 1]};
          const bf16x2 h23 = {(__bf16)acc[c][q][4 * j + 2], (__bf16)acc[c][q][4 * j + 3]};
          part[q][j] = __builtin_amdgcn_fdot2_f32_bf16(h01, w01, part[q][j], false);
          part[q][j] = __builtin_amdgcn_fdot2_f32_bf16(h23, w23, part[q][j], false);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < NBT; ++q)
      ldsPart[(2 * w + ge) * VBM + q * 32 + (lane_e & 31)] = (part[q][0] + part[q][1]) + (part[q][2] + part[q][3]);
  };

  // ---- set-up: first input tile, first agent's vectors, first weight blocks
  const int64_t t_first = blockIdx.x;
  if (t_first >= ntiles) return;
  fetch(t_first, std::false_type{});
  {
    const Net net0 = net_of(a.net, agent_of_tile(t_first));
    stage_biases(net0, tid, NT);
    stage_w3(net0, tid, NT);
  }
  hold(std::false_type{});
  fetch(t_first, std::true_type{});
  stash(std::false_type{});
  hold(std::true_type{});
  stash(std::true_type{});
  // which tile a chunk-1 request of step (e) is for: the next one (group A), the one after it (group B); past the
  // end it re-reads the last tile (never used)
  auto tile_for_e = [&](int64_t t) {
    const int64_t want = t + (grpB ? 2 : 1) * (int64_t)gridDim.x;
    return want < ntiles ? want : ntiles - 1;
  };
  if (grpB) {
    // group B's chunk 1 of the second tile (its step (e) of a tile before the first)
    fetch(tile_for_e(t_first - gridDim.x), std::true_type{});
    hold(std::true_type{});
  }
  auto wptr = [&](int layer, int ag) {
    return reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(a.net.W[layer]) + (size_t)ag * a.net.w_stride[layer]);
  };
  const int nkb1 = a.net.nkb[0];
  u32x4 ring[PD][CTH];
  prime<CTH, PD>(ring, wptr(0, agent_of_tile(t_first)), nkb1, nct, ct0, lane);
  int agent_b = agent_of_tile(t_first), agent_w3 = agent_b;  // whose vectors sit in LDS
  float b3_prev = 0.0f;
  // hidden halves as this wavefront sees them: its own group's (written by its epilogue 1, first half of its
  // layer 2) and the other group's (second half of its layer 2); k-blocks of layer 2 in the same order
  unsigned char *const ldsOwn = grpB ? ldsXB : ldsHA;
  const unsigned char *const ldsOther = grpB ? ldsHA : ldsXB;
  const int kb_own = grpB ? NKBH : 0, kb_other = grpB ? 0 : NKBH;
  __syncthreads();
  // Both groups run the same five steps per tile -- (a) layer 1, (b) epilogue 1, (c) layer 2 over the own half,
  // (d) layer 2 over the other half, (e) epilogue 2 + output dot -- with a workgroup barrier after each; group B
  // starts one barrier late, which puts it one step behind group A for the whole launch (the table above).
  // Matrix steps run at raised wavefront priority: a matrix instruction occupies the pipe for 32 cycles, so the
  // epilogue wavefront of the SIMD loses one issue slot in eight, while without it the older wavefront of a SIMD
  // wins every arbitration and a younger matrix wavefront starves behind an older epilogue wavefront.
  if (grpB) __syncthreads();

  for (int64_t t = t_first; t < ntiles; t += gridDim.x) {
    const int64_t tn = t + gridDim.x;
    const int64_t tf = tn < ntiles ? tn : t;  // tile fetched during this one (the last one re-reads itself)
    const int agent = agent_of_tile(t);
    const int agent_n = tn < ntiles ? agent_of_tile(tn) : agent;
    const u32x4 *W1 = wptr(0, agent), *W2 = wptr(1, agent);
    f32x16 acc[CTH][NBT];

    // ---- (a) layer 1, accumulators start from b1.  [A: phase 1, B: phase 2]
    __builtin_amdgcn_s_setprio(kMatrixPrio);
    {
      int lane_1 = lane;
      asm volatile("" : "+v"(lane_1));
      bias_acc<CTH, NBT>(acc, ldsBias, ct0, lane_1);
      if (NKB1 > 0) {
        mma_range_static<true, CTH, NBT, PD, (NKB1 > 0 ? NKB1 : PD)>(acc, ring, ldsXB, a.xpitch, W1, nct, 0, W2, nct,
                                                                    kb_own, ct0, 0, lane_1);
      } else {
        mma_layer<true, CTH, NBT, PD>(acc, ring, ldsXB, a.xpitch, nkb1, W1, nct, ct0, 0, lane_1);
        prime<CTH, PD>(ring, W2 + (size_t)kb_own * nct * 64, NKBH, nct, ct0, lane_1);
      }
    }
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();

    // ---- (b) epilogue 1 -> own hidden half; first chunk of the next rows.
    //      [A: phase 2, B: phase 3: every wavefront is done with the input tile]
    fetch(tf, std::false_type{});  // chunk 0 of the next tile
    if (!grpB) {
      if (t != t_first) {
        // the previous tile's values: group B delivered its partial sums in phase 1
        int tid_y = threadIdx.x;
        asm volatile("" : "+v"(tid_y));
        if (tid_y < VBM) {
          float y = b3_prev;
#pragma unroll
          for (int p = 0; p < 2 * NW; ++p) y += ldsPart[p * VBM + tid_y];
          __builtin_nontemporal_store(y, &a.Y[(t - gridDim.x) * VBM + tid_y]);
        }
      }
      // output weights of this tile's agent: last read (previous tile, group B) in phase 1, next in phase 5
      if (agent != agent_w3) stage_w3(net_of(a.net, agent), tid, NT / 2);
    }
    agent_w3 = agent;
    {
      int lane_2 = lane;
      asm volatile("" : "+v"(lane_2));
      // (column f of a row-major half sits at byte 2 (f - first feature of the half))
      epilogue_hidden_biased<CTH, NBT>(acc, ldsOwn - (size_t)kb_own * 32, VHPITCH, ct0, 0, lane_2);
    }
    hold(std::false_type{});
    __syncthreads();

    // ---- (c) layer 2 over the own half, accumulators start from b2.  [A: phase 3, B: phase 4]
    __builtin_amdgcn_s_setprio(kMatrixPrio);
    {
      int lane_3 = lane;
      asm volatile("" : "+v"(lane_3));
      bias_acc<CTH, NBT>(acc, ldsBias + nct * 32, ct0, lane_3);
      mma_range_static<true, CTH, NBT, PD, NKBH>(acc, ring, ldsOwn, VHPITCH, W2, nct, kb_own, W2, nct, kb_other, ct0, 0,
                                                 lane_3);
    }
    __syncthreads();

    // ---- (d) layer 2 over the other half.  [A: phase 4; B: phase 5 -- the input region is free: B writes its
    //      rows, both chunks].  No weight blocks of the next tile yet.
    if (grpB) {
      stash(std::false_type{});
      stash(std::true_type{});
    }
    {
      int lane_4 = lane;
      asm volatile("" : "+v"(lane_4));
      mma_range_static<true, CTH, NBT, PD, NKBH, false>(acc, ring, ldsOther, VHPITCH, W2, nct, kb_other, W2, nct, 0, ct0,
                                                        0, lane_4);
    }
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();

    // ---- (e) epilogue 2 + output dot.  [A: phase 5 -- writes its rows of the next input tile; B: phase 1 of the
    //      next tile]
    if (!grpB) {
      stash(std::false_type{});
      // hidden biases of the next tile's agent: last read in phase 4 (group B), next in phase 1
      if (agent_n != agent_b) stage_biases(net_of(a.net, agent_n), tid, NT / 2);
    }
    agent_b = agent_n;
    fetch(tile_for_e(t), std::true_type{});
    epilogue_out_dot(acc);
    hold(std::true_type{});
    if (!grpB) stash(std::true_type{});
    {
      int lane_5 = lane;
      asm volatile("" : "+v"(lane_5));
      prime<CTH, PD>(ring, wptr(0, agent_n), nkb1, nct, ct0, lane_5);  // in flight across the barrier
    }
    b3_prev = a.net.b[2][(size_t)agent * a.net.b_stride[2]];
    __syncthreads();
  }
  // drain: group A waits out group B's last step, then writes the last tile's values
  if (!grpB) {
    __syncthreads();
    int tid_y = threadIdx.x;
    asm volatile("" : "+v"(tid_y));
    if (tid_y < VBM) {
      // (the last tile this workgroup took)
      const int64_t t_last = t_first + (ntiles - 1 - t_first) / gridDim.x * gridDim.x;
      float y = b3_prev;
#pragma unroll
      for (int p = 0; p < 2 * NW; ++p) y += ldsPart[p * VBM + tid_y];
      __builtin_nontemporal_store(y, &a.Y[t_last * VBM + tid_y]);
    }
  }
}

// ------------------------------------------------------------- weight packing
__global__ void pack_layer_kernel(const float *__restrict__ W, const float *__restrict__ b, int P, int in_dim,
                                  int out_dim, int bf16, int k_rot, int nkb, int nct, void *__restrict__ Wp,
                                  float *__restrict__ bp) {
  const size_t per_agent = (size_t)nct * nkb * 64;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < per_agent * P) {
    const int agent = (int)(i / per_agent);
    const size_t j = i - (size_t)agent * per_agent;
    const int lane = (int)(j & 63);
    const int ct = (int)((j >> 6) % nct);
    const int kb = (int)((j >> 6) / nct);
    const int col = ct * 32 + (lane & 31), g = lane >> 5;
    const float *Wa = W + (size_t)agent * in_dim * out_dim;
    if (bf16) {
      __bf16 v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int k = kb * 16 + 8 * g + e;
        const int ks = k < k_rot ? in_dim - k_rot + k : k - k_rot;
        v[e] = (__bf16)((k < in_dim && col < out_dim) ? Wa[(size_t)ks * out_dim + col] : 0.0f);
      }
      __bf16 *dst = reinterpret_cast<__bf16 *>(Wp) + i * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e] = v[e];
    } else {
      float *dst = reinterpret_cast<float *>(Wp) + i * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = kb * 8 + 4 * g + e;
        const int ks = k < k_rot ? in_dim - k_rot + k : k - k_rot;
        dst[e] = (k < in_dim && col < out_dim) ? Wa[(size_t)ks * out_dim + col] : 0.0f;
      }
    }
  }
  const size_t nb = (size_t)P * nct * 32;
  if (i < nb) {
    const int agent = (int)(i / (nct * 32));
    const int col = (int)(i % (nct * 32));
    bp[i] = col < out_dim ? b[(size_t)agent * out_dim + col] : 0.0f;
  }
}

int kblock(int bf16) { return bf16 ? 16 : 8; }

struct Shape {
  int cth, cto;  // column tiles per wavefront, hidden / output layers
};

bool pick_shape(int Hd, int O, int bf16, Shape *s) {
  if (Hd < 32 || Hd % 32 != 0 || O < 1) return false;
  const int nh = Hd / 32, no = (O + 31) / 32;
  const int need_h = (nh + kWaves - 1) / kWaves, need_o = (no + kWaves - 1) / kWaves;
  int cth = need_h <= 1 ? 1 : need_h <= 2 ? 2 : need_h <= 4 ? 4 : need_h <= 8 ? 8 : 0;
  int cto = need_o <= 1 ? 1 : need_o <= 4 ? 4 : 0;
  if (!cth || !cto) return false;
  if (!bf16 && cth > 4) return false;       // fp32 hidden tile of 1024 columns exceeds LDS
  if (cto == 4 && cth < 4) return false;    // wide outputs only with wide hidden layers
  s->cth = cth;
  s->cto = cto;
  return true;
}

}  // namespace

int64_t split_scratch_rows(int64_t n_envs, int hidden) {
  return (hidden >= 128 && n_envs >= 64 && (n_envs + 63) / 64 * 2 <= 256) ? n_envs : 0;
}

bool mlp_supported(int S, int Hd, int O, int bf16) {
  Shape s;
  return S >= 1 && pick_shape(Hd, O, bf16, &s);
}

int padded_out(int out_dim) { return (out_dim + 31) / 32 * 32; }

size_t packed_weight_bytes(int in_dim, int out_dim, int bf16) {
  const int KB = kblock(bf16);
  const size_t nkb = (in_dim + KB - 1) / KB, nct = (out_dim + 31) / 32;
  return nkb * nct * 64 * 16;
}

hipError_t launch_pack_layer(hipStream_t st, const float *W, const float *b, int P, int in_dim, int out_dim, int bf16,
                             int k_rot, void *Wp, float *bp) {
  const int KB = kblock(bf16);
  const int nkb = (in_dim + KB - 1) / KB, nct = (out_dim + 31) / 32;
  const size_t n = (size_t)P * nct * nkb * 64;
  const size_t nb = (size_t)P * nct * 32;
  const size_t total = n > nb ? n : nb;
  hipLaunchKernelGGL(pack_layer_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, W, b, P, in_dim,
                     out_dim, bf16, k_rot, nkb, nct, Wp, bp);
  return hipGetLastError();
}

template <bool BF16, int CTH, int CTO, int TAG, int RT = 2>
static hipError_t launch_tagged(hipStream_t st, const MlpArgs &a, unsigned blocks, size_t lds) {
  constexpr auto kern = mlp3_kernel<BF16, RT, CTH, CTO, TAG>;
  const hipError_t e = allow_full_lds<kern>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds, st, a);
  return hipGetLastError();
}

template <bool BF16, int CTH, int CTO>
static hipError_t launch_one(hipStream_t st, const MlpArgs &a, unsigned blocks, size_t lds) {
  return a.rows > a.N ? launch_tagged<BF16, CTH, CTO, 1>(st, a, blocks, lds)
                      : launch_tagged<BF16, CTH, CTO, 0>(st, a, blocks, lds);
}


template <bool BF16, int NW, int CTH, int NKB1, int NKB2, int TAG>
static hipError_t launch_tiles_tagged(hipStream_t st, const TileArgs &a, unsigned blocks, size_t lds) {
  constexpr auto kern = mlp_tiles_kernel<BF16, NW, CTH, NKB1, NKB2, TAG>;
  const hipError_t e = allow_full_lds<kern>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(NW * 64), lds, st, a);
  return hipGetLastError();
}

template <bool BF16, int NW, int CTH, int NKB1 = 0, int NKB2 = 0>
static hipError_t launch_tiles(hipStream_t st, const TileArgs &a, unsigned blocks, size_t lds) {
  return a.rows > a.N ? launch_tiles_tagged<BF16, NW, CTH, NKB1, NKB2, 1>(st, a, blocks, lds)
                      : launch_tiles_tagged<BF16, NW, CTH, NKB1, NKB2, 0>(st, a, blocks, lds);
}

int compute_units() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      n = prop.multiProcessorCount;
    if (n <= 0) n = 256;
  }
  return n;
}

// The whole-tile kernel covers dense rows, one output feature tile, hidden widths up to 512 and S up to 320.
// `rows` must be a multiple of 64.
static bool try_launch_tiles(hipStream_t st, const PackedNet &net, int64_t rows, int64_t row_base, const float *X,
                             int64_t ldx, float *Y, int32_t N, int32_t envs_per_agent, hipError_t *err) {
  const int S = net.in_dim[0], Hd = net.out_dim[0];
  // (S >= 5: at least two 16-byte groups per row, the reciprocal of one group does not fit the 32-bit magic)
  if (ldx != S || S < 5 || (reinterpret_cast<uintptr_t>(X) & 3u) || net.nct[2] != 1 || Hd > 512) return false;
  const int G = (S + 3) / 4;
  // eight wavefronts when every one of them gets at least one feature tile
  const int nct = net.nct[0];
  const int NW = nct >= 8 ? 8 : 4;
  const int cth = (nct + NW - 1) / NW;
  if ((tile::BM * G + NW * 64 - 1) / (NW * 64) > XPRE_MAX) return false;
  const int esz = net.bf16 ? 2 : 4, KB = kblock(net.bf16);
  TileArgs a;
  a.X = X;
  a.rows = rows;
  a.row_base = row_base;
  a.Y = Y;
  a.net = net;
  a.N = N;
  a.envs_per_agent = envs_per_agent;
  a.S = S;
  a.groups = G;
  a.g_magic = (int32_t)(uint32_t)((0x100000000ull + (uint64_t)G - 1) / (uint64_t)G);
  a.xpitch = tile::tile_pitch(net.nkb[0] * KB, esz);
  a.hpitch = tile::tile_pitch(Hd, esz);
  const size_t lds = (size_t)tile::BM * (a.xpitch + a.hpitch) + (size_t)net.nkb[2] * 1024 +
                     (size_t)(net.nct[0] + net.nct[1] + net.nct[2]) * 32 * 4;
  if (lds > 160 * 1024) return false;
  const int64_t ntiles = rows / tile::BM;
  const unsigned blocks = (unsigned)(ntiles < compute_units() ? ntiles : compute_units());
  const bool bf = net.bf16 != 0;
  // shapes of the named workloads get straight-line k loops (S = 301: 19 bf16 / 38 fp32 k-blocks)
  if (bf && NW == 8 && cth == 2 && net.nkb[0] == 19 && net.nkb[1] == 32) *err = launch_tiles<true, 8, 2, 19, 32>(st, a, blocks, lds);
  else if (!bf && NW == 8 && cth == 1 && net.nkb[0] == 38 && net.nkb[1] == 32) *err = launch_tiles<false, 8, 1, 38, 32>(st, a, blocks, lds);
  else if (NW == 8 && cth == 2) *err = bf ? launch_tiles<true, 8, 2>(st, a, blocks, lds) : launch_tiles<false, 8, 2>(st, a, blocks, lds);
  else if (NW == 8 && cth == 1) *err = bf ? launch_tiles<true, 8, 1>(st, a, blocks, lds) : launch_tiles<false, 8, 1>(st, a, blocks, lds);
  else if (NW == 4 && cth == 1) *err = bf ? launch_tiles<true, 4, 1>(st, a, blocks, lds) : launch_tiles<false, 4, 1>(st, a, blocks, lds);
  else if (NW == 4 && cth == 2) *err = bf ? launch_tiles<true, 4, 2>(st, a, blocks, lds) : launch_tiles<false, 4, 2>(st, a, blocks, lds);
  else return false;
  return true;
}


template <int NKB1, int SS>
static hipError_t launch_value(hipStream_t st, const ValueArgs &a, unsigned blocks, size_t lds) {
  constexpr auto kern = value_kernel<NKB1, SS>;
  const hipError_t e = allow_full_lds<kern>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), lds, st, a);
  return hipGetLastError();
}

// The value kernel covers a bf16 critic with 512 hidden units on dense rows of at most 304 columns, when
// there are enough rows to give every compute unit several tiles and agents own multiples of 128 envs.
// `rows` must be a multiple of 128 and X must start at a multiple of N rows of the caller's buffer.
static bool try_launch_value(hipStream_t st, const PackedNet &net, int64_t rows, const float *X, int64_t ldx,
                             float *Y, int32_t N, int32_t envs_per_agent, hipError_t *err) {
  const int S = net.in_dim[0], Hd = net.out_dim[0];
  if (!net.bf16 || net.out_dim[2] != 1 || Hd != 2 * VHALF || net.out_dim[1] != Hd || ldx != S || S < 4) return false;
  if ((reinterpret_cast<uintptr_t>(X) & 3u) || N % VBM != 0 || envs_per_agent % VBM != 0) return false;
  if (net.nkb[0] > VPRE_MAX || net.nkb[0] < 4 || rows < (int64_t)VBM * 4 * compute_units()) return false;
  ValueArgs a;
  a.X = X;
  a.rows = rows;
  a.Y = Y;
  a.net = net;
  a.N = N;
  a.envs_per_agent = envs_per_agent;
  a.S = S;
  a.groups = net.nkb[0] * 4;
  a.g_magic = (uint32_t)((0x100000000ull + (uint64_t)a.groups - 1) / (uint64_t)a.groups);
  a.xpitch = tile::tile_pitch(net.nkb[0] * 16, 2);
  // LDS: hidden half A | input tile or hidden half B | b1, b2 | output weights | partial sums
  size_t off = (size_t)VBM * VHPITCH;
  a.off_xb = (int32_t)off;
  off += (size_t)VBM * (a.xpitch > VHPITCH ? a.xpitch : VHPITCH);
  a.off_bias = (int32_t)off;
  off += (size_t)2 * Hd * 4;
  a.off_w3 = (int32_t)off;
  off += (size_t)Hd * 2;
  a.off_part = (int32_t)off;
  off += (size_t)16 * VBM * 4;
  const size_t lds = off;
  if (lds > (size_t)kMaxLdsBytes) return false;
  const int64_t ntiles = rows / VBM;
  const unsigned blocks = (unsigned)(ntiles < compute_units() ? ntiles : compute_units());
  // the observation width of the named workloads gets compile-time index arithmetic and k loops
  if (S == 301) *err = launch_value<19, 301>(st, a, blocks, lds);
  else *err = launch_value<0, 0>(st, a, blocks, lds);
  return true;
}

template <int CTH, bool WIDE_OUT, int CC>
static hipError_t launch_wide(hipStream_t st, const WideArgs &a, unsigned blocks, size_t lds) {
  constexpr auto kern = mlp_wide_kernel<8, CTH, WIDE_OUT, CC>;
  const hipError_t e = allow_full_lds<kern>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(512), lds, st, a);
  return hipGetLastError();
}

// The wide-input kernel covers bf16 networks with 512 or 1024 hidden units whatever the input width, with one
// output feature tile (weights in LDS) or several (streamed); any row stride, any number of rows.
static bool try_launch_wide(hipStream_t st, const PackedNet &net, int64_t rows, int64_t row_base, const float *X,
                            int64_t ldx, float *Y, int32_t N, int32_t envs_per_agent, hipError_t *err) {
  const int Hd = net.out_dim[0];
  if (!net.bf16 || (Hd != 512 && Hd != 1024) || net.out_dim[1] != Hd || (reinterpret_cast<uintptr_t>(X) & 3u)) return false;
  if (net.nct[2] > 32) return false;
  if (envs_per_agent < N && envs_per_agent % tile::BM != 0) return false;  // a tile must not straddle two agents
  // measured: with 512 hidden units and at most a tile or two per compute unit the chunk-staged kernel below is
  // as fast or faster (its four-wavefront workgroups start sooner); long buffers and 1024 hidden units win here
  if (Hd == 512 && rows < (int64_t)4 * tile::BM * compute_units()) return false;
  const bool wide_out = net.nct[2] > 1;
  const int cc = Hd == 512 ? 128 : 64;
  WideArgs a;
  a.X = X, a.ldx = ldx, a.rows = rows, a.row_base = row_base, a.Y = Y, a.net = net, a.N = N;
  a.envs_per_agent = envs_per_agent, a.S = net.in_dim[0];
  a.cpitch = tile::tile_pitch(cc, 2);
  a.hpitch = tile::tile_pitch(Hd, 2);
  const size_t lds = (size_t)tile::BM * a.hpitch + 2 * (size_t)tile::BM * a.cpitch +
                     (wide_out ? 0 : (size_t)net.nkb[2] * 1024) +
                     (size_t)(net.nct[0] + net.nct[1] + net.nct[2]) * 32 * 4;
  if (lds > 160 * 1024) return false;
  const int64_t ntiles = (rows + tile::BM - 1) / tile::BM;
  const unsigned blocks = (unsigned)(ntiles < compute_units() ? ntiles : compute_units());
  if (Hd == 512)
    *err = wide_out ? launch_wide<2, true, 128>(st, a, blocks, lds) : launch_wide<2, false, 128>(st, a, blocks, lds);
  else
    *err = wide_out ? launch_wide<4, true, 64>(st, a, blocks, lds) : launch_wide<4, false, 64>(st, a, blocks, lds);
  return true;
}

// Few rows: one launch per layer (see dense_layer_kernel).  Needs the scratch of the packed network (two fp32
// activation buffers of split_rows x hidden).
static bool try_launch_split(hipStream_t st, const PackedNet &net, int64_t rows, const float *X, int64_t ldx, float *Y,
                             int32_t N, int32_t envs_per_agent, hipError_t *err) {
  const int Hd = net.out_dim[0];
  if (!net.split_h[0] || !net.split_h[1] || rows > net.split_rows || rows < 64 || Hd < 128) return false;
  if ((rows + 63) / 64 * 2 > compute_units()) return false;  // enough tiles for the whole-network kernels
  if (envs_per_agent < N && envs_per_agent % 32 != 0) return false;  // a row tile never spans two agents
  const int64_t tiles = (rows + 31) / 32;
  const int esz = net.bf16 ? 2 : 4, KB = kblock(net.bf16);
  const float *in = X;
  int64_t ld_in = ldx;
  for (int l = 0; l < 3; ++l) {
    LayerArgs a;
    a.X = in, a.ldx = ld_in, a.rows = rows, a.row_offset = 0;
    a.Y = l == 2 ? Y : net.split_h[l];
    a.ldy = l == 2 ? net.out_dim[2] : Hd;
    a.W = net.W[l], a.b = net.b[l], a.w_stride = net.w_stride[l], a.b_stride = net.b_stride[l];
    a.in_dim = net.in_dim[l], a.out_dim = net.out_dim[l], a.nkb = net.nkb[l], a.nct = net.nct[l];
    a.act = l < 2 ? 1 : (net.out_tanh ? 2 : 0);
    a.N = N, a.envs_per_agent = envs_per_agent;
    a.xpitch = kSplitPD * KB * esz + 16;
    const size_t lds = 2 * (size_t)32 * a.xpitch;
    const dim3 grid((unsigned)tiles, (unsigned)((net.nct[l] + kWaves - 1) / kWaves));
    if (net.bf16) {
      *err = allow_full_lds<dense_layer_kernel<true, 1, kSplitPD>>();
      if (*err != hipSuccess) return true;
      hipLaunchKernelGGL((dense_layer_kernel<true, 1, kSplitPD>), grid, dim3(kThreads), lds, st, a);
    } else {
      *err = allow_full_lds<dense_layer_kernel<false, 1, kSplitPD>>();
      if (*err != hipSuccess) return true;
      hipLaunchKernelGGL((dense_layer_kernel<false, 1, kSplitPD>), grid, dim3(kThreads), lds, st, a);
    }
    *err = hipGetLastError();
    if (*err != hipSuccess) return true;
    in = net.split_h[l < 2 ? l : 0];
    ld_in = Hd;
  }
  return true;
}

hipError_t launch_mlp(hipStream_t st, const PackedNet &net, int64_t rows, const float *X, int64_t ldx, float *Y,
                      int32_t N, int32_t envs_per_agent) {
  {
    hipError_t terr = hipSuccess;
    if (try_launch_split(st, net, rows, X, ldx, Y, N, envs_per_agent, &terr)) return terr;
  }
  Shape s;
  if (!pick_shape(net.out_dim[0], net.out_dim[2], net.bf16, &s)) return hipErrorInvalidValue;
  constexpr int BM = 64;
  int64_t row_offset = 0;
  if (rows >= VBM) {
    // a long value-head buffer: 128-row tiles first
    hipError_t terr = hipSuccess;
    const int64_t full = rows / VBM * VBM;
    if (try_launch_value(st, net, full, X, ldx, Y, N, envs_per_agent, &terr)) {
      if (terr != hipSuccess || full == rows) return terr;
      X += full * ldx;
      Y += full * net.out_dim[2];
      row_offset = full;
      rows -= full;
    }
  }
  if (rows >= BM) {
    // full tiles through the persistent whole-tile kernel when it covers the shape; the ragged tail below
    hipError_t terr = hipSuccess;
    const int64_t full = rows / BM * BM;
    if (try_launch_tiles(st, net, full, row_offset, X, ldx, Y, N, envs_per_agent, &terr)) {
      if (terr != hipSuccess || full == rows) return terr;
      X += full * ldx;
      Y += full * net.out_dim[2];
      row_offset += full;
      rows -= full;
    }
  }
  if (rows > 0) {
    // wide inputs or outputs: the chunked whole-tile kernel, ragged tail included
    hipError_t terr = hipSuccess;
    if (try_launch_wide(st, net, rows, row_offset, X, ldx, Y, N, envs_per_agent, &terr)) return terr;
  }
  const int esz = net.bf16 ? 2 : 4, KB = kblock(net.bf16);
  const int pd = s.cth >= 8 ? 2 : 4;
  MlpArgs a;
  a.X = X;
  a.ldx = ldx;
  a.rows = rows;
  a.Y = Y;
  a.net = net;
  a.N = N;
  a.envs_per_agent = envs_per_agent;
  a.row_offset = row_offset;
  a.xpitch = pd * KB * esz + 16;
  a.hpitch = net.out_dim[0] * esz + 16;
  const size_t lds = (size_t)BM * a.hpitch + 2 * (size_t)BM * a.xpitch;
  if (lds > 160 * 1024) return hipErrorInvalidValue;
  const unsigned blocks = (unsigned)((rows + BM - 1) / BM);
  // fp32 networks on fewer 64-row tiles than compute units (4096 envs per step): 32-row tiles put twice as many
  // compute units to work, and the fp32 matrix time per tile halves
  if (!net.bf16 && s.cto == 1 && rows > 32 && (rows + BM - 1) / BM < compute_units()) {
    const unsigned blocks32 = (unsigned)((rows + 31) / 32);
    if (s.cth == 1) return launch_tagged<false, 1, 1, 0, 1>(st, a, blocks32, lds);
    if (s.cth == 2) return launch_tagged<false, 2, 1, 0, 1>(st, a, blocks32, lds);
    if (s.cth == 4) return launch_tagged<false, 4, 1, 0, 1>(st, a, blocks32, lds);
  }
#define POD_CASE(B, H, O_) \
  if ((net.bf16 != 0) == B && s.cth == H && s.cto == O_) return launch_one<B, H, O_>(st, a, blocks, lds);
  POD_CASE(true, 1, 1)
  POD_CASE(true, 2, 1)
  POD_CASE(true, 4, 1)
  POD_CASE(true, 4, 4)
  POD_CASE(true, 8, 1)
  POD_CASE(true, 8, 4)
  POD_CASE(false, 1, 1)
  POD_CASE(false, 2, 1)
  POD_CASE(false, 4, 1)
  POD_CASE(false, 4, 4)
#undef POD_CASE
  return hipErrorInvalidValue;
}

}  // namespace pod
