// Matrix-core building blocks for one 64-row batch tile of the 3-layer
// perceptron (actor / critic networks, Sec. 4.1 and 4.2 of the paper), shared
// by the batched forward kernel and the persistent rollout kernel.
//
// Formulation.  Every layer is computed transposed, C^T = W^T * A^T: the packed
// weights are the MFMA "A" operand (32 output features x k-block) and the
// activation tile in LDS is the "B" operand (k-block x 32 batch rows).  In the
// 32x32 accumulator a lane then owns ONE batch row (l % 32) and, per group
// j = 0..3, FOUR CONSECUTIVE output features 8 j + 4 (l / 32) + {0..3}.  Four
// consecutive features are four consecutive k of the next layer, so the
// epilogue packs them and writes them with a single 8-byte (bf16) or 16-byte
// (fp32) LDS store into the row-major [batch][feature] tile the next layer
// reads its B operand from.
//
// The NW wavefronts of a workgroup split the output features; each streams
// its own weight blocks from global/L2 through a small register ring that is
// primed for the next layer before the current layer's epilogue starts.  With
// NW = 8 two wavefronts share a SIMD, so one's waits on weight loads or its
// epilogue arithmetic overlap with the other's matrix instructions.  The small
// output layer's weights sit in LDS.
#pragma once

#include "pod_internal.h"
#include <type_traits>

namespace pod {
namespace tile {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 64;  // batch rows per tile (two 32-row MFMA tiles)

template <bool BF16>
struct Op;

template <>
struct Op<true> {
  static constexpr int KB = 16;
  static constexpr int ESZ = 2;
  // acc += W_block (features x k) * X_block (k x batch)
  static __device__ inline void mma(const u32x4 &w, const u32x4 &x, f32x16 &c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), c, 0, 0,
                                                0);
  }
  static __device__ inline void store1(unsigned char *p, float v) { *reinterpret_cast<__bf16 *>(p) = (__bf16)v; }
  static __device__ inline void store4(unsigned char *p, float a, float b, float c, float d) {
    bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    *reinterpret_cast<u32x2 *>(p) = __builtin_bit_cast(u32x2, v);
  }
};

template <>
struct Op<false> {
  static constexpr int KB = 8;
  static constexpr int ESZ = 4;
  static __device__ inline void mma(const u32x4 &w, const u32x4 &x, f32x16 &c) {
    const f32x4 wf = __builtin_bit_cast(f32x4, w), xf = __builtin_bit_cast(f32x4, x);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[0], xf[0], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[1], xf[1], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[2], xf[2], c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[3], xf[3], c, 0, 0, 0);
  }
  static __device__ inline void store1(unsigned char *p, float v) { *reinterpret_cast<float *>(p) = v; }
  static __device__ inline void store4(unsigned char *p, float a, float b, float c, float d) {
    f32x4 v = {a, b, c, d};
    *reinterpret_cast<f32x4 *>(p) = v;
  }
};

constexpr float kTwoLog2e = 2.8853900817779268f;

// tanh to a few 1e-7 relative: odd Taylor polynomial below 1/4, 1 - 2/(e^{2|x|}+1) above.
__device__ inline float tanh_accurate(float x) {
  const float ax = fabsf(x);
  const float x2 = x * x;
  float ps = fmaf(x2, 62.0f / 2835.0f, -17.0f / 315.0f);
  ps = fmaf(x2, ps, 2.0f / 15.0f);
  ps = fmaf(x2, ps, -1.0f / 3.0f);
  const float small = fmaf(x2 * x, ps, x);
  const float e = __builtin_amdgcn_exp2f(ax * kTwoLog2e);
  const float big = copysignf(1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f), x);
  return ax < 0.25f ? small : big;
}

// tanh(z) from t = z * 2 log2(e); ~1e-7 absolute, for results that are rounded to bf16.
__device__ inline float tanh_from_scaled(float t) {
  const float e = __builtin_amdgcn_exp2f(t);
  return fmaf(-2.0f, __builtin_amdgcn_rcpf(e + 1.0f), 1.0f);
}

// One agent's packed network (pointers already offset to the agent).
struct Net {
  const u32x4 *W[3];
  const float *b[3];
  int nkb[3], nct[3];
  int out_dim, out_tanh;
};

__device__ inline Net net_of(const PackedNet &p, int agent) {
  Net n;
#pragma unroll
  for (int l = 0; l < 3; ++l) {
    n.W[l] = reinterpret_cast<const u32x4 *>(static_cast<const unsigned char *>(p.W[l]) +
                                             (size_t)agent * p.w_stride[l]);
    n.b[l] = p.b[l] + (size_t)agent * p.b_stride[l];
    n.nkb[l] = p.nkb[l];
    n.nct[l] = p.nct[l];
  }
  n.out_dim = p.out_dim[2];
  n.out_tanh = p.out_tanh;
  return n;
}

// Weight block (feature tile ct, k-block kb) for this lane.  Blocks are stored k-major ([kb][ct][lane]):
// the blocks a workgroup needs for one k-block are one contiguous run, so the requests of a k-step spread
// over all L2 channels instead of piling onto the few channels a power-of-two stride would select.
__device__ inline u32x4 load_w(const u32x4 *W, int nct, int ct, int kb, int lane) {
  return W[((size_t)kb * nct + ct) * 64 + lane];
}

// Fill the ring with k-blocks 0..PD-1 of a layer (feature tiles ct0..ct0+CT-1, clamped to the last tile).
template <int CT, int PD>
__device__ inline void prime(u32x4 (&ring)[PD][CT], const u32x4 *W, int nkb, int nct, int ct0, int lane) {
#pragma unroll
  for (int s = 0; s < PD; ++s)
    if (s < nkb) {
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = load_w(W, nct, min(ct0 + c, nct - 1), s, lane);
    }
}

// acc[c][t] += W(feature tile ct0 + c) * X(batch tile bt0 + t) over all k-blocks.  The activation tile is
// row-major [batch][k] in LDS with `pitch` bytes per row.  The ring must be primed for this layer.
// The main loop has no branches (refills past the end re-read the last block), so the compiler's wait
// counters stay exact and PD k-blocks of weights are really in flight behind the matrix instructions.
template <bool BF16, int CT, int NBT, int PD>
__device__ inline void mma_layer(f32x16 (&acc)[CT][NBT], u32x4 (&ring)[PD][CT], const unsigned char *ldsX, int pitch,
                                 int nkb, const u32x4 *W, int nct, int ct0, int bt0, int lane) {
  using O = Op<BF16>;
  const int brow = lane & 31, g = lane >> 5;
  const unsigned char *xbase = ldsX + (size_t)(bt0 * 32 + brow) * pitch + 16 * g;
  const u32x4 *wp[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) wp[c] = W + (size_t)min(ct0 + c, nct - 1) * 64 + lane;
  int kb0 = 0;
  for (; kb0 + PD <= nkb; kb0 += PD) {
#pragma unroll
    for (int s = 0; s < PD; ++s) {
      const int kb = kb0 + s;
      u32x4 x[NBT];
#pragma unroll
      for (int t = 0; t < NBT; ++t) x[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + kb * 32);
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int t = 0; t < NBT; ++t) O::mma(ring[s][c], x[t], acc[c][t]);
      const int kn = min(kb + PD, nkb - 1);
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = wp[c][(size_t)kn * nct * 64];
      // keep each refill right behind the matrix instructions that freed its slot: left alone, the
      // scheduler sinks all refills to the end of the loop body and the ring is one k-group deep
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const int rem = nkb - kb0;  // < PD blocks left, already in ring[0 .. rem-1]
#pragma unroll
  for (int s = 0; s < PD - 1; ++s) {
    if (s < rem) {
      const int kb = kb0 + s;
      u32x4 x[NBT];
#pragma unroll
      for (int t = 0; t < NBT; ++t) x[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + kb * 32);
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int t = 0; t < NBT; ++t) O::mma(ring[s][c], x[t], acc[c][t]);
    }
  }
}

// k-blocks [kb_lo, kb_hi) of a layer whose activations arrive in chunks: ldsX holds the chunk that starts at k-block
// kb_lo.  kb_lo is a multiple of PD; kb_hi is a multiple of PD or equals nkb.  The ring runs on across the calls
// (primed once for the layer; refills are addressed by the layer-wide k-block index).
template <bool BF16, int CT, int NBT, int PD>
__device__ inline void mma_layer_range(f32x16 (&acc)[CT][NBT], u32x4 (&ring)[PD][CT], const unsigned char *ldsX,
                                       int pitch, int kb_lo, int kb_hi, int nkb, const u32x4 *W, int nct, int ct0,
                                       int bt0, int lane) {
  using O = Op<BF16>;
  const int brow = lane & 31, g = lane >> 5;
  const unsigned char *xbase = ldsX + (size_t)(bt0 * 32 + brow) * pitch + 16 * g;
  const u32x4 *wp[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) wp[c] = W + (size_t)min(ct0 + c, nct - 1) * 64 + lane;
  int kb0 = kb_lo;
  for (; kb0 + PD <= kb_hi; kb0 += PD) {
#pragma unroll
    for (int s = 0; s < PD; ++s) {
      const int kb = kb0 + s;
      u32x4 x[NBT];
#pragma unroll
      for (int t = 0; t < NBT; ++t)
        x[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + (kb - kb_lo) * 32);
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int t = 0; t < NBT; ++t) O::mma(ring[s][c], x[t], acc[c][t]);
      const int kn = min(kb + PD, nkb - 1);
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = wp[c][(size_t)kn * nct * 64];
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const int rem = kb_hi - kb0;  // < PD blocks left (only at the end of the layer), already in ring[0 .. rem-1]
#pragma unroll
  for (int s = 0; s < PD - 1; ++s) {
    if (s < rem) {
      const int kb = kb0 + s;
      u32x4 x[NBT];
#pragma unroll
      for (int t = 0; t < NBT; ++t)
        x[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + (kb - kb_lo) * 32);
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int t = 0; t < NBT; ++t) O::mma(ring[s][c], x[t], acc[c][t]);
    }
  }
}

// The same with the number of k-blocks known at compile time: straight-line code, so every wait on a
// weight load is placed exactly (across a loop back-edge the compiler falls back to waiting for all loads,
// which exposes one L2 round trip per loop iteration).
template <bool BF16, int CT, int NBT, int PD, int NKB>
__device__ inline void mma_layer_static(f32x16 (&acc)[CT][NBT], u32x4 (&ring)[PD][CT], const unsigned char *ldsX,
                                        int pitch, const u32x4 *W, int nct, int ct0, int bt0, int lane) {
  using O = Op<BF16>;
  const int brow = lane & 31, g = lane >> 5;
  const unsigned char *xbase = ldsX + (size_t)(bt0 * 32 + brow) * pitch + 16 * g;
  const u32x4 *wp[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) wp[c] = W + (size_t)min(ct0 + c, nct - 1) * 64 + lane;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    constexpr int dummy = 0;
    (void)dummy;
    const int s = kb % PD;
    u32x4 x[NBT];
#pragma unroll
    for (int t = 0; t < NBT; ++t) x[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + kb * 32);
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
      for (int t = 0; t < NBT; ++t) O::mma(ring[s][c], x[t], acc[c][t]);
    if (kb + PD < NKB) {
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = wp[c][(size_t)(kb + PD) * nct * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// NKB consecutive k-blocks of a layer, straight-line, for callers that walk a layer in pieces or chain layers
// without a stall: LDS column block i of `ldsX` pairs with weight block kbw0 + i of W.  On entry ring slot s must
// hold weight block kbw0 + s (s < PD).  Inside the range a consumed slot is refilled with the block PD ahead; the
// last PD steps refill their slots with blocks kbn0 + (slot) of Wn (nctn feature tiles per k-block): the ring is
// then primed, slot for slot, for a range that starts at block kbn0 of Wn.  NEXT = false: no refills in the last PD
// steps (the ring's registers are free afterwards; the caller primes it again before the next range).
template <bool BF16, int CT, int NBT, int PD, int NKB, bool NEXT = true, bool XAHEAD = false>
__device__ inline void mma_range_static(f32x16 (&acc)[CT][NBT], u32x4 (&ring)[PD][CT], const unsigned char *ldsX,
                                        int pitch, const u32x4 *W, int nct, int kbw0, const u32x4 *Wn, int nctn,
                                        int kbn0, int ct0, int bt0, int lane) {
  using O = Op<BF16>;
  static_assert(NKB >= PD, "a range must be at least as long as the ring");
  const int brow = lane & 31, g = lane >> 5;
  const unsigned char *xbase = ldsX + (size_t)(bt0 * 32 + brow) * pitch + 16 * g;
  const u32x4 *wp[CT], *wn[CT];
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    wp[c] = W + ((size_t)kbw0 * nct + min(ct0 + c, nct - 1)) * 64 + lane;
    wn[c] = Wn + ((size_t)kbn0 * nctn + min(ct0 + c, nctn - 1)) * 64 + lane;
  }
  // XAHEAD: the activation block of step i + 1 is requested before the matrix instructions of step i, for a
  // wavefront that has its SIMD's matrix pipe to itself (nobody else's instructions cover the LDS round trip)
  u32x4 xn[NBT];
  if (XAHEAD) {
#pragma unroll
    for (int t = 0; t < NBT; ++t) xn[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch);
  }
#pragma unroll
  for (int i = 0; i < NKB; ++i) {
    constexpr int dummy = 0;
    (void)dummy;
    const int s = i % PD;
    u32x4 x[NBT];
    if (XAHEAD) {
#pragma unroll
      for (int t = 0; t < NBT; ++t) x[t] = xn[t];
      if (i + 1 < NKB) {
#pragma unroll
        for (int t = 0; t < NBT; ++t)
          xn[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + (i + 1) * 32);
      }
    } else {
#pragma unroll
      for (int t = 0; t < NBT; ++t) x[t] = *reinterpret_cast<const u32x4 *>(xbase + (size_t)t * 32 * pitch + i * 32);
    }
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
      for (int t = 0; t < NBT; ++t) O::mma(ring[s][c], x[t], acc[c][t]);
    if (i + PD < NKB) {
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = wp[c][(size_t)(i + PD) * nct * 64];
    } else if (NEXT) {
#pragma unroll
      for (int c = 0; c < CT; ++c) ring[s][c] = wn[c][(size_t)s * nctn * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <int CT, int NBT>
__device__ inline void zero_acc(f32x16 (&acc)[CT][NBT]) {
#pragma unroll
  for (int c = 0; c < CT; ++c)
#pragma unroll
    for (int t = 0; t < NBT; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[c][t][i] = 0.0f;
}

// acc = bias of the wavefront's features (every batch row alike): a layer started this way needs no bias add in
// its epilogue.  bias: LDS, padded to whole feature tiles.
template <int CT, int NBT>
__device__ inline void bias_acc(f32x16 (&acc)[CT][NBT], const float *bias, int ct0, int lane) {
  const int g = lane >> 5;
#pragma unroll
  for (int c = 0; c < CT; ++c)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias + (ct0 + c) * 32 + 8 * j + 4 * g);
#pragma unroll
      for (int t = 0; t < NBT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[c][t][4 * j + i] = bv[i];
    }
}

// acc <- tanh(acc), in place, one feature tile (all NBT batch tiles of it: 16 NBT values per lane) at a time and
// one operation at a time over all of them: every instruction's operand was produced 16 NBT instructions earlier,
// so a wavefront that has a SIMD's vector unit to itself never waits for a result.  (Written value by value, the
// compiler keeps four chains in flight -- all the registers it has next to live accumulators -- and the
// transcendental latencies are exposed.)  The barriers keep the scheduler from interleaving the stages again.
template <int NBT>
__device__ inline void tanh_in_place(f32x16 (&acc)[NBT]) {
#pragma unroll
  for (int t = 0; t < NBT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] *= kTwoLog2e;
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < NBT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = __builtin_amdgcn_exp2f(acc[t][i]);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < NBT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] += 1.0f;
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < NBT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = __builtin_amdgcn_rcpf(acc[t][i]);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < NBT; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[t][i] = fmaf(-2.0f, acc[t][i], 1.0f);
  __builtin_amdgcn_sched_barrier(0);
}

// hidden = tanh(acc) -> LDS, for bf16 layers whose accumulators started from the bias (bias_acc).  Overwrites acc.
template <int CT, int NBT>
__device__ inline void epilogue_hidden_biased(f32x16 (&acc)[CT][NBT], unsigned char *ldsH, int hpitch, int ct0,
                                              int bt0, int lane) {
  using O = Op<true>;
  const int brow = lane & 31, g = lane >> 5;
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    tanh_in_place<NBT>(acc[c]);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int f0 = (ct0 + c) * 32 + 8 * j + 4 * g;
#pragma unroll
      for (int t = 0; t < NBT; ++t)
        O::store4(ldsH + (size_t)((bt0 + t) * 32 + brow) * hpitch + f0 * O::ESZ, acc[c][t][4 * j], acc[c][t][4 * j + 1],
                  acc[c][t][4 * j + 2], acc[c][t][4 * j + 3]);
    }
  }
}

// hidden = tanh(acc + bias) -> row-major [batch][feature] LDS tile in the operand type.
template <bool BF16, int CT, int NBT>
__device__ inline void epilogue_hidden(const f32x16 (&acc)[CT][NBT], const float *bias, unsigned char *ldsH,
                                       int hpitch, int nct, int ct0, int bt0, int lane) {
  using O = Op<BF16>;
  const int brow = lane & 31, g = lane >> 5;
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    if (ct0 + c < nct) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int f0 = (ct0 + c) * 32 + 8 * j + 4 * g;
        const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias + f0);
#pragma unroll
        for (int t = 0; t < NBT; ++t) {
          float h[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (BF16)
              h[i] = tanh_from_scaled(fmaf(acc[c][t][4 * j + i], kTwoLog2e, bv[i] * kTwoLog2e));
            else
              h[i] = tanh_accurate(acc[c][t][4 * j + i] + bv[i]);
          }
          O::store4(ldsH + (size_t)((bt0 + t) * 32 + brow) * hpitch + f0 * O::ESZ, h[0], h[1], h[2], h[3]);
        }
      }
    }
  }
}

// Bias and activation of the last layer.
__device__ inline float finish_out(float acc, float bias, int out_tanh) {
  const float z = acc + bias;
  return out_tanh ? tanh_accurate(z) : z;
}

// Last layer: y = acc + bias (tanh for the actor) handed to sink(batch_row_in_tile, feature, value).
// RAW: hand over the bare accumulator instead; the caller applies finish_out itself (spread over more lanes
// than the two wavefronts that hold the accumulators).
template <int CT, int NBT, bool RAW, class Sink>
__device__ inline void epilogue_out(const f32x16 (&acc)[CT][NBT], const float *bias, int out_dim, int out_tanh,
                                    int nct, int ct0, int bt0, int lane, Sink sink) {
  const int brow = lane & 31, g = lane >> 5;
#pragma unroll
  for (int c = 0; c < CT; ++c) {
    if (ct0 + c < nct) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int f0 = (ct0 + c) * 32 + 8 * j + 4 * g;
        const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias + f0);
#pragma unroll
        for (int t = 0; t < NBT; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float y = RAW ? acc[c][t][4 * j + i] : finish_out(acc[c][t][4 * j + i], bv[i], out_tanh);
            if (f0 + i < out_dim) sink((bt0 + t) * 32 + brow, f0 + i, y);
          }
      }
    }
  }
}

// Copy one agent's three bias vectors (padded to multiples of 32) into LDS: [b1 | b2 | b3], and, when the
// output layer is a single feature tile, its packed weights (nkb[2] blocks of 1 KiB) into ldsW3.
template <int NT>
__device__ inline void stage_net(const Net &net, float *ldsBias, u32x4 *ldsW3, int tid) {
  int off = 0;
#pragma unroll
  for (int l = 0; l < 3; ++l) {
    const int n = net.nct[l] * 32;
    for (int i = tid; i < n; i += NT) ldsBias[off + i] = net.b[l][i];
    off += n;
  }
  if (ldsW3 && net.nct[2] == 1) {
    // four loads in flight per thread before the first LDS store (a plain copy loop pays one round trip per pass)
    const int n3 = net.nkb[2] * 64;
    for (int base = tid; base < n3; base += 4 * NT) {
      u32x4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = net.W[2][min(base + j * NT, n3 - 1)];
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (base + j * NT < n3) ldsW3[base + j * NT] = v[j];
    }
  }
}

// Output layer with one feature tile: weights from LDS (block kb = 64 lanes x 16 B), activations from ldsH.
// NKB > 0: straight-line code over a compile-time number of k-blocks with two accumulators (even / odd
// k-blocks), which halves the dependent chain of matrix instructions and lets the LDS reads run ahead.
// kb0: first k-block (NKB > 0 only), for callers that split the k range over several wavefronts.
template <bool BF16, int NKB>
__device__ inline void mma_out_lds(f32x16 &acc, const u32x4 *ldsW3, const unsigned char *ldsH, int hpitch, int nkb,
                                   int bt, int lane, int kb0 = 0) {
  using O = Op<BF16>;
  const int brow = lane & 31, g = lane >> 5;
  const unsigned char *xbase = ldsH + (size_t)(bt * 32 + brow) * hpitch + 16 * g + (NKB > 0 ? kb0 * 32 : 0);
  if (NKB > 0) ldsW3 += kb0 * 64;
  if (NKB > 0) {
    f32x16 acc2;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc2[i] = 0.0f;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      const u32x4 wv = ldsW3[kb * 64 + lane];
      const u32x4 xv = *reinterpret_cast<const u32x4 *>(xbase + kb * 32);
      if (kb & 1)
        O::mma(wv, xv, acc2);
      else
        O::mma(wv, xv, acc);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] += acc2[i];
  } else {
    for (int kb = 0; kb < nkb; ++kb) {
      const u32x4 wv = ldsW3[kb * 64 + lane];
      const u32x4 xv = *reinterpret_cast<const u32x4 *>(xbase + kb * 32);
      O::mma(wv, xv, acc);
    }
  }
}

// Layers 1-3 for the 64-row tile whose layer-1 input already sits in ldsX (row-major, xpitch bytes per row,
// padded k columns zero).  ldsH receives the hidden tiles; ldsBias / ldsW3 as filled by stage_net.
// NW wavefronts (4 or 8); CTH = feature tiles per wavefront in the hidden layers; NKB1 / NKB2 = k-blocks
// of layers 1 / 2 when known at compile time (0: read them from `net`).
// WIDE_OUT = false: the output layer has at most 32 features (one feature tile, weights in ldsW3).
// Hooks: early() runs after layer 1's matrix work, before its epilogue -- the place to issue global loads that
// are not needed soon.  late() runs once layer 2's epilogue is complete workgroup-wide; ldsX has been free
// since layer 1 and may be refilled there.
// Ends without a trailing barrier: the caller must synchronise before ldsH or ldsX are read or written again.
constexpr int ring_depth(int cth) { return cth >= 8 ? 2 : 4; }

// PRIMED: the caller has already called prime() for layer 1 on `ring` (to get the first weight blocks in flight
// before the input tile is complete).  RAW_OUT: see epilogue_out.
// KSPLIT > 1 (RAW_OUT, one output feature tile, NKB2 known): the output layer's k range is split over KSPLIT
// wavefronts per batch tile, so that all 2 KSPLIT wavefronts share its matrix work; the sink is then called
// as sink(row, feature, partial_sum, part) and the caller adds the KSPLIT parts.
// Layer1: by default layer 1 reads a whole input tile from ldsX.  A caller whose input rows do not fit in LDS passes
// a functor instead; it is called by EVERY wavefront as layer1(acc, ring, active) (it may contain barriers), must
// leave layer 1's sums of the active wavefronts in acc, and owns the ring while it runs.
struct WholeTileLayer1 {};
// NBT: 32-row batch tiles of the tile (2: the usual 64 rows; 1: a 32-row tile, for shapes whose 64-row tiles do not
// fit in LDS).
template <bool BF16, int NW, int CTH, bool WIDE_OUT, int NKB1, int NKB2, bool PRIMED, bool RAW_OUT, int KSPLIT = 1,
          int NBT = 2, class Early, class Late, class Sink, class Layer1 = WholeTileLayer1>
__device__ inline void mlp_tile(const Net &net, u32x4 (&ring)[ring_depth(CTH)][CTH], const unsigned char *ldsX,
                                int xpitch, unsigned char *ldsH, int hpitch, const float *ldsBias,
                                const u32x4 *ldsW3, int tid, Early early, Late late, Sink sink,
                                Layer1 layer1 = Layer1()) {
  constexpr int PD = ring_depth(CTH);
  // the wavefront index is uniform: tell the compiler, so that block addresses live in scalar registers
  const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ct0 = w * CTH;
  const bool act = ct0 < net.nct[0];
  const float *lb1 = ldsBias, *lb2 = ldsBias + net.nct[0] * 32, *lb3 = lb2 + net.nct[1] * 32;
  {
    f32x16 acc[CTH][NBT];
    zero_acc<CTH, NBT>(acc);
    if constexpr (!std::is_same<Layer1, WholeTileLayer1>::value) {
      layer1(acc, ring, act);
      if (act) prime<CTH, PD>(ring, net.W[1], net.nkb[1], net.nct[1], ct0, lane);
    } else if (act) {
      if (!PRIMED) prime<CTH, PD>(ring, net.W[0], net.nkb[0], net.nct[0], ct0, lane);
      if (NKB1 > 0)
        mma_layer_static<BF16, CTH, NBT, PD, NKB1>(acc, ring, ldsX, xpitch, net.W[0], net.nct[0], ct0, 0, lane);
      else
        mma_layer<BF16, CTH, NBT, PD>(acc, ring, ldsX, xpitch, net.nkb[0], net.W[0], net.nct[0], ct0, 0, lane);
      prime<CTH, PD>(ring, net.W[1], net.nkb[1], net.nct[1], ct0, lane);
    }
    early();
    if (act) epilogue_hidden<BF16, CTH, NBT>(acc, lb1, ldsH, hpitch, net.nct[0], ct0, 0, lane);
    __syncthreads();
    zero_acc<CTH, NBT>(acc);
    if (act) {
      if (NKB2 > 0)
        mma_layer_static<BF16, CTH, NBT, PD, NKB2>(acc, ring, ldsH, hpitch, net.W[1], net.nct[1], ct0, 0, lane);
      else
        mma_layer<BF16, CTH, NBT, PD>(acc, ring, ldsH, hpitch, net.nkb[1], net.W[1], net.nct[1], ct0, 0, lane);
    }
    __syncthreads();  // every wavefront has consumed the layer-1 tile; it is overwritten in place
    if (act) epilogue_hidden<BF16, CTH, NBT>(acc, lb2, ldsH, hpitch, net.nct[1], ct0, 0, lane);
    __syncthreads();
  }
  // output layer: few features.  One feature tile: the first NBT wavefronts take one 32-row batch tile each while
  // the others run late().  More feature tiles: split them over the wavefronts like the hidden layers.
  if constexpr (!WIDE_OUT && KSPLIT > 1) {
    static_assert(KSPLIT == 1 || (RAW_OUT && NKB2 > 0 && NKB2 % (KSPLIT > 0 ? KSPLIT : 1) == 0), "k split of the output layer");
    if (w < NBT * KSPLIT) {
      const int bt = w % NBT, part = w / NBT;
      f32x16 acc[1][1];
      zero_acc<1, 1>(acc);
      mma_out_lds<BF16, NKB2 / KSPLIT>(acc[0][0], ldsW3, ldsH, hpitch, net.nkb[2], bt, lane, part * (NKB2 / KSPLIT));
      epilogue_out<1, 1, true>(acc, lb3, net.out_dim, net.out_tanh, 1, 0, bt, lane,
                               [&](int b, int f, float z) { sink(b, f, z, part); });
    }
    late();
  } else if constexpr (!WIDE_OUT) {
    if (w < NBT) {
      f32x16 acc[1][1];
      zero_acc<1, 1>(acc);
      mma_out_lds<BF16, NKB2>(acc[0][0], ldsW3, ldsH, hpitch, net.nkb[2], w, lane);  // nkb[2] == nkb[1]
      epilogue_out<1, 1, RAW_OUT>(acc, lb3, net.out_dim, net.out_tanh, 1, 0, w, lane, sink);
    }
    late();
  } else {
    late();
    constexpr int CTO = 4;
    const int co0 = w * CTO;
    if (co0 < net.nct[2]) {
      u32x4 r4[2][CTO];
      f32x16 acc[CTO][NBT];
      zero_acc<CTO, NBT>(acc);
      prime<CTO, 2>(r4, net.W[2], net.nkb[2], net.nct[2], co0, lane);
      mma_layer<BF16, CTO, NBT, 2>(acc, r4, ldsH, hpitch, net.nkb[2], net.W[2], net.nct[2], co0, 0, lane);
      epilogue_out<CTO, NBT, RAW_OUT>(acc, lb3, net.out_dim, net.out_tanh, net.nct[2], co0, 0, lane, sink);
    }
  }
}

// Geometry of the LDS tiles.
__host__ __device__ inline int tile_pitch(int k_elems_padded, int esz) { return k_elems_padded * esz + 16; }

}  // namespace tile
}  // namespace pod
