// Persistent rollout kernel: one workgroup keeps a tile of envs (64 with bf16
// networks, 32 with fp32 networks) on its compute unit for all T steps of a
// rollout (the worker of Sec. 4.2: actor x batched environment; stock-trading
// task of Table 1 / Sec. 5.3).
//
// Envs are independent, so no grid-wide synchronisation is needed: each
// workgroup loops   obs_t (LDS) -> actor (matrix cores) -> sample -> trade ->
// reward / done / reset -> obs_{t+1} (LDS + HBM)   on its own.  The env state
// (cash, cursor, episode sums: registers of one "ledger" lane per env; holdings
// and current prices: LDS) never leaves the compute unit during the rollout, and
// the next observation is assembled directly in the LDS tile the actor reads
// its input from.  Per env-step the kernel therefore moves only the bytes the
// method itself needs: noise and the next market row in, observation, raw
// action, reward / done / log-prob out.
//
// For the 301-512-512 bf16 shape the actor runs as two wavefront groups half a
// layer out of step, so that the tanh epilogues of one group execute under the
// matrix instructions of the other, and the first k-blocks of the next step's
// layer 1 run while the ledger of this step is still walking ("split schedule",
// described at the step loop); other shapes run the layers with all wavefronts
// in step.
//
// Trade execution reproduces, operation for operation in binary32, the serial
// rule "all sales in stock order, then all purchases in stock order, each
// limited by the cash left": everything that does not depend on the running
// cash (wanted shares, sale quantities and proceeds, unit costs) is computed
// by all 512 lanes in parallel; one ledger lane per env then walks the cash
// chain in branch-free code, where the latency of the dependent operations on
// the running cash is what bounds the step.
//
// Compiled with floating-point contraction off (integer decisions depend on
// one rounding per operation); the network code uses explicit fmaf.
#include "pod_internal.h"
#include <type_traits>

#include "pod_tile.h"

namespace pod {

namespace {

using namespace tile;

constexpr int NW = 8;
constexpr int NT = NW * 64;
// envs per workgroup: 64 (bf16 networks) or 32 (fp32 networks, whose 64-row tiles do not fit in LDS); a template
// parameter E of the kernel
constexpr int DMAX = 32;         // stock slots per env row in LDS; slots D..31 hold neutral values (k = 0, h = 0)
constexpr int kDp = DMAX + 1;    // odd row pitch: the per-env serial walks of the ledger hit distinct banks
// Lane maps of the parallel env work (no index divisions anywhere in the step loop):
//  * (env, stock) slots: a half-wavefront per env row, lane % 32 = stock slot; wavefront w owns envs
//    [w E/8, (w + 1) E/8), two per pass, E/16 passes;
//  * market rows (prices and indicators of the next observation): one env row per instruction, wavefronts 1..7
//    take rows w - 1, w + 6, ...; lane l carries price l and the 16-byte indicator group l (D K <= 252, D K % 4 == 0).
//    The ledger wavefront carries none: a load of its own in flight would sit in front of whatever its serial
//    pass waits for next (a wavefront's memory operations complete in order).

constexpr int kLagPrio = 2;  // wavefront priority of the lagging group's matrix steps in the split schedule (1..3 measure alike)
constexpr int MUP = 33;         // row pitch of a policy-mean plane (lanes of one store differ in the row: 32 would hit one bank)
// Planes the output layer's k range is split into (one per group of wavefronts), by the compile-time k-block count
// of the kernel instance.
constexpr int mu_planes(int nkb2) { return (nkb2 > 0 && nkb2 % 4 == 0) ? 4 : 1; }

struct Row {
  int32_t row_val;  // market row the portfolio is valued at (cursor + 1)
  int32_t row_obs;  // market row of the next observation (row 0 of the path after an episode end)
  int32_t done;
  int32_t pad;
};

// Byte offsets of the LDS regions, computed once on the host (the launch size, the shape check and the kernel
// all read this one carve-up).  The env scratch arrays alias the hidden tile: they live between the end of the
// output layer and the next step's first epilogue.  The policy-mean planes alias the head of the input region,
// which is dead between layer 1 and the write of the next observation; the region is sized for whichever of the
// two is larger.
struct FusedLayout {
  int32_t xpitch, hpitch;  // bytes per row of the input / hidden tile
  int32_t off_x, off_w3, off_bias, off_h, off_p, off_row, off_cash, off_done;
  int32_t total;
};

struct FusedArgs {
  EnvDims d;
  FusedLayout L;
  EnvState st;
  const float *price, *ind;
  PackedNet actor;
  int32_t envs_per_agent;
  int32_t T;
  const float *noise;      // [T, N, D]
  const float *mu_forced;  // [T, N, D] or null (then the actor runs)
  float *obs;              // [T+1, N, S]
  float *act_raw;          // [T, N, D]
  float *reward;           // [T, N]
  uint8_t *done;           // [T, N]
  float *logp;             // opt [T, N]
  float *mu_out;           // opt [T, N, D]
  int32_t *shares;         // opt [T, N, D]
};

// Ledger input of one (env, stock) slot, written by the parallel lanes.
struct __attribute__((aligned(16))) Slot {
  int32_t k;   // wanted shares, signed
  float val;   // sale proceeds (k < 0) or unit cost of a purchase (k > 0)
  double rcp;  // 1 / unit cost in binary64 (k > 0), else 0
};

__device__ inline Row row_of(const EnvDims &d, int32_t tau, int32_t start, int32_t n) {
  const int32_t m = d.M == 1 ? 0 : n;
  Row r;
  r.row_val = (tau + 1) * d.M + m;
  r.done = (tau + 1 - start == d.H);
  r.row_obs = r.done ? start * d.M + m : r.row_val;
  r.pad = 0;
  return r;
}

template <bool BF16, int E, int CTH, int NKB1, int NKB2, bool ACTOR>
__global__ __launch_bounds__(NT) void rollout_fused_kernel(FusedArgs a) {
  static_assert(E == 64 || E == 32, "one or two 32-row batch tiles");
  constexpr int NBT = E / 32;
  using O = tile::Op<BF16>;
  // the named bf16 shape runs its actor as two wavefront groups half a layer out of step (see the step loop)
  constexpr bool SPLIT = ACTOR && BF16 && E == 64 && CTH == 2 && NKB2 == 32 && NKB1 >= 16;
  constexpr int PDR = SPLIT ? 8 : ring_depth(CTH);  // weight blocks in flight per feature tile
  // Roles of the wavefronts outside the actor.  The ledger wavefront LW walks the cash chains; MW others carry
  // the market rows of the next observation.  In the split schedule these are the four wavefronts of group A,
  // which then also run the first NK1A k-blocks of the next step's layer 1 (indicator columns only, complete
  // once the market rows are written) while the ledger -- a wavefront of group B -- is still walking.
  // (Measured alternatives that were no faster: the three idle wavefronts of group B sharing the market rows;
  // a raised priority for the ledger wavefront.)
  constexpr int LW = SPLIT ? NW / 2 : 0;
  constexpr int MW = SPLIT ? NW / 2 : NW - 1;
  constexpr int NK1A = SPLIT ? NKB1 - 8 : 0;
  extern __shared__ __align__(16) unsigned char lds[];
  const EnvDims &d = a.d;
  const int D = d.D, DK = D * d.K, S = d.S;
  constexpr int Dp = kDp;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n0 = blockIdx.x * E;
  const size_t N = (size_t)d.N;
  const bool is_market = SPLIT ? wave < NW / 2 : wave != 0;
  const int mw = SPLIT ? wave : wave - 1;  // index among the market wavefronts

  // ---- LDS carve-up (see FusedLayout)
  unsigned char *ldsH = lds;
  unsigned char *ldsX = lds + a.L.off_x;
  u32x4 *ldsW3 = reinterpret_cast<u32x4 *>(lds + a.L.off_w3);
  float *ldsBias = reinterpret_cast<float *>(lds + a.L.off_bias);
  int32_t *s_h = reinterpret_cast<int32_t *>(lds + a.L.off_h);
  float *s_p = reinterpret_cast<float *>(lds + a.L.off_p);  // prices the trades execute at
  Row *s_row = reinterpret_cast<Row *>(lds + a.L.off_row);
  float *s_cash = reinterpret_cast<float *>(lds + a.L.off_cash);
  int32_t *s_done = reinterpret_cast<int32_t *>(lds + a.L.off_done);  // episode-end flags of the step just taken
  int32_t *s_sync = s_done + E;  // arrivals of group A's wavefronts at their own meeting point, counted up all rollout
  // scratch in the hidden tile
  Slot *s_slot = reinterpret_cast<Slot *>(ldsH);            // what the ledger needs per (env, stock), one 16-byte read
  int32_t *s_q = reinterpret_cast<int32_t *>(s_slot + E * Dp);  // executed shares, signed
  float *s_pv = reinterpret_cast<float *>(s_q + E * Dp);    // valuation prices
  float *s_e2 = s_pv + E * Dp;                              // squared noise
  // output-layer accumulators of the actor, one [E][32] plane per k part of that layer (summed in the pre-compute)
  constexpr int KS = mu_planes(NKB2);
  float *s_mu = reinterpret_cast<float *>(ldsX);

  // ---- ledger lanes (wavefront LW, see below): per-env scalars in registers for the whole rollout
  float cash = 0.0f;
  int32_t tau = 0, start = 0, ep_cnt = 0;
  double asset = 0.0, ep_ret = 0.0, ep_sum = 0.0, ep_sqsum = 0.0;

  Net net;
  if (ACTOR) {
    net = net_of(a.actor, (n0 % d.N) / a.envs_per_agent);
    stage_net<NT>(net, ldsBias, ldsW3, tid);
    if constexpr (SPLIT) {
      // Output-layer blocks in the k order of an accumulator half: the lane of half g takes, from the standard
      // block's two lanes of its output feature, the four k of each that an accumulator lane of half g holds.
      __syncthreads();
      u32x4 v[NKB2 * 64 / NT];
#pragma unroll
      for (int j = 0; j < NKB2 * 64 / NT; ++j) {
        const int idx = tid + NT * j, blk = idx >> 6, l = idx & 63, o = l & 31, g = l >> 5;
        const uint32_t *lo = reinterpret_cast<const uint32_t *>(ldsW3 + blk * 64 + o);
        const uint32_t *hi = reinterpret_cast<const uint32_t *>(ldsW3 + blk * 64 + 32 + o);
        v[j] = u32x4{lo[2 * g], lo[2 * g + 1], hi[2 * g], hi[2 * g + 1]};
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < NKB2 * 64 / NT; ++j) ldsW3[tid + NT * j] = v[j];
    }
    // padded k columns of the input tile must read as zero
    for (int i = tid; i < E * a.L.xpitch / 4; i += NT) reinterpret_cast<uint32_t *>(ldsX)[i] = 0u;
    if (tid == 0) *s_sync = 0;
  }
  __syncthreads();

  // ---- prologue: load the state, emit observation 0
  if (wave == LW && lane < E) {
    const int n = n0 + lane;
    cash = a.st.cash[n];
    tau = a.st.tau[n];
    start = a.st.start[n];
    ep_ret = a.st.ep_ret[n];
    ep_sum = a.st.ep_sum[n];
    ep_sqsum = a.st.ep_sqsum[n];
    ep_cnt = a.st.ep_cnt[n];
    Row r;  // "next observation" of a virtual step before the rollout = the current cursor
    const int32_t m = d.M == 1 ? 0 : n;
    r.row_val = tau * d.M + m;
    r.row_obs = r.row_val;
    r.done = 0;
    r.pad = 0;
    s_row[lane] = r;
    s_cash[lane] = cash;
  }
  for (int idx = tid; idx < E * D; idx += NT) {
    const int dd = idx / E, e = idx - dd * E;
    s_h[e * Dp + dd] = a.st.h[(size_t)dd * N + n0 + e];
  }
  if (tid < E)
    for (int dd = D; dd < DMAX; ++dd) {
      s_h[tid * Dp + dd] = 0;
      s_p[tid * Dp + dd] = 0.0f;
    }
  __syncthreads();

  constexpr int PAIRS = E / 16;                   // (env, stock) slots per lane
  constexpr int MROWS = (E + MW - 1) / MW;        // market rows per market wavefront
  // (Each helper starts from an opaque copy of the thread index: what it derives from it is loop invariant, and
  // the compiler would otherwise keep it in registers across the matrix-core code instead of recomputing a few
  // integer operations.)
  // Writes the market part of an observation (prices, indicators at row_obs) to HBM row `obs_row` and into the
  // LDS input tile, and refreshes the execution prices.  `p_obs` / `ind_v`: values already in registers.
  auto emit_market = [&](float *obs_row, const float (&p_obs)[MROWS], const f32x4 (&ind_v)[MROWS]) {
    int l = threadIdx.x & 63;
    asm volatile("" : "+v"(l));
    if (is_market) {
      // Straight-line code without lane masks: lanes beyond the row's prices / indicator groups, and passes beyond
      // the tile's last row, repeat the last valid item -- they loaded the same value and store it to the same
      // place again.
      const int lp = min(l, D - 1), li = min(l, (DK >> 2) - 1);
#pragma unroll
      for (int i = 0; i < MROWS; ++i) {
        const int e = min(mw + MW * i, E - 1);
        float *orow = obs_row + (size_t)(n0 + e) * S;
        const float v = p_obs[i];
        s_p[e * Dp + lp] = v;
        const float pv = v * d.s_price;
        __builtin_nontemporal_store(pv, &orow[1 + lp]);
        if (ACTOR) O::store1(ldsX + (size_t)e * a.L.xpitch + (DK + 1 + lp) * O::ESZ, pv);
        f32x4 sv = ind_v[i];
        sv[0] *= d.s_ind;
        sv[1] *= d.s_ind;
        sv[2] *= d.s_ind;
        sv[3] *= d.s_ind;
        // observation rows are 4-byte aligned only; a 16-byte store needs no more than that
        __builtin_nontemporal_store(sv, reinterpret_cast<f32x4 *>(orow + 1 + 2 * D) + li);
        // (indicators lead the LDS tile, so a group of four is one aligned store)
        if (ACTOR) O::store4(ldsX + (size_t)e * a.L.xpitch + 4 * li * O::ESZ, sv[0], sv[1], sv[2], sv[3]);
      }
    }
  };
  // Portfolio part of an observation: cash and holdings from the ledger.
  // AFTER_STEP: also writes the executed trades of step t out and clears the holdings of envs whose episode
  // ended (the same thread owns an (env, stock) slot in both roles, so no barrier is needed in between).
  auto emit_portfolio = [&](float *obs_row, auto after_step, size_t g0) {
    constexpr bool AFTER_STEP = decltype(after_step)::value;
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    if (tid < E) {
      const float sv = s_cash[tid] * d.s_cash;
      __builtin_nontemporal_store(sv, &obs_row[(size_t)(n0 + tid) * S]);
      if (ACTOR) {
        O::store1(ldsX + (size_t)tid * a.L.xpitch + DK * O::ESZ, sv);
        // the policy means were parked over the head of this tile: restore the zero k padding of every row
        const int kp = (a.L.xpitch - 16) / O::ESZ;
        for (int c = S; c < kp; ++c) O::store1(ldsX + (size_t)tid * a.L.xpitch + c * O::ESZ, 0.0f);
      }
    }
    const int dd = tid & 31, e0 = (tid >> 6) * (E / NW) + ((tid >> 5) & 1);
    if (dd < D) {
#pragma unroll
      for (int i = 0; i < PAIRS; ++i) {
        const int e = e0 + 2 * i;
        int32_t h = s_h[e * Dp + dd];
        if (AFTER_STEP) {
          // sales were booked when they were sized; purchases (q > 0) are booked here
          const int32_t q = s_q[e * Dp + dd];
          if (a.shares) a.shares[g0 + (size_t)e * D + dd] = q;
          h = s_done[e] ? 0 : h + max(q, 0);
          s_h[e * Dp + dd] = h;
        }
        const float sv = (float)h * d.s_hold;
        __builtin_nontemporal_store(sv, &obs_row[(size_t)(n0 + e) * S + 1 + D + dd]);
        if (ACTOR) O::store1(ldsX + (size_t)e * a.L.xpitch + (DK + 1 + D + dd) * O::ESZ, sv);
      }
    }
  };
  // Loads into registers: the step's noise and valuation prices are requested at the start of the step and
  // consumed after the actor; the market row of the next observation is requested at the start of the ledger
  // phase and written out at its end (it does not depend on the step's outcome, and this way its registers are
  // not live while the matrix steps need them for weight blocks in flight).
  float r_eps[PAIRS], r_mu[PAIRS], r_pv[PAIRS], r_po[MROWS];
  f32x4 r_ind[MROWS];
  // (s_row is double-buffered by the step's parity: the ledger lanes write the rows of step t + 1 while other
  // wavefronts may still read those of step t)
  auto fetch_valuation = [&](const Row *rows) {
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int dd = min(tid & 31, D - 1), e0 = (tid >> 6) * (E / NW) + ((tid >> 5) & 1);
#pragma unroll
    for (int i = 0; i < PAIRS; ++i)
      r_pv[i] = __builtin_nontemporal_load(&a.price[(size_t)rows[e0 + 2 * i].row_val * D + dd]);
  };
  auto fetch_market = [&](const Row *rows) {
    int l = threadIdx.x & 63;
    asm volatile("" : "+v"(l));
    if (is_market) {
      const int lp = min(l, D - 1), li = min(l, (DK >> 2) - 1);
      const int row_of_lane = rows[min(l, E - 1)].row_obs;  // one LDS read; the rows are then picked lane by lane
#pragma unroll
      for (int i = 0; i < MROWS; ++i) {
        const int e = min(mw + MW * i, E - 1);
        const size_t ro = (size_t)__builtin_amdgcn_readlane(row_of_lane, e);
        r_po[i] = __builtin_nontemporal_load(&a.price[ro * D + lp]);
        r_ind[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.ind + ro * DK) + li);
      }
    } else {
      // (defined on every path: otherwise the values of the previous step count as live all around the loop)
#pragma unroll
      for (int i = 0; i < MROWS; ++i) {
        r_po[i] = 0.0f;
        r_ind[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
      }
    }
  };
  auto fetch_step_inputs = [&](int t) {
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int dd = min(tid & 31, D - 1), e0 = (tid >> 6) * (E / NW) + ((tid >> 5) & 1);
    const size_t g0 = ((size_t)t * N + n0) * D;
#pragma unroll
    for (int i = 0; i < PAIRS; ++i) {
      r_eps[i] = __builtin_nontemporal_load(&a.noise[g0 + (size_t)(e0 + 2 * i) * D + dd]);
      if (!ACTOR) r_mu[i] = a.mu_forced[g0 + (size_t)(e0 + 2 * i) * D + dd];
    }
  };

  {
    fetch_market(s_row);
    emit_market(a.obs, r_po, r_ind);
    emit_portfolio(a.obs, std::false_type{}, 0);
  }
  __syncthreads();
  if (wave == LW && lane < E) {
    // account value the first reward is measured against; cursor rows of step 0
    const int e = lane;
    double v = (double)cash;
    for (int dd = 0; dd < D; ++dd) v += (double)s_h[e * Dp + dd] * (double)s_p[e * Dp + dd];
    asset = v;
    s_row[e] = row_of(d, tau, start, n0 + e);  // (step 0 reads buffer 0 again: the barrier at the loop top orders it)
  }

  // Weight ring of the actor.  Layer 1's first blocks are requested a phase early (here, and after each step's
  // ledger) so that they are in flight while the observation is completed.
  u32x4 ring[PDR][CTH];
  const float *lb3 = ldsBias + (ACTOR ? (a.actor.nct[0] + a.actor.nct[1]) * 32 : 0);
  if (ACTOR) prime<CTH, PDR>(ring, net.W[0], net.nkb[0], net.nct[0], wave * CTH, lane);
  // split schedule: layer-1 accumulators of group A, carried from the ledger phase of one step into the next
  f32x16 acc1[SPLIT ? CTH : 1][SPLIT ? NBT : 1];
  auto layer1_head = [&]() {  // group A: bias and the first NK1A k-blocks; leaves the ring primed with the rest
    if constexpr (SPLIT) {
      int lane_h = lane;
      asm volatile("" : "+v"(lane_h));
      bias_acc<CTH, NBT>(acc1, ldsBias, wave * CTH, lane_h);
      mma_range_static<true, CTH, NBT, PDR, NK1A, true, true>(acc1, ring, ldsX, a.L.xpitch, net.W[0], net.nct[0], 0,
                                                             net.W[0], net.nct[0], NK1A, wave * CTH, 0, lane_h);
    }
  };
  if constexpr (SPLIT) {
    if (wave < NW / 2) layer1_head();  // (observation 0 is complete: the barrier above)
  }
  // Group B's wavefronts start every step by overwriting the layer-1 accumulators and the ring, but the compiler
  // cannot tell that the ledger code only runs on a wavefront of group B and would keep both live (128
  // registers) through it.  An empty statement that "produces" them ends their live range there at no cost.
  auto forget_actor_registers = [&]() {
    if constexpr (SPLIT) {
#pragma unroll
      for (int c = 0; c < CTH; ++c)
#pragma unroll
        for (int b = 0; b < NBT; ++b) asm volatile("" : "=v"(acc1[c][b]));
#pragma unroll
      for (int s = 0; s < PDR; ++s)
#pragma unroll
        for (int c = 0; c < CTH; ++c) asm volatile("" : "=v"(ring[s][c]));
    }
  };

  for (int t = 0; t < a.T; ++t) {
    __syncthreads();  // observation t complete in LDS; ledger rows of step t visible
    float *obs_next = a.obs + (size_t)(t + 1) * N * S;
    const size_t g0 = ((size_t)t * N + n0) * D;
    const Row *rows_t = s_row + (t & 1) * E;
    Row *rows_next = s_row + ((t + 1) & 1) * E;

    if constexpr (SPLIT) {
      // ---- the actor, two wavefront groups half a layer out of step
      // Group A (wavefronts 0-3) owns hidden features 0-255, group B (4-7) features 256-511.  Both run the same
      // five steps with a barrier after each -- (a) layer 1, (b) its tanh -> own half of the hidden tile,
      // (c) layer 2 over the own half, (d) layer 2 over the other group's half, (e) tanh of layer 2 and the output
      // layer's partial sums over the own features -- but B runs them one barrier later than A, so the tanh steps
      // of one group fall under matrix steps of the other on the same SIMDs.  The slot a group has no step in
      // (B the first, A the last) is where its lanes request the step's market rows and noise.
      // Step (e) feeds the output layer from registers: the eight values a lane holds of a feature tile's half
      // are one k-block of the transposed product, in the k order the output weights were permuted to at set-up.
      // The partial sums of a wavefront pair (w, w + 4) meet in plane w of the policy means.
      constexpr int PDS = PDR, HALF = NKB2 / 2;
      const bool grpB = wave >= NW / 2;
      const int ct0 = wave * CTH;
      const int own0 = grpB ? HALF : 0, oth0 = grpB ? 0 : HALF;
      const float *lb1 = ldsBias, *lb2 = ldsBias + net.nct[0] * 32;
      f32x16 (&acc)[CTH][NBT] = acc1;
      int lane_s = lane;  // (opaque per step, or the addresses of all weight blocks are hoisted out of the step loop)
      asm volatile("" : "+v"(lane_s));
      if (grpB) {
        fetch_step_inputs(t);
        fetch_valuation(rows_t);
        __syncthreads();
        bias_acc<CTH, NBT>(acc, lb1, ct0, lane_s);
        // (group B is the one the barriers wait for: its matrix steps go first on the SIMDs it shares with A)
        __builtin_amdgcn_s_setprio(kLagPrio);
        mma_range_static<true, CTH, NBT, PDS, NKB1, true, true>(acc, ring, ldsX, a.L.xpitch, net.W[0], net.nct[0], 0,
                                                                net.W[1], net.nct[1], own0, ct0, 0, lane_s);
      } else {
        // (the head of layer 1 ran during the previous step's ledger phase)
        mma_range_static<true, CTH, NBT, PDS, NKB1 - NK1A, true, true>(acc, ring, ldsX + NK1A * 32, a.L.xpitch, net.W[0],
                                                                       net.nct[0], NK1A, net.W[1], net.nct[1], own0, ct0,
                                                                       0, lane_s);
      }
      __builtin_amdgcn_s_setprio(0);
      __syncthreads();
      epilogue_hidden_biased<CTH, NBT>(acc, ldsH, a.L.hpitch, ct0, 0, lane_s);
      __syncthreads();
      bias_acc<CTH, NBT>(acc, lb2, ct0, lane_s);
      if (grpB) __builtin_amdgcn_s_setprio(kLagPrio);
      mma_range_static<true, CTH, NBT, PDS, HALF, true, true>(acc, ring, ldsH + own0 * 32, a.L.hpitch, net.W[1], net.nct[1], own0,
                                                   net.W[1], net.nct[1], oth0, ct0, 0, lane_s);
      __syncthreads();
      mma_range_static<true, CTH, NBT, PDS, HALF, false, true>(acc, ring, ldsH + oth0 * 32, a.L.hpitch, net.W[1], net.nct[1],
                                                          oth0, net.W[1], net.nct[1], 0, ct0, 0, lane_s);
      __builtin_amdgcn_s_setprio(0);
      __syncthreads();
      {
        f32x16 o3[NBT];
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
          for (int i = 0; i < 16; ++i) o3[b][i] = 0.0f;
#pragma unroll
        for (int c = 0; c < CTH; ++c) {
          tanh_in_place<NBT>(acc[c]);
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            const u32x4 wb = ldsW3[((ct0 + c) * 2 + kk) * 64 + lane_s];
#pragma unroll
            for (int b = 0; b < NBT; ++b) {
              const bf16x8 v = {(__bf16)acc[c][b][8 * kk],     (__bf16)acc[c][b][8 * kk + 1], (__bf16)acc[c][b][8 * kk + 2],
                                (__bf16)acc[c][b][8 * kk + 3], (__bf16)acc[c][b][8 * kk + 4], (__bf16)acc[c][b][8 * kk + 5],
                                (__bf16)acc[c][b][8 * kk + 6], (__bf16)acc[c][b][8 * kk + 7]};
              O::mma(wb, __builtin_bit_cast(u32x4, v), o3[b]);
            }
          }
        }
        float *plane = s_mu + (wave & 3) * (E * MUP) + (lane_s & 31) * MUP + 4 * (lane_s >> 5);
        if (grpB) {
          // (all reads in flight before the first sum: one LDS round trip, not one per value)
          f32x16 old[NBT];
#pragma unroll
          for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) old[b][i] = plane[b * 32 * MUP + 8 * (i >> 2) + (i & 3)];
#pragma unroll
          for (int b = 0; b < NBT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) o3[b][i] += old[b][i];
        }
#pragma unroll
        for (int b = 0; b < NBT; ++b)
#pragma unroll
          for (int i = 0; i < 16; ++i) plane[b * 32 * MUP + 8 * (i >> 2) + (i & 3)] = o3[b][i];
      }
      __syncthreads();
      // (group A has passed five barriers, group B six; A's sixth is in its branch below, behind the requests for
      // its noise, valuation prices and market rows -- the slot in which B runs step (e))
    } else {
      if (ACTOR) {
        mlp_tile<BF16, NW, CTH, false, NKB1, NKB2, true, true, KS, NBT>(
            net, ring, ldsX, a.L.xpitch, ldsH, a.L.hpitch, ldsBias, ldsW3, tid,
            [&]() {
              fetch_step_inputs(t);
              fetch_valuation(rows_t);
            },
            [&]() {},
            [&](int b, int f, float z, int part = 0) { s_mu[part * (E * MUP) + b * MUP + f] = z; });  // finished below
      } else {
        fetch_step_inputs(t);
        fetch_valuation(rows_t);
      }
      __syncthreads();  // means in LDS; the hidden tile is free for the env scratch
    }

    // ---- everything that does not depend on the running cash, all lanes (slots D..31 get neutral values)
    auto size_orders = [&]() {
      int tid_p = threadIdx.x;
      asm volatile("" : "+v"(tid_p));
      const int dd = tid_p & 31, e0 = (tid_p >> 6) * (E / NW) + ((tid_p >> 5) & 1);
      const bool live = dd < D;
#pragma unroll
      for (int i = 0; i < PAIRS; ++i) {
        const int e = e0 + 2 * i, o = e * Dp + dd;
        float mu;
        if (ACTOR) {
          float z = s_mu[e * MUP + dd];
#pragma unroll
          for (int part = 1; part < KS; ++part) z += s_mu[part * (E * MUP) + e * MUP + dd];
          mu = finish_out(z, lb3[dd], 1);
        } else {
          mu = r_mu[i];
        }
        const float eps = live ? r_eps[i] : 0.0f;
        const float a_raw = live ? mu + d.sigma * eps : 0.0f;
        if (live) {
          __builtin_nontemporal_store(a_raw, &a.act_raw[g0 + (size_t)e * D + dd]);
          if (ACTOR && a.mu_out) a.mu_out[g0 + (size_t)e * D + dd] = mu;
        }
        const float ac = fminf(1.0f, fmaxf(-1.0f, a_raw));
        const int32_t k = (int32_t)truncf(ac * d.hmax);
        const float p = s_p[o];
        int32_t q = 0;
        float val = 0.0f;
        double rcp = 0.0;
        if (k < 0) {
          const int32_t h = s_h[o];
          q = min(-k, h);
          s_h[o] = h - q;
          const float gross = p * (float)q;
          val = gross * d.one_minus_c;
          q = -q;
        } else if (k > 0) {
          val = p * d.one_plus_c;
          rcp = 1.0 / (double)val;
        }
        Slot sl;
        sl.k = k;
        sl.val = val;
        sl.rcp = rcp;
        s_slot[o] = sl;
        s_q[o] = q;
        s_pv[o] = live ? r_pv[i] : 0.0f;
        s_e2[o] = eps * eps;
      }
    };

    auto run_ledger = [&]() {
      // ---- the ledger: one lane per env walks the cash chain in stock order
      // Each pass stages a chunk of the lane's row in registers first, so that the LDS reads of a chunk are
      // all in flight together and the dependent chain on `cash` runs on registers only.
      int e = lane;
      asm volatile("" : "+v"(e));  // per-step opaque, or the chunk addresses are hoisted out of the step loop
      const int n = n0 + e, o0 = e * Dp;
      constexpr int CH = 16;
#pragma unroll
      for (int c0 = 0; c0 < DMAX; c0 += CH) {
        Slot sl[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) sl[j] = s_slot[o0 + c0 + j];
#pragma unroll
        for (int j = 0; j < CH; ++j) cash = sl[j].k < 0 ? cash + sl[j].val : cash;
      }
      // Purchases in stock order, the trading rule in straight-line code:
      //   m = floor(cash / u); q = min(k, max(m, 0)); if (q u > cash) q -= 1; cash -= q u        (binary32)
      // One lane per env walks a dependent chain on `cash`, so what counts is the length of that chain, not
      // the instruction count: no data-dependent branches (a branch taken for one lane costs all 64 the round
      // trip through the scalar unit), and everything that does not depend on `cash` sits off the chain.
      // The binary32 quotient comes from one binary64 product with the reciprocal of u prepared by the other
      // lanes: the product is within 2^-52 of cash / u, a quotient of two binary32 numbers is at least 2^-49
      // (relative) away from every binary32 rounding boundary it does not hit exactly, so rounding the product
      // to binary32 gives the correctly rounded cash / u -- the same value as the division, in 3 dependent
      // operations instead of 11.
      int32_t hn[DMAX];  // holdings after the trades (written back by the pass that emits them)
#pragma unroll
      for (int c0 = 0; c0 < DMAX; c0 += CH) {
        Slot sl[CH];
        int32_t hh[CH], qq[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
          sl[j] = s_slot[o0 + c0 + j];
          hh[j] = s_h[o0 + c0 + j];
          qq[j] = s_q[o0 + c0 + j];
        }
#pragma unroll
        for (int j = 0; j < CH; ++j) {
          // On the chain through `cash`: widen, multiply, narrow, truncate, min, multiply, subtract | compare,
          // select -- eight operations.  Sales and holds have k = 0 and reciprocal 0: q = 0, outlay 0.  The
          // quotient is never negative (cash is not), so truncation is the floor and needs no clamp at 0; the
          // outlay of one share less, (q - 1) u rounded once, is the fused q u - u (the same real number, one
          // rounding); both candidate balances are formed before the comparison is known.
          const float kf = (float)max(sl[j].k, 0);
          const float u = sl[j].val;
          const float ratio = (float)((double)cash * sl[j].rcp);
          const float q0 = fminf(kf, truncf(ratio));
          const float out_q = q0 * u, out_q1 = fmaf(q0, u, -u);
          const float bal0 = cash - out_q, bal1 = cash - out_q1;
          const bool over = out_q > cash;
          cash = over ? bal1 : bal0;
          const int32_t q = (int32_t)(over ? q0 - 1.0f : q0);
          hn[c0 + j] = hh[j] + q;
          s_q[o0 + c0 + j] = qq[j] + q;  // (a purchase slot held 0)
        }
      }
      double asset1 = (double)cash;
#pragma unroll
      for (int c0 = 0; c0 < DMAX; c0 += CH) {
        float pp[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) pp[j] = s_pv[o0 + c0 + j];
#pragma unroll
        for (int j = 0; j < CH; ++j) asset1 += (double)hn[c0 + j] * (double)pp[j];  // empty slots add +0
      }
      const double r = (asset1 - asset) * (double)d.rho;
      asset = asset1;
      ep_ret += r;
      const int dn = rows_t[e].done;
      const size_t tn = (size_t)t * N + n;
      a.reward[tn] = (float)r;
      a.done[tn] = (uint8_t)dn;
      if (dn) {
        ep_sum += ep_ret;
        ep_sqsum += ep_ret * ep_ret;
        ep_cnt += 1;
        ep_ret = 0.0;
        cash = d.cash0;
        asset = (double)d.cash0;
        tau = start;
      } else {
        tau += 1;
      }
      s_cash[e] = cash;
      s_done[e] = dn;
      rows_next[e] = row_of(d, tau, start, n);  // cursor rows of step t + 1
    };
    auto run_logp = [&]() {
      // ---- log-probability of the sampled action: squared noise summed in stock order, one lane per env
      int e = lane;
      asm volatile("" : "+v"(e));
      const int o0 = e * Dp;
      float e2 = 0.0f;
#pragma unroll
      for (int c0 = 0; c0 < DMAX; c0 += 16) {
        float ee[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) ee[j] = s_e2[o0 + c0 + j];
#pragma unroll
        for (int j = 0; j < 16; ++j) e2 += ee[j];  // empty slots add +0
      }
      a.logp[(size_t)t * N + n0 + e] = fmaf(-0.5f, e2, d.logp_const);

    };

    // The ledger wavefront and the others run separate code from here to the end of the ledger phase (with the
    // same barrier between the two phases), so that the registers of the market row the others carry through
    // the ledger phase are not live in the ledger's code.
    if constexpr (SPLIT) {
      if (wave < NW / 2) {
        // group A: market row of observation t + 1 (requested in its last actor slot), then -- once all four of
        // its wavefronts have written their rows -- the head of the next step's layer 1
        fetch_step_inputs(t);
        fetch_valuation(rows_t);
        fetch_market(rows_t);
        __syncthreads();  // the means are complete and the hidden tile is free
        size_orders();
        __syncthreads();
        {
          // (also after the last step, like the head of layer 1 below: harmless, and the ring and the accumulators
          // are then defined on every path through this branch -- nothing of the previous step stays live in it)
          int lane_p = lane;  // (opaque per step: the block addresses are recomputed here, not kept across the step)
          asm volatile("" : "+v"(lane_p));
          prime<CTH, PDR>(ring, net.W[0], net.nkb[0], net.nct[0], wave * CTH, lane_p);
        }
        emit_market(obs_next, r_po, r_ind);
        // meeting point of group A alone (the other wavefronts are busy and meet everybody at the barrier below):
        // a counter in LDS that every wavefront of the group bumps once per step and then waits on, with a bound
        // on the wait so that a mistake elsewhere shows as a wrong result, never as a hang
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(s_sync, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int target = MW * (t + 1);
        for (int spin = 0; spin < (1 << 20); ++spin) {
          if (__hip_atomic_load(s_sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= target) break;
          __builtin_amdgcn_s_sleep(1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        layer1_head();
      } else if (wave == LW) {
        size_orders();
        __syncthreads();
        if (lane < E) run_ledger();
        forget_actor_registers();
      } else {
        size_orders();
        __syncthreads();
        if (wave == LW + 1 && lane < E && a.logp) run_logp();
        forget_actor_registers();
      }
      __syncthreads();
      if (wave >= NW / 2) {  // (also after the last step: the loads are harmless, and the ring is defined on every path)
        int lane_p = lane;
        asm volatile("" : "+v"(lane_p));
        prime<CTH, PDR>(ring, net.W[0], net.nkb[0], net.nct[0], wave * CTH, lane_p);
      }
    } else {
      if (wave == 0) {
        size_orders();
        __syncthreads();
        if (lane < E) run_ledger();
      } else {
        size_orders();
        __syncthreads();
        // ---- meanwhile, the other wavefronts: the market row of observation t + 1 (requested here, written out
        // at the end of the phase), and on one of them the log-probabilities
        fetch_market(rows_t);
        if (wave == 1 && lane < E && a.logp) run_logp();
        emit_market(obs_next, r_po, r_ind);
      }
      __syncthreads();
      if (ACTOR && t + 1 < a.T) {
        int lane_p = lane;  // (opaque per step: the block addresses are recomputed here, not kept across the step)
        asm volatile("" : "+v"(lane_p));
        prime<CTH, PDR>(ring, net.W[0], net.nkb[0], net.nct[0], wave * CTH, lane_p);
      }
    }

    // ---- executed trades out; episode ends clear the holdings; portfolio part of observation t+1
    emit_portfolio(obs_next, std::true_type{}, g0);
  }

  // ---- epilogue: state back to the workspace
  __syncthreads();
  if (wave == LW && lane < E) {
    const int n = n0 + lane;
    a.st.cash[n] = cash;
    a.st.tau[n] = tau;
    a.st.ep_ret[n] = ep_ret;
    a.st.ep_sum[n] = ep_sum;
    a.st.ep_sqsum[n] = ep_sqsum;
    a.st.ep_cnt[n] = ep_cnt;
  }
  for (int idx = tid; idx < E * D; idx += NT) {
    const int dd = idx / E, e = idx - dd * E;
    a.st.h[(size_t)dd * N + n0 + e] = s_h[e * Dp + dd];
  }
}

// Kernel instance for a configuration: feature tiles per wavefront and, for the named shape, compile-time k-block
// counts of layers 1 and 2 (0: read at run time).
struct FusedShape {
  int envs, cth, nkb1, nkb2;  // envs per workgroup; feature tiles per wavefront; k-blocks of layers 1, 2 (0: run time)
};

FusedShape fused_shape(const pr_config &c) {
  const int S = 1 + 2 * c.n_stocks + c.n_stocks * c.n_ind;
  const int KB = c.mlp_dtype == PR_MLP_BF16 ? 16 : 8;
  FusedShape f;
  f.envs = c.mlp_dtype == PR_MLP_BF16 ? 64 : 32;
  f.cth = (c.hidden / 32) / NW;
  f.nkb1 = f.nkb2 = 0;
  // the named shapes: 301 inputs with 512 hidden units in bf16 / 256 hidden units in fp32
  // (the split schedule of this instance runs the first 11 k-blocks of layer 1 before the portfolio columns
  // exist: they must all be indicator columns)
  if (KB == 16 && f.cth == 2 && (S + 15) / 16 == 19 && c.hidden / 16 == 32 && c.n_stocks * c.n_ind >= 11 * 16)
    f.nkb1 = 19, f.nkb2 = 32;
  if (KB == 8 && f.cth == 1 && (S + 7) / 8 == 38 && c.hidden / 8 == 32) f.nkb1 = 38, f.nkb2 = 32;
  return f;
}

// The one carve-up of the kernel's LDS.
FusedLayout fused_layout(const pr_config &c, bool with_actor) {
  const int D = c.n_stocks, S = 1 + 2 * D + D * c.n_ind, Hd = c.hidden;
  const bool bf = c.mlp_dtype == PR_MLP_BF16;
  const int KB = bf ? 16 : 8, esz = bf ? 2 : 4;
  const FusedShape fs = fused_shape(c);
  const int E = fs.envs;
  const int nkb1 = (S + KB - 1) / KB, nct = Hd / 32;
  FusedLayout L;
  L.xpitch = tile_pitch(nkb1 * KB, esz);
  L.hpitch = tile_pitch(Hd, esz);
  // the env scratch (slots 16 B, executed shares, valuation prices, squared noise) must fit in the hidden tile
  const size_t env_scratch = (size_t)7 * E * kDp * 4;
  if ((size_t)E * L.hpitch < env_scratch) L.hpitch = (int32_t)(((env_scratch + E - 1) / E + 15) / 16 * 16);
  size_t off = (size_t)E * L.hpitch;
  L.off_x = (int32_t)off;
  size_t xbytes = (size_t)E * L.xpitch;
  const size_t mu_bytes = with_actor ? (size_t)mu_planes(fs.nkb2) * E * MUP * 4 : 0;
  if (xbytes < mu_bytes) xbytes = (mu_bytes + 15) / 16 * 16;
  off += xbytes;
  L.off_w3 = (int32_t)off;
  if (with_actor) off += (size_t)(Hd / KB) * 1024;  // output layer: one feature tile, Hd / KB k-blocks of 1 KiB
  L.off_bias = (int32_t)off;
  if (with_actor) off += (size_t)(2 * nct + 1) * 32 * 4;
  L.off_h = (int32_t)off;
  off += (size_t)E * kDp * 4;
  L.off_p = (int32_t)off;
  off += (size_t)E * kDp * 4;
  L.off_row = (int32_t)off;
  off += (size_t)2 * E * sizeof(Row);  // two buffers, by the step's parity
  L.off_cash = (int32_t)off;
  off += (size_t)E * 4;
  L.off_done = (int32_t)off;
  off += (size_t)E * 4 + 16;  // episode-end flags, and the meeting counter of the split schedule behind them
  L.total = (int32_t)off;
  return L;
}

constexpr size_t kLdsMax = kMaxLdsBytes;

}  // namespace

// Shapes the persistent kernel covers: networks whose whole input tile, hidden tile and output-layer weights fit
// in LDS next to the env arrays -- bf16 with 256 or 512 hidden units on 64-env tiles, fp32 with 256 hidden units
// on 32-env tiles; N (and the envs of an agent) a multiple of the tile; D <= 32; D K <= 252 and a multiple of 4
// (the indicator rows are moved in 16-byte groups; the market tensors must be 16-byte aligned); one output
// feature tile.
bool fused_supported(const pr_config &c) {
  const int D = c.n_stocks, DK = c.n_stocks * c.n_ind, S = 1 + 2 * D + DK, Hd = c.hidden;
  if (c.mlp_dtype != PR_MLP_BF16 && c.mlp_dtype != PR_MLP_F32) return false;
  const int E = fused_shape(c).envs;
  if (c.n_envs % E != 0 || D > 32 || DK > 252 || DK < 4 || DK % 4 != 0 || S < 4) return false;
  if (Hd % 32 != 0 || Hd < 256 || Hd > 512 || (Hd / 32) % NW != 0) return false;
  if (c.mlp_dtype == PR_MLP_F32 && Hd != 256) return false;
  if (c.n_agents > 1 && (c.n_envs / c.n_agents) % E != 0) return false;
  return fused_lds_bytes(c, true) <= kLdsMax;
}

size_t fused_lds_bytes(const pr_config &c, bool with_actor) { return (size_t)fused_layout(c, with_actor).total; }

template <bool BF16, int E, bool ACTOR, int CTH, int NKB1, int NKB2>
static hipError_t launch_fused_inst(hipStream_t st, const FusedArgs &a, unsigned blocks, size_t lds) {
  constexpr auto kern = rollout_fused_kernel<BF16, E, CTH, NKB1, NKB2, ACTOR>;
  const hipError_t e = allow_full_lds<kern>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(NT), lds, st, a);
  return hipGetLastError();
}

hipError_t launch_rollout_fused(hipStream_t st, const pr_config &c, const EnvDims &d, const EnvState &s,
                                const float *price, const float *ind, const PackedNet &actor, int32_t envs_per_agent,
                                int32_t T, const float *noise, const float *mu_forced, const pr_buffers &out) {
  if (!fused_supported(c)) return hipErrorInvalidValue;
  FusedArgs a;
  a.d = d;
  a.st = s;
  a.price = price;
  a.ind = ind;
  a.actor = actor;
  a.envs_per_agent = envs_per_agent;
  a.T = T;
  a.noise = noise;
  a.mu_forced = mu_forced;
  a.obs = out.obs;
  a.act_raw = out.act_raw;
  a.reward = out.reward;
  a.done = out.done;
  a.logp = out.logp;
  a.mu_out = mu_forced ? nullptr : out.mu;
  a.shares = out.shares;
  const int DK = d.D * d.K;
  const bool with_actor = mu_forced == nullptr;
  a.L = fused_layout(c, with_actor);
  if (reinterpret_cast<uintptr_t>(ind) & 15u) return hipErrorInvalidValue;  // 16-byte indicator loads
  const size_t lds = (size_t)a.L.total;
  if (lds > kLdsMax) return hipErrorInvalidValue;
  const FusedShape fs = fused_shape(c);
  const unsigned blocks = (unsigned)(d.N / fs.envs);
  const int KB = actor.bf16 ? 16 : 8, esz = actor.bf16 ? 2 : 4;
  if (with_actor && ((actor.bf16 != 0) != (c.mlp_dtype == PR_MLP_BF16) || tile_pitch(actor.nkb[0] * KB, esz) != a.L.xpitch ||
                     tile_pitch(actor.nkb[1] * KB, esz) > a.L.hpitch || actor.nkb[2] != actor.nkb[1] || actor.nct[2] != 1))
    return hipErrorInvalidValue;  // the packed network is not the one the layout was made for
  if (c.mlp_dtype == PR_MLP_BF16) {
    if (!with_actor) return launch_fused_inst<true, 64, false, 1, 0, 0>(st, a, blocks, lds);
    if (fs.cth == 2 && fs.nkb1 == 19 && fs.nkb2 == 32) return launch_fused_inst<true, 64, true, 2, 19, 32>(st, a, blocks, lds);
    if (fs.cth == 2) return launch_fused_inst<true, 64, true, 2, 0, 0>(st, a, blocks, lds);
    if (fs.cth == 1) return launch_fused_inst<true, 64, true, 1, 0, 0>(st, a, blocks, lds);
  } else {
    if (!with_actor) return launch_fused_inst<false, 32, false, 1, 0, 0>(st, a, blocks, lds);
    if (fs.cth == 1 && fs.nkb1 == 38 && fs.nkb2 == 32) return launch_fused_inst<false, 32, true, 1, 38, 32>(st, a, blocks, lds);
    if (fs.cth == 1) return launch_fused_inst<false, 32, true, 1, 0, 0>(st, a, blocks, lds);
  }
  return hipErrorInvalidValue;
}

}  // namespace pod
