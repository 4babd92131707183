// The whole decode-time MoE layer in ONE persistent kernel (gfx950): one workgroup per CU.
//
//   phase R1  router GEMV, spread over all workgroups (fp64 accumulation, one dot product per
//             wavefront); x of the batch is staged into LDS meanwhile; `out` is cleared
//   -- grid barrier (two-level arrival counters, no cache maintenance) --
//   phase R2  OEA routing (Algorithm 1), computed redundantly by EVERY workgroup from the logits
//             into its own LDS: no second barrier, no routing metadata read back from memory;
//             then the cost-weighted cut of both stages' rows over the workgroups
//   phase A   gate/up mat-vec stage over the active experts: the wavefronts take tiles from a
//             counter in LDS, stream them double-buffered, collect the hidden units in LDS and
//             write them out at the end; then the workgroup adds its rows to the completion
//             counters of its experts
//   phase B   down mat-vec stage: first tiles requested, then the workgroup waits (bounded) for the
//             completion counters of ITS experts only, stages their hidden vectors and streams;
//             results are added into `out` with the gate weights at the end (Eq. 1)
//
// Compared with three back-to-back kernels this removes two dispatch gaps with their pipeline
// drain/fill and every dependent metadata load.  All 256 workgroups must be resident at once: the
// launcher checks that a workgroup fits on every CU and every wait spins for a bounded time only.
#include "oea_ffn_dev.h"
#include "oea_timeline.h"
#include "oea_route_dev.h"

namespace oea {

namespace {

constexpr size_t kFusedLdsMax = 156 * 1024;
#define OEA_MAX_FUSED_N 128  // experts the fused kernel handles (completion words in the control area)
constexpr int kFusedStage = 8;  // staging loads kept in flight per thread
// Small-batch kernel, down stage: two wavefronts (few active experts) or one request no weight
// tiles before the hidden vectors are there, and stage them (see fused_stage).
// Measured at B=16: -1.2 us with two at T=36, but +0.4 us at T=73, where one is neutral.
constexpr int kStageWaves = 2;
constexpr int kBalBase = 1024 + 2 * OEA_MAX_FUSED_N * 32;  // ctrl word of the speed-weight state: w[2][256], rate[256]
constexpr int kBalMaxWg = 256;                             // workgroups it covers

struct FusedParams {
  const void* x;
  const void* w_router;
  const void* w_gate;
  const void* w_up;
  const void* w_down;
  const float* bias;
  const uint8_t* token_mask;
  float* out;
  float* acc;      // what the down stage adds into: out [B,d], or (deterministic combine) y [B*k, d], one row per pair
  int acc_rows;    // its rows: B or B*k
  float* logits;   // [B,N] workspace
  void* h;         // [B*k, I] workspace
  RouteOut ro;     // global copies of the routing result, written by workgroup 0
  uint32_t* ctrl;  // [3] error flag, [32] and [256 + 32 i] barrier arrivals, [64] barrier generation (separate
                   // 128-byte lines), from [1024] the per-expert completion counters (done_count)
  int B, d, N, I, k, k0;
  int cap_vec;     // most (expert, token) pairs one workgroup can meet in one stage (large batches: vectors per
                   // piece in the gate/up stage)
  int cap_vec1;    // large batches: vectors per piece in the down stage
  int ecap0, ecap1;  // floats of LDS result buffer per wavefront, gate/up and down stage (0 = none)
  uint32_t spin_limit;
  // general OEA (Algorithm 2) in the kernel: top-p threshold and rank window; k is k_max
  int general;
  int gen_max_p;
  double gen_p;
};

// words of LDS in front of the vector area (after the 16-byte dump slot)
__host__ __device__ inline size_t fused_meta_words(int B, int N, int k) {
  const size_t P = (size_t)B * k;
  size_t w = route_lds_words(B, N) + 4 * P + (size_t)B + (size_t)N + 4 + (size_t)N + 4 + kBalMaxWg + 4;
  return (w + 3) & ~size_t(3);
}

// Barrier over all workgroups of the grid: an arrival counter that returns to 0 and a generation
// word that only grows, on separate 128-byte lines (the pollers read the generation, the arrivals
// hit the counter).  The generation is read ONCE per call, at the start of the kernel (no barrier of
// this call can complete before this workgroup has arrived); barrier i of the call is passed when
// the generation has reached gen0 + i.  The workgroup whose arrival completes the count (which
// wraps back to 0 by itself) publishes the next generation.
//
// There is no cache maintenance here (a device-scope fence writes back / invalidates the whole L2
// of the XCD, far too slow): data that crosses workgroups in this kernel is written with
// device-coherent stores and read with device-coherent loads.  grid_arrive drains the wavefront's
// stores before the workgroup's __syncthreads, so they have reached memory before thread 0
// announces the workgroup.
// The wait is bounded: after spin_limit polls the workgroup raises the error flag and goes on
// (its results are then meaningless, but every access stays in bounds and the kernel ends).
__device__ __forceinline__ uint32_t grid_generation(uint32_t* ctrl) {
  return __hip_atomic_load(ctrl + 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Arrivals go through two levels: workgroup b adds to leaf counter b % kBarrierLeaves, the arrival
// that completes a leaf adds to the root, the one that completes the root publishes the generation.
// Atomics on one line execute one after the other (about 20 ns each), so 256 arrivals on a single
// counter cost 4-5 us; with 16 leaves on lines of their own the two levels take 2 x 16 steps.
constexpr int kBarrierLeaves = 16;
constexpr int kBarrierLeafBase = 256;  // ctrl word of leaf 0; one 128-byte line per leaf

// next = the generation that completes this barrier (thread 0's value is the one used)
__device__ __forceinline__ void grid_arrive(uint32_t* ctrl, uint32_t next) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's stores have reached memory
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t G = gridDim.x, b = blockIdx.x;
    const uint32_t leaf = b % kBarrierLeaves;
    const uint32_t n_leaves = G < kBarrierLeaves ? G : kBarrierLeaves;
    const uint32_t members = (G - leaf + kBarrierLeaves - 1) / kBarrierLeaves;  // workgroups on this leaf
    // wrapping increments: the arrival that completes a counter also returns it to 0, in one atomic
    if (atomicInc(ctrl + kBarrierLeafBase + 32 * leaf, members - 1) == members - 1)
      if (atomicInc(ctrl + 32, n_leaves - 1) == n_leaves - 1)
        __hip_atomic_store(ctrl + 64, next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

__device__ __forceinline__ void grid_wait(uint32_t* ctrl, uint32_t next, uint32_t spin_limit) {
  if (threadIdx.x == 0) {
    uint32_t spins = 0;
    // signed distance: correct across the wrap of the 32-bit generation
    while (int(__hip_atomic_load(ctrl + 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - next) < 0) {
      __builtin_amdgcn_s_sleep(2);
      if (++spins > spin_limit) {
        atomicExch(ctrl + kCtrlErrWord, 1u);
        break;
      }
    }
  }
  __syncthreads();
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---- cost-weighted split of a stage over the workgroups.
// A weight row of an expert with c pairs costs about (kRowCost + beta*c): streaming its bytes plus c
// dot products per weight.  Cutting the concatenated rows of the active experts by BYTES leaves the
// workgroups that own popular experts (many tokens) computing after the others have finished (in
// the gate/up stage about 1.6 us per extra token at B=16, and the down stage of an expert cannot
// start before its slowest gate/up part); cutting by COST lets everyone finish together.
// With off[] the CSR offsets of the pairs, the cost of all rows of the active experts before
// position a is rows * (kRowCost*a + beta*off[a]); workgroup b starts at the row at cost total*b/G.
constexpr int kRowCost = 64;
#ifndef OEA_BETA_UP
#define OEA_BETA_UP 3
#endif
#ifndef OEA_BETA_DOWN
#define OEA_BETA_DOWN 12
#endif
constexpr int kBetaUp = OEA_BETA_UP;      // per pair, gate/up stage
constexpr int kBetaDown = OEA_BETA_DOWN;  // per pair, down stage (also makes up for what is left of the gate/up skew)

// ---- speed weights of the workgroups.
// Workgroups do not stream equally fast (on the measured device the odd-numbered XCDs ran 2-4 %
// behind the even ones, every call), and the layer ends with the slowest.  The workspace keeps a
// weight per workgroup, an exponential average of its measured share-per-time; the cost range is
// cut in proportion to the weights.  Call n reads buffer n%2 and the rates of call n-1 and writes
// buffer (n+1)%2 (workgroup 0 only), so every workgroup of a call derives the same boundaries.

// First row of workgroup b (b in [0,G]) in the concatenated numbering.  Called by whole wavefronts
// (every lane tests two positions of the active list, T <= 128); the result is wave-uniform and the
// same in every workgroup.
__device__ __forceinline__ int wg_first_row(const int* l_off, int T, int rows, int beta, int b, int G, int lane,
                                            const float* l_frac = nullptr) {
  if (b <= 0 || T <= 0) return 0;
  if (b >= G) return T * rows;
  // All quantities are integers below 2^40, exact in double; the divisions go through double because
  // 64-bit integer division is a long instruction sequence on this GPU.  Every workgroup evaluates
  // the same expression for boundary b, so neighbours agree on it.
  const double total = double(kRowCost) * T + double(beta) * l_off[T];  // in units of one row
  // l_frac[b]: share of the total cost given to the workgroups before b (speed-weighted); else equal shares
  const double x = l_frac ? floor(total * rows * double(l_frac[b])) : floor(total * rows * b / G);
  const int a0 = lane, a1 = lane + 64;
  const double p0 = double(rows) * (double(kRowCost) * a0 + double(beta) * l_off[a0 < T ? a0 : T]);
  const double p1 = double(rows) * (double(kRowCost) * a1 + double(beta) * l_off[a1 < T ? a1 : T]);
  const int below = __popcll(__ballot(a0 < T && p0 <= x)) + __popcll(__ballot(a1 < T && p1 <= x));
  const int lo = below > 0 ? below - 1 : 0;  // largest position whose prefix cost is <= x
  const int off_lo = l_off[lo];
  const double w = kRowCost + double(beta) * (l_off[lo + 1] - off_lo);
  double r = floor((x - double(rows) * (double(kRowCost) * lo + double(beta) * off_lo)) / w);
  r = r < 0 ? 0 : (r > rows ? rows : r);
  return uniform(lo * rows + int(r));
}

// The state is READ before the workgroup arrives at the grid barrier (balance_load) and evaluated after
// (balance_shares): no workgroup can pass that barrier, let alone reach the end of the kernel where it
// writes its new rate, before every workgroup has arrived, so all of them read the same values.
struct BalanceIn {
  float w[4], r[4];  // lane l holds workgroups 4 l .. 4 l + 3
};
__device__ __forceinline__ BalanceIn balance_load(uint32_t* ctrl, uint32_t parity, int G, int lane) {
  const float* const st = reinterpret_cast<const float*>(ctrl + kBalBase);
  const float* const w_old = st + (parity & 1u) * kBalMaxWg;
  const float* const rate = st + 2 * kBalMaxWg;
  BalanceIn in;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int b = lane * 4 + j;
    in.w[j] = b < G ? __hip_atomic_load(w_old + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
    in.r[j] = b < G ? __hip_atomic_load(rate + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
  }
  return in;
}

// Executed by ONE wavefront: new weights from the state and the rates of the previous call, their
// cumulative shares -> l_frac[0..G] (l_frac[0] = 0, l_frac[G] = 1).  write_back: store the new state.
__device__ __forceinline__ void balance_shares(uint32_t* ctrl, uint32_t parity, int G, bool write_back, float* l_frac,
                                               int lane, const BalanceIn in) {
  float* const st = reinterpret_cast<float*>(ctrl + kBalBase);
  float* const w_new = st + ((parity & 1u) ^ 1u) * kBalMaxWg;
  float w[4], r[4];
  float sum_r = 0.f, n_r = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    w[j] = in.w[j];
    r[j] = in.r[j];
    if (!(w[j] > 0.5f && w[j] < 2.f)) w[j] = 1.f;  // fresh (zeroed) or damaged state
    if (!(r[j] > 0.f && r[j] < 1e30f)) r[j] = 0.f;  // no measurement
    sum_r += r[j];
    n_r += r[j] > 0.f ? 1.f : 0.f;
  }
  sum_r = wave_sum_f32(sum_r);
  n_r = wave_sum_f32(n_r);
  const float mean = n_r > 0.f ? sum_r / n_r : 1.f;
  float local = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int b = lane * 4 + j;
    if (r[j] > 0.f) {
      float rel = r[j] / mean;  // this workgroup's speed relative to the average of the last call
      rel = rel < 0.8f ? 0.8f : (rel > 1.25f ? 1.25f : rel);
      // the measured speed was obtained WITH the old weight's share, so it estimates the speed itself.
      // A slow average: most of a call's deviation is that call's own (routing pattern, memory
      // system), and a weight that chases it adds noise to the next call's shares (a quarter per
      // call instead of a twentieth was 0.3 us slower with rotating token batches)
      w[j] = 0.95f * w[j] + 0.05f * rel;
      w[j] = w[j] < 0.7f ? 0.7f : (w[j] > 1.4f ? 1.4f : w[j]);
    }
    if (b >= G) w[j] = 0.f;
    if (write_back && b < G) __hip_atomic_store(w_new + b, w[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    local += w[j];
  }
  float incl = local;  // inclusive scan of the lanes' sums
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const float v = __shfl_up(incl, off, 64);
    if (lane >= off) incl += v;
  }
  const float total = __shfl(incl, 63, 64);
  float run = incl - local;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int b = lane * 4 + j;
    if (b < G) l_frac[b] = run / total;
    run += w[j];
  }
  if (lane == 0) l_frac[G] = 1.f;
}

// A workgroup whose experts' pairs exceed the vectors its LDS holds (cap) walks them in pieces.  The
// piece that starts at pair c0 ends at a boundary between experts whenever one lies within reach:
// the rows of an expert are then streamed for one piece only (fused_stage hands out no tiles for a
// segment without pairs in the piece); only a single expert with more than cap pairs has its rows
// streamed once per piece.  e1 <= e2: ends of the first and second expert in the pair list [0, nvec).
__device__ __forceinline__ int piece_end(int c0, int nvec, int cap, int e1, int e2) {
  int c1 = c0 + cap < nvec ? c0 + cap : nvec;
  if (c1 < nvec) {
    if (e2 > c0 && e2 <= c1)
      c1 = e2;
    else if (e1 > c0 && e1 <= c1)
      c1 = e1;
  }
  return c1;
}

// One mat-vec stage of the fused kernel.  Same tile loop as expert_stream_kernel; the routing
// metadata comes from LDS, and `mid` runs once the first two weight tiles are in flight (it holds
// the wait for the hidden vectors and their staging for the down stage).  Every workgroup calls mid.
// The first n_defer wavefronts request their tiles only after mid (see below).
//
// The workgroup's rows [R0,R1) are cut into tiles that the wavefronts TAKE one at a time from a
// counter in LDS (l_next, zero on entry) instead of owning fixed shares: measured with fixed shares,
// the four wavefronts that start second on their SIMDs stream about 15 % slower than the first four,
// and the workgroup waited for them.  Only a wavefront's first two tiles are fixed.
// Results are collected in an LDS buffer and written out after the last tile: a store or atomic
// issued between the weight loads would have to complete (the memory counter retires in order)
// before the NEXT tile's data counts as arrived.  If they do not fit (many rows of a very popular
// expert) they are written directly instead.
// The pairs of the workgroup's experts are numbered 0..nvec-1 in the grouped order; only those in
// [c0, c1) are processed (their vectors are what l_vec holds, in that order), which lets a caller with
// little LDS walk a long pair list in pieces.  GATHER: see token_step.
template <typename WT, int STAGE, int LPR, int NCH, int RG, bool GATHER = false, typename Mid>
__device__ __forceinline__ void fused_stage(const WT* wa, const WT* wb, WT* h_out, float* out, int rows, int L,
                                            int R0, int R1, int N, int pairs_max, int cap_vec, const int* l_active,
                                            const int* l_off, const int* l_tok, const float* l_gw,
                                            const uint4* l_vec, float* ebuf, int ecap, uint32_t* l_next, Mid mid,
                                            int c0 = 0, int c1 = 0x7fffffff, int n_defer = 0) {
  constexpr int EPL = 16 / int(sizeof(WT));
  constexpr int R = 64 / LPR;
  constexpr int NM = STAGE == 0 ? 2 : 1;
  constexpr int TROWS = RG * R;
  const int tid = threadIdx.x, lane = tid & 63;
  const int lsub = lane % LPR, lrow = lane / LPR;
  const int L16 = L / EPL;

  bool wg_has = R0 < R1;
  const int a0 = wg_has ? R0 / rows : 0;
  const int nseg = wg_has ? (R1 - 1) / rows - a0 + 1 : 0;
  const int e0 = uniform(l_active[a0]);
  const int e1 = nseg > 1 ? uniform(l_active[a0 + 1]) : 0;
  const int e2 = nseg > 2 ? uniform(l_active[a0 + 2]) : 0;
  // never true for a routing computed by this kernel; keeps every access in bounds regardless
  if (nseg > kMaxSeg || (unsigned)e0 >= (unsigned)N || (unsigned)e1 >= (unsigned)N || (unsigned)e2 >= (unsigned)N)
    wg_has = false;
  const int lo = R0, hi = wg_has ? R1 : R0;

  // pair lists of this workgroup's experts
  const int off0 = uniform(l_off[a0]);
  const int off1 = uniform(l_off[a0 + 1]);
  const int off2 = nseg > 1 ? uniform(l_off[a0 + 2]) : off1;
  const int off3 = nseg > 2 ? uniform(l_off[a0 + 3]) : off2;
  const int nvec = off3 - off0;
  if (off0 < 0 || off1 < off0 || off2 < off1 || off3 < off2 || off0 + nvec > pairs_max) wg_has = false;  // never true
  // pairs of each segment inside [c0, c1)
  const int q0 = c0 < 0 ? 0 : c0, q1 = c1 < nvec ? c1 : nvec;
  auto clip = [&](int from, int to) __attribute__((always_inline)) {  // pairs [from,to) of the list, cut to [q0,q1)
    const int a = from > q0 ? from : q0, b = to < q1 ? to : q1;
    return b > a ? b - a : 0;
  };
  const int n0 = clip(0, off1 - off0), n1 = clip(off1 - off0, off2 - off0), n2 = clip(off2 - off0, off3 - off0);
  if (n0 + n1 + n2 > cap_vec) wg_has = false;  // the caller staged at most cap_vec vectors
  const int base = wg_has ? off0 + q0 : 0;     // first pair of the piece
  const int hi_w = wg_has ? hi : lo;
  const SegView sv{rows, a0, e0, e1, e2, n0, n1, n2, hi_w, lo};
  const int* const s_tok = l_tok + base;
  const float* const s_gw = l_gw + base;
  const int n_res = result_entries(sv);
  const bool use_buf = n_res <= ecap * kFfnWaves;

  // tile i of the workgroup: the tiles of segment 0, then of segment 1, ...; none crosses an expert boundary.
  // A segment none of whose pairs belongs to this piece has no tiles: its rows are not streamed.
  const int nt0 = n0 > 0 ? (seg_n(sv, 0) + TROWS - 1) / TROWS : 0;
  const int nt1 = n1 > 0 ? (seg_n(sv, 1) + TROWS - 1) / TROWS : 0;
  const int nt2 = n2 > 0 ? (seg_n(sv, 2) + TROWS - 1) / TROWS : 0;
  // The wavefronts that start right away take their first two tiles by number (tile w, then tile
  // nw + w): with few tiles everybody gets one before anybody gets two.  The counter hands out the
  // tiles behind those (i < 0: the next tile from the counter).
  const int wave = uniform(tid >> 6);
  const bool deferred = wave < n_defer;  // see below
  const int nw = kFfnWaves - n_defer;
  auto take_tile = [&](int& r, int& n, int i = -1) __attribute__((always_inline)) {
    if (i < 0) {
      if (lane == 0) i = 2 * nw + int(atomicAdd(l_next, 1u));
      i = uniform(i);
    }
    const int sgm = i < nt0 ? 0 : (i < nt0 + nt1 ? 1 : 2);
    const int j = i - (sgm > 0 ? nt0 : 0) - (sgm > 1 ? nt1 : 0);
    r = seg_lo(sv, sgm) + j * TROWS;
    n = i < nt0 + nt1 + nt2 ? tile_rows(sv, r, TROWS) : 0;
    if (n <= 0) r = lo;
  };

  uint4 wA[NM][RG][NCH], wB[NM][RG][NCH];
  int rA = lo, nA = 0, rB = lo, nB = 0;
  // The first n_defer wavefronts request nothing before mid: what they load IN mid (polled counters,
  // staged vectors) then does not queue behind two weight tiles (loads return in issue order).
  if (wg_has && !deferred) {  // a wavefront that finds no tile requests a placeholder
    take_tile(rA, nA, wave - n_defer);
    take_tile(rB, nB, nw + wave - n_defer);
    load_tile<WT, NM, LPR, NCH, RG, true>(wA, wa, wb, rows, L, lsub, lrow, tile_ref(sv, rA), nA);
    load_tile<WT, NM, LPR, NCH, RG, true>(wB, wa, wb, rows, L, lsub, lrow, tile_ref(sv, rB), nB);
  }
  __builtin_amdgcn_sched_barrier(0);  // the requests above are issued before anything in mid

  mid(a0, wg_has ? nseg : 0);

  if (wg_has && deferred) {
    take_tile(rA, nA);
    take_tile(rB, nB);
    load_tile<WT, NM, LPR, NCH, RG, true>(wA, wa, wb, rows, L, lsub, lrow, tile_ref(sv, rA), nA);
    load_tile<WT, NM, LPR, NCH, RG, true>(wB, wa, wb, rows, L, lsub, lrow, tile_ref(sv, rB), nB);
  }

  if (wg_has && nA > 0) {
    while (true) {
      compute_tile<WT, STAGE, NM, LPR, NCH, RG, true, true, true, GATHER>(wA, s_tok, s_gw, l_vec, h_out, out, rows, L16, base,
                                                                  lsub, lrow, tile_ref_buffered(sv, rA), nA, ebuf, use_buf);
      take_tile(rA, nA);
      load_tile<WT, NM, LPR, NCH, RG, true>(wA, wa, wb, rows, L, lsub, lrow, tile_ref(sv, rA), nA);
      if (nB <= 0) break;
      compute_tile<WT, STAGE, NM, LPR, NCH, RG, true, true, true, GATHER>(wB, s_tok, s_gw, l_vec, h_out, out, rows, L16, base,
                                                                  lsub, lrow, tile_ref_buffered(sv, rB), nB, ebuf, use_buf);
      take_tile(rB, nB);
      load_tile<WT, NM, LPR, NCH, RG, true>(wB, wa, wb, rows, L, lsub, lrow, tile_ref(sv, rB), nB);
      if (nA <= 0) break;
    }
  }
  __syncthreads();  // every wavefront's results are in the buffer
  if (wg_has && use_buf) flush_results<WT, STAGE>(sv, ebuf, s_tok, s_gw, h_out, out, base, tid);
}

// Layout of the per-expert completion words in the control area: the counter of the expert at
// position a of the active list sits on a 128-byte line of its own (same-line atomics and polls
// from many workgroups serialise badly).
constexpr int kDoneBase = 1024;  // first word
constexpr int kDoneStride = 32;  // words between experts
__device__ __forceinline__ uint32_t* done_count(uint32_t* ctrl, int a) { return ctrl + kDoneBase + a * kDoneStride; }

// After the gate/up stage: tell the down stage which hidden vectors are complete.  Called by the whole
// workgroup; every wavefront first drains its h stores.  Thread 0 adds the rows this workgroup
// produced to the counter of each expert it touched; an expert is complete when its counter has
// reached `rows` hidden units, which is what the consumers poll for.  (A separate flag raised by the
// arrival that completes an expert cost that arrival a second trip to memory: about 1 us per layer.)
// (Signalling only after the down stage's first tiles are requested, with the h stores completing
// underneath, was measured slower: early finishers then compete with the gate/up stragglers that
// everyone waits for.)
__device__ __forceinline__ void signal_hidden_done(uint32_t* ctrl, int R0, int R1, int rows) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x != 0) return;
  if (R0 >= R1) return;
  const int a0 = R0 / rows, a1 = (R1 - 1) / rows;
#pragma unroll
  for (int sgm = 0; sgm < kMaxSeg; ++sgm) {
    const int a = a0 + sgm;
    if (a <= a1) {
      const int lo = R0 > a * rows ? R0 : a * rows;
      const int hi = R1 < (a + 1) * rows ? R1 : (a + 1) * rows;
      // no value comes back: the thread does not wait for the counter's round trip
      __hip_atomic_fetch_add(done_count(ctrl, a), uint32_t(hi - lo), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// d == LPR0*EPL*NCH0 and I == LPR1*EPL*NCH1 exactly; N <= 64*NV; B <= 32; k <= 16.
// GEN: the routing is the general OEA (Algorithm 2) instead of Algorithm 1; an instantiation of its
// own, so that the code of the default kernel does not depend on it (as a run-time branch it
// changed the register allocation of the stages and cost the default path 0.4 us).
template <typename WT, int LPR0, int NCH0, int LPR1, int NCH1, int NV, bool GEN = false>
__global__ __launch_bounds__(kFfnThreads) void moe_fused_kernel(FusedParams p) {
  extern __shared__ uint4 lds4[];
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  constexpr int EPL = 16 / int(sizeof(WT));
  const int B = p.B, d = p.d, N = p.N, I = p.I, k = p.k;
  const int P = B * k;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int G = gridDim.x, wg = blockIdx.x;
  const WT* const x = static_cast<const WT*>(p.x);

  // ---- LDS: [dump 16 B][routing scratch][routing result][vectors: x (phases R,A) then h (phase B)]
  uint32_t* const l_route = reinterpret_cast<uint32_t*>(lds4 + 1);
  int* const l_idx = reinterpret_cast<int*>(l_route + route_lds_words(B, N));
  float* const l_gatew = reinterpret_cast<float*>(l_idx + P);
  int* const l_nsel = reinterpret_cast<int*>(l_gatew + P);
  int* const l_active = l_nsel + B;
  int* const l_nact = l_active + N;
  int* const l_off = l_nact + 4;
  int* const l_tok = l_off + N + 4;
  float* const l_gw = reinterpret_cast<float*>(l_tok + P);
  float* const l_frac = l_gw + P;  // [G+1] cumulative cost shares of the workgroups
  uint4* const l_vec = lds4 + 1 + fused_meta_words(B, N, k) / 4;

  OEA_TL(0);
  // every thread reads the same word (one request per wavefront); tested before the grid barrier
  const uint32_t magic = __hip_atomic_load(p.ctrl + kCtrlMagicWord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  uint32_t gen0 = 0;  // thread 0: barrier generation at the start of this call
  if (tid == 0 || tid == 64) gen0 = grid_generation(p.ctrl);  // thread 64: parity of the call for the speed weights
  const bool balanced = G <= kBalMaxWg;
  BalanceIn bal_in{};
  if (balanced && wave == 1) bal_in = balance_load(p.ctrl, uint32_t(__builtin_amdgcn_readfirstlane(int(gen0))), G, lane);
  // ---- phase R1.  x of the batch -> LDS: loads first, written after the logits
  const int d16 = d / EPL;
  const int n16_x = B * d16;
  // the operands of this wavefront's (first) logit are requested first: loads return in issue
  // order, and the logits are what the other workgroups wait for
  constexpr int XC = LPR0 * NCH0 / 64;  // 16-byte chunks of a row per lane (d == LPR0 * EPL * NCH0)
  const WT* const wr = static_cast<const WT*>(p.w_router);
  const int idx0 = wg * kFfnWaves + wave;
  const bool has0 = idx0 < B * N;
  uint4 la[XC], lb[XC];
  {
    const int ii = has0 ? idx0 : 0;
    const int t = ii / N, e = ii - t * N;
#pragma unroll
    for (int c = 0; c < XC; ++c) {
      la[c] = *reinterpret_cast<const uint4*>(x + (size_t)t * d + (lane + 64 * c) * EPL);
      lb[c] = *reinterpret_cast<const uint4*>(wr + (size_t)e * d + (lane + 64 * c) * EPL);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  u32x4 stg[kFusedStage];
  {
    const u32x4* src = reinterpret_cast<const u32x4*>(x);
#pragma unroll
    for (int j = 0; j < kFusedStage; ++j) {
      const int i = j * kFfnThreads + tid;
      stg[j] = src[i < n16_x ? i : n16_x - 1];
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  {  // clear this workgroup's slice of out[B,d] (d is a multiple of 8: float4 granules)
    // written through to memory: phase B adds to these words with device-scope atomics from every XCD
    const int total = p.acc_rows * d;
    const int per = (total + G - 1) / G;
    const int lo = per * wg, hi = lo + per < total ? lo + per : total;
    for (int i = lo + tid; i < hi; i += kFfnThreads)
      __hip_atomic_store(p.acc + i, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // per-expert completion counters of the gate/up stage: cleared here, before the first grid barrier
  if (wg == 0 && tid < N) {
    __hip_atomic_store(done_count(p.ctrl, tid), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // router logits: one (token, expert) dot product per wavefront, fp64 accumulation, one rounding
  {
    if (has0) {
      double acc = 0.0;
#pragma unroll
      for (int c = 0; c < XC; ++c) acc = frag_dot_f64<WT>(la[c], lb[c], acc);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
      if (lane == 0) {
        if (p.bias) acc += double(p.bias[idx0 % N]);
        __hip_atomic_store(p.logits + idx0, float(acc), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    for (int idx = idx0 + G * kFfnWaves; idx < B * N; idx += G * kFfnWaves) {
      const int t = idx / N, e = idx - t * N;
      const WT* xr = x + (size_t)t * d;
      const WT* wre = wr + (size_t)e * d;
      double acc = 0.0;
      for (int c = lane * EPL; c < d; c += 64 * EPL) {
        uint4 a = *reinterpret_cast<const uint4*>(xr + c);
        uint4 b = *reinterpret_cast<const uint4*>(wre + c);
        acc = frag_dot_f64<WT>(a, b, acc);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
      if (lane == 0) {
        if (p.bias) acc += double(p.bias[e]);
        __hip_atomic_store(p.logits + idx, float(acc), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }

#pragma unroll
  for (int j = 0; j < kFusedStage; ++j) {
    const int i16 = j * kFfnThreads + tid;
    *reinterpret_cast<u32x4*>(i16 < n16_x ? l_vec + i16 : lds4) = stg[j];
  }
  for (int base = kFusedStage * kFfnThreads; base < n16_x; base += kFusedStage * kFfnThreads) {  // larger x
    const u32x4* src = reinterpret_cast<const u32x4*>(x);
#pragma unroll
    for (int j = 0; j < kFusedStage; ++j) {
      const int i16 = base + j * kFfnThreads + tid;
      stg[j] = src[i16 < n16_x ? i16 : n16_x - 1];
    }
#pragma unroll
    for (int j = 0; j < kFusedStage; ++j) {
      const int i16 = base + j * kFfnThreads + tid;
      *reinterpret_cast<u32x4*>(i16 < n16_x ? l_vec + i16 : lds4) = stg[j];
    }
  }

  OEA_TL(1);
  // A workspace that oea_workspace_init has not prepared holds arbitrary barrier words: nobody
  // arrives, nobody waits, the kernel ends here in every workgroup (they all read the same word).
  if (magic != kWsMagic) return;
  grid_arrive(p.ctrl, gen0 + 1);  // logits and cleared out words are in memory
  if (balanced && wave == 1)  // while thread 0 waits at the barrier
    balance_shares(p.ctrl, uint32_t(__builtin_amdgcn_readfirstlane(int(gen0))), G, wg == 0, l_frac, lane, bal_in);
  grid_wait(p.ctrl, gen0 + 1, p.spin_limit);
  OEA_TL(2);

  // ---- phase R2: routing, replicated per workgroup, result in LDS.  Every row of 16 lanes reads
  // its token's logits straight from memory (device-coherent loads: written by other workgroups).
  if (tid == 0) l_nact[1] = l_nact[2] = 0;  // tile counters of the two stages (a barrier follows in the routing)
  // (the positions of the pairs in the grouped order go straight to memory, from workgroup 0 only)
  const RouteOut lo{l_idx, l_gatew, l_nsel, l_active, l_nact, l_off, l_tok, l_gw, wg == 0 ? p.ro.grp_pos : nullptr};
  uint32_t* const ctrl = p.ctrl;
  const float* const frac = balanced ? l_frac : nullptr;
  uint32_t* const l_cut = l_route + 48;  // [4] inside the routing scratch's block-scan words, unused at N <= 128
  {
    // The four cut points of this workgroup (both ends, both stages) need only the CSR offsets: the
    // last four wavefronts compute one each while the rows' lanes write the pair lists.
    auto cuts = [&]() {
      if (wave >= kFfnWaves - 4) {
        const int q = wave - (kFfnWaves - 4);
        int T_ = uniform(l_nact[0]);
        T_ = T_ < 0 ? 0 : (T_ > N ? N : T_);
        const int cut = wg_first_row(l_off, T_, q < 2 ? I : d, q < 2 ? kBetaUp : kBetaDown, wg + (q & 1), G, lane, frac);
        if (lane == 0) l_cut[q] = uint32_t(cut);
      }
    };
    if constexpr (GEN) {  // Algorithm 2: top-p cut of the baseline, rank window; k is k_max
      route_rows_general<4 * NV, kFfnThreads, true>(p.logits, p.token_mask, B, N, p.k0,
                                                    RouteGeneral{p.gen_p, k, p.gen_max_p, nullptr}, lo, l_route, cuts);
    } else {
      RowCarry<4 * NV> carry;  // one DPP row of 16 lanes per token, 4 * NV keys per lane
      route_union_rows<4 * NV, kFfnThreads, true>(p.logits, p.token_mask, B, N, p.k0, lo, l_route, carry);
      route_fill_rows<4 * NV, kFfnThreads>(B, N, k, p.k0, lo, l_route, carry, cuts);
    }
  }
  __syncthreads();
  if (wg == 0) {  // publish the routing result
    for (int i = tid; i < P; i += kFfnThreads) {
      p.ro.expert_idx[i] = l_idx[i];
      p.ro.gate_w[i] = l_gatew[i];
    }
    for (int i = tid; i < B; i += kFfnThreads) p.ro.n_sel[i] = l_nsel[i];
    for (int i = tid; i < N; i += kFfnThreads) p.ro.active_list[i] = l_active[i];
    if (tid == 0) *p.ro.n_active = l_nact[0];
  }
  int T = uniform(l_nact[0]);
  T = T < 0 ? 0 : (T > N ? N : T);
  const int RA0 = uniform(int(l_cut[0])), RA1 = uniform(int(l_cut[1]));
  const int RB0 = uniform(int(l_cut[2])), RB1 = uniform(int(l_cut[3]));
  const unsigned long long tA0 = wall_clock64();
  OEA_TL(7);
  OEA_TL_VAL(16, RA0);
  OEA_TL_VAL(17, RA1);
  OEA_TL_VAL(18, RB0);
  OEA_TL_VAL(19, RB1);

  // ---- phase A: gate/up
  fused_stage<WT, 0, LPR0, NCH0, 1>(static_cast<const WT*>(p.w_gate), static_cast<const WT*>(p.w_up),
                                    static_cast<WT*>(p.h), p.out, I, d, RA0, RA1, N, P, p.cap_vec, l_active, l_off,
                                    l_tok, l_gw, l_vec, reinterpret_cast<float*>(l_vec + (size_t)B * d16), p.ecap0,
                                    reinterpret_cast<uint32_t*>(l_nact + 1), [](int, int) {});
  const unsigned long long tA1 = wall_clock64();
  OEA_TL(8);
  signal_hidden_done(p.ctrl, RA0, RA1, I);
  OEA_TL(9);
  // Row of p.acc a pair adds into: its token, or with one row per pair the pair itself (the list of
  // selected experts in LDS has been published and is not read any more: it becomes that identity)
  const bool per_pair = p.acc_rows != B;
  if (per_pair)
    for (int i = tid; i < P; i += kFfnThreads) l_idx[i] = i;  // ordered before its use by the barriers in mid_b
  const int* const l_rowof = per_pair ? l_idx : l_tok;
  // ---- phase B: down.  mid = barrier (h complete everywhere), then this workgroup's h rows -> LDS
  const WT* const hsrc = static_cast<const WT*>(p.h);
  const int I16 = I / EPL;
  const uint32_t spin_limit = p.spin_limit;
  const int cap_vec = p.cap_vec;
  unsigned long long tB0 = 0;
  const int n_defer = 2 * T <= N ? kStageWaves : 1;
  auto mid_b = [&](int a0, int nseg) {  // runs once the first weight tiles are requested
        OEA_TL(10);
        // No grid barrier here: this workgroup only needs the hidden vectors of ITS experts, which
        // its neighbours produce (both stages cut the expert list in about the same proportions).
        // Wait, bounded, until the counter of each of them says complete.
        if (tid == 0) {
          uint32_t spins = 0;
          for (int sgm = 0; sgm < nseg; ++sgm)
            while (__hip_atomic_load(done_count(ctrl, a0 + sgm), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < uint32_t(I)) {
              __builtin_amdgcn_s_sleep(2);
              if (++spins > spin_limit) {
                atomicExch(ctrl + kCtrlErrWord, 1u);
                break;
              }
            }
        }
        __syncthreads();
        OEA_TL(11);
        const int off0 = uniform(l_off[a0]);
        int nvec = uniform(l_off[a0 + nseg]) - off0;
        if (off0 < 0 || nvec < 0 || nvec > cap_vec || off0 + nvec > P) nvec = 0;  // never true; bounds the copy
        // h was written by other workgroups (other XCDs): device-coherent 16-byte loads, which
        // exist as buffer loads with the sc0 sc1 bits; the descriptor also bounds the access
        const int n16 = nvec * I16;
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<WT*>(hsrc + (size_t)off0 * I), 0, n16 * 16, 0x00020000);
        // staged by the wavefronts that have no weight tiles in flight, unless that would take them
        // more than two rounds of loads (many pairs): then by everybody
        const int kStagers = n16 <= 2 * kFusedStage * n_defer * 64 ? n_defer * 64 : kFfnThreads;
        if (tid < kStagers)
          for (int base = 0; base < n16; base += kFusedStage * kStagers) {
            u32x4 t4[kFusedStage];
#pragma unroll
            for (int j = 0; j < kFusedStage; ++j) {
              const int i16 = base + j * kStagers + tid;
              t4[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (i16 < n16 ? i16 : n16 - 1) * 16, 0, 1 | 16);
            }
#pragma unroll
            for (int j = 0; j < kFusedStage; ++j) {
              const int i16 = base + j * kStagers + tid;
              *reinterpret_cast<u32x4*>(i16 < n16 ? l_vec + i16 : lds4) = t4[j];
            }
          }
        __syncthreads();
        OEA_TL(12);
        tB0 = wall_clock64();
      };
  fused_stage<WT, 1, LPR1, NCH1, 2>(
      static_cast<const WT*>(p.w_down), static_cast<const WT*>(nullptr), static_cast<WT*>(nullptr), p.acc, d, I, RB0,
      RB1, N, P, p.cap_vec, l_active, l_off, l_rowof, l_gw, l_vec,
      reinterpret_cast<float*>(l_vec + (size_t)cap_vec * I16), p.ecap1, reinterpret_cast<uint32_t*>(l_nact + 2), mid_b,
      0, 0x7fffffff, n_defer);
  if (balanced && tid == 0) {  // this workgroup's speed in this call: cost share per clock tick of streaming
    const unsigned long long tB1 = wall_clock64();
    const float ticks = float((tA1 - tA0) + (tB1 - tB0));
    const float share = l_frac[wg + 1] - l_frac[wg];
    const bool measured = RA1 - RA0 >= 16 && RB1 - RB0 >= 64 && tB0 != 0 && ticks > 100.f && share > 0.f;
    __hip_atomic_store(reinterpret_cast<float*>(ctrl + kBalBase) + 2 * kBalMaxWg + wg, measured ? share / ticks : 0.f,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  OEA_TL(13);
  OEA_TL_DRAINED(14);
}

// ---------------------------------------------------------------------------------------------
// The same single-kernel layer for larger batches (32 < B <= 128), where x of the whole batch no
// longer fits in LDS: a workgroup stages only the vectors of ITS experts' pairs (gathered rows of x
// for the gate/up stage, rows of h for the down stage) and, should they exceed its LDS share, walks
// them in pieces (streaming its weight rows once per piece).  The routing takes the tokens in groups
// of 32 (four per wavefront).
template <typename WT, int LPR0, int NCH0, int LPR1, int NCH1, int NV, bool GEN = false>
__global__ __launch_bounds__(kFfnThreads) void moe_fused_gather_kernel(FusedParams p) {
  extern __shared__ uint4 lds4[];
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  constexpr int EPL = 16 / int(sizeof(WT));
  const int B = p.B, d = p.d, N = p.N, I = p.I, k = p.k;
  const int P = B * k;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uniform(tid >> 6);
  const int G = gridDim.x, wg = blockIdx.x;
  const WT* const x = static_cast<const WT*>(p.x);
  uint32_t* const ctrl = p.ctrl;

  uint32_t* const l_route = reinterpret_cast<uint32_t*>(lds4 + 1);
  int* const l_idx = reinterpret_cast<int*>(l_route + route_lds_words(B, N));
  float* const l_gatew = reinterpret_cast<float*>(l_idx + P);
  int* const l_nsel = reinterpret_cast<int*>(l_gatew + P);
  int* const l_active = l_nsel + B;
  int* const l_nact = l_active + N;
  int* const l_off = l_nact + 4;
  int* const l_tok = l_off + N + 4;
  float* const l_gw = reinterpret_cast<float*>(l_tok + P);
  float* const l_frac = l_gw + P;
  uint4* const l_vec = lds4 + 1 + fused_meta_words(B, N, k) / 4;
  const int d16 = d / EPL, I16 = I / EPL;

  OEA_TL(0);
  const uint32_t magic = __hip_atomic_load(ctrl + kCtrlMagicWord, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  uint32_t gen0 = 0;
  if (tid == 0 || tid == 64) gen0 = grid_generation(ctrl);
  const bool balanced = G <= kBalMaxWg;
  BalanceIn bal_in{};
  if (balanced && wave == 1) bal_in = balance_load(ctrl, uint32_t(__builtin_amdgcn_readfirstlane(int(gen0))), G, lane);
  {  // clear this workgroup's slice of out[B,d]
    const int total = p.acc_rows * d;
    const int per = (total + G - 1) / G;
    const int lo = per * wg, hi = lo + per < total ? lo + per : total;
    for (int i = lo + tid; i < hi; i += kFfnThreads)
      __hip_atomic_store(p.acc + i, 0.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (wg == 0 && tid < N) {
    __hip_atomic_store(done_count(ctrl, tid), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  {  // router logits: a wavefront takes one expert and four tokens at a time (the router row chunk is
     // loaded once for the four, their loads and reductions overlap)
    constexpr int TB = 4;
    const WT* const wr = static_cast<const WT*>(p.w_router);
    const int nblk = (B + TB - 1) / TB;
    for (int u = wg * kFfnWaves + wave; u < N * nblk; u += G * kFfnWaves) {
      const int e = u / nblk, t0 = (u - e * nblk) * TB;
      const WT* wre = wr + (size_t)e * d;
      double acc[TB];
#pragma unroll
      for (int i = 0; i < TB; ++i) acc[i] = 0.0;
      for (int c = lane * EPL; c < d; c += 64 * EPL) {
        const uint4 b = *reinterpret_cast<const uint4*>(wre + c);
        uint4 a[TB];
#pragma unroll
        for (int i = 0; i < TB; ++i) a[i] = *reinterpret_cast<const uint4*>(x + (size_t)(t0 + i < B ? t0 + i : B - 1) * d + c);
#pragma unroll
        for (int i = 0; i < TB; ++i) acc[i] = frag_dot_f64<WT>(a[i], b, acc[i]);
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
        for (int i = 0; i < TB; ++i) acc[i] += __shfl_xor(acc[i], off, 64);
      if (lane == 0) {
#pragma unroll
        for (int i = 0; i < TB; ++i)
          if (t0 + i < B)
            __hip_atomic_store(p.logits + (size_t)(t0 + i) * N + e, float(acc[i] + (p.bias ? double(p.bias[e]) : 0.0)),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  OEA_TL(1);
  if (magic != kWsMagic) return;  // unprepared workspace: see moe_fused_kernel
  grid_arrive(ctrl, gen0 + 1);
  if (balanced && wave == 1)
    balance_shares(ctrl, uint32_t(__builtin_amdgcn_readfirstlane(int(gen0))), G, wg == 0, l_frac, lane, bal_in);
  grid_wait(ctrl, gen0 + 1, p.spin_limit);
  OEA_TL(2);

  if (tid == 0) l_nact[1] = l_nact[2] = 0;
  // (the positions of the pairs in the grouped order go straight to memory, from workgroup 0 only)
  const RouteOut lo{l_idx, l_gatew, l_nsel, l_active, l_nact, l_off, l_tok, l_gw, wg == 0 ? p.ro.grp_pos : nullptr};
  if constexpr (GEN)  // Algorithm 2 (see moe_fused_kernel)
    route_rows_general_any<4 * NV, kFfnThreads, true>(p.logits, p.token_mask, B, N, p.k0,
                                                      RouteGeneral{p.gen_p, k, p.gen_max_p, nullptr}, lo, l_route);
  else
    route_rows_groups<4 * NV, kFfnThreads, 4, true>(p.logits, p.token_mask, B, N, k, p.k0, lo, l_route);  // B <= 128
  __syncthreads();
  if (wg == 0) {  // publish the routing result
    for (int i = tid; i < P; i += kFfnThreads) {
      p.ro.expert_idx[i] = l_idx[i];
      p.ro.gate_w[i] = l_gatew[i];
    }
    for (int i = tid; i < B; i += kFfnThreads) p.ro.n_sel[i] = l_nsel[i];
    for (int i = tid; i < N; i += kFfnThreads) p.ro.active_list[i] = l_active[i];
    if (tid == 0) *p.ro.n_active = l_nact[0];
  }
  int T = uniform(l_nact[0]);
  T = T < 0 ? 0 : (T > N ? N : T);
  const float* const frac = balanced ? l_frac : nullptr;
  // the four cut points of this workgroup (both ends, both stages): one wavefront each, shared through
  // the routing scratch, which nothing reads any more
  if (wave < 4) {
    const int cut = wg_first_row(l_off, T, wave < 2 ? I : d, wave < 2 ? kBetaUp : kBetaDown, wg + (wave & 1), G, lane,
                                 frac);
    if (lane == 0) l_route[wave] = uint32_t(cut);
  }
  __syncthreads();
  const int RA0 = uniform(int(l_route[0])), RA1 = uniform(int(l_route[1]));
  const int RB0 = uniform(int(l_route[2])), RB1 = uniform(int(l_route[3]));

  // pairs of the experts a row range touches: [first pair, count)
  // ... and where the first and the second expert end in that list (for piece_end)
  auto pairs_of = [&](int R0, int R1, int rows, int& off0, int& nvec, int& e1, int& e2) __attribute__((always_inline)) {
    off0 = 0;
    nvec = e1 = e2 = 0;
    if (R0 >= R1) return;
    const int a0 = R0 / rows, a1 = (R1 - 1) / rows;
    off0 = uniform(l_off[a0]);
    nvec = uniform(l_off[a1 + 1]) - off0;
    if (off0 < 0 || nvec < 0 || off0 + nvec > P) nvec = 0;  // never true for a valid routing
    e1 = uniform(l_off[a0 + 1]) - off0;
    e2 = a1 > a0 ? uniform(l_off[a0 + 2]) - off0 : nvec;
    e1 = e1 < 0 ? 0 : (e1 > nvec ? nvec : e1);
    e2 = e2 < e1 ? e1 : (e2 > nvec ? nvec : e2);
  };
  const unsigned long long tA0 = wall_clock64();
  OEA_TL(7);
  OEA_TL_VAL(16, RA0);
  OEA_TL_VAL(17, RA1);
  OEA_TL_VAL(18, RB0);
  OEA_TL_VAL(19, RB1);

  // ---- phase A: gate/up, in pieces of at most cap0 pairs
  {
    int off0, nvec, end1, end2;
    pairs_of(RA0, RA1, I, off0, nvec, end1, end2);
    const int cap0 = p.cap_vec;
    float* const ebuf = reinterpret_cast<float*>(l_vec + (size_t)cap0 * d16);
    int c0 = 0, c1 = 0;
    do {  // at least once: a workgroup without rows still takes part in the barriers inside
      c1 = piece_end(c0, nvec, cap0, end1, end2);
      if (c0 > 0) {  // the previous piece is flushed; hand the tiles out again
        __syncthreads();
        if (tid == 0) l_nact[1] = 0;
        __syncthreads();
      }
      fused_stage<WT, 0, LPR0, NCH0, 1, true>(
          static_cast<const WT*>(p.w_gate), static_cast<const WT*>(p.w_up), static_cast<WT*>(p.h), p.out, I, d, RA0,
          RA1, N, P, cap0, l_active, l_off, l_tok, l_gw, l_vec, ebuf, p.ecap0, reinterpret_cast<uint32_t*>(l_nact + 1),
          [&](int, int) {  // runs once the first weight tiles are requested: x rows of the piece's pairs -> LDS
            const u32x4* src = reinterpret_cast<const u32x4*>(x);
            const int n16 = (c1 - c0) * d16;
            for (int base = 0; base < n16; base += kFusedStage * kFfnThreads) {
              u32x4 t4[kFusedStage];
#pragma unroll
              for (int j = 0; j < kFusedStage; ++j) {
                int i16 = base + j * kFfnThreads + tid;
                i16 = i16 < n16 ? i16 : n16 - 1;
                const int v = i16 / d16, c = i16 - v * d16;
                t4[j] = src[(size_t)l_tok[off0 + c0 + v] * d16 + c];
              }
#pragma unroll
              for (int j = 0; j < kFusedStage; ++j) {
                const int i16 = base + j * kFfnThreads + tid;
                *reinterpret_cast<u32x4*>(i16 < n16 ? l_vec + i16 : lds4) = t4[j];
              }
            }
            __syncthreads();
          },
          c0, c1);
      c0 = c1;
    } while (c0 < nvec);
  }
  const unsigned long long tA1 = wall_clock64();
  OEA_TL(8);
  signal_hidden_done(ctrl, RA0, RA1, I);
  OEA_TL(9);
  const bool per_pair = p.acc_rows != B;  // see moe_fused_kernel
  if (per_pair)
    for (int i = tid; i < P; i += kFfnThreads) l_idx[i] = i;
  const int* const l_rowof = per_pair ? l_idx : l_tok;

  // ---- phase B: down, in pieces of at most cap1 pairs
  unsigned long long tB0 = 0;
  {
    int off0, nvec, end1, end2;
    pairs_of(RB0, RB1, d, off0, nvec, end1, end2);
    const int cap1 = p.cap_vec1;
    float* const ebuf = reinterpret_cast<float*>(l_vec + (size_t)cap1 * I16);
    const WT* const hsrc = static_cast<const WT*>(p.h);
    const uint32_t spin_limit = p.spin_limit;
    int c0 = 0, c1 = 0;
    do {
      c1 = piece_end(c0, nvec, cap1, end1, end2);
      if (c0 > 0) {
        __syncthreads();
        if (tid == 0) l_nact[2] = 0;
        __syncthreads();
      }
      fused_stage<WT, 1, LPR1, NCH1, 2, true>(
          static_cast<const WT*>(p.w_down), static_cast<const WT*>(nullptr), static_cast<WT*>(nullptr), p.acc, d, I,
          RB0, RB1, N, P, cap1, l_active, l_off, l_rowof, l_gw, l_vec, ebuf, p.ecap1,
          reinterpret_cast<uint32_t*>(l_nact + 2),
          [&](int a0, int nseg) {
            if (c0 == 0) {  // wait, bounded, until the hidden vectors of this workgroup's experts are complete
              if (tid == 0) {
                uint32_t spins = 0;
                for (int sgm = 0; sgm < nseg; ++sgm)
                  while (__hip_atomic_load(done_count(ctrl, a0 + sgm), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < uint32_t(I)) {
                    __builtin_amdgcn_s_sleep(2);
                    if (++spins > spin_limit) {
                      atomicExch(ctrl + kCtrlErrWord, 1u);
                      break;
                    }
                  }
              }
              __syncthreads();
            }
            // h rows of the piece's pairs: written by other workgroups, device-coherent 16-byte loads
            const int n16 = (c1 - c0) * I16;
            __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<WT*>(hsrc + (size_t)(off0 + c0) * I), 0, n16 * 16, 0x00020000);
            for (int base = 0; base < n16; base += kFusedStage * kFfnThreads) {
              u32x4 t4[kFusedStage];
#pragma unroll
              for (int j = 0; j < kFusedStage; ++j) {
                const int i16 = base + j * kFfnThreads + tid;
                t4[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (i16 < n16 ? i16 : n16 - 1) * 16, 0, 1 | 16);
              }
#pragma unroll
              for (int j = 0; j < kFusedStage; ++j) {
                const int i16 = base + j * kFfnThreads + tid;
                *reinterpret_cast<u32x4*>(i16 < n16 ? l_vec + i16 : lds4) = t4[j];
              }
            }
            __syncthreads();
            if (c0 == 0) {
              tB0 = wall_clock64();
              OEA_TL(12);
            }
          },
          c0, c1);
      c0 = c1;
    } while (c0 < nvec);
  }
  if (balanced && tid == 0) {
    const unsigned long long tB1 = wall_clock64();
    const float ticks = float((tA1 - tA0) + (tB1 - tB0));
    const float share = l_frac[wg + 1] - l_frac[wg];
    const bool measured = RA1 - RA0 >= 16 && RB1 - RB0 >= 64 && tB0 != 0 && ticks > 100.f && share > 0.f;
    __hip_atomic_store(reinterpret_cast<float*>(ctrl + kBalBase) + 2 * kBalMaxWg + wg, measured ? share / ticks : 0.f,
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  OEA_TL(13);
  OEA_TL_DRAINED(14);
}

// ---------------------------------------------------------------------------------------------
// One expert stage as a kernel of its own, for batches the fused kernel does not take (B > 32):
// the routing result is read from the workspace, the work is cut by cost as above, and every
// workgroup stages only the token vectors of ITS experts' pairs (gathered rows of x for the gate/up
// stage, rows of h for the down stage).  If a workgroup's pairs exceed its LDS share it walks them
// in pieces and streams its weight rows once per piece: always correct, rarely needed.
struct StageParams {
  const void* wa;   // stage 0: W_gate; stage 1: W_down   [N, rows, L]
  const void* wb;   // stage 0: W_up
  const void* vec;  // stage 0: x [B, L]; stage 1: h [P, L]
  void* h_out;      // stage 0: h [P, rows]
  float* out;       // stage 1: out [B, rows]
  Grouping g;
  int rows, L, N, B, pairs_max;
  int cap_vec;   // vectors of length L the LDS vector area holds
  int cap_list;  // entries of the staged pair lists
  int ecap;      // floats of result buffer per wavefront
  int per_pair;  // stage 1: `out` has one row per pair (deterministic combine)
};

template <typename WT, int STAGE, int LPR, int NCH, int RG>
__global__ __launch_bounds__(kFfnThreads) void expert_stage_kernel(StageParams p) {
  extern __shared__ uint4 lds4[];
  constexpr int EPL = 16 / int(sizeof(WT));
  const int tid = threadIdx.x, lane = tid & 63;
  const int N = p.N, rows = p.rows, L = p.L;
  const int L16 = L / EPL;
  // LDS: [dump 16 B][active N][off N+4][counter 4][tok cap_list][gw cap_list][vectors][results]
  int* const l_active = reinterpret_cast<int*>(lds4 + 1);
  int* const l_off = l_active + N;
  uint32_t* const l_next = reinterpret_cast<uint32_t*>(l_off + N + 4);
  int* const l_tok = reinterpret_cast<int*>(l_next + 4);
  float* const l_gw = reinterpret_cast<float*>(l_tok + p.cap_list);
  uint4* const l_vec = lds4 + 1 + (2 * (size_t)N + 8 + 2 * (size_t)p.cap_list + 3) / 4;
  float* const ebuf = reinterpret_cast<float*>(l_vec + (size_t)p.cap_vec * L16);

  int T = *p.g.n_active;
  T = T < 0 ? 0 : (T > N ? N : T);
  for (int i = tid; i < N; i += kFfnThreads) l_active[i] = i < T ? p.g.active_list[i] : 0;
  for (int i = tid; i <= N; i += kFfnThreads) l_off[i] = p.g.grp_off[i <= T ? i : T];
  __syncthreads();
  const int beta = STAGE == 0 ? kBetaUp : kBetaDown;
  const int R0 = wg_first_row(l_off, T, rows, beta, blockIdx.x, gridDim.x, lane);
  const int R1 = wg_first_row(l_off, T, rows, beta, blockIdx.x + 1, gridDim.x, lane);
  if (R0 >= R1) return;  // uniform over the workgroup
  const int a0 = R0 / rows, a1 = (R1 - 1) / rows;
  if (a1 - a0 + 1 > kMaxSeg) return;  // excluded by the launcher's choice of grid; keeps the code below in bounds
  const int off0 = l_off[a0];
  int nvec = l_off[a1 + 1] - off0;
  if (off0 < 0 || nvec < 0 || off0 + nvec > p.pairs_max) return;  // never true after a valid routing
  if (nvec > p.cap_list) nvec = p.cap_list;  // cap_list >= kMaxSeg * B covers every valid routing
  // pair lists of this workgroup's experts; addressed by the global pair number below
  for (int i = tid; i < nvec; i += kFfnThreads) {
    const bool rowof_pair = STAGE == 1 && p.per_pair;
    const int t = rowof_pair ? off0 + i : p.g.grp_tok[off0 + i];
    const int lim = rowof_pair ? p.pairs_max : p.B;
    l_tok[i] = t < 0 ? 0 : (t >= lim ? lim - 1 : t);
    l_gw[i] = p.g.grp_gw[off0 + i];
  }
  const uint4* const vsrc = reinterpret_cast<const uint4*>(p.vec);
  int end1 = l_off[a0 + 1] - off0, end2 = a1 > a0 ? l_off[a0 + 2] - off0 : nvec;
  end1 = end1 < 0 ? 0 : (end1 > nvec ? nvec : end1);
  end2 = end2 < end1 ? end1 : (end2 > nvec ? nvec : end2);
  for (int c0 = 0, c1 = 0; c0 < nvec; c0 = c1) {
    c1 = piece_end(c0, nvec, p.cap_vec, end1, end2);
    __syncthreads();  // the lists are written; the previous piece is done with the vector area
    if (tid == 0) *l_next = 0;
    for (int i16 = tid; i16 < (c1 - c0) * L16; i16 += kFfnThreads) {
      const int v = i16 / L16, c = i16 - v * L16;
      const size_t row = STAGE == 0 ? (size_t)l_tok[c0 + v] : (size_t)(off0 + c0 + v);
      l_vec[i16] = vsrc[row * L16 + c];
    }
    __syncthreads();
    fused_stage<WT, STAGE, LPR, NCH, RG, true>(
        static_cast<const WT*>(p.wa), static_cast<const WT*>(p.wb), static_cast<WT*>(p.h_out), p.out, rows, L, R0, R1,
        N, p.pairs_max, p.cap_vec, l_active, l_off, l_tok - off0, l_gw - off0, l_vec, ebuf, p.ecap, l_next,
        [](int, int) {}, c0, c1);
  }
}

template <typename WT, int STAGE, int LPR, int NCH, int RG>
hipError_t launch_stage_one(StageParams p, int grid, hipStream_t s) {
  auto kern = expert_stage_kernel<WT, STAGE, LPR, NCH, RG>;
  // LDS plan: lists, then as many vectors as fit beside a result buffer of 1024 floats per wavefront
  p.cap_list = kMaxSeg * p.B < p.pairs_max ? kMaxSeg * p.B : p.pairs_max;
  const size_t fixed = 16 + ((2 * (size_t)p.N + 8 + 2 * (size_t)p.cap_list + 3) / 4) * 16;
  p.ecap = 1024;
  const size_t res = (size_t)p.ecap * kFfnWaves * sizeof(float);
  if (fixed + res + (size_t)p.L * sizeof(WT) > kFusedLdsMax) return hipErrorNotSupported;
  size_t cap = (kFusedLdsMax - fixed - res) / ((size_t)p.L * sizeof(WT));
  if (cap > (size_t)p.cap_list) cap = p.cap_list;
  p.cap_vec = (int)cap;
  const size_t lds = fixed + cap * p.L * sizeof(WT) + res;
  static PerDevice attr_set;
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kFusedLdsMax, attr_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kFfnThreads), lds, s, p);
  return hipGetLastError();
}


// Launch of a persistent layer kernel: one workgroup per compute unit, all resident at once.  The
// occupancy query (once per kernel and device) shows that a workgroup fits on a compute unit; that
// the compute units are FREE when the kernel starts is the caller's part (see oea.h).
// cooperative: launch through hipLaunchCooperativeKernel, with which the runtime itself guarantees
// that the whole grid is resident or refuses the launch (measured: 18 us more per launch, so it is
// an option for callers that share the device, not the default).
template <typename Kern>
hipError_t launch_persistent(Kern kern, const FusedParams& p, int grid, size_t lds_bytes, PerDevice& attr,
                             PerDevice& fits, bool cooperative, hipStream_t s) {
  int dev = 0;
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kFusedLdsMax, attr, &dev);
  if (e != hipSuccess) return e;
  int ok = fits.v[dev].load(std::memory_order_relaxed);  // 1 = a workgroup fits on a compute unit, -1 = not
  if (ok == 0) {
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kFfnThreads, kFusedLdsMax);
    if (e != hipSuccess) return e;
    ok = per_cu >= 1 ? 1 : -1;
    fits.v[dev].store(ok, std::memory_order_relaxed);
  }
  if (ok < 0) return hipErrorNotSupported;
  if (cooperative) {
    FusedParams pc = p;
    void* args[] = {&pc};
    return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(kern), dim3(grid), dim3(kFfnThreads), args,
                                      (unsigned)lds_bytes, s);
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kFfnThreads), lds_bytes, s, p);
  return hipGetLastError();
}

template <typename WT, int LPR0, int NCH0, int LPR1, int NCH1, int NV>
hipError_t launch_fused_one(const FusedParams& p, int grid, size_t lds_bytes, bool coop, hipStream_t s) {
  if (p.general) {
    static PerDevice attr_g, fits_g;
    return launch_persistent(moe_fused_kernel<WT, LPR0, NCH0, LPR1, NCH1, NV, true>, p, grid, lds_bytes, attr_g,
                             fits_g, coop, s);
  }
  static PerDevice attr, fits;
  return launch_persistent(moe_fused_kernel<WT, LPR0, NCH0, LPR1, NCH1, NV>, p, grid, lds_bytes, attr, fits, coop, s);
}

template <typename WT, int LPR0, int NCH0, int LPR1, int NCH1, int NV>
hipError_t launch_fused_gather_one(const FusedParams& p, int grid, size_t lds_bytes, bool coop, hipStream_t s) {
  if (p.general) {
    static PerDevice attr_g, fits_g;
    return launch_persistent(moe_fused_gather_kernel<WT, LPR0, NCH0, LPR1, NCH1, NV, true>, p, grid, lds_bytes,
                             attr_g, fits_g, coop, s);
  }
  static PerDevice attr, fits;
  return launch_persistent(moe_fused_gather_kernel<WT, LPR0, NCH0, LPR1, NCH1, NV>, p, grid, lds_bytes, attr, fits,
                           coop, s);
}

}  // namespace

// The fused kernel when the shape is one it is built for; hipErrorNotSupported otherwise.
hipError_t try_launch_fused(const void* x, const void* w_router, const void* w_gate, const void* w_up,
                            const void* w_down, const float* bias, const uint8_t* token_mask, float* out,
                            float* logits, void* h, RouteOut ro, uint32_t* ctrl, int B, int d, int N, int I,
                            int k, int k0, oea_dtype dt, hipStream_t s, uint32_t spin_limit, bool cooperative,
                            float* y_per_pair, const RouteGeneralArgs* general) {
  if (dt != OEA_BF16 || N > 128 || B > 128 || k > 16) return hipErrorNotSupported;
  const bool shape30 = d == 2048 && I == 768, shape235 = d == 4096 && I == 1536;
  if (!shape30 && !shape235) return hipErrorNotSupported;
  int dev = 0, grid = 0;
  if (!current_device(&dev, &grid)) return hipErrorUnknown;
  if (grid < 1) return hipErrorNotSupported;
  // most experts one workgroup's cost share can touch: share / cheapest expert, plus the two it may cut
  const int beta_hi = kBetaUp > kBetaDown ? kBetaUp : kBetaDown, beta_lo = kBetaUp < kBetaDown ? kBetaUp : kBetaDown;
  const long long share_num = (long long)kRowCost * N + (long long)beta_hi * B * k;
  const int nseg_max = int(share_num / ((long long)grid * (kRowCost + beta_lo))) + 2;
  if (nseg_max > kMaxSeg) return hipErrorNotSupported;
  const size_t fixed = 16 + fused_meta_words(B, N, k) * 4;
  const bool gather = B > 32;  // x of the whole batch does not fit beside the rest: stage per workgroup
  long long cap_vec = (long long)nseg_max * B, cap_vec1 = 0;
  if (cap_vec > (long long)B * k) cap_vec = (long long)B * k;
  int ecap0 = 0, ecap1 = 0;
  size_t lds_bytes = 0;
  if (!gather) {
    const size_t vec_x = (size_t)B * d * 2, vec_h = (size_t)cap_vec * I * 2;
    if (fixed + (vec_x > vec_h ? vec_x : vec_h) > kFusedLdsMax) return hipErrorNotSupported;
    // what is left of the LDS holds the wavefronts' result buffers (at most 2048 floats each)
    auto result_cap = [&](size_t vec) {
      size_t per_wave = (kFusedLdsMax - fixed - vec) / (kFfnWaves * sizeof(float));
      per_wave = per_wave > 2048 ? 2048 : per_wave & ~size_t(3);
      return per_wave >= 64 ? (int)per_wave : 0;
    };
    ecap0 = result_cap(vec_x);
    ecap1 = result_cap(vec_h);
    const size_t need0 = vec_x + (size_t)ecap0 * kFfnWaves * sizeof(float);
    const size_t need1 = vec_h + (size_t)ecap1 * kFfnWaves * sizeof(float);
    lds_bytes = fixed + (need0 > need1 ? need0 : need1);
  } else {
    // result buffers of 1024 (gate/up) and 2048 (down: more rows per workgroup, shorter vectors) floats
    // per wavefront; the rest of the LDS holds the staged vectors of a piece
    ecap0 = 1024;
    ecap1 = 2048;
    const size_t res0 = (size_t)ecap0 * kFfnWaves * sizeof(float), res1 = (size_t)ecap1 * kFfnWaves * sizeof(float);
    if (fixed + res0 + 4 * (size_t)d * 2 > kFusedLdsMax || fixed + res1 + 4 * (size_t)I * 2 > kFusedLdsMax)
      return hipErrorNotSupported;
    const long long c0 = (long long)((kFusedLdsMax - fixed - res0) / ((size_t)d * 2));
    const long long c1 = (long long)((kFusedLdsMax - fixed - res1) / ((size_t)I * 2));
    cap_vec1 = c1 < cap_vec ? c1 : cap_vec;
    cap_vec = c0 < cap_vec ? c0 : cap_vec;
    const size_t need0 = (size_t)cap_vec * d * 2 + res0, need1 = (size_t)cap_vec1 * I * 2 + res1;
    lds_bytes = fixed + (need0 > need1 ? need0 : need1);
  }
  const size_t alone = 84 * 1024;  // more than half of a CU's LDS: exactly one workgroup per CU
  if (lds_bytes < alone) lds_bytes = alone;

  FusedParams p{};
  p.x = x;
  p.w_router = w_router;
  p.w_gate = w_gate;
  p.w_up = w_up;
  p.w_down = w_down;
  p.bias = bias;
  p.token_mask = token_mask;
  p.out = out;
  p.acc = y_per_pair ? y_per_pair : out;
  p.acc_rows = y_per_pair ? B * k : B;
  p.logits = logits;
  p.h = h;
  p.ro = ro;
  p.ctrl = ctrl;
  p.B = B;
  p.d = d;
  p.N = N;
  p.I = I;
  p.k = k;
  p.k0 = k0;
  p.general = general ? 1 : 0;
  p.gen_p = general ? general->p : 1.0;
  p.gen_max_p = general ? general->max_p : N;
  p.cap_vec = (int)cap_vec;
  p.cap_vec1 = (int)cap_vec1;
  p.ecap0 = ecap0;
  p.ecap1 = ecap1;
  p.spin_limit = spin_limit ? spin_limit : 4u << 20;  // polls of >= 100 ns each: gives up after about a second
  if (gather) {
    if (shape30) return launch_fused_gather_one<uint16_t, 32, 8, 16, 6, 2>(p, grid, lds_bytes, cooperative, s);
    return launch_fused_gather_one<uint16_t, 64, 8, 32, 6, 2>(p, grid, lds_bytes, cooperative, s);
  }
  if (shape30) return launch_fused_one<uint16_t, 32, 8, 16, 6, 2>(p, grid, lds_bytes, cooperative, s);
  return launch_fused_one<uint16_t, 64, 8, 32, 6, 2>(p, grid, lds_bytes, cooperative, s);
}

// The two expert stages as separate kernels built from the fused kernel's stage code (batches the
// fused kernel does not take); hipErrorNotSupported for shapes they are not built for.
hipError_t try_launch_stage_kernels(int stage, const void* vec, const void* wa, const void* wb, void* h_out,
                                    float* out, int B, int d, int N, int I, int k, oea_dtype dt, Grouping g,
                                    bool per_pair, hipStream_t s) {
  if (dt != OEA_BF16 || N > 128) return hipErrorNotSupported;
  const bool shape30 = d == 2048 && I == 768, shape235 = d == 4096 && I == 1536;
  if (!shape30 && !shape235) return hipErrorNotSupported;
  int dev = 0, grid = 0;
  if (!current_device(&dev, &grid)) return hipErrorUnknown;
  if (grid < 1) return hipErrorNotSupported;
  // a workgroup's cost share must not span more than kMaxSeg experts (see try_launch_fused)
  const int beta_hi = kBetaUp > kBetaDown ? kBetaUp : kBetaDown, beta_lo = kBetaUp < kBetaDown ? kBetaUp : kBetaDown;
  const long long share_num = (long long)kRowCost * N + (long long)beta_hi * B * k;
  if (int(share_num / ((long long)grid * (kRowCost + beta_lo))) + 2 > kMaxSeg) return hipErrorNotSupported;
  StageParams p{};
  p.wa = wa;
  p.wb = wb;
  p.vec = vec;
  p.h_out = h_out;
  p.out = out;
  p.g = g;
  p.rows = stage == 0 ? I : d;
  p.L = stage == 0 ? d : I;
  p.N = N;
  p.B = B;
  p.pairs_max = B * k;
  p.per_pair = per_pair ? 1 : 0;
  if (shape30)
    return stage == 0 ? launch_stage_one<uint16_t, 0, 32, 8, 1>(p, grid, s)
                      : launch_stage_one<uint16_t, 1, 16, 6, 2>(p, grid, s);
  return stage == 0 ? launch_stage_one<uint16_t, 0, 64, 8, 1>(p, grid, s)
                    : launch_stage_one<uint16_t, 1, 32, 6, 2>(p, grid, s);
}

}  // namespace oea

#ifdef OEA_TIMELINE
// Timeline build only: copy the stamps of the last layer kernel to the host (kTlSlots x kTlWgs
// 64-bit wall-clock values, slot-major).  Synchronises the device.
extern "C" int oea_timeline_read(unsigned long long* h_dst, size_t bytes) {
  if (!h_dst || bytes < sizeof(unsigned long long) * oea::kTlSlots * oea::kTlWgs) return OEA_ERR_SHAPE;
  if (hipDeviceSynchronize() != hipSuccess) return OEA_ERR_HIP;
  return hipMemcpyFromSymbol(h_dst, HIP_SYMBOL(oea::g_timeline), sizeof(unsigned long long) * oea::kTlSlots * oea::kTlWgs) ==
                 hipSuccess
             ? OEA_OK
             : OEA_ERR_HIP;
}
#endif
