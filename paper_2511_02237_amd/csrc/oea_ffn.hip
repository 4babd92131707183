// Grouped SwiGLU expert FFN over the ACTIVE experts only (gfx950).
//
// The paper's premise (Section 2 and Section 3.1, Eq. 2) is that at decode batch sizes the layer is
// bound by streaming each activated expert's weights from HBM once; per-expert token counts are
// tiny (1-4 at B=16).  So both mat-vec stages are bandwidth kernels built from one primitive:
// a wavefront streams a tile of weight rows with 16-byte loads (fully coalesced: LPR consecutive
// lanes cover LPR*16 contiguous bytes of one row), keeps the tile in registers, and takes its dot
// products with the few token vectors of that expert, which sit in LDS.
//
//   stage 0 (gate/up): rows j of W_gate[e], W_up[e] (length d) . x_t      -> h[p,j] = silu(g)*u
//   stage 1 (down)   : rows c of W_down[e] (length I) . h[p,:]            -> out[t,c] += g_{t,e} * y
//
// Work split: the T*rows weight rows of the active experts are cut into gridDim.x equal contiguous
// ranges, one per workgroup (so every CU streams the same number of bytes whatever T is); inside a
// workgroup each (expert, row-range) segment is cut again into equal ranges, one per wavefront.
#include "oea_ffn_dev.h"

namespace oea {

namespace {

constexpr size_t kLdsBudget = 128 * 1024;     // generic kernel: LDS bytes for the staged token vectors
constexpr size_t kStreamLdsMax = 152 * 1024;  // streaming kernel: most LDS one workgroup may ask for

struct FfnParams {
  const void* wa;    // stage 0: W_gate [N,rows,L]; stage 1: W_down [N,rows,L]
  const void* wb;    // stage 0: W_up; stage 1: unused
  const void* vec;   // stage 0: x [B,L]; stage 1: h [P,L]
  void* h_out;       // stage 0: h [P,rows]
  float* out;        // stage 1: out [B,rows]
  int rows;          // weight rows per expert (stage 0: I, stage 1: d)
  int L;             // row length            (stage 0: d, stage 1: I)
  int N;
  int B;
  int pairs_max;     // B*k: size of the grouping arrays
  int per_pair;      // stage 1: `out` has one row per PAIR (deterministic combine): pair p adds into row p
  int tok_cap;       // generic kernel: token vectors that fit in LDS at once
  int cap_vec;       // streaming kernel: capacity of the staged (expert, token) pair list
  Grouping g;
};

// STAGE 0: two matrices (gate, up), RG must be 1.  STAGE 1: one matrix, RG row groups per tile.
// LPR lanes share a row (64/LPR rows per group); NCH 16-byte chunks per lane cover a row.
template <typename WT, int STAGE, int LPR, int NCH, int RG>
__global__ __launch_bounds__(kFfnThreads) void expert_kernel(FfnParams p) {
  extern __shared__ uint4 lds4[];
  constexpr int EPL = 16 / int(sizeof(WT));  // elements per 16-byte load
  constexpr int R = 64 / LPR;                // rows per row group
  constexpr int CH = LPR * EPL;              // elements per chunk of a row
  constexpr int NM = STAGE == 0 ? 2 : 1;
  static_assert(STAGE == 1 || RG == 1, "gate/up stage uses one row group");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lsub = lane % LPR, lrow = lane / LPR;
  const int rows = p.rows, L = p.L;
  const int nch = (L + CH - 1) / CH;  // <= NCH, checked on the host
  const int L16 = L / EPL;            // 16-byte granules per vector

  int T = *p.g.n_active;
  T = T < 0 ? 0 : (T > p.N ? p.N : T);
  const long long total = (long long)T * rows;
  const long long R0 = total * blockIdx.x / gridDim.x;
  const long long R1 = total * (blockIdx.x + 1) / gridDim.x;
  if (R0 >= R1) return;

  const WT* wa = static_cast<const WT*>(p.wa);
  const WT* wb = static_cast<const WT*>(p.wb);
  const WT* vec = static_cast<const WT*>(p.vec);

  for (int a = int(R0 / rows); (long long)a * rows < R1; ++a) {
    const long long base = (long long)a * rows;
    const int seg_lo = int((R0 > base ? R0 : base) - base);
    const int seg_hi = int((R1 < base + rows ? R1 : base + rows) - base);
    const int e = p.g.active_list[a];
    const int off = p.g.grp_off[a];
    const int cnt = p.g.grp_off[a + 1] - off;
    // never taken after a valid routing; keeps every access in bounds if the workspace was not prepared
    if ((unsigned)e >= (unsigned)p.N || cnt <= 0 || off < 0 || off + cnt > p.pairs_max) continue;
    const WT* wae = wa + (size_t)e * rows * L;
    const WT* wbe = STAGE == 0 ? wb + (size_t)e * rows * L : nullptr;

    // this wavefront's equal share of the segment
    const int nseg = seg_hi - seg_lo;
    const int my_lo = seg_lo + int((long long)nseg * wave / kFfnWaves);
    const int my_hi = seg_lo + int((long long)nseg * (wave + 1) / kFfnWaves);

    for (int q0 = 0; q0 < cnt; q0 += p.tok_cap) {
      const int nq = cnt - q0 < p.tok_cap ? cnt - q0 : p.tok_cap;
      __syncthreads();  // the previous segment's readers are done with the LDS vectors
      for (int i = tid; i < nq * L16; i += kFfnThreads) {
        const int q = i / L16, c = i - q * L16;
        int src_row = off + q0 + q;
        if (STAGE == 0) {
          src_row = p.g.grp_tok[src_row];
          src_row = src_row < 0 ? 0 : (src_row >= p.B ? p.B - 1 : src_row);
        }
        lds4[i] = reinterpret_cast<const uint4*>(vec + (size_t)src_row * L)[c];
      }
      __syncthreads();

      for (int r0 = my_lo; r0 < my_hi; r0 += RG * R) {
        // ---- stream the tile: RG*R rows (x2 matrices in stage 0), NCH chunks each
        uint4 w[NM][RG][NCH];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
          const int row = r0 + rg * R + lrow;
          const bool row_ok = row < my_hi;
#pragma unroll
          for (int c = 0; c < NCH; ++c) {
            const int col = c * CH + lsub * EPL;
            const bool ok = row_ok && c < nch && col < L;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
              const WT* src = (m == 0 ? wae : wbe) + (size_t)row * L + col;
              w[m][rg][c] = ok ? load_stream16(src) : make_uint4(0, 0, 0, 0);
            }
          }
        }
        // ---- dot products with each token vector of this expert
        for (int q = 0; q < nq; ++q) {
          float acc[NM][RG];
#pragma unroll
          for (int m = 0; m < NM; ++m)
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) acc[m][rg] = 0.f;
          const uint4* vq = lds4 + q * L16 + lsub;
#pragma unroll
          for (int c = 0; c < NCH; ++c) {
            if (c < nch) {
              const int g16 = c * LPR + lsub;
              const uint4 v = g16 < L16 ? vq[c * LPR] : make_uint4(0, 0, 0, 0);
#pragma unroll
              for (int m = 0; m < NM; ++m)
#pragma unroll
                for (int rg = 0; rg < RG; ++rg) acc[m][rg] = frag_dot<WT>(w[m][rg][c], v, acc[m][rg]);
            }
          }
          const int pidx = off + q0 + q;
#pragma unroll
          for (int rg = 0; rg < RG; ++rg) {
            const int row = r0 + rg * R + lrow;
            if (STAGE == 0) {
              const float gsum = row_sum<LPR>(acc[0][rg]);
              const float usum = row_sum<LPR>(acc[NM - 1][rg]);
              if (lsub == 0 && row < my_hi) {
                const float hval = gsum / (1.f + __expf(-gsum)) * usum;
                store_h(static_cast<WT*>(p.h_out) + (size_t)pidx * rows + row, hval);
              }
            } else {
              const float y = row_sum<LPR>(acc[0][rg]);
              if (lsub == 0 && row < my_hi) {
                const int t = p.per_pair ? pidx : p.g.grp_tok[pidx];
                if ((unsigned)t < (unsigned)(p.per_pair ? p.pairs_max : p.B))
                  unsafeAtomicAdd(p.out + (size_t)t * rows + row, p.g.grp_gw[pidx] * y);
              }
            }
          }
        }
      }
    }
  }
}


// ---------------------------------------------------------------------------------------------
// Streaming kernel: the fast path.  Same split of the work as above, but
//   * the token vectors of ALL the (at most kMaxSeg) experts a workgroup touches are staged into
//     LDS once, before the main loop, so the loop has no barrier;
//   * every wavefront keeps two weight tiles in registers and always has the next tile's loads in
//     flight while it computes on the current one (continuous HBM streaming).  The loads are
//     unconditional (clamped to valid rows/columns, never predicated), so the compiler can count
//     them and wait only for the older tile.
// Stage 0 keeps x of the whole batch resident (indexed by token); stage 1 stages the hidden
// vectors of its experts' pairs (contiguous in the grouped order).
// FULL: the row length is exactly LPR*EPL*NCH (no ragged last chunk), so no column masks.

template <typename WT, int STAGE, int LPR, int NCH, int RG, bool FULL>
__global__ __launch_bounds__(kFfnThreads) void expert_stream_kernel(FfnParams p) {
  extern __shared__ uint4 lds4[];
  constexpr int EPL = 16 / int(sizeof(WT));
  constexpr int R = 64 / LPR;
  constexpr int NM = STAGE == 0 ? 2 : 1;
  constexpr int TROWS = RG * R;  // weight rows per tile

  const int rows = p.rows, L = p.L, N = p.N;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps the row bookkeeping scalar
  const int lsub = lane % LPR, lrow = lane / LPR;
  const int L16 = L / EPL;
  const WT* const vec = static_cast<const WT*>(p.vec);

  // Staging loads are issued as early as possible and in batches of kStageBatch per thread, all in
  // flight together; they are written to LDS only after the first weight tiles have been requested.
  constexpr int kStageBatch = 8;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a native vector: stays in registers
  u32x4 stg[kStageBatch];
  const int n16_x = p.B * L16;  // stage 0: x of the whole batch, needs no routing result
  if (STAGE == 0) {
    const u32x4* src = reinterpret_cast<const u32x4*>(vec);
#pragma unroll
    for (int j = 0; j < kStageBatch; ++j) {
      const int i = j * kFfnThreads + tid;
      stg[j] = src[i < n16_x ? i : n16_x - 1];
    }
  }
  __builtin_amdgcn_sched_barrier(0);  // keep the staging loads up here, ahead of everything else

  int T = *p.g.n_active;
  T = T < 0 ? 0 : (T > N ? N : T);
  const int total = T * rows;  // <= OEA_MAX_N * OEA_MAX_D: fits an int
  const int R0 = int((long long)total * blockIdx.x / gridDim.x);
  const int R1 = int((long long)total * (blockIdx.x + 1) / gridDim.x);
  if (R0 >= R1) return;

  // ---- the (at most kMaxSeg = 3) experts this workgroup touches: uniform scalar loads
  const int a0 = R0 / rows;
  const int nseg = (R1 - 1) / rows - a0 + 1;
  const int off0 = p.g.grp_off[a0];
  const int off1 = p.g.grp_off[a0 + 1];
  const int off2 = nseg > 1 ? p.g.grp_off[a0 + 2] : off1;
  const int off3 = nseg > 2 ? p.g.grp_off[a0 + 3] : off2;
  const int e0 = p.g.active_list[a0];
  const int e1 = nseg > 1 ? p.g.active_list[a0 + 1] : 0;
  const int e2 = nseg > 2 ? p.g.active_list[a0 + 2] : 0;
  const int nvec = off3 - off0;
  // never true after a valid routing; keeps every access in bounds otherwise
  if (nseg > kMaxSeg || off0 < 0 || off1 < off0 || off2 < off1 || off3 < off2 || nvec > p.cap_vec ||
      off0 + nvec > p.pairs_max || (unsigned)e0 >= (unsigned)N || (unsigned)e1 >= (unsigned)N ||
      (unsigned)e2 >= (unsigned)N)
    return;

  // LDS: [dump slot: 16 B][pair tokens: cap_vec int][pair weights: cap_vec float][vectors].
  // The dump slot takes the writes of threads that have nothing to stage, so staging is branch-free
  // and its loads stay where they are issued (ahead of the weight tiles).
  int* l_tok = reinterpret_cast<int*>(lds4 + 1);
  float* l_gw = reinterpret_cast<float*>(l_tok + p.cap_vec);
  uint4* l_vec = lds4 + 1 + (p.cap_vec * 8 + 15) / 16;

  // pair lists and (stage 1) the hidden vectors of this workgroup's pairs: first batch of loads
  const int n16 = STAGE == 0 ? n16_x : nvec * L16;
  const uint4* const vsrc = reinterpret_cast<const uint4*>(STAGE == 0 || nvec == 0 ? vec : vec + (size_t)off0 * L);
  const int i_first = nvec == 0 ? 0 : (tid < nvec ? tid : nvec - 1);
  const int src_first = off0 + i_first < p.pairs_max ? off0 + i_first : 0;
  // the row of `out` a pair adds into: its token, or (per_pair) the pair itself
  const int row_limit = STAGE == 1 && p.per_pair ? p.pairs_max : p.B;
  const int tok_first = STAGE == 1 && p.per_pair ? src_first : p.g.grp_tok[src_first];
  const float gw_first = p.g.grp_gw[src_first];
  if (STAGE == 1) {
#pragma unroll
    for (int j = 0; j < kStageBatch; ++j) {
      const int i16 = j * kFfnThreads + tid;
      stg[j] = reinterpret_cast<const u32x4*>(vsrc)[i16 < n16 ? i16 : (n16 > 0 ? n16 - 1 : 0)];
    }
  }
  __builtin_amdgcn_sched_barrier(0);

  // this wavefront's equal share [my_lo, my_hi) of the workgroup's rows (concatenated numbering)
  const int n_wg = R1 - R0;
  const int my_lo = R0 + int((long long)n_wg * wave / kFfnWaves);
  const int my_hi = R0 + int((long long)n_wg * (wave + 1) / kFfnWaves);
  const bool has_work = my_lo < my_hi;

  const SegView sv{rows, a0, e0, e1, e2, off1 - off0, off2 - off1, off3 - off2, my_hi};
  const WT* const wa = static_cast<const WT*>(p.wa);
  const WT* const wb = static_cast<const WT*>(p.wb);
  WT* const h_out = static_cast<WT*>(p.h_out);
  float* const out = p.out;

  // ---- prologue: first two tiles in flight, then the staged data goes to LDS
  uint4 wA[NM][RG][NCH], wB[NM][RG][NCH];
  // Requests past the end of the wavefront's rows (and those of a wavefront without rows) are placeholders
  // on the row r_first: the loads stay unconditional, which keeps the compiler's count of outstanding
  // loads exact, but they read one granule only.
  const int r_first = has_work ? my_lo : R0;
  int rA = r_first, nA = has_work ? tile_rows(sv, my_lo, TROWS) : 0;
  int rB = rA + nA, nB = tile_rows(sv, rB, TROWS);
  load_tile<WT, NM, LPR, NCH, RG, FULL>(wA, wa, wb, rows, L, lsub, lrow, tile_ref(sv, r_first), nA);
  load_tile<WT, NM, LPR, NCH, RG, FULL>(wB, wa, wb, rows, L, lsub, lrow, tile_ref(sv, nB > 0 ? rB : r_first), nB);

  __builtin_amdgcn_sched_barrier(0);  // weight tiles are requested before the staged data is consumed
  {
    int* const dump_i = reinterpret_cast<int*>(lds4);
    float* const dump_f = reinterpret_cast<float*>(lds4) + 1;
    *(tid < nvec ? l_tok + tid : dump_i) = tok_first < 0 ? 0 : (tok_first >= row_limit ? row_limit - 1 : tok_first);
    *(tid < nvec ? l_gw + tid : dump_f) = gw_first;
#pragma unroll
    for (int j = 0; j < kStageBatch; ++j) {
      const int i16 = j * kFfnThreads + tid;
      *reinterpret_cast<u32x4*>(i16 < n16 ? l_vec + i16 : lds4) = stg[j];
    }
  }
  for (int i = tid + kFfnThreads; i < nvec; i += kFfnThreads) {  // only for very large batches
    int t = STAGE == 1 && p.per_pair ? off0 + i : p.g.grp_tok[off0 + i];
    l_tok[i] = t < 0 ? 0 : (t >= row_limit ? row_limit - 1 : t);
    l_gw[i] = p.g.grp_gw[off0 + i];
  }
  for (int i16 = kStageBatch * kFfnThreads + tid; i16 < n16; i16 += kFfnThreads) l_vec[i16] = vsrc[i16];
  __syncthreads();
  if (!has_work) return;

  // ---- main loop: compute on one buffer while the other one's loads are in flight
  while (true) {
    compute_tile<WT, STAGE, NM, LPR, NCH, RG, FULL>(wA, l_tok, l_gw, l_vec, h_out, out, rows, L16, off0, lsub, lrow,
                                                    tile_ref(sv, rA), nA);
    rA = rB + nB;
    nA = tile_rows(sv, rA, TROWS);
    load_tile<WT, NM, LPR, NCH, RG, FULL>(wA, wa, wb, rows, L, lsub, lrow, tile_ref(sv, nA > 0 ? rA : r_first), nA);
    if (nB <= 0) break;
    compute_tile<WT, STAGE, NM, LPR, NCH, RG, FULL>(wB, l_tok, l_gw, l_vec, h_out, out, rows, L16, off0, lsub, lrow,
                                                    tile_ref(sv, rB), nB);
    rB = rA + nA;
    nB = tile_rows(sv, rB, TROWS);
    load_tile<WT, NM, LPR, NCH, RG, FULL>(wB, wa, wb, rows, L, lsub, lrow, tile_ref(sv, nB > 0 ? rB : r_first), nB);
    if (nA <= 0) break;
  }
}

// Measurement aid: read `n16` 16-byte granules once with the access pattern of the expert kernels
// (each wavefront a contiguous share, 16 non-temporal 1 KB requests in flight) and do nothing with
// them.  Its rate is the practical ceiling for streaming weights on the device at hand.
__global__ __launch_bounds__(kFfnThreads) void read_probe_kernel(const uint4* __restrict__ src, size_t n16,
                                                                  uint32_t* sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * kFfnWaves + (threadIdx.x >> 6);
  const size_t nwaves = (size_t)gridDim.x * kFfnWaves;
  const size_t per = (n16 / nwaves) & ~size_t(1023);  // whole batches of 16 x 64 granules; the remainder is skipped
  const uint4* p = src + wave * per;
  uint32_t acc = 0;
  for (size_t i = 0; i < per; i += 1024) {
    uint4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = load_stream16(p + i + j * 64 + lane);
#pragma unroll
    for (int j = 0; j < 16; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  if (acc == 0x9e3779b9u && sink) *sink = acc;  // keeps the loads alive; practically never taken
}

int num_cus() {
  int dev = 0, cus = 0;
  return current_device(&dev, &cus) && cus > 0 ? cus : 256;
}

template <typename WT, int STAGE, int LPR, int NCH, int RG>
hipError_t launch_one(const FfnParams& p, size_t lds_bytes, hipStream_t s) {
  auto kern = expert_kernel<WT, STAGE, LPR, NCH, RG>;
  static PerDevice attr_done;
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kLdsBudget, attr_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(num_cus()), dim3(kFfnThreads), lds_bytes, s, p);
  return hipGetLastError();
}

// pick lanes-per-row so that a row fits in NCH chunks
template <typename WT, int STAGE, int NCH, int RG>
hipError_t launch_lpr(const FfnParams& p, size_t lds_bytes, hipStream_t s) {
  constexpr int EPL = 16 / int(sizeof(WT));
  if (p.L <= 16 * EPL * NCH) return launch_one<WT, STAGE, 16, NCH, RG>(p, lds_bytes, s);
  if (p.L <= 32 * EPL * NCH) return launch_one<WT, STAGE, 32, NCH, RG>(p, lds_bytes, s);
  if (p.L <= 64 * EPL * NCH) return launch_one<WT, STAGE, 64, NCH, RG>(p, lds_bytes, s);
  return hipErrorInvalidValue;
}

template <typename WT, int STAGE, int LPR, int NCH, int RG, bool FULL>
hipError_t launch_stream_one(const FfnParams& p, size_t lds_bytes, hipStream_t s) {
  auto kern = expert_stream_kernel<WT, STAGE, LPR, NCH, RG, FULL>;
  static PerDevice attr_done;
  hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kStreamLdsMax, attr_done);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(num_cus()), dim3(kFfnThreads), lds_bytes, s, p);
  return hipGetLastError();
}

template <typename WT, int STAGE, int LPR>
hipError_t launch_stream_lpr(const FfnParams& p, size_t lds_bytes, hipStream_t s) {
  constexpr int EPL = 16 / int(sizeof(WT));
  constexpr int RG = STAGE == 0 ? 1 : 2;
  if (p.L == LPR * EPL * 8) return launch_stream_one<WT, STAGE, LPR, 8, RG, true>(p, lds_bytes, s);
  if (p.L == LPR * EPL * 6) return launch_stream_one<WT, STAGE, LPR, 6, RG, true>(p, lds_bytes, s);
  return launch_stream_one<WT, STAGE, LPR, 8, RG, false>(p, lds_bytes, s);
}

// Streaming kernel if a row fits 8 chunks of some lanes-per-row and the staged vectors fit LDS.
// Returns hipErrorNotSupported when the generic kernel has to be used.
template <typename WT>
hipError_t try_launch_stream(int stage, FfnParams p, int B, int k, hipStream_t s) {
  constexpr int EPL = 16 / int(sizeof(WT));
  const int grid = num_cus();
  const int nseg_max = (p.N + grid - 1) / grid + 1;
  if (nseg_max > kMaxSeg || p.L > 64 * EPL * 8) return hipErrorNotSupported;
  long long cap_vec = (long long)nseg_max * B;
  if (cap_vec > (long long)B * k) cap_vec = (long long)B * k;
  const size_t list_bytes = 16 + (((size_t)cap_vec * 8 + 15) / 16) * 16;  // dump slot + pair lists
  const size_t vec_bytes = (size_t)(stage == 0 ? B : cap_vec) * p.L * sizeof(WT);
  size_t lds_bytes = list_bytes + vec_bytes;
  if (lds_bytes > kStreamLdsMax) return hipErrorNotSupported;
  const size_t alone = 84 * 1024;  // more than half of the CU's 160 KB: one workgroup per CU
  if (lds_bytes < alone) lds_bytes = alone;
  p.cap_vec = (int)cap_vec;
  // fewest lanes per row (most rows per tile) that covers a row in at most 8 chunks
  const int lpr = p.L <= 16 * EPL * 8 ? 16 : (p.L <= 32 * EPL * 8 ? 32 : 64);
  if (stage == 0) {
    if (lpr == 16) return launch_stream_lpr<WT, 0, 16>(p, lds_bytes, s);
    if (lpr == 32) return launch_stream_lpr<WT, 0, 32>(p, lds_bytes, s);
    return launch_stream_lpr<WT, 0, 64>(p, lds_bytes, s);
  }
  if (lpr == 16) return launch_stream_lpr<WT, 1, 16>(p, lds_bytes, s);
  if (lpr == 32) return launch_stream_lpr<WT, 1, 32>(p, lds_bytes, s);
  return launch_stream_lpr<WT, 1, 64>(p, lds_bytes, s);
}

template <typename WT>
hipError_t launch_stage(int stage, FfnParams p, int B, int k, bool generic_only, hipStream_t s) {
  if (!generic_only) {
    hipError_t e = try_launch_stream<WT>(stage, p, B, k, s);
    if (e != hipErrorNotSupported) return e;
  }
  // generic kernel.  LDS: as many token vectors as fit (at most B), one workgroup per CU
  const size_t vec_bytes = (size_t)p.L * sizeof(WT);
  int cap = int(kLdsBudget / vec_bytes);
  if (cap < 1) return hipErrorInvalidValue;
  if (cap > B) cap = B;
  p.tok_cap = cap;
  size_t lds_bytes = (size_t)cap * vec_bytes;
  const size_t alone = 84 * 1024;
  if (lds_bytes < alone) lds_bytes = alone;
  constexpr int EPL = 16 / int(sizeof(WT));
  if (stage == 0) return launch_lpr<WT, 0, 16, 1>(p, lds_bytes, s);
  // down stage: one matrix, so the 32-load tile holds several row groups
  if (p.L <= 16 * EPL * 8) return launch_one<WT, 1, 16, 8, 4>(p, lds_bytes, s);
  return launch_lpr<WT, 1, 16, 2>(p, lds_bytes, s);
}

}  // namespace

bool current_device(int* dev, int* cus) {
  static PerDevice cached;  // compute units + 1, 0 = not looked up yet
  int d = -1;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) return false;
  int c = cached.v[d].load(std::memory_order_relaxed);
  if (c == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, d) != hipSuccess || n < 0) return false;
    c = n + 1;
    cached.v[d].store(c, std::memory_order_relaxed);
  }
  *dev = d;
  *cus = c - 1;
  return true;
}

namespace {
// Deterministic combine (Eq. 1 with the sum over the selected experts taken in slot order): one
// thread per four output coordinates of a token.  y holds gate weight x expert output per pair.
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ y, const int32_t* __restrict__ grp_pos,
                                                      const int32_t* __restrict__ n_sel, float* __restrict__ out,
                                                      int B, int d, int k, int pairs) {
  const int t = blockIdx.x;
  int n = n_sel[t];
  n = n < 0 ? 0 : (n > k ? k : n);
  for (int c4 = blockIdx.y * 256 + threadIdx.x; c4 < d / 4; c4 += gridDim.y * 256) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < n; ++s) {
      const int pos = grp_pos[t * k + s];
      if ((unsigned)pos >= (unsigned)pairs) continue;  // never true after a valid routing
      const float4 v = reinterpret_cast<const float4*>(y + (size_t)pos * d)[c4];
      acc.x += v.x;
      acc.y += v.y;
      acc.z += v.z;
      acc.w += v.w;
    }
    reinterpret_cast<float4*>(out + (size_t)t * d)[c4] = acc;
  }
}
}  // namespace

hipError_t launch_combine(const float* y, const int32_t* grp_pos, const int32_t* n_sel, float* out, int B, int d,
                          int k, hipStream_t s) {
  const int chunks = (d / 4 + 255) / 256;
  hipLaunchKernelGGL(combine_kernel, dim3(B, chunks > 8 ? 8 : chunks), dim3(256), 0, s, y, grp_pos, n_sel, out, B, d, k,
                     B * k);
  return hipGetLastError();
}

hipError_t launch_read_probe(const void* buf, size_t bytes, uint32_t* sink, hipStream_t s) {
  hipLaunchKernelGGL(read_probe_kernel, dim3(num_cus()), dim3(kFfnThreads), 0, s, static_cast<const uint4*>(buf),
                     bytes / 16, sink);
  return hipGetLastError();
}

hipError_t launch_expert_gate_up(const void* x, const void* w_gate, const void* w_up, void* h, int B,
                                 int d, int N, int I, int k, oea_dtype dt, Grouping g, bool generic_only,
                                 hipStream_t s) {
  FfnParams p{};
  p.B = B;
  p.pairs_max = B * k;
  p.wa = w_gate;
  p.wb = w_up;
  p.vec = x;
  p.h_out = h;
  p.out = nullptr;
  p.rows = I;
  p.L = d;
  p.N = N;
  p.g = g;
  return dt == OEA_F32 ? launch_stage<float>(0, p, B, k, generic_only, s)
                       : launch_stage<uint16_t>(0, p, B, k, generic_only, s);
}

hipError_t launch_expert_down(const void* h, const void* w_down, float* out, int B, int d, int N, int I,
                              int k, oea_dtype dt, Grouping g, bool generic_only, bool per_pair, hipStream_t s) {
  FfnParams p{};
  p.B = B;
  p.pairs_max = B * k;
  p.wa = w_down;
  p.wb = nullptr;
  p.vec = h;
  p.h_out = nullptr;
  p.out = out;
  p.rows = d;
  p.L = I;
  p.N = N;
  p.g = g;
  p.per_pair = per_pair ? 1 : 0;
  return dt == OEA_F32 ? launch_stage<float>(1, p, B, k, generic_only, s)
                       : launch_stage<uint16_t>(1, p, B, k, generic_only, s);
}

}  // namespace oea
