// Expert stages on the matrix cores, for batches in which an expert serves many tokens.
//
// The dot-product stages multiply every weight once per token of its expert on the vector ALUs:
// fine while an expert has a handful of tokens (the layer is then bound by the weight stream,
// Section 3.1, Eq. 2: the b T term), but with B*k/N of 16 and more the a B k term takes over and the
// vector ALUs, not HBM, set the latency.  Here a weight tile meets 16 tokens per instruction
// instead: v_mfma_f32_16x16x32_bf16 multiplies 16 weight rows x 32 columns with the same 32
// entries of 16 token vectors (bf16 products, fp32 accumulation).
//
// A workgroup (8 wavefronts) takes units of 128 rows of W_gate AND W_up of one expert (gate/up
// stage; 16 rows of each per wavefront) or 256 rows of W_down (down stage; 32 per wavefront) and
// walks the inner dimension in slabs of 64 columns, against up to 128 tokens of the expert at a
// time (accumulators for 8 groups of 16 tokens x 2 weight tiles stay in registers; an expert with
// more tokens takes further passes over the same rows).
//   * Every operand is loaded from memory with whole 128-byte row pieces per 8 lanes (a lane
//     pattern in the instruction's operand layout, 16 different rows per 16 lanes, costs several
//     times the cache look-ups and was measured to stream at half the rate), four slabs ahead,
//     into registers; loads are issued and consumed in one order, so the in-order completion of
//     the memory counter costs nothing.  The pipeline runs on across units.
//   * A slab goes through LDS to reach the operand layout (lane l: row l % 16, columns
//     8 (l / 16) .. + 8 of a step's 32): a wavefront's weight rows through a region of its own, the
//     token rows (x, or h rows of the expert's pairs, gathered through the pair list; each
//     wavefront loads an eighth) through a shared one, two buffers each and one workgroup barrier
//     per slab.  Rows are 144 bytes apart in LDS, so both directions are free of bank conflicts.
// Results leave the registers directly: silu(gate) * up rounded to the storage type into h, or
// gate-weighted atomic adds into out (Eq. 1).
#include "oea_ffn_dev.h"

namespace oea {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kDenseGroups = 8;     // groups of 16 tokens per pass
constexpr int kDenseTokens = 16 * kDenseGroups;
constexpr int kDenseBLoads = kDenseTokens / 64;  // token-row pieces a lane loads per slab (8 rows per wavefront and load)
constexpr int kDenseSlab = 64;      // columns per slab: two matrix-core steps of 32
constexpr int kDenseLook = 4;       // slabs requested ahead
constexpr int kDenseRowQuads = 9;   // 16-byte pieces between consecutive rows of a slab in LDS (8 + 1 of padding)
constexpr int kDenseLdsA = 2 * 2 * 16 * kDenseRowQuads;          // per wavefront: [buffer][tile][row]
constexpr int kDenseLdsB = 2 * kDenseTokens * kDenseRowQuads;    // [buffer][token]
constexpr int kDenseMeta = 4096;    // pairs whose token and gate weight a workgroup keeps in LDS
constexpr size_t kDenseLdsBytes = (size_t)(kFfnWaves * kDenseLdsA + kDenseLdsB) * 16 + (size_t)kDenseMeta * 8;

struct DenseParams {
  const uint16_t* wa;   // gate/up stage: W_gate; down stage: W_down   [N, rows, L]
  const uint16_t* wb;   // gate/up stage: W_up
  const uint16_t* vec;  // gate/up stage: x [B, L]; down stage: h [pairs, L] in grouped order
  uint16_t* h_out;      // gate/up stage: h [pairs, rows]
  float* out;           // down stage: out [B, rows] (or [pairs, rows], one row per pair)
  Grouping g;
  int rows, L, N, B, pairs_max;
  int per_pair;
};

// One job of a workgroup: a unit (expert, block of rows) against one pass of at most kDenseTokens pairs.
struct DenseJob {
  int u;      // unit number; units are numbered expert-major over the active list
  int pass;
  int e;      // expert id
  int row0;   // first row of the unit inside the expert
  int pair0;  // first pair of the pass (grouped order)
  int cnt;    // pairs in the pass, 1..kDenseTokens
  int mbase;  // entry of pair0 in the token / gate-weight copy in LDS
  bool valid;
};

// Token and gate weight of the pairs of the workgroup's experts are copied to LDS before the first
// weight request: a load from memory inside the pipeline would have to wait for every weight load
// issued before it (the memory counter completes in order).  A workgroup's units span at most
// ceil(N / workgroups) + 1 experts of at most B pairs each; the launcher only starts the kernel if
// that many fit.
struct DenseMeta {
  int* tok;     // LDS [kDenseMeta]: tokens, clamped to [0, B)
  float* gw;    // LDS [kDenseMeta]
  int first;    // pair number of entry 0
};

// Where one wavefront finds a job's operands: wave-uniform base addresses (they stay in scalar
// registers, with the slab's column offset added there) and one 32-bit byte offset per lane and
// operand kind.  The weight offset is the same for every job.
struct DenseOperands {
  const char* a0;   // first row of the wavefront's tile 0
  const char* a1;   // ... of tile 1: W_up (gate/up stage) or the next 16 rows of W_down
  uint32_t off_b[kDenseBLoads];  // per lane: its piece of its token rows
};

__device__ __forceinline__ u32x4_t load_stream_q(const char* base, uint32_t off) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + off));
}
__device__ __forceinline__ u32x4_t load_plain_q(const char* base, uint32_t off) {
  return *reinterpret_cast<const u32x4_t*>(base + off);
}

__device__ __forceinline__ int sgpr(int v) { return __builtin_amdgcn_readfirstlane(v); }

template <int STAGE>
__device__ __forceinline__ DenseJob dense_job(const int* l_active, const int* l_off, int u, int pass, int u1, int upe,
                                              int pairs_max) {
  constexpr int kUnitRows = STAGE == 0 ? 128 : 256;
  DenseJob j{};
  j.valid = false;
  while (u < u1) {  // experts without usable pairs never occur after a valid routing
    const int a = u / upe;
    const int off = sgpr(l_off[a]), cnt = sgpr(l_off[a + 1]) - off;
    if (off >= 0 && cnt > 0 && off + cnt <= pairs_max && pass * kDenseTokens < cnt) {
      j.u = u;
      j.pass = pass;
      j.e = sgpr(l_active[a]);
      j.row0 = (u - a * upe) * kUnitRows;
      j.pair0 = off + pass * kDenseTokens;
      const int rem = cnt - pass * kDenseTokens;
      j.cnt = rem < kDenseTokens ? rem : kDenseTokens;
      j.valid = true;
      return j;
    }
    ++u;
    pass = 0;
  }
  return j;
}

template <int STAGE>
__device__ __forceinline__ DenseOperands dense_operands(const DenseParams& p, const DenseMeta& mv, const DenseJob& j,
                                                       int wave, int lane) {
  constexpr int kWaveRows = STAGE == 0 ? 16 : 32;
  DenseOperands o;
  const size_t first = ((size_t)j.e * p.rows + (size_t)(j.row0 + wave * kWaveRows)) * p.L * sizeof(uint16_t);
  o.a0 = reinterpret_cast<const char*>(p.wa) + first;
  o.a1 = STAGE == 0 ? reinterpret_cast<const char*>(p.wb) + first : o.a0 + (size_t)16 * p.L * sizeof(uint16_t);
#pragma unroll
  for (int h = 0; h < kDenseBLoads; ++h) {
    const int n = h * 64 + wave * 8 + (lane >> 3);  // a token row this lane helps to load; past the last one: the last again
    const int nn = n < j.cnt ? n : j.cnt - 1;
    int pi = j.pair0 + nn;
    pi = pi < 0 ? 0 : (pi >= p.pairs_max ? p.pairs_max - 1 : pi);
    const int vrow = STAGE == 0 ? mv.tok[j.mbase + nn] : pi;
    // below 2^31 by the entry points' limits on B, k, d and I
    o.off_b[h] = (uint32_t(vrow) * uint32_t(p.L) + (lane & 7) * 8) * uint32_t(sizeof(uint16_t));
  }
  return o;
}

// registers of one slab in flight: four pieces of weight rows (tile 0 rows 0-7, 8-15, tile 1 likewise), one of a token row
struct DenseSlab {
  u32x4_t a[4], b[kDenseBLoads];
};

template <int STAGE>
__device__ __forceinline__ void dense_request(DenseSlab& r, const DenseParams& p, const DenseOperands& q,
                                              uint32_t off_a, int slab) {
  const size_t col = (size_t)slab * kDenseSlab * sizeof(uint16_t);
  const size_t rows8 = (size_t)8 * p.L * sizeof(uint16_t);
  r.a[0] = load_stream_q(q.a0 + col, off_a);
  r.a[1] = load_stream_q(q.a0 + rows8 + col, off_a);
  r.a[2] = load_stream_q(q.a1 + col, off_a);
  r.a[3] = load_stream_q(q.a1 + rows8 + col, off_a);
#pragma unroll
  for (int h = 0; h < kDenseBLoads; ++h) r.b[h] = load_plain_q(reinterpret_cast<const char*>(p.vec) + col, q.off_b[h]);
}

// The slab loop of one job with ng token groups.  ring[] holds the slabs in flight (slot = slab % 4).
// One instance of the loop serves every group count (a branch per group, wave-uniform): with an
// instance per count the compiler moves the ring between their register assignments from job to
// job, which waits for every load in flight.
template <int STAGE>
__device__ __forceinline__ void dense_run(DenseSlab (&ring)[kDenseLook], const DenseParams& p, const DenseOperands& cur,
                                          const DenseOperands& nxt, uint32_t off_a, u32x4_t* lds_a, u32x4_t* lds_b,
                                          f32x4_t (&acc)[kDenseGroups][2], int ng, int wave, int lane) {
  const int r = lane & 15, q = lane >> 4;
  const int wrow = lane >> 3, wcol = lane & 7;
  const int slabs = p.L / kDenseSlab;  // a multiple of kDenseLook (launcher)
  for (int sl = 0; sl < slabs; sl += kDenseLook) {
    const bool last = sl + kDenseLook >= slabs;  // refills then belong to the next job
#pragma unroll
    for (int s = 0; s < kDenseLook; ++s) {
      const int buf = s & 1;
      u32x4_t* const wa_ = lds_a + buf * (2 * 16 * kDenseRowQuads);
      u32x4_t* const wb_ = lds_b + buf * (kDenseTokens * kDenseRowQuads);
      wa_[(wrow)*kDenseRowQuads + wcol] = ring[s].a[0];
      wa_[(wrow + 8) * kDenseRowQuads + wcol] = ring[s].a[1];
      wa_[(16 + wrow) * kDenseRowQuads + wcol] = ring[s].a[2];
      wa_[(24 + wrow) * kDenseRowQuads + wcol] = ring[s].a[3];
#pragma unroll
      for (int h = 0; h < kDenseBLoads; ++h) wb_[(h * 64 + wave * 8 + wrow) * kDenseRowQuads + wcol] = ring[s].b[h];
      {  // selected without a branch: the bases are scalars
        DenseOperands src;
        src.a0 = last ? nxt.a0 : cur.a0;
        src.a1 = last ? nxt.a1 : cur.a1;
#pragma unroll
        for (int h = 0; h < kDenseBLoads; ++h) src.off_b[h] = last ? nxt.off_b[h] : cur.off_b[h];
        dense_request<STAGE>(ring[s], p, src, off_a, last ? s : sl + kDenseLook + s);
      }
      __syncthreads();
#pragma unroll
      for (int i2 = 0; i2 < 2; ++i2) {
        const bf16x8_t a0 = __builtin_bit_cast(bf16x8_t, wa_[r * kDenseRowQuads + i2 * 4 + q]);
        const bf16x8_t a1 = __builtin_bit_cast(bf16x8_t, wa_[(16 + r) * kDenseRowQuads + i2 * 4 + q]);
#pragma unroll
        for (int c = 0; c < kDenseGroups; ++c) {
          if (c >= ng) break;
          const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, wb_[(16 * c + r) * kDenseRowQuads + i2 * 4 + q]);
          if (STAGE == 0) {  // result tile [weight row][token]: a lane holds four rows of one token
            acc[c][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bv, acc[c][0], 0, 0, 0);
            acc[c][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bv, acc[c][1], 0, 0, 0);
          } else {  // [token][weight row]: 16 lanes hold 16 consecutive output coordinates of one token
            acc[c][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv, a0, acc[c][0], 0, 0, 0);
            acc[c][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv, a1, acc[c][1], 0, 0, 0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);  // a slot is refilled as soon as it is free, slab by slab
    }
  }
}

template <int STAGE>
__device__ __forceinline__ void dense_store(const DenseParams& p, const DenseMeta& mv, const DenseJob& j,
                                            const f32x4_t (&acc)[kDenseGroups][2], int wave, int lane) {
  constexpr int kWaveRows = STAGE == 0 ? 16 : 32;
  const int r = lane & 15, q = lane >> 4;
  const int rows = p.rows;
  if (STAGE == 0) {
    // the lane holds rows 4 q .. 4 q + 3 of the gate and the up tile for token r of each group
    const int row = j.row0 + wave * kWaveRows + 4 * q;
#pragma unroll
    for (int c = 0; c < kDenseGroups; ++c) {
      const int n = c * 16 + r;
      if (n < j.cnt) {
        int pi = j.pair0 + n;
        pi = pi < 0 ? 0 : (pi >= p.pairs_max ? p.pairs_max - 1 : pi);
        uint16_t hv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float gsum = acc[c][0][i], usum = acc[c][1][i];
          hv[i] = f32_to_bf16_rne(gsum / (1.f + __expf(-gsum)) * usum);
        }
        uint2 packed;
        packed.x = uint32_t(hv[0]) | (uint32_t(hv[1]) << 16);
        packed.y = uint32_t(hv[2]) | (uint32_t(hv[3]) << 16);
        *reinterpret_cast<uint2*>(p.h_out + (size_t)pi * rows + row) = packed;
      }
    }
  } else {
    // the lane holds output coordinate r of both tiles for tokens 4 q .. 4 q + 3 of each group: an
    // atomic instruction adds 64 consecutive bytes to each of four rows of out
    const int row = j.row0 + wave * kWaveRows + r;
#pragma unroll
    for (int c = 0; c < kDenseGroups; ++c)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = c * 16 + 4 * q + i;
        if (n < j.cnt) {
          int pi = j.pair0 + n;
          pi = pi < 0 ? 0 : (pi >= p.pairs_max ? p.pairs_max - 1 : pi);
          const int orow = p.per_pair ? pi : mv.tok[j.mbase + n];
          const float gw = mv.gw[j.mbase + n];
          float* const o = p.out + (size_t)orow * rows + row;
          unsafeAtomicAdd(o, gw * acc[c][0][i]);
          unsafeAtomicAdd(o + 16, gw * acc[c][1][i]);
        }
      }
  }
}

template <int STAGE>
__global__ __launch_bounds__(kFfnThreads) void expert_dense_kernel(DenseParams p) {
  extern __shared__ uint4 lds4[];
  __shared__ int l_active[OEA_MAX_N];
  __shared__ int l_off[OEA_MAX_N + 1];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int N = p.N;
  int T = *p.g.n_active;
  T = T < 0 ? 0 : (T > N ? N : T);
  for (int i = tid; i < N; i += kFfnThreads) {
    const int e = i < T ? p.g.active_list[i] : 0;
    l_active[i] = e < 0 ? 0 : (e >= N ? N - 1 : e);
  }
  for (int i = tid; i <= N; i += kFfnThreads) l_off[i] = p.g.grp_off[i <= T ? i : T];
  __syncthreads();

  // units of this workgroup: a contiguous, equal share of all active experts' row blocks
  constexpr int kUnitRows = STAGE == 0 ? 128 : 256;
  const int upe = p.rows / kUnitRows;
  const long long U = (long long)T * upe;
  const int u0 = int(U * blockIdx.x / gridDim.x), u1 = int(U * (blockIdx.x + 1) / gridDim.x);
  u32x4_t* const lds_a = reinterpret_cast<u32x4_t*>(lds4) + wave * kDenseLdsA;
  u32x4_t* const lds_b = reinterpret_cast<u32x4_t*>(lds4) + kFfnWaves * kDenseLdsA;

  DenseJob cur = dense_job<STAGE>(l_active, l_off, u0, 0, u1, upe, p.pairs_max);
  if (!cur.valid) return;  // uniform over the workgroup
  // token and gate weight of every pair of this workgroup's experts -> LDS
  DenseMeta mv{};
  mv.tok = reinterpret_cast<int*>(lds_b + kDenseLdsB);
  mv.gw = reinterpret_cast<float*>(mv.tok + kDenseMeta);
  {
    const int a_first = u0 / upe, a_last = (u1 - 1) / upe;  // u1 > u0: there is a valid job
    const int m0 = sgpr(l_off[a_first]), m1 = sgpr(l_off[a_last + 1]);
    mv.first = m0;
    // never false after a valid routing (see DenseMeta); keeps the copy inside its LDS area
    if (!(m0 >= 0 && m1 >= m0 && m1 - m0 <= kDenseMeta && m1 <= p.pairs_max)) return;
    for (int i = tid; i < m1 - m0; i += kFfnThreads) {
      const int t = p.g.grp_tok[m0 + i];
      mv.tok[i] = t < 0 ? 0 : (t >= p.B ? p.B - 1 : t);
      mv.gw[i] = p.g.grp_gw[m0 + i];
    }
  }
  cur.mbase = cur.pair0 - mv.first;
  __syncthreads();
  DenseOperands pc = dense_operands<STAGE>(p, mv, cur, wave, lane);
  // per lane: row lane / 8 of a group of eight rows, 16-byte piece lane % 8 of the slab's 128 bytes
  const uint32_t off_a = (uint32_t(lane >> 3) * uint32_t(p.L) + (lane & 7) * 8) * uint32_t(sizeof(uint16_t));
  DenseSlab ring[kDenseLook];
#pragma unroll
  for (int s = 0; s < kDenseLook; ++s) dense_request<STAGE>(ring[s], p, pc, off_a, s);
  while (cur.valid) {
    // the job after this one; without one the last refills read this job's first slabs again (unused)
    DenseJob nxt = dense_job<STAGE>(l_active, l_off, cur.u, cur.pass + 1, u1, upe, p.pairs_max);
    nxt.mbase = nxt.pair0 - mv.first;
    const DenseOperands pn = nxt.valid ? dense_operands<STAGE>(p, mv, nxt, wave, lane) : pc;
    f32x4_t acc[kDenseGroups][2];
#pragma unroll
    for (int c = 0; c < kDenseGroups; ++c) acc[c][0] = acc[c][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    dense_run<STAGE>(ring, p, pc, pn, off_a, lds_a, lds_b, acc, (cur.cnt + 15) >> 4, wave, lane);
    dense_store<STAGE>(p, mv, cur, acc, wave, lane);
    cur = nxt;
    pc = pn;
  }
}

}  // namespace

// One expert stage (0 gate/up, 1 down) on the matrix cores; hipErrorNotSupported for storage types
// and shapes it is not built for (bf16; rows a multiple of a workgroup's unit, inner dimension of 256).
hipError_t try_launch_dense_stage(int stage, const void* vec, const void* wa, const void* wb, void* h_out, float* out,
                                  int B, int d, int N, int I, int k, oea_dtype dt, Grouping g, bool per_pair,
                                  hipStream_t s) {
  if (dt != OEA_BF16 || N > OEA_MAX_N) return hipErrorNotSupported;
  const int rows = stage == 0 ? I : d, L = stage == 0 ? d : I;
  if (rows % (stage == 0 ? 128 : 256) != 0 || L % (kDenseLook * kDenseSlab) != 0) return hipErrorNotSupported;
  int dev = 0, grid = 0;
  if (!current_device(&dev, &grid)) return hipErrorUnknown;
  if (grid < 1) return hipErrorNotSupported;
  // the pairs of the experts one workgroup can touch must fit its LDS copy of their tokens and weights
  if (((long long)(N + grid - 1) / grid + 1) * B > kDenseMeta) return hipErrorNotSupported;
  DenseParams p{};
  p.wa = static_cast<const uint16_t*>(wa);
  p.wb = static_cast<const uint16_t*>(wb);
  p.vec = static_cast<const uint16_t*>(vec);
  p.h_out = static_cast<uint16_t*>(h_out);
  p.out = out;
  p.g = g;
  p.rows = rows;
  p.L = L;
  p.N = N;
  p.B = B;
  p.pairs_max = B * k;
  p.per_pair = per_pair ? 1 : 0;
  static PerDevice attr0, attr1;
  const void* kern = stage == 0 ? reinterpret_cast<const void*>(expert_dense_kernel<0>)
                                : reinterpret_cast<const void*>(expert_dense_kernel<1>);
  hipError_t e = ensure_dynamic_lds(kern, (int)kDenseLdsBytes, stage == 0 ? attr0 : attr1);
  if (e != hipSuccess) return e;
  if (stage == 0)
    hipLaunchKernelGGL(expert_dense_kernel<0>, dim3(grid), dim3(kFfnThreads), kDenseLdsBytes, s, p);
  else
    hipLaunchKernelGGL(expert_dense_kernel<1>, dim3(grid), dim3(kFfnThreads), kDenseLdsBytes, s, p);
  return hipGetLastError();
}

}  // namespace oea
