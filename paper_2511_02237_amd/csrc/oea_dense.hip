// Expert stages on the matrix cores, for batches in which an expert serves many tokens.
//
// The dot-product stages multiply every weight once per token of its expert on the vector ALUs:
// fine while an expert has a handful of tokens (the layer is then bound by the weight stream,
// Section 3.1, Eq. 2: the b T term), but with B*k/N of 16 and more the a B k term takes over and the
// vector ALUs, not HBM, set the latency.  Here a weight tile meets 16 tokens per instruction
// instead: v_mfma_f32_16x16x32_bf16 multiplies 16 weight rows x 32 columns with the same 32
// entries of 16 token vectors (bf16 products, fp32 accumulation).
//
// Work unit of a wavefront: 16 rows of W_gate AND W_up of one expert (gate/up stage), or 32 rows
// of W_down (down stage), over the whole inner dimension, against up to 64 tokens of that expert
// at a time (accumulators for 4 groups of 16 tokens x 2 weight tiles stay in registers; an expert
// with more tokens takes further passes over the same rows).  Weight operands come straight from
// memory in the instruction's operand layout (lane l: row l % 16, columns 8 (l / 16) .. + 8 of the
// step's 32), requested several steps ahead with streaming loads; token operands (x or h rows of
// the expert's pairs, gathered through the pair list) come the same way and mostly hit in the
// caches, since the eight wavefronts of a workgroup work on neighbouring rows of the same expert.
// Results leave the registers directly: silu(gate) * up rounded to the storage type into h, or
// gate-weighted atomic adds into out (Eq. 1).
#include "oea_ffn_dev.h"

namespace oea {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kDenseMaxGroups = 4;  // groups of 16 tokens per pass
constexpr int kDenseStep = 32;      // columns per matrix-core instruction

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

__device__ __forceinline__ uint4 load_plain16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// One unit against the pairs [pair0, pair0 + cnt) of its expert, cnt <= 16 * NG.  LOOK steps of
// operands are in flight; loads are issued and consumed in the same order, so the in-order
// completion of the memory counter costs nothing.
template <int STAGE, int NG, int LOOK>
__device__ __forceinline__ void dense_unit(const DenseParams& p, int e, int row0, int pair0, int cnt, int lane) {
  const int r = lane & 15, q = lane >> 4;
  const int L = p.L, rows = p.rows;
  const uint16_t* pa[2];
  {
    const size_t base = ((size_t)e * rows + (size_t)(row0 + r)) * L + q * 8;
    pa[0] = p.wa + base;
    pa[1] = STAGE == 0 ? p.wb + base : p.wa + base + (size_t)16 * L;
  }
  const uint16_t* pb[NG];
  int pair_of[NG];
#pragma unroll
  for (int c = 0; c < NG; ++c) {
    const int n = c * 16 + r;
    // lanes past the last token read a valid row; their result columns are never stored
    int pi = pair0 + (n < cnt ? n : 0);
    pi = pi < 0 ? 0 : (pi >= p.pairs_max ? p.pairs_max - 1 : pi);
    pair_of[c] = pi;
    int vrow = pi;
    if (STAGE == 0) {
      vrow = p.g.grp_tok[pi];
      vrow = vrow < 0 ? 0 : (vrow >= p.B ? p.B - 1 : vrow);
    }
    pb[c] = p.vec + (size_t)vrow * L + q * 8;
  }

  uint4 a[LOOK][2], b[LOOK][NG];
  f32x4_t acc[NG][2];
#pragma unroll
  for (int c = 0; c < NG; ++c) acc[c][0] = acc[c][1] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  auto request = [&](int s, int step) {
#pragma unroll
    for (int m = 0; m < 2; ++m) a[s][m] = load_stream16(pa[m] + (size_t)step * kDenseStep);
#pragma unroll
    for (int c = 0; c < NG; ++c) b[s][c] = load_plain16(pb[c] + (size_t)step * kDenseStep);
  };
  auto multiply = [&](int s) {
#pragma unroll
    for (int c = 0; c < NG; ++c) {
      const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, b[s][c]);
#pragma unroll
      for (int m = 0; m < 2; ++m)
        acc[c][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[s][m]), bv, acc[c][m], 0, 0, 0);
    }
  };

  const int steps = L / kDenseStep;  // a multiple of LOOK (launcher)
#pragma unroll
  for (int s = 0; s < LOOK; ++s) request(s, s);
  for (int kk = 0; kk + LOOK < steps; kk += LOOK) {
#pragma unroll
    for (int s = 0; s < LOOK; ++s) {
      multiply(s);
      request(s, kk + LOOK + s);
      __builtin_amdgcn_sched_barrier(0);  // a slot is refilled as soon as it is free, not at the end of the round
    }
  }
#pragma unroll
  for (int s = 0; s < LOOK; ++s) multiply(s);

  // the lane holds rows 4 q .. 4 q + 3 of each tile for token r of each group
#pragma unroll
  for (int c = 0; c < NG; ++c) {
    const int n = c * 16 + r;
    if (n < cnt) {
      const int pi = pair_of[c];
      if (STAGE == 0) {
        uint16_t hv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float gsum = acc[c][0][j], usum = acc[c][1][j];
          hv[j] = f32_to_bf16_rne(gsum / (1.f + __expf(-gsum)) * usum);
        }
        uint2 packed;
        packed.x = uint32_t(hv[0]) | (uint32_t(hv[1]) << 16);
        packed.y = uint32_t(hv[2]) | (uint32_t(hv[3]) << 16);
        *reinterpret_cast<uint2*>(p.h_out + (size_t)pi * rows + row0 + 4 * q) = packed;
      } else {
        int orow = pi;
        if (!p.per_pair) {
          orow = p.g.grp_tok[pi];
          orow = orow < 0 ? 0 : (orow >= p.B ? p.B - 1 : orow);
        }
        const float gw = p.g.grp_gw[pi];
        float* const o = p.out + (size_t)orow * rows + row0 + 4 * q;
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
          for (int j = 0; j < 4; ++j) unsafeAtomicAdd(o + 16 * m + j, gw * acc[c][m][j]);
      }
    }
  }
}

template <int STAGE>
__global__ __launch_bounds__(kFfnThreads) void expert_dense_kernel(DenseParams p) {
  __shared__ int l_active[OEA_MAX_N];
  __shared__ int l_off[OEA_MAX_N + 1];
  __shared__ uint32_t l_next;
  const int tid = threadIdx.x, lane = tid & 63;
  const int N = p.N;
  int T = *p.g.n_active;
  T = T < 0 ? 0 : (T > N ? N : T);
  for (int i = tid; i < N; i += kFfnThreads) {
    const int e = i < T ? p.g.active_list[i] : 0;
    l_active[i] = e < 0 ? 0 : (e >= N ? N - 1 : e);
  }
  for (int i = tid; i <= N; i += kFfnThreads) l_off[i] = p.g.grp_off[i <= T ? i : T];
  if (tid == 0) l_next = 0;
  __syncthreads();

  // units of this workgroup: a contiguous, equal share of all active experts' row blocks; its
  // wavefronts take them one by one from a counter
  constexpr int kUnitRows = STAGE == 0 ? 16 : 32;
  const int upe = p.rows / kUnitRows;
  const long long U = (long long)T * upe;
  const int u0 = int(U * blockIdx.x / gridDim.x), u1 = int(U * (blockIdx.x + 1) / gridDim.x);
  for (;;) {
    uint32_t t = 0;
    if (lane == 0) t = atomicAdd(&l_next, 1u);
    const int u = u0 + __builtin_amdgcn_readfirstlane(int(t));
    if (u >= u1) break;
    const int a = u / upe;
    const int row0 = (u - a * upe) * kUnitRows;
    const int e = l_active[a];
    const int off = l_off[a], cnt = l_off[a + 1] - off;
    if (off < 0 || cnt <= 0 || off + cnt > p.pairs_max) continue;  // never true after a valid routing
    for (int q0 = 0; q0 < cnt; q0 += 16 * kDenseMaxGroups) {
      const int rem = cnt - q0;
      const int here = rem < 16 * kDenseMaxGroups ? rem : 16 * kDenseMaxGroups;
      const int groups = (here + 15) >> 4;
      if (groups == 1)
        dense_unit<STAGE, 1, 8>(p, e, row0, off + q0, here, lane);
      else if (groups == 2)
        dense_unit<STAGE, 2, 8>(p, e, row0, off + q0, here, lane);
      else if (groups == 3)
        dense_unit<STAGE, 3, 4>(p, e, row0, off + q0, here, lane);
      else
        dense_unit<STAGE, 4, 4>(p, e, row0, off + q0, here, lane);
    }
  }
}

}  // namespace

// One expert stage (0 gate/up, 1 down) on the matrix cores; hipErrorNotSupported for storage types
// and shapes it is not built for (bf16; rows a multiple of the unit, inner dimension of 256).
hipError_t try_launch_dense_stage(int stage, const void* vec, const void* wa, const void* wb, void* h_out, float* out,
                                  int B, int d, int N, int I, int k, oea_dtype dt, Grouping g, bool per_pair,
                                  hipStream_t s) {
  if (dt != OEA_BF16 || N > OEA_MAX_N) return hipErrorNotSupported;
  const int rows = stage == 0 ? I : d, L = stage == 0 ? d : I;
  if (rows % (stage == 0 ? 16 : 32) != 0 || L % (8 * kDenseStep) != 0) return hipErrorNotSupported;
  int dev = 0, grid = 0;
  if (!current_device(&dev, &grid)) return hipErrorUnknown;
  if (grid < 1) return hipErrorNotSupported;
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
  if (stage == 0)
    hipLaunchKernelGGL(expert_dense_kernel<0>, dim3(grid), dim3(kFfnThreads), 0, s, p);
  else
    hipLaunchKernelGGL(expert_dense_kernel<1>, dim3(grid), dim3(kFfnThreads), 0, s, p);
  return hipGetLastError();
}

}  // namespace oea
