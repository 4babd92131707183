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
#include "oea_internal.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace oea {

namespace {

constexpr int kFfnThreads = 512;
constexpr int kFfnWaves = kFfnThreads / 64;
constexpr size_t kLdsBudget = 128 * 1024;  // bytes of LDS used for the staged token vectors

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// sum over the LPR consecutive lanes that share one weight row; every lane gets the total
template <int LPR>
__device__ __forceinline__ float row_sum(float v) {
  v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);  // row_half_mirror
  v += dpp_move<0x140>(v);  // row_mirror
  if (LPR >= 32) v += __shfl_xor(v, 16, 64);
  if (LPR >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

template <typename WT>
__device__ __forceinline__ float frag_dot(const uint4& w, const uint4& v, float acc);

template <>
__device__ __forceinline__ float frag_dot<float>(const uint4& w, const uint4& v, float acc) {
  acc = fmaf(__uint_as_float(w.x), __uint_as_float(v.x), acc);
  acc = fmaf(__uint_as_float(w.y), __uint_as_float(v.y), acc);
  acc = fmaf(__uint_as_float(w.z), __uint_as_float(v.z), acc);
  acc = fmaf(__uint_as_float(w.w), __uint_as_float(v.w), acc);
  return acc;
}

template <>
__device__ __forceinline__ float frag_dot<uint16_t>(const uint4& w, const uint4& v, float acc) {
  // v_dot2c_f32_bf16: acc += w.lo*v.lo + w.hi*v.hi with fp32 accumulation
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x), __builtin_bit_cast(bf16x2_t, v.x), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y), __builtin_bit_cast(bf16x2_t, v.y), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z), __builtin_bit_cast(bf16x2_t, v.z), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w), __builtin_bit_cast(bf16x2_t, v.w), acc, false);
  return acc;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7f800000u) == 0x7f800000u) return uint16_t((u >> 16) | ((u & 0xffffu) ? 0x40u : 0u));  // inf/nan
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

__device__ __forceinline__ void store_h(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_h(uint16_t* p, float v) { *p = f32_to_bf16_rne(v); }

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
  int tok_cap;       // token vectors that fit in LDS at once
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
              w[m][rg][c] = ok ? *reinterpret_cast<const uint4*>(src) : make_uint4(0, 0, 0, 0);
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
                const int t = p.g.grp_tok[pidx];
                if ((unsigned)t < (unsigned)p.B)
                  unsafeAtomicAdd(p.out + (size_t)t * rows + row, p.g.grp_gw[pidx] * y);
              }
            }
          }
        }
      }
    }
  }
}

int g_num_cus = 0;

int num_cus() {
  if (g_num_cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      g_num_cus = prop.multiProcessorCount;
    if (g_num_cus <= 0) g_num_cus = 256;
  }
  return g_num_cus;
}

template <typename WT, int STAGE, int LPR, int NCH, int RG>
hipError_t launch_one(const FfnParams& p, size_t lds_bytes, hipStream_t s) {
  auto kern = expert_kernel<WT, STAGE, LPR, NCH, RG>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
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

template <typename WT>
hipError_t launch_stage(int stage, FfnParams p, int B, hipStream_t s) {
  // LDS: as many token vectors as fit (at most B), at least one workgroup per CU alone on its CU
  const size_t vec_bytes = (size_t)p.L * sizeof(WT);
  int cap = int(kLdsBudget / vec_bytes);
  if (cap < 1) return hipErrorInvalidValue;
  if (cap > B) cap = B;
  p.tok_cap = cap;
  size_t lds_bytes = (size_t)cap * vec_bytes;
  const size_t alone = 84 * 1024;  // more than half of the CU's 160 KB: one workgroup per CU
  if (lds_bytes < alone) lds_bytes = alone;
  constexpr int EPL = 16 / int(sizeof(WT));
  if (stage == 0) return launch_lpr<WT, 0, 16, 1>(p, lds_bytes, s);
  // down stage: one matrix, so the 32-load tile holds several row groups
  if (p.L <= 16 * EPL * 8) return launch_one<WT, 1, 16, 8, 4>(p, lds_bytes, s);
  return launch_lpr<WT, 1, 16, 2>(p, lds_bytes, s);
}

}  // namespace

hipError_t launch_expert_gate_up(const void* x, const void* w_gate, const void* w_up, void* h, int B,
                                 int d, int N, int I, int k, oea_dtype dt, Grouping g, hipStream_t s) {
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
  return dt == OEA_F32 ? launch_stage<float>(0, p, B, s) : launch_stage<uint16_t>(0, p, B, s);
}

hipError_t launch_expert_down(const void* h, const void* w_down, float* out, int B, int d, int N, int I,
                              int k, oea_dtype dt, Grouping g, hipStream_t s) {
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
  return dt == OEA_F32 ? launch_stage<float>(1, p, B, s) : launch_stage<uint16_t>(1, p, B, s);
}

}  // namespace oea
