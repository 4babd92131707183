// Router GEMV + OEA routing kernels (gfx950).
//
// Routing follows Algorithm 1 of the paper in its closed form: every token's Phase-1 set is a
// subset of the union U, and the k0 best experts overall are also the k0 best inside U, so the
// final set of a token is "the min(k,|U|) best-ranked members of U".  The kernel therefore does
//   pass 1: per token (one wavefront each) top-k0 by repeated wave arg-max -> OR into a bit mask in LDS
//   barrier
//   pass 2: per token top-k of the logits restricted to U -> S_i in rank order, gate weights
//           (softmax scores renormalised over S_i: Eq. 1 / Section 3.2 "Weighting after rerouting")
//   pass 3: ascending active list, and the expert -> (token, weight) grouping the FFN kernels use.
// Ranking is on the fp32 logits, ties to the lower expert id, -0.0 equal to +0.0.
#include "oea_internal.h"

namespace oea {

namespace {

constexpr int kRouteThreads = 1024;
constexpr int kRouteWaves = kRouteThreads / 64;

__device__ __forceinline__ uint32_t orderable_bits(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u << 1) == 0u) u = 0u;  // -0.0 ranks equal to +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_orderable(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
  return __uint_as_float(u);
}

// key: larger = better rank.  High word orders by logit, low word prefers the lower expert id.
// A valid key is never 0, so 0 marks "not a candidate".
__device__ __forceinline__ uint64_t make_key(float logit, uint32_t id) {
  return (uint64_t(orderable_bits(logit)) << 32) | uint64_t(0xffffffffu - id);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return uint32_t(__builtin_amdgcn_update_dpp(0, int(v), CTRL, 0xF, 0xF, true));
}

template <int CTRL>
__device__ __forceinline__ uint64_t dpp_max_u64(uint64_t v) {
  const uint64_t o = (uint64_t(dpp_u32<CTRL>(uint32_t(v >> 32))) << 32) | dpp_u32<CTRL>(uint32_t(v));
  return o > v ? o : v;
}

// max over the 64 lanes, result in every lane: 4 DPP steps inside each row of 16, 2 cross-row steps
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
  v = dpp_max_u64<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_max_u64<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_max_u64<0x141>(v);  // row_half_mirror
  v = dpp_max_u64<0x140>(v);  // row_mirror
  uint64_t o = __shfl_xor(v, 16, 64);
  v = o > v ? o : v;
  o = __shfl_xor(v, 32, 64);
  return o > v ? o : v;
}

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// One arg-max round over the wave's candidate keys; removes the winner.  Returns 0 if none left.
template <int NV>
__device__ __forceinline__ uint64_t pick_best(uint64_t (&key)[NV], int lane) {
  uint64_t local = key[0];
#pragma unroll
  for (int j = 1; j < NV; ++j) local = key[j] > local ? key[j] : local;
  uint64_t best = wave_max_u64(local);
  if (best != 0) {
    uint32_t id = 0xffffffffu - uint32_t(best);
#pragma unroll
    for (int j = 0; j < NV; ++j)
      if (id == uint32_t(lane + 64 * j)) key[j] = 0;
  }
  return best;
}

// LDS words used by route_block
__host__ __device__ inline size_t route_lds_words(int B, int N) {
  return 64 + (size_t)N * ((B + 31) / 32) + (size_t)N;
}

// Executed by ONE workgroup of kRouteThreads threads.  lds: route_lds_words(B,N) words.
// SINGLE: B <= kRouteWaves, one token per wavefront; its candidate keys stay in registers across
// the barrier, so Phase 2 continues where Phase 1 stopped instead of starting over.
template <int NV, bool SINGLE>
__device__ void route_block(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                            int B, int N, int k, int k0, RouteOut o, uint32_t* lds) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NWB = (B + 31) >> 5;
  uint32_t* U = lds;                 // [16] union bit mask over experts
  uint32_t* scan = lds + 16;         // [48] scratch for block scans
  uint32_t* colmask = lds + 64;      // [N*NWB] per expert: bit mask of the tokens routed to it
  uint32_t* eoff = colmask + N * NWB;  // [N] per expert: first pair in the grouped order

  for (int i = tid; i < int(route_lds_words(B, N)); i += kRouteThreads) lds[i] = 0;
  __syncthreads();

  uint64_t keep[NV];  // SINGLE: this wavefront's keys after Phase 1
  int my_id = -1;     // lane r holds the expert of rank r (SINGLE: filled from Phase 1 on)
  float my_logit = 0.f;
  int n_single = 0;

  // ---- pass 1: Phase 1 of Algorithm 1, S_i^base = k0 best experts; U = union over the batch
  for (int t = wave; t < B; t += kRouteWaves) {
    const bool live = !(token_mask && token_mask[t] == 0);
    uint64_t key[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      int e = lane + 64 * j;
      key[j] = (live && e < N) ? make_key(logits[(size_t)t * N + e], uint32_t(e)) : 0;
    }
    for (int r = 0; r < k0; ++r) {
      uint64_t best = pick_best<NV>(key, lane);
      if (best == 0) break;
      uint32_t id = 0xffffffffu - uint32_t(best);
      if (lane == 0) atomicOr(&U[id >> 5], 1u << (id & 31));
      if (SINGLE) {
        if (lane == r) {
          my_id = int(id);
          my_logit = from_orderable(uint32_t(best >> 32));
        }
        ++n_single;
      }
    }
    if (SINGLE) {
#pragma unroll
      for (int j = 0; j < NV; ++j) keep[j] = key[j];
    }
  }
  __syncthreads();

  // ---- pass 2: Phase 2 in closed form: the token's best members of U up to k in all, then weights.
  // Every Phase-1 pick is in U and outranks the rest, so SINGLE just continues on the kept keys.
  for (int t = wave; t < B; t += kRouteWaves) {
    const bool live = !(token_mask && token_mask[t] == 0);
    int n = SINGLE ? n_single : 0;
    if (!SINGLE) {
      my_id = -1;
      my_logit = 0.f;
    }
    uint64_t key[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      int e = lane + 64 * j;
      bool cand = live && e < N && ((U[e >> 5] >> (e & 31)) & 1u);
      if (SINGLE)
        key[j] = cand ? keep[j] : 0;
      else
        key[j] = cand ? make_key(logits[(size_t)t * N + e], uint32_t(e)) : 0;
    }
    for (int r = n; r < k; ++r) {
      uint64_t best = pick_best<NV>(key, lane);
      if (best == 0) break;
      if (lane == r) {
        my_id = int(0xffffffffu - uint32_t(best));
        my_logit = from_orderable(uint32_t(best >> 32));
      }
      ++n;
    }
    // g_s = exp(l_s - m) / sum_{s'} exp(l_s' - m): the softmax denominator cancels in Eq. 1
    float m = __shfl(my_logit, 0, 64);
    float w = lane < n ? expf(my_logit - m) : 0.f;
    float z = wave_sum_f32(w);
    if (lane < k) {
      o.expert_idx[(size_t)t * k + lane] = lane < n ? my_id : -1;
      o.gate_w[(size_t)t * k + lane] = lane < n ? w / z : 0.f;
    }
    if (lane < n) atomicOr(&colmask[my_id * NWB + (t >> 5)], 1u << (t & 31));
    if (lane == 0) o.n_sel[t] = n;
  }
  __syncthreads();

  // ---- pass 3a: active list (ascending ids), pairs per expert, CSR offsets
  const int e = tid;
  const bool in_u = e < N && ((U[e >> 5] >> (e & 31)) & 1u);
  uint64_t ballot = __ballot(in_u);
  if (lane == 0) scan[wave] = uint32_t(__popcll(ballot));
  int cnt = 0;
  if (in_u)
    for (int w = 0; w < NWB; ++w) cnt += __popc(colmask[e * NWB + w]);
  int incl = cnt;  // inclusive scan of cnt inside the wave
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int v = __shfl_up(incl, off, 64);
    if (lane >= off) incl += v;
  }
  if (lane == 63) scan[16 + wave] = uint32_t(incl);
  __syncthreads();
  int pos_base = 0, cnt_base = 0, T = 0, P = 0;
  for (int w = 0; w < kRouteWaves; ++w) {
    int a = int(scan[w]), c = int(scan[16 + w]);
    if (w < wave) {
      pos_base += a;
      cnt_base += c;
    }
    T += a;
    P += c;
  }
  const int pos = pos_base + __popcll(ballot & ((1ull << lane) - 1ull));
  const int excl = cnt_base + incl - cnt;
  if (in_u) o.active_list[pos] = e;
  if (e < N && e >= T) o.active_list[e] = -1;
  if (tid == 0) *o.n_active = T;
  if (!o.grp_off) return;
  if (in_u) {
    o.grp_off[pos] = excl;
    eoff[e] = uint32_t(excl);
  }
  if (tid == 0) o.grp_off[T] = P;
  __syncthreads();

  // ---- pass 3b: one thread per (token, slot) pair; inside an expert, pairs are in token order
  for (int p = tid; p < B * k; p += kRouteThreads) {
    const int ex = o.expert_idx[p];
    if (ex < 0) continue;
    const int t = p / k;
    int rank = __popc(colmask[ex * NWB + (t >> 5)] & ((1u << (t & 31)) - 1u));
    for (int w = 0; w < (t >> 5); ++w) rank += __popc(colmask[ex * NWB + w]);
    const int dst = int(eoff[ex]) + rank;
    o.grp_tok[dst] = t;
    o.grp_gw[dst] = o.gate_w[p];
  }
}

template <int NV>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const float* logits, const uint8_t* token_mask,
                                                              int B, int N, int k, int k0, RouteOut o) {
  extern __shared__ uint32_t lds[];
  if (B <= kRouteWaves)
    route_block<NV, true>(logits, token_mask, B, N, k, k0, o, lds);
  else
    route_block<NV, false>(logits, token_mask, B, N, k, k0, o, lds);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// fp64 dot product of one 16-byte fragment pair
template <typename WT>
__device__ __forceinline__ double frag_dot_f64(const uint4& a, const uint4& b, double acc);

template <>
__device__ __forceinline__ double frag_dot_f64<float>(const uint4& a, const uint4& b, double acc) {
  acc = fma(double(__uint_as_float(a.x)), double(__uint_as_float(b.x)), acc);
  acc = fma(double(__uint_as_float(a.y)), double(__uint_as_float(b.y)), acc);
  acc = fma(double(__uint_as_float(a.z)), double(__uint_as_float(b.z)), acc);
  acc = fma(double(__uint_as_float(a.w)), double(__uint_as_float(b.w)), acc);
  return acc;
}

template <>
__device__ __forceinline__ double frag_dot_f64<uint16_t>(const uint4& a, const uint4& b, double acc) {
  const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // a bf16 x bf16 product is exact in fp32
    acc += double(bf16_bits_to_f32(av[i] & 0xffffu) * bf16_bits_to_f32(bv[i] & 0xffffu));
    acc += double(__uint_as_float(av[i] & 0xffff0000u) * __uint_as_float(bv[i] & 0xffff0000u));
  }
  return acc;
}

// grid = N workgroups (one per expert e), kRouteThreads threads.
//   part A: logits[t,e] = fp32( sum_c x[t,c] W_router[e,c] + bias[e] ), fp64 accumulation;
//           the workgroups also clear `out` for the atomically accumulating down-projection.
//   part B: the workgroup that arrives last at the counter routes the whole batch.
template <typename WT, int NV>
__global__ __launch_bounds__(kRouteThreads) void router_route_kernel(
    const WT* __restrict__ x, const WT* __restrict__ w_router, const float* __restrict__ bias,
    const uint8_t* token_mask, int B, int d, int N, int k, int k0, float* logits, float* out_to_zero,
    uint32_t* counter, RouteOut o) {
  extern __shared__ uint32_t lds[];
  constexpr int EPL = 16 / int(sizeof(WT));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e = blockIdx.x;

  {  // clear this workgroup's slice of out[B,d] (d is a multiple of 8, so float4 granules)
    const size_t total4 = (size_t)B * d / 4;
    const size_t per = (total4 + gridDim.x - 1) / gridDim.x;
    const size_t lo = per * e, hi = lo + per < total4 ? lo + per : total4;
    float4* o4 = reinterpret_cast<float4*>(out_to_zero);
    for (size_t i = lo + tid; i < hi; i += kRouteThreads) o4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }

  const WT* wr = w_router + (size_t)e * d;
  for (int t = wave; t < B; t += kRouteWaves) {
    const WT* xr = x + (size_t)t * d;
    double acc = 0.0;
    for (int c = lane * EPL; c < d; c += 64 * EPL) {
      uint4 a = *reinterpret_cast<const uint4*>(xr + c);
      uint4 b = *reinterpret_cast<const uint4*>(wr + c);
      acc = frag_dot_f64<WT>(a, b, acc);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
      if (bias) acc += double(bias[e]);
      logits[(size_t)t * N + e] = float(acc);
    }
  }

  // One device-scope release per workgroup (not per thread: each one writes back the L2): the barrier
  // orders every wavefront's stores before thread 0's fence, the fence before the counter update.
  __syncthreads();
  if (tid == 0) {
    __threadfence();
    uint32_t old = atomicAdd(counter, 1u);
    const bool is_last = old == gridDim.x - 1;
    if (is_last) {
      __threadfence();          // acquire: the other workgroups' logits
      atomicExch(counter, 0u);  // leave the control word zero for the next call
    }
    lds[0] = is_last ? 1u : 0u;
  }
  __syncthreads();
  const bool last = lds[0] != 0u;
  __syncthreads();
  if (!last) return;
  if (B <= kRouteWaves)
    route_block<NV, true>(logits, token_mask, B, N, k, k0, o, lds);
  else
    route_block<NV, false>(logits, token_mask, B, N, k, k0, o, lds);
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

int nv_for(int N) {
  int nv = (N + 63) / 64;
  return nv <= 1 ? 1 : nv <= 2 ? 2 : nv <= 4 ? 4 : 8;
}

}  // namespace

size_t route_lds_bytes(int B, int N) { return sizeof(uint32_t) * route_lds_words(B, N); }

hipError_t launch_fill_zero(uint32_t* p, size_t n_words, hipStream_t s) {
  if (n_words == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, s, p, n_words);
  return hipGetLastError();
}

hipError_t launch_route(const float* logits, const uint8_t* token_mask, int B, int N, int k, int k0,
                        RouteOut o, hipStream_t s) {
  const size_t lds = route_lds_bytes(B, N);
  switch (nv_for(N)) {
#define OEA_CASE(NV)                                                                                      \
  case NV: {                                                                                              \
    if (lds > 48 * 1024) {                                                                                \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&route_kernel<NV>),                \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);           \
      if (e != hipSuccess) return e;                                                                      \
    }                                                                                                     \
    hipLaunchKernelGGL(route_kernel<NV>, dim3(1), dim3(kRouteThreads), lds, s, logits, token_mask, B, N, k, \
                       k0, o);                                                                            \
  } break;
    OEA_CASE(1)
    OEA_CASE(2)
    OEA_CASE(4)
    OEA_CASE(8)
#undef OEA_CASE
  }
  return hipGetLastError();
}

template <typename WT>
static hipError_t launch_rr(const void* x, const void* w_router, const float* bias, const uint8_t* token_mask,
                            int B, int d, int N, int k, int k0, float* logits, float* out_to_zero,
                            uint32_t* counter, RouteOut o, hipStream_t s) {
  const size_t lds = route_lds_bytes(B, N);
  switch (nv_for(N)) {
#define OEA_CASE(NV)                                                                                       \
  case NV: {                                                                                               \
    if (lds > 48 * 1024) {                                                                                 \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&router_route_kernel<WT, NV>),      \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);            \
      if (e != hipSuccess) return e;                                                                       \
    }                                                                                                      \
    hipLaunchKernelGGL((router_route_kernel<WT, NV>), dim3(N), dim3(kRouteThreads), lds, s,                \
                       static_cast<const WT*>(x), static_cast<const WT*>(w_router), bias, token_mask, B, d, \
                       N, k, k0, logits, out_to_zero, counter, o);                                         \
  } break;
    OEA_CASE(1)
    OEA_CASE(2)
    OEA_CASE(4)
    OEA_CASE(8)
#undef OEA_CASE
  }
  return hipGetLastError();
}

hipError_t launch_router_and_route(const void* x, const void* w_router, const float* bias,
                                   const uint8_t* token_mask, int B, int d, int N, int k, int k0,
                                   oea_dtype dt, float* logits, float* out_to_zero, uint32_t* counter,
                                   RouteOut o, hipStream_t s) {
  if (dt == OEA_F32)
    return launch_rr<float>(x, w_router, bias, token_mask, B, d, N, k, k0, logits, out_to_zero, counter, o, s);
  return launch_rr<uint16_t>(x, w_router, bias, token_mask, B, d, N, k, k0, logits, out_to_zero, counter, o, s);
}

}  // namespace oea
