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

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    uint64_t o = __shfl_xor(v, off, 64);
    v = o > v ? o : v;
  }
  return v;
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

// Executed by ONE workgroup of kRouteThreads threads.  lds: see route_lds_bytes().
template <int NV>
__device__ void route_block(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                            int B, int N, int k, int k0, RouteOut o, uint32_t* lds) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NW = (N + 31) >> 5;
  uint32_t* U = lds;              // [16] union bit mask
  uint32_t* scan = lds + 16;      // [48] scratch for block scans
  uint32_t* selmask = lds + 64;   // [B*NW] per-token membership of the final sets

  for (int i = tid; i < 64 + B * NW; i += kRouteThreads) lds[i] = 0;
  __syncthreads();

  // ---- pass 1: Phase 1 of Algorithm 1, S_i^base = k0 best experts; U = union over the batch
  for (int t = wave; t < B; t += kRouteWaves) {
    if (token_mask && token_mask[t] == 0) continue;
    uint64_t key[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      int e = lane + 64 * j;
      key[j] = e < N ? make_key(logits[(size_t)t * N + e], uint32_t(e)) : 0;
    }
    for (int r = 0; r < k0; ++r) {
      uint64_t best = pick_best<NV>(key, lane);
      if (best == 0) break;
      uint32_t id = 0xffffffffu - uint32_t(best);
      if (lane == 0) atomicOr(&U[id >> 5], 1u << (id & 31));
    }
  }
  __syncthreads();

  // ---- pass 2: Phase 2 in closed form: top-k of the logits restricted to U, then weights
  for (int t = wave; t < B; t += kRouteWaves) {
    int n = 0;
    int my_id = -1;
    float my_logit = 0.f;
    if (!(token_mask && token_mask[t] == 0)) {
      uint64_t key[NV];
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        int e = lane + 64 * j;
        bool cand = e < N && ((U[e >> 5] >> (e & 31)) & 1u);
        key[j] = cand ? make_key(logits[(size_t)t * N + e], uint32_t(e)) : 0;
      }
      for (int r = 0; r < k; ++r) {
        uint64_t best = pick_best<NV>(key, lane);
        if (best == 0) break;
        if (lane == r) {
          my_id = int(0xffffffffu - uint32_t(best));
          my_logit = from_orderable(uint32_t(best >> 32));
        }
        ++n;
      }
    }
    // g_s = exp(l_s - m) / sum_{s'} exp(l_s' - m): the softmax denominator cancels in Eq. 1
    float m = __shfl(my_logit, 0, 64);
    float w = lane < n ? expf(my_logit - m) : 0.f;
    float z = wave_sum_f32(w);
    if (lane < k) {
      o.expert_idx[(size_t)t * k + lane] = lane < n ? my_id : -1;
      o.gate_w[(size_t)t * k + lane] = lane < n ? w / z : 0.f;
    }
    if (lane < n) atomicOr(&selmask[t * NW + (my_id >> 5)], 1u << (my_id & 31));
    if (lane == 0) o.n_sel[t] = n;
  }
  __syncthreads();

  // ---- pass 3: active list (ascending ids) and expert -> token grouping
  const int e = tid;
  const bool in_u = e < N && ((U[e >> 5] >> (e & 31)) & 1u);
  uint64_t ballot = __ballot(in_u);
  if (lane == 0) scan[wave] = uint32_t(__popcll(ballot));
  int cnt = 0;
  if (in_u)
    for (int t = 0; t < B; ++t) cnt += int((selmask[t * NW + (e >> 5)] >> (e & 31)) & 1u);
  // inclusive scan of cnt inside the wave
  int incl = cnt;
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
  if (o.grp_off) {
    if (in_u) {
      o.grp_off[pos] = excl;
      int p = excl;
      for (int t = 0; t < B; ++t) {
        if ((selmask[t * NW + (e >> 5)] >> (e & 31)) & 1u) {
          float g = 0.f;
          for (int s = 0; s < k; ++s)
            if (o.expert_idx[(size_t)t * k + s] == e) g = o.gate_w[(size_t)t * k + s];
          o.grp_tok[p] = t;
          o.grp_gw[p] = g;
          ++p;
        }
      }
    }
    if (tid == 0) o.grp_off[T] = P;
  }
}

template <int NV>
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const float* logits, const uint8_t* token_mask,
                                                              int B, int N, int k, int k0, RouteOut o) {
  extern __shared__ uint32_t lds[];
  route_block<NV>(logits, token_mask, B, N, k, k0, o, lds);
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
  route_block<NV>(logits, token_mask, B, N, k, k0, o, lds);
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

size_t route_lds_bytes(int B, int N) { return sizeof(uint32_t) * (64 + (size_t)B * ((N + 31) / 32)); }

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
