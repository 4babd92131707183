// Router GEMV + OEA routing kernels (gfx950): the stand-alone routing entry point and the first
// kernel of the three-kernel layer path.  The routing itself is in oea_route_dev.h.
#include "oea_route_dev.h"

namespace oea {

namespace {

constexpr int kRouteThreads = 1024;

// One workgroup routes one decode position (blockIdx.x): its B rows of logits and its own output slices.
// Positions are independent (Section 4: every position and layer is routed separately), so a grid
// of L workgroups routes L positions in one launch.
// NT threads (>= N): 1024 for one or few positions (most parallelism for a single routing); 256 for
// many positions of a small batch, where four wavefronts hold the 16 token rows and four times as
// many positions are resident per compute unit.
template <int NV, int NT>
__global__ __launch_bounds__(NT) void route_kernel(const float* logits, const uint8_t* token_mask, int B, int N,
                                                   int k, int k0, RouteOut o) {
  extern __shared__ uint32_t lds[];
  const size_t pos = blockIdx.x;
  logits += pos * B * N;
  if (token_mask) token_mask += pos * B;
  o.expert_idx += pos * B * k;
  o.gate_w += pos * B * k;
  o.n_sel += pos * B;
  o.active_list += pos * N;
  o.n_active += pos;
  if constexpr (NT == 256) {
    // launch_route picks this size only for NV <= 2, k <= 16, B <= 16: the row-per-token routing is
    // the only path compiled in, which keeps the kernel at 8 wavefronts per SIMD (with many
    // positions the launch is bound by how many are resident to hide each other's LDS round trips)
    RowCarry<4 * NV> c;
    route_union_rows<4 * NV, NT>(logits, token_mask, B, N, k0, o, lds, c);
    route_fill_rows<4 * NV, NT>(B, N, k, k0, o, lds, c);
  } else if (NV <= 2 && k <= 16 && B <= 4 * (NT / 64)) {
    // few experts: one DPP row of 16 lanes per token, four tokens per wavefront
    RowCarry<4 * NV> c;
    route_union_rows<4 * NV, NT>(logits, token_mask, B, N, k0, o, lds, c);
    route_fill_rows<4 * NV, NT>(B, N, k, k0, o, lds, c);
  } else if (NV <= 2 && k <= 16 && B <= 16 * (NT / 64)) {
    route_rows_groups<4 * NV, NT, 4>(logits, token_mask, B, N, k, k0, o, lds);  // up to four groups, keys kept
  } else if (NV <= 2 && k <= 16) {
    route_rows_any<4 * NV, NT>(logits, token_mask, B, N, k, k0, o, lds);
  } else if (B <= NT / 64) {
    route_block<NV, NT, 1>(logits, token_mask, B, N, k, k0, o, lds);
  } else {
    route_block<NV, NT, 0>(logits, token_mask, B, N, k, k0, o, lds);
  }
}

template <int NV>
__global__ __launch_bounds__(kRouteThreads) void route_general_kernel(const float* logits, const uint8_t* token_mask,
                                                                      int B, int N, int k0, RouteGeneral g, RouteOut o) {
  extern __shared__ uint32_t lds[];
  route_block_general<NV, kRouteThreads>(logits, token_mask, B, N, k0, g, o, lds);
}

// First kernel of the three-kernel layer.  grid = N workgroups (one per expert e), kRouteThreads threads.
//   part A: logits[t,e] = fp32( sum_c x[t,c] W_router[e,c] + bias[e] ), fp64 accumulation;
//           the workgroups also clear `out` for the atomically accumulating down-projection.
//   part B: the workgroup that arrives last at the counter routes the whole batch.
template <typename WT, int NV>
__global__ __launch_bounds__(kRouteThreads) void router_route_kernel(
    const WT* __restrict__ x, const WT* __restrict__ w_router, const float* __restrict__ bias,
    const uint8_t* token_mask, int B, int d, int N, int k, int k0, float* logits, float* out_to_zero,
    size_t n_zero, uint32_t* counter, RouteOut o, RouteGeneral g, int general) {
  extern __shared__ uint32_t lds[];
  constexpr int EPL = 16 / int(sizeof(WT));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e = blockIdx.x;
  // `counter` is the first control word of the workspace; every thread reads the same magic word
  const uint32_t magic = counter[kCtrlMagicWord];

  {  // clear this workgroup's slice of what the down projection adds into: out[B,d], or the per-pair
     // buffer of the deterministic combine (n_zero floats, a multiple of 8: float4 granules)
    const size_t total4 = n_zero / 4;
    const size_t per = (total4 + gridDim.x - 1) / gridDim.x;
    const size_t lo = per * e, hi = lo + per < total4 ? lo + per : total4;
    float4* o4 = reinterpret_cast<float4*>(out_to_zero);
    for (size_t i = lo + tid; i < hi; i += kRouteThreads) o4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }

  // A workspace that was never prepared holds an arbitrary arrival count: no workgroup would know
  // that it is the last.  The layer then ends with out = 0 and an empty routing (no active expert).
  if (magic != kWsMagic) {
    if (e == 0 && tid == 0) *o.n_active = 0;
    return;
  }

  // TB tokens at a time per wavefront: the router row chunk is loaded once for all of them and their
  // loads and reductions overlap (one token at a time was bound by load latency)
  constexpr int TB = 4;
  const WT* wr = w_router + (size_t)e * d;
  for (int t0 = wave * TB; t0 < B; t0 += (kRouteThreads / 64) * TB) {
    double acc[TB];
#pragma unroll
    for (int i = 0; i < TB; ++i) acc[i] = 0.0;
    for (int c = lane * EPL; c < d; c += 64 * EPL) {
      const uint4 b = *reinterpret_cast<const uint4*>(wr + c);
      uint4 a[TB];
#pragma unroll
      for (int i = 0; i < TB; ++i) {
        const int t = t0 + i < B ? t0 + i : B - 1;
        a[i] = *reinterpret_cast<const uint4*>(x + (size_t)t * d + c);
      }
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
        if (t0 + i < B) logits[(size_t)(t0 + i) * N + e] = float(acc[i] + (bias ? double(bias[e]) : 0.0));
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
  if (general) {
    route_block_general<NV, kRouteThreads>(logits, token_mask, B, N, k0, g, o, lds);
  } else if (NV <= 2 && k <= 16 && B <= 4 * (kRouteThreads / 64)) {
    RowCarry<4 * NV> c;  // few experts: one DPP row of 16 lanes per token
    route_union_rows<4 * NV, kRouteThreads>(logits, token_mask, B, N, k0, o, lds, c);
    route_fill_rows<4 * NV, kRouteThreads>(B, N, k, k0, o, lds, c);
  } else if (NV <= 2 && k <= 16 && B <= 16 * (kRouteThreads / 64)) {
    route_rows_groups<4 * NV, kRouteThreads, 4>(logits, token_mask, B, N, k, k0, o, lds);
  } else if (NV <= 2 && k <= 16) {
    route_rows_any<4 * NV, kRouteThreads>(logits, token_mask, B, N, k, k0, o, lds);
  } else if (B <= kRouteThreads / 64)
    route_block<NV, kRouteThreads, 1>(logits, token_mask, B, N, k, k0, o, lds);
  else
    route_block<NV, kRouteThreads, 0>(logits, token_mask, B, N, k, k0, o, lds);
}

__global__ void ws_prepare_kernel(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = i == (size_t)kCtrlMagicWord ? kWsMagic : 0u;
}

int nv_for(int N) {
  int nv = (N + 63) / 64;
  return nv <= 1 ? 1 : nv <= 2 ? 2 : nv <= 4 ? 4 : 8;
}

}  // namespace

size_t route_lds_bytes(int B, int N) { return sizeof(uint32_t) * (route_lds_words(B, N) + (size_t)B); }

hipError_t launch_ws_prepare(uint32_t* ctrl, size_t n_words, hipStream_t s) {
  if (n_words <= (size_t)kCtrlMagicWord) return hipErrorInvalidValue;
  hipLaunchKernelGGL(ws_prepare_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, s, ctrl, n_words);
  return hipGetLastError();
}

template <int NV, int NT>
static hipError_t launch_route_one(const float* logits, const uint8_t* token_mask, int L, int B, int N, int k, int k0,
                                   RouteOut o, size_t lds, hipStream_t s) {
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&route_kernel<NV, NT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((route_kernel<NV, NT>), dim3(L), dim3(NT), lds, s, logits, token_mask, B, N, k, k0, o);
  return hipGetLastError();
}

hipError_t launch_route(const float* logits, const uint8_t* token_mask, int L, int B, int N, int k, int k0,
                        RouteOut o, hipStream_t s) {
  const size_t lds = route_lds_bytes(B, N);
  // many positions of a small batch: small workgroups (the row-per-token routing needs B <= 16 for 256 threads)
  const bool small = L >= 8 && B <= 16 && N <= 128 && k <= 16;
  switch (nv_for(N)) {
    case 1: return small ? launch_route_one<1, 256>(logits, token_mask, L, B, N, k, k0, o, lds, s)
                         : launch_route_one<1, kRouteThreads>(logits, token_mask, L, B, N, k, k0, o, lds, s);
    case 2: return small ? launch_route_one<2, 256>(logits, token_mask, L, B, N, k, k0, o, lds, s)
                         : launch_route_one<2, kRouteThreads>(logits, token_mask, L, B, N, k, k0, o, lds, s);
    case 4: return launch_route_one<4, kRouteThreads>(logits, token_mask, L, B, N, k, k0, o, lds, s);
    default: return launch_route_one<8, kRouteThreads>(logits, token_mask, L, B, N, k, k0, o, lds, s);
  }
}

template <typename WT>
static hipError_t launch_rr(const void* x, const void* w_router, const float* bias, const uint8_t* token_mask,
                            int B, int d, int N, int k, int k0, float* logits, float* out_to_zero, size_t n_zero,
                            uint32_t* counter, RouteOut o, const RouteGeneralArgs* ga, hipStream_t s) {
  RouteGeneral g{1.0, k, N, nullptr};
  const int general = ga && (ga->p < 1.0 || ga->max_p < N) ? 1 : 0;
  if (general) g = RouteGeneral{ga->p, k, ga->max_p, nullptr};
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
                       N, k, k0, logits, out_to_zero, n_zero, counter, o, g, general);                     \
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
                                   oea_dtype dt, float* logits, float* to_zero, size_t n_zero, uint32_t* counter,
                                   RouteOut o, const RouteGeneralArgs* ga, hipStream_t s) {
  if (dt == OEA_F32)
    return launch_rr<float>(x, w_router, bias, token_mask, B, d, N, k, k0, logits, to_zero, n_zero, counter, o, ga, s);
  return launch_rr<uint16_t>(x, w_router, bias, token_mask, B, d, N, k, k0, logits, to_zero, n_zero, counter, o, ga, s);
}

hipError_t launch_route_general(const float* logits, const uint8_t* token_mask, int B, int N, int k0,
                                const RouteGeneralArgs& ga, int32_t* n_base, RouteOut o, hipStream_t s) {
  const size_t lds = route_lds_bytes(B, N);
  const RouteGeneral g{ga.p, ga.k_max, ga.max_p, n_base};
  switch (nv_for(N)) {
#define OEA_CASE(NV)                                                                                        \
  case NV: {                                                                                                \
    if (lds > 48 * 1024) {                                                                                  \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&route_general_kernel<NV>),          \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);             \
      if (e != hipSuccess) return e;                                                                        \
    }                                                                                                       \
    hipLaunchKernelGGL(route_general_kernel<NV>, dim3(1), dim3(kRouteThreads), lds, s, logits, token_mask, B, \
                       N, k0, g, o);                                                                        \
  } break;
    OEA_CASE(1)
    OEA_CASE(2)
    OEA_CASE(4)
    OEA_CASE(8)
#undef OEA_CASE
  }
  return hipGetLastError();
}

}  // namespace oea
