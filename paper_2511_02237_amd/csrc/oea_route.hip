// Router GEMV + OEA routing kernels (gfx950): the stand-alone routing entry point and the first
// kernel of the three-kernel layer path.  The routing itself is in oea_route_dev.h.
#include "oea_route_dev.h"

namespace oea {

namespace {

constexpr int kRouteThreads = 1024;
constexpr int kWideFromBatch = 128;  // larger batches route over many workgroups (see wide_logits_kernel)

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

// ---------------------------------------------------------------------------------------------
// Batches above 128 tokens: router and routing over many workgroups, as four kernels in stream
// order (a kernel boundary is the grid-wide synchronisation Algorithm 1 needs twice: the union of
// Phase 1 before Phase 2, all pair counts before the grouped lists).  The union and the counts live
// in control words of the workspace that the first kernel clears.  With one workgroup per expert
// for the logits and one workgroup routing the whole batch this step took 50 / 104 / 230 us at
// B = 256 / 512 / 1024.
//
// 1. wide_logits_kernel: a workgroup of four wavefronts computes the logits of 8 tokens x 16 experts,
//    each wavefront a 4 x 8 block: operands are widened to fp64 once per block and multiplied with
//    fused multiply-adds (a bf16 or fp32 product is exact in fp64, so this is the same arithmetic,
//    in the same order, as the other router kernels: the same bits), 1.75 instructions per
//    multiply-add instead of 3.  It also clears a slice of what the down stage adds into, and the
//    control words of the routing kernels that follow.
constexpr int kWideThreads = 256;

// element q of a 16-byte piece, widened to fp64 (exact)
template <typename WT>
__device__ __forceinline__ double widen_elem(const uint4& v, int q);
template <>
__device__ __forceinline__ double widen_elem<uint16_t>(const uint4& v, int q) {
  const uint32_t w = q < 2 ? v.x : q < 4 ? v.y : q < 6 ? v.z : v.w;
  return double((q & 1) ? __uint_as_float(w & 0xffff0000u) : bf16_bits_to_f32(w & 0xffffu));
}
template <>
__device__ __forceinline__ double widen_elem<float>(const uint4& v, int q) {
  return double(__uint_as_float(q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w));
}

template <typename WT>
__global__ __launch_bounds__(kWideThreads) void wide_logits_kernel(const WT* __restrict__ x,
                                                                   const WT* __restrict__ w_router,
                                                                   const float* __restrict__ bias, int B, int d, int N,
                                                                   float* logits, float* out_to_zero, size_t n_zero,
                                                                   uint32_t* ctrl, int32_t* n_active) {
  constexpr int EPL = 16 / int(sizeof(WT));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wg = blockIdx.y * gridDim.x + blockIdx.x, n_wg = gridDim.x * gridDim.y;
  {
    const size_t total4 = n_zero / 4;
    const size_t per = (total4 + n_wg - 1) / n_wg;
    const size_t lo = per * wg, hi = lo + per < total4 ? lo + per : total4;
    float4* o4 = reinterpret_cast<float4*>(out_to_zero);
    for (size_t i = lo + tid; i < hi; i += kWideThreads) o4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (ctrl[kCtrlMagicWord] != kWsMagic) {  // unprepared workspace: an empty routing, out = 0
    if (wg == 0 && tid == 0) *n_active = 0;
    return;
  }
  if (wg == 0) {
    if (tid < 16) ctrl[kCtrlWideUnion + tid] = 0u;
    for (int i = tid; i < N; i += kWideThreads) ctrl[kCtrlWideCount + i * wide_count_stride(N)] = 0u;
  }
  const int t0 = blockIdx.x * 8 + (wave >> 1) * 4, e0 = blockIdx.y * 16 + (wave & 1) * 8;
  if (t0 >= B || e0 >= N) return;
  double acc[4][8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.0;
  for (int c = lane * EPL; c < d; c += 64 * EPL) {
    uint4 a[4], b[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int t = t0 + i < B ? t0 + i : B - 1;
      a[i] = *reinterpret_cast<const uint4*>(x + (size_t)t * d + c);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int e = e0 + j < N ? e0 + j : N - 1;
      b[j] = *reinterpret_cast<const uint4*>(w_router + (size_t)e * d + c);
    }
#pragma unroll
    for (int q = 0; q < EPL; ++q) {  // element by element: every sum takes its terms in ascending order
      double af[4], bf[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) af[i] = widen_elem<WT>(a[i], q);
#pragma unroll
      for (int j = 0; j < 8; ++j) bf[j] = widen_elem<WT>(b[j], q);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = fma(af[i], bf[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] += __shfl_xor(acc[i][j], off, 64);
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (t0 + i < B && e0 + j < N)
          logits[(size_t)(t0 + i) * N + e0 + j] = float(acc[i][j] + (bias ? double(bias[e0 + j]) : 0.0));
  }
}

// 2. wide_phase1_kernel: a wavefront per token takes its k0 best experts (Phase 1 of Algorithm 1; with
//    GEN the baseline of Algorithm 2: cut where the cumulative softmax mass, fp64, reaches p, its size
//    parked in n_sel for the next kernel); the workgroup's four tokens are united in LDS first, and
//    only bits that the union in memory does not show yet are added there (one atomic per token and
//    pick on the same few words serialises: 60 us at B = 1024).
template <int NV, bool GEN>
__global__ __launch_bounds__(kWideThreads) void wide_phase1_kernel(const float* __restrict__ logits,
                                                                    const uint8_t* __restrict__ token_mask, int B, int N,
                                                                    int k0, RouteGeneral g, uint32_t* ctrl, int32_t* n_sel) {
  __shared__ uint32_t s_u[16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int t = blockIdx.x * (kWideThreads / 64) + (tid >> 6);
  if (ctrl[kCtrlMagicWord] != kWsMagic) return;
  if (tid < 16) s_u[tid] = 0u;
  __syncthreads();
  if (t < B) {
    const bool live = !(token_mask && token_mask[t] == 0);
    int n = 0;
    if (live) {
      uint32_t key[NV];
      float lg[NV];
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int e = lane + 64 * j;
        lg[j] = e < N ? logits[(size_t)t * N + e] : 0.f;
        key[j] = e < N ? make_key(lg[j]) : 0;
      }
      const bool capped = GEN && g.p < 1.0;
      double m = 0.0, z = 1.0;
      if (capped) {  // softmax denominator over all N experts
        uint32_t lm = key[0];
#pragma unroll
        for (int j = 1; j < NV; ++j) lm = key[j] > lm ? key[j] : lm;
        m = double(from_orderable(wave_max_u32(lm)));
        double zl = 0.0;
#pragma unroll
        for (int j = 0; j < NV; ++j)
          if (key[j] != 0) zl += exp(double(lg[j]) - m);
        z = wave_sum_f64(zl);
      }
      double cum = 0.0;
      for (int r = 0; r < k0; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        if (lane == 0) atomicOr(&s_u[id >> 5], 1u << (id & 31));
        ++n;
        if (capped) {
          cum += exp(double(from_orderable(bk)) - m) / z;
          if (cum >= g.p) break;
        }
      }
    }
    if (GEN && lane == 0) n_sel[t] = n;
  }
  __syncthreads();
  if (tid < 16) {
    uint32_t* const gu = ctrl + kCtrlWideUnion + tid;
    const uint32_t fresh = s_u[tid] & ~__hip_atomic_load(gu, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (fresh) atomicOr(gu, fresh);
  }
}

// 3. wide_phase2_kernel: a wavefront per token takes its best members of the union, up to k (Phase 2
//    in closed form; with GEN the baseline again, then the walk over the ranks below max_p of
//    Algorithm 2), computes the weights of Eq. 1, and draws a place in each chosen expert's group
//    from that expert's counter (kept in grp_pos until the last kernel knows where the group starts;
//    the counters lie on cache lines of their own where they fit: side by side, their atomics took
//    16 us at B = 1024 instead of 5).
//    The order of the pairs inside a group is the order of arrival: nothing depends on it.
template <int NV, bool GEN>
__global__ __launch_bounds__(kWideThreads) void wide_phase2_kernel(const float* __restrict__ logits,
                                                                    const uint8_t* __restrict__ token_mask, int B, int N,
                                                                    int k, RouteGeneral g, uint32_t* ctrl, RouteOut o) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * (kWideThreads / 64) + (threadIdx.x >> 6);
  if (ctrl[kCtrlMagicWord] != kWsMagic || t >= B) return;
  const bool live = !(token_mask && token_mask[t] == 0);
  const uint32_t* U = ctrl + kCtrlWideUnion;
  auto in_union = [&](int e) { return e < N && ((U[e >> 5] >> (e & 31)) & 1u); };
  uint32_t key[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int e = lane + 64 * j;
    const bool cand = live && e < N && (GEN || in_union(e));
    key[j] = cand ? make_key(logits[(size_t)t * N + e]) : 0;
  }
  int n = 0, my_id = -1;
  float my_logit = 0.f;
  auto take = [&](int id, uint32_t bk) __attribute__((always_inline)) {
    if (lane == n) {
      my_id = id;
      my_logit = from_orderable(bk);
    }
    ++n;
  };
  if (!GEN) {
    for (int r = 0; r < k; ++r) {
      uint32_t bk;
      int id;
      if (!pick_best<NV>(key, lane, bk, id)) break;
      take(id, bk);
    }
  } else {
    const int nbase = live ? o.n_sel[t] : 0;
    if (g.max_p >= N) {
      // no window: after the baseline, the piggybacked experts are the best remaining members of the union
      for (int r = 0; r < nbase; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        take(id, bk);
      }
#pragma unroll
      for (int j = 0; j < NV; ++j)
        if (!in_union(lane + 64 * j)) key[j] = 0;
      while (n < g.k_max) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        take(id, bk);
      }
    } else {
      // walk the ranks in order; an expert outside the union uses up its rank without being taken
      const int last = nbase > g.max_p ? nbase : g.max_p;
      for (int r = 0; r < last; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        if (r < nbase) {
          take(id, bk);
        } else {
          if (n >= g.k_max) break;
          if (in_union(id)) take(id, bk);
        }
      }
    }
  }
  // g_s = exp(l_s - m) / sum_{s'} exp(l_s' - m): the softmax denominator cancels in Eq. 1
  const float m = __shfl(my_logit, 0, 64);
  const float w = lane < n ? expf(my_logit - m) : 0.f;
  const float z = wave_sum_f32(w);
  if (lane < k) {
    o.expert_idx[(size_t)t * k + lane] = lane < n ? my_id : -1;
    o.gate_w[(size_t)t * k + lane] = lane < n ? w / z : 0.f;
    uint32_t* const counter_of_mine = ctrl + kCtrlWideCount + (lane < n ? my_id : 0) * wide_count_stride(N);
    o.grp_pos[(size_t)t * k + lane] = lane < n ? int(atomicAdd(counter_of_mine, 1u)) : -1;
  }
  if (lane == 0) o.n_sel[t] = n;
}

// 4. wide_group_kernel: every workgroup derives the active list and the group offsets from the union
//    and the counts (workgroup 0 writes them out), then sends its share of the pairs to their places.
__global__ __launch_bounds__(kRouteThreads) void wide_group_kernel(int B, int N, int k, const uint32_t* ctrl, RouteOut o) {
  __shared__ int s_off[OEA_MAX_N];   // first pair of expert e's group
  __shared__ int s_wave[2][kRouteThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (ctrl[kCtrlMagicWord] != kWsMagic) return;
  // thread e: member of the union?  how many pairs?  (N <= 512 <= threads)
  const bool member = tid < N && ((ctrl[kCtrlWideUnion + (tid >> 5)] >> (tid & 31)) & 1u);
  const int cnt = member ? int(ctrl[kCtrlWideCount + tid * wide_count_stride(N)]) : 0;
  const int inc_m = wave_incl_scan_i32(member ? 1 : 0, lane), inc_c = wave_incl_scan_i32(cnt, lane);
  if (lane == 63) {
    s_wave[0][wave] = inc_m;
    s_wave[1][wave] = inc_c;
  }
  __syncthreads();
  int base_m = 0, base_c = 0, T = 0, total = 0;
  for (int w = 0; w < kRouteThreads / 64; ++w) {
    if (w < wave) {
      base_m += s_wave[0][w];
      base_c += s_wave[1][w];
    }
    T += s_wave[0][w];
    total += s_wave[1][w];
  }
  const int a = base_m + inc_m - 1, off = base_c + inc_c - cnt;
  if (tid < N) s_off[tid] = off;
  if (blockIdx.x == 0) {
    if (member) {
      o.active_list[a] = tid;
      o.grp_off[a] = off;
    }
    if (tid >= T && tid < N) o.active_list[tid] = -1;
    if (tid == 0) {
      *o.n_active = T;
      o.grp_off[T] = total;
    }
  }
  __syncthreads();
  const int P = B * k;
  for (int i = blockIdx.x * kRouteThreads + tid; i < P; i += gridDim.x * kRouteThreads) {
    const int e = o.expert_idx[i];
    if (e >= 0 && e < N) {
      const int dst = s_off[e] + o.grp_pos[i];
      if (dst >= 0 && dst < P) {  // always true; bounds the stores
        o.grp_tok[dst] = i / k;
        o.grp_gw[dst] = o.gate_w[i];
        o.grp_pos[i] = dst;
      }
    }
  }
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
  if (B > kWideFromBatch && o.grp_off && o.grp_tok && o.grp_gw && o.grp_pos) {
    // large batch: router and routing over many workgroups, four kernels in stream order
    const int per_wg = kWideThreads / 64;  // a wavefront per token; small workgroups spread them over the compute units
    hipLaunchKernelGGL((wide_logits_kernel<WT>), dim3((B + 7) / 8, (N + 15) / 16), dim3(kWideThreads), 0, s,
                       static_cast<const WT*>(x), static_cast<const WT*>(w_router), bias, B, d, N, logits, out_to_zero,
                       n_zero, counter, o.n_active);
    switch (nv_for(N)) {
#define OEA_CASE(NV)                                                                                           \
  case NV:                                                                                                     \
    if (general) {                                                                                             \
      hipLaunchKernelGGL((wide_phase1_kernel<NV, true>), dim3((B + per_wg - 1) / per_wg), dim3(kWideThreads),  \
                         0, s, logits, token_mask, B, N, k0, g, counter, o.n_sel);                             \
      hipLaunchKernelGGL((wide_phase2_kernel<NV, true>), dim3((B + per_wg - 1) / per_wg), dim3(kWideThreads),  \
                         0, s, logits, token_mask, B, N, k, g, counter, o);                                    \
    } else {                                                                                                   \
      hipLaunchKernelGGL((wide_phase1_kernel<NV, false>), dim3((B + per_wg - 1) / per_wg),                     \
                         dim3(kWideThreads), 0, s, logits, token_mask, B, N, k0, g, counter, o.n_sel);        \
      hipLaunchKernelGGL((wide_phase2_kernel<NV, false>), dim3((B + per_wg - 1) / per_wg),                     \
                         dim3(kWideThreads), 0, s, logits, token_mask, B, N, k, g, counter, o);               \
    }                                                                                                          \
    break;
      OEA_CASE(1)
      OEA_CASE(2)
      OEA_CASE(4)
      OEA_CASE(8)
#undef OEA_CASE
    }
    const int group_wgs = (B * k + 2 * kRouteThreads - 1) / (2 * kRouteThreads);
    hipLaunchKernelGGL(wide_group_kernel, dim3(group_wgs), dim3(kRouteThreads), 0, s, B, N, k, counter, o);
    return hipGetLastError();
  }
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
