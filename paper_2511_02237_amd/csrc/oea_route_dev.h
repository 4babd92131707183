// Device-side routing code shared by the routing kernels and the fused layer kernel (gfx950).
//
// Routing follows Algorithm 1 of the paper in its closed form: every token's Phase-1 set is a
// subset of the union U, and the k0 best experts overall are also the k0 best inside U, so the
// final set of a token is "the min(k,|U|) best-ranked members of U".  route_block does
//   pass 1: per token (one wavefront each) top-k0 by repeated wave arg-max -> OR into a bit mask in LDS
//   barrier
//   pass 2: per token the best members of U up to k -> S_i in rank order, gate weights
//           (softmax scores renormalised over S_i: Eq. 1 / Section 3.2 "Weighting after rerouting")
//   pass 3: ascending active list, and the expert -> (token, weight) grouping the FFN kernels use.
// Ranking is on the fp32 logits, ties to the lower expert id, -0.0 equal to +0.0.
//
// Variants, all with the same results:
//   route_block             one wavefront per token, any N <= 512 (routing kernels, large expert counts)
//   route_union_rows +      one DPP row of 16 lanes per token, four tokens per wavefront, N <= 128,
//   route_fill_rows         B <= 4 * wavefronts: the single-kernel layer (B <= 32) and the routing kernels
//   route_rows_groups / _any  the same for more tokens, in groups of 4 * wavefronts
//   route_rows_general      Algorithm 2 (top-p cut, rank window) in the row form, for the single-kernel layer
//   route_block_general     Algorithm 2, one wavefront per token (routing kernels)
// The row forms end in route_rows_finish / route_group_with: gate weights, token masks per expert,
// CSR offsets (one wavefront), pair lists (from the rows' registers).
#pragma once
#include "oea_internal.h"

#include "oea_timeline.h"

#include <type_traits>

namespace oea {
namespace {

__device__ __forceinline__ uint32_t orderable_bits(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u << 1) == 0u) u = 0u;  // -0.0 ranks equal to +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_orderable(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
  return __uint_as_float(u);
}

// Ranking key of a logit: its order-preserving bit pattern; larger = better rank.  0 marks "not a
// candidate" (only one negative-NaN pattern maps to 0, and routing of NaN logits is unspecified).
// Equal keys are separated by expert id when the winner is looked up (lowest id first).
__device__ __forceinline__ uint32_t make_key(float logit) { return orderable_bits(logit); }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max_u32(uint32_t v) {
  const uint32_t o = uint32_t(__builtin_amdgcn_update_dpp(0, int(v), CTRL, 0xF, 0xF, true));
  return o > v ? o : v;
}

// max over the 64 lanes as a wave-uniform value: 4 DPP steps inside each row of 16 lanes, then the
// four row results are read into scalar registers and compared there
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = dpp_max_u32<0xB1>(v);   // quad_perm [1,0,3,2]
  v = dpp_max_u32<0x4E>(v);   // quad_perm [2,3,0,1]
  v = dpp_max_u32<0x141>(v);  // row_half_mirror
  v = dpp_max_u32<0x140>(v);  // row_mirror
  uint32_t m = 0;
#pragma unroll
  for (int row = 0; row < 4; ++row) {
    const uint32_t r = uint32_t(__builtin_amdgcn_readlane(int(v), row * 16));
    m = r > m ? r : m;
  }
  return m;
}

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// One arg-max round over the wave's candidate keys (lane l, slot j holds expert l + 64 j); removes
// the winner.  Returns false if no candidate is left; else the winner's key and expert id (uniform).
template <int NV>
__device__ __forceinline__ bool pick_best(uint32_t (&key)[NV], int lane, uint32_t& best_key, int& best_id) {
  uint32_t local = key[0];
#pragma unroll
  for (int j = 1; j < NV; ++j) local = key[j] > local ? key[j] : local;
  const uint32_t m = wave_max_u32(local);
  if (m == 0) return false;
  int id = -1;  // equal keys: the lowest expert id wins
#pragma unroll
  for (int j = NV - 1; j >= 0; --j) {
    const uint64_t hit = __ballot(key[j] == m);
    if (hit != 0) id = 64 * j + int(__builtin_ctzll(hit));
  }
#pragma unroll
  for (int j = 0; j < NV; ++j)
    if (id == lane + 64 * j) key[j] = 0;
  best_key = m;
  best_id = id;
  return true;
}

// LDS words used by route_block
__host__ __device__ inline size_t route_lds_words(int B, int N) {
  return 64 + (size_t)N * ((B + 31) / 32) + (size_t)N;
}

// inclusive prefix sum over the 64 lanes: shifts inside each row of 16 lanes by DPP (zero shifted in),
// then the three row totals are added through scalar registers
template <int CTRL>
__device__ __forceinline__ int dpp_shr_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ int wave_incl_scan_i32(int v, int lane) {
  v += dpp_shr_i32<0x111>(v);  // row_shr:1
  v += dpp_shr_i32<0x112>(v);  // row_shr:2
  v += dpp_shr_i32<0x114>(v);  // row_shr:4
  v += dpp_shr_i32<0x118>(v);  // row_shr:8
  const int r0 = __builtin_amdgcn_readlane(v, 15), r1 = __builtin_amdgcn_readlane(v, 31);
  const int r2 = __builtin_amdgcn_readlane(v, 47);
  const int row = lane >> 4;
  return v + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

// the same with the row totals passed on by DPP broadcasts (lane 15 of a row to the next row, lane 31
// to the upper two rows) instead of scalar registers: six dependent steps, no lane reads
__device__ __forceinline__ int wave_incl_scan_dpp_i32(int v) {
  v += dpp_shr_i32<0x111>(v);  // row_shr:1
  v += dpp_shr_i32<0x112>(v);  // row_shr:2
  v += dpp_shr_i32<0x114>(v);  // row_shr:4
  v += dpp_shr_i32<0x118>(v);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

// Tail of the first half: the members of the union bit mask U (lds[0..15]) in ascending order ->
// o.active_list, their number -> *o.n_active.  Called by all NT threads after a barrier that
// completes U; the results are complete after the caller's next barrier.
// Expert e is handled by thread ebase + e (ebase a multiple of 64): with ebase > 0 the wavefronts
// below it have nothing to do here and go on at once.
template <int NT>
__device__ __forceinline__ void route_active(int N, RouteOut o, uint32_t* lds, int ebase = 0) {
  const int e = int(threadIdx.x) - ebase;
  if (e < 0) return;
  const uint32_t* U = lds;
  // position of expert e among the members = members below it, counted from the mask words
  // themselves (at most 16 of them): no scan across the wavefronts, no barrier
  const int nw = (N + 31) >> 5;
  int T = 0, pos = 0;
  for (int w = 0; w < nw; ++w) {
    const int c = __popc(U[w]);
    T += c;
    pos += w < (e >> 5) ? c : 0;
  }
  const uint32_t mine = e < N ? U[e >> 5] : 0u;
  const bool in_u = (mine >> (e & 31)) & 1u;
  pos += __popc(mine & ((1u << (e & 31)) - 1u));
  if (in_u) o.active_list[pos] = e;
  if (e < N && e >= T) o.active_list[e] = -1;
  if (e == 0) *o.n_active = T;
}


// Tail of the second half: pairs per expert (from the token bit masks colmask), CSR offsets by
// position in the active list, and the grouped (token, weight) lists.  Called by all NT threads
// after a barrier that completes colmask, o.expert_idx and o.gate_w.
// after_offsets() runs in every thread once the CSR offsets are complete (after the barrier that
// publishes them), beside the loop that fills the pair lists: work that needs only the offsets
// (the fused kernel cuts its rows there) overlaps with that loop.
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};
// What the offsets need from the union mask alone (complete since the end of Phase 1): computed
// before the barrier that ends Phase 2, by the threads that will compute the offsets after it.
// N <= 128: ONE wavefront (the one of thread ebase) computes the offsets, lane l those of experts
// 2l and 2l+1, with a single scan.  Larger N: thread e expert e, scan across the wavefronts.
struct GroupPre {
  int e;           // this thread's (first) expert; < 0: none
  int T;           // members of U
  int pos;         // members below e
  bool in_u, in1;  // e, e + 1 (N <= 128 only) is a member
};
template <int NT>
__device__ __forceinline__ GroupPre route_group_pre(int N, const uint32_t* lds, int ebase) {
  GroupPre g{-1, 0, 0, false, false};
  const int rel = int(threadIdx.x) - ebase;
  if (N <= 128) {
    if (rel < 0 || rel >= 64) return g;
    g.e = 2 * rel;
  } else {
    g.e = rel;  // ebase == 0
  }
  const uint32_t* U = lds;
  const int nw = (N + 31) >> 5;
  for (int w = 0; w < nw; ++w) {
    const int c = __popc(U[w]);
    g.T += c;
    g.pos += w < (g.e >> 5) ? c : 0;
  }
  const uint32_t mine = g.e < N ? U[g.e >> 5] : 0u;  // e even: e + 1 is in the same word
  g.in_u = (mine >> (g.e & 31)) & 1u;
  g.in1 = N <= 128 && g.e + 1 < N && ((mine >> ((g.e + 1) & 31)) & 1u);
  g.pos += __popc(mine & ((1u << (g.e & 31)) - 1u));
  return g;
}
// LISTS = false: the caller fills the pair lists itself (route_fill_rows does, from registers).
template <int NT, typename Hook = NoHook, bool LISTS = true>
__device__ __forceinline__ void route_group_with(int B, int N, int k, RouteOut o, uint32_t* lds, const GroupPre g,
                                                 Hook after_offsets = Hook()) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NWB = (B + 31) >> 5;
  uint32_t* scan = lds + 16;
  uint32_t* colmask = lds + 64;
  uint32_t* eoff = colmask + N * NWB;
  if (!o.grp_off) return;
  // ---- pairs per expert, CSR offsets by position in the active list
  const int e = g.e, T = g.T, pos = g.pos;
  const bool in_u = g.in_u;
  if (N <= 128) {
    if (e >= 0) {  // one wavefront
      // unconditional reads at clamped addresses (experts >= N have no words), all in flight together
      const uint32_t* m0 = colmask + (e < N ? e : N - 1) * NWB;
      const uint32_t* m1 = colmask + (e + 1 < N ? e + 1 : N - 1) * NWB;
      int c0 = __popc(m0[0]), c1 = __popc(m1[0]);
      for (int w = 1; w < NWB; ++w) {
        c0 += __popc(m0[w]);
        c1 += __popc(m1[w]);
      }
      c0 = in_u ? c0 : 0;
      c1 = g.in1 ? c1 : 0;
      const int incl = wave_incl_scan_dpp_i32(c0 + c1);
      const int excl0 = incl - c0 - c1, excl1 = excl0 + c0;
      if (in_u) {
        o.grp_off[pos] = excl0;
        eoff[e] = uint32_t(excl0);
      }
      if (g.in1) {
        o.grp_off[pos + (in_u ? 1 : 0)] = excl1;
        eoff[e + 1] = uint32_t(excl1);
      }
      if (lane == 63) o.grp_off[T] = incl;  // all pairs
    }
  } else {  // thread base 0 (see route_union_rows): e == tid
    int cnt = 0;
    if (in_u)
      for (int w = 0; w < NWB; ++w) cnt += __popc(colmask[e * NWB + w]);
    const int incl = wave_incl_scan_i32(cnt, lane);
    if (lane == 63) scan[16 + wave] = uint32_t(incl);
    __syncthreads();
    int cnt_base = 0, P = 0;
    for (int w = 0; w < NW; ++w) {
      const int cw = int(scan[16 + w]);
      cnt_base += w < wave ? cw : 0;
      P += cw;
    }
    const int excl = cnt_base + incl - cnt;
    if (tid == 0) o.grp_off[T] = P;
    if (in_u) {
      o.grp_off[pos] = excl;
      eoff[e] = uint32_t(excl);
    }
  }
  __syncthreads();
  OEA_TL(6);
  after_offsets();

  if (!LISTS) return;
  // ---- one thread per (token, slot) pair; inside an expert, pairs are in token order
  for (int p = tid; p < B * k; p += NT) {
    const int ex = o.expert_idx[p];
    if (ex < 0) {
      if (o.grp_pos) o.grp_pos[p] = -1;
      continue;
    }
    const int t = p / k;
    int rank = __popc(colmask[ex * NWB + (t >> 5)] & ((1u << (t & 31)) - 1u));
    for (int w = 0; w < (t >> 5); ++w) rank += __popc(colmask[ex * NWB + w]);
    const int dst = int(eoff[ex]) + rank;
    o.grp_tok[dst] = t;
    o.grp_gw[dst] = o.gate_w[p];
    if (o.grp_pos) o.grp_pos[p] = dst;
  }
}
template <int NT, typename Hook = NoHook>
__device__ __forceinline__ void route_group(int B, int N, int k, RouteOut o, uint32_t* lds, Hook after_offsets = Hook()) {
  route_group_with<NT>(B, N, k, o, lds, route_group_pre<NT>(N, lds, 0), after_offsets);
}


// Routing state that a wavefront carries from the first half of route_block to the second.
template <int NV, int TPW>
struct RouteCarry {
  static constexpr int TP = TPW > 0 ? TPW : 1;
  uint32_t keep[TP][NV];  // TPW > 0: the wavefront's candidate keys after Phase 1
  int sel_id[TP];         // lane r holds the expert of rank r
  float sel_logit[TP];
  int sel_n[TP];
};

// Executed by ONE workgroup of NT threads (NT/64 wavefronts, NT >= N).  lds: route_lds_words(B,N) words.
// TPW > 0 (requires B <= TPW * NT/64): every wavefront owns at most TPW tokens and keeps their
// candidate keys in registers across the barrier, so Phase 2 continues where Phase 1 stopped.
// TPW == 0: any B; Phase 2 starts over from the logits.
// The RouteOut pointers may point to global memory or to LDS.
//
// First half: Phase 1 of Algorithm 1 and the union.  On return (after the caller's next
// __syncthreads) o.active_list and *o.n_active are complete: everything the expert stages need to
// know WHICH weights will be read.
template <int NV, int NT, int TPW>
__device__ __forceinline__ void route_union(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                                            int B, int N, int k0, RouteOut o, uint32_t* lds,
                                            RouteCarry<NV, TPW>& c) {
  constexpr int NW = NT / 64;
  constexpr int TP = RouteCarry<NV, TPW>::TP;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t* U = lds;  // [16] union bit mask over experts ([16..63]: scratch for block scans)

  for (int i = tid; i < int(route_lds_words(B, N)); i += NT) lds[i] = 0;
  __syncthreads();
  OEA_TL(3);

  // ---- pass 1: Phase 1 of Algorithm 1, S_i^base = k0 best experts; U = union over the batch
  if (TPW > 0) {
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      const int t = wave + i * NW;
      const bool live = t < B && !(token_mask && token_mask[t] == 0);
      c.sel_n[i] = 0;
      c.sel_id[i] = -1;
      c.sel_logit[i] = 0.f;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        int e = lane + 64 * j;
        c.keep[i][j] = (live && e < N) ? make_key(logits[(size_t)(live ? t : 0) * N + e]) : 0;
      }
    }
    // rounds outside, tokens inside: the wavefront's tokens form independent dependency chains
    for (int r = 0; r < k0; ++r) {
#pragma unroll
      for (int i = 0; i < TP; ++i) {
        uint32_t bk;
        int id;
        if (pick_best<NV>(c.keep[i], lane, bk, id)) {
          if (lane == 0) atomicOr(&U[id >> 5], 1u << (id & 31));
          if (lane == r) {
            c.sel_id[i] = id;
            c.sel_logit[i] = from_orderable(bk);
          }
          ++c.sel_n[i];
        }
      }
    }
  } else {
    for (int t = wave; t < B; t += NW) {
      const bool live = !(token_mask && token_mask[t] == 0);
      uint32_t key[NV];
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        int e = lane + 64 * j;
        key[j] = (live && e < N) ? make_key(logits[(size_t)t * N + e]) : 0;
      }
      for (int r = 0; r < k0; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        if (lane == 0) atomicOr(&U[id >> 5], 1u << (id & 31));
      }
    }
  }
  __syncthreads();
  OEA_TL(4);

  route_active<NT>(N, o, lds);
}

// Second half: Phase 2 in closed form (the token's best members of U up to k in all), the weights of
// Eq. 1, and the expert -> (token, weight) grouping.  Needs a __syncthreads between route_union and
// this call only if o.active_list / o.n_active are read in between; its own barriers order the rest.
template <int NV, int NT, int TPW>
__device__ __forceinline__ void route_fill(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                                           int B, int N, int k, int k0, RouteOut o, uint32_t* lds,
                                           RouteCarry<NV, TPW>& c) {
  constexpr int NW = NT / 64;
  constexpr int TP = RouteCarry<NV, TPW>::TP;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NWB = (B + 31) >> 5;
  uint32_t* U = lds;
  uint32_t* colmask = lds + 64;  // [N*NWB] per expert: bit mask of the tokens routed to it ([N] more: CSR scratch)

  // Every Phase-1 pick is in U and outranks the rest, so with kept keys Phase 2 just continues.
  auto finish = [&](int t, int n, int my_id, float my_logit) __attribute__((always_inline)) {
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
  };
  if (TPW > 0) {
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        int e = lane + 64 * j;
        bool cand = e < N && ((U[e >> 5] >> (e & 31)) & 1u);
        if (!cand) c.keep[i][j] = 0;
      }
    for (int r = k0; r < k; ++r) {  // every live token holds exactly k0 picks here
#pragma unroll
      for (int i = 0; i < TP; ++i) {
        uint32_t bk;
        int id;
        if (pick_best<NV>(c.keep[i], lane, bk, id)) {
          if (lane == c.sel_n[i]) {
            c.sel_id[i] = id;
            c.sel_logit[i] = from_orderable(bk);
          }
          ++c.sel_n[i];
        }
      }
    }
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      const int t = wave + i * NW;
      if (t < B) finish(t, c.sel_n[i], c.sel_id[i], c.sel_logit[i]);
    }
  } else {
    for (int t = wave; t < B; t += NW) {
      const bool live = !(token_mask && token_mask[t] == 0);
      uint32_t key[NV];
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        int e = lane + 64 * j;
        bool cand = live && e < N && ((U[e >> 5] >> (e & 31)) & 1u);
        key[j] = cand ? make_key(logits[(size_t)t * N + e]) : 0;
      }
      int n = 0, my_id = -1;
      float my_logit = 0.f;
      for (int r = 0; r < k; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        if (lane == r) {
          my_id = id;
          my_logit = from_orderable(bk);
        }
        ++n;
      }
      finish(t, n, my_id, my_logit);
    }
  }
  __syncthreads();
  OEA_TL(5);
  route_group<NT>(B, N, k, o, lds);
}

// ---------------------------------------------------------------------------------------------
// Row-per-token variant for small expert counts (N <= 16*NK, k <= 16, B <= 4*NT/64): a token is
// handled by one DPP row of 16 lanes (lane li of the row holds the keys of experts li + 16 j), so a
// wavefront ranks four tokens with the same instructions, and a round of the arg-max is pure vector
// code: row-wide max of the keys, then row-wide min of the expert ids that hold that key (ties go to
// the lower id), no scalar round trip and no branch.  Token t sits in wavefront t / RPW, row t % RPW.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_min_u32(uint32_t v) {
  const uint32_t o = uint32_t(__builtin_amdgcn_update_dpp(0, int(v), CTRL, 0xF, 0xF, true));
  return o < v ? o : v;
}
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v) {  // all 16 lanes of a row get the row's max
  v = dpp_max_u32<0xB1>(v);
  v = dpp_max_u32<0x4E>(v);
  v = dpp_max_u32<0x141>(v);
  v = dpp_max_u32<0x140>(v);
  return v;
}
__device__ __forceinline__ uint32_t row_min_u32(uint32_t v) {
  v = dpp_min_u32<0xB1>(v);
  v = dpp_min_u32<0x4E>(v);
  v = dpp_min_u32<0x141>(v);
  v = dpp_min_u32<0x140>(v);
  return v;
}
__device__ __forceinline__ float row_sum_f32(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));
  return v;
}

__device__ __forceinline__ double row_sum_f64(double v) {  // the two halves travel by DPP
  auto step = [&](auto ctrl) __attribute__((always_inline)) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), decltype(ctrl)::value, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), decltype(ctrl)::value, 0xF, 0xF, true);
    v += __hiloint2double(hi, lo);
  };
  step(std::integral_constant<int, 0xB1>());
  step(std::integral_constant<int, 0x4E>());
  step(std::integral_constant<int, 0x141>());
  step(std::integral_constant<int, 0x140>());
  return v;
}

template <int NK>
struct RowCarry {
  uint32_t key[NK];  // candidate keys of the row's token (0 = taken / not a candidate)
  uint32_t sel_id;   // lane r of the row: expert of rank r
  uint32_t sel_key;  // and its key
  uint32_t top_key;  // key of rank 0 (every lane of the row)
  int n;             // picks so far (every lane of the row)
  int t;             // the row's token, -1 if none
  bool any;          // wave-uniform: some row of this wavefront holds a token
  int ebase;         // workgroup-uniform: thread ebase + e does the per-expert bookkeeping of expert e
};

// The data path of one round for eight keys per lane, as one block of machine code: m = the row's
// best key, win = the lowest expert id holding it, and that expert's key cleared.  Same steps as the
// generic code in row_pick; what differs is the order of the instructions.  On gfx950 a select may
// not read a lane mask that a compare wrote less than two instructions earlier, and the compiler
// pairs every compare with its select (two idle issue slots per pair, an idle slot costs as much as
// an instruction: 32 of a round's 98 slots).  Here the eight compares of a step write eight masks
// first and the selects follow.  The idle slots that remain (s_nop 1) are the two a DPP operand
// needs after the instruction that wrote it.
__device__ __forceinline__ void row_pick_core8(uint32_t (&key)[8], const uint32_t (&id)[8], uint32_t& m,
                                               uint32_t& win) {
  uint32_t t, u;
  unsigned long long s0, s1, s2, s3, s4, s5, s6, s7;
  asm("v_max3_u32 %[t], %[k0], %[k1], %[k2]\n"
      "v_max3_u32 %[u], %[k3], %[k4], %[k5]\n"
      "v_max3_u32 %[t], %[t], %[k6], %[k7]\n"
      "v_max_u32 %[t], %[t], %[u]\n"
      "s_nop 1\n"
      "v_max_u32_dpp %[t], %[t], %[t] quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      "s_nop 1\n"
      "v_max_u32_dpp %[t], %[t], %[t] quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      "s_nop 1\n"
      "v_max_u32_dpp %[t], %[t], %[t] row_half_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      "s_nop 1\n"
      "v_max_u32_dpp %[m], %[t], %[t] row_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      // lowest id among this lane's keys equal to m (0xffff: none), then the lowest of the row
      "v_cmp_eq_u32 %[s7], %[k7], %[m]\n"
      "v_cmp_eq_u32 %[s6], %[k6], %[m]\n"
      "v_cmp_eq_u32 %[s5], %[k5], %[m]\n"
      "v_cmp_eq_u32 %[s4], %[k4], %[m]\n"
      "v_cmp_eq_u32 %[s3], %[k3], %[m]\n"
      "v_cmp_eq_u32 %[s2], %[k2], %[m]\n"
      "v_cmp_eq_u32 %[s1], %[k1], %[m]\n"
      "v_cmp_eq_u32 %[s0], %[k0], %[m]\n"
      "v_mov_b32 %[u], 0xffff\n"
      "v_cndmask_b32 %[u], %[u], %[i7], %[s7]\n"
      "v_cndmask_b32 %[u], %[u], %[i6], %[s6]\n"
      "v_cndmask_b32 %[u], %[u], %[i5], %[s5]\n"
      "v_cndmask_b32 %[u], %[u], %[i4], %[s4]\n"
      "v_cndmask_b32 %[u], %[u], %[i3], %[s3]\n"
      "v_cndmask_b32 %[u], %[u], %[i2], %[s2]\n"
      "v_cndmask_b32 %[u], %[u], %[i1], %[s1]\n"
      "v_cndmask_b32 %[u], %[u], %[i0], %[s0]\n"
      "s_nop 1\n"
      "v_min_u32_dpp %[u], %[u], %[u] quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      "s_nop 1\n"
      "v_min_u32_dpp %[u], %[u], %[u] quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      "s_nop 1\n"
      "v_min_u32_dpp %[u], %[u], %[u] row_half_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      "s_nop 1\n"
      "v_min_u32_dpp %[w], %[u], %[u] row_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1\n"
      // clear the winner's key
      "v_cmp_ne_u32 %[s0], %[i0], %[w]\n"
      "v_cmp_ne_u32 %[s1], %[i1], %[w]\n"
      "v_cmp_ne_u32 %[s2], %[i2], %[w]\n"
      "v_cmp_ne_u32 %[s3], %[i3], %[w]\n"
      "v_cmp_ne_u32 %[s4], %[i4], %[w]\n"
      "v_cmp_ne_u32 %[s5], %[i5], %[w]\n"
      "v_cmp_ne_u32 %[s6], %[i6], %[w]\n"
      "v_cmp_ne_u32 %[s7], %[i7], %[w]\n"
      "v_cndmask_b32 %[k0], 0, %[k0], %[s0]\n"
      "v_cndmask_b32 %[k1], 0, %[k1], %[s1]\n"
      "v_cndmask_b32 %[k2], 0, %[k2], %[s2]\n"
      "v_cndmask_b32 %[k3], 0, %[k3], %[s3]\n"
      "v_cndmask_b32 %[k4], 0, %[k4], %[s4]\n"
      "v_cndmask_b32 %[k5], 0, %[k5], %[s5]\n"
      "v_cndmask_b32 %[k6], 0, %[k6], %[s6]\n"
      "v_cndmask_b32 %[k7], 0, %[k7], %[s7]\n"
      : [k0] "+v"(key[0]), [k1] "+v"(key[1]), [k2] "+v"(key[2]), [k3] "+v"(key[3]), [k4] "+v"(key[4]),
        [k5] "+v"(key[5]), [k6] "+v"(key[6]), [k7] "+v"(key[7]), [t] "=&v"(t), [u] "=&v"(u), [m] "=&v"(m),
        [w] "=&v"(win), [s0] "=&s"(s0), [s1] "=&s"(s1), [s2] "=&s"(s2), [s3] "=&s"(s3), [s4] "=&s"(s4),
        [s5] "=&s"(s5), [s6] "=&s"(s6), [s7] "=&s"(s7)
      : [i0] "v"(id[0]), [i1] "v"(id[1]), [i2] "v"(id[2]), [i3] "v"(id[3]), [i4] "v"(id[4]), [i5] "v"(id[5]),
        [i6] "v"(id[6]), [i7] "v"(id[7]));
}

// one round for all rows: pick the best remaining candidate of every row's token, store it at rank
// `rank` (wave-uniform).  ALONE: the wavefront has its SIMD (nearly) to itself, as in a workgroup
// that fills a compute unit; the hand-scheduled block is then a quarter faster.  With many
// wavefronts per SIMD (many small workgroups) the idle slots of the compiler's code are filled by
// the other wavefronts and its shorter encodings win by 3 %.
template <int NK, bool ALONE = true>
__device__ __forceinline__ void row_pick(RowCarry<NK>& c, int li, int rank) {
  uint32_t m, win;
#ifndef OEA_ROW_PICK_PLAIN  // (build switch: the compiler's code everywhere, for comparison)
  if constexpr (NK == 8 && ALONE) {
    uint32_t id[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) id[j] = uint32_t(li + 16 * j);
    row_pick_core8(c.key, id, m, win);
  } else
#endif
  {
    uint32_t lm = c.key[0];
#pragma unroll
    for (int j = 1; j < NK; ++j) lm = c.key[j] > lm ? c.key[j] : lm;
    m = row_max_u32(lm);
    uint32_t cand = 0xffffu;  // lowest expert id among this lane's keys equal to m
#pragma unroll
    for (int j = NK - 1; j >= 0; --j) cand = c.key[j] == m ? uint32_t(li + 16 * j) : cand;
    win = row_min_u32(cand);
#pragma unroll
    for (int j = 0; j < NK; ++j) c.key[j] = uint32_t(li + 16 * j) == win ? 0u : c.key[j];
  }
  const bool valid = m != 0;
  if (valid && li == rank) {
    c.sel_id = win;
    c.sel_key = m;
  }
  if (rank == 0) c.top_key = m;
  c.n += valid ? 1 : 0;
}

// COHERENT: the logits were written by other workgroups of the same launch (device-coherent stores);
// they are read with device-coherent loads instead of plain ones.
template <int NK, int NT, bool COHERENT = false>
__device__ __forceinline__ void route_union_rows(const float* __restrict__ logits,
                                                 const uint8_t* __restrict__ token_mask, int B, int N, int k0,
                                                 RouteOut o, uint32_t* lds, RowCarry<NK>& c) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, row = lane >> 4;
  // rows in use per wavefront: four as soon as that leaves wavefronts without tokens.  The rounds
  // are bound by instruction issue, and the wavefronts of a workgroup share four SIMDs in turn
  // (wavefront w on SIMD w % 4): tokens packed into the first wavefronts run one wavefront per SIMD
  // (B=16: 3.5 instead of 3.9 us per routing)
  const int RPW = B <= NW / 2 ? 1 : 4;
  uint32_t* U = lds;

  for (int i = tid; i < int(route_lds_words(B, N)); i += NT) lds[i] = 0;
  const int t = wave * RPW + row;
  const bool have = row < RPW && t < B;
  const bool live = have && !(token_mask && token_mask[t] == 0);
  c.t = have ? t : -1;
  c.any = wave * RPW < B;
  // Wavefronts without tokens, if there are enough of them for one thread per expert, do the
  // per-expert bookkeeping (active list, offsets) beside the selection rounds of the others
  const int nbusy = (B + RPW - 1) / RPW;
  c.ebase = (N <= 128 && (NW - nbusy) * 64 >= N) ? nbusy * 64 : 0;
  c.n = 0;
  c.sel_id = 0;
  c.sel_key = 0;
  c.top_key = 0;
  float lg[NK];
#pragma unroll
  for (int j = 0; j < NK; ++j) {  // unconditional loads (clamped address): all in flight together
    const int e = li + 16 * j;
    const float* src = logits + (size_t)(live ? t : 0) * N + (e < N ? e : N - 1);
    lg[j] = COHERENT ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *src;
  }
#pragma unroll
  for (int j = 0; j < NK; ++j) c.key[j] = (live && li + 16 * j < N) ? make_key(lg[j]) : 0;
  __syncthreads();  // U is cleared
  OEA_TL(3);
  // ---- Phase 1 of Algorithm 1: S_i^base = the k0 best experts (wavefronts without tokens leave
  // the SIMDs to the others)
  if (c.any) {
    for (int r = 0; r < k0; ++r) row_pick<NK, (NT > 256)>(c, li, r);
    if (li < c.n) atomicOr(&U[c.sel_id >> 5], 1u << (c.sel_id & 31));
  }
  __syncthreads();
  OEA_TL(4);
  route_active<NT>(N, o, lds, c.ebase);
}

// Common tail of the row-per-token routings, entered with every row's selection complete (lane r of
// a row: expert and key of rank r; c.n picks): gate weights, the selection written out, the
// token masks per expert, then (after the barrier) offsets and pair lists.  gp: see route_group_pre.
template <int NK, int NT, typename Hook = NoHook>
__device__ __forceinline__ void route_rows_finish(int B, int N, int k, RouteOut o, uint32_t* lds, RowCarry<NK>& c,
                                                  const GroupPre gp, Hook after_offsets = Hook()) {
  const int li = threadIdx.x & 15;
  const int NWB = (B + 31) >> 5;
  uint32_t* colmask = lds + 64;
  float gate = 0.f;
  if (c.any) {
    // weights: g_s = exp(l_s - l_top) / sum_s' exp(l_s' - l_top) (Eq. 1; the softmax denominator cancels)
    const float w = li < c.n ? expf(from_orderable(c.sel_key) - from_orderable(c.top_key)) : 0.f;
    const float z = row_sum_f32(w);
    gate = li < c.n ? w / z : 0.f;
    if (c.t >= 0) {
      const int t = c.t;
      if (li < k) {
        o.expert_idx[(size_t)t * k + li] = li < c.n ? int(c.sel_id) : -1;
        o.gate_w[(size_t)t * k + li] = gate;
      }
      if (li < c.n) atomicOr(&colmask[c.sel_id * NWB + (t >> 5)], 1u << (t & 31));
      if (li == 0) o.n_sel[t] = c.n;
    }
  }
  __syncthreads();
  OEA_TL(5);
  // The pair lists straight from the rows' registers: lane r of a token's row holds its pair of
  // rank r.  Its place inside the expert's group (tokens in ascending order) comes from the token
  // masks, which are complete here; only the expert's offset has to wait for the next barrier.
  const bool pair = c.any && c.t >= 0 && li < c.n && o.grp_off;
  int rank = 0;
  if (c.any) {
    const int t = pair ? c.t : 0;
    const uint32_t* cm = colmask + (pair ? int(c.sel_id) : 0) * NWB;
    rank = __popc(cm[t >> 5] & ((1u << (t & 31)) - 1u));
    for (int wd = 0; wd < (t >> 5); ++wd) rank += __popc(cm[wd]);
  }
  route_group_with<NT, Hook, false>(B, N, k, o, lds, gp, after_offsets);
  if (c.any && o.grp_off) {
    const uint32_t* eoff = colmask + N * NWB;
    if (pair) {
      const int dst = int(eoff[c.sel_id]) + rank;
      o.grp_tok[dst] = c.t;
      o.grp_gw[dst] = gate;
      if (o.grp_pos) o.grp_pos[(size_t)c.t * k + li] = dst;
    } else if (o.grp_pos && c.t >= 0 && li < k) {
      o.grp_pos[(size_t)c.t * k + li] = -1;
    }
  }
}

template <int NK, int NT, typename Hook = NoHook>
__device__ __forceinline__ void route_fill_rows(int B, int N, int k, int k0, RouteOut o, uint32_t* lds,
                                                RowCarry<NK>& c, Hook after_offsets = Hook()) {
  const int li = threadIdx.x & 15;
  uint32_t* U = lds;
  const GroupPre gp = route_group_pre<NT>(N, lds, c.ebase);
  // ---- Phase 2 in closed form: continue on the candidates that are in U, up to k picks.
  // A live token holds exactly k0 picks here (k0 <= N), so the next rank is the round number.
  if (c.any) {
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      // expert li + 16 j (< 16*NK <= 512: inside U's 16 words): word j/2, bit li + 16 (j%2)
      if (!((U[j >> 1] >> (li + 16 * (j & 1))) & 1u)) c.key[j] = 0;
    }
    for (int r = k0; r < k; ++r) row_pick<NK, (NT > 256)>(c, li, r);
  }
  route_rows_finish<NK, NT>(B, N, k, o, lds, c, gp, after_offsets);
}

template <int NV, int NT, int TPW>
__device__ void route_block(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                            int B, int N, int k, int k0, RouteOut o, uint32_t* lds) {
  RouteCarry<NV, TPW> c;
  route_union<NV, NT, TPW>(logits, token_mask, B, N, k0, o, lds, c);
  route_fill<NV, NT, TPW>(logits, token_mask, B, N, k, k0, o, lds, c);
}

// Row-per-token routing for any B: the tokens are taken in groups of 4*NT/64 (four per wavefront).
// Nothing is carried between the phases; Phase 2 is the closed form on its own (the k best members
// of U, which contain the baseline).  N <= 16*NK, k <= 16.
template <int NK, int NT, bool COHERENT = false>
__device__ void route_rows_any(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask, int B,
                               int N, int k, int k0, RouteOut o, uint32_t* lds) {
  constexpr int GROUP = 4 * (NT / 64);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, row = lane >> 4;
  const int NWB = (B + 31) >> 5;
  uint32_t* U = lds;
  uint32_t* colmask = lds + 64;
  // the logits of the row's token in group t0 (clamped addresses: every lane loads, all in flight
  // together).  COHERENT: see route_union_rows.  The next group's are requested before the current
  // group's selection rounds, so that only the first load of each phase is waited for.
  auto load_group = [&](float (&lg)[NK], int t0) __attribute__((always_inline)) {
    const int t = t0 + wave * 4 + row;
    const float* src = logits + (size_t)(t < B ? t : B - 1) * N;
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      const int e = li + 16 * j;
      const float* q = src + (e < N ? e : N - 1);
      lg[j] = COHERENT ? __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *q;
    }
  };

  float cur[NK], nxt[NK];
  load_group(cur, 0);
  for (int i = tid; i < int(route_lds_words(B, N)); i += NT) lds[i] = 0;
  __syncthreads();
  for (int t0 = 0; t0 < B; t0 += GROUP) {  // ---- Phase 1: baselines and their union
    // after the last group: the first group again, for Phase 2
    load_group(nxt, t0 + GROUP < B ? t0 + GROUP : 0);
    const int t = t0 + wave * 4 + row;
    const bool live = t < B && !(token_mask && token_mask[t] == 0);
    RowCarry<NK> c;
    c.n = 0;
    c.sel_id = c.sel_key = c.top_key = 0;
#pragma unroll
    for (int j = 0; j < NK; ++j) c.key[j] = (live && li + 16 * j < N) ? make_key(cur[j]) : 0;
    for (int r = 0; r < k0; ++r) row_pick<NK>(c, li, r);
    if (li < c.n) atomicOr(&U[c.sel_id >> 5], 1u << (c.sel_id & 31));
#pragma unroll
    for (int j = 0; j < NK; ++j) cur[j] = nxt[j];
  }
  __syncthreads();
  route_active<NT>(N, o, lds);
  for (int t0 = 0; t0 < B; t0 += GROUP) {  // ---- Phase 2 in closed form, weights
    if (t0 + GROUP < B) load_group(nxt, t0 + GROUP);
    const int t = t0 + wave * 4 + row;
    const bool have = t < B;
    const bool live = have && !(token_mask && token_mask[t] == 0);
    RowCarry<NK> c;
    c.n = 0;
    c.sel_id = c.sel_key = c.top_key = 0;
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      const int e = li + 16 * j;
      const bool cand = live && e < N && ((U[e >> 5] >> (e & 31)) & 1u);
      c.key[j] = cand ? make_key(cur[j]) : 0;
    }
    for (int r = 0; r < k; ++r) row_pick<NK>(c, li, r);
    const float w = li < c.n ? expf(from_orderable(c.sel_key) - from_orderable(c.top_key)) : 0.f;
    const float z = row_sum_f32(w);
    if (have) {
      if (li < k) {
        o.expert_idx[(size_t)t * k + li] = li < c.n ? int(c.sel_id) : -1;
        o.gate_w[(size_t)t * k + li] = li < c.n ? w / z : 0.f;
      }
      if (li < c.n) atomicOr(&colmask[c.sel_id * NWB + (t >> 5)], 1u << (t & 31));
      if (li == 0) o.n_sel[t] = c.n;
    }
#pragma unroll
    for (int j = 0; j < NK; ++j) cur[j] = nxt[j];
  }
  __syncthreads();
  route_group<NT>(B, N, k, o, lds);
}

// The same for up to MAXG token groups with the candidate keys of ALL groups in registers (as
// route_union_rows / route_fill_rows hold one group's): the logits are read once, Phase 2 continues
// after the k0 picks of Phase 1 instead of starting over.  B <= MAXG * 4 * NT/64.
template <int NK, int NT, int MAXG, bool COHERENT = false>
__device__ void route_rows_groups(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask, int B,
                                  int N, int k, int k0, RouteOut o, uint32_t* lds) {
  constexpr int GROUP = 4 * (NT / 64);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, row = lane >> 4;
  const int NWB = (B + 31) >> 5;
  uint32_t* U = lds;
  uint32_t* colmask = lds + 64;
  auto load_group = [&](float (&lg)[NK], int t0) __attribute__((always_inline)) {
    const int t = t0 + wave * 4 + row;
    const float* src = logits + (size_t)(t < B ? t : B - 1) * N;
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      const int e = li + 16 * j;
      const float* q = src + (e < N ? e : N - 1);
      lg[j] = COHERENT ? __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *q;
    }
  };

  // The groups' selection rounds are independent chains of dependent instructions: they are
  // interleaved round by round, which hides most of each chain's latency.
  RowCarry<NK> c[MAXG];
  for (int i = tid; i < int(route_lds_words(B, N)); i += NT) lds[i] = 0;
#pragma unroll
  for (int g = 0; g < MAXG; ++g) {
    if (g * GROUP < B) {  // uniform over the workgroup
      float lg[NK];
      load_group(lg, g * GROUP);
      const int t = g * GROUP + wave * 4 + row;
      const bool live = t < B && !(token_mask && token_mask[t] == 0);
      c[g].t = t < B ? t : -1;
      c[g].n = 0;
      c[g].sel_id = c[g].sel_key = c[g].top_key = 0;
#pragma unroll
      for (int j = 0; j < NK; ++j) c[g].key[j] = (live && li + 16 * j < N) ? make_key(lg[j]) : 0;
    }
  }
  __syncthreads();  // U is cleared
  for (int r = 0; r < k0; ++r) {  // ---- Phase 1: baselines
#pragma unroll
    for (int g = 0; g < MAXG; ++g)
      if (g * GROUP < B) row_pick<NK>(c[g], li, r);
  }
#pragma unroll
  for (int g = 0; g < MAXG; ++g)  // ... and their union
    if (g * GROUP < B && li < c[g].n) atomicOr(&U[c[g].sel_id >> 5], 1u << (c[g].sel_id & 31));
  __syncthreads();
  route_active<NT>(N, o, lds);
  // ---- Phase 2: continue on the candidates that are in U, up to k picks
#pragma unroll
  for (int g = 0; g < MAXG; ++g) {
    if (g * GROUP < B) {
#pragma unroll
      for (int j = 0; j < NK; ++j) {
        const int e = li + 16 * j;  // e < 16*NK <= 512: inside U's 16 words
        if (!((U[e >> 5] >> (e & 31)) & 1u)) c[g].key[j] = 0;
      }
    }
  }
  // a live token holds exactly k0 picks here (k0 <= N), so the next rank is the round number
  for (int r = k0; r < k; ++r) {
#pragma unroll
    for (int g = 0; g < MAXG; ++g)
      if (g * GROUP < B) row_pick<NK>(c[g], li, r);
  }
#pragma unroll
  for (int g = 0; g < MAXG; ++g) {
    if (g * GROUP < B) {
      const float w = li < c[g].n ? expf(from_orderable(c[g].sel_key) - from_orderable(c[g].top_key)) : 0.f;
      const float z = row_sum_f32(w);
      if (c[g].t >= 0) {
        const int t = c[g].t;
        if (li < k) {
          o.expert_idx[(size_t)t * k + li] = li < c[g].n ? int(c[g].sel_id) : -1;
          o.gate_w[(size_t)t * k + li] = li < c[g].n ? w / z : 0.f;
        }
        if (li < c[g].n) atomicOr(&colmask[c[g].sel_id * NWB + (t >> 5)], 1u << (t & 31));
        if (li == 0) o.n_sel[t] = c[g].n;
      }
    }
  }
  __syncthreads();
  route_group<NT>(B, N, k, o, lds);
}

// ---------------------------------------------------------------------------------------------
// General OEA (Algorithm 2 of the paper): the baseline of a token is cut by a top-p rule as well
// (n_i = min(k0, t_i), t_i = least t whose t best experts hold softmax mass >= p), piggybacking
// stops at k_max experts and only looks at ranks up to max_p.  p >= 1 switches the top-p cut off,
// max_p >= N the window; with both off and k_max = k this is Algorithm 1.
struct RouteGeneral {
  double p;         // top-p threshold, (0,1]
  int k_max;        // cap on |S_i| for piggybacking (a baseline larger than k_max is kept)
  int max_p;        // piggyback only from ranks <= max_p (1-based), i.e. rank indices < max_p
  int32_t* n_base;  // [B] out: n_i (may be nullptr)
};

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// General OEA with one DPP row of 16 lanes per token (N <= 16*NK, max(k0, k_max) <= 16,
// B <= 4*NT/64): the form the single-kernel layer uses.  Same decisions as route_block_general:
// the baseline ends with the pick that brings the cumulative softmax mass (fp64) to p; a row that
// has stopped takes no part in later rounds (its keys stay as they are); Phase 2 either continues
// on the members of U (no window) or walks the ranks up to max_p, where an expert outside U uses
// up its rank.  Slot r of a row is the r-th expert taken, so the output is in rank order.
template <int NK, int NT, bool COHERENT = false, typename Hook = NoHook>
__device__ __forceinline__ void route_rows_general(const float* __restrict__ logits,
                                                   const uint8_t* __restrict__ token_mask, int B, int N, int k0,
                                                   RouteGeneral g, RouteOut o, uint32_t* lds,
                                                   Hook after_offsets = Hook()) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, row = lane >> 4;
  const int kw = k0 > g.k_max ? k0 : g.k_max;
  const int RPW = B <= NW / 2 ? 1 : 4;
  uint32_t* U = lds;
  RowCarry<NK> c;
  for (int i = tid; i < int(route_lds_words(B, N)); i += NT) lds[i] = 0;
  const int t = wave * RPW + row;
  const bool have = row < RPW && t < B;
  const bool live = have && !(token_mask && token_mask[t] == 0);
  c.t = have ? t : -1;
  c.any = wave * RPW < B;
  const int nbusy = (B + RPW - 1) / RPW;
  c.ebase = (N <= 128 && (NW - nbusy) * 64 >= N) ? nbusy * 64 : 0;
  c.n = 0;
  c.sel_id = c.sel_key = c.top_key = 0;
  float lg[NK];
#pragma unroll
  for (int j = 0; j < NK; ++j) {
    const int e = li + 16 * j;
    const float* src = logits + (size_t)(live ? t : 0) * N + (e < N ? e : N - 1);
    lg[j] = COHERENT ? __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *src;
  }
#pragma unroll
  for (int j = 0; j < NK; ++j) c.key[j] = (live && li + 16 * j < N) ? make_key(lg[j]) : 0;
  __syncthreads();  // U is cleared

  // One round for the rows with `active` set: their best remaining candidate is removed; it is
  // taken (next slot of the row) unless `members_only` and it is not in U.  Returns its key, 0 if
  // the row was not active or had no candidate left.
  auto pick = [&](bool active, bool members_only) __attribute__((always_inline)) {
    uint32_t lm = c.key[0];
#pragma unroll
    for (int j = 1; j < NK; ++j) lm = c.key[j] > lm ? c.key[j] : lm;
    const uint32_t m = row_max_u32(lm);
    uint32_t cand = 0xffffu;
#pragma unroll
    for (int j = NK - 1; j >= 0; --j) cand = c.key[j] == m ? uint32_t(li + 16 * j) : cand;
    const uint32_t win = row_min_u32(cand);
    const bool valid = active && m != 0;
    const uint32_t wq = valid ? win : 0u;  // < N when valid
    const bool member = !members_only || ((U[wq >> 5] >> (wq & 31)) & 1u);
    const bool rec = valid && member;
#pragma unroll
    for (int j = 0; j < NK; ++j) c.key[j] = (valid && uint32_t(li + 16 * j) == win) ? 0u : c.key[j];
    if (rec && li == c.n) {
      c.sel_id = win;
      c.sel_key = m;
    }
    if (rec && c.n == 0) c.top_key = m;
    c.n += rec ? 1 : 0;
    return valid ? m : 0u;
  };

  // ---- Phase 1: the baseline, cut by the top-p rule as well
  const bool capped = g.p < 1.0;
  int nbase = 0;
  if (c.any) {
    double mtop = 0.0, z = 1.0;
    if (capped) {  // softmax denominator over all experts of the row's token
      uint32_t lm = c.key[0];
#pragma unroll
      for (int j = 1; j < NK; ++j) lm = c.key[j] > lm ? c.key[j] : lm;
      mtop = double(from_orderable(row_max_u32(lm)));
      double zl = 0.0;
#pragma unroll
      for (int j = 0; j < NK; ++j)
        if (c.key[j] != 0) zl += exp(double(from_orderable(c.key[j])) - mtop);
      z = row_sum_f64(zl);
    }
    bool active = true;
    double cum = 0.0;
    for (int r = 0; r < k0; ++r) {
      if (__ballot(active) == 0) break;
      const uint32_t m = pick(active, false);
      if (m == 0) active = false;
      if (capped && m != 0) {
        cum += exp(double(from_orderable(m)) - mtop) / z;
        if (cum >= g.p) active = false;
      }
    }
    nbase = c.n;
    if (li < nbase) atomicOr(&U[c.sel_id >> 5], 1u << (c.sel_id & 31));
    if (g.n_base && c.t >= 0 && li == 0) g.n_base[c.t] = nbase;
  }
  __syncthreads();
  route_active<NT>(N, o, lds, c.ebase);
  const GroupPre gp = route_group_pre<NT>(N, lds, c.ebase);

  // ---- Phase 2: piggyback on U in rank order, ranks below max_p, until k_max experts are held
  if (c.any) {
    if (g.max_p >= N) {  // no window: the best remaining members of U
#pragma unroll
      for (int j = 0; j < NK; ++j)
        if (!((U[j >> 1] >> (li + 16 * (j & 1))) & 1u)) c.key[j] = 0;
      for (int r = 0; r < g.k_max; ++r) {
        const bool active = c.n < g.k_max;
        if (__ballot(active) == 0) break;
        pick(active, false);
      }
    } else {  // the ranks in order; rk = candidates removed so far = rank of the next one
      int rk = nbase;
      bool open = true;  // candidates left
      for (int r = 0; r < g.max_p; ++r) {
        const bool active = open && rk < g.max_p && c.n < g.k_max;
        if (__ballot(active) == 0) break;
        const uint32_t m = pick(active, true);
        if (active && m == 0) open = false;
        rk += m != 0 ? 1 : 0;
      }
    }
  }
  route_rows_finish<NK, NT>(B, N, kw, o, lds, c, gp, after_offsets);
}

// General OEA in the row form for any B (the single-kernel layer for larger batches): the tokens are
// taken in groups of 4*NT/64, nothing but the baseline sizes (parked in o.n_sel) is carried between
// the phases; Phase 2 reloads a group's logits, takes the baseline again and goes on from there.
// N <= 16*NK, max(k0, k_max) <= 16.
template <int NK, int NT, bool COHERENT = false>
__device__ void route_rows_general_any(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                                       int B, int N, int k0, RouteGeneral g, RouteOut o, uint32_t* lds) {
  constexpr int GROUP = 4 * (NT / 64);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, row = lane >> 4;
  const int NWB = (B + 31) >> 5;
  const int kw = k0 > g.k_max ? k0 : g.k_max;
  uint32_t* U = lds;
  uint32_t* colmask = lds + 64;
  const bool capped = g.p < 1.0;
  for (int i = tid; i < int(route_lds_words(B, N)); i += NT) lds[i] = 0;
  __syncthreads();

  RowCarry<NK> c;
  auto load_keys = [&](int t, bool live) __attribute__((always_inline)) {
    const float* src = logits + (size_t)(t < B ? t : B - 1) * N;
#pragma unroll
    for (int j = 0; j < NK; ++j) {
      const int e = li + 16 * j;
      const float* q = src + (e < N ? e : N - 1);
      const float v = COHERENT ? __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : *q;
      c.key[j] = (live && e < N) ? make_key(v) : 0;
    }
    c.n = 0;
    c.sel_id = c.sel_key = c.top_key = 0;
  };
  // one round for the rows with `active` set (see route_rows_general)
  auto pick = [&](bool active, bool members_only) __attribute__((always_inline)) {
    uint32_t lm = c.key[0];
#pragma unroll
    for (int j = 1; j < NK; ++j) lm = c.key[j] > lm ? c.key[j] : lm;
    const uint32_t m = row_max_u32(lm);
    uint32_t cand = 0xffffu;
#pragma unroll
    for (int j = NK - 1; j >= 0; --j) cand = c.key[j] == m ? uint32_t(li + 16 * j) : cand;
    const uint32_t win = row_min_u32(cand);
    const bool valid = active && m != 0;
    const uint32_t wq = valid ? win : 0u;
    const bool member = !members_only || ((U[wq >> 5] >> (wq & 31)) & 1u);
    const bool rec = valid && member;
#pragma unroll
    for (int j = 0; j < NK; ++j) c.key[j] = (valid && uint32_t(li + 16 * j) == win) ? 0u : c.key[j];
    if (rec && li == c.n) {
      c.sel_id = win;
      c.sel_key = m;
    }
    if (rec && c.n == 0) c.top_key = m;
    c.n += rec ? 1 : 0;
    return valid ? m : 0u;
  };

  // ---- Phase 1: baselines (top-p cut) and their union; the baseline size of token t -> o.n_sel[t]
  for (int t0 = 0; t0 < B; t0 += GROUP) {
    const int t = t0 + wave * 4 + row;
    const bool live = t < B && !(token_mask && token_mask[t] == 0);
    load_keys(t, live);
    double mtop = 0.0, z = 1.0;
    if (capped) {
      uint32_t lm = c.key[0];
#pragma unroll
      for (int j = 1; j < NK; ++j) lm = c.key[j] > lm ? c.key[j] : lm;
      mtop = double(from_orderable(row_max_u32(lm)));
      double zl = 0.0;
#pragma unroll
      for (int j = 0; j < NK; ++j)
        if (c.key[j] != 0) zl += exp(double(from_orderable(c.key[j])) - mtop);
      z = row_sum_f64(zl);
    }
    bool active = true;
    double cum = 0.0;
    for (int r = 0; r < k0; ++r) {
      if (__ballot(active) == 0) break;
      const uint32_t m = pick(active, false);
      if (m == 0) active = false;
      if (capped && m != 0) {
        cum += exp(double(from_orderable(m)) - mtop) / z;
        if (cum >= g.p) active = false;
      }
    }
    if (li < c.n) atomicOr(&U[c.sel_id >> 5], 1u << (c.sel_id & 31));
    if (t < B && li == 0) {
      o.n_sel[t] = c.n;
      if (g.n_base) g.n_base[t] = c.n;
    }
  }
  __syncthreads();
  route_active<NT>(N, o, lds);

  // ---- Phase 2 per group: the baseline again, then piggybacking as in route_rows_general
  for (int t0 = 0; t0 < B; t0 += GROUP) {
    const int t = t0 + wave * 4 + row;
    const bool have = t < B;
    const bool live = have && !(token_mask && token_mask[t] == 0);
    const int nbase = have ? o.n_sel[t] : 0;  // written by this row's lane 0 before the barrier above
    load_keys(t, live);
    for (int r = 0; r < k0; ++r) {
      const bool active = c.n < nbase;
      if (__ballot(active) == 0) break;
      pick(active, false);
    }
    if (g.max_p >= N) {
#pragma unroll
      for (int j = 0; j < NK; ++j)
        if (!((U[j >> 1] >> (li + 16 * (j & 1))) & 1u)) c.key[j] = 0;
      for (int r = 0; r < g.k_max; ++r) {
        const bool active = c.n < g.k_max;
        if (__ballot(active) == 0) break;
        pick(active, false);
      }
    } else {
      int rk = nbase;
      bool open = true;
      for (int r = 0; r < g.max_p; ++r) {
        const bool active = open && rk < g.max_p && c.n < g.k_max;
        if (__ballot(active) == 0) break;
        const uint32_t m = pick(active, true);
        if (active && m == 0) open = false;
        rk += m != 0 ? 1 : 0;
      }
    }
    const float w = li < c.n ? expf(from_orderable(c.sel_key) - from_orderable(c.top_key)) : 0.f;
    const float z = row_sum_f32(w);
    if (have) {
      if (li < kw) {
        o.expert_idx[(size_t)t * kw + li] = li < c.n ? int(c.sel_id) : -1;
        o.gate_w[(size_t)t * kw + li] = li < c.n ? w / z : 0.f;
      }
      if (li < c.n) atomicOr(&colmask[c.sel_id * NWB + (t >> 5)], 1u << (t & 31));
      if (li == 0) o.n_sel[t] = c.n;
    }
  }
  __syncthreads();
  route_group<NT>(B, N, kw, o, lds);
}

// One workgroup of NT threads, one wavefront per token at a time, any B.  Output rows have
// kw = max(k0, k_max) slots.  lds: route_lds_words(B,N) + B words.
// The top-p decision compares fp64 sums of fp64 softmax values (the softmax of Section 2 taken in
// double, like the weights it decides about are defined), so it can differ from an evaluation in
// another summation order only when the mass is within rounding of p.
template <int NV, int NT>
__device__ void route_block_general(const float* __restrict__ logits, const uint8_t* __restrict__ token_mask,
                                    int B, int N, int k0, RouteGeneral g, RouteOut o, uint32_t* lds) {
  constexpr int NW = NT / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int NWB = (B + 31) >> 5;
  const int kw = k0 > g.k_max ? k0 : g.k_max;
  uint32_t* U = lds;
  uint32_t* colmask = lds + 64;
  int* nb = reinterpret_cast<int*>(lds + route_lds_words(B, N));  // [B] baseline sizes

  for (int i = tid; i < int(route_lds_words(B, N)) + B; i += NT) lds[i] = 0;
  __syncthreads();
  const bool capped = g.p < 1.0;

  // ---- Phase 1: baseline S_i^base = the n_i best experts; U = union over the batch
  for (int t = wave; t < B; t += NW) {
    const bool live = !(token_mask && token_mask[t] == 0);
    uint32_t key[NV];
    float lg[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int e = lane + 64 * j;
      lg[j] = (live && e < N) ? logits[(size_t)t * N + e] : 0.f;
      key[j] = (live && e < N) ? make_key(lg[j]) : 0;
    }
    double m = 0.0, z = 1.0;
    if (capped && live) {  // softmax denominator over all N experts
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
    int n = 0;
    double cum = 0.0;
    for (int r = 0; r < k0; ++r) {
      uint32_t bk;
      int id;
      if (!pick_best<NV>(key, lane, bk, id)) break;
      if (lane == 0) atomicOr(&U[id >> 5], 1u << (id & 31));
      ++n;
      if (capped) {
        cum += exp(double(from_orderable(bk)) - m) / z;
        if (cum >= g.p) break;
      }
    }
    if (lane == 0) {
      nb[t] = n;
      if (g.n_base) g.n_base[t] = n;
    }
  }
  __syncthreads();
  route_active<NT>(N, o, lds);
  __syncthreads();

  // ---- Phase 2: piggyback on U in rank order, ranks below max_p, until k_max experts are held
  for (int t = wave; t < B; t += NW) {
    const bool live = !(token_mask && token_mask[t] == 0);
    const int nbase = nb[t];
    uint32_t key[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int e = lane + 64 * j;
      key[j] = (live && e < N) ? make_key(logits[(size_t)t * N + e]) : 0;
    }
    int cnt = 0, my_id = -1;
    float my_logit = 0.f;
    auto take = [&](int id, uint32_t bk) __attribute__((always_inline)) {
      if (lane == cnt) {
        my_id = id;
        my_logit = from_orderable(bk);
      }
      ++cnt;
    };
    if (g.max_p >= N) {
      // no window: the piggybacked experts are simply the best remaining members of U
      for (int r = 0; r < nbase; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        take(id, bk);
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int e = lane + 64 * j;
        if (!(e < N && ((U[e >> 5] >> (e & 31)) & 1u))) key[j] = 0;
      }
      while (cnt < g.k_max) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        take(id, bk);
      }
    } else {
      // walk the ranks in order; an expert outside U uses up its rank without being taken
      const int last = nbase > g.max_p ? nbase : g.max_p;
      for (int r = 0; r < last; ++r) {
        uint32_t bk;
        int id;
        if (!pick_best<NV>(key, lane, bk, id)) break;
        if (r < nbase) {
          take(id, bk);
        } else {
          if (cnt >= g.k_max) break;
          if ((U[id >> 5] >> (id & 31)) & 1u) take(id, bk);
        }
      }
    }
    // weights: original scores renormalised over S_i (Eq. 1; the softmax denominator cancels)
    const float mtop = __shfl(my_logit, 0, 64);
    const float w = lane < cnt ? expf(my_logit - mtop) : 0.f;
    const float zz = wave_sum_f32(w);
    if (lane < kw) {
      o.expert_idx[(size_t)t * kw + lane] = lane < cnt ? my_id : -1;
      o.gate_w[(size_t)t * kw + lane] = lane < cnt ? w / zz : 0.f;
    }
    if (lane < cnt) atomicOr(&colmask[my_id * NWB + (t >> 5)], 1u << (t & 31));
    if (lane == 0) o.n_sel[t] = cnt;
  }
  __syncthreads();
  route_group<NT>(B, N, kw, o, lds);
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

}  // namespace
}  // namespace oea
