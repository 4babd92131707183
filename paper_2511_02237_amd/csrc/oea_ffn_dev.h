// Device-side building blocks of the expert mat-vec stages, shared by the streaming kernels and
// the fused layer kernel (gfx950): 16-byte fragment dot products, lane reductions, and the
// register-tile load / compute helpers of the streaming design.
#pragma once
#include "oea_internal.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace oea {
namespace {

constexpr int kFfnThreads = 512;
constexpr int kFfnWaves = kFfnThreads / 64;

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

// 16-byte streaming load of expert weights: each byte is read once per layer call, so the load is
// marked non-temporal (on this GPU that streams markedly faster from HBM than a plain load,
// 6.9 against 6.1 TB/s in a read-only probe, and leaves the caches to x, h and the metadata)
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7f800000u) == 0x7f800000u) return uint16_t((u >> 16) | ((u & 0xffffu) ? 0x40u : 0u));  // inf/nan
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

__device__ __forceinline__ void store_h(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_h(uint16_t* p, float v) { *p = f32_to_bf16_rne(v); }
// device-coherent variants: written through to memory, no dirty line stays in this XCD's L2, so
// workgroups on other XCDs can read the value after a grid barrier without cache maintenance
__device__ __forceinline__ void store_h_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_h_coherent(uint16_t* p, float v) {
  __hip_atomic_store(p, f32_to_bf16_rne(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kMaxSeg = 3;

// Per-wavefront description of the rows it streams.  All members are wave-uniform scalars; the
// helpers take it BY VALUE and select between plain scalars only, so it never lives in memory.
struct SegView {
  int rows;              // weight rows per expert
  int a0;                // position (in the active list) of the workgroup's first expert
  int e0, e1, e2;        // expert ids of the (up to 3) segments
  int cnt0, cnt1, cnt2;  // (expert, token) pairs per segment
  int my_hi;             // end of this wavefront's rows (concatenated numbering)
  int my_lo;             // their start (only used for the result buffer in LDS)
};

struct TileRef {
  int e;     // expert id
  int rloc;  // first row inside the expert
  int cnt;   // pairs of that expert
  int vb;    // index of its first pair in the staged lists
  int ebase;    // result buffer in LDS: entry of the tile's first row for the expert's first pair ...
  int estride;  // ... and the distance between consecutive pairs (= rows of this segment the wavefront owns)
};

__device__ __forceinline__ int seg_of(const SegView sv, int r) {
  return (r >= (sv.a0 + 1) * sv.rows ? 1 : 0) + (r >= (sv.a0 + 2) * sv.rows ? 1 : 0);
}

// rows of the tile that starts at concatenated row r: at most trows, never across an expert boundary
__device__ __forceinline__ int tile_rows(const SegView sv, int r, int trows) {
  if (r >= sv.my_hi) return 0;
  int lim = (sv.a0 + seg_of(sv, r) + 1) * sv.rows;
  lim = lim < sv.my_hi ? lim : sv.my_hi;
  const int n = lim - r;
  return n < trows ? n : trows;
}

__device__ __forceinline__ TileRef tile_ref(const SegView sv, int r) {
  const int s = seg_of(sv, r);
  TileRef t;
  t.e = s == 0 ? sv.e0 : (s == 1 ? sv.e1 : sv.e2);
  t.cnt = s == 0 ? sv.cnt0 : (s == 1 ? sv.cnt1 : sv.cnt2);
  t.vb = s == 0 ? 0 : (s == 1 ? sv.cnt0 : sv.cnt0 + sv.cnt1);
  t.rloc = r - (sv.a0 + s) * sv.rows;
  t.ebase = 0;
  t.estride = 0;
  return t;
}

// Result buffer (LDS, floats) for the rows [my_lo, my_hi): the rows of segment s form a block [pair][row],
// the blocks of the segments follow each other.
__device__ __forceinline__ int seg_lo(const SegView sv, int s) {
  const int start = (sv.a0 + s) * sv.rows;
  return start > sv.my_lo ? start : sv.my_lo;
}
__device__ __forceinline__ int seg_n(const SegView sv, int s) {  // rows of segment s inside [my_lo, my_hi)
  const int end = (sv.a0 + s + 1) * sv.rows;
  const int n = (end < sv.my_hi ? end : sv.my_hi) - seg_lo(sv, s);
  return n > 0 ? n : 0;
}
__device__ __forceinline__ int seg_cnt(const SegView sv, int s) { return s == 0 ? sv.cnt0 : (s == 1 ? sv.cnt1 : sv.cnt2); }
__device__ __forceinline__ int seg_entries(const SegView sv, int s) {  // buffer entries of segment s
  return seg_n(sv, s) * seg_cnt(sv, s);
}
__device__ __forceinline__ int seg_ebase(const SegView sv, int s) {
  return (s > 0 ? seg_entries(sv, 0) : 0) + (s > 1 ? seg_entries(sv, 1) : 0);
}
__device__ __forceinline__ int result_entries(const SegView sv) {
  return seg_entries(sv, 0) + seg_entries(sv, 1) + seg_entries(sv, 2);
}
__device__ __forceinline__ TileRef tile_ref_buffered(const SegView sv, int r) {
  TileRef t = tile_ref(sv, r);
  const int s = seg_of(sv, r);
  t.ebase = seg_ebase(sv, s) + (r - seg_lo(sv, s));
  t.estride = seg_n(sv, s);
  return t;
}

// Always issues NM*RG*NCH loads.  nrows >= 1 rows of the tile are wanted; lanes of missing rows
// re-read the tile's last row, columns past the end re-read the row's last granule (their products
// are masked in compute).  nrows == 0 is a placeholder request past the end of the wavefront's work
// (it keeps the number of outstanding loads fixed): every lane then reads the same 16 bytes, so it
// costs one cache line per load instead of a tile.
template <typename WT, int NM, int LPR, int NCH, int RG, bool FULL>
__device__ __forceinline__ void load_tile(uint4 (&w)[NM][RG][NCH], const WT* wa, const WT* wb, int rows, int L,
                                          int lsub, int lrow, const TileRef t, int nrows) {
  constexpr int EPL = 16 / int(sizeof(WT));
  constexpr int R = 64 / LPR;
  constexpr int CH = LPR * EPL;
  const size_t ebase = (size_t)t.e * rows * L;
  const bool real = nrows > 0;
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    int rr = rg * R + lrow;
    rr = rr < nrows ? rr : nrows - 1;
    rr = real ? rr : 0;
    const size_t rbase = ebase + (size_t)(t.rloc + rr) * L;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      int col = ch * CH + lsub * EPL;
      if (!FULL) col = col < L ? col : L - EPL;
      col = real ? col : 0;
#pragma unroll
      for (int m = 0; m < NM; ++m) w[m][rg][ch] = load_stream16((m == 0 ? wa : wb) + rbase + col);
    }
  }
}

// one (expert, token) pair against the tile held in w: dot products, reduction over the row's lanes, epilogue
// use_buf: the results go to the wavefront's result buffer in LDS (entry eidx + row of the
// tile) instead of memory; flush_results writes them out when the wavefront has streamed all its rows.
// GATHER: the staged vectors are indexed by pair in the gate/up stage too (x rows gathered per pair).
template <typename WT, int STAGE, int NM, int LPR, int NCH, int RG, bool FULL, bool COH = false, bool EBUF = false,
          bool GATHER = false>
__device__ __forceinline__ void token_step(const uint4 (&w)[NM][RG][NCH], const int* l_tok, const float* l_gw,
                                           const uint4* l_vec, WT* h_out, float* out, int rows, int L16, int off0,
                                           int lsub, int lrow, int rloc, int nrows, int pair, float* ebuf = nullptr,
                                           bool use_buf = false, int eidx = 0) {
  constexpr int R = 64 / LPR;
  const int tok = l_tok[pair];
  const uint4* vq = l_vec + (size_t)(STAGE == 0 && !GATHER ? tok : pair) * L16;
  uint4 v[NCH];
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    const int g16 = ch * LPR + lsub;
    if (FULL) {
      v[ch] = vq[g16];
    } else {
      const uint4 t4 = vq[g16 < L16 ? g16 : L16 - 1];
      const uint32_t keep = g16 < L16 ? 0xffffffffu : 0u;  // a zero vector element kills the product
      v[ch] = make_uint4(t4.x & keep, t4.y & keep, t4.z & keep, t4.w & keep);
    }
  }
  float acc[NM][RG];
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) acc[m][rg] = 0.f;
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
    for (int m = 0; m < NM; ++m)
#pragma unroll
      for (int rg = 0; rg < RG; ++rg) acc[m][rg] = frag_dot<WT>(w[m][rg][ch], v[ch], acc[m][rg]);
#pragma unroll
  for (int rg = 0; rg < RG; ++rg) {
    const int rr = rg * R + lrow;
    if (STAGE == 0) {
      const float gsum = row_sum<LPR>(acc[0][rg]);
      const float usum = row_sum<LPR>(acc[NM - 1][rg]);
      if (lsub == 0 && rr < nrows) {
        const float hval = gsum / (1.f + __expf(-gsum)) * usum;
        if (EBUF && use_buf)
          ebuf[eidx + rr] = hval;
        else if (COH)
          store_h_coherent(h_out + (size_t)(off0 + pair) * rows + rloc + rr, hval);
        else
          store_h(h_out + (size_t)(off0 + pair) * rows + rloc + rr, hval);
      }
    } else {
      const float y = row_sum<LPR>(acc[0][rg]);
      if (lsub == 0 && rr < nrows) {
        if (EBUF && use_buf)
          ebuf[eidx + rr] = y;
        else
          unsafeAtomicAdd(out + (size_t)tok * rows + rloc + rr, l_gw[pair] * y);
      }
    }
  }
}

// The first kUnrollTok pairs of an expert are handled by straight-line code with forward branches
// only.  A loop here would make the compiler drain ALL outstanding loads (also the prefetched
// tile) in the loop pre-header, because the loop stores to memory; the loop form is kept for the
// rare expert with more pairs than that.
constexpr int kUnrollTok = 8;

template <typename WT, int STAGE, int NM, int LPR, int NCH, int RG, bool FULL, bool COH = false, bool EBUF = false,
          bool GATHER = false>
__device__ __forceinline__ void compute_tile(const uint4 (&w)[NM][RG][NCH], const int* l_tok, const float* l_gw,
                                             const uint4* l_vec, WT* h_out, float* out, int rows, int L16,
                                             int off0, int lsub, int lrow, const TileRef t, int nrows,
                                             float* ebuf = nullptr, bool use_buf = false) {
#pragma unroll
  for (int q = 0; q < kUnrollTok; ++q)
    if (q < t.cnt)
      token_step<WT, STAGE, NM, LPR, NCH, RG, FULL, COH, EBUF, GATHER>(w, l_tok, l_gw, l_vec, h_out, out, rows, L16, off0, lsub,
                                                               lrow, t.rloc, nrows, t.vb + q, ebuf, use_buf,
                                                               t.ebase + q * t.estride);
  if (t.cnt > kUnrollTok)
    for (int q = kUnrollTok; q < t.cnt; ++q)
      token_step<WT, STAGE, NM, LPR, NCH, RG, FULL, COH, EBUF, GATHER>(w, l_tok, l_gw, l_vec, h_out, out, rows, L16, off0, lsub,
                                                               lrow, t.rloc, nrows, t.vb + q, ebuf, use_buf,
                                                               t.ebase + q * t.estride);
}

// Write the workgroup's buffered results to memory (all kFfnThreads threads): for every segment
// and pair its rows are consecutive addresses, so neighbouring threads store (or add) neighbours.
//   STAGE 0: h[(off0 + pair), row] = value (device-coherent store, rounded to the storage type)
//   STAGE 1: out[token, row] += gate weight * value
template <typename WT, int STAGE>
__device__ __forceinline__ void flush_results(const SegView sv, const float* ebuf, const int* s_tok, const float* s_gw,
                                              WT* h_out, float* out, int off0, int tid) {
  int vb = 0;
#pragma unroll
  for (int s = 0; s < kMaxSeg; ++s) {
    const int n = seg_n(sv, s), cnt = seg_cnt(sv, s);
    const int rloc = seg_lo(sv, s) - (sv.a0 + s) * sv.rows;
    const int base = seg_ebase(sv, s);
    // one thread per (pair, row) entry, rows fastest
    for (int i = tid; i < n * cnt; i += kFfnThreads) {
      const int q = i / n, r = i - q * n;
      const int pair = vb + q;
      const float v = ebuf[base + i];
      if (STAGE == 0)
        store_h_coherent(h_out + (size_t)(off0 + pair) * sv.rows + rloc + r, v);
      else
        unsafeAtomicAdd(out + (size_t)s_tok[pair] * sv.rows + rloc + r, s_gw[pair] * v);
    }
    vb += cnt;
  }
}

}  // namespace
}  // namespace oea
