/*
 * CPU oracle for the decode-time MoE layer with Opportunistic Expert Activation (OEA).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table or helper with the
 * HIP library; it never calls it and is never called by it.
 *
 * Written from the paper (arxiv 2511.02237), plain and slow on purpose:
 *   - Section 2, Eq. 1      : moe(x) = sum_{i in S} R(x)_i / sum_{j in S} R(x)_j * E_i(x)
 *   - Section 3.2, Notation : e_{i,j} = experts of token i sorted by descending router score
 *   - Algorithm 1           : simplified OEA (Phase 1 top-k0, Phase 2 piggybacking up to k)
 *   - Algorithm 2           : general OEA (top-p cap n_i = min(k0,t_i), k^max, maxP)
 *   - Section 3.2, "Weighting after rerouting": router scores kept, renormalised over S_i
 *   - Section 4, "Hardware and model": each expert is a SwiGLU FFN made of three mat-muls
 *   - Section 6, "A note on padding": a padding mask that removes padded tokens' expert choices
 *
 * Arithmetic: every floating-point accumulation is fp64, taken left to right in the order the
 * definition is written.  Router logits are rounded ONCE to fp32 after the fp64 sum, because the
 * ranking (an integer decision) is taken on fp32 logits: that is the precision the routing entry
 * point of the library receives them in.  bf16 inputs are widened exactly.
 *
 * Readings of the paper taken here (each one is listed again in the design notes):
 *   R1  The Phase-2 cap.  The listing breaks when |S_i| > k, which would allow k+1 experts; the
 *       prose says the number of selected experts "does not exceed" the cap and that the base
 *       model is k0 = k.  So: a token stops as soon as it holds k (or k^max) experts.
 *   R2  R = softmax(W_router x) (+ optional per-expert bias used only by synthetic skewed inputs).
 *   R3  Ranking is on the fp32 logits (softmax is monotone), descending, ties -> lower expert id.
 *       -0.0 and +0.0 are equal.
 *   R4  S_i is reported in rank order; unused slots hold -1 / weight 0.
 *   R5  If the union holds fewer than k experts a token simply ends with fewer than k.
 *   R6  SwiGLU: E(x) = W_down ( silu(W_gate x) * (W_up x) ), silu(z) = z / (1 + exp(-z)), no bias.
 *   R7  Top-p threshold t_i uses the scores in SORTED order (as in Algorithm 2).
 *   R8  A masked (padding) token selects nothing, adds nothing to the union, and its output is 0.
 *
 * Pinning: see tests/test_oracle_*.py (not gpu).  Every exported function below is pinned there
 * against closed forms, invariants, brute force on tiny inputs, or numpy fp64 definitions.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* exact widening of one stored element to double */
static double elem(const void *p, long idx, int dtype) {
  if (dtype == ORACLE_F32) return (double)((const float *)p)[idx];
  uint32_t bits = ((uint32_t)((const uint16_t *)p)[idx]) << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Router pre-activations (Section 2: the router maps a token to one score per expert).
 * logits[i][e] = fp32( sum_c x[i][c] * W_router[e][c]  (+ bias[e]) ), sum in fp64, c ascending. */
void oracle_router_logits(const void *x, const void *w_router, const float *bias, int B, int d,
                          int N, int dtype, float *logits) {
  for (int i = 0; i < B; ++i)
    for (int e = 0; e < N; ++e) {
      double s = 0.0;
      for (int c = 0; c < d; ++c) s += elem(x, (long)i * d + c, dtype) * elem(w_router, (long)e * d + c, dtype);
      if (bias) s += (double)bias[e];
      logits[(long)i * N + e] = (float)s;
    }
}

/* Normalised router scores R(x_i) in the simplex (Section 2), as fp64 softmax of the fp32 logits. */
void oracle_softmax(const float *logits, int B, int N, double *R) {
  for (int i = 0; i < B; ++i) {
    const float *l = logits + (long)i * N;
    double m = (double)l[0];
    for (int e = 1; e < N; ++e)
      if ((double)l[e] > m) m = (double)l[e];
    double z = 0.0;
    for (int e = 0; e < N; ++e) z += exp((double)l[e] - m);
    for (int e = 0; e < N; ++e) R[(long)i * N + e] = exp((double)l[e] - m) / z;
  }
}

/* e_{i,.} (Section 3.2, Notation): insertion sort, descending logit, equal logits keep ascending
 * expert id (stable).  rank[i][j] = expert holding rank j for token i (0-based). */
void oracle_rank(const float *logits, int B, int N, int32_t *rank) {
  for (int i = 0; i < B; ++i) {
    const float *l = logits + (long)i * N;
    int32_t *r = rank + (long)i * N;
    for (int e = 0; e < N; ++e) {
      int pos = e;
      while (pos > 0 && l[r[pos - 1]] < l[e]) { /* strictly smaller moves down: ties stay put */
        r[pos] = r[pos - 1];
        --pos;
      }
      r[pos] = e;
    }
  }
}

/* General OEA routing (Algorithm 2); Algorithm 1 is the call p = 1, k_max = k, max_p = N.
 *
 * in : logits [B,N] fp32; token_mask [B] (NULL = all live; 0 = padded token, reading R8)
 * out: expert_idx [B,width] rank order, -1 padded; gate_w [B,width] fp64, 0 padded, with
 *      width = max(k0, k_max): the listing starts S_i from the whole baseline, so a baseline
 *      larger than k_max is kept as it is and simply receives no piggybacked expert;
 *      n_sel [B]; n_base [B] (= n_i); active_list [N] ascending ids, first *n_active valid.
 * Returns 0, or -1 on an illegal parameter combination.
 */
int oracle_oea_route_general(const float *logits, const uint8_t *token_mask, int B, int N, int k0,
                             double p, int k_max, int max_p, int32_t *expert_idx, double *gate_w,
                             int32_t *n_sel, int32_t *n_base, int32_t *active_list,
                             int32_t *n_active) {
  if (B < 1 || N < 1 || k0 < 1 || k0 > N || k_max < 1 || k_max > N || max_p < 1 || max_p > N ||
      !(p > 0.0) || p > 1.0)
    return -1;
  const int width = k0 > k_max ? k0 : k_max;
  int32_t *rank = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * N);
  double *R = (double *)malloc(sizeof(double) * (size_t)B * N);
  uint8_t *in_union = (uint8_t *)calloc((size_t)N, 1);
  oracle_rank(logits, B, N, rank);
  oracle_softmax(logits, B, N, R);

  /* Phase 1: baseline experts.  t_i = least t with cumulative sorted mass >= p; n_i = min(k0,t_i). */
  for (int i = 0; i < B; ++i) {
    int ni = 0;
    if (!token_mask || token_mask[i]) {
      int ti = N; /* p = 1 switches the top-p cap off (Section 4.1, footnote on p = 1) */
      double cum = 0.0;
      for (int j = 0; j < N && p < 1.0; ++j) {
        cum += R[(long)i * N + rank[(long)i * N + j]];
        if (cum >= p) {
          ti = j + 1;
          break;
        }
      }
      ni = k0 < ti ? k0 : ti;
    }
    n_base[i] = ni;
    for (int j = 0; j < ni; ++j) in_union[rank[(long)i * N + j]] = 1;
  }

  /* S^base = union of the baselines; T = |S^base|. */
  int T = 0;
  for (int e = 0; e < N; ++e)
    if (in_union[e]) active_list[T++] = e;
  for (int e = T; e < N; ++e) active_list[e] = -1;
  *n_active = T;

  /* Phase 2: piggybacking.  Walk ranks n_i+1 .. maxP, take experts already in S^base, stop at
   * the cap (reading R1). */
  for (int i = 0; i < B; ++i) {
    int32_t *S = expert_idx + (long)i * width;
    double *g = gate_w + (long)i * width;
    int cnt = 0;
    for (int s = 0; s < width; ++s) {
      S[s] = -1;
      g[s] = 0.0;
    }
    if (!token_mask || token_mask[i]) {
      for (int j = 0; j < n_base[i]; ++j) S[cnt++] = rank[(long)i * N + j];
      for (int j = n_base[i]; j < max_p; ++j) {
        if (cnt >= k_max) break;
        int e = rank[(long)i * N + j];
        if (in_union[e]) S[cnt++] = e;
      }
    }
    n_sel[i] = cnt;
    /* Weighting after rerouting: original scores, renormalised over S_i (Eq. 1). */
    double z = 0.0;
    for (int s = 0; s < cnt; ++s) z += R[(long)i * N + S[s]];
    for (int s = 0; s < cnt; ++s) g[s] = R[(long)i * N + S[s]] / z;
  }
  free(rank);
  free(R);
  free(in_union);
  return 0;
}

/* Simplified OEA (Algorithm 1).  k0 = k is the unmodified top-k router. */
int oracle_oea_route(const float *logits, const uint8_t *token_mask, int B, int N, int k, int k0,
                     int32_t *expert_idx, double *gate_w, int32_t *n_sel, int32_t *active_list,
                     int32_t *n_active) {
  if (k < 1 || k > N || k0 < 1 || k0 > k) return -1;
  int32_t *n_base = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B > 0 ? B : 1));
  int rc = oracle_oea_route_general(logits, token_mask, B, N, k0, 1.0, k, N, expert_idx, gate_w,
                                    n_sel, n_base, active_list, n_active);
  free(n_base);
  return rc;
}

/* One expert on one token (Section 4: SwiGLU FFN, three mat-muls; reading R6).
 * w_gate, w_up : [I,d] row-major; w_down : [d,I] row-major; y : [d] fp64. */
void oracle_expert_ffn(const void *x_row, const void *w_gate, const void *w_up, const void *w_down,
                       int d, int I, int dtype, double *h_scratch, double *y) {
  for (int j = 0; j < I; ++j) {
    double g = 0.0, u = 0.0;
    for (int c = 0; c < d; ++c) g += elem(w_gate, (long)j * d + c, dtype) * elem(x_row, c, dtype);
    for (int c = 0; c < d; ++c) u += elem(w_up, (long)j * d + c, dtype) * elem(x_row, c, dtype);
    h_scratch[j] = g / (1.0 + exp(-g)) * u;
  }
  for (int c = 0; c < d; ++c) {
    double s = 0.0;
    for (int j = 0; j < I; ++j) s += elem(w_down, (long)c * I + j, dtype) * h_scratch[j];
    y[c] = s;
  }
}

/* Eq. 1 over given sets: out[i] = sum_s gate_w[i][s] * E_{S_i[s]}(x_i), slots in stored order.
 * x [B,d]; w_gate, w_up [N,I,d]; w_down [N,d,I]; expert_idx/gate_w [B,kk]; out [B,d] fp64.
 * The (token, slot) pairs are independent and are spread over OpenMP threads; the weighted sum
 * over slots is taken afterwards in slot order, so the result does not depend on the thread count. */
void oracle_moe_combine(const void *x, const void *w_gate, const void *w_up, const void *w_down,
                        const int32_t *expert_idx, const double *gate_w, int B, int d, int N, int I,
                        int kk, int dtype, double *out) {
  (void)N;
  size_t esz = dtype == ORACLE_F32 ? 4 : 2;
  double *y = (double *)calloc((size_t)B * kk * d, sizeof(double));
#pragma omp parallel
  {
    double *h = (double *)malloc(sizeof(double) * (size_t)I);
#pragma omp for schedule(dynamic, 1)
    for (int q = 0; q < B * kk; ++q) {
      int i = q / kk;
      int e = expert_idx[q];
      if (e < 0) continue;
      const char *xr = (const char *)x + (size_t)i * d * esz;
      const char *wg = (const char *)w_gate + (size_t)e * I * d * esz;
      const char *wu = (const char *)w_up + (size_t)e * I * d * esz;
      const char *wd = (const char *)w_down + (size_t)e * d * I * esz;
      oracle_expert_ffn(xr, wg, wu, wd, d, I, dtype, h, y + (size_t)q * d);
    }
    free(h);
  }
  for (int i = 0; i < B; ++i)
    for (int c = 0; c < d; ++c) {
      double s = 0.0;
      for (int sl = 0; sl < kk; ++sl)
        if (expert_idx[(long)i * kk + sl] >= 0)
          s += gate_w[(long)i * kk + sl] * y[((size_t)i * kk + sl) * d + c];
      out[(long)i * d + c] = s;
    }
  free(y);
}

/* The whole decode-time layer: router -> simplified OEA -> Eq. 1.
 * Any of logits_out / expert_idx / gate_w / n_sel / active_list / n_active may be NULL. */
int oracle_moe_decode(const void *x, const void *w_router, const void *w_gate, const void *w_up,
                      const void *w_down, const float *router_bias, const uint8_t *token_mask,
                      int B, int d, int N, int I, int k, int k0, int dtype, double *out,
                      float *logits_out, int32_t *expert_idx, double *gate_w, int32_t *n_sel,
                      int32_t *active_list, int32_t *n_active) {
  if (B < 1 || d < 1 || N < 1 || I < 1) return -1;
  float *logits = (float *)malloc(sizeof(float) * (size_t)B * N);
  int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * k);
  double *gw = (double *)malloc(sizeof(double) * (size_t)B * k);
  int32_t *ns = (int32_t *)malloc(sizeof(int32_t) * (size_t)B);
  int32_t *al = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
  int32_t T = 0;
  oracle_router_logits(x, w_router, router_bias, B, d, N, dtype, logits);
  int rc = oracle_oea_route(logits, token_mask, B, N, k, k0, idx, gw, ns, al, &T);
  if (rc == 0) {
    oracle_moe_combine(x, w_gate, w_up, w_down, idx, gw, B, d, N, I, k, dtype, out);
    if (logits_out) memcpy(logits_out, logits, sizeof(float) * (size_t)B * N);
    if (expert_idx) memcpy(expert_idx, idx, sizeof(int32_t) * (size_t)B * k);
    if (gate_w) memcpy(gate_w, gw, sizeof(double) * (size_t)B * k);
    if (n_sel) memcpy(n_sel, ns, sizeof(int32_t) * (size_t)B);
    if (active_list) memcpy(active_list, al, sizeof(int32_t) * (size_t)N);
    if (n_active) *n_active = T;
  }
  free(logits);
  free(idx);
  free(gw);
  free(ns);
  free(al);
  return rc;
}
