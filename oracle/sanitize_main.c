/*
 * Driver for a sanitizer build of the oracle (test infrastructure): calls every exported function
 * of oea_oracle.c on small seeded inputs, including the edge shapes (one token, one expert, k = N,
 * padded tokens, every knob of the general routing), with output buffers of exactly the
 * documented sizes.  Built by oracle/build.py with -fsanitize=address,undefined; any report makes
 * the run fail.  Prints "oracle sanitize: ok" at the end.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_set_num_threads(int n);
int oracle_num_threads(void);
void oracle_router_logits(const void *x, const void *w_router, const float *bias, int B, int d, int N, int dtype,
                          float *logits);
void oracle_softmax(const float *logits, int B, int N, double *R);
void oracle_rank(const float *logits, int B, int N, int32_t *rank);
int oracle_oea_route_general(const float *logits, const uint8_t *token_mask, int B, int N, int k0, double p, int k_max,
                             int max_p, int32_t *expert_idx, double *gate_w, int32_t *n_sel, int32_t *n_base,
                             int32_t *active_list, int32_t *n_active);
int oracle_oea_route(const float *logits, const uint8_t *token_mask, int B, int N, int k, int k0, int32_t *expert_idx,
                     double *gate_w, int32_t *n_sel, int32_t *active_list, int32_t *n_active);
void oracle_expert_ffn(const void *x_row, const void *w_gate, const void *w_up, const void *w_down, int d, int I,
                       int dtype, double *h_scratch, double *y);
void oracle_moe_combine(const void *x, const void *w_gate, const void *w_up, const void *w_down,
                        const int32_t *expert_idx, const double *gate_w, int B, int d, int N, int I, int kk, int dtype,
                        double *out);
int oracle_moe_decode(const void *x, const void *w_router, const void *w_gate, const void *w_up, const void *w_down,
                      const float *router_bias, const uint8_t *token_mask, int B, int d, int N, int I, int k, int k0,
                      int dtype, double *out, float *logits_out, int32_t *expert_idx, double *gate_w, int32_t *n_sel,
                      int32_t *active_list, int32_t *n_active);

static uint32_t seed_state = 12345u;
static float frand(void) { /* uniform in (-1, 1) */
  seed_state = seed_state * 1664525u + 1013904223u;
  return (float)((seed_state >> 8) & 0xffffff) / 8388608.0f - 1.0f;
}
static uint16_t to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
/* n values in the given storage type (0 = fp32, 1 = bf16 bits), scaled */
static void *draw(size_t n, int dtype, float scale) {
  if (dtype == 0) {
    float *p = (float *)malloc(n * 4);
    for (size_t i = 0; i < n; ++i) p[i] = frand() * scale;
    return p;
  }
  uint16_t *p = (uint16_t *)malloc(n * 2);
  for (size_t i = 0; i < n; ++i) p[i] = to_bf16(frand() * scale);
  return p;
}

static int check_routing(const int32_t *idx, const int32_t *n_sel, const int32_t *al, int T, int B, int N, int width) {
  if (T < 0 || T > N) return 1;
  for (int a = 0; a < T; ++a)
    if (al[a] < 0 || al[a] >= N) return 1;
  for (int i = 0; i < B; ++i) {
    if (n_sel[i] < 0 || n_sel[i] > width) return 1;
    for (int s = 0; s < width; ++s) {
      int e = idx[i * width + s];
      if (s < n_sel[i] ? (e < 0 || e >= N) : e != -1) return 1;
    }
  }
  return 0;
}

static int one_layer(int B, int d, int N, int I, int k, int k0, int dtype, int with_mask, int with_bias) {
  void *x = draw((size_t)B * d, dtype, 1.0f), *wr = draw((size_t)N * d, dtype, 0.2f);
  void *wg = draw((size_t)N * I * d, dtype, 0.05f), *wu = draw((size_t)N * I * d, dtype, 0.05f);
  void *wd = draw((size_t)N * d * I, dtype, 0.05f);
  float *bias = with_bias ? (float *)draw((size_t)N, 0, 1.0f) : NULL;
  uint8_t *mask = NULL;
  if (with_mask) {
    mask = (uint8_t *)malloc((size_t)B);
    for (int i = 0; i < B; ++i) mask[i] = (uint8_t)(i % 3 != 1);
  }
  double *out = (double *)malloc(sizeof(double) * (size_t)B * d);
  float *lg = (float *)malloc(sizeof(float) * (size_t)B * N);
  int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * k), *ns = (int32_t *)malloc(sizeof(int32_t) * B);
  double *gw = (double *)malloc(sizeof(double) * (size_t)B * k);
  int32_t *al = (int32_t *)malloc(sizeof(int32_t) * N), T = -1;
  int bad = oracle_moe_decode(x, wr, wg, wu, wd, bias, mask, B, d, N, I, k, k0, dtype, out, lg, idx, gw, ns, al, &T);
  bad |= check_routing(idx, ns, al, T, B, N, k);
  /* the pieces on their own, with buffers of exactly the documented sizes */
  double *R = (double *)malloc(sizeof(double) * (size_t)B * N);
  int32_t *rk = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * N);
  oracle_router_logits(x, wr, bias, B, d, N, dtype, lg);
  oracle_softmax(lg, B, N, R);
  oracle_rank(lg, B, N, rk);
  double *hs = (double *)malloc(sizeof(double) * I), *y = (double *)malloc(sizeof(double) * d);
  oracle_expert_ffn(x, wg, wu, wd, d, I, dtype, hs, y);
  oracle_moe_combine(x, wg, wu, wd, idx, gw, B, d, N, I, k, dtype, out);
  /* the same call with every optional output left out */
  bad |= oracle_moe_decode(x, wr, wg, wu, wd, bias, mask, B, d, N, I, k, k0, dtype, out, NULL, NULL, NULL, NULL, NULL, NULL);
  free(x); free(wr); free(wg); free(wu); free(wd); free(bias); free(mask); free(out); free(lg); free(idx); free(ns);
  free(gw); free(al); free(R); free(rk); free(hs); free(y);
  return bad;
}

static int general_routing(int B, int N) {
  float *lg = (float *)draw((size_t)B * N, 0, 2.0f);
  for (int i = 0; i + 1 < B * N; i += 5) lg[i + 1] = lg[i]; /* exact ties */
  uint8_t *mask = (uint8_t *)malloc((size_t)B);
  for (int i = 0; i < B; ++i) mask[i] = (uint8_t)(i % 4 != 2);
  int bad = 0;
  const double ps[] = {1.0, 0.9, 0.3, 1e-9};
  for (int k0 = 1; k0 <= N; k0 += (N > 4 ? N / 3 : 1))
    for (int k_max = 1; k_max <= N; k_max += (N > 4 ? N / 3 : 1))
      for (int max_p = 1; max_p <= N; max_p += (N > 4 ? N / 2 : 1))
        for (int pi = 0; pi < 4; ++pi)
          for (int m = 0; m < 2; ++m) {
            const int width = k0 > k_max ? k0 : k_max;
            int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * width);
            double *gw = (double *)malloc(sizeof(double) * (size_t)B * width);
            int32_t *ns = (int32_t *)malloc(sizeof(int32_t) * B), *nb = (int32_t *)malloc(sizeof(int32_t) * B);
            int32_t *al = (int32_t *)malloc(sizeof(int32_t) * N), T = -1;
            bad |= oracle_oea_route_general(lg, m ? mask : NULL, B, N, k0, ps[pi], k_max, max_p, idx, gw, ns, nb, al, &T);
            bad |= check_routing(idx, ns, al, T, B, N, width);
            free(idx); free(gw); free(ns); free(nb); free(al);
          }
  /* illegal parameters are refused without touching the outputs */
  bad |= oracle_oea_route_general(lg, NULL, B, N, 0, 1.0, 1, 1, NULL, NULL, NULL, NULL, NULL, NULL) != -1;
  bad |= oracle_oea_route_general(lg, NULL, B, N, 1, 0.0, 1, 1, NULL, NULL, NULL, NULL, NULL, NULL) != -1;
  bad |= oracle_oea_route_general(lg, NULL, B, N, 1, 1.0, N + 1, 1, NULL, NULL, NULL, NULL, NULL, NULL) != -1;
  bad |= oracle_oea_route(lg, NULL, B, N, 1, 2, NULL, NULL, NULL, NULL, NULL) != -1;
  free(lg); free(mask);
  return bad;
}

int main(void) {
  int bad = 0;
  oracle_set_num_threads(2);
  if (oracle_num_threads() < 1) bad = 1;
  /* B, d, N, I, k, k0, dtype, mask, bias */
  bad |= one_layer(4, 64, 16, 32, 4, 2, 0, 0, 0);
  bad |= one_layer(5, 40, 7, 24, 7, 3, 1, 1, 1); /* k = N */
  bad |= one_layer(1, 8, 1, 8, 1, 1, 1, 0, 0);   /* one token, one expert */
  bad |= one_layer(3, 16, 5, 8, 2, 2, 0, 1, 0);  /* k0 = k */
  bad |= one_layer(9, 24, 12, 16, 6, 1, 1, 1, 1);
  bad |= general_routing(6, 9);
  bad |= general_routing(1, 4);
  bad |= general_routing(33, 3);
  if (bad) {
    printf("oracle sanitize: FAILED\n");
    return 1;
  }
  printf("oracle sanitize: ok\n");
  return 0;
}
