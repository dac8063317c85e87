/*
 * Driver for a sanitizer build of the CPU oracle (test infrastructure).
 *
 * tests/test_oracle_sanitize.py compiles this file together with oracle/scmoe_oracle.c under
 * -fsanitize=address,undefined, runs it in a child process and compares the printed sums with
 * what the ordinary build of the oracle returns for the same inputs.  Every exported function
 * is called, on shapes chosen to reach the ends of its arrays: empty inputs, an empty expert
 * segment, capacity 0, expert indices outside [0, E), k up to 4, rows past offsets[E].
 *
 * Inputs come from a 32-bit linear congruential generator that the Python test repeats.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle_weights {
  const float *Wg, *bias, *W1, *b1, *W2, *b2, *W1s, *b1s, *W2s, *b2s, *Wcg;
} oracle_weights;

double oracle_round_to_bf16(double v);
double oracle_gelu(double v, int mode);
int oracle_capacity(int T, int E, int k, double cf);
void oracle_gate_logits(const float*, long, const float*, const float*, int, int, int, float*);
void oracle_gate_logits_f64(const float*, long, const float*, const float*, int, int, int, double*);
void oracle_gate_topk(const float*, int, int, int, int, int32_t*, float*, float*);
void oracle_dispatch(const int32_t*, int, int, int, int, int32_t*, int32_t*, int32_t*, int32_t*);
void oracle_expert_ffn(const float*, long, const int32_t*, int, int, int, const float*, const float*,
                       const float*, const float*, int, int, double*);
void oracle_coef_gate(const float*, long, const float*, int, int, int, double*);
void oracle_combine(const double*, const int32_t*, const float*, int, int, int, const double*,
                    const double*, const double*, double*);
void oracle_layer_rows(const float*, long, const float*, long, const oracle_weights*, int, int, int, int,
                       int, int, int, int, const int32_t*, const float*, const int32_t*, const int32_t*,
                       int, double*);
void oracle_layer_forward(const float*, long, const float*, long, const oracle_weights*, int, int, int, int,
                          int, int, int, int, int, int, int, int, int32_t*, float*, int32_t*, int32_t*,
                          int32_t*, int32_t*, double*);

static uint32_t lcg_state = 1u;
static uint32_t lcg(void) {
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return lcg_state;
}
/* uniform in [-0.5, 0.5) with 24 bits: exactly representable in fp32 */
static float unif(void) { return (float)(lcg() >> 8) / 16777216.0f - 0.5f; }

/* exactly-sized heap arrays, so that the sanitizer sees every step past an end */
static float* fvec(size_t n, float scale) {
  float* p = (float*)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) p[i] = scale * unif();
  return p;
}
static double dsum(const double* a, size_t n) {
  double s = 0.0;
  for (size_t i = 0; i < n; ++i) s += a[i] * (double)(1 + (i % 7));
  return s;
}
static double fsum(const float* a, size_t n) {
  double s = 0.0;
  for (size_t i = 0; i < n; ++i) s += (double)a[i] * (double)(1 + (i % 7));
  return s;
}
static long isum(const int32_t* a, size_t n) {
  long s = 0;
  for (size_t i = 0; i < n; ++i) s += (long)a[i] * (long)(1 + (i % 11));
  return s;
}

static void case_gate(int T, int d, int E, int k, int normalize, int with_bias) {
  float* x = fvec((size_t)T * d, 2.0f);
  float* Wg = fvec((size_t)d * E, 1.0f);
  float* bias = with_bias ? fvec((size_t)E, 0.5f) : NULL;
  float* lg = (float*)malloc(sizeof(float) * ((size_t)T * E + 1));
  double* lg64 = (double*)malloc(sizeof(double) * ((size_t)T * E + 1));
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * ((size_t)T * k + 1));
  float* w = (float*)malloc(sizeof(float) * ((size_t)T * k + 1));
  float* probs = (float*)malloc(sizeof(float) * ((size_t)T * E + 1));
  oracle_gate_logits(x, d, Wg, bias, T, d, E, lg);
  oracle_gate_logits_f64(x, d, Wg, bias, T, d, E, lg64);
  oracle_gate_topk(lg, T, E, k, normalize, idx, w, probs);
  printf("gate T=%d d=%d E=%d k=%d n=%d b=%d %.17g %.17g %ld %.17g %.17g\n", T, d, E, k, normalize, with_bias,
         fsum(lg, (size_t)T * E), dsum(lg64, (size_t)T * E), isum(idx, (size_t)T * k), fsum(w, (size_t)T * k),
         fsum(probs, (size_t)T * E));
  free(x); free(Wg); free(bias); free(lg); free(lg64); free(idx); free(w); free(probs);
}

static void case_dispatch(int T, int E, int k, int C, int with_invalid) {
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * ((size_t)T * k + 1));
  for (int i = 0; i < T * k; ++i) {
    idx[i] = (int32_t)(lcg() >> 8) % E;
    if (with_invalid && (i % 13) == 5) idx[i] = (i % 2) ? -1 : E;
  }
  int32_t* counts = (int32_t*)calloc((size_t)E, sizeof(int32_t));
  int32_t* offsets = (int32_t*)calloc((size_t)E + 1, sizeof(int32_t));
  int32_t* dst = (int32_t*)malloc(sizeof(int32_t) * ((size_t)T * k + 1));
  size_t cap = (size_t)E * (size_t)C < (size_t)T * k ? (size_t)E * (size_t)C : (size_t)T * k;
  int32_t* src = (int32_t*)malloc(sizeof(int32_t) * (cap + 1));   /* room for exactly the rows that can be kept */
  for (size_t i = 0; i < cap + 1; ++i) src[i] = -7;
  oracle_dispatch(idx, T, E, k, C, counts, offsets, dst, src);
  printf("dispatch T=%d E=%d k=%d C=%d inv=%d %ld %ld %ld %ld\n", T, E, k, C, with_invalid, isum(counts, (size_t)E),
         isum(offsets, (size_t)E + 1), isum(dst, (size_t)T * k), isum(src, (size_t)offsets[E]));
  free(idx); free(counts); free(offsets); free(dst); free(src);
}

static void case_ffn(int E, const int* lens, int extra, int d, int F, int biases, int gelu_mode, int mimic) {
  int32_t* offsets = (int32_t*)malloc(sizeof(int32_t) * ((size_t)E + 1));
  offsets[0] = 0;
  for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + lens[e];
  const int K = offsets[E] + extra;
  float* x = fvec((size_t)K * d, 2.0f);
  float* W1 = fvec((size_t)E * F * d, 0.6f);
  float* W2 = fvec((size_t)E * d * F, 0.6f);
  float* b1 = biases ? fvec((size_t)E * F, 0.3f) : NULL;
  float* b2 = biases ? fvec((size_t)E * d, 0.3f) : NULL;
  double* y = (double*)calloc((size_t)K * d + 1, sizeof(double));
  oracle_expert_ffn(x, d, offsets, E, d, F, W1, b1, W2, b2, gelu_mode, mimic, y);
  printf("ffn E=%d K=%d d=%d F=%d b=%d g=%d m=%d %.17g\n", E, K, d, F, biases, gelu_mode, mimic, dsum(y, (size_t)K * d));
  free(offsets); free(x); free(W1); free(W2); free(b1); free(b2); free(y);
}

static void case_combine(int T, int d, int k, int use_base, int use_res, int use_coef) {
  const int K = T * k;
  double* yp = (double*)malloc(sizeof(double) * ((size_t)K * d + 1));
  for (size_t i = 0; i < (size_t)K * d; ++i) yp[i] = (double)unif();
  int32_t* dst = (int32_t*)malloc(sizeof(int32_t) * ((size_t)K + 1));
  for (int i = 0; i < K; ++i) dst[i] = (i % 5 == 3) ? -1 : (K - 1 - i);
  float* w = fvec((size_t)K, 1.0f);
  double* base = NULL; double* res = NULL; double* coef = NULL;
  if (use_base) { base = (double*)malloc(sizeof(double) * ((size_t)T * d + 1)); for (size_t i = 0; i < (size_t)T * d; ++i) base[i] = (double)unif(); }
  if (use_res) { res = (double*)malloc(sizeof(double) * ((size_t)T * d + 1)); for (size_t i = 0; i < (size_t)T * d; ++i) res[i] = (double)unif(); }
  if (use_coef) { coef = (double*)malloc(sizeof(double) * ((size_t)T * 2 + 1)); for (size_t i = 0; i < (size_t)T * 2; ++i) coef[i] = (double)unif(); }
  double* y = (double*)malloc(sizeof(double) * ((size_t)T * d + 1));
  oracle_combine(yp, dst, w, T, d, k, base, res, coef, y);
  printf("combine T=%d d=%d k=%d %d%d%d %.17g\n", T, d, k, use_base, use_res, use_coef, dsum(y, (size_t)T * d));
  free(yp); free(dst); free(w); free(base); free(res); free(coef); free(y);
}

static void case_layer(int T, int d, int F, int E, int k, int C, int shared, int normalize, int cg, int gelu_mode,
                       int mimic, int residual, int biases) {
  float* xp = fvec((size_t)T * d, 2.0f);
  float* xc = fvec((size_t)T * d, 2.0f);
  oracle_weights W;
  memset(&W, 0, sizeof(W));
  float* Wg = fvec((size_t)d * E, 1.0f);
  float* gb = biases ? fvec((size_t)E, 0.3f) : NULL;
  float* W1 = fvec((size_t)E * F * d, 0.6f);
  float* W2 = fvec((size_t)E * d * F, 0.6f);
  float* W1s = fvec((size_t)F * d, 0.6f);
  float* W2s = fvec((size_t)d * F, 0.6f);
  float* b1 = biases ? fvec((size_t)E * F, 0.3f) : NULL;
  float* b2 = biases ? fvec((size_t)E * d, 0.3f) : NULL;
  float* b1s = biases ? fvec((size_t)F, 0.3f) : NULL;
  float* b2s = biases ? fvec((size_t)d, 0.3f) : NULL;
  float* Wcg = cg ? fvec((size_t)cg * d, 1.0f) : NULL;
  W.Wg = Wg; W.bias = gb; W.W1 = W1; W.b1 = b1; W.W2 = W2; W.b2 = b2;
  W.W1s = W1s; W.b1s = b1s; W.W2s = W2s; W.b2s = b2s; W.Wcg = Wcg;
  const size_t n = (size_t)T * k;
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (n + 1));
  float* w = (float*)malloc(sizeof(float) * (n + 1));
  int32_t* counts = (int32_t*)calloc((size_t)E, sizeof(int32_t));
  int32_t* offsets = (int32_t*)calloc((size_t)E + 1, sizeof(int32_t));
  int32_t* dst = (int32_t*)malloc(sizeof(int32_t) * (n + 1));
  int32_t* src = (int32_t*)malloc(sizeof(int32_t) * (n + 1));
  double* y = (double*)malloc(sizeof(double) * ((size_t)T * d + 1));
  oracle_layer_forward(xp, d, xc, d, &W, T, d, F, E, k, C, shared, normalize, cg, gelu_mode, mimic, residual, idx, w,
                       counts, offsets, dst, src, y);
  /* the same rows once more through the per-token entry, last token first */
  int32_t* tokens = (int32_t*)malloc(sizeof(int32_t) * ((size_t)T + 1));
  for (int t = 0; t < T; ++t) tokens[t] = T - 1 - t;
  double* y2 = (double*)malloc(sizeof(double) * ((size_t)T * d + 1));
  oracle_layer_rows(xp, d, xc, d, &W, d, F, k, shared, cg, gelu_mode, mimic, residual, idx, w, dst, tokens, T, y2);
  double* cf = (double*)malloc(sizeof(double) * ((size_t)T * 2 + 1));
  if (cg) oracle_coef_gate(xc, d, Wcg, cg, T, d, cf);
  printf("layer T=%d d=%d F=%d E=%d k=%d C=%d s=%d n=%d cg=%d g=%d m=%d r=%d b=%d %.17g %.17g %ld %ld %.17g\n", T, d, F, E,
         k, C, shared, normalize, cg, gelu_mode, mimic, residual, biases, dsum(y, (size_t)T * d), dsum(y2, (size_t)T * d),
         isum(idx, n), isum(dst, n), cg ? dsum(cf, (size_t)T * 2) : 0.0);
  free(xp); free(xc); free(Wg); free(gb); free(W1); free(W2); free(W1s); free(W2s); free(b1); free(b2); free(b1s);
  free(b2s); free(Wcg); free(idx); free(w); free(counts); free(offsets); free(dst); free(src); free(y); free(tokens);
  free(y2); free(cf);
}

int main(void) {
  printf("scalar %.17g %.17g %.17g %.17g %d %d %d\n", oracle_round_to_bf16(1.00390625), oracle_round_to_bf16(-3.1415926),
         oracle_gelu(0.7, 0), oracle_gelu(-1.3, 1), oracle_capacity(8192, 8, 1, 1.25), oracle_capacity(100, 7, 2, 1.0),
         oracle_capacity(0, 3, 1, 2.0));
  case_gate(37, 24, 5, 1, 0, 1);
  case_gate(37, 24, 5, 2, 1, 0);
  case_gate(9, 8, 4, 4, 1, 1);
  case_gate(5, 16, 1, 1, 0, 0);
  case_gate(0, 8, 3, 1, 0, 1);
  case_dispatch(70, 4, 1, 10, 0);
  case_dispatch(70, 4, 2, 0, 1);
  case_dispatch(64, 3, 3, 200, 1);
  case_dispatch(1, 1, 1, 1, 0);
  case_dispatch(0, 5, 2, 4, 0);
  { const int lens[3] = {5, 0, 9}; case_ffn(3, lens, 4, 12, 20, 1, 0, 0); }
  { const int lens[2] = {7, 1}; case_ffn(2, lens, 0, 8, 16, 0, 1, 1); }
  { const int lens[1] = {0}; case_ffn(1, lens, 3, 8, 8, 1, 0, 1); }
  case_combine(11, 6, 1, 1, 0, 0);
  case_combine(11, 6, 2, 1, 1, 1);
  case_combine(4, 3, 4, 0, 0, 0);
  case_combine(0, 5, 1, 1, 1, 1);
  case_layer(23, 12, 20, 4, 1, 4, 1, 0, 0, 0, 0, 0, 1);
  case_layer(23, 12, 20, 4, 2, 9, 1, 1, 2, 1, 1, 1, 0);
  case_layer(19, 8, 16, 3, 3, 57, 0, 1, 0, 0, 0, 0, 1);
  case_layer(17, 8, 16, 5, 1, 0, 1, 0, 1, 0, 0, 1, 0);
  case_layer(0, 8, 8, 2, 1, 3, 1, 0, 0, 0, 0, 0, 0);
  printf("done\n");
  return 0;
}
