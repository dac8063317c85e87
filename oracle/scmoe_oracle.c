/*
 * scmoe_oracle.c — plain CPU statement of what one ScMoE block's forward pass computes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is compared with;
 * nothing in the product path may call it, and it shares no code, header, table or helper
 * with the HIP sources.  It is written for checking by eye against the paper, not for
 * speed: scalar loops, one token / one expert / one output element at a time, fp64
 * accumulation everywhere except where a rounding decides an integer (the gate logits).
 *
 * Passages followed (ScMoE paper):
 *   Eq. (1)      MoE(x) = sum_i G(x)_i E_i(x)
 *   Eq. (2)-(3)  G(x) = Softmax(TopK-masked H(x))
 *   Eq. (4)      H(x)_i = (x . W_gate)_i + eps_i      (eps: a fixed additive bias or 0)
 *   Eq. (6)      shared-expert MoE: SE(x) + sum_i G(x)_i E_i(x)
 *   Eq. (7)      ScMoE block: H_cur + SE(H_cur) + sum_i G(H_prev)_i E_i(H_prev)
 *   Eq. (14)-(17) coefficient gates CG-1 / CG-2
 *   Sec. 2.2     workflow: gate routing, input encode, expert computation, output decode
 *
 * Readings taken where the paper is silent (each is a stated choice, not a fact of the
 * paper): capacity drop policy = token order, first choices before second choices;
 * expert = Linear -> GELU (erf form, tanh optional) -> Linear; top-1 gate weight = full
 * softmax probability of the chosen expert; ties -> lowest expert index.
 *
 * Parity pins: every function below is pinned by the CPU tests (brute force on tiny
 * inputs, closed forms, library cross-checks, invariants); none is "parity unpinned"
 * with respect to the stated readings.  Parity with the paper authors' own code is
 * unpinned: the paper prints no input/output values.
 *
 * Inputs are fp32 arrays.  For bf16 workloads the caller passes the bf16 values widened
 * to fp32 (exact), so both sides start from identical numbers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_GELU_ERF 0
#define ORACLE_GELU_TANH 1
#define ORACLE_MAX_TOPK 8

/* Round a double to the nearest bf16 value (ties to even) and return it as a double.
 * Used only by the optional "mimic" mode, which rounds intermediates where a bf16
 * pipeline stores them so that a disagreement can be localised. */
static double round_to_bf16(double v) {
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* The rounding above, exported so that the tests can pin its tie rule and direction. */
double oracle_round_to_bf16(double v) { return round_to_bf16(v); }

/* GELU.  Exact form: v * Phi(v) with Phi the standard normal CDF written through erf.
 * Tanh form: 0.5 v (1 + tanh( sqrt(2/pi) (v + 0.044715 v^3) )). */
static double gelu(double v, int mode) {
  if (mode == ORACLE_GELU_TANH) {
    const double c = 0.7978845608028654; /* sqrt(2/pi) */
    return 0.5 * v * (1.0 + tanh(c * (v + 0.044715 * v * v * v)));
  }
  return 0.5 * v * (1.0 + erf(v * 0.7071067811865476));
}

double oracle_gelu(double v, int mode) { return gelu(v, mode); }

/*
 * Eq. (4): gate logits.  The rounding of the logits decides the arg max, so the
 * arithmetic is fixed: fp32, one fused multiply-add per input feature in ascending
 * feature order starting from 0, then one rounded add of the bias.
 * x: [T, d] stride ldx; Wg: [d, E]; bias: [E] or NULL; logits: [T, E].
 */
void oracle_gate_logits(const float* x, long ldx, const float* Wg, const float* bias, int T,
                        int d, int E, float* logits) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    for (int e = 0; e < E; ++e) {
      float acc = 0.0f;
      for (int i = 0; i < d; ++i) acc = fmaf(x[(long)t * ldx + i], Wg[(long)i * E + e], acc);
      if (bias) acc = acc + bias[e];
      logits[(long)t * E + e] = acc;
    }
  }
}

/* The same logits in fp64 with plain multiply and add: the "true" value, used by the
 * tests to tell tokens whose arg max is decided by rounding from the rest. */
void oracle_gate_logits_f64(const float* x, long ldx, const float* Wg, const float* bias,
                            int T, int d, int E, double* logits) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    for (int e = 0; e < E; ++e) {
      double acc = 0.0;
      for (int i = 0; i < d; ++i) acc += (double)x[(long)t * ldx + i] * (double)Wg[(long)i * E + e];
      if (bias) acc += (double)bias[e];
      logits[(long)t * E + e] = acc;
    }
  }
}

/*
 * Eq. (2)-(3): top-k selection and gate weights from given logits, 1 <= k <= min(E,
 * ORACLE_MAX_TOPK) (the paper's layers use k = 1, 2 and, in the Table 4 baselines, 3).
 * Selection: largest logit, lowest index on ties, a NaN never wins over a number (a row
 * of NaNs selects the lowest indices); each further choice the same over the experts not
 * chosen yet, so idx[t] lists the k largest logits in descending order.
 * probs = softmax over all E logits (fp64, max subtracted).
 * normalize == 0: w_j = probs[idx_j].  normalize == 1: softmax over the k selected logits
 * only, which is Eq. (2) taken literally (k = 1 gives 1).
 * idx, w: [T, k]; probs: [T, E] or NULL.
 */
void oracle_gate_topk(const float* logits, int T, int E, int k, int normalize, int32_t* idx,
                      float* w, float* probs) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    const float* l = logits + (long)t * E;
    int sel[ORACLE_MAX_TOPK];
    for (int j = 0; j < k; ++j) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        int taken = 0;                     /* the j-th choice skips the j earlier ones */
        for (int i = 0; i < j; ++i) taken |= (sel[i] == e);
        if (taken) continue;
        if (best < 0) { best = e; continue; }
        /* a candidate replaces the best only if strictly larger, or if the best so far
         * is NaN and the candidate is not */
        if (l[e] > l[best] || (isnan(l[best]) && !isnan(l[e]))) best = e;
      }
      sel[j] = best;
      idx[(long)t * k + j] = best;
    }
    /* full softmax */
    double m = -INFINITY;
    for (int e = 0; e < E; ++e)
      if ((double)l[e] > m) m = (double)l[e];
    double sum = 0.0;
    for (int e = 0; e < E; ++e) sum += exp((double)l[e] - m);
    if (probs)
      for (int e = 0; e < E; ++e) probs[(long)t * E + e] = (float)(exp((double)l[e] - m) / sum);
    if (!normalize) {
      for (int j = 0; j < k; ++j) w[(long)t * k + j] = (float)(exp((double)l[sel[j]] - m) / sum);
    } else {
      double ms = (double)l[sel[0]];
      double ssum = 0.0;
      for (int j = 0; j < k; ++j) ssum += exp((double)l[sel[j]] - ms);
      for (int j = 0; j < k; ++j) w[(long)t * k + j] = (float)(exp((double)l[sel[j]] - ms) / ssum);
    }
  }
}

/*
 * Sec. 2.2 "input encode" under a capacity C (capacity factor of Tables 8-9).
 * Walk the items in order (all first choices by ascending token, then all second
 * choices, and so on for each further choice).  An item's slot in its expert is the number of earlier items sent there; it
 * is kept iff slot < C.  Kept items are packed expert by expert, in slot order.
 * idx: [T, k]; counts: [E]; offsets: [E+1]; dst_row: [T, k] (-1 = dropped);
 * src_token: [>= number kept].
 * An index outside [0, E) is treated as dropped.
 */
void oracle_dispatch(const int32_t* idx, int T, int E, int k, int C, int32_t* counts,
                     int32_t* offsets, int32_t* dst_row, int32_t* src_token) {
  int64_t* seen = (int64_t*)calloc((size_t)E, sizeof(int64_t));
  int32_t* slot = (int32_t*)malloc(sizeof(int32_t) * (size_t)T * (size_t)k + 4);
  for (int j = 0; j < k; ++j)
    for (int t = 0; t < T; ++t) {
      int e = idx[(long)t * k + j];
      if (e < 0 || e >= E) { slot[(long)t * k + j] = -1; continue; }
      slot[(long)t * k + j] = (seen[e] < C) ? (int32_t)seen[e] : -1;
      seen[e] += 1;
    }
  offsets[0] = 0;
  for (int e = 0; e < E; ++e) {
    counts[e] = (int32_t)(seen[e] < C ? seen[e] : C);
    offsets[e + 1] = offsets[e] + counts[e];
  }
  for (int t = 0; t < T; ++t)
    for (int j = 0; j < k; ++j) {
      long i = (long)t * k + j;
      if (slot[i] < 0) { dst_row[i] = -1; continue; }
      dst_row[i] = offsets[idx[i]] + slot[i];
      src_token[dst_row[i]] = t;
    }
  free(seen);
  free(slot);
}

/*
 * One expert applied to one token (Sec. 2.1: an expert is an MLP):
 *   h = GELU(W1 x + b1),  out = W2 h + b2.
 * W1: [F, d], W2: [d, F] ([out, in]); b1 [F], b2 [d] or NULL.  fp64 throughout.
 * mimic != 0 rounds h to bf16 after the GELU and `out` to bf16 at the end.
 * scratch: F doubles.
 */
static void expert_token(const float* x, int d, int F, const float* W1, const float* b1,
                         const float* W2, const float* b2, int gelu_mode, int mimic,
                         double* scratch, double* out) {
  for (int f = 0; f < F; ++f) {
    double acc = 0.0;
    const float* wrow = W1 + (long)f * d;
    for (int i = 0; i < d; ++i) acc += (double)wrow[i] * (double)x[i];
    if (b1) acc += (double)b1[f];
    double h = gelu(acc, gelu_mode);
    scratch[f] = mimic ? round_to_bf16(h) : h;
  }
  for (int j = 0; j < d; ++j) {
    double acc = 0.0;
    const float* wrow = W2 + (long)j * F;
    for (int f = 0; f < F; ++f) acc += (double)wrow[f] * scratch[f];
    if (b2) acc += (double)b2[j];
    out[j] = mimic ? round_to_bf16(acc) : acc;
  }
}

/*
 * Expert computation over packed segments (Eq. (1), Sec. 2.2 "expert computation"):
 * rows offsets[e] .. offsets[e+1]-1 of x_perm go through expert e.
 * x_perm: [K, d] stride ldx; W1: [E, F, d]; W2: [E, d, F]; b1 [E, F], b2 [E, d] or NULL;
 * y_perm: [K, d] fp64, stride d.
 */
void oracle_expert_ffn(const float* x_perm, long ldx, const int32_t* offsets, int E, int d,
                       int F, const float* W1, const float* b1, const float* W2,
                       const float* b2, int gelu_mode, int mimic, double* y_perm) {
  for (int e = 0; e < E; ++e) {
    const float* W1e = W1 + (long)e * F * d;
    const float* W2e = W2 + (long)e * d * F;
    const float* b1e = b1 ? b1 + (long)e * F : NULL;
    const float* b2e = b2 ? b2 + (long)e * d : NULL;
#pragma omp parallel
    {
      double* scratch = (double*)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(dynamic, 4)
      for (int r = offsets[e]; r < offsets[e + 1]; ++r)
        expert_token(x_perm + (long)r * ldx, d, F, W1e, b1e, W2e, b2e, gelu_mode, mimic,
                     scratch, y_perm + (long)r * d);
      free(scratch);
    }
  }
}

/*
 * Eq. (14)-(17): coefficients of the coefficient gate for one token, fp64.
 * mode 0: (1, 1).  CG-1: (sigmoid(Wcg . x), 1).  CG-2: softmax of the two dot products.
 */
static void coef_token(const float* x, int d, const float* Wcg, int mode, double* c0,
                       double* c1) {
  *c0 = 1.0;
  *c1 = 1.0;
  if (mode == 1) {
    double a = 0.0;
    for (int i = 0; i < d; ++i) a += (double)Wcg[i] * (double)x[i];
    *c0 = 1.0 / (1.0 + exp(-a));
  } else if (mode == 2) {
    double a = 0.0, b = 0.0;
    for (int i = 0; i < d; ++i) {
      a += (double)Wcg[i] * (double)x[i];
      b += (double)Wcg[d + i] * (double)x[i];
    }
    double m = a > b ? a : b;
    double ea = exp(a - m), eb = exp(b - m);
    *c0 = ea / (ea + eb);
    *c1 = eb / (ea + eb);
  }
}

void oracle_coef_gate(const float* x, long ldx, const float* Wcg, int mode, int T, int d,
                      double* coef) {
  for (int t = 0; t < T; ++t) coef_token(x + (long)t * ldx, d, Wcg, mode, &coef[2 * t], &coef[2 * t + 1]);
}

/*
 * Output decode + merge for given per-row expert outputs (Sec. 2.2 "output decode",
 * Eq. (6)/(7)):  y[t] = c0 base[t] + c1 sum_j w[t,j] y_perm[dst_row[t,j]] + residual[t].
 * y_perm, base, residual: fp64 arrays of stride d (base/residual/coef may be NULL).
 */
void oracle_combine(const double* y_perm, const int32_t* dst_row, const float* w, int T,
                    int d, int k, const double* base, const double* residual,
                    const double* coef, double* y) {
  for (int t = 0; t < T; ++t) {
    double c0 = coef ? coef[2 * t] : 1.0, c1 = coef ? coef[2 * t + 1] : 1.0;
    for (int i = 0; i < d; ++i) {
      double routed = 0.0;
      for (int j = 0; j < k; ++j) {
        int r = dst_row[(long)t * k + j];
        if (r >= 0) routed += (double)w[(long)t * k + j] * y_perm[(long)r * d + i];
      }
      double v = c1 * routed;
      if (base) v += c0 * base[(long)t * d + i];
      if (residual) v += residual[(long)t * d + i];
      y[(long)t * d + i] = v;
    }
  }
}

/* Bundle of layer weights (all fp32 host arrays; NULL where optional). */
typedef struct oracle_weights {
  const float* Wg;   /* [d, E] */
  const float* bias; /* [E]    */
  const float* W1;   /* [E, F, d] */
  const float* b1;   /* [E, F] */
  const float* W2;   /* [E, d, F] */
  const float* b2;   /* [E, d] */
  const float* W1s;  /* [F, d] */
  const float* b1s;  /* [F] */
  const float* W2s;  /* [d, F] */
  const float* b2s;  /* [d] */
  const float* Wcg;  /* [1 or 2, d] */
} oracle_weights;

/*
 * Rows of the ScMoE block output, Eq. (7), for a list of tokens, given the routing
 * (expert index, gate weight, kept flag) already decided for every token:
 *
 *   y[t] = c0 SE(x_cur[t]) + c1 sum_j kept(t,j) w[t,j] E_{idx[t,j]}(x_src[t]) (+ x_cur[t])
 *
 * `shared` selects the ScMoE / shared-expert form (SE term present, routed experts read
 * x_prev); with shared == 0 it is the standard top-k layer of Eq. (1) (routed experts
 * read x_cur, no SE term).  tokens: [n] token ids; y: [n, d] fp64.
 * dst_row is used only for its sign (kept or dropped).
 */
void oracle_layer_rows(const float* x_prev, long ld_prev, const float* x_cur, long ld_cur,
                       const oracle_weights* W, int d, int F, int k, int shared, int cg_mode,
                       int gelu_mode, int mimic, int add_residual, const int32_t* idx,
                       const float* w, const int32_t* dst_row, const int32_t* tokens, int n,
                       double* y) {
#pragma omp parallel
  {
    double* scratch = (double*)malloc(sizeof(double) * (size_t)F);
    double* tmp = (double*)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
    for (int q = 0; q < n; ++q) {
      int t = tokens[q];
      double* yt = y + (long)q * d;
      double c0 = 1.0, c1 = 1.0;
      if (cg_mode) coef_token(x_cur + (long)t * ld_cur, d, W->Wcg, cg_mode, &c0, &c1);
      for (int i = 0; i < d; ++i) yt[i] = 0.0;
      const float* xr = shared ? x_prev + (long)t * ld_prev : x_cur + (long)t * ld_cur;
      for (int j = 0; j < k; ++j) {
        long it = (long)t * k + j;
        if (dst_row[it] < 0) continue; /* dropped: contributes exactly zero */
        int e = idx[it];
        expert_token(xr, d, F, W->W1 + (long)e * F * d, W->b1 ? W->b1 + (long)e * F : NULL,
                     W->W2 + (long)e * d * F, W->b2 ? W->b2 + (long)e * d : NULL, gelu_mode,
                     mimic, scratch, tmp);
        for (int i = 0; i < d; ++i) yt[i] += (double)w[it] * tmp[i];
      }
      for (int i = 0; i < d; ++i) yt[i] *= c1;
      if (shared) {
        expert_token(x_cur + (long)t * ld_cur, d, F, W->W1s, W->b1s, W->W2s, W->b2s, gelu_mode,
                     mimic, scratch, tmp);
        for (int i = 0; i < d; ++i) yt[i] += c0 * tmp[i];
      }
      if (add_residual)
        for (int i = 0; i < d; ++i) yt[i] += (double)x_cur[(long)t * ld_cur + i];
    }
    free(scratch);
    free(tmp);
  }
}

/*
 * The whole block for all tokens: gate (Eq. (2)-(4)) on x_prev (ScMoE) or x_cur (standard
 * layer), capacity-bounded encode, experts, decode and merge.  Returns the routing too.
 * y: [T, d] fp64.  idx, w, dst_row: [T, k]; counts [E]; offsets [E+1]; src_token [T*k].
 */
void oracle_layer_forward(const float* x_prev, long ld_prev, const float* x_cur, long ld_cur,
                          const oracle_weights* W, int T, int d, int F, int E, int k, int C,
                          int shared, int normalize, int cg_mode, int gelu_mode, int mimic,
                          int add_residual, int32_t* idx, float* w, int32_t* counts,
                          int32_t* offsets, int32_t* dst_row, int32_t* src_token, double* y) {
  float* logits = (float*)malloc(sizeof(float) * (size_t)T * (size_t)E + 4);
  const float* xg = shared ? x_prev : x_cur;
  long ldg = shared ? ld_prev : ld_cur;
  oracle_gate_logits(xg, ldg, W->Wg, W->bias, T, d, E, logits);
  oracle_gate_topk(logits, T, E, k, normalize, idx, w, NULL);
  oracle_dispatch(idx, T, E, k, C, counts, offsets, dst_row, src_token);
  int32_t* tokens = (int32_t*)malloc(sizeof(int32_t) * (size_t)T + 4);
  for (int t = 0; t < T; ++t) tokens[t] = t;
  oracle_layer_rows(x_prev, ld_prev, x_cur, ld_cur, W, d, F, k, shared, cg_mode, gelu_mode,
                    mimic, add_residual, idx, w, dst_row, tokens, T, y);
  free(tokens);
  free(logits);
}

/* Capacity from the capacity factor: C = ceil(cf * k * T / E).  The product is formed in
 * long double and a ceiling within 1e-9 of an integer is taken as that integer, so that
 * factors like 1.25 or 1.0 give the exact value. */
int oracle_capacity(int T, int E, int k, double cf) {
  long double v = (long double)cf * (long double)k * (long double)T / (long double)E;
  long double r = roundl(v);
  if (fabsl(v - r) < 1e-9L) return (int)r;
  return (int)ceill(v);
}
