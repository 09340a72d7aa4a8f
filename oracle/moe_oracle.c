/*
 * CPU oracle for one GPU's share of an expert-parallel MoE layer.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be checked against a plain,
 * slow, obviously-correct statement of what the layer computes.  It shares no code, header, table
 * or helper with the GPU library, and nothing in the product path may call it.
 *
 * What is computed follows the paper's problem statement:
 *   - MoE structure (Sec. II-A): every token activates its top-k experts as chosen by the gate; each
 *     activated expert runs its FFN (GEMM-1, GEMM-2); the k outputs are aggregated.
 *   - Weighted aggregation (Sec. III-C): expert output o_i is scaled by gate weight w_i and the scaled
 *     outputs are summed without further weighting, y = sum_i (w_i * o_i).
 *   - Expert -> GPU map (Sec. III-D, switch routing): rank(e) = e / experts_per_rank.
 *   - Layout allocation (Sec. III-D, AL Table): each expert owns a dense layout tensor whose rows are
 *     handed out one after the other; here in ascending token order, which makes the table unique.
 *   - Per-expert active counts are known from routing before Dispatch (Sec. III-E, nactive[expert]).
 * The paper does not state the gate function or the FFN activation; the readings used are: softmax over
 * the logits, top-k on the raw logits with ties broken towards the lower expert index, weights
 * renormalised over the k picks, and a SwiGLU FFN  (silu(x Wg) * (x Wu)) Wd  without biases.
 *
 * Floating point: inputs are fp32 (or bf16 bit patterns widened exactly); all sums are accumulated in
 * MOE_ACC_T (double unless overridden at compile time with -DMOE_ACC_T=float) in ascending index order;
 * exp() is evaluated in double.  Nothing is blocked, fused or reordered beyond that.
 *
 * Pins (tests/, -m "not gpu"): brute-force NumPy re-derivations on tiny inputs, a hand-worked 4-token
 * example, the gate network against a library matrix product and unit-vector / hand-worked cases, sum-to-one and permutation invariants, the identical-experts == dense-FFN identity, the
 * closed-form expected dedup count, and the float-vs-double accumulation twin; for the FP8 layer the format's
 * definition and a library's conversions on all codes, midpoints and random values, and the layer restated with
 * that library's conversions and float64 library products.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef MOE_ACC_T
#define MOE_ACC_T double
#endif
typedef MOE_ACC_T acc_t;

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_NOMEM (-2)

/* element type codes of activations and weights */
#define ELT_F32 0
#define ELT_BF16 1

static inline float load_elt(const void *base, size_t i, int elt) {
  if (elt == ELT_F32) return ((const float *)base)[i];
  uint32_t bits = ((uint32_t)((const uint16_t *)base)[i]) << 16; /* bf16 -> fp32 is exact */
  float v;
  memcpy(&v, &bits, sizeof v);
  return v;
}

int moe_oracle_acc_bytes(void) { return (int)sizeof(acc_t); }

int moe_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * Gate network (Sec. II-A: the experts of a token are "selected by the gate network").  The paper does not
 * spell the network out; the reading used is the usual bias-free linear map: logit[t][e] = sum_c x[t][c] *
 * W_r[e][c], one row of W_r per expert, summed in ascending c.  logits is [T, E] in double.
 */
int moe_oracle_router_logits(int T, int d, int E, int elt, const void *x, const void *W_r, double *logits) {
  if (T < 0 || d < 1 || E < 1 || !x || !W_r || !logits) return ORACLE_BAD_ARG;
  if (elt != ELT_F32 && elt != ELT_BF16) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    for (int e = 0; e < E; ++e) {
      acc_t sum = 0;
      for (int c = 0; c < d; ++c)
        sum += (acc_t)load_elt(x, (size_t)t * d + c, elt) * (acc_t)load_elt(W_r, (size_t)e * d + c, elt);
      logits[(size_t)t * E + e] = (double)sum;
    }
  }
  return ORACLE_OK;
}

/*
 * Routing (Sec. II-A "topk experts selected by the gate network").
 * For each token: repeatedly take the not-yet-taken expert with the largest logit (lowest index on
 * ties); slot order is pick order.  w_j = exp(l_j - l_0) / sum_i exp(l_i - l_0), sum in slot order.
 * Returns ORACLE_BAD_ARG on a non-finite logit.
 */
int moe_oracle_route_topk(int T, int E, int k, const float *logits, int32_t *topk_idx, float *topk_w) {
  if (T < 0 || E < 1 || k < 1 || k > E || !logits || !topk_idx || !topk_w) return ORACLE_BAD_ARG;
  unsigned char *taken = (unsigned char *)malloc((size_t)E);
  if (!taken) return ORACLE_NOMEM;
  for (int t = 0; t < T; ++t) {
    const float *row = logits + (size_t)t * E;
    for (int e = 0; e < E; ++e) {
      if (!isfinite(row[e])) { free(taken); return ORACLE_BAD_ARG; }
      taken[e] = 0;
    }
    for (int j = 0; j < k; ++j) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        if (taken[e]) continue;
        if (best < 0 || row[e] > row[best]) best = e; /* strict '>' keeps the lowest index on ties */
      }
      taken[best] = 1;
      topk_idx[(size_t)t * k + j] = best;
    }
    double m = (double)row[topk_idx[(size_t)t * k]];
    double sum = 0.0;
    for (int j = 0; j < k; ++j) sum += exp((double)row[topk_idx[(size_t)t * k + j]] - m);
    for (int j = 0; j < k; ++j)
      topk_w[(size_t)t * k + j] = (float)(exp((double)row[topk_idx[(size_t)t * k + j]] - m) / sum);
  }
  free(taken);
  return ORACLE_OK;
}

/*
 * Routing with the gate variants of recent MoE models (the paper evaluates DeepSeek-V3, whose gate is of this kind,
 * and leaves the gate function open, Sec. II-A):
 *   gate 0 (softmax): selection value v_e = l_e + b_e; weights as in moe_oracle_route_topk (softmax over the
 *                     logits, renormalised over the picks);
 *   gate 1 (sigmoid): s_e = 1 / (1 + exp(-l_e)); selection value v_e = s_e + b_e; weights w_j = s_j / sum of the
 *                     picked s.
 * b (may be NULL = 0) is a per-expert bias that steers the selection only and never enters the weights.
 * Selection values are formed in fp32 (they decide an index, and fp32 is what the GPU kernel uses); the k largest
 * are taken, lowest index on ties, slot order = pick order.  sel_out (may be NULL) receives the [T, E] selection
 * values so that a caller can tell decisive picks from near-ties.
 */
int moe_oracle_route_topk_gate(int T, int E, int k, const float *logits, const float *bias, int gate,
                               int32_t *topk_idx, float *topk_w, float *sel_out) {
  if (T < 0 || E < 1 || k < 1 || k > E || !logits || !topk_idx || !topk_w || (gate != 0 && gate != 1))
    return ORACLE_BAD_ARG;
  unsigned char *taken = (unsigned char *)malloc((size_t)E);
  float *sel = (float *)malloc(sizeof(float) * (size_t)E);
  if (!taken || !sel) { free(taken); free(sel); return ORACLE_NOMEM; }
  for (int t = 0; t < T; ++t) {
    const float *row = logits + (size_t)t * E;
    for (int e = 0; e < E; ++e) {
      const float b = bias ? bias[e] : 0.0f;
      if (!isfinite(row[e]) || !isfinite(b)) { free(taken); free(sel); return ORACLE_BAD_ARG; }
      const float base = gate == 0 ? row[e] : 1.0f / (1.0f + expf(-row[e]));
      sel[e] = base + b;
      if (sel_out) sel_out[(size_t)t * E + e] = sel[e];
      taken[e] = 0;
    }
    for (int j = 0; j < k; ++j) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        if (taken[e]) continue;
        if (best < 0 || sel[e] > sel[best]) best = e;
      }
      taken[best] = 1;
      topk_idx[(size_t)t * k + j] = best;
    }
    double m = -INFINITY, sum = 0.0;
    for (int j = 0; j < k; ++j) {
      const double l = (double)row[topk_idx[(size_t)t * k + j]];
      if (l > m) m = l;
    }
    for (int j = 0; j < k; ++j) {
      const double l = (double)row[topk_idx[(size_t)t * k + j]];
      sum += gate == 0 ? exp(l - m) : 1.0 / (1.0 + exp(-l));
    }
    for (int j = 0; j < k; ++j) {
      const double l = (double)row[topk_idx[(size_t)t * k + j]];
      topk_w[(size_t)t * k + j] = (float)((gate == 0 ? exp(l - m) : 1.0 / (1.0 + exp(-l))) / sum);
    }
  }
  free(taken);
  free(sel);
  return ORACLE_OK;
}

/*
 * Dispatch tables (Sec. III-D AL Table; Sec. III-E nactive[expert]).
 * counts[e]  = number of (token, slot) pairs routed to e; offsets = exclusive prefix sum (E+1 entries).
 * Pairs are visited in ascending pair id p = t*k + j; the pair takes the next free row of its expert:
 * inv_perm[p] = row, perm[row] = p.
 */
int moe_oracle_build_tables(int T, int E, int k, const int32_t *topk_idx, int32_t *counts, int32_t *offsets,
                            int32_t *perm, int32_t *inv_perm) {
  if (T < 0 || E < 1 || k < 1 || !topk_idx || !counts || !offsets || !perm || !inv_perm) return ORACLE_BAD_ARG;
  for (int e = 0; e < E; ++e) counts[e] = 0;
  for (size_t p = 0; p < (size_t)T * k; ++p) {
    int e = topk_idx[p];
    if (e < 0 || e >= E) return ORACLE_BAD_ARG;
    counts[e]++;
  }
  offsets[0] = 0;
  for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
  int32_t *cursor = (int32_t *)calloc((size_t)E, sizeof(int32_t));
  if (!cursor) return ORACLE_NOMEM;
  for (size_t p = 0; p < (size_t)T * k; ++p) {
    int e = topk_idx[p];
    int32_t row = offsets[e] + cursor[e]++;
    inv_perm[p] = row;
    perm[row] = (int32_t)p;
  }
  free(cursor);
  return ORACLE_OK;
}

/*
 * Dedup table (Sec. II-B redundancy: one transfer per distinct (token, destination GPU);
 * Sec. III-D: destination = expert / experts_per_rank).
 * Entries are the distinct (rank, token) pairs in (rank ascending, token ascending) order;
 * dedup_mask has bit j set iff slot j of that token lies in that rank.  Needs k <= 32.
 */
int moe_oracle_build_dedup(int T, int E, int k, int R, const int32_t *topk_idx, int32_t *rank_counts,
                           int32_t *rank_offsets, int32_t *dedup_tok, uint32_t *dedup_mask,
                           int32_t *pair_to_dedup) {
  if (T < 0 || E < 1 || k < 1 || k > 32 || R < 1 || E % R != 0) return ORACLE_BAD_ARG;
  if (!topk_idx || !rank_counts || !rank_offsets || !dedup_tok || !dedup_mask || !pair_to_dedup)
    return ORACLE_BAD_ARG;
  const int epr = E / R;
  int32_t n = 0;
  rank_offsets[0] = 0;
  for (int r = 0; r < R; ++r) {
    rank_counts[r] = 0;
    for (int t = 0; t < T; ++t) {
      uint32_t mask = 0;
      for (int j = 0; j < k; ++j)
        if (topk_idx[(size_t)t * k + j] / epr == r) mask |= (uint32_t)1 << j;
      if (!mask) continue;
      dedup_tok[n] = t;
      dedup_mask[n] = mask;
      for (int j = 0; j < k; ++j)
        if (mask >> j & 1u) pair_to_dedup[(size_t)t * k + j] = n;
      ++n;
      rank_counts[r]++;
    }
    rank_offsets[r + 1] = n;
  }
  return ORACLE_OK;
}

/*
 * Forward for a list of tokens (Sec. II-A GEMM-1 / GEMM-2; Sec. III-C weighted sum).
 *   for each selected token t, for each slot j whose expert e is hosted by local ranks [lrb, lre):
 *     g = x_t Wg[le], u = x_t Wu[le], h = silu(g) * u, o = h Wd[le], y_t += w[t,j] * o
 * tokens == NULL means tokens 0..n_tok-1.  y_out is [n_tok, d] in double; rows without a local slot are 0.
 * Weights are indexed by local expert le = e - lrb*E/R and stored input-major: Wg,Wu [E_loc,d,f], Wd [E_loc,f,d].
 */
int moe_oracle_forward(int T, int d, int f, int E, int k, int R, int lrb, int lre, int elt, const void *x,
                       const int32_t *topk_idx, const float *topk_w, const void *W_gate, const void *W_up,
                       const void *W_down, const int32_t *tokens, int n_tok, double *y_out) {
  if (T < 0 || d < 1 || f < 1 || E < 1 || k < 1 || R < 1 || E % R != 0) return ORACLE_BAD_ARG;
  if (lrb < 0 || lre <= lrb || lre > R || (elt != ELT_F32 && elt != ELT_BF16)) return ORACLE_BAD_ARG;
  if (!x || !topk_idx || !topk_w || !W_gate || !W_up || !W_down || !y_out || n_tok < 0) return ORACLE_BAD_ARG;
  const int epr = E / R;
  const int e_lo = lrb * epr, e_hi = lre * epr;
  int status = ORACLE_OK;
#pragma omp parallel
  {
    acc_t *g = (acc_t *)malloc(sizeof(acc_t) * (size_t)f);
    acc_t *u = (acc_t *)malloc(sizeof(acc_t) * (size_t)f);
    acc_t *o = (acc_t *)malloc(sizeof(acc_t) * (size_t)d);
    acc_t *acc = (acc_t *)malloc(sizeof(acc_t) * (size_t)d);
    if (!g || !u || !o || !acc) {
#pragma omp critical
      status = ORACLE_NOMEM;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int i = 0; i < n_tok; ++i) {
        const int t = tokens ? tokens[i] : i;
        for (int m = 0; m < d; ++m) acc[m] = 0;
        if (t >= 0 && t < T) {
          for (int j = 0; j < k; ++j) {
            const int e = topk_idx[(size_t)t * k + j];
            if (e < e_lo || e >= e_hi) continue;
            const size_t le = (size_t)(e - e_lo);
            const size_t wgu = le * (size_t)d * f, wdn = le * (size_t)f * d;
            for (int n = 0; n < f; ++n) { g[n] = 0; u[n] = 0; }
            for (int c = 0; c < d; ++c) {
              const acc_t xc = (acc_t)load_elt(x, (size_t)t * d + c, elt);
              const size_t rowb = wgu + (size_t)c * f;
              for (int n = 0; n < f; ++n) {
                g[n] += xc * (acc_t)load_elt(W_gate, rowb + n, elt);
                u[n] += xc * (acc_t)load_elt(W_up, rowb + n, elt);
              }
            }
            for (int n = 0; n < f; ++n) {
              const double gv = (double)g[n];
              g[n] = (acc_t)((gv / (1.0 + exp(-gv))) * (double)u[n]); /* h = silu(g) * u, kept unrounded */
            }
            for (int m = 0; m < d; ++m) o[m] = 0;
            for (int n = 0; n < f; ++n) {
              const acc_t hn = g[n];
              const size_t rowb = wdn + (size_t)n * d;
              for (int m = 0; m < d; ++m) o[m] += hn * (acc_t)load_elt(W_down, rowb + m, elt);
            }
            const acc_t w = (acc_t)topk_w[(size_t)t * k + j];
            for (int m = 0; m < d; ++m) acc[m] += w * o[m];
          }
        }
        for (int m = 0; m < d; ++m) y_out[(size_t)i * d + m] = (double)acc[m];
      }
    }
    free(g); free(u); free(o); free(acc);
  }
  return status;
}

/* ------------------------------------------------------------------------------------------------------------
 * FP8 expert GEMMs.  The paper's DeepSeek-V3 runs use FP8 GEMM kernels (Sec. V-A) and says nothing more about
 * them; the reading used here:
 *   - number format: the 8-bit E4M3 format of the OCP 8-bit floating point specification (1 sign, 4 exponent bits
 *     with bias 7, 3 mantissa bits; no infinities; S.1111.111 is NaN; largest finite value 448; subnormals
 *     m/8 * 2^-6), the format the matrix cores of the target read;
 *   - conversion: round to nearest, ties to even; magnitudes above 448 saturate to 448;
 *   - scaling: one fp32 scale per token for x (amax of the row / 448), one per output column and expert for every
 *     weight matrix (amax over the reduction index / 448), a given (calibrated, static) scale per expert for h;
 *     a group that is all zero gets scale 1;  code = convert(value / scale) with the division in fp32;
 *   - GEMM-1: g, u = (sum of products of codes) * s_x[t] * s_w[le][n];  h = silu(g) * u, rounded to fp32, divided
 *     by s_h[le] in fp32 and converted;  GEMM-2: o = (sum of products of codes) * s_h[le] * s_wd[le][m];
 *     then the weighted sum of Sec. III-C as in the unquantised layer.
 * ------------------------------------------------------------------------------------------------------------ */

/* value of an E4M3 code (NaN codes give NaN) */
double moe_oracle_fp8_decode(uint8_t code) {
  const int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m / 8.0, -6);
  else v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return s ? -v : v;
}

/* fp32 -> E4M3: nearest code, ties to the code with even mantissa, saturating at +-448; NaN -> S.1111.111 */
uint8_t moe_oracle_fp8_encode(float value) {
  const uint8_t sign = signbit(value) ? 0x80 : 0x00;
  if (isnan(value)) return (uint8_t)(sign | 0x7F);
  const double a = fabs((double)value);
  if (a >= 448.0) return (uint8_t)(sign | 0x7E);
  if (a < ldexp(1.0, -6)) {
    /* subnormal range: multiples of 2^-9; rint() rounds ties to even in the default rounding mode */
    const int q = (int)rint(ldexp(a, 9)); /* 0..8; 8 is the smallest normal number, code 0x08 */
    return (uint8_t)(sign | q);
  }
  int ex;
  const double fr = frexp(a, &ex); /* a = fr * 2^ex, fr in [0.5, 1) */
  int e = ex - 1;                  /* a = (2 fr) * 2^e, 2 fr in [1, 2) */
  int q = (int)rint((2.0 * fr - 1.0) * 8.0); /* 0..8 */
  if (q == 8) { q = 0; ++e; }
  return (uint8_t)(sign | ((e + 7) << 3) | q); /* a < 448 keeps (e, q) at or below (8, 6) */
}

/*
 * Quantise n_groups groups of group_len values each: element i of group g is a[g * group_stride + i * elem_stride]
 * (rows of a matrix: group_stride = row length, elem_stride = 1; columns: group_stride = 1, elem_stride = row
 * length).  codes uses the same indexing, scales is [n_groups].
 */
int moe_oracle_fp8_quantize(const float *a, int64_t n_groups, int64_t group_len, int64_t group_stride,
                            int64_t elem_stride, uint8_t *codes, float *scales) {
  if (!a || !codes || !scales || n_groups < 0 || group_len < 1) return ORACLE_BAD_ARG;
#pragma omp parallel for schedule(static)
  for (int64_t g = 0; g < n_groups; ++g) {
    float amax = 0.0f;
    for (int64_t i = 0; i < group_len; ++i) {
      const float v = fabsf(a[g * group_stride + i * elem_stride]);
      if (v > amax) amax = v;
    }
    const float scale = amax > 0.0f ? amax / 448.0f : 1.0f;
    scales[g] = scale;
    for (int64_t i = 0; i < group_len; ++i) {
      const float v = a[g * group_stride + i * elem_stride] / scale; /* fp32 division */
      codes[g * group_stride + i * elem_stride] = moe_oracle_fp8_encode(v);
    }
  }
  return ORACLE_OK;
}

/*
 * Forward with FP8 operands (see the reading above).  xq [T,d] codes with s_x [T]; Wg, Wu codes [E_loc,d,f] with
 * scales [E_loc,f]; Wd codes [E_loc,f,d] with scales [E_loc,d]; s_h [E_loc].  Everything else as moe_oracle_forward.
 */
int moe_oracle_forward_fp8(int T, int d, int f, int E, int k, int R, int lrb, int lre, const uint8_t *xq,
                           const float *s_x, const int32_t *topk_idx, const float *topk_w, const uint8_t *Wg,
                           const float *s_g, const uint8_t *Wu, const float *s_u, const uint8_t *Wd,
                           const float *s_d, const float *s_h, const int32_t *tokens, int n_tok, double *y_out) {
  if (T < 0 || d < 1 || f < 1 || E < 1 || k < 1 || R < 1 || E % R != 0) return ORACLE_BAD_ARG;
  if (lrb < 0 || lre <= lrb || lre > R || n_tok < 0) return ORACLE_BAD_ARG;
  if (!xq || !s_x || !topk_idx || !topk_w || !Wg || !s_g || !Wu || !s_u || !Wd || !s_d || !s_h || !y_out)
    return ORACLE_BAD_ARG;
  const int epr = E / R;
  const int e_lo = lrb * epr, e_hi = lre * epr;
  double value[256];
  for (int c = 0; c < 256; ++c) value[c] = moe_oracle_fp8_decode((uint8_t)c);
  int status = ORACLE_OK;
#pragma omp parallel
  {
    acc_t *g = (acc_t *)malloc(sizeof(acc_t) * (size_t)f);
    acc_t *u = (acc_t *)malloc(sizeof(acc_t) * (size_t)f);
    acc_t *o = (acc_t *)malloc(sizeof(acc_t) * (size_t)d);
    acc_t *acc = (acc_t *)malloc(sizeof(acc_t) * (size_t)d);
    if (!g || !u || !o || !acc) {
#pragma omp critical
      status = ORACLE_NOMEM;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int i = 0; i < n_tok; ++i) {
        const int t = tokens ? tokens[i] : i;
        for (int m = 0; m < d; ++m) acc[m] = 0;
        if (t >= 0 && t < T) {
          for (int j = 0; j < k; ++j) {
            const int e = topk_idx[(size_t)t * k + j];
            if (e < e_lo || e >= e_hi) continue;
            const size_t le = (size_t)(e - e_lo);
            const size_t wgu = le * (size_t)d * f, wdn = le * (size_t)f * d;
            for (int n = 0; n < f; ++n) { g[n] = 0; u[n] = 0; }
            for (int c = 0; c < d; ++c) {
              const acc_t xc = (acc_t)value[xq[(size_t)t * d + c]];
              const size_t rowb = wgu + (size_t)c * f;
              for (int n = 0; n < f; ++n) {
                g[n] += xc * (acc_t)value[Wg[rowb + n]];
                u[n] += xc * (acc_t)value[Wu[rowb + n]];
              }
            }
            for (int n = 0; n < f; ++n) {
              const double gv = (double)g[n] * (double)s_x[t] * (double)s_g[le * f + n];
              const double uv = (double)u[n] * (double)s_x[t] * (double)s_u[le * f + n];
              const float h = (float)((gv / (1.0 + exp(-gv))) * uv);
              g[n] = (acc_t)value[moe_oracle_fp8_encode(h / s_h[le])]; /* h as the code GEMM-2 reads */
            }
            for (int m = 0; m < d; ++m) o[m] = 0;
            for (int n = 0; n < f; ++n) {
              const acc_t hn = g[n];
              const size_t rowb = wdn + (size_t)n * d;
              for (int m = 0; m < d; ++m) o[m] += hn * (acc_t)value[Wd[rowb + m]];
            }
            const double w = (double)topk_w[(size_t)t * k + j];
            for (int m = 0; m < d; ++m)
              acc[m] += (acc_t)(w * ((double)o[m] * (double)s_h[le] * (double)s_d[le * d + m]));
          }
        }
        for (int m = 0; m < d; ++m) y_out[(size_t)i * d + m] = (double)acc[m];
      }
    }
    free(g); free(u); free(o); free(acc);
  }
  return status;
}

/* ------------------------------------------------------------------------------------------------------------
 * Backward pass of the layer (the paper's end-to-end results cover forward and backward, Sec. V; it gives no
 * formulas, these are the derivatives of the forward above).  For a local row (token t, slot j, local expert le,
 * gate weight w) and the incoming gradient dy_t of y_t:
 *   dh_raw = dy_t Wd^T,  dw = <h, dh_raw>  (= <o, dy_t>),  dh = w * dh_raw,
 *   dg = dh * u * silu'(g),  du = dh * silu(g),   silu'(g) = s (1 + g (1 - s)),  s = 1 / (1 + exp(-g)),
 *   dx_t += dg Wg^T + du Wu^T,
 *   dWg += x_t^T dg,  dWu += x_t^T du,  dWd += h^T (w dy_t).
 * Only the local slots contribute (one GPU's share, like the forward).  Everything in double, sums in ascending
 * index order, rows of an expert in ascending token order.
 * ------------------------------------------------------------------------------------------------------------ */

/* g, u (full length f) of token t under local expert le */
static void oracle_gate_up(const void *x, int elt, int t, int d, int f, const void *W_gate, const void *W_up, size_t le,
                           int n0, int n1, double *g, double *u) {
  for (int n = n0; n < n1; ++n) { g[n] = 0; u[n] = 0; }
  for (int c = 0; c < d; ++c) {
    const double xc = (double)load_elt(x, (size_t)t * d + c, elt);
    const size_t rowb = le * (size_t)d * f + (size_t)c * f;
    for (int n = n0; n < n1; ++n) {
      g[n] += xc * (double)load_elt(W_gate, rowb + n, elt);
      u[n] += xc * (double)load_elt(W_up, rowb + n, elt);
    }
  }
}

/*
 * Gradients that belong to tokens: dx rows [n_tok, d] and d_topk_w rows [n_tok, k] (0 for slots whose expert is
 * not local) for the listed tokens (tokens == NULL: 0..n_tok-1).
 */
int moe_oracle_backward_tokens(int T, int d, int f, int E, int k, int R, int lrb, int lre, int elt, const void *x,
                               const void *dy, const int32_t *topk_idx, const float *topk_w, const void *W_gate,
                               const void *W_up, const void *W_down, const int32_t *tokens, int n_tok,
                               double *dx_out, double *dw_out) {
  if (T < 0 || d < 1 || f < 1 || E < 1 || k < 1 || R < 1 || E % R != 0) return ORACLE_BAD_ARG;
  if (lrb < 0 || lre <= lrb || lre > R || (elt != ELT_F32 && elt != ELT_BF16) || n_tok < 0) return ORACLE_BAD_ARG;
  if (!x || !dy || !topk_idx || !topk_w || !W_gate || !W_up || !W_down || !dx_out || !dw_out) return ORACLE_BAD_ARG;
  const int epr = E / R;
  const int e_lo = lrb * epr, e_hi = lre * epr;
  int status = ORACLE_OK;
#pragma omp parallel
  {
    double *g = (double *)malloc(sizeof(double) * (size_t)f);
    double *u = (double *)malloc(sizeof(double) * (size_t)f);
    double *dg = (double *)malloc(sizeof(double) * (size_t)f);
    double *du = (double *)malloc(sizeof(double) * (size_t)f);
    if (!g || !u || !dg || !du) {
#pragma omp critical
      status = ORACLE_NOMEM;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int i = 0; i < n_tok; ++i) {
        const int t = tokens ? tokens[i] : i;
        double *dx = dx_out + (size_t)i * d;
        for (int c = 0; c < d; ++c) dx[c] = 0;
        for (int j = 0; j < k; ++j) dw_out[(size_t)i * k + j] = 0;
        if (t < 0 || t >= T) continue;
        for (int j = 0; j < k; ++j) {
          const int e = topk_idx[(size_t)t * k + j];
          if (e < e_lo || e >= e_hi) continue;
          const size_t le = (size_t)(e - e_lo);
          const double w = (double)topk_w[(size_t)t * k + j];
          oracle_gate_up(x, elt, t, d, f, W_gate, W_up, le, 0, f, g, u);
          double dwsum = 0;
          for (int n = 0; n < f; ++n) {
            double dh_raw = 0;
            const size_t rowb = le * (size_t)f * d + (size_t)n * d;
            for (int m = 0; m < d; ++m)
              dh_raw += (double)load_elt(dy, (size_t)t * d + m, elt) * (double)load_elt(W_down, rowb + m, elt);
            const double s = 1.0 / (1.0 + exp(-g[n]));
            dwsum += (g[n] * s * u[n]) * dh_raw;
            const double dh = w * dh_raw;
            dg[n] = dh * u[n] * (s * (1.0 + g[n] * (1.0 - s)));
            du[n] = dh * (g[n] * s);
          }
          dw_out[(size_t)i * k + j] = dwsum;
          for (int c = 0; c < d; ++c) {
            const size_t rowb = le * (size_t)d * f + (size_t)c * f;
            double acc = 0;
            for (int n = 0; n < f; ++n)
              acc += dg[n] * (double)load_elt(W_gate, rowb + n, elt) + du[n] * (double)load_elt(W_up, rowb + n, elt);
            dx[c] += acc;
          }
        }
      }
    }
    free(g); free(u); free(dg); free(du);
  }
  return status;
}

/*
 * Weight gradients of local expert le for the hidden indices n in [n0, n1):  dWg[:, n0:n1] and dWu[:, n0:n1]
 * ([d, n1-n0] each, row-major) and dWd[n0:n1, :] ([n1-n0, d]).  All tokens, ascending.
 */
int moe_oracle_backward_weights(int T, int d, int f, int E, int k, int R, int lrb, int lre, int elt, const void *x,
                                const void *dy, const int32_t *topk_idx, const float *topk_w, const void *W_gate,
                                const void *W_up, const void *W_down, int le, int n0, int n1, double *dWg,
                                double *dWu, double *dWd) {
  if (T < 0 || d < 1 || f < 1 || E < 1 || k < 1 || R < 1 || E % R != 0) return ORACLE_BAD_ARG;
  if (lrb < 0 || lre <= lrb || lre > R || (elt != ELT_F32 && elt != ELT_BF16)) return ORACLE_BAD_ARG;
  if (!x || !dy || !topk_idx || !topk_w || !W_gate || !W_up || !W_down || !dWg || !dWu || !dWd) return ORACLE_BAD_ARG;
  const int epr = E / R;
  if (le < 0 || le >= (lre - lrb) * epr || n0 < 0 || n1 > f || n0 >= n1) return ORACLE_BAD_ARG;
  const int e = lrb * epr + le, nn = n1 - n0;
  double *g = (double *)malloc(sizeof(double) * (size_t)f);
  double *u = (double *)malloc(sizeof(double) * (size_t)f);
  if (!g || !u) { free(g); free(u); return ORACLE_NOMEM; }
  for (size_t i = 0; i < (size_t)d * nn; ++i) { dWg[i] = 0; dWu[i] = 0; dWd[i] = 0; }
  for (int t = 0; t < T; ++t) {
    for (int j = 0; j < k; ++j) {
      if (topk_idx[(size_t)t * k + j] != e) continue;
      const double w = (double)topk_w[(size_t)t * k + j];
      oracle_gate_up(x, elt, t, d, f, W_gate, W_up, (size_t)le, n0, n1, g, u);
      for (int n = n0; n < n1; ++n) {
        double dh_raw = 0;
        const size_t rowb = (size_t)le * f * d + (size_t)n * d;
        for (int m = 0; m < d; ++m)
          dh_raw += (double)load_elt(dy, (size_t)t * d + m, elt) * (double)load_elt(W_down, rowb + m, elt);
        const double s = 1.0 / (1.0 + exp(-g[n]));
        const double h = g[n] * s * u[n];
        const double dh = w * dh_raw;
        const double dgn = dh * u[n] * (s * (1.0 + g[n] * (1.0 - s)));
        const double dun = dh * (g[n] * s);
        for (int c = 0; c < d; ++c) {
          const double xc = (double)load_elt(x, (size_t)t * d + c, elt);
          dWg[(size_t)c * nn + (n - n0)] += xc * dgn;
          dWu[(size_t)c * nn + (n - n0)] += xc * dun;
        }
        for (int m = 0; m < d; ++m)
          dWd[(size_t)(n - n0) * d + m] += h * (w * (double)load_elt(dy, (size_t)t * d + m, elt));
      }
    }
  }
  free(g); free(u);
  return ORACLE_OK;
}

/*
 * Backward of the routing weights of moe_oracle_route_topk (softmax over the logits, renormalised over the picks,
 * i.e. a softmax over the k picked logits): with w_j the weights and dw_j the incoming gradients of token t,
 *   dlogit[e_j] = w_j * (dw_j - sum_i w_i dw_i),   0 for the experts that were not picked
 * (the selection itself is piecewise constant).  dlogits is [T, E] in double; the weights are recomputed from the
 * logits in double.
 */
int moe_oracle_route_backward(int T, int E, int k, const float *logits, const int32_t *topk_idx, const double *dw,
                              double *dlogits) {
  if (T < 0 || E < 1 || k < 1 || k > E || !logits || !topk_idx || !dw || !dlogits) return ORACLE_BAD_ARG;
  for (int t = 0; t < T; ++t) {
    const float *row = logits + (size_t)t * E;
    for (int e = 0; e < E; ++e) dlogits[(size_t)t * E + e] = 0.0;
    double m = -INFINITY, sum = 0.0, dot = 0.0;
    for (int j = 0; j < k; ++j) {
      const int e = topk_idx[(size_t)t * k + j];
      if (e < 0 || e >= E) return ORACLE_BAD_ARG;
      if ((double)row[e] > m) m = (double)row[e];
    }
    for (int j = 0; j < k; ++j) sum += exp((double)row[topk_idx[(size_t)t * k + j]] - m);
    for (int j = 0; j < k; ++j)
      dot += exp((double)row[topk_idx[(size_t)t * k + j]] - m) / sum * dw[(size_t)t * k + j];
    for (int j = 0; j < k; ++j) {
      const int e = topk_idx[(size_t)t * k + j];
      const double w = exp((double)row[e] - m) / sum;
      dlogits[(size_t)t * E + e] = w * (dw[(size_t)t * k + j] - dot);
    }
  }
  return ORACLE_OK;
}
