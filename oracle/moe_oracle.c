/*
 * moe_oracle.c -- plain CPU definition of the sparse-MoE FFN layer forward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * compared with; it is loaded by the tests, by the smoke check and by the
 * benchmark's CPU-baseline leg, and by nothing else.  It shares no code with
 * the GPU path and must never be called from it.
 *
 * What it computes.  The paper (MoESD, arXiv 2505.19645) describes the layer
 * only in words (Introduction: several expert networks plus a router that
 * activates K of them per token; Sec. 3.2: K per token out of E) and models
 * its cost through the number of activated experts N (Eq. N(t)).  The layer's
 * arithmetic is the standard SwiGLU mixture, fixed by the benchmark configs:
 *
 *   logit[t,e] = sum_j X[t,j] * Wr[e,j]  (+ bias[e])
 *   key[t,e]   = fp32(logit[t,e])                       (one rounding)
 *   ids[t,:]   = the K experts with the largest key, equal keys -> lower index,
 *                listed in that order
 *                (group-limited variant, n_group > 1: the E experts form n_group
 *                equal consecutive groups; a group's score is the sum of the scores
 *                of its two members with the largest key, rounded once to fp32; the
 *                topk_group groups with the largest group score, equal -> lower
 *                index, stay; ids are taken among their members only.  This is the
 *                routing rule published for the model family of benchmark config 4,
 *                without its selection bias.)
 *   score      = softmax over all E of logit, or sigmoid(logit)
 *   w[t,s]     = score[ids[t,s]] / sum_s' score[ids[t,s']]   (if renormalize)
 *                times routed_scale
 *   permutation= stable counting sort of the flat slots f = t*K+s by expert
 *   y[p,:]     = Wd_e . ( silu(Wg_e . x) * (Wu_e . x) ),  x = X[perm[p]/K],
 *                e = expert owning sorted row p
 *   out[t,:]   = sum_s w[t,s] * y[inv[t*K+s],:]  +  g_t * shared(x_t)
 *   g_t        = sigmoid(x_t . w_sg) or 1
 *
 * Low-precision expert weights (outside the paper, whose Appendix C.2 only notes that the
 * floor of the expert-loading term scales with the weights' bit width): the expert matrices
 * may be given as 8-bit floating-point codes, format E4M3 of the OCP OFP8 specification
 * (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinities,
 * S.1111.111 = NaN), with one fp32 scale per output row; the weight is then
 * decode(code) * scale[row] as a real number, and everything else is unchanged.
 *
 * Everything is evaluated in fp64 from the bf16-valued inputs, sums run over
 * the contraction index in ascending order, and nothing is rounded in between
 * except the selection key.  Loops are parallelised with OpenMP over
 * independent outputs only; no sum is split or reordered.
 *
 * Pins (tests/test_oracle_*.py): brute-force subset routing on tiny inputs,
 * sum_s w = 1, numpy stable argsort for the permutation, reductions to plain
 * matrix products (E=1,K=1; K=E; identical experts; expert relabelling), the
 * closed form N(t) against Monte-Carlo and against exact enumeration; the
 * group-limited rule against a sort-based restatement, a hand-made case and
 * its two degenerate settings (one group; all groups kept); the E4M3 decoder
 * against a table of all 256 code points written with rational arithmetic and
 * against a library cast, the fp8 layer against the bf16 layer on weights
 * that both formats hold exactly (tests/test_oracle_fp8.py).
 * Absolute output values have no worked example in the paper: they are pinned
 * only through those reductions ("parity unpinned" by the paper itself).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t d, E, top_k, inter, shared_inter;
  int32_t score_func;  /* 0 softmax, 1 sigmoid */
  int32_t renormalize;
  int32_t shared_gate;
  double  routed_scale;
  int32_t n_group;     /* 0 or 1: no groups */
  int32_t topk_group;  /* groups kept per token */
} oracle_desc;

/* bf16 word -> double (exact) */
static double bf16_to_f64(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* double -> bf16 word, round to nearest even in ONE step (no detour via fp32,
 * which could round twice).  Finite inputs of ordinary magnitude only. */
static uint16_t f64_to_bf16(double v) {
  if (v == 0.0 || !isfinite(v)) {
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
  }
  int ex;
  double m = frexp(v, &ex);         /* v = m * 2^ex, 0.5 <= |m| < 1 */
  double r = nearbyint(ldexp(m, 8)); /* 8 significant bits, ties to even */
  float f = (float)ldexp(r, ex - 8); /* exactly representable */
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

/* E4M3 code -> double, from the format's definition (OCP OFP8 specification, Sec. 5):
 * s eeee mmm; exponent field 0: subnormal, m/8 * 2^-6; otherwise (1 + m/8) * 2^(e - 7);
 * no infinities; exponent 15 with mantissa 7 is NaN (so the largest finite value is 448). */
static double fp8_e4m3_to_f64(uint8_t c) {
  const int s = c >> 7, e = (c >> 3) & 15, m = c & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m / 8.0, -6);
  else v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return s ? -v : v;
}

void oracle_fp8_e4m3_decode(const uint8_t *codes, int64_t n, double *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = fp8_e4m3_to_f64(codes[i]);
}

/* x . (decode(code) * scale): the weight row as real numbers, then the same ascending sum */
static double dot_bf16_fp8(const uint16_t *a, const uint8_t *codes, double scale, int64_t n) {
  double s = 0.0;
  for (int64_t j = 0; j < n; ++j) s += bf16_to_f64(a[j]) * (fp8_e4m3_to_f64(codes[j]) * scale);
  return s;
}

static double dot_bf16(const uint16_t *a, const uint16_t *b, int64_t n) {
  double s = 0.0;
  for (int64_t j = 0; j < n; ++j) s += bf16_to_f64(a[j]) * bf16_to_f64(b[j]);
  return s;
}

static double sigmoid64(double z) { return 1.0 / (1.0 + exp(-z)); }
static double silu64(double z) { return z / (1.0 + exp(-z)); }

/* ---- closed forms of Sec. 3.2 ------------------------------------------- */

/* Eq. N(t) */
double oracle_expected_active_experts(int32_t E, int32_t K, int64_t t) {
  if (E < 1 || K < 0 || K > E || t < 0) return NAN;
  return (double)E * (1.0 - pow((double)(E - K) / (double)E, (double)t));
}

/* N(t) without the uniformity assumption.  The step before Eq. N(t) (an expert is
 * activated unless none of the t tokens activates it) holds for every expert on its
 * own: with p[e] the probability that one token activates expert e (sum_e p[e] = K)
 * and independent tokens, N(t) = sum_e (1 - (1 - p[e])^t).  p[e] = K/E gives Eq. N(t). */
double oracle_expected_active_experts_p(const double *p, int32_t E, int64_t t) {
  if (E < 1 || t < 0 || !p) return NAN;
  double n = 0.0;
  for (int e = 0; e < E; ++e) {
    if (!(p[e] >= 0.0) || !(p[e] <= 1.0)) return NAN;
    n += 1.0 - pow(1.0 - p[e], (double)t);
  }
  return n;
}

/* Eq. Texp */
double oracle_expected_tokens_per_expert(int32_t E, int32_t K, int64_t t) {
  if (E < 1 || K < 0 || K > E || t < 0) return NAN;
  if (t == 0 || K == 0) return 0.0;
  return (double)t * (double)K / oracle_expected_active_experts(E, K, t);
}

/* Eq. T_thres: smallest t with N(t) >= tau*E, found by stepping t (no log) */
int64_t oracle_token_threshold(int32_t E, int32_t K, double tau) {
  if (E < 1 || K < 1 || K > E || !(tau >= 0.0) || !(tau < 1.0)) return -1;
  double miss = 1.0; /* (1-rho)^t */
  double q = (double)(E - K) / (double)E;
  for (int64_t t = 0; t < (int64_t)1 << 40; ++t) {
    if (1.0 - miss >= tau) return t < 1 ? 1 : t;
    miss *= q;
  }
  return -1;
}

/* ---- routing -------------------------------------------------------------- */

/* logits [T,E] f64 (may be NULL), ids [T,K], w [T,K] f64 */
int32_t oracle_route(const oracle_desc *c, const uint16_t *x, const uint16_t *wr,
                     const float *bias, int32_t T, double *logits_out, int32_t *ids,
                     double *w) {
  const int E = c->E, K = c->top_k, d = c->d;
  if (E < 1 || K < 1 || K > E || T < 0 || c->n_group > 1024) return 1;
  const int G = c->n_group > 1 ? c->n_group : 1;
  const int Gk = G > 1 ? c->topk_group : 1;
  if (E % G != 0 || Gk < 1 || Gk > G || K > Gk * (E / G)) return 1;
  const int gs = E / G;
#pragma omp parallel
  {
    double *l = (double *)malloc(sizeof(double) * E);
    double *p = (double *)malloc(sizeof(double) * E);
    float *key = (float *)malloc(sizeof(float) * E);
    char *taken = (char *)malloc(E);
#pragma omp for schedule(static)
    for (int t = 0; t < T; ++t) {
      for (int e = 0; e < E; ++e) {
        l[e] = dot_bf16(x + (int64_t)t * d, wr + (int64_t)e * d, d);
        if (bias) l[e] += (double)bias[e];
        key[e] = (float)l[e];
        if (logits_out) logits_out[(int64_t)t * E + e] = l[e];
      }
      /* scores from the fp64 logits */
      if (c->score_func == 0) {
        double mx = l[0];
        for (int e = 1; e < E; ++e) if (l[e] > mx) mx = l[e];
        double z = 0.0;
        for (int e = 0; e < E; ++e) { p[e] = exp(l[e] - mx); z += p[e]; }
        for (int e = 0; e < E; ++e) p[e] /= z;
      } else {
        for (int e = 0; e < E; ++e) p[e] = sigmoid64(l[e]);
      }
      /* K rounds of "largest remaining key, first index on equality" */
      memset(taken, 0, E);
      if (G > 1) {
        /* group-limited selection: everything outside the kept groups is "taken" */
        float gkey[1024];
        char gkeep[1024];
        for (int g = 0; g < G; ++g) {
          int a = -1, b = -1; /* the two largest keys of the group, first index on equality */
          for (int e = g * gs; e < (g + 1) * gs; ++e) {
            if (a < 0 || key[e] > key[a]) { b = a; a = e; }
            else if (b < 0 || key[e] > key[b]) b = e;
          }
          gkey[g] = (float)(p[a] + (b >= 0 ? p[b] : 0.0));
          gkeep[g] = 0;
        }
        for (int s = 0; s < Gk; ++s) {
          int best = -1;
          for (int g = 0; g < G; ++g) {
            if (gkeep[g]) continue;
            if (best < 0 || gkey[g] > gkey[best]) best = g;
          }
          gkeep[best] = 1;
        }
        for (int e = 0; e < E; ++e) taken[e] = !gkeep[e / gs];
      }
      for (int s = 0; s < K; ++s) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
          if (taken[e]) continue;
          if (best < 0 || key[e] > key[best]) best = e;
        }
        taken[best] = 1;
        ids[(int64_t)t * K + s] = best;
      }
      double den = 1.0;
      if (c->renormalize) {
        den = 0.0;
        for (int s = 0; s < K; ++s) den += p[ids[(int64_t)t * K + s]];
      }
      for (int s = 0; s < K; ++s)
        w[(int64_t)t * K + s] = p[ids[(int64_t)t * K + s]] / den * c->routed_scale;
    }
    free(l); free(p); free(key); free(taken);
  }
  return 0;
}

/* ---- permutation ---------------------------------------------------------- */

int32_t oracle_permute(int32_t E, int32_t K, int32_t T, const int32_t *ids, int32_t *counts,
                       int32_t *offsets, int32_t *perm, int32_t *inv, int32_t *n_active) {
  if (E < 1 || K < 1 || T < 0) return 1;
  const int64_t n = (int64_t)T * K;
  for (int e = 0; e < E; ++e) counts[e] = 0;
  for (int64_t f = 0; f < n; ++f) {
    if (ids[f] < 0 || ids[f] >= E) return 1;
    counts[ids[f]]++;
  }
  offsets[0] = 0;
  for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
  int32_t *rank = (int32_t *)calloc(E, sizeof(int32_t));
  for (int64_t f = 0; f < n; ++f) {
    int e = ids[f];
    int32_t p = offsets[e] + rank[e]++;
    perm[p] = (int32_t)f;
    inv[f] = p;
  }
  free(rank);
  int na = 0;
  for (int e = 0; e < E; ++e) na += counts[e] > 0;
  *n_active = na;
  return 0;
}

/* ---- one SwiGLU FFN on one token: y[0..d) ---------------------------------- */
static void ffn_row(const uint16_t *xrow, const uint16_t *wg, const uint16_t *wu,
                    const uint16_t *wd, int d, int I, double *h, double *y) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < I; ++i) {
    double g = dot_bf16(xrow, wg + (int64_t)i * d, d);
    double u = dot_bf16(xrow, wu + (int64_t)i * d, d);
    h[i] = silu64(g) * u;
  }
#pragma omp parallel for schedule(static)
  for (int cidx = 0; cidx < d; ++cidx) {
    const uint16_t *row = wd + (int64_t)cidx * I;
    double s = 0.0;
    for (int i = 0; i < I; ++i) s += h[i] * bf16_to_f64(row[i]);
    y[cidx] = s;
  }
}

/* The same FFN with E4M3 weight codes and one scale per output row (sg, su: [I]; sd: [d]). */
static void ffn_row_fp8(const uint16_t *xrow, const uint8_t *wg, const float *sg, const uint8_t *wu,
                        const float *su, const uint8_t *wd, const float *sd, int d, int I, double *h,
                        double *y) {
#pragma omp parallel for schedule(static)
  for (int i = 0; i < I; ++i) {
    double g = dot_bf16_fp8(xrow, wg + (int64_t)i * d, (double)sg[i], d);
    double u = dot_bf16_fp8(xrow, wu + (int64_t)i * d, (double)su[i], d);
    h[i] = silu64(g) * u;
  }
#pragma omp parallel for schedule(static)
  for (int cidx = 0; cidx < d; ++cidx) {
    const uint8_t *row = wd + (int64_t)cidx * I;
    const double sc = (double)sd[cidx];
    double s = 0.0;
    for (int i = 0; i < I; ++i) s += h[i] * (fp8_e4m3_to_f64(row[i]) * sc);
    y[cidx] = s;
  }
}

/* Expert weights of one layer in either format.  bf16: wg/wu/wd (and the shared sg/su/sd) are
 * uint16 words and the scale pointers are NULL; fp8: they are E4M3 codes and every matrix has
 * one fp32 scale per output row ([E, I], [E, I], [E, d]; shared [S], [S], [d]). */
typedef struct {
  int fp8;
  const void *wg, *wu, *wd, *sg, *su, *sd;
  const float *wg_s, *wu_s, *wd_s, *sg_s, *su_s, *sd_s;
} expert_weights;

static void ffn_row_any(const expert_weights *w, int shared, int e, const uint16_t *xrow, int d, int I,
                        double *h, double *y) {
  const int64_t gu = shared ? 0 : (int64_t)e * I * d, dn = shared ? 0 : (int64_t)e * d * I;
  if (!w->fp8) {
    const uint16_t *g = (const uint16_t *)(shared ? w->sg : w->wg) + gu;
    const uint16_t *u = (const uint16_t *)(shared ? w->su : w->wu) + gu;
    const uint16_t *dd = (const uint16_t *)(shared ? w->sd : w->wd) + dn;
    ffn_row(xrow, g, u, dd, d, I, h, y);
  } else {
    const uint8_t *g = (const uint8_t *)(shared ? w->sg : w->wg) + gu;
    const uint8_t *u = (const uint8_t *)(shared ? w->su : w->wu) + gu;
    const uint8_t *dd = (const uint8_t *)(shared ? w->sd : w->wd) + dn;
    const float *gs = shared ? w->sg_s : w->wg_s + (int64_t)e * I;
    const float *us = shared ? w->su_s : w->wu_s + (int64_t)e * I;
    const float *ds = shared ? w->sd_s : w->wd_s + (int64_t)e * d;
    ffn_row_fp8(xrow, g, gs, u, us, dd, ds, d, I, h, y);
  }
}

/*
 * Whole layer.  tok_list/n_list select the tokens whose output is wanted
 * (NULL / 0 = all T, in order); routing and the permutation always cover all T.
 * out_f64 / out_bf16: [n_out, d].  Optional outputs (NULL to skip): ids [T,K],
 * w [T,K], counts [E], offsets [E+1], perm [T*K], inv [T*K], n_active [1],
 * gate [T] (shared-expert gate of every token).
 */
static int32_t forward_impl(const oracle_desc *c, const uint16_t *x, const uint16_t *wr,
                            const float *bias, const expert_weights *ew, const uint16_t *wsg, int32_t T,
                            const int32_t *tok_list, int32_t n_list, double *out_f64,
                            uint16_t *out_bf16, int32_t *ids_o, double *w_o, int32_t *counts_o,
                            int32_t *offsets_o, int32_t *perm_o, int32_t *inv_o,
                            int32_t *n_active_o, double *gate_o) {
  const int E = c->E, K = c->top_k, d = c->d, I = c->inter, S = c->shared_inter;
  if (T < 0) return 1;
  const int64_t n = (int64_t)T * K;
  int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (n ? n : 1));
  double *w = (double *)malloc(sizeof(double) * (n ? n : 1));
  int32_t *counts = (int32_t *)malloc(sizeof(int32_t) * E);
  int32_t *offsets = (int32_t *)malloc(sizeof(int32_t) * (E + 1));
  int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (n ? n : 1));
  int32_t *inv = (int32_t *)malloc(sizeof(int32_t) * (n ? n : 1));
  int32_t n_active = 0;
  int32_t rc = oracle_route(c, x, wr, bias, T, NULL, ids, w);
  if (!rc) rc = oracle_permute(E, K, T, ids, counts, offsets, perm, inv, &n_active);
  if (rc) goto done;

  {
    const int n_out = tok_list ? n_list : T;
    const int Imax = I > S ? I : S;
    double *h = (double *)malloc(sizeof(double) * (Imax ? Imax : 1));
    double *y = (double *)malloc(sizeof(double) * d * K);
    double *sh = (double *)malloc(sizeof(double) * d);
    for (int o = 0; o < n_out; ++o) {
      const int t = tok_list ? tok_list[o] : o;
      /* routed experts: the K sorted rows that belong to token t */
      for (int s = 0; s < K; ++s) {
        const int32_t p = inv[(int64_t)t * K + s];
        int e = 0;
        while (!(offsets[e] <= p && p < offsets[e + 1])) ++e; /* owner of row p */
        const int tok = perm[p] / K;                          /* == t */
        ffn_row_any(ew, 0, e, x + (int64_t)tok * d, d, I, h, y + (int64_t)s * d);
      }
      double g = 1.0;
      if (S > 0) {
        ffn_row_any(ew, 1, 0, x + (int64_t)t * d, d, S, h, sh);
        if (c->shared_gate) g = sigmoid64(dot_bf16(x + (int64_t)t * d, wsg, d));
      }
      if (gate_o) gate_o[t] = g;
      for (int cidx = 0; cidx < d; ++cidx) {
        double acc = 0.0;
        for (int s = 0; s < K; ++s) acc += w[(int64_t)t * K + s] * y[(int64_t)s * d + cidx];
        if (S > 0) acc += g * sh[cidx];
        if (out_f64) out_f64[(int64_t)o * d + cidx] = acc;
        if (out_bf16) out_bf16[(int64_t)o * d + cidx] = f64_to_bf16(acc);
      }
    }
    free(h); free(y); free(sh);
  }
  if (ids_o) memcpy(ids_o, ids, sizeof(int32_t) * n);
  if (w_o) memcpy(w_o, w, sizeof(double) * n);
  if (counts_o) memcpy(counts_o, counts, sizeof(int32_t) * E);
  if (offsets_o) memcpy(offsets_o, offsets, sizeof(int32_t) * (E + 1));
  if (perm_o) memcpy(perm_o, perm, sizeof(int32_t) * n);
  if (inv_o) memcpy(inv_o, inv, sizeof(int32_t) * n);
  if (n_active_o) *n_active_o = n_active;
done:
  free(ids); free(w); free(counts); free(offsets); free(perm); free(inv);
  return rc;
}

int32_t oracle_moe_forward(const oracle_desc *c, const uint16_t *x, const uint16_t *wr,
                           const float *bias, const uint16_t *wg, const uint16_t *wu,
                           const uint16_t *wd, const uint16_t *sg, const uint16_t *su,
                           const uint16_t *sd, const uint16_t *wsg, int32_t T,
                           const int32_t *tok_list, int32_t n_list, double *out_f64,
                           uint16_t *out_bf16, int32_t *ids_o, double *w_o, int32_t *counts_o,
                           int32_t *offsets_o, int32_t *perm_o, int32_t *inv_o,
                           int32_t *n_active_o, double *gate_o) {
  expert_weights ew = {0, wg, wu, wd, sg, su, sd, NULL, NULL, NULL, NULL, NULL, NULL};
  return forward_impl(c, x, wr, bias, &ew, wsg, T, tok_list, n_list, out_f64, out_bf16, ids_o, w_o,
                      counts_o, offsets_o, perm_o, inv_o, n_active_o, gate_o);
}

/* The layer with E4M3 expert weights: codes [E,I,d], [E,I,d], [E,d,I] (shared [S,d], [S,d], [d,S]) and
 * scales [E,I], [E,I], [E,d] (shared [S], [S], [d]); router and shared gate stay bf16. */
int32_t oracle_moe_forward_fp8(const oracle_desc *c, const uint16_t *x, const uint16_t *wr,
                               const float *bias, const uint8_t *wg, const float *wg_s,
                               const uint8_t *wu, const float *wu_s, const uint8_t *wd,
                               const float *wd_s, const uint8_t *sg, const float *sg_s,
                               const uint8_t *su, const float *su_s, const uint8_t *sd,
                               const float *sd_s, const uint16_t *wsg, int32_t T,
                               const int32_t *tok_list, int32_t n_list, double *out_f64,
                               uint16_t *out_bf16, int32_t *ids_o, double *w_o, int32_t *counts_o,
                               int32_t *offsets_o, int32_t *perm_o, int32_t *inv_o,
                               int32_t *n_active_o, double *gate_o) {
  expert_weights ew = {1, wg, wu, wd, sg, su, sd, wg_s, wu_s, wd_s, sg_s, su_s, sd_s};
  return forward_impl(c, x, wr, bias, &ew, wsg, T, tok_list, n_list, out_f64, out_bf16, ids_o, w_o,
                      counts_o, offsets_o, perm_o, inv_o, n_active_o, gate_o);
}

/* The same forward with every sum carried in fp32 instead of fp64: used only
 * by a cross-precision test that guards the fp64 code against a typo. */
static float dot_bf16_f32(const uint16_t *a, const uint16_t *b, int64_t n) {
  float s = 0.0f;
  for (int64_t j = 0; j < n; ++j) s += (float)bf16_to_f64(a[j]) * (float)bf16_to_f64(b[j]);
  return s;
}

int32_t oracle_ffn_row_f32(const uint16_t *xrow, const uint16_t *wg, const uint16_t *wu,
                           const uint16_t *wd, int32_t d, int32_t I, float *y) {
  float *h = (float *)malloc(sizeof(float) * I);
  for (int i = 0; i < I; ++i) {
    float g = dot_bf16_f32(xrow, wg + (int64_t)i * d, d);
    float u = dot_bf16_f32(xrow, wu + (int64_t)i * d, d);
    h[i] = g / (1.0f + expf(-g)) * u;
  }
  for (int cidx = 0; cidx < d; ++cidx) {
    float s = 0.0f;
    for (int i = 0; i < I; ++i) s += h[i] * (float)bf16_to_f64(wd[(int64_t)cidx * I + i]);
    y[cidx] = s;
  }
  free(h);
  return 0;
}

int32_t oracle_ffn_row_f64(const uint16_t *xrow, const uint16_t *wg, const uint16_t *wu,
                           const uint16_t *wd, int32_t d, int32_t I, double *y) {
  double *h = (double *)malloc(sizeof(double) * I);
  ffn_row(xrow, wg, wu, wd, d, I, h, y);
  free(h);
  return 0;
}

/* bf16 rounding of a double array, exposed for the rounding-floor check */
void oracle_round_bf16(const double *v, int64_t n, uint16_t *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = f64_to_bf16(v[i]);
}
