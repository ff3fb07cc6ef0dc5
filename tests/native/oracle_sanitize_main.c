/* Driver for the sanitizer build of the oracle (tests/test_sanitizers.py): small layers of every kind
 * (softmax / sigmoid, groups, shared expert with and without gate, bf16 and E4M3 weights, token lists,
 * T = 0) through every entry point, under -fsanitize=address,undefined.  Values are pseudo-random;
 * only memory safety and defined behaviour are checked here, the arithmetic has its own pins. */
#include <stdio.h>
#include "../../oracle/moe_oracle.c"

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
static uint16_t rnd_bf16(void) { return (uint16_t)(0x3C00u + (rnd() & 0x3FFu) + ((rnd() & 1u) << 15)); } /* ~ +-0.01..0.1 */
static uint8_t rnd_fp8(void) { uint8_t c = (uint8_t)rnd(); return (c & 0x7F) == 0x7F ? 0x30 : c; }

static int run(int d, int E, int K, int I, int S, int score, int gate, int groups, int topg, int T, int fp8) {
  oracle_desc c = {d, E, K, I, S, score, 1, gate, 1.0, groups, topg};
  size_t nx = (size_t)(T ? T : 1) * d;
  uint16_t *x = malloc(2 * nx), *wr = malloc(2 * (size_t)E * d), *wsg = malloc(2 * (size_t)d);
  size_t ng = (size_t)E * I * d, ns = (size_t)(S ? S : 1) * d;
  void *wg = malloc(2 * ng), *wu = malloc(2 * ng), *wd = malloc(2 * ng), *sg = malloc(2 * ns), *su = malloc(2 * ns),
       *sd = malloc(2 * ns);
  float *sc = malloc(4 * ((size_t)E * (I > d ? I : d) + S + d));
  for (size_t i = 0; i < nx; ++i) x[i] = rnd_bf16();
  for (size_t i = 0; i < (size_t)E * d; ++i) wr[i] = rnd_bf16();
  for (int i = 0; i < d; ++i) wsg[i] = rnd_bf16();
  for (size_t i = 0; i < ng; ++i) {
    if (fp8) { ((uint8_t *)wg)[i] = rnd_fp8(); ((uint8_t *)wu)[i] = rnd_fp8(); ((uint8_t *)wd)[i] = rnd_fp8(); }
    else { ((uint16_t *)wg)[i] = rnd_bf16(); ((uint16_t *)wu)[i] = rnd_bf16(); ((uint16_t *)wd)[i] = rnd_bf16(); }
  }
  for (size_t i = 0; i < ns; ++i) {
    if (fp8) { ((uint8_t *)sg)[i] = rnd_fp8(); ((uint8_t *)su)[i] = rnd_fp8(); ((uint8_t *)sd)[i] = rnd_fp8(); }
    else { ((uint16_t *)sg)[i] = rnd_bf16(); ((uint16_t *)su)[i] = rnd_bf16(); ((uint16_t *)sd)[i] = rnd_bf16(); }
  }
  for (size_t i = 0; i < (size_t)E * (I > d ? I : d) + S + d; ++i) sc[i] = 0.001f + (float)(rnd() & 255) * 1e-5f;
  size_t n = (size_t)(T ? T : 1) * K;
  const size_t no = (size_t)(T > 2 ? T : 2) * d;  /* the token-list pass asks for two rows */
  double *out = malloc(8 * no), *w = malloc(8 * n), *gt = malloc(8 * (size_t)(T ? T : 1));
  uint16_t *outb = malloc(2 * no);
  int32_t *ids = malloc(4 * n), *perm = malloc(4 * n), *inv = malloc(4 * n), *cnt = malloc(4 * (size_t)E),
          *off = malloc(4 * (size_t)(E + 1)), na = -1;
  int32_t toks[2] = {T > 1 ? T - 1 : 0, 0};
  int rc = 0;
  for (int pass = 0; pass < 2 && !rc; ++pass) { /* all tokens, then a token list */
    const int32_t *tl = pass ? toks : NULL;
    const int nl = pass ? (T > 0 ? 2 : 0) : 0;
    if (pass && T == 0) break;
    if (fp8)
      rc = oracle_moe_forward_fp8(&c, x, wr, NULL, wg, sc, wu, sc, wd, sc, S ? sg : NULL, sc, S ? su : NULL, sc,
                                  S ? sd : NULL, sc, gate ? wsg : NULL, T, tl, nl, out, outb, ids, w, cnt, off, perm,
                                  inv, &na, gt);
    else
      rc = oracle_moe_forward(&c, x, wr, NULL, wg, wu, wd, S ? sg : NULL, S ? su : NULL, S ? sd : NULL,
                              gate ? wsg : NULL, T, tl, nl, out, outb, ids, w, cnt, off, perm, inv, &na, gt);
  }
  if (!rc && T > 0) {
    double y[64];
    float y32[64];
    if (!fp8 && d <= 64) {
      oracle_ffn_row_f64(x, wg, wu, wd, d, I, y);
      oracle_ffn_row_f32(x, wg, wu, wd, d, I, y32);
    }
    oracle_round_bf16(out, (int64_t)d, outb);
  }
  free(x); free(wr); free(wsg); free(wg); free(wu); free(wd); free(sg); free(su); free(sd); free(sc);
  free(out); free(w); free(gt); free(outb); free(ids); free(perm); free(inv); free(cnt); free(off);
  return rc;
}

int main(void) {
  int bad = 0;
  bad += run(32, 6, 2, 24, 0, 0, 0, 0, 0, 9, 0);
  bad += run(48, 8, 3, 16, 40, 1, 1, 4, 2, 7, 0);
  bad += run(64, 5, 5, 8, 16, 0, 0, 0, 0, 1, 0);
  bad += run(32, 6, 2, 32, 16, 0, 1, 0, 0, 5, 1);
  bad += run(48, 4, 1, 16, 0, 1, 0, 2, 1, 3, 1);
  bad += run(32, 6, 2, 24, 8, 0, 1, 0, 0, 0, 0);   /* empty batch */
  {
    uint8_t codes[256];
    double v[256];
    for (int i = 0; i < 256; ++i) codes[i] = (uint8_t)i;
    oracle_fp8_e4m3_decode(codes, 256, v);
    double p[3] = {0.2, 0.3, 0.5};
    if (!(oracle_expected_active_experts(8, 2, 5) > 2.0) || oracle_token_threshold(8, 2, 0.95) != 11 ||
        !(oracle_expected_active_experts_p(p, 3, 2) > 0.0) || !(oracle_expected_tokens_per_expert(8, 2, 3) > 0.0) ||
        v[0x7e] != 448.0)
      ++bad;
    int32_t ids[4] = {1, 0, 1, 9}, cnt[2], off[3], pm[4], iv[4], na;
    if (oracle_permute(2, 2, 2, ids, cnt, off, pm, iv, &na) != 1) ++bad;  /* an id out of range is refused */
  }
  printf(bad ? "oracle_sanitize: %d FAILED\n" : "oracle_sanitize: ok\n", bad);
  return bad ? 1 : 0;
}
