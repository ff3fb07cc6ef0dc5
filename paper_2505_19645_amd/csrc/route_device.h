// Device code shared by the routing kernels: wave reductions and the per-token
// top-K (see route.hip for the method).
#pragma once
#include "common.h"

// 64-lane unsigned max, result in every lane.  Within each row of 16 lanes the
// exchange uses DPP lane permutes (xor 1, xor 2, mirror within 8, mirror within
// 16: max is idempotent, so mirrored partners work as a butterfly); the four row
// results are then read out as scalars.  This is the inner step of the K top-k
// rounds, and a shuffle-based reduction would put ~12 LDS-crossbar round trips
// on each round's critical path.
#define MOESD_DPP_MAX(v, CTRL)                                                              \
  {                                                                                         \
    const uint32_t lo_ = (uint32_t)(v), hi_ = (uint32_t)((v) >> 32);                        \
    const uint32_t olo_ = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo_, CTRL, 0xF, 0xF, false); \
    const uint32_t ohi_ = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)hi_, CTRL, 0xF, 0xF, false); \
    const unsigned long long o_ = ((unsigned long long)ohi_ << 32) | olo_;                   \
    (v) = o_ > (v) ? o_ : (v);                                                               \
  }
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
  MOESD_DPP_MAX(v, 0xB1)   // quad_perm [1,0,3,2]
  MOESD_DPP_MAX(v, 0x4E)   // quad_perm [2,3,0,1]
  MOESD_DPP_MAX(v, 0x141)  // row_half_mirror
  MOESD_DPP_MAX(v, 0x140)  // row_mirror
  unsigned long long best = 0ull;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, r * 16);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), r * 16);
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    best = o > best ? o : best;
  }
  return best;
}

// value of lane `src` (wave-uniform) in every lane
__device__ __forceinline__ double readlane_f64(double v, int src) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, src);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), src);
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ double wave_max_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off, 64));
  return v;
}

// Top-K of one token by one wave (all 64 lanes must call it together).
template <int SLOTS>  // experts per lane: E <= 64 * SLOTS
__device__ __forceinline__ void topk_token(const double *__restrict__ logits, int t, int lane, int E,
                                           int Etot, int K, int score_func, int renorm, float scale,
                                           int groups, int32_t *__restrict__ ids,
                                           float *__restrict__ w, float *__restrict__ gate) {
  const double *lrow = logits + (size_t)t * Etot;

  unsigned long long key[SLOTS];
  double lval[SLOTS];  // the fp64 logits of this lane's experts
#pragma unroll
  for (int j = 0; j < SLOTS; ++j) {
    const int e = lane + 64 * j;
    key[j] = 0ull;  // below every real key (real keys have a non-zero low word)
    lval[j] = 0.0;
    if (e < E) {
      lval[j] = lrow[e];
      const float kf = (float)lval[j] + 0.0f;  // the one rounding; +0 folds -0 into +0
      uint32_t u = __float_as_uint(kf);
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      key[j] = ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)e);
    }
  }

  // groups = n_group | topk_group << 16; n_group <= 1: unconstrained selection
  const int n_group = groups & 0xFFFF, topk_group = groups >> 16;

  // full-softmax normaliser, needed when the winners are not renormalised and for group scores
  double mx = 0.0, z = 1.0;
  if (score_func == MOESD_SCORE_SOFTMAX && (!renorm || n_group > 1)) {
    double m = -1.0e300;
#pragma nounroll
    for (int e = lane; e < E; e += 64) m = fmax(m, lrow[e]);
    mx = wave_max_f64(m);
    double sacc = 0.0;
#pragma nounroll
    for (int e = lane; e < E; e += 64) sacc += exp(lrow[e] - mx);
    z = wave_sum_f64(sacc);
  }

  // Group-limited selection: a group's score is the sum of the scores of its two members with
  // the largest keys, rounded once to fp32; the topk_group best groups (equal scores: the lower
  // index) keep their members, every other expert's key is cleared.  Lane g holds group g's score.
  if (n_group > 1) {
    const int gs = E / n_group;
    int grp[SLOTS];
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) grp[j] = (lane + 64 * j) / gs;
    unsigned long long gkey = 0ull;
#pragma nounroll
    for (int g = 0; g < n_group; ++g) {
      unsigned long long b1 = 0ull;
#pragma unroll
      for (int j = 0; j < SLOTS; ++j)
        if (grp[j] == g && key[j] > b1) b1 = key[j];
      b1 = wave_max_u64(b1);  // never 0: a group has at least one member
      unsigned long long b2 = 0ull;
#pragma unroll
      for (int j = 0; j < SLOTS; ++j)
        if (grp[j] == g && key[j] != b1 && key[j] > b2) b2 = key[j];
      b2 = wave_max_u64(b2);  // 0: the group has one member
      const int e1 = (int)(0xFFFFFFFFu - (uint32_t)(b1 & 0xFFFFFFFFull));
      const int e2 = b2 ? (int)(0xFFFFFFFFu - (uint32_t)(b2 & 0xFFFFFFFFull)) : e1;
      const double l1 = lrow[e1], l2 = lrow[e2];
      double s1, s2;
      if (score_func == MOESD_SCORE_SOFTMAX) {
        s1 = exp(l1 - mx) / z;
        s2 = exp(l2 - mx) / z;
      } else {
        s1 = 1.0 / (1.0 + exp(-l1));
        s2 = 1.0 / (1.0 + exp(-l2));
      }
      const float gf = (float)(s1 + (b2 ? s2 : 0.0));  // >= 0: its bit pattern is ordered as it is
      if (lane == g)
        gkey = ((unsigned long long)(__float_as_uint(gf) | 0x80000000u) << 32) |
               (unsigned long long)(0xFFFFFFFFu - (uint32_t)g);
    }
    unsigned long long keep = 0ull;
#pragma nounroll
    for (int s = 0; s < topk_group; ++s) {
      const unsigned long long best = wave_max_u64(gkey);
      const int g = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
      keep |= 1ull << g;
      if (lane == g) gkey = 0ull;
    }
#pragma unroll
    for (int j = 0; j < SLOTS; ++j)
      if (!((keep >> (grp[j] & 63)) & 1ull)) key[j] = 0ull;
  }

  int my_id = 0;        // lane s keeps the s-th winner
  double my_logit = 0.0;
  double first_logit = 0.0;
#pragma nounroll
  for (int s = 0; s < K; ++s) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) best = key[j] > best ? key[j] : best;
    best = wave_max_u64(best);
    const int e = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
    // owner removes it; everyone takes its fp64 logit from the owner's register (a read of memory
    // here would put one load latency into each of the K rounds)
#pragma unroll
    for (int j = 0; j < SLOTS; ++j)
      if (lane + 64 * j == e) key[j] = 0ull;
    const int owner = __builtin_amdgcn_readfirstlane(e & 63), oslot = e >> 6;
    double cand = lval[0];
#pragma unroll
    for (int j = 1; j < SLOTS; ++j)
      if (j == oslot) cand = lval[j];
    const double lv = readlane_f64(cand, owner);
    if (s == 0) first_logit = lv;
    if (lane == s) { my_id = e; my_logit = lv; }
  }

  // scores of the winners (lanes 0..K-1), fp64
  double sc = 0.0;
  if (lane < K) {
    if (score_func == MOESD_SCORE_SOFTMAX) {
      sc = renorm ? exp(my_logit - first_logit) : exp(my_logit - mx) / z;
    } else {
      sc = 1.0 / (1.0 + exp(-my_logit));
    }
  }
  double den = 1.0;
  if (renorm) den = wave_sum_f64(sc);
  if (lane < K) {
    ids[(size_t)t * K + lane] = my_id;
    w[(size_t)t * K + lane] = (float)(sc / den * (double)scale);
  }
  if (gate && lane == 0) {
    gate[t] = (Etot > E) ? (float)(1.0 / (1.0 + exp(-lrow[E]))) : 1.0f;
  }
}

