// Routing: router logits in fp64, then per-token top-K with wavefront shuffles.
//
// The paper's Sec. 3.2 counts how many of the E experts t tokens activate when
// each token picks K of them; this file is the picking.  The logits are
// accumulated in fp64 (products of two bf16 values are exact there) and rounded
// once to fp32: that fp32 value is the selection key, so any summation order
// gives the same expert ids.
#include "common.h"

// ---------------------------------------------------------------------------
// logits[t, e] = sum_j x[t,j] * w[e,j] (+ bias[e]),  e in [0, E]; column E (only
// when w_shared_gate != NULL) is x . w_shared_gate, the shared expert's gate logit.
// One wave computes a 4-token x 4-expert tile; its 64 lanes split the hidden
// dimension in 16-byte pieces and fold their partial sums with xor-shuffles.
// ---------------------------------------------------------------------------
#define RL_TT 4
#define RL_EE 4

__global__ __launch_bounds__(256) void router_logits_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr, const float *__restrict__ bias,
    const uint16_t *__restrict__ wsg, int T, int d, int E, int Etot, double *__restrict__ logits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e0 = (blockIdx.y * 4 + wave) * RL_EE;
  const int t0 = blockIdx.x * RL_TT;
  if (e0 >= Etot) return;

  const uint16_t *xr[RL_TT];
  const uint16_t *wrow[RL_EE];
#pragma unroll
  for (int i = 0; i < RL_TT; ++i) xr[i] = x + (size_t)min(t0 + i, T - 1) * d;
#pragma unroll
  for (int j = 0; j < RL_EE; ++j) {
    const int e = min(e0 + j, Etot - 1);
    wrow[j] = (e < E) ? wr + (size_t)e * d : wsg;
  }
  double acc[RL_TT][RL_EE];
#pragma unroll
  for (int i = 0; i < RL_TT; ++i)
#pragma unroll
    for (int j = 0; j < RL_EE; ++j) acc[i][j] = 0.0;

  for (int k = lane * 8; k < d; k += 64 * 8) {  // d is a multiple of 8
    u32x4 xv[RL_TT], wv[RL_EE];
#pragma unroll
    for (int i = 0; i < RL_TT; ++i) xv[i] = ld16(xr[i] + k);
#pragma unroll
    for (int j = 0; j < RL_EE; ++j) wv[j] = ld16(wrow[j] + k);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      double xd[RL_TT], wd[RL_EE];
#pragma unroll
      for (int i = 0; i < RL_TT; ++i) {
        const uint32_t u = xv[i][kk >> 1];
        xd[i] = (double)__uint_as_float((kk & 1) ? (u & 0xFFFF0000u) : (u << 16));
      }
#pragma unroll
      for (int j = 0; j < RL_EE; ++j) {
        const uint32_t u = wv[j][kk >> 1];
        wd[j] = (double)__uint_as_float((kk & 1) ? (u & 0xFFFF0000u) : (u << 16));
      }
#pragma unroll
      for (int i = 0; i < RL_TT; ++i)
#pragma unroll
        for (int j = 0; j < RL_EE; ++j) acc[i][j] = fma(xd[i], wd[j], acc[i][j]);
    }
  }
#pragma unroll
  for (int i = 0; i < RL_TT; ++i)
#pragma unroll
    for (int j = 0; j < RL_EE; ++j) {
      double v = acc[i][j];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
      acc[i][j] = v;
    }
  if (lane < RL_TT * RL_EE) {
    const int i = lane / RL_EE, j = lane % RL_EE;
    double v = 0.0;
#pragma unroll
    for (int ii = 0; ii < RL_TT; ++ii)
#pragma unroll
      for (int jj = 0; jj < RL_EE; ++jj)
        if (ii == i && jj == j) v = acc[ii][jj];
    const int t = t0 + i, e = e0 + j;
    if (t < T && e < Etot) {
      if (e < E && bias) v += (double)bias[e];
      logits[(size_t)t * Etot + e] = v;
    }
  }
}

hipError_t launch_router_logits(const uint16_t *x, const uint16_t *w_router, const float *bias,
                                const uint16_t *w_shared_gate, int T, int d, int E, double *logits,
                                hipStream_t s) {
  const int Etot = E + (w_shared_gate ? 1 : 0);
  dim3 grid((T + RL_TT - 1) / RL_TT, (Etot + 4 * RL_EE - 1) / (4 * RL_EE));
  hipLaunchKernelGGL(router_logits_kernel, grid, dim3(256), 0, s, x, w_router, bias, w_shared_gate, T,
                     d, E, Etot, logits);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Per-token top-K.  One wave per token; lane l owns experts l, l+64, ...
// A key is packed as (order-preserving u32 of the fp32 logit) << 32 | ~index, so
// one unsigned max picks the largest key and, among equals, the lowest index.
// K rounds of a 64-lane max reduction produce the ids in descending order.
// Scores and weights are evaluated in fp64 from the fp64 logits and rounded
// once to fp32.
// ---------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(v, off, 64);
    v = o > v ? o : v;
  }
  return v;
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

template <int SLOTS>  // experts per lane: E <= 64 * SLOTS
__global__ __launch_bounds__(256) void topk_kernel(const double *__restrict__ logits, int T, int E,
                                                   int Etot, int K, int score_func, int renorm,
                                                   float scale, int32_t *__restrict__ ids,
                                                   float *__restrict__ w, float *__restrict__ gate) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  const double *lrow = logits + (size_t)t * Etot;

  unsigned long long key[SLOTS];
#pragma unroll
  for (int j = 0; j < SLOTS; ++j) {
    const int e = lane + 64 * j;
    key[j] = 0ull;  // below every real key (real keys have a non-zero low word)
    if (e < E) {
      const float kf = (float)lrow[e] + 0.0f;  // the one rounding; +0 folds -0 into +0
      uint32_t u = __float_as_uint(kf);
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      key[j] = ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)e);
    }
  }

  // full-softmax normaliser, needed only when the winners are not renormalised
  double mx = 0.0, z = 1.0;
  if (score_func == MOESD_SCORE_SOFTMAX && !renorm) {
    double m = -1.0e300;
#pragma nounroll
    for (int e = lane; e < E; e += 64) m = fmax(m, lrow[e]);
    mx = wave_max_f64(m);
    double sacc = 0.0;
#pragma nounroll
    for (int e = lane; e < E; e += 64) sacc += exp(lrow[e] - mx);
    z = wave_sum_f64(sacc);
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
    // owner removes it; everyone re-reads its fp64 logit (a broadcast load)
#pragma unroll
    for (int j = 0; j < SLOTS; ++j)
      if (lane + 64 * j == e) key[j] = 0ull;
    const double lv = lrow[e];
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

hipError_t launch_topk(const double *logits, int T, int E, int K, int score_func, int renorm,
                       float scale, int has_shared_gate, int32_t *ids, float *w, float *gate,
                       hipStream_t s) {
  const int Etot = E + (has_shared_gate ? 1 : 0);
  const dim3 grid((T + 3) / 4), block(256);
  if (E <= 64)
    hipLaunchKernelGGL(topk_kernel<1>, grid, block, 0, s, logits, T, E, Etot, K, score_func, renorm,
                       scale, ids, w, gate);
  else if (E <= 256)
    hipLaunchKernelGGL(topk_kernel<4>, grid, block, 0, s, logits, T, E, Etot, K, score_func, renorm,
                       scale, ids, w, gate);
  else
    hipLaunchKernelGGL(topk_kernel<MOESD_MAX_E / 64>, grid, block, 0, s, logits, T, E, Etot, K,
                       score_func, renorm, scale, ids, w, gate);
  return hipGetLastError();
}
