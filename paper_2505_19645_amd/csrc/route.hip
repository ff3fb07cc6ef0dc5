// Routing: router logits in fp64, then per-token top-K with wavefront shuffles.
//
// The paper's Sec. 3.2 counts how many of the E experts t tokens activate when
// each token picks K of them; this file is the picking.  The logits are
// accumulated in fp64 (products of two bf16 values are exact there) and rounded
// once to fp32: that fp32 value is the selection key.  Two summation orders give
// fp64 sums that differ by about 1e-16 relative, so the key, and with it the
// expert ids, can differ only when a logit lies within that distance of an fp32
// rounding boundary: the ids are order-independent by margin, not by construction
// (logits built from a few powers of two are exact in any order; a test puts such
// logits on and next to rounding boundaries).
#include "common.h"
#include "route_device.h"

// ---------------------------------------------------------------------------
// logits[t, e] = sum_j x[t,j] * w[e,j] (+ bias[e]),  e in [0, E]; column E (only
// when w_shared_gate != NULL) is x . w_shared_gate, the shared expert's gate logit.
// One workgroup computes 8 tokens x 1 expert: its four waves take interleaved
// 1 KB pieces of the hidden dimension (64 lanes x 16 bytes), fold their partial
// sums with xor-shuffles and add the four wave sums through LDS.  The grid
// covers (token blocks) x (experts), so even a single token spreads the router
// matrix over E workgroups and no wave walks more than d/2048 dependent steps.
// ---------------------------------------------------------------------------
#define RL_TT 8
// the register-tiled kernels below run when they have at least this many workgroups
#define RL_TILED8_MIN_WGS 288  // 8 tokens x 8 experts per wave
#define RL_TILED4_MIN_WGS 192  // 8 tokens x 4 experts per wave

__device__ __forceinline__ double bf16_pair_lo(uint32_t u) { return (double)__uint_as_float(u << 16); }
__device__ __forceinline__ double bf16_pair_hi(uint32_t u) { return (double)__uint_as_float(u & 0xFFFF0000u); }

__global__ __launch_bounds__(256) void router_logits_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr, const float *__restrict__ bias,
    const uint16_t *__restrict__ wsg, int T, int d, int E, int Etot, double *__restrict__ logits) {
  __shared__ double part[4][RL_TT];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e = blockIdx.y;
  const int t0 = blockIdx.x * RL_TT;
  const uint16_t *wrow = (e < E) ? wr + (size_t)e * d : wsg;
  const int nt = min(RL_TT, T - t0);  // tokens of this block (uniform)
  double acc[RL_TT];
#pragma unroll
  for (int i = 0; i < RL_TT; ++i) acc[i] = 0.0;

#pragma unroll 2
  for (int k = (wave * 64 + lane) * 8; k < d; k += 256 * 8) {  // d is a multiple of 8
    const u32x4 wv = ld16(wrow + k);
    u32x4 xv[RL_TT];
#pragma unroll
    for (int i = 0; i < RL_TT; ++i)
      if (i < nt) xv[i] = ld16(x + (size_t)(t0 + i) * d + k);
    double wd[8];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      wd[2 * c] = bf16_pair_lo(wv[c]);
      wd[2 * c + 1] = bf16_pair_hi(wv[c]);
    }
#pragma unroll
    for (int i = 0; i < RL_TT; ++i)
      if (i < nt) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          acc[i] = fma(bf16_pair_lo(xv[i][c]), wd[2 * c], acc[i]);
          acc[i] = fma(bf16_pair_hi(xv[i][c]), wd[2 * c + 1], acc[i]);
        }
      }
  }
#pragma unroll
  for (int i = 0; i < RL_TT; ++i)
    if (i < nt) {
      double v = acc[i];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0) part[wave][i] = v;
    }
  __syncthreads();
  if (threadIdx.x < nt) {
    const int i = threadIdx.x;
    double v = ((part[0][i] + part[1][i]) + part[2][i]) + part[3][i];
    if (e < E && bias) v += (double)bias[e];
    logits[(size_t)(t0 + i) * Etot + e] = v;
  }
}

// Many tokens: register-tiled variant.  A wave owns 8 tokens x RLT_EB (8 or 4) experts over
// the whole contraction (lane l takes the 16-byte pieces l, l+64, ...), so a converted token
// value feeds RLT_EB FMAs and a converted weight value 8: a quarter (three eighths) of a
// conversion per FMA instead of more than one above, and the token rows are read once per
// 4 * RLT_EB experts (the 4 waves of a workgroup take 4 expert blocks of the same 8 tokens).
// The narrower block has twice the workgroups, for the sizes where the wider one would leave
// compute units idle.
// The partial sums of a lane are reduced across the wave by halving: in each of six
// steps a lane keeps the half of its (zero-padded to 64) values that its partner does not,
// so lane l ends with the full sum of value index l = RLT_EB * token + expert.
#define RLT_TT 8
template <int RLT_EB>
__global__ __launch_bounds__(256) void router_logits_tiled_kernel(
    const uint16_t *__restrict__ x, const uint16_t *__restrict__ wr, const float *__restrict__ bias,
    const uint16_t *__restrict__ wsg, int T, int d, int E, int Etot, double *__restrict__ logits) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * RLT_TT;
  const int e0 = (blockIdx.y * 4 + wave) * RLT_EB;
  if (e0 >= Etot) return;
  const uint16_t *xrow[RLT_TT];
  const uint16_t *wrow[RLT_EB];
#pragma unroll
  for (int i = 0; i < RLT_TT; ++i) xrow[i] = x + (size_t)min(t0 + i, T - 1) * d;
#pragma unroll
  for (int j = 0; j < RLT_EB; ++j) {
    const int e = min(e0 + j, Etot - 1);
    wrow[j] = (e < E) ? wr + (size_t)e * d : wsg;
  }
  double acc[RLT_TT][RLT_EB];
#pragma unroll
  for (int i = 0; i < RLT_TT; ++i)
#pragma unroll
    for (int j = 0; j < RLT_EB; ++j) acc[i][j] = 0.0;

  // the pieces of the next step are fetched before the FMAs of the current one
  u32x4 xv[RLT_TT], wv[RLT_EB];
  {
    const int k = min(lane * 8, d - 8);
#pragma unroll
    for (int i = 0; i < RLT_TT; ++i) xv[i] = ld16(xrow[i] + k);
#pragma unroll
    for (int j = 0; j < RLT_EB; ++j) wv[j] = ld16(wrow[j] + k);
  }
  for (int k = lane * 8; k < d; k += 64 * 8) {  // d is a multiple of 8
    u32x4 xc[RLT_TT], wc[RLT_EB];
#pragma unroll
    for (int i = 0; i < RLT_TT; ++i) xc[i] = xv[i];
#pragma unroll
    for (int j = 0; j < RLT_EB; ++j) wc[j] = wv[j];
    const int kn = min(k + 64 * 8, d - 8);  // (a step past the end re-reads the last piece; unused)
#pragma unroll
    for (int i = 0; i < RLT_TT; ++i) xv[i] = ld16(xrow[i] + kn);
#pragma unroll
    for (int j = 0; j < RLT_EB; ++j) wv[j] = ld16(wrow[j] + kn);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      double xl[RLT_TT], xh[RLT_TT];
#pragma unroll
      for (int i = 0; i < RLT_TT; ++i) {
        xl[i] = bf16_pair_lo(xc[i][c]);
        xh[i] = bf16_pair_hi(xc[i][c]);
      }
#pragma unroll
      for (int j = 0; j < RLT_EB; ++j) {
        const double wl = bf16_pair_lo(wc[j][c]), wh = bf16_pair_hi(wc[j][c]);
#pragma unroll
        for (int i = 0; i < RLT_TT; ++i) {
          acc[i][j] = fma(xl[i], wl, acc[i][j]);
          acc[i][j] = fma(xh[i], wh, acc[i][j]);
        }
      }
    }
  }
  // halving reduction over the 64 lanes; value index v = RLT_EB * token + expert, the
  // values beyond RLT_TT * RLT_EB are zero padding
  double v[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) v[i] = 0.0;
#pragma unroll
  for (int i = 0; i < RLT_TT; ++i)
#pragma unroll
    for (int j = 0; j < RLT_EB; ++j) v[i * RLT_EB + j] = acc[i][j];
#pragma unroll
  for (int step = 0; step < 6; ++step) {
    const int half = 32 >> step;          // values kept per lane after this step
    const bool upper = (lane >> (5 - step)) & 1;  // lane bit that decides which half it keeps
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      if (i < half) {
        const double keep = upper ? v[i + half] : v[i];
        const double send = upper ? v[i] : v[i + half];
        v[i] = keep + __shfl_xor(send, 32 >> step, 64);
      }
    }
  }
  // lane l now holds value index: bit (5 - step) of l chose the upper half at step `step`,
  // i.e. index l itself
  const int ti = lane / RLT_EB, ej = lane % RLT_EB;
  const int t = t0 + ti, e = e0 + ej;
  if (ti < RLT_TT && t < T && e < Etot) {
    double r = v[0];
    if (e < E && bias) r += (double)bias[e];
    logits[(size_t)t * Etot + e] = r;
  }
}

hipError_t launch_router_logits(const uint16_t *x, const uint16_t *w_router, const float *bias,
                                const uint16_t *w_shared_gate, int T, int d, int E, double *logits,
                                hipStream_t s) {
  const int Etot = E + (w_shared_gate ? 1 : 0);
  // the tiled kernels have 16x or 32x fewer workgroups: only when those still fill the chip
  const int tb = (T + RLT_TT - 1) / RLT_TT;
  const int eb8 = (Etot + 31) / 32, eb4 = (Etot + 15) / 16;
  if ((long)tb * eb8 >= RL_TILED8_MIN_WGS) {
    hipLaunchKernelGGL(router_logits_tiled_kernel<8>, dim3(tb, eb8), dim3(256), 0, s, x, w_router, bias,
                       w_shared_gate, T, d, E, Etot, logits);
    return hipGetLastError();
  }
  if ((long)tb * eb4 >= RL_TILED4_MIN_WGS) {
    hipLaunchKernelGGL(router_logits_tiled_kernel<4>, dim3(tb, eb4), dim3(256), 0, s, x, w_router, bias,
                       w_shared_gate, T, d, E, Etot, logits);
    return hipGetLastError();
  }
  dim3 grid((T + RL_TT - 1) / RL_TT, Etot);
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
template <int SLOTS>
__global__ __launch_bounds__(256) void topk_kernel(const double *__restrict__ logits, int T, int E,
                                                   int Etot, int K, int score_func, int renorm,
                                                   float scale, int groups, int32_t *__restrict__ ids,
                                                   float *__restrict__ w, float *__restrict__ gate) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  topk_token<SLOTS>(logits, t, lane, E, Etot, K, score_func, renorm, scale, groups, ids, w, gate);
}

hipError_t launch_topk(const double *logits, int T, int E, int K, int score_func, int renorm,
                       float scale, int groups, int has_shared_gate, int32_t *ids, float *w,
                       float *gate, hipStream_t s) {
  const int Etot = E + (has_shared_gate ? 1 : 0);
  const dim3 grid((T + 3) / 4), block(256);
  if (E <= 64)
    hipLaunchKernelGGL(topk_kernel<1>, grid, block, 0, s, logits, T, E, Etot, K, score_func, renorm,
                       scale, groups, ids, w, gate);
  else if (E <= 256)
    hipLaunchKernelGGL(topk_kernel<4>, grid, block, 0, s, logits, T, E, Etot, K, score_func, renorm,
                       scale, groups, ids, w, gate);
  else
    hipLaunchKernelGGL(topk_kernel<MOESD_MAX_E / 64>, grid, block, 0, s, logits, T, E, Etot, K,
                       score_func, renorm, scale, groups, ids, w, gate);
  return hipGetLastError();
}
