// Internal helpers shared by the HIP kernels of libmoesd (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/moesd.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

#define MOESD_WAVE 64

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round to nearest even; finite inputs
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ u32x4 ld16(const uint16_t *p) { return *reinterpret_cast<const u32x4 *>(p); }

// streaming 16-byte load: the weights are read exactly once, keep them out of the caches' way
__device__ __forceinline__ u32x4 ld16_stream(const uint16_t *p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// silu(z) = z / (1 + e^-z) with the hardware exp2 and reciprocal (each about 1 ulp): a few
// ulp of fp32 in all, far below the bf16 rounding of the activation that follows.  e^-z
// overflows to +inf for z < -88 and the result is -0, as it should be.
__device__ __forceinline__ float silu_f32(float z) {
  const float e = __builtin_amdgcn_exp2f(z * -1.44269504088896340736f);
  return z * __builtin_amdgcn_rcpf(1.0f + e);
}

// ---- launch descriptors (host fills, passed by value) ------------------------

// Plan written by the permutation kernel for the expert kernels (int32 words):
//   [0] n_small:  experts with 1..16 rows
//   [1] n_big64:  experts with 17..64 rows
//   [2] n_large:  (expert, 256-row block) entries of the experts with more than 128 rows
//   [3] n_big128: experts with 65..128 rows
//   [PLAN_CTR], [PLAN_CTR+1]  zero: the counters from which the gate/up and the down streaming
//                kernel draw units of tiles
//   [PLAN_HDR .. +E)        ids of the small experts, ascending
//   [PLAN_HDR+E .. +2E)     ids of the experts with 17..64 rows, ascending
//   [PLAN_HDR+2E .. +3E)    ids of the experts with 65..128 rows, ascending
//   [PLAN_HDR+5E .. )       n_large pairs (expert id, block index), ascending by expert, block
#define PLAN_HDR 8
#define PLAN_CTR 4
#define PLAN_BIG_MAX_ROWS 128
#define PLAN_BIG64_OFF(E) (PLAN_HDR + (E))
#define PLAN_BIG128_OFF(E) (PLAN_HDR + 2 * (E))
#define PLAN_LARGE_OFF(E) (PLAN_HDR + 5 * (E))
#define PLAN_WORDS(E, TK) (PLAN_LARGE_OFF(E) + 2 * ((E) + (TK) / 256 + 2))

struct StreamArgs {
  // routed experts: bf16 words, or (fp8 != 0) E4M3 bytes with one fp32 scale per output row
  const void *w_gate, *w_up, *w_down;         // [E,I,d] [E,I,d] [E,d,I]
  // shared expert
  const void *ws_gate, *ws_up, *ws_down;      // [S,d] [S,d] [d,S]
  const float *s_gate, *s_up, *s_down;        // [E,I] [E,I] [E,d] row scales (fp8 only)
  const float *ss_gate, *ss_up, *ss_down;     // [S] [S] [d]
  int32_t fp8;
  const uint16_t *x;                          // [T,d]
  uint16_t *h;                                // [T*K, I] bf16
  uint16_t *hs;                               // [T, S]   bf16
  float *y;                                   // [T*K, d] f32
  float *ys;                                  // [parts, T, d] f32: partial sums over k-parts of S
  const int32_t *offsets;                     // [E+1]
  const int32_t *row_token;                   // [T*K] sorted row -> token
  const int32_t *plan;
  int32_t d, E, K, I, S, T;
  int32_t part_k;                             // k-part length of the shared down projection
  int32_t shared_stream;                      // 1: the streaming kernels take the shared expert, 0: the tiled ones
};

// ---- per-device facts (moesd_api.cpp) --------------------------------------------
// The device the calling thread has current and its compute-unit count.  The counts are cached
// per device ordinal in atomics: every thread that fills a cache entry writes the same value.
#define MOESD_MAX_DEVICES 64
hipError_t current_device(int *dev, int *n_cu);
// Kernels that need more dynamic LDS than the default limit raise it once per (kernel, device):
// one bit per device ordinal; a repeated call is harmless, so a race between two first calls is too.
struct LdsLimitOnce {
  std::atomic<unsigned long long> done{0ull};
};
hipError_t raise_dynamic_lds_limit(LdsLimitOnce &once, int dev, const void *kernel, int bytes);

// host-side launch entry points, one per source file
hipError_t launch_router_logits(const uint16_t *x, const uint16_t *w_router, const float *bias,
                                const uint16_t *w_shared_gate, int T, int d, int E, double *logits,
                                hipStream_t s);
// groups = n_group | topk_group << 16 (0: unconstrained selection)
hipError_t launch_topk(const double *logits, int T, int E, int K, int score_func, int renorm,
                       float scale, int groups, int has_shared_gate, int32_t *ids, float *w,
                       float *gate, hipStream_t s);
// row_token / plan may be NULL (standalone permutation).  wide_fill_min: experts with 65..128 rows
// go to the tiled kernels' list if some expert has more than 128 rows and fewer than that many
// experts have 17..128 rows (0: never).
hipError_t launch_permute(const int32_t *ids, int64_t n, int E, int K, int32_t *counts,
                          int32_t *offsets, int32_t *perm, int32_t *inv, int32_t *n_active,
                          int32_t *row_token, int32_t *plan, int wide_fill_min, hipStream_t s);
// top-K and permutation in one launch; only for E <= 256 and few tokens
hipError_t launch_topk_permute(const double *logits, int T, int E, int K, int score_func, int renorm,
                               float scale, int groups, int has_shared_gate, int32_t *ids, float *w,
                               float *gate, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                               int32_t *n_active, int32_t *row_token, int32_t *plan, int wide_fill_min,
                               hipStream_t s);
hipError_t launch_gate_up(const StreamArgs &a, hipStream_t s);
hipError_t launch_down(const StreamArgs &a, hipStream_t s);
// The tiled kernels are persistent and cut the work into equal shares; a tile cut by a
// share boundary is completed through `partials` (tiled_partials_bytes() bytes, the same on
// every device).
size_t tiled_partials_bytes();
// Which kernels should take the shared expert of S x d at T > 128 tokens (K of E experts per token): 1 = the streaming
// kernels (its weights pass once per 64 tokens), 0 = the MFMA-tiled kernels (a few 256-row tiles
// can leave most of the chip idle for as long as one tile takes).
int shared_expert_streams(int T, int d, int S, int part_k, int K, int E, int n_cu);
hipError_t launch_gate_up_tiled(const StreamArgs &a, float *partials, hipStream_t s);
hipError_t launch_down_tiled(const StreamArgs &a, float *partials, hipStream_t s);
hipError_t launch_combine(const float *y, const float *ys, int n_parts, const float *w,
                          const float *gate, const int32_t *inv, int T, int K, int d, uint16_t *out,
                          float *out_f32, hipStream_t s);
