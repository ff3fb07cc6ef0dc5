/*
 * moesd.h -- C ABI of libmoesd: the sparse-MoE FFN layer forward over a
 * speculative-decoding verification batch of T = B*(gamma+1) tokens, written
 * for one AMD MI355X (gfx950).
 *
 * The paper (MoESD, arXiv 2505.19645) models the cost of this layer: Sec. 3.2
 * counts the experts that t tokens activate (Eq. N(t)), and Sec. 3.3 prices a
 * target forward as  bias + k1*G(t) + k2*N + k3*G(Texp).  This library is the
 * layer that those formulas describe, plus the three closed forms themselves.
 *
 * Conventions for every entry point
 *   - "device" pointers are plain HIP device addresses owned by the caller;
 *     "host" pointers are ordinary process memory.  Nothing here allocates,
 *     frees or synchronises; all work is enqueued on `stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and the call returns at once.
 *   - bf16 tensors are arrays of 16-bit words (upper half of an IEEE fp32).
 *   - Matrices are row-major, [out, in]: the contraction index is contiguous.
 *   - Arguments are validated on the host before anything is launched.  On
 *     MOESD_INVALID_ARG, MOESD_UNSUPPORTED and MOESD_WORKSPACE_TOO_SMALL nothing
 *     has been enqueued and no output was touched.  MOESD_HIP_ERROR reports a
 *     failure of the HIP runtime itself (a launch or an event record refused);
 *     kernels enqueued before it stay enqueued and the outputs are undefined.
 *   - T == 0 is a successful no-op.
 *   - Calls that use the same workspace or outputs on different streams race.
 *     Besides that the library keeps, per process: the last HIP error code, and
 *     per device ordinal the compute-unit count and which kernels already had
 *     their dynamic-LDS limit raised (atomics; every writer stores the same
 *     value, so concurrent first calls are safe).  Work is launched on the
 *     device the calling thread has current.
 *
 * The interface is the four calls of the problem statement (route, permute,
 * forward, expected activated experts) with these additions, each for a stated
 * reason: moesd_route takes a workspace (the fp64 logits live there);
 * moesd_moe_forward also returns inv_perm and, on request, the output before its
 * final rounding (out_f32), both for checking; the descriptor carries n_group /
 * topk_group (group-limited selection) and weight_format (low-precision expert
 * weights); moesd_moe_forward_staged records events at the stage boundaries for
 * timing; moesd_moe_forward_static is the variant for callers that cannot
 * allocate; moesd_expected_active_experts_p, moesd_expected_tokens_per_expert
 * and moesd_token_threshold are further closed forms of Sec. 3.2.
 */
#ifndef MOESD_H
#define MOESD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define MOESD_OK                  0
#define MOESD_INVALID_ARG         1  /* null pointer, K<1, K>E, E<1, T<0, T*K >= 2^31,
                                        d / inter / shared_inter not a multiple of 8   */
#define MOESD_UNSUPPORTED         2  /* E > MOESD_MAX_E, K > MOESD_MAX_K, unknown enum,
                                        T*d*2 >= 2^32 (a token row's byte offset is 32-bit) */
#define MOESD_WORKSPACE_TOO_SMALL 3
#define MOESD_HIP_ERROR           4  /* see moesd_last_hip_error()                     */

#define MOESD_MAX_E 1024             /* experts: 16 keys per lane of a 64-wide wave    */
#define MOESD_MAX_K 32

#define MOESD_SCORE_SOFTMAX 0
#define MOESD_SCORE_SIGMOID 1

/* expert weight formats (routed and shared expert matrices; the router stays bf16) */
#define MOESD_WEIGHTS_BF16     0
#define MOESD_WEIGHTS_FP8_E4M3 1  /* 8-bit codes, E4M3 of the OCP OFP8 specification (1 sign, 4 exponent
                                     bits with bias 7, 3 mantissa bits, subnormals, no infinities,
                                     S.1111.111 = NaN, largest finite value 448), one fp32 scale per
                                     output row: weight = decode(code) * scale[row].  Halves the bytes of
                                     the expert-loading term k2*N of Sec. 3.3, whose floor scales with the
                                     weights' bit width (Appendix C.2).  Codes are assumed finite.  d,
                                     inter and shared_inter must be multiples of 16. */

/* One MoE layer's shape, in the paper's notation (Sec. 3.2: E experts, K per
 * token; rho = K/E).  The arithmetic choices below are not in the paper, which
 * never spells the layer out; they follow the usual SwiGLU MoE block. */
typedef struct {
  int32_t d;            /* hidden size                                           */
  int32_t E;            /* number of routed experts                              */
  int32_t top_k;        /* K: experts per token                                  */
  int32_t inter;        /* I: intermediate size of one routed expert             */
  int32_t shared_inter; /* S: intermediate size of the shared expert, 0 = none   */
  int32_t score_func;   /* MOESD_SCORE_SOFTMAX (over all E) or MOESD_SCORE_SIGMOID */
  int32_t renormalize;  /* 1: top-k scores are divided by their sum              */
  int32_t shared_gate;  /* 1: shared expert scaled by sigmoid(x . w_shared_gate) */
  float   routed_scale; /* multiplies every routed weight (1.0 = none)           */
  int32_t n_group;      /* > 1: group-limited selection, see moesd_route; else off */
  int32_t topk_group;   /* groups kept per token (1 .. n_group)                    */
  int32_t weight_format; /* MOESD_WEIGHTS_BF16 or MOESD_WEIGHTS_FP8_E4M3           */
} moesd_layer_desc;

/* All weights: device pointers, read-only, caller-owned.  Router, bias and shared gate as stated;
 * the six expert matrices are bf16, or uint8 E4M3 codes with the same shapes when
 * desc->weight_format == MOESD_WEIGHTS_FP8_E4M3; then each has an fp32 scale per output row. */
typedef struct {
  const void  *w_router;      /* [E, d]                                          */
  const float *router_bias;   /* [E] fp32, added to the logits; may be NULL      */
  const void  *w_gate;        /* [E, I, d]                                       */
  const void  *w_up;          /* [E, I, d]                                       */
  const void  *w_down;        /* [E, d, I]                                       */
  const void  *ws_gate;       /* [S, d]   (NULL iff S == 0)                      */
  const void  *ws_up;         /* [S, d]                                          */
  const void  *ws_down;       /* [d, S]                                          */
  const void  *w_shared_gate; /* [d]      (NULL iff shared_gate == 0)            */
  /* row scales, fp32; NULL unless the weights are MOESD_WEIGHTS_FP8_E4M3 */
  const float *w_gate_scale;  /* [E, I]                                          */
  const float *w_up_scale;    /* [E, I]                                          */
  const float *w_down_scale;  /* [E, d]                                          */
  const float *ws_gate_scale; /* [S]                                             */
  const float *ws_up_scale;   /* [S]                                             */
  const float *ws_down_scale; /* [d]                                             */
} moesd_weights;

/* ---------------------------------------------------------------------------
 * Closed forms of Sec. 3.2 (host only, pure, no GPU needed).
 * ------------------------------------------------------------------------- */

/* Expected number of activated experts after t tokens under uniform routing,
 * Eq. N(t):  E * (1 - ((E-K)/E)^t).  NaN if E<1, K<0, K>E or t<0. */
double moesd_expected_active_experts(int32_t E, int32_t K, int64_t t);

/* The same expectation without the uniformity assumption that Sec. 3.2 makes:
 * the step before Eq. N(t) (an expert is activated unless none of the t tokens
 * activates it) applied to each expert with its own probability p[e] of being
 * activated by one token (host array of E values in [0,1], summing to K), tokens
 * independent:  sum_e (1 - (1 - p[e])^t).  p[e] = K/E gives Eq. N(t); any other p
 * with the same sum gives less.  NaN on bad input. */
double moesd_expected_active_experts_p(const double *p, int32_t E, int64_t t);

/* Mean tokens per activated expert, Eq. Texp:  t*K / N(t)  =
 * rho*t / (1 - (1-rho)^t).  Returns 0 for t == 0 or K == 0; NaN on bad input. */
double moesd_expected_tokens_per_expert(int32_t E, int32_t K, int64_t t);

/* Token threshold of near-full activation, Eq. T_thres: the smallest integer t
 * with N(t) >= tau*E, i.e. ceil(log_{1-rho}(1-tau)).  K == E gives 1.
 * Returns -1 on bad input (E<1, K<1, K>E, tau outside [0,1)). */
int64_t moesd_token_threshold(int32_t E, int32_t K, double tau);

/* ---------------------------------------------------------------------------
 * Workspace
 * ------------------------------------------------------------------------- */

/* Bytes of device scratch that moesd_route / moesd_moe_forward need for up to
 * T_max tokens (256-byte aligned pieces; the caller's buffer must itself be
 * 256-byte aligned).  Besides the per-token buffers (logits, routing outputs,
 * the bf16 activation [T*K, I] and the fp32 expert outputs [T*K, d]) it holds,
 * for T_max > 128, 128 MB of partial-sum space for the
 * MFMA-tiled expert kernels (512 KB for each of at most 256 persistent workgroups).  The size depends on
 * the arguments only, not on the device.  Returns 0 if the descriptor or T_max
 * is invalid. */
size_t moesd_workspace_bytes(const moesd_layer_desc *desc, int32_t T_max);

/* ---------------------------------------------------------------------------
 * Hot path.  The steps are those a verification forward of the target model
 * runs once per layer (Sec. 3.1: T_T(B, gamma) is one forward over all drafted
 * tokens of all B requests); their cost is what Sec. 3.3 models.
 * ------------------------------------------------------------------------- */

/* Router: logits = x . w_router^T (+ bias), accumulated in fp64 and rounded once
 * to fp32; that fp32 value is the selection key.  Per token the K largest keys
 * win, equal keys go to the lower expert index, and ids are emitted in that
 * (descending key, ascending index) order.  Weights are softmax-over-E or
 * sigmoid scores of the winners, optionally divided by their sum, times
 * routed_scale.
 * With desc->n_group > 1 the selection is group-limited (the rule published for
 * the model family of benchmark config 4, without its selection bias; Sec. 3.2
 * models unconstrained selection): the experts form n_group equal consecutive
 * groups (E divisible by n_group, n_group <= 64), a group's score is the sum of
 * the scores of its two members with the largest keys, rounded once to fp32,
 * the topk_group groups with the largest score stay (equal scores: the lower
 * group index) and the K winners are taken among their members
 * (K <= topk_group * E / n_group).
 *   x          device [T, d] bf16
 *   w_router   device [E, d] bf16;  router_bias device [E] fp32 or NULL
 *   topk_ids   device [T, K] int32 (out);  topk_w  device [T, K] fp32 (out)
 *   workspace  device, >= moesd_workspace_bytes(desc, T)
 */
int32_t moesd_route(const moesd_layer_desc *desc, const void *x, const void *w_router,
                    const float *router_bias, int32_t T, int32_t *topk_ids, float *topk_w,
                    void *workspace, size_t workspace_bytes, void *stream);

/* Token-to-expert permutation: the stable counting sort of the T*K flat slots
 * f = t*K + s by expert id.
 *   topk_ids  device [T*K] int32, every value in [0, E) (not checked)
 *   counts    device [E]    tokens per expert (m_e)
 *   offsets   device [E+1]  exclusive prefix sum of counts, offsets[E] = T*K
 *   perm      device [T*K]  perm[p] = f, the slot that lands at sorted row p
 *   inv_perm  device [T*K]  inv_perm[f] = p
 *   n_active  device [1]    number of experts with counts > 0: the paper's N
 * No workspace.  Deterministic: equal inputs give equal bytes. */
int32_t moesd_permute(int32_t E, int32_t K, int32_t T, const int32_t *topk_ids,
                      int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                      int32_t *n_active, void *stream);

/* The whole layer: route, permute, grouped SwiGLU expert FFN over the activated
 * experts only, shared expert, weighted combine.
 *   out[t,:] = sum_s w[t,s] * FFN_{ids[t,s]}(x_t)  +  g_t * FFN_shared(x_t)
 *   FFN_e(x) = W_down_e . ( silu(W_gate_e . x) * (W_up_e . x) )
 * bf16 operands, fp32 accumulation, the intermediate activation is rounded to
 * bf16 once, the output is rounded to bf16 once.  E4M3 weights are widened to bf16
 * (exactly) for the multiplication and the row scale is applied to the fp32 sum.
 *   x    device [T, d] bf16;   out  device [T, d] bf16
 *   out_f32   device [T, d] fp32 or NULL: the same result before rounding
 *   topk_ids .. n_active: optional device outputs (any may be NULL), shaped as
 *   in moesd_route / moesd_permute, for checking the intermediate steps.
 */
int32_t moesd_moe_forward(const moesd_layer_desc *desc, const moesd_weights *weights,
                          const void *x, int32_t T, void *out, float *out_f32,
                          void *workspace, size_t workspace_bytes,
                          int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets,
                          int32_t *perm, int32_t *inv_perm, int32_t *n_active, void *stream);

/* Same as moesd_moe_forward, and additionally records caller-created
 * hipEvent_t handles on `stream` at the stage boundaries, so a harness can
 * time each stage of one real forward:
 *   events[0] before routing, [1] after routing + permutation,
 *   [2] after the gate/up kernel, [3] after the down kernel, [4] after combine.
 * events: host array of MOESD_N_STAGE_EVENTS hipEvent_t (as void*). */
#define MOESD_N_STAGE_EVENTS 5
int32_t moesd_moe_forward_staged(const moesd_layer_desc *desc, const moesd_weights *weights,
                                 const void *x, int32_t T, void *out, float *out_f32,
                                 void *workspace, size_t workspace_bytes,
                                 int32_t *topk_ids, float *topk_w, int32_t *counts,
                                 int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                                 int32_t *n_active, void *stream, void *const *events);

/* For callers that cannot allocate device memory around the call (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * moesd_moe_forward without the workspace arguments.  The scratch is a
 * MOESD_STATIC_SCRATCH_BYTES array inside the library's device image; every GPU
 * the library runs on holds its own copy until the process ends.  The call
 * allocates nothing and frees nothing.  It returns MOESD_WORKSPACE_TOO_SMALL
 * (nothing enqueued) when moesd_workspace_bytes(desc, T) exceeds
 * MOESD_STATIC_SCRATCH_BYTES: 32 MB hold every benchmark shape up to T = 64
 * (config 1 up to T = 128); T > 128 never fits, the MFMA-tiled kernels' 128 MB of
 * partial-sum space alone exceed it.  All calls on one GPU share the one array:
 * calls that overlap in time on one GPU race, also on different streams.  Nothing
 * in the array needs clearing between calls (the permutation kernel zeroes the two
 * counters the expert kernels draw from, as it does in a caller's workspace).
 * Inputs, outputs and the optional outputs are as in moesd_moe_forward. */
#define MOESD_STATIC_SCRATCH_BYTES (32u << 20)
int32_t moesd_moe_forward_static(const moesd_layer_desc *desc, const moesd_weights *weights,
                                 const void *x, int32_t T, void *out, float *out_f32,
                                 int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets,
                                 int32_t *perm, int32_t *inv_perm, int32_t *n_active, void *stream);

/* ---------------------------------------------------------------------------
 * Diagnostics
 * ------------------------------------------------------------------------- */
const char *moesd_status_string(int32_t status);
int32_t     moesd_last_hip_error(void);   /* hipError_t of the last MOESD_HIP_ERROR, else 0 */

#ifdef __cplusplus
}
#endif
#endif /* MOESD_H */
