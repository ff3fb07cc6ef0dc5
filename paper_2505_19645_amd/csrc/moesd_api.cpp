// Host side of libmoesd: argument checks, workspace carving, launch order.
#include <atomic>
#include <cstring>

#include "common.h"

// up to this many tokens one workgroup picks every top-K and sorts (one launch instead of two)
#ifndef MOESD_FUSED_TOPK_MAX_T
#define MOESD_FUSED_TOPK_MAX_T 32
#endif

namespace {

std::atomic<int32_t> g_last_hip_error{0};

int32_t hip_fail(hipError_t e) {
  g_last_hip_error.store((int32_t)e);
  return MOESD_HIP_ERROR;
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int32_t check_desc(const moesd_layer_desc *c) {
  if (!c) return MOESD_INVALID_ARG;
  if (c->E < 1 || c->top_k < 1 || c->top_k > c->E) return MOESD_INVALID_ARG;
  if (c->d < 8 || c->d % 8 || c->inter < 8 || c->inter % 8) return MOESD_INVALID_ARG;
  if (c->shared_inter < 0 || c->shared_inter % 8) return MOESD_INVALID_ARG;
  if (c->E > MOESD_MAX_E || c->top_k > MOESD_MAX_K) return MOESD_UNSUPPORTED;
  if (c->n_group > 1) {
    if (c->E % c->n_group != 0 || c->topk_group < 1 || c->topk_group > c->n_group ||
        (int64_t)c->top_k > (int64_t)c->topk_group * (c->E / c->n_group))
      return MOESD_INVALID_ARG;
    if (c->n_group > 64) return MOESD_UNSUPPORTED;
  }
  if (c->score_func != MOESD_SCORE_SOFTMAX && c->score_func != MOESD_SCORE_SIGMOID)
    return MOESD_UNSUPPORTED;
  if ((c->renormalize | 1) != 1 || (c->shared_gate | 1) != 1) return MOESD_UNSUPPORTED;
  if (c->weight_format != MOESD_WEIGHTS_BF16 && c->weight_format != MOESD_WEIGHTS_FP8_E4M3)
    return MOESD_UNSUPPORTED;
  if (c->weight_format == MOESD_WEIGHTS_FP8_E4M3 && (c->d % 16 || c->inter % 16 || c->shared_inter % 16))
    return MOESD_INVALID_ARG;  // 16-byte pieces of 8-bit weights
  return MOESD_OK;
}

int32_t check_T(const moesd_layer_desc *c, int32_t T) {
  if (T < 0) return MOESD_INVALID_ARG;
  if ((int64_t)T * c->top_k >= ((int64_t)1 << 31)) return MOESD_INVALID_ARG;
  // the MFMA-tiled kernels keep a token row's byte offset in 32 bits
  if ((int64_t)T * c->d * 2 >= ((int64_t)1 << 32)) return MOESD_UNSUPPORTED;
  return MOESD_OK;
}

// Workspace pieces, in order.  Every piece starts on a 256-byte boundary.
struct Workspace {
  double *logits;  // [T, E+1] fp64 router logits (+ shared-gate logit)
  int32_t *ids;    // [T, K]
  float *w;        // [T, K]
  int32_t *counts, *offsets, *perm, *inv, *n_active;
  int32_t *row_token;  // [T*K] sorted row -> token
  int32_t *plan;       // work lists for the expert kernels (see common.h)
  float *gate;     // [T]
  uint16_t *h;     // [T*K, I] bf16
  uint16_t *hs;    // [T, S]   bf16
  float *y;        // [T*K, d] f32
  float *ys;       // [parts, T, d] f32
  float *tiled_partials;     // partial accumulator tiles of the MFMA-tiled kernels (T > 128 only)
  int32_t part_k, parts;
  size_t bytes;
};

// Above how many tokens the MFMA-tiled kernels run (and need their partial-sum space): they take
// the experts with more than 128 rows.
inline int32_t tiled_from(const moesd_layer_desc *) { return PLAN_BIG_MAX_ROWS; }

// the group-limited selection's two settings in one launch argument (0: unconstrained)
inline int groups_of(const moesd_layer_desc *c) {
  return c->n_group > 1 ? (c->n_group | (c->topk_group << 16)) : 0;
}

// The shared expert's down projection is cut along its intermediate dimension
// into parts about as long as a routed expert's, so that every tile of the down
// kernel costs the same; the combine adds the parts.
inline int32_t shared_part_k(const moesd_layer_desc *c) {
  const int32_t pk = (c->inter + 255) / 256 * 256;
  return pk;
}

Workspace carve(const moesd_layer_desc *c, int64_t T, char *base) {
  Workspace ws;
  size_t off = 0;
  auto take = [&](size_t n) {
    char *p = base ? base + off : nullptr;
    off += align256(n ? n : 1);
    return p;
  };
  const int64_t K = c->top_k, E = c->E, d = c->d, I = c->inter, S = c->shared_inter;
  ws.logits = (double *)take(sizeof(double) * T * (E + 1));
  ws.ids = (int32_t *)take(sizeof(int32_t) * T * K);
  ws.w = (float *)take(sizeof(float) * T * K);
  ws.counts = (int32_t *)take(sizeof(int32_t) * E);
  ws.offsets = (int32_t *)take(sizeof(int32_t) * (E + 1));
  ws.perm = (int32_t *)take(sizeof(int32_t) * T * K);
  ws.inv = (int32_t *)take(sizeof(int32_t) * T * K);
  ws.n_active = (int32_t *)take(sizeof(int32_t));
  ws.row_token = (int32_t *)take(sizeof(int32_t) * T * K);
  ws.plan = (int32_t *)take(sizeof(int32_t) * PLAN_WORDS(E, T * K));
  ws.part_k = shared_part_k(c);
  ws.parts = S > 0 ? (int32_t)((S + ws.part_k - 1) / ws.part_k) : 0;
  ws.gate = (float *)take(sizeof(float) * T);
  ws.h = (uint16_t *)take(sizeof(uint16_t) * T * K * I);
  ws.hs = (uint16_t *)take(sizeof(uint16_t) * T * S);
  ws.y = (float *)take(sizeof(float) * T * K * d);
  ws.ys = (float *)take(sizeof(float) * ws.parts * T * d);
  ws.tiled_partials = (float *)take(T > tiled_from(c) ? tiled_partials_bytes() : 0);
  ws.bytes = off;
  return ws;
}

}  // namespace

hipError_t current_device(int *dev, int *n_cu) {
  static std::atomic<int> cus[MOESD_MAX_DEVICES];  // zero-initialised: not yet known
  hipError_t e = hipGetDevice(dev);
  if (e != hipSuccess) return e;
  const bool cached = *dev >= 0 && *dev < MOESD_MAX_DEVICES;
  int n = cached ? cus[*dev].load(std::memory_order_relaxed) : 0;
  if (n == 0) {
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, *dev);
    if (e != hipSuccess) return e;
    if (n < 1) return hipErrorInvalidDevice;
    if (cached) cus[*dev].store(n, std::memory_order_relaxed);
  }
  *n_cu = n;
  return hipSuccess;
}

hipError_t raise_dynamic_lds_limit(LdsLimitOnce &once, int dev, const void *kernel, int bytes) {
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && ((once.done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  if (tracked) once.done.fetch_or(1ull << dev, std::memory_order_release);
  return hipSuccess;
}

extern "C" {

const char *moesd_status_string(int32_t status) {
  switch (status) {
    case MOESD_OK: return "ok";
    case MOESD_INVALID_ARG: return "invalid argument";
    case MOESD_UNSUPPORTED: return "unsupported configuration";
    case MOESD_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MOESD_HIP_ERROR: return "HIP error (see moesd_last_hip_error)";
    default: return "unknown status";
  }
}

int32_t moesd_last_hip_error(void) { return g_last_hip_error.load(); }

size_t moesd_workspace_bytes(const moesd_layer_desc *desc, int32_t T_max) {
  if (check_desc(desc) != MOESD_OK || check_T(desc, T_max) != MOESD_OK) return 0;
  return carve(desc, T_max, nullptr).bytes;
}

int32_t moesd_route(const moesd_layer_desc *desc, const void *x, const void *w_router,
                    const float *router_bias, int32_t T, int32_t *topk_ids, float *topk_w,
                    void *workspace, size_t workspace_bytes, void *stream) {
  int32_t st = check_desc(desc);
  if (st) return st;
  if ((st = check_T(desc, T))) return st;
  if (T == 0) return MOESD_OK;
  if (!x || !w_router || !topk_ids || !topk_w || !workspace) return MOESD_INVALID_ARG;
  if (((uintptr_t)workspace & 255) != 0) return MOESD_INVALID_ARG;
  Workspace ws = carve(desc, T, (char *)workspace);
  if (workspace_bytes < ws.bytes) return MOESD_WORKSPACE_TOO_SMALL;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = launch_router_logits((const uint16_t *)x, (const uint16_t *)w_router, router_bias,
                                      nullptr, T, desc->d, desc->E, ws.logits, s);
  if (e != hipSuccess) return hip_fail(e);
  e = launch_topk(ws.logits, T, desc->E, desc->top_k, desc->score_func, desc->renormalize,
                  desc->routed_scale, groups_of(desc), 0, topk_ids, topk_w, nullptr, s);
  if (e != hipSuccess) return hip_fail(e);
  return MOESD_OK;
}

int32_t moesd_permute(int32_t E, int32_t K, int32_t T, const int32_t *topk_ids, int32_t *counts,
                      int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *n_active,
                      void *stream) {
  if (E < 1 || K < 1 || K > E || T < 0) return MOESD_INVALID_ARG;
  if ((int64_t)T * K >= ((int64_t)1 << 31)) return MOESD_INVALID_ARG;
  if (E > MOESD_MAX_E || K > MOESD_MAX_K) return MOESD_UNSUPPORTED;
  if (!counts || !offsets || !n_active) return MOESD_INVALID_ARG;
  if (T > 0 && (!topk_ids || !perm || !inv_perm)) return MOESD_INVALID_ARG;
  hipError_t e = launch_permute(topk_ids, (int64_t)T * K, E, K, counts, offsets, perm, inv_perm,
                                n_active, nullptr, nullptr, 0, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  return MOESD_OK;
}

}  // extern "C"

namespace {

// Everything that can be checked without the runtime, in the order the header documents.
// need_bytes: the scratch the call needs (0 for T == 0).
int32_t check_forward(const moesd_layer_desc *desc, const moesd_weights *wt, const void *x, int32_t T,
                      const void *out, size_t *need_bytes) {
  int32_t st = check_desc(desc);
  if (st) return st;
  if ((st = check_T(desc, T))) return st;
  if (!wt) return MOESD_INVALID_ARG;
  const bool has_shared = desc->shared_inter > 0;
  if (!wt->w_router || !wt->w_gate || !wt->w_up || !wt->w_down) return MOESD_INVALID_ARG;
  if (has_shared && (!wt->ws_gate || !wt->ws_up || !wt->ws_down)) return MOESD_INVALID_ARG;
  if (has_shared && desc->shared_gate && !wt->w_shared_gate) return MOESD_INVALID_ARG;
  if (desc->weight_format == MOESD_WEIGHTS_FP8_E4M3) {
    if (!wt->w_gate_scale || !wt->w_up_scale || !wt->w_down_scale) return MOESD_INVALID_ARG;
    if (has_shared && (!wt->ws_gate_scale || !wt->ws_up_scale || !wt->ws_down_scale)) return MOESD_INVALID_ARG;
  }
  *need_bytes = 0;
  if (T == 0) return MOESD_OK;
  if (!x || !out) return MOESD_INVALID_ARG;
  *need_bytes = carve(desc, T, nullptr).bytes;
  return MOESD_OK;
}

// The launches of one forward; every argument has been checked, `workspace` is 256-byte aligned and
// large enough.  From here on only the runtime can fail.
int32_t run_forward(const moesd_layer_desc *desc, const moesd_weights *wt, const void *x, int32_t T,
                    void *out, float *out_f32, void *workspace, int32_t *topk_ids, float *topk_w,
                    int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                    int32_t *n_active, void *stream, void *const *events) {
  const bool has_shared = desc->shared_inter > 0;
  hipStream_t s = (hipStream_t)stream;
  hipError_t e;
  if (T == 0) {
    // nothing to compute; keep the counting outputs well defined if asked for
    if (counts && offsets && n_active) {
      e = launch_permute(nullptr, 0, desc->E, desc->top_k, counts, offsets, nullptr, nullptr,
                         n_active, nullptr, nullptr, 0, s);
      if (e != hipSuccess) return hip_fail(e);
    }
    return MOESD_OK;
  }
  Workspace ws = carve(desc, T, (char *)workspace);
  int dev = 0, n_cu = 0;
  if ((e = current_device(&dev, &n_cu)) != hipSuccess) return hip_fail(e);

  int32_t *ids = topk_ids ? topk_ids : ws.ids;
  float *w = topk_w ? topk_w : ws.w;
  int32_t *cnt = counts ? counts : ws.counts;
  int32_t *off = offsets ? offsets : ws.offsets;
  int32_t *pm = perm ? perm : ws.perm;
  int32_t *iv = inv_perm ? inv_perm : ws.inv;
  int32_t *na = n_active ? n_active : ws.n_active;
  const bool gated = has_shared && desc->shared_gate;

#define MOESD_EVENT(i)                                             \
  if (events) {                                                    \
    e = hipEventRecord((hipEvent_t)events[i], s);                  \
    if (e != hipSuccess) return hip_fail(e);                       \
  }
#define MOESD_TRY(call)                                            \
  e = (call);                                                      \
  if (e != hipSuccess) return hip_fail(e);

  MOESD_EVENT(0)
  MOESD_TRY(launch_router_logits((const uint16_t *)x, (const uint16_t *)wt->w_router,
                                 wt->router_bias, gated ? (const uint16_t *)wt->w_shared_gate : nullptr,
                                 T, desc->d, desc->E, ws.logits, s))
  const bool fp8 = desc->weight_format == MOESD_WEIGHTS_FP8_E4M3;
  const bool tiled = T > tiled_from(desc);
  if (T <= MOESD_FUSED_TOPK_MAX_T && desc->E <= 256) {
    MOESD_TRY(launch_topk_permute(ws.logits, T, desc->E, desc->top_k, desc->score_func,
                                  desc->renormalize, desc->routed_scale, groups_of(desc), gated ? 1 : 0, ids, w,
                                  ws.gate, cnt, off, pm, iv, na, ws.row_token, ws.plan, 0, s))
  } else {
    MOESD_TRY(launch_topk(ws.logits, T, desc->E, desc->top_k, desc->score_func, desc->renormalize,
                          desc->routed_scale, groups_of(desc), gated ? 1 : 0, ids, w, ws.gate, s))
    // the wide classes of the streaming kernels fill the chip when their tiles of the down projection
    // (128 output rows each), the shorter of the two lists, number at least one per compute unit
    const int wide_rt = (desc->d + 127) / 128;
    const int wide_fill_min = T > PLAN_BIG_MAX_ROWS ? (n_cu + wide_rt - 1) / wide_rt : 0;
    MOESD_TRY(launch_permute(ids, (int64_t)T * desc->top_k, desc->E, desc->top_k, cnt, off, pm, iv, na,
                             ws.row_token, ws.plan, wide_fill_min, s))
  }
  MOESD_EVENT(1)

  StreamArgs a;
  a.w_gate = wt->w_gate;
  a.w_up = wt->w_up;
  a.w_down = wt->w_down;
  a.ws_gate = wt->ws_gate;
  a.ws_up = wt->ws_up;
  a.ws_down = wt->ws_down;
  a.s_gate = wt->w_gate_scale;
  a.s_up = wt->w_up_scale;
  a.s_down = wt->w_down_scale;
  a.ss_gate = wt->ws_gate_scale;
  a.ss_up = wt->ws_up_scale;
  a.ss_down = wt->ws_down_scale;
  a.fp8 = fp8 ? 1 : 0;
  a.x = (const uint16_t *)x;
  a.h = ws.h;
  a.hs = ws.hs;
  a.y = ws.y;
  a.ys = ws.ys;
  a.offsets = off;
  a.row_token = ws.row_token;
  a.plan = ws.plan;
  a.part_k = ws.part_k;
  a.d = desc->d;
  a.E = desc->E;
  a.K = desc->top_k;
  a.I = desc->inter;
  a.S = desc->shared_inter;
  a.T = T;
  a.shared_stream = shared_expert_streams(T, desc->d, desc->shared_inter, ws.part_k, desc->top_k, desc->E, n_cu);
  // A shared expert that goes to the tiled kernels need not be split into k-parts: their own schedule cuts
  // contractions where that balances the chip, and every extra part costs T * d * 4 bytes written by the
  // down projection and read again by the combine.  That schedule counts every stage alike, though, and
  // a stage of a half-empty token block is cheaper than one of the shared expert's full blocks, and it
  // cuts only where there are many stages to share out: the parts go only where the routed experts'
  // blocks are many and well filled (512 rows per expert on average).
  int n_parts = ws.parts;
  if (desc->shared_inter > 0 && !a.shared_stream && (long)T * desc->top_k >= 512L * desc->E) {
    a.part_k = desc->shared_inter;
    n_parts = 1;
  }
  // experts with at most 128 rows stream (8-bit weights: at most 16); the others are tiled
  MOESD_TRY(launch_gate_up(a, s))
  if (tiled) {
    MOESD_TRY(launch_gate_up_tiled(a, ws.tiled_partials, s))
  }
  MOESD_EVENT(2)
  MOESD_TRY(launch_down(a, s))
  if (tiled) { MOESD_TRY(launch_down_tiled(a, ws.tiled_partials, s)) }
  MOESD_EVENT(3)
  MOESD_TRY(launch_combine(ws.y, ws.ys, n_parts, w, ws.gate, iv, T, desc->top_k, desc->d,
                           (uint16_t *)out, out_f32, s))
  MOESD_EVENT(4)
#undef MOESD_EVENT
#undef MOESD_TRY
  return MOESD_OK;
}

}  // namespace

// Scratch of moesd_moe_forward_static: one array per GPU, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[MOESD_STATIC_SCRATCH_BYTES];

namespace {

// The device address of `scratch` on the device the calling thread has current, looked up once per
// device ordinal (every thread that fills an entry stores the same address).
hipError_t static_scratch(void **ptr) {
  static std::atomic<void *> addr[MOESD_MAX_DEVICES];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MOESD_MAX_DEVICES) return hipErrorInvalidDevice;
  void *p = addr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || ((uintptr_t)p & 255) != 0) return hipErrorInvalidSymbol;
    addr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return hipSuccess;
}

}  // namespace

extern "C" {

int32_t moesd_moe_forward_staged(const moesd_layer_desc *desc, const moesd_weights *wt,
                                 const void *x, int32_t T, void *out, float *out_f32,
                                 void *workspace, size_t workspace_bytes, int32_t *topk_ids,
                                 float *topk_w, int32_t *counts, int32_t *offsets, int32_t *perm,
                                 int32_t *inv_perm, int32_t *n_active, void *stream,
                                 void *const *events) {
  size_t need = 0;
  int32_t st = check_forward(desc, wt, x, T, out, &need);
  if (st) return st;
  if (T > 0) {
    if (!workspace || ((uintptr_t)workspace & 255) != 0) return MOESD_INVALID_ARG;
    if (workspace_bytes < need) return MOESD_WORKSPACE_TOO_SMALL;
  }
  return run_forward(desc, wt, x, T, out, out_f32, workspace, topk_ids, topk_w, counts, offsets, perm,
                     inv_perm, n_active, stream, events);
}

int32_t moesd_moe_forward(const moesd_layer_desc *desc, const moesd_weights *weights, const void *x,
                          int32_t T, void *out, float *out_f32, void *workspace,
                          size_t workspace_bytes, int32_t *topk_ids, float *topk_w, int32_t *counts,
                          int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *n_active,
                          void *stream) {
  return moesd_moe_forward_staged(desc, weights, x, T, out, out_f32, workspace, workspace_bytes,
                                  topk_ids, topk_w, counts, offsets, perm, inv_perm, n_active,
                                  stream, nullptr);
}

int32_t moesd_moe_forward_static(const moesd_layer_desc *desc, const moesd_weights *weights,
                                 const void *x, int32_t T, void *out, float *out_f32,
                                 int32_t *topk_ids, float *topk_w, int32_t *counts, int32_t *offsets,
                                 int32_t *perm, int32_t *inv_perm, int32_t *n_active, void *stream) {
  size_t need = 0;
  int32_t st = check_forward(desc, weights, x, T, out, &need);
  if (st) return st;
  if (need > (size_t)MOESD_STATIC_SCRATCH_BYTES) return MOESD_WORKSPACE_TOO_SMALL;
  void *ws = nullptr;
  if (T > 0) {
    hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return hip_fail(e);
  }
  return run_forward(desc, weights, x, T, out, out_f32, ws, topk_ids, topk_w, counts, offsets, perm,
                     inv_perm, n_active, stream, nullptr);
}

}  // extern "C"
