// Token-to-expert permutation: a stable counting sort of the T*K flat slots by
// expert id, done by one workgroup with per-wave LDS histograms.
//
// counts[e] > 0 is the activation indicator X_e of the paper's Sec. 3.2 and
// n_active = sum_e X_e is its N.  Every step is integer work whose result does
// not depend on scheduling: a wave walks its contiguous segment in order, lanes
// that hold the same expert find each other with ballots, and only the lowest of
// them touches that wave's private histogram row, so ranks are deterministic.
#include "common.h"
#include "route_device.h"

#define PERM_WAVES 16
#define PERM_THREADS (PERM_WAVES * 64)
#define PERM_MAX_LDS (156 * 1024)  // dynamic LDS a launch may ask for (the kernel has a few hundred bytes of its own)

// mask of the lanes (among `valid`) whose value equals this lane's
__device__ __forceinline__ unsigned long long match_lanes(int v, int nbits, unsigned long long valid) {
  unsigned long long m = valid;
  for (int b = 0; b < nbits; ++b) {
    const bool bit = (v >> b) & 1;
    const unsigned long long bal = __ballot(bit);
    m &= bit ? bal : ~bal;
  }
  return m;
}

__device__ __forceinline__ void permute_body(
    const int32_t *ids, int64_t n, int E, int K, int nbits, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ perm, int32_t *__restrict__ inv,
    int32_t *__restrict__ n_active, int32_t *__restrict__ row_token, int32_t *__restrict__ plan,
    int wide_fill_min, int32_t *smem, bool staged) {
  int32_t *hist = smem;                     // [PERM_WAVES][E]
  int32_t *scan = smem + PERM_WAVES * E;    // [PERM_THREADS] scratch for the scan over experts
  // (staged) [n] the sorted order, collected here and written out in whole lines afterwards: scattered
  // 4-byte stores from one compute unit were most of this kernel's time
  int32_t *sorted = scan + PERM_THREADS;
  __shared__ int32_t wave_tot[5][PERM_WAVES];
  __shared__ int32_t active_tot, wide_tot, large_tot;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // contiguous segment per wave, a whole number of 64-slot steps
  int64_t seg = (n + PERM_WAVES - 1) / PERM_WAVES;
  seg = (seg + 63) / 64 * 64;
  const int64_t beg = (int64_t)wave * seg;
  const int64_t end = beg + seg < n ? beg + seg : n;

  for (int i = tid; i < PERM_WAVES * E; i += PERM_THREADS) hist[i] = 0;
  if (tid == 0) {
    active_tot = 0;
    wide_tot = 0;
    large_tot = 0;
  }
  __syncthreads();

  // pass 1: per-wave histogram
  int32_t *myhist = hist + wave * E;
  for (int64_t f0 = beg; f0 < end; f0 += 64) {
    const int64_t f = f0 + lane;
    const bool ok = f < end;
    const int e = ok ? min(max(ids[f], 0), E - 1) : 0;  // out-of-range ids are the caller's bug; stay in bounds
    const unsigned long long valid = __ballot(ok);
    const unsigned long long peers = match_lanes(e, nbits, valid);
    if (ok && (peers & ((1ull << lane) - 1ull)) == 0ull) atomicAdd(&myhist[e], __popcll(peers));
  }
  __syncthreads();

  // per expert: total, and each wave's starting rank inside the expert
  int total = 0;
  for (int e = tid; e < E; e += PERM_THREADS) {  // E <= PERM_THREADS: at most one pass
    int run = 0;
    for (int w = 0; w < PERM_WAVES; ++w) {
      const int c = hist[w * E + e];
      hist[w * E + e] = run;
      run += c;
    }
    total = run;
    counts[e] = total;
  }
  // exclusive scans over experts (tid == expert index): the totals give the
  // offsets; the others place each expert in the expert kernels' work lists
  // (1..16 rows: "small"; 17..64 and 65..128: the two wide classes of the streaming
  // kernels; more: one "large" entry per 256-row block for the MFMA-tiled kernels)
  // An expert with 65..128 rows streams its weights once through a 128-row wide tile, unless the wide
  // classes together have too few tiles to fill the chip (fewer than wide_fill_min experts with 17..128
  // rows; the streaming kernels cannot split a tile's contraction over workgroups) while the tiled
  // kernels, which can, run anyway for some expert with more rows: then it joins their list as one
  // half-empty 256-row block.
  const int v = (tid < E) ? total : 0;
  const unsigned long long wideb = __ballot(v > 16 && v <= PLAN_BIG_MAX_ROWS);
  const unsigned long long largeb = __ballot(v > PLAN_BIG_MAX_ROWS);
  if (lane == 0 && wideb) atomicAdd(&wide_tot, __popcll(wideb));
  if (lane == 0 && largeb) atomicAdd(&large_tot, __popcll(largeb));
  __syncthreads();
  const int b128_max = (large_tot > 0 && wide_tot < wide_fill_min) ? 64 : PLAN_BIG_MAX_ROWS;
  const int v_small = (v >= 1 && v <= 16) ? 1 : 0;
  const int v_b64 = (v > 16 && v <= 64) ? 1 : 0;
  const int v_b128 = (v > 64 && v <= b128_max) ? 1 : 0;
  const int v_large = (v > b128_max) ? (v + 255) / 256 : 0;
  int incl = v, incl_s = v_small, incl_b = v_b64, incl_c = v_b128, incl_l = v_large;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off, 64);
    const int os = __shfl_up(incl_s, off, 64);
    const int ob = __shfl_up(incl_b, off, 64);
    const int oc = __shfl_up(incl_c, off, 64);
    const int ol = __shfl_up(incl_l, off, 64);
    if (lane >= off) {
      incl += o;
      incl_s += os;
      incl_b += ob;
      incl_c += oc;
      incl_l += ol;
    }
  }
  if (lane == 63) {
    wave_tot[0][wave] = incl;
    wave_tot[1][wave] = incl_s;
    wave_tot[2][wave] = incl_b;
    wave_tot[3][wave] = incl_l;
    wave_tot[4][wave] = incl_c;
  }
  const unsigned long long act = __ballot(tid < E && total > 0);
  if (lane == 0 && act) atomicAdd(&active_tot, __popcll(act));
  __syncthreads();
  int wbase = 0, wbase_s = 0, wbase_b = 0, wbase_c = 0, wbase_l = 0;
  for (int w = 0; w < wave; ++w) {
    wbase += wave_tot[0][w];
    wbase_s += wave_tot[1][w];
    wbase_b += wave_tot[2][w];
    wbase_l += wave_tot[3][w];
    wbase_c += wave_tot[4][w];
  }
  const int excl = wbase + incl - v;
  if (tid < E) {
    offsets[tid] = excl;
    scan[tid] = excl;
    if (plan) {
      if (v_small) plan[PLAN_HDR + wbase_s + incl_s - 1] = tid;
      if (v_b64) plan[PLAN_BIG64_OFF(E) + wbase_b + incl_b - 1] = tid;
      if (v_b128) plan[PLAN_BIG128_OFF(E) + wbase_c + incl_c - 1] = tid;
      const int pos = wbase_l + incl_l - v_large;
      for (int b = 0; b < v_large; ++b) {
        plan[PLAN_LARGE_OFF(E) + 2 * (pos + b)] = tid;
        plan[PLAN_LARGE_OFF(E) + 2 * (pos + b) + 1] = b;
      }
    }
  }
  if (tid == 0) {
    offsets[E] = (int32_t)n;
    *n_active = active_tot;
    if (plan) {
      int ns = 0, nb = 0, nl = 0, nc = 0;
      for (int w = 0; w < PERM_WAVES; ++w) {
        ns += wave_tot[1][w];
        nb += wave_tot[2][w];
        nl += wave_tot[3][w];
        nc += wave_tot[4][w];
      }
      plan[0] = ns;
      plan[1] = nb;
      plan[2] = nl;
      plan[3] = nc;
      plan[PLAN_CTR] = 0;
      plan[PLAN_CTR + 1] = 0;
    }
  }
  __syncthreads();
  for (int i = tid; i < PERM_WAVES * E; i += PERM_THREADS) hist[i] += scan[i % E];
  __syncthreads();

  // pass 2: same walk; the group leader reserves the group's rows
  for (int64_t f0 = beg; f0 < end; f0 += 64) {
    const int64_t f = f0 + lane;
    const bool ok = f < end;
    const int e = ok ? min(max(ids[f], 0), E - 1) : 0;  // out-of-range ids are the caller's bug; stay in bounds
    const unsigned long long valid = __ballot(ok);
    const unsigned long long peers = match_lanes(e, nbits, valid);
    const unsigned long long below = peers & ((1ull << lane) - 1ull);
    int base = 0;
    if (ok && below == 0ull) base = atomicAdd(&myhist[e], __popcll(peers));
    const int leader = ok ? __ffsll((long long)peers) - 1 : 0;
    base = __shfl(base, leader, 64);
    if (ok) {
      const int p = base + __popcll(below);
      inv[f] = p;
      if (staged) {
        sorted[p] = (int32_t)f;
      } else {
        perm[p] = (int32_t)f;
        if (row_token) row_token[p] = (int32_t)(f / K);
      }
    }
  }
  if (staged) {
    __syncthreads();
    for (int64_t i = tid; i < n; i += PERM_THREADS) {
      const int32_t f = sorted[i];
      perm[i] = f;
      if (row_token) row_token[i] = f / K;
    }
  }
}

__global__ __launch_bounds__(PERM_THREADS) void permute_kernel(
    const int32_t *__restrict__ ids, int64_t n, int E, int K, int nbits,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv, int32_t *__restrict__ n_active, int32_t *__restrict__ row_token,
    int32_t *__restrict__ plan, int wide_fill_min, int staged) {
  extern __shared__ int32_t smem[];
  permute_body(ids, n, E, K, nbits, counts, offsets, perm, inv, n_active, row_token, plan, wide_fill_min, smem,
               staged != 0);
}

// Few tokens: the same workgroup first picks every token's top-K (wave w takes
// tokens w, w+16, ...) and then sorts, which saves a kernel launch.
template <int SLOTS>
__global__ __launch_bounds__(PERM_THREADS) void topk_permute_kernel(
    const double *__restrict__ logits, int T, int E, int Etot, int K, int score_func, int renorm,
    float scale, int groups, int32_t *ids, float *__restrict__ w, float *__restrict__ gate, int nbits,
    int32_t *__restrict__ counts, int32_t *__restrict__ offsets, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv, int32_t *__restrict__ n_active, int32_t *__restrict__ row_token,
    int32_t *__restrict__ plan, int wide_fill_min) {
  extern __shared__ int32_t smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t = wave; t < T; t += PERM_WAVES)
    topk_token<SLOTS>(logits, t, lane, E, Etot, K, score_func, renorm, scale, groups, ids, w, gate);
  __threadfence_block();
  __syncthreads();
  permute_body(ids, (int64_t)T * K, E, K, nbits, counts, offsets, perm, inv, n_active, row_token, plan,
               wide_fill_min, smem, false);  // (few tokens: no expert has more than 128 rows)
}

hipError_t launch_permute(const int32_t *ids, int64_t n, int E, int K, int32_t *counts,
                          int32_t *offsets, int32_t *perm, int32_t *inv, int32_t *n_active,
                          int32_t *row_token, int32_t *plan, int wide_fill_min, hipStream_t s) {
  int nbits = 1;
  while ((1 << nbits) < E) ++nbits;
  size_t smem = sizeof(int32_t) * ((size_t)PERM_WAVES * E + PERM_THREADS);
  // the sorted order is staged in LDS when it fits beside the histograms (gfx950 has 160 KB per CU)
  const int staged = n > 0 && smem + sizeof(int32_t) * (size_t)n <= PERM_MAX_LDS ? 1 : 0;
  if (staged) smem += sizeof(int32_t) * (size_t)n;
  if (smem > 48 * 1024) {  // above the default dynamic-LDS limit
    static LdsLimitOnce once;
    int dev = 0, n_cu = 0;
    hipError_t e = current_device(&dev, &n_cu);
    if (e != hipSuccess) return e;
    e = raise_dynamic_lds_limit(once, dev, reinterpret_cast<const void *>(permute_kernel), PERM_MAX_LDS);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(PERM_THREADS), smem, s, ids, n, E, K, nbits,
                     counts, offsets, perm, inv, n_active, row_token, plan, wide_fill_min, staged);
  return hipGetLastError();
}

hipError_t launch_topk_permute(const double *logits, int T, int E, int K, int score_func, int renorm,
                               float scale, int groups, int has_shared_gate, int32_t *ids, float *w,
                               float *gate, int32_t *counts, int32_t *offsets, int32_t *perm, int32_t *inv,
                               int32_t *n_active, int32_t *row_token, int32_t *plan, int wide_fill_min,
                               hipStream_t s) {
  const int Etot = E + (has_shared_gate ? 1 : 0);
  int nbits = 1;
  while ((1 << nbits) < E) ++nbits;
  const size_t smem = sizeof(int32_t) * ((size_t)PERM_WAVES * E + PERM_THREADS);
  if (E <= 64) {
    hipLaunchKernelGGL(topk_permute_kernel<1>, dim3(1), dim3(PERM_THREADS), smem, s, logits, T, E, Etot,
                       K, score_func, renorm, scale, groups, ids, w, gate, nbits, counts, offsets, perm, inv,
                       n_active, row_token, plan, wide_fill_min);
  } else if (E <= 256) {
    hipLaunchKernelGGL(topk_permute_kernel<4>, dim3(1), dim3(PERM_THREADS), smem, s, logits, T, E, Etot,
                       K, score_func, renorm, scale, groups, ids, w, gate, nbits, counts, offsets, perm, inv,
                       n_active, row_token, plan, wide_fill_min);
  } else {
    return hipErrorInvalidValue;  // callers use the two-kernel path for wider routers
  }
  return hipGetLastError();
}
