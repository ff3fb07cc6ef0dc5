// Expert FFN for many rows per expert: MFMA-tiled grouped GEMM through LDS.
//
// Once an expert's load T_exp passes the ridge point the layer turns from
// loading weights to computing (the k3*G(T_exp) term of the paper's Sec. 3.3
// model).  Experts (or the shared expert) with more than 128 token rows are cut
// into blocks of 256 rows and handled here: a workgroup computes a 256-token x
// 256-weight-row tile (128 w_gate rows + the same 128 w_up rows with SwiGLU
// fused, or 256 w_down rows), marching over the contraction dimension in
// 64-element stages through two LDS buffers, with v_mfma_f32_32x32x16_bf16.
//
//  * Eight waves (two per SIMD, so one multiplies while the other waits) as
//    2 (row halves) x 4 (token quarters); a wave owns 2 x 2 32-row tiles (gate
//    and up rows 64wr..64wr+63, or two 64-row groups of w_down) x two 32-token
//    tiles = 8 accumulator tiles; 131 flops per byte brought into LDS.
//  * Operands travel global memory -> registers -> LDS: every lane fetches eight
//    16-byte pieces of a stage (whole 128-byte lines per row) one stage ahead of
//    the multiplication and stores them when the other buffer has been read.
//    (Measured on this chip: the same traffic through global_load_lds tops out at
//    about two thirds of this path's rate, and 64-byte row pieces at less again.)
//  * Rows are 128 bytes in LDS, their eight 16-byte pieces XOR-swizzled by
//    (row >> 1) & 7: two rows share a 256-byte bank line, so the 16 rows a
//    quarter-wave reads, and the 2 rows x 8 pieces it writes, fall into 16
//    different 16-byte bank groups.
//  * The MFMA fragments of a 16-element half step are double-buffered in
//    registers: the LDS reads of the next half step run under the MFMAs of the
//    current one; one s_barrier per stage.
//  * Workgroup ids are remapped so that runs of 4 consecutive tiles (the token blocks
//    of one expert that share a weight tile) land on the same XCD and meet in its L2.
//
// MFMA operand use (32x32x16): lane l = 32*q + r supplies 8 consecutive
// contraction elements (piece 2*s + q of half step s) of weight row r as A and of
// token row r as B; it receives, for token r, output features
// 8*g + 4*q + c (g, c = 0..3) in accumulator register 4*g + c.
#include <type_traits>

#include "common.h"

#define TBM 256  // token rows per tile
#define TBN 256  // weight rows per tile (two halves of 128)
#define TBK 64   // contraction elements per stage
#define T_ROW_BYTES 128
#define T_A_BYTES (TBN * T_ROW_BYTES)  // 32 KB
#define T_B_BYTES (TBM * T_ROW_BYTES)  // 32 KB
#define T_STAGE_BYTES (T_A_BYTES + T_B_BYTES)
#define T_LW 8  // 16-byte pieces per lane per stage
#define T_THREADS 512
#define TILED_LDS_BYTES (2 * T_STAGE_BYTES)

enum { TMODE_GATE_UP = 0, TMODE_DOWN = 1 };

// LDS accesses done, then the workgroup barrier; deliberately no vmcnt wait: the global
// loads of the next stage stay in flight across it.  The lgkmcnt(0) wait is a builtin (not
// part of the asm) so that the compiler's wait-count bookkeeping knows about it.
__device__ __forceinline__ void t_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // vmcnt and expcnt unconstrained, lgkmcnt(0)
  asm volatile("s_barrier" ::: "memory");
}

__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                 c, 0, 0, 0);
}

template <int MODE>
__global__ __launch_bounds__(T_THREADS) void expert_tiled_kernel(StreamArgs a, int n_shared_entries,
                                                           int rt_shared, int rt_routed) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave & 1, wt = wave >> 1;  // wt: 0..3
  const int r32 = lane & 31, q = lane >> 5;

  // ---- which tile ---------------------------------------------------------------------
  // The tiles with work are numbered densely: first the shared expert's (row tile major,
  // its token blocks adjacent), then the routed experts' (row tile major over the actual
  // number of large entries, blocks of one expert adjacent).  Workgroup ids are dealt to
  // the 8 XCDs round-robin; the remap hands each XCD runs of 4 consecutive tile numbers
  // (blocks that share a weight tile) and deals those runs round-robin.
  const int xcd = blockIdx.x % 8, g = blockIdx.x / 8;
  const int lin = ((g / 4) * 8 + xcd) * 4 + (g % 4);
  const int n_large = a.plan[2];
  const int n_sh_tiles = n_shared_entries * rt_shared;
  int rt, entry;
  if (lin < n_sh_tiles) {
    rt = lin / n_shared_entries;
    entry = lin % n_shared_entries;
  } else {
    const int lr = lin - n_sh_tiles;
    if (n_large == 0 || lr >= n_large * rt_routed) return;
    rt = lr / n_large;
    entry = n_shared_entries + lr % n_large;
  }

  const int parts = (MODE == TMODE_DOWN && a.S > 0) ? (a.S + a.part_k - 1) / a.part_k : 1;
  const uint16_t *A0, *A1;  // the two 64-row operand halves, row 0, at this entry's k origin
  const uint16_t *B;
  long a_stride, b_stride;
  int n_rows, row0, m, klen, out_n;
  bool use_map;
  void *out;
  if (entry < n_shared_entries) {
    const int part = (MODE == TMODE_DOWN) ? entry % parts : 0;
    const int blk = (MODE == TMODE_DOWN) ? entry / parts : entry;
    row0 = blk * TBM;
    m = min(a.T - row0, TBM);
    use_map = false;
    if (MODE == TMODE_GATE_UP) {
      A0 = a.ws_gate; A1 = a.ws_up; a_stride = a.d; n_rows = a.S;
      B = a.x; b_stride = a.d; klen = a.d; out = a.hs; out_n = a.S;
    } else {
      const int k0 = part * a.part_k;
      A0 = a.ws_down + k0; A1 = A0 + (size_t)128 * a.S; a_stride = a.S; n_rows = a.d;
      B = a.hs + k0; b_stride = a.S; klen = min(a.part_k, a.S - k0);
      out = a.ys + (size_t)part * a.T * a.d; out_n = a.d;
    }
  } else {
    const int le = entry - n_shared_entries;
    const int base = PLAN_LARGE_OFF(a.E);
    const int e = a.plan[base + 2 * le], blk = a.plan[base + 2 * le + 1];
    const int beg = a.offsets[e], end = a.offsets[e + 1];
    row0 = beg + blk * TBM;
    m = min(end - row0, TBM);
    if (MODE == TMODE_GATE_UP) {
      A0 = a.w_gate + (size_t)e * a.I * a.d; A1 = a.w_up + (size_t)e * a.I * a.d; a_stride = a.d;
      n_rows = a.I; B = a.x; b_stride = a.d; use_map = true; klen = a.d; out = a.h; out_n = a.I;
    } else {
      A0 = a.w_down + (size_t)e * a.d * a.I; A1 = A0 + (size_t)128 * a.I; a_stride = a.I;
      n_rows = a.d; B = a.h; b_stride = a.I; use_map = false; klen = a.I; out = a.y; out_n = a.d;
    }
  }
  // first output feature of this tile; gate/up: 128 features (rows i0.. of both matrices),
  // down: 256 features (rows i0.. and i0+128..)
  const int i0 = (MODE == TMODE_GATE_UP) ? rt * 128 : rt * 256;
  if (i0 >= n_rows) return;
  const int rv0 = min(128, n_rows - i0);                                               // valid rows, first half
  const int rv1 = (MODE == TMODE_GATE_UP) ? rv0 : max(1, min(128, n_rows - i0 - 128));  // second half
  const bool second_ok = (MODE == TMODE_GATE_UP) || (n_rows - i0 > 128);

  // ---- loader: a stage is 512 rows x 128 bytes; wave w fetches rows 64(w&3).. of the weight
  // rows (w < 4) or of the token rows (w >= 4), instruction i rows 8i..8i+7, lane l row
  // (l >> 3), piece (l & 7)
  const int lrow = lane >> 3, piece = lane & 7;
  const bool load_b = wave >= 4;
  const int lw = wave & 3;
  const char *wbase;    // wave-uniform: first row this wave may touch, at the k origin
  uint32_t off[T_LW];   // this lane's rows (clamped into the valid rows), in bytes from wbase
  if (!load_b) {
    const bool second = lw >= 2;
    const uint16_t *base = (second && second_ok) ? A1 : A0;
    const int rv = second ? rv1 : rv0;
    wbase = reinterpret_cast<const char *>(base + (size_t)i0 * a_stride);
#pragma unroll
    for (int i = 0; i < T_LW; ++i) {
      const int hrow = 64 * (lw & 1) + 8 * i + lrow;
      off[i] = (uint32_t)min(hrow, rv - 1) * (uint32_t)(a_stride * 2);
    }
  } else {
    wbase = reinterpret_cast<const char *>(use_map ? B : B + (size_t)row0 * b_stride);
#pragma unroll
    for (int i = 0; i < T_LW; ++i) {
      const int row = min(64 * lw + 8 * i + lrow, m - 1);
      const int tr = use_map ? a.row_token[row0 + row] : row;
      off[i] = (uint32_t)tr * (uint32_t)(b_stride * 2);
    }
  }
  // this lane's eight LDS store positions (stage buffer 0)
  const int srow0 = (load_b ? TBN : 0) + 64 * lw + lrow;
  auto load_stage = [&](int s, u32x4 (&pre)[T_LW]) __attribute__((always_inline)) {
    // a piece past the end of the rows is pulled back inside (it is zeroed before the store)
    const uint32_t kk = 2u * (uint32_t)min(s * TBK + piece * 8, klen - 8);
#pragma unroll
    for (int i = 0; i < T_LW; ++i) pre[i] = *reinterpret_cast<const u32x4 *>(wbase + (off[i] + kk));
  };
  auto store_stage = [&](int s, int buf, u32x4 (&pre)[T_LW], bool ragged) __attribute__((always_inline)) {
    if (ragged && s * TBK + piece * 8 >= klen) {
#pragma unroll
      for (int i = 0; i < T_LW; ++i) pre[i] = (u32x4){0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < T_LW; ++i) {
      const int row = srow0 + 8 * i;
      *reinterpret_cast<u32x4 *>(smem + buf * T_STAGE_BYTES + row * T_ROW_BYTES + ((piece ^ ((row >> 1) & 7)) << 4)) =
          pre[i];
    }
  };

  f32x16 acc[4][2];  // [weight tile: 2 of the first half, 2 of the second][token tile]
#pragma unroll
  for (int h = 0; h < 4; ++h)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[h][t][v] = 0.f;

  // Operand fragments of one 16-element half step: 4 weight tiles and 2 token tiles.
  const int key = (r32 >> 1) & 7;
  const char *pa0 = smem + (64 * wr + r32) * T_ROW_BYTES;
  const char *pb0 = smem + T_A_BYTES + (64 * wt + r32) * T_ROW_BYTES;
  auto read_half = [&](int buf, int hs, u32x4 (&fa)[4], u32x4 (&fb)[2]) __attribute__((always_inline)) {
    const int so = buf * T_STAGE_BYTES + (((2 * hs + q) ^ key) << 4);
#pragma unroll
    for (int h = 0; h < 4; ++h)
      fa[h] = *reinterpret_cast<const u32x4 *>(pa0 + so + ((h >> 1) * 128 + (h & 1) * 32) * T_ROW_BYTES);
#pragma unroll
    for (int t = 0; t < 2; ++t) fb[t] = *reinterpret_cast<const u32x4 *>(pb0 + so + t * 32 * T_ROW_BYTES);
  };
  auto mfma_half = [&](const u32x4 (&fa)[4], const u32x4 (&fb)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
      for (int t = 0; t < 2; ++t) acc[h][t] = mfma32(fa[h], fb[t], acc[h][t]);
  };

  const int nkb = (klen + TBK - 1) / TBK;
  const bool ragged = (klen % TBK) != 0;  // then the last stage is zero-padded
  u32x4 pre[T_LW], fa0[4], fb0[2], fa1[4], fb1[2];
  load_stage(0, pre);
  store_stage(0, 0, pre, ragged && nkb == 1);
  if (nkb > 1) load_stage(1, pre);
  t_barrier();
  read_half(0, 0, fa0, fb0);
  read_half(0, 1, fa1, fb1);
  // One stage: four half steps from buffer kb & 1.  Before the third half step's MFMAs
  // retire, the prefetched registers (stage kb+1) go to the other buffer, whose last
  // readers passed the previous barrier, and the loads of stage kb+2 are issued; after the
  // barrier the first fragments of stage kb+1 are read under the last MFMAs of stage kb.
  // (The scheduling fences keep the compiler from sinking the reads below the MFMAs.)
  auto step = [&](int kb, auto has_next, auto has_next2) __attribute__((always_inline)) {
    const int buf = kb & 1;
    mfma_half(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    read_half(buf, 2, fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_half(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    read_half(buf, 3, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_half(fa0, fb0);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(has_next)::value) {
      store_stage(kb + 1, buf ^ 1, pre, ragged && !decltype(has_next2)::value);
      if constexpr (decltype(has_next2)::value) load_stage(kb + 2, pre);
      t_barrier();  // stage kb+1 is in LDS for everyone; everyone has stage kb in registers
      read_half(buf ^ 1, 0, fa0, fb0);
    }
    __builtin_amdgcn_sched_barrier(0);
    mfma_half(fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(has_next)::value) read_half(buf ^ 1, 1, fa1, fb1);
    __builtin_amdgcn_sched_barrier(0);
  };
  {
    int kb = 0;
    for (; kb + 2 < nkb; ++kb) step(kb, std::true_type{}, std::true_type{});
    if (kb + 1 < nkb) {
      step(kb, std::true_type{}, std::false_type{});
      ++kb;
    }
    step(kb, std::false_type{}, std::false_type{});
  }

  // ---- epilogue: lane holds, for token (64wt + 32t + r32), features 8g + 4q + c -------------
  // weight tile h: half (h >> 1), rows 64wr + 32(h & 1) .. +31 of that half
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = 64 * wt + 32 * t + r32;
    if (j < m) {
      const size_t orow = (size_t)(row0 + j);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int f = 64 * wr + 32 * hh + 8 * g + 4 * q;  // feature inside the 128 of a half
          if (MODE == TMODE_GATE_UP) {
            const int i = i0 + f;
            if (i < out_n) {
              uint32_t hb[4];
#pragma unroll
              for (int c = 0; c < 4; ++c)
                hb[c] = f32_to_bf16_bits(silu_f32(acc[hh][t][4 * g + c]) * acc[2 + hh][t][4 * g + c]);
              u32x2 o;
              o[0] = hb[0] | (hb[1] << 16);
              o[1] = hb[2] | (hb[3] << 16);
              *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(out) + orow * out_n + i) = o;
            }
          } else {
            float *y = reinterpret_cast<float *>(out);
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
              const int i = i0 + 128 * h2 + f;
              if (i < out_n) {
                const f32x16 &v = acc[2 * h2 + hh][t];
                f32x4 o = {v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
                *reinterpret_cast<f32x4 *>(y + orow * out_n + i) = o;
              }
            }
          }
        }
    }
  }
}

static hipError_t launch_tiled(int mode, const StreamArgs &a, hipStream_t s) {
  static bool attr_set[2] = {false, false};
  const void *fn = mode == TMODE_GATE_UP ? reinterpret_cast<const void *>(expert_tiled_kernel<TMODE_GATE_UP>)
                                         : reinterpret_cast<const void *>(expert_tiled_kernel<TMODE_DOWN>);
  if (!attr_set[mode]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, TILED_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set[mode] = true;
  }
  // row offsets are kept as 32-bit byte counts inside the kernel
  if ((unsigned long long)a.T * (unsigned long long)a.d * 2ull >= (1ull << 32)) return hipErrorInvalidValue;
  const int parts = (mode == TMODE_DOWN && a.S > 0) ? (a.S + a.part_k - 1) / a.part_k : 1;
  const int n_shared = (a.S > 0 && a.T > PLAN_BIG_MAX_ROWS) ? ((a.T + TBM - 1) / TBM) * parts : 0;
  // experts with more than 128 rows: at most T*K/129 of them, each with ceil(m/256) blocks
  const long tk = (long)a.T * a.K;
  long n_large_ub = tk / (PLAN_BIG_MAX_ROWS + 1);
  if (n_large_ub > a.E) n_large_ub = a.E;
  n_large_ub += tk / TBM;
  if (n_shared + n_large_ub == 0) return hipSuccess;
  int rt_s, rt_r;
  if (mode == TMODE_GATE_UP) {
    rt_s = (a.S + 127) / 128;
    rt_r = (a.I + 127) / 128;
  } else {
    rt_s = rt_r = (a.d + 255) / 256;
  }
  const long n_lin = (long)n_shared * rt_s + n_large_ub * rt_r;
  const long grid = ((n_lin + 31) / 32) * 32;
  if (mode == TMODE_GATE_UP)
    hipLaunchKernelGGL(expert_tiled_kernel<TMODE_GATE_UP>, dim3((unsigned)grid), dim3(T_THREADS), TILED_LDS_BYTES, s, a,
                       n_shared, rt_s, rt_r);
  else
    hipLaunchKernelGGL(expert_tiled_kernel<TMODE_DOWN>, dim3((unsigned)grid), dim3(T_THREADS), TILED_LDS_BYTES, s, a,
                       n_shared, rt_s, rt_r);
  return hipGetLastError();
}

hipError_t launch_gate_up_tiled(const StreamArgs &a, hipStream_t s) { return launch_tiled(TMODE_GATE_UP, a, s); }
hipError_t launch_down_tiled(const StreamArgs &a, hipStream_t s) { return launch_tiled(TMODE_DOWN, a, s); }
