// Expert FFN for many rows per expert: MFMA-tiled grouped GEMM through LDS.
//
// Once an expert's load T_exp passes the ridge point the layer turns from
// loading weights to computing (the k3*G(T_exp) term of the paper's Sec. 3.3
// model).  Experts (or the shared expert) with more than 128 token rows are cut
// into equal blocks of at most 256 rows and handled here: a workgroup computes a 256-token x
// 256-weight-row tile (128 w_gate rows + the same 128 w_up rows with SwiGLU
// fused, or 256 w_down rows), marching over the contraction dimension in
// 64-element stages through LDS (three weight buffers and two token buffers of
// 32 KB), with v_mfma_f32_16x16x32_bf16.
//
//  * The card runs these kernels against its power limit, not its clock limit (registers-only
//    MFMA loops on random bf16 data sustain 0.80 of the 2.5 PFLOP/s peak with the 32x32x16
//    shape and 0.91 with 16x16x32, whose accumulator traffic per flop is half), hence the
//    16x16x32 shape although it needs twice the instructions.
//  * Eight waves (two per SIMD, so one multiplies while the other waits) as
//    2 (row halves) x 4 (token quarters); a wave owns 2 x 4 16-row tiles (gate
//    and up rows 64wr..64wr+63, or two 64-row groups of w_down) x four 16-token
//    tiles (tiles wt, wt+4, wt+8, wt+12 of the block's 16) = 32 accumulator tiles; 131 flops
//    per byte brought into LDS.
//  * Operands travel global memory -> LDS by global_load_lds (no registers, no LDS store
//    instructions): every wave moves 32 rows of each operand per stage, whole 128-byte lines per
//    row, the weights two stages ahead of the multiplication and the tokens (which come from L2)
//    one.  E4M3 weights are widened to bf16 on the way and pass through registers instead.
//  * Rows are 128 bytes in LDS, their eight 16-byte pieces XOR-swizzled by
//    (row >> 1) & 7: two rows share a 256-byte bank line, so the 16 rows a
//    quarter-wave reads, and the 2 rows x 8 pieces it writes, fall into 16
//    different 16-byte bank groups.
//  * Token tiles that are all padding are neither read nor multiplied (the stage loop is a template
//    over the number of a wave's tiles that hold rows; every wave still moves its share of the
//    stages): the MFMA time of a block follows its rows in steps of 32.
//  * A stage is two steps of 32 contraction elements.  The 8 weight fragments of a step are
//    refilled in place, each right after the four MFMAs that read it, with the fragment of the
//    next step; the 4 token fragments alternate between two register sets.  One s_barrier per
//    stage, between its two steps.
//  * Persistent launch, one workgroup per CU.  Four workgroups on one XCD form a team
//    that walks runs of 4 consecutive tiles in lockstep (the token blocks of one expert
//    that share a weight tile meet in that XCD's L2).  Normally whole runs are dealt
//    round-robin.  When that would leave the busiest team more than 15 % above the mean,
//    the list of (run, stage) units is instead cut into equal contiguous shares, one per
//    team, so every CU gets the same number of stages whatever the tile count.  A tile
//    that straddles a cut is not finished here:
//    each of its workgroups writes its partial accumulators, and a small second kernel
//    adds the partials of every cut tile in k order (the same order on every run) and
//    runs the epilogue.  No atomics, no fences, nobody waits for anybody.
//
// MFMA operand use (16x16x32): lane l = 16*q + r supplies 8 consecutive
// contraction elements (piece 4*s + q of step s) of weight row r as A and of
// token row r as B; it receives, for token r, output features 4*q .. 4*q+3.
#include <type_traits>

#include "common.h"

#define TBM 256  // token rows per tile
#define TBN 256  // weight rows per tile (two halves of 128)
#define TBK 64   // contraction elements per stage
#define T_ROW_BYTES 128
#define T_A_BYTES (TBN * T_ROW_BYTES)  // 32 KB
#define T_B_BYTES (TBM * T_ROW_BYTES)  // 32 KB
// LDS: NAB weight buffers, then 2 token buffers.  bf16 weights come from HBM by LDS-DMA and get three
// buffers (two stages of lead); the tokens come from L2 and get two.  E4M3 weights pass through registers:
// two buffers.
#define T_NAB(fp8) ((fp8) ? 2 : 3)
#define T_LDS_BYTES(fp8) (T_NAB(fp8) * T_A_BYTES + 2 * T_B_BYTES)
#define T_WAVES 8
#define T_THREADS (64 * T_WAVES)
#define T_LW (4096 / T_THREADS)  // 16-byte pieces per lane per stage
#define T_LROWS (512 / T_WAVES)  // rows of one operand a loader wave fetches

enum { TMODE_GATE_UP = 0, TMODE_DOWN = 1 };

// LDS accesses done, then the workgroup barrier; deliberately no vmcnt wait: the global
// loads of the next stage stay in flight across it.  The lgkmcnt(0) wait is a builtin (not
// part of the asm) so that the compiler's wait-count bookkeeping knows about it.
__device__ __forceinline__ void t_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);  // vmcnt and expcnt unconstrained, lgkmcnt(0)
  asm volatile("s_barrier" ::: "memory");
}

// The barrier that opens a piece also waits for every vector memory operation of the wave (nothing of this
// piece is in flight yet; what remains are the previous piece's output stores and register reloads the
// compiler placed before the stage loop).  As a builtin it tells the compiler's wait-count bookkeeping that
// those reloads have landed; otherwise it puts a wait for them inside the stage loop, where, not knowing of
// the LDS-DMA loads the asm statements issue, it waits for all of those as well, every stage.
__device__ __forceinline__ void t_barrier_opening() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0), expcnt unconstrained, lgkmcnt(0)
  asm volatile("s_barrier" ::: "memory");
}

// Global memory -> LDS without passing through registers: lane l's 16 bytes land at lds_base + 16 l
// (lds_base wave-uniform, in m0).  The compiler does not track m0 across inline asm (it warns on seeing it
// in a clobber list; the clobber is what keeps any value of its own out of m0 here).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void t_dma16(const void *g, uint32_t lds_base) {
  const uint32_t b = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(b) : "memory", "m0");
}
#pragma clang diagnostic pop

// Launch-wide schedule, filled by the host.
struct TiledSched {
  int n_shared_entries;   // token blocks (x k-parts for the down projection) of the shared expert
  int rt_shared, rt_routed;  // row tiles per shared / routed entry
  int nkb_s, nkb_r;       // stages per shared / routed tile (upper bound over the region)
  float *partials;        // [2 * workgroups of the main kernel] slots of T_THREADS * 128 floats
  int n_teams;            // teams of the main kernel (its grid / 4)
};
#define T_SLOT_FLOATS (T_THREADS * 128)  // a workgroup's accumulators

// The schedule both kernels derive from the plan: units of (run, stage), two regions.
struct TiledWork {
  int n_large, n_sh_tiles, n_r_tiles;
  long runs_s, runs;  // runs of the shared region, of both
  long W_s, W;        // units of the shared region, of both
  int nkb_s, nkb_r, n_teams;
  bool cut;           // shares end inside runs (else on run boundaries)
};
// Whether the shares of the teams end inside runs.  Cutting runs costs a round trip of partial sums through
// memory and a second epilogue pass: only worth it when whole runs would leave the busiest team more than 15 %
// above the mean, or when at least half the teams would idle and every team still gets 32 stages.  (Whole
// runs are dealt region by region; the shared expert's runs are as long as its whole contraction, the routed
// experts' as theirs.)  The host evaluates the same rule over every number of routed tiles a launch can have,
// to leave out the second kernel where no launch can cut.
__host__ __device__ inline bool tiled_cuts(long runs_s, long runs, int nkb_s, int nkb_r, long nt) {
  const long W = runs_s * nkb_s + (runs - runs_s) * nkb_r;
  const long busiest = (runs_s + nt - 1) / nt * nkb_s + (runs - runs_s + nt - 1) / nt * nkb_r;
  const bool mixed = runs_s > 0 && runs > runs_s && nkb_s != nkb_r;
  return ((runs > nt || (mixed && W >= 8 * nt)) && busiest * nt * 100 > W * 115) ||
         (2 * runs <= nt && W >= 32L * nt);  // half the teams idle, and long contractions
}

__device__ __forceinline__ TiledWork tiled_work(const StreamArgs &a, const TiledSched &sc) {
  // Tiles are numbered densely per region: the shared expert's first (row tile major, its
  // token blocks adjacent), then the routed experts' (row tile major over the actual number
  // of large entries, blocks of one expert adjacent).  A run is 4 consecutive tiles.
  TiledWork w;
  w.n_large = a.plan[2];
  w.n_sh_tiles = sc.n_shared_entries * sc.rt_shared;
  w.n_r_tiles = w.n_large * sc.rt_routed;
  w.runs_s = (w.n_sh_tiles + 3) / 4;
  w.runs = w.runs_s + (w.n_r_tiles + 3) / 4;
  w.nkb_s = sc.nkb_s;
  w.nkb_r = sc.nkb_r;
  w.n_teams = sc.n_teams;
  w.W_s = w.runs_s * sc.nkb_s;
  w.W = w.W_s + (w.runs - w.runs_s) * sc.nkb_r;
  w.cut = tiled_cuts(w.runs_s, w.runs, sc.nkb_s, sc.nkb_r, w.n_teams);
  return w;
}
// when runs are cut: first unit of team g's share (g = n_teams: one past the end)
__device__ __forceinline__ long tiled_team_start(const TiledWork &w, int g) { return (w.W * g) / w.n_teams; }

// The rows of an expert (or the tokens of the shared expert) go into nb = ceil(rows / 256) blocks.  The
// multiplying work of a tile follows its rows in steps of 32 (see idle token tiles below), and the blocks of
// one expert are walked in step by a team, so an even split (in multiples of 16 rows) is taken where it
// makes every block cheaper than a whole tile: three blocks of 176 rows instead of 256 + 256 + 16.  Where
// the even blocks would be (nearly) whole tiles anyway, the blocks are 256 rows and the last one holds the
// rest.  Block blk holds rows [blk * per, min(rows, (blk + 1) * per)); (nb - 1) * per < rows either way.
__device__ __forceinline__ int tiled_block_rows(int rows) {
  const int nb = (rows + TBM - 1) / TBM;
  const int per = ((rows + nb - 1) / nb + 15) & ~15;
  return per > TBM - 32 ? TBM : per;
}

// One piece: stages [st0, st1) of one tile (stage numbers in units of the region's nkb_reg).
// FIXUP: no multiplication; the accumulators are the sum of the tile's stored pieces, and the workgroup
// finishes only token tile tq of every wave (a quarter of the tile: 32 accumulator registers instead of
// 128, so that enough waves fit a CU to hide the latency of reading the pieces).
template <int MODE, bool FIXUP, bool FP8>
__device__ __forceinline__ void tiled_piece(const StreamArgs &a, const TiledSched &sc, char *smem, bool shared_region,
                                            int tile, int st0, int st1, int nkb_reg, long run_base, int slot,
                                            int team_member, const TiledWork &w, int tq = 0) {
  constexpr int NT = FIXUP ? 1 : 4;  // token tiles held per wave
  const int n_large = w.n_large;
  // (the thread id passes through an empty asm so that what is derived from it is computed anew for every
  // piece: kept across pieces, those values were spilled, and a reload placed before the stage loop made
  // the compiler wait, inside the loop, for everything in flight)
  int tid_ = threadIdx.x;
  asm volatile("" : "+v"(tid_));
  const int tid = tid_, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wr = wave & 1, wt = wave >> 1;  // weight row half, token quarter
  const int r16 = lane & 15, q = lane >> 4;
  const int n_shared_entries = sc.n_shared_entries;
  int rt, entry;
  if (shared_region) {
    rt = tile / n_shared_entries;
    entry = tile % n_shared_entries;
  } else {
    rt = tile / n_large;
    entry = n_shared_entries + tile % n_large;
  }

  const int parts = (MODE == TMODE_DOWN && a.S > 0) ? (a.S + a.part_k - 1) / a.part_k : 1;
  // Weights: bf16 words, or (FP8) E4M3 codes that the loading waves widen to bf16 on their way into
  // LDS, with one scale per output row applied in the epilogue.
  constexpr long esz = FP8 ? 1 : 2;
  const char *A0, *A1;  // the two 128-row operand halves, row 0, at this entry's k origin
  const uint16_t *B;
  long a_stride, b_stride;  // a_stride: bytes per weight row; b_stride: elements per token row
  int n_rows, row0, m, klen, out_n;
  bool use_map;
  void *out;
  const float *sc0 = nullptr, *sc1 = nullptr;  // (FP8) row scales of the two halves' matrices
  if (entry < n_shared_entries) {
    const int part = (MODE == TMODE_DOWN) ? entry % parts : 0;
    const int blk = (MODE == TMODE_DOWN) ? entry / parts : entry;
    const int per = tiled_block_rows(a.T);
    row0 = blk * per;
    m = min(a.T - row0, per);
    use_map = false;
    if (MODE == TMODE_GATE_UP) {
      A0 = reinterpret_cast<const char *>(a.ws_gate); A1 = reinterpret_cast<const char *>(a.ws_up);
      a_stride = a.d * esz; n_rows = a.S;
      B = a.x; b_stride = a.d; klen = a.d; out = a.hs; out_n = a.S;
      sc0 = a.ss_gate; sc1 = a.ss_up;
    } else {
      const int k0 = part * a.part_k;
      a_stride = a.S * esz;
      A0 = reinterpret_cast<const char *>(a.ws_down) + k0 * esz; A1 = A0 + (size_t)128 * a_stride; n_rows = a.d;
      B = a.hs + k0; b_stride = a.S; klen = min(a.part_k, a.S - k0);
      out = a.ys + (size_t)part * a.T * a.d; out_n = a.d;
      sc0 = sc1 = a.ss_down;
    }
  } else {
    const int le = entry - n_shared_entries;
    const int base = PLAN_LARGE_OFF(a.E);
    const int e = a.plan[base + 2 * le], blk = a.plan[base + 2 * le + 1];
    const int beg = a.offsets[e], end = a.offsets[e + 1];
    const int per = tiled_block_rows(end - beg);
    row0 = beg + blk * per;
    m = min(end - row0, per);
    if (MODE == TMODE_GATE_UP) {
      A0 = reinterpret_cast<const char *>(a.w_gate) + (size_t)e * a.I * a.d * esz;
      A1 = reinterpret_cast<const char *>(a.w_up) + (size_t)e * a.I * a.d * esz;
      a_stride = a.d * esz;
      n_rows = a.I; B = a.x; b_stride = a.d; use_map = true; klen = a.d; out = a.h; out_n = a.I;
      sc0 = a.s_gate + (size_t)e * a.I; sc1 = a.s_up + (size_t)e * a.I;
    } else {
      a_stride = a.I * esz;
      A0 = reinterpret_cast<const char *>(a.w_down) + (size_t)e * a.d * a.I * esz; A1 = A0 + (size_t)128 * a_stride;
      n_rows = a.d; B = a.h; b_stride = a.I; use_map = false; klen = a.I; out = a.y; out_n = a.d;
      sc0 = sc1 = a.s_down + (size_t)e * a.d;
    }
  }
  // first output feature of this tile; gate/up: 128 features (rows i0.. of both matrices),
  // down: 256 features (rows i0.. and i0+128..)
  const int i0 = (MODE == TMODE_GATE_UP) ? rt * 128 : rt * 256;
  const int rv0 = min(128, n_rows - i0);                                               // valid rows, first half
  const int rv1 = (MODE == TMODE_GATE_UP) ? rv0 : max(1, min(128, n_rows - i0 - 128));  // second half
  const bool second_ok = (MODE == TMODE_GATE_UP) || (n_rows - i0 > 128);

  f32x4 acc[8][NT];  // [weight tile: 4 of the first half, 4 of the second][token tile]
#pragma unroll
  for (int h = 0; h < 8; ++h)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[h][t] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if constexpr (!FIXUP) {
  // ---- loader: a stage is 256 weight rows + 256 token rows x 128 bytes.  Wave w moves weight rows
  // 32w .. 32w+31 of the tile's 256 (waves 4..7: the second half) and token rows 32w .. 32w+31, 8 rows
  // per instruction: lane l row (l >> 3), LDS position (l & 7) of that row.  The data travel by LDS-DMA
  // (no registers, no LDS store instructions); the DMA writes a wave's 64 x 16 bytes linearly, so the
  // swizzle is done on the way in: position p of row r receives piece p ^ ((r >> 1) & 7).  E4M3 weights
  // cannot take that road (they are widened to bf16 on the way): their 8-byte pieces go through
  // registers, rows 16w' + 8i + (l >> 3) of each half for the wave pair.
  const int lrow = lane >> 3, pos = lane & 7;
  const bool second = wave >= T_WAVES / 2;
  const char *abase = ((second && second_ok) ? A1 : A0) + (size_t)i0 * a_stride;  // wave-uniform
  const char *bbase = reinterpret_cast<const char *>(use_map ? B : B + (size_t)row0 * b_stride);
  const int rvh = second ? rv1 : rv0;
  uint32_t offA[4], offB[4];  // this lane's rows (clamped into the valid rows), in bytes
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int hrow = 32 * (wave & 3) + 8 * i + lrow;  // row inside its half
    offA[i] = (uint32_t)min(hrow, rvh - 1) * (uint32_t)a_stride;
    const int row = min(32 * wave + 8 * i + lrow, m - 1);
    const int tr = use_map ? a.row_token[row0 + row] : row;
    offB[i] = (uint32_t)tr * (uint32_t)(b_stride * 2);
  }
  // rows 32w + 8i + lrow: (row >> 1) & 7 = (4i + (lrow >> 1)) & 7, two values by the parity of i
  const int pc0 = pos ^ ((lrow >> 1) & 7), pc1 = pos ^ ((4 + (lrow >> 1)) & 7);
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  // a piece past the end of the rows is pulled back inside (and zeroed in LDS once it has landed)
  auto k_off = [&](int s, int pc) __attribute__((always_inline)) {
    return (uint32_t)min(s * TBK + pc * 8, klen - 8);
  };
  u32x4 pre[4];  // (E4M3) this lane's weight codes of one stage on their way to LDS: 4 x 8 bytes
  constexpr int NAB = T_NAB(FP8);
  constexpr int B_BASE = NAB * T_A_BYTES;
  // instruction ii of the 4 that bring a wave's share of the weights of stage s into weight buffer ab
  auto issue_a = [&](int s, int ab, int ii) __attribute__((always_inline)) {
    const uint32_t kk = k_off(s, (ii & 1) ? pc1 : pc0);
    if constexpr (FP8) {
      const u32x2 v = *reinterpret_cast<const u32x2 *>(abase + (offA[ii] + kk));
      pre[ii][0] = v[0];
      pre[ii][1] = v[1];
    } else {
      t_dma16(abase + (offA[ii] + 2u * kk), lds0 + ab * T_A_BYTES + (32 * wave + 8 * ii) * T_ROW_BYTES);
    }
  };
  // the same for the tokens of stage s into token buffer bb
  auto issue_b = [&](int s, int bb, int ii) __attribute__((always_inline)) {
    const uint32_t kk = k_off(s, (ii & 1) ? pc1 : pc0);
    t_dma16(bbase + (offB[ii] + 2u * kk), lds0 + B_BASE + bb * T_B_BYTES + (32 * wave + 8 * ii) * T_ROW_BYTES);
  };
  // What remains to do before the barrier that publishes stage s (weights in buffer ab): (E4M3) widen and
  // store the weight pieces; wait for the DMA (all but the `later` youngest instructions, which belong to a
  // later stage); zero the weight pieces past the end of a ragged contraction.
  auto finish_stage = [&](int s, int ab, bool rag, auto later) __attribute__((always_inline)) {
    constexpr int LATER = decltype(later)::value;
    char *dst = smem + ab * T_A_BYTES + (32 * wave + lrow) * T_ROW_BYTES + (pos << 4);
    if constexpr (FP8) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t c0 = pre[i][0], c1 = pre[i][1];
        u32x4 v;
        v[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c0, 1.0f, false));
        v[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c0, 1.0f, true));
        v[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c1, 1.0f, false));
        v[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(c1, 1.0f, true));
        const int pc = (i & 1) ? pc1 : pc0;
        if (rag && s * TBK + pc * 8 >= klen) v = (u32x4){0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4 *>(dst + 8 * i * T_ROW_BYTES) = v;
      }
    }
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(FP8 ? 0 : LATER) : "memory");
    if (!FP8 && rag) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int pc = (i & 1) ? pc1 : pc0;
        if (s * TBK + pc * 8 >= klen) *reinterpret_cast<u32x4 *>(dst + 8 * i * T_ROW_BYTES) = (u32x4){0u, 0u, 0u, 0u};
      }
    }
  };

  // Operand fragments of one 32-element step: 8 weight tiles and 4 token tiles of 16 rows.
  const int key = (r16 >> 1) & 7;
  const char *pa0 = smem + (64 * wr + r16) * T_ROW_BYTES;
  const char *pb0 = smem + B_BASE + (16 * wt + r16) * T_ROW_BYTES;  // token tile t of this wave: rows 16 (wt + 4 t) ..
  auto frag_off = [&](int ks) __attribute__((always_inline)) { return ((4 * ks + q) ^ key) << 4; };
  auto read_a = [&](int ab, int ks, int h) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4 *>(pa0 + ab * T_A_BYTES + frag_off(ks) + ((h >> 2) * 128 + (h & 3) * 16) * T_ROW_BYTES);
  };
  auto read_b = [&](int bb, int ks, int t) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4 *>(pb0 + bb * T_B_BYTES + frag_off(ks) + t * 64 * T_ROW_BYTES);
  };

  const int nkb = (klen + TBK - 1) / TBK;          // this tile's own stage count (<= nkb_reg)
  const int s0 = min(st0, nkb), s1 = min(st1, nkb);  // the part of the piece that exists
  const bool ragged = (klen % TBK) != 0 && s1 == nkb;  // then the piece's last stage is zero-padded
  u32x4 fa[8], fb[2][4];
  const int n = s1 - s0;  // stages of this piece; stage s0 + j lives in weight buffer j % NAB and token buffer j & 1
  // One stage: two steps of 32 MFMAs; on entry fa and fb[0] hold the fragments of its first step.  Each
  // weight fragment is refilled in place right after the four MFMAs that read it (one weight fragment
  // against the four token fragments), the token fragments alternate between two register sets.  In the
  // shadow of the first step the fragments of the second are read; then the next stage must have landed,
  // and the barrier; in the shadow of the second step the fragments of the next stage's first step are
  // read and loads are issued into the buffers just left: the tokens of stage j + 2, then the weights of
  // stage j + NAB.  (Scheduling groups: 0x008 MFMA, 0x100 DS read.)
  auto mfma_group = [&](int h, int set, auto ntv) __attribute__((always_inline)) {
    constexpr int NTV = decltype(ntv)::value;
#pragma unroll
    for (int t = 0; t < NTV; ++t) acc[h][t] = mfma16(fa[h], fb[set][t], acc[h][t]);
  };
  auto group_shadow = [&](bool reads, bool two, auto ntv) __attribute__((always_inline)) {
    constexpr int NTV = decltype(ntv)::value;
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    if constexpr (NTV >= 2) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if (reads && two) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    if constexpr (NTV > 2) __builtin_amdgcn_sched_group_barrier(0x008, NTV - 2, 0);
    __builtin_amdgcn_sched_barrier(0);
  };
  using std::integral_constant;
  using Y = std::true_type;
  using N = std::false_type;
  // ab: weight buffer of stage j.  H1, H2, H3: stages j+1, j+2, j+3 exist in this piece.  At the wait,
  // the youngest instructions in flight are the 4 weight loads of stage j + 2 (3 weight buffers), if any.
  auto step = [&](int j, int ab, auto h1, auto h2, auto h3, auto ntv) __attribute__((always_inline)) {
    constexpr bool H1 = decltype(h1)::value, H2 = decltype(h2)::value, H3 = decltype(h3)::value;
    constexpr int NTV = decltype(ntv)::value;  // this wave's token tiles that hold rows (they are its first ones)
    constexpr bool MULT = NTV > 0;             // false: a wave whose token rows are all padding
    constexpr bool HA = NAB == 3 ? H3 : H2;       // the weights to issue in this stage exist
    const int bb = j & 1;
    const int ab1 = ab + 1 == NAB ? 0 : ab + 1;
    if constexpr (MULT) {
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        mfma_group(h, 0, ntv);
        fa[h] = read_a(ab, 1, h);
        if (h < NTV) fb[1][h] = read_b(bb, 1, h);
        group_shadow(true, h < NTV, ntv);
      }
    }
    if constexpr (H1) {
      // (stage j + 1 is the last one, the only one that can be ragged, exactly when stage j + 2 does not exist)
      finish_stage(s0 + j + 1, ab1, H2 ? false : ragged, integral_constant<int, (NAB == 3 && H2) ? 4 : 0>{});
      t_barrier();  // the next stage is in LDS for everyone; everyone has read this one
    }
    if constexpr (MULT) {
#pragma unroll
      for (int h = 0; h < 8; ++h) {
        mfma_group(h, 1, ntv);
        if constexpr (H1) {
          fa[h] = read_a(ab1, 0, h);
          if (h < NTV) fb[0][h] = read_b(bb ^ 1, 0, h);
        }
        group_shadow(H1, h < NTV, ntv);
        if (h < 4) {
          if constexpr (H2) issue_b(s0 + j + 2, bb, h);
        } else {
          if constexpr (HA) issue_a(s0 + j + NAB, ab, h - 4);
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if constexpr (H2) issue_b(s0 + j + 2, bb, i);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if constexpr (HA) issue_a(s0 + j + NAB, ab, i);
    }
  };
  // Idle token tiles.  The 16 token tiles of a block are dealt round-robin to the four token quarters (wave
  // wt holds tiles wt, wt + 4, wt + 8, wt + 12), so a block of m rows leaves every wave its first
  // ceil((ceil(m / 16) - wt) / 4) tiles; the others are padding and are neither read nor multiplied.  With the
  // usual placement of a workgroup's waves (wave i on SIMD i mod 4) the multiplying work of every SIMD then
  // follows the rows in steps of 32.  A wave without any tile only keeps moving its share of the stages and
  // keeps the barriers.
  const int n_tiles16 = (m + 15) >> 4;
  const int my_tiles = min(4, (n_tiles16 - wt + 3) >> 2);
  // the stages of a piece; the last ones are straight-line sequences chosen by how many remain, so the
  // steady state is branch-free
  auto run_stages = [&](auto mult) __attribute__((always_inline)) {
    constexpr int NTV = decltype(mult)::value;
    if constexpr (NTV > 0) {
#pragma unroll
      for (int h = 0; h < 8; ++h) fa[h] = read_a(0, 0, h);
#pragma unroll
      for (int t = 0; t < NTV; ++t) fb[0][t] = read_b(0, 0, t);
    }
    int j = 0, ab = 0;
    for (; j + 3 < n; ++j) {
      step(j, ab, Y{}, Y{}, Y{}, mult);
      ab = ab + 1 == NAB ? 0 : ab + 1;
    }
    if (j + 2 < n) {
      step(j, ab, Y{}, Y{}, N{}, mult);
      ab = ab + 1 == NAB ? 0 : ab + 1;
      ++j;
    }
    if (j + 1 < n) {
      step(j, ab, Y{}, N{}, N{}, mult);
      ab = ab + 1 == NAB ? 0 : ab + 1;
      ++j;
    }
    step(j, ab, N{}, N{}, N{}, mult);
  };
  if (!FIXUP && n > 0) {
    t_barrier_opening();  // everyone is done with the LDS of the previous piece
    // in flight before the loop: stage 0; the tokens of stage 1; the weights of stages 1 .. NAB-1
#pragma unroll
    for (int i = 0; i < 4; ++i) issue_b(s0, 0, i);
#pragma unroll
    for (int i = 0; i < 4; ++i) issue_a(s0, 0, i);
    if constexpr (FP8) finish_stage(s0, 0, ragged && n == 1, integral_constant<int, 0>{});
    if (1 < n) {
#pragma unroll
      for (int i = 0; i < 4; ++i) issue_b(s0 + 1, 1, i);
#pragma unroll
      for (int i = 0; i < 4; ++i) issue_a(s0 + 1, 1, i);
    }
    if constexpr (!FP8) {
      if (2 < n) {
#pragma unroll
        for (int i = 0; i < 4; ++i) issue_a(s0 + 2, 2, i);
        finish_stage(s0, 0, false, integral_constant<int, 12>{});
      } else if (1 < n) {
        finish_stage(s0, 0, false, integral_constant<int, 8>{});
      } else {
        finish_stage(s0, 0, ragged, integral_constant<int, 0>{});
      }
    }
    t_barrier();
    switch (my_tiles) {  // wave-uniform; every variant keeps the same barriers
      case 0: run_stages(integral_constant<int, 0>{}); break;
      case 1: run_stages(integral_constant<int, 1>{}); break;
      case 2: run_stages(integral_constant<int, 2>{}); break;
      case 3: run_stages(integral_constant<int, 3>{}); break;
      default: run_stages(integral_constant<int, 4>{}); break;
    }
  }

  // ---- a tile cut by the schedule: its pieces meet in memory, the second kernel finishes it --
  if (!(st0 == 0 && st1 == nkb_reg)) {
    f32x4 *mine = reinterpret_cast<f32x4 *>(sc.partials + (size_t)slot * T_SLOT_FLOATS);
#pragma unroll
    for (int h = 0; h < 8; ++h)
#pragma unroll
      for (int t = 0; t < NT; ++t) mine[(h * 4 + t) * T_THREADS + tid] = acc[h][t];
    return;
  }
  }  // !FIXUP
  if constexpr (FIXUP) {
    // contributors: the teams whose shares meet this run's units, in k order
    const int n_teams = w.n_teams;
    auto team_start = [&](int g) -> long { return tiled_team_start(w, g); };
    auto team_of = [&](long u) -> int {
      int g = (int)min((long)n_teams - 1, (u * n_teams) / w.W);
      while (g + 1 < n_teams && team_start(g + 1) <= u) ++g;
      while (g > 0 && team_start(g) > u) --g;
      return g;
    };
    const int g_lo = team_of(run_base), g_hi = team_of(run_base + nkb_reg - 1);
    for (int gg = g_lo; gg <= g_hi; ++gg) {
      const long ts = team_start(gg);
      if (ts == team_start(gg + 1)) continue;  // an empty share
      const int wg = ((gg / 8) * 4 + team_member) * 8 + (gg % 8);
      const int sl = 2 * wg + (ts >= run_base ? 0 : 1);  // its first piece, or its last
      const f32x4 *theirs = reinterpret_cast<const f32x4 *>(sc.partials + (size_t)sl * T_SLOT_FLOATS);
#pragma unroll
      for (int h = 0; h < 8; ++h) acc[h][0] += theirs[(h * 4 + tq) * T_THREADS + tid];
    }
  }

  // ---- epilogue: lane holds, for token 16 (wt + 4t) + r16, features 4q .. 4q+3 of every weight tile ------
  // weight tile h: half (h >> 2), rows 64wr + 16(h & 3) .. +15 of that half
#pragma unroll
  for (int tl = 0; tl < NT; ++tl) {
    const int t = FIXUP ? tq : tl;  // which of the wave's four token tiles acc[.][tl] is
    const int j = 16 * (wt + 4 * t) + r16;
    if (j < m) {
      const size_t orow = (size_t)(row0 + j);
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) {
        const int f = 64 * wr + 16 * hh + 4 * q;  // feature inside the 128 of a half
        if (MODE == TMODE_GATE_UP) {
          const int i = i0 + f;
          if (i < out_n) {
            f32x4 cg = {1.f, 1.f, 1.f, 1.f}, cu = {1.f, 1.f, 1.f, 1.f};
            if (FP8) {  // one scale per weight row = per output feature
              cg = *reinterpret_cast<const f32x4 *>(sc0 + i);
              cu = *reinterpret_cast<const f32x4 *>(sc1 + i);
            }
            uint32_t hb[4];
#pragma unroll
            for (int c = 0; c < 4; ++c)
              hb[c] = f32_to_bf16_bits(silu_f32(acc[hh][tl][c] * cg[c]) * (acc[4 + hh][tl][c] * cu[c]));
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
              f32x4 o = acc[4 * h2 + hh][tl];
              if (FP8) {
                const f32x4 cd = *reinterpret_cast<const f32x4 *>(sc0 + i);
#pragma unroll
                for (int c = 0; c < 4; ++c) o[c] *= cd[c];
              }
              *reinterpret_cast<f32x4 *>(y + orow * out_n + i) = o;
            }
          }
        }
      }
    }
  }
}

template <int MODE, bool FP8>
__global__ __launch_bounds__(T_THREADS) void expert_tiled_kernel(StreamArgs a, TiledSched sc) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  // Workgroup ids are dealt to the 8 XCDs round-robin: team g lives on XCD g % 8.
  const int xcd = blockIdx.x % 8, j = blockIdx.x / 8;
  const int team = (j / 4) * 8 + xcd, member = j % 4;
  const TiledWork w = tiled_work(a, sc);
  if (w.W == 0) return;
  if (!w.cut) {
    // Whole tiles.  The shared expert's runs (4 consecutive tiles) are dealt round-robin over
    // the teams.  The routed experts' work is the grid (entry group of 4 token blocks) x (row
    // tile); it is walked entry group by entry group and handed out 8 cells at a time to the
    // 8 teams of one XCD, so an XCD's workgroups read the same 4 token blocks (and each team
    // its own weight tile): on the Mixtral-shaped layer at T = 4096 this took the gate/up kernel's
    // L2 fill traffic from 8.8 GB to 4.7 GB per launch (1.9 GB of weights are the floor).
    // (With few large entries the groups of 4 would be mostly empty: then the routed tiles are
    // dealt as plain runs of 4 consecutive tiles too.)
    const int tl = team / 8, tpx = w.n_teams / 8;  // team within its XCD, teams per XCD
    const int eg_n = (w.n_large + 3) / 4;
    // at most 10 % of the group slots empty, and enough work that the two phases (shared, then
    // routed) starting at team 0 each cost nothing
    const bool grid = (4 * eg_n - w.n_large) * 10 <= w.n_large && w.runs > 2 * w.n_teams;
    const long sh_rounds = (w.runs_s + w.n_teams - 1) / w.n_teams;
    const long cells = (long)eg_n * sc.rt_routed;
    const long n_it = grid ? sh_rounds + ((cells + tpx - 1) / tpx + 7) / 8 : (w.runs + w.n_teams - 1) / w.n_teams;
    for (long it = 0; it < n_it; ++it) {
      bool shared_region, valid;
      int tile;
      if (!grid) {  // shared and routed runs as one list, dealt round-robin
        const long run = team + it * w.n_teams;
        shared_region = run < w.runs_s;
        tile = (int)(4 * (shared_region ? run : run - w.runs_s) + member);
        valid = run < w.runs && tile < (shared_region ? w.n_sh_tiles : w.n_r_tiles);
      } else if (it < sh_rounds) {
        const long run = team + it * w.n_teams;
        shared_region = true;
        tile = (int)(4 * run + member);
        valid = run < w.runs_s && tile < w.n_sh_tiles;
      } else {
        const long q = (xcd + 8 * (it - sh_rounds)) * tpx + tl;
        const int eg = (int)(q / sc.rt_routed), rt = (int)(q % sc.rt_routed);
        const int entry = 4 * eg + member;
        shared_region = false;
        valid = q < cells && entry < w.n_large;
        tile = rt * w.n_large + entry;
      }
      const int nkb_reg = shared_region ? sc.nkb_s : sc.nkb_r;
      if (valid) tiled_piece<MODE, false, FP8>(a, sc, smem, shared_region, tile, 0, nkb_reg, nkb_reg, 0, 0, member, w);
    }
    return;
  }
  long u = tiled_team_start(w, team);
  const long u_end = tiled_team_start(w, team + 1);
  int piece = 0;
  while (u < u_end) {
    const bool shared_region = u < w.W_s;
    const int nkb_reg = shared_region ? sc.nkb_s : sc.nkb_r;
    const long ur = shared_region ? u : u - w.W_s;
    const long run = ur / nkb_reg;
    const int st0 = (int)(ur % nkb_reg);
    const int st1 = (int)min((long)nkb_reg, st0 + (u_end - u));
    const int tile = (int)(4 * run + member);
    if (tile < (shared_region ? w.n_sh_tiles : w.n_r_tiles))
      tiled_piece<MODE, false, FP8>(a, sc, smem, shared_region, tile, st0, st1, nkb_reg, u - st0,
                               2 * (int)blockIdx.x + (piece == 0 ? 0 : 1), member, w);
    u += st1 - st0;
    ++piece;
  }
}

// Finishes the tiles the main kernel's share boundaries cut.  Workgroup (g, member, tq): if the
// boundary between teams g and g+1 is the first one inside its run, sum that run's pieces for token
// tile tq of every wave.
template <int MODE, bool FP8>
__global__ __launch_bounds__(T_THREADS) void expert_tiled_fixup_kernel(StreamArgs a, TiledSched sc) {
  const int tq = blockIdx.x & 3, g = blockIdx.x / 16, member = (blockIdx.x / 4) % 4;
  const TiledWork w = tiled_work(a, sc);
  if (w.W == 0 || !w.cut || g + 1 >= w.n_teams) return;
  const long b = tiled_team_start(w, g + 1);  // first unit of team g+1
  if (b >= w.W) return;
  const bool shared_region = b < w.W_s;
  const int nkb_reg = shared_region ? sc.nkb_s : sc.nkb_r;
  const long ur = shared_region ? b : b - w.W_s;
  const int st = (int)(ur % nkb_reg);
  if (st == 0) return;  // the boundary falls between two runs: nothing is cut
  const long run_base = b - st;
  if (tiled_team_start(w, g) > run_base) return;  // an earlier boundary inside this run does the work
  const int tile = (int)(4 * (ur / nkb_reg) + member);
  if (tile >= (shared_region ? w.n_sh_tiles : w.n_r_tiles)) return;
  tiled_piece<MODE, true, FP8>(a, sc, nullptr, shared_region, tile, 0, nkb_reg, nkb_reg, run_base, 0, member, w, tq);
}

// The persistent grid: whole teams of 4 on each of the 8 XCDs, at most TILED_MAX_WGS workgroups
// (the partial-sum space in the workspace is sized for that many, whatever the device).
#define TILED_MAX_WGS 256
static int tiled_grid_for(int n_cu) {
  const int g = (n_cu / 32) * 32;
  return g < 32 ? 32 : (g > TILED_MAX_WGS ? TILED_MAX_WGS : g);
}
// Estimated microseconds either way, from measurements on the MI355X: the streaming kernels move
// the shared expert's 3*S*d*2 bytes once per 128 tokens at about 4.8 TB/s when they share the chip
// with the routed experts' wide tiles; a tiled kernel needs ceil(tiles / CUs) rounds of a tile's
// stages, 1.5 us (gate/up) and 1.8 us (down) each, plus a fix-up launch.
int shared_expert_streams(int T, int d, int S, int part_k, int K, int E, int n_cus) {
  if (S <= 0 || T <= PLAN_BIG_MAX_ROWS) return 1;
  // routed experts with more than 128 rows on average keep the tiled kernels busy anyway: the shared
  // expert's tiles then fill gaps there instead of leaving the chip idle
  if ((long)T * K > 128L * E) return 0;
  const double n_cu = (double)tiled_grid_for(n_cus);
  const double stream_us = (double)((T + 127) / 128) * (3.0 * S * (double)d * 2.0) / 4.8e6;
  const double tb = (double)((T + TBM - 1) / TBM);
  const int parts = (S + part_k - 1) / part_k;
  const double gu_rounds = ceil(tb * ((S + 127) / 128) / n_cu), dn_rounds = ceil(tb * parts * ((d + 255) / 256) / n_cu);
  const double gu_stages = (double)((d + TBK - 1) / TBK), dn_stages = (double)(((S < part_k ? S : part_k) + TBK - 1) / TBK);
  const double tiled_us = gu_rounds * gu_stages * 1.5 + dn_rounds * dn_stages * 1.8 + 8.0;
  return stream_us < tiled_us ? 1 : 0;
}

size_t tiled_partials_bytes() { return (size_t)2 * TILED_MAX_WGS * T_SLOT_FLOATS * sizeof(float); }
static hipError_t launch_tiled(int mode, const StreamArgs &a, float *partials, hipStream_t s) {
  static LdsLimitOnce lds_once[4];
  typedef void (*kern_t)(StreamArgs, TiledSched);
  static const kern_t mains[4] = {expert_tiled_kernel<TMODE_GATE_UP, false>, expert_tiled_kernel<TMODE_DOWN, false>,
                                  expert_tiled_kernel<TMODE_GATE_UP, true>, expert_tiled_kernel<TMODE_DOWN, true>};
  static const kern_t fixups[4] = {
      expert_tiled_fixup_kernel<TMODE_GATE_UP, false>, expert_tiled_fixup_kernel<TMODE_DOWN, false>,
      expert_tiled_fixup_kernel<TMODE_GATE_UP, true>, expert_tiled_fixup_kernel<TMODE_DOWN, true>};
  const int which = (a.fp8 ? 2 : 0) + mode;
  int dev = 0, n_cu = 0;
  hipError_t e = current_device(&dev, &n_cu);
  if (e != hipSuccess) return e;
  e = raise_dynamic_lds_limit(lds_once[which], dev, reinterpret_cast<const void *>(mains[which]), T_LDS_BYTES(a.fp8));
  if (e != hipSuccess) return e;
  // (row offsets are kept as 32-bit byte counts inside the kernel: T * d * 2 < 2^32, checked by the caller,
  // which also decides whether these kernels have anything to do at this T)
  const int parts = (mode == TMODE_DOWN && a.S > 0) ? (a.S + a.part_k - 1) / a.part_k : 1;
  TiledSched sc;
  sc.n_shared_entries = (a.S > 0 && !a.shared_stream) ? ((a.T + TBM - 1) / TBM) * parts : 0;
  if (mode == TMODE_GATE_UP) {
    sc.rt_shared = (a.S + 127) / 128;
    sc.rt_routed = (a.I + 127) / 128;
    sc.nkb_s = sc.nkb_r = (a.d + TBK - 1) / TBK;
  } else {
    sc.rt_shared = sc.rt_routed = (a.d + 255) / 256;
    sc.nkb_s = a.S > 0 ? ((a.S < a.part_k ? a.S : a.part_k) + TBK - 1) / TBK : 1;
    sc.nkb_r = (a.I + TBK - 1) / TBK;
  }
  sc.partials = partials;
  const unsigned grid = (unsigned)tiled_grid_for(n_cu);
  sc.n_teams = (int)grid / 4;
  hipLaunchKernelGGL(mains[which], dim3(grid), dim3(T_THREADS), T_LDS_BYTES(a.fp8), s, a, sc);
  // The second kernel only where some launch of this shape and size can cut.  The plan is on the device; what
  // the host knows is a bound: an entry is an expert with more than 64 rows (fewer than T*K/64 of them, at
  // most E) or one more 256-row block of one (fewer than T*K/256 in all).
  const long tk = (long)a.T * a.K;
  const long max_large = tk / 256 + (tk / 65 < a.E ? tk / 65 : a.E);
  const long runs_s = ((long)sc.n_shared_entries * sc.rt_shared + 3) / 4;
  bool may_cut = false;
  for (long n_large = 0; n_large <= max_large && !may_cut; ++n_large)
    may_cut = tiled_cuts(runs_s, runs_s + (n_large * sc.rt_routed + 3) / 4, sc.nkb_s, sc.nkb_r, sc.n_teams);
  if (may_cut) hipLaunchKernelGGL(fixups[which], dim3(4 * grid), dim3(T_THREADS), 0, s, a, sc);
  return hipGetLastError();
}

hipError_t launch_gate_up_tiled(const StreamArgs &a, float *partials, hipStream_t s) {
  return launch_tiled(TMODE_GATE_UP, a, partials, s);
}
hipError_t launch_down_tiled(const StreamArgs &a, float *partials, hipStream_t s) {
  return launch_tiled(TMODE_DOWN, a, partials, s);
}
