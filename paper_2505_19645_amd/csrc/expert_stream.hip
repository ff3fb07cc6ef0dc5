// Expert FFN: persistent weight-streaming kernels (gate/up + SwiGLU, and down).
//
// While an expert sees few tokens the layer is bound by loading the activated
// experts' parameters (the k2*N term of the paper's Sec. 3.3 forward-time model;
// Sec. 3.2 shows that sparser models stay in this regime for longer).  These
// kernels are therefore built around the weight stream, not around the MFMA:
//
//  * One persistent workgroup per compute unit.  All tiles of a launch are laid
//    on one line, weighted by their cost, and every workgroup takes an equal,
//    contiguous share of that line.  A workgroup therefore reads long
//    contiguous runs of weight rows and all workgroups finish together.
//  * A tile is 32 weight rows (16 of w_gate + the same 16 of w_up, or 32 rows of
//    w_down) against one block of token rows of one expert: up to 16 rows
//    ("small" tile) or up to 64 rows ("big" tile).
//  * The contraction dimension is cut into 256-element blocks.  A block is
//    fetched with global_load_lds_dwordx4 into 24 KB ring slots: every wave
//    instruction moves two 512-byte row pieces, contiguous in HBM, straight
//    into LDS without touching a register; the weights carry the non-temporal
//    hint (each byte is read exactly once).  A small tile's block fills one
//    slot (16 KB of weights + 8 KB of tokens), a big tile's block two (the
//    second holds token rows 16..63).  Every slot is exactly six loads per
//    wave, so the hand-written s_waitcnt counts are compile-time constants.
//  * Loads are issued and awaited by hand (s_waitcnt vmcnt, one s_barrier per
//    slot): the compiler sees no vector memory load in the loop, so it cannot
//    serialise the prefetch, which runs four slots ahead across tile borders.
//  * MFMA operands come from LDS.  The 16-byte pieces of a row are stored
//    XOR-swizzled by (row & 7), which keeps the operand reads free of bank
//    conflicts while the DMA writes stay linear.
//  * Small tiles: the four waves split the eight 32-element MFMA steps of a
//    block and add their partial 16x16 tiles through LDS in a fixed order.
//    Big tiles: wave w owns token rows 16w..16w+15 and needs no reduction.
//    Either way results do not depend on scheduling.
//
// MFMA operand use (v_mfma_f32_16x16x32_bf16): lane l = 16*q + r supplies 8
// consecutive contraction elements (piece 4*s + q of step s) of weight row r
// as A and of token row r as B; it receives, for token r, output features
// 4*q .. 4*q+3.
#include "common.h"

#define KB 256             // contraction elements per block
#define ROW_BYTES 512      // KB * 2
#define A_BYTES 16384      // 2 operand halves x 16 rows x 512 B
#define SLOT_BYTES 24576   // A_BYTES + 16 token rows
#define RING 6             // slots in the ring
#define AHEAD 4            // slots in flight
#define LW 6               // loads per wave per slot
#define RED_BYTES 8192     // 4 waves x 2 halves x 256 floats
#define SMALL_M 16
#define BIG_TB 64
#define STREAM_LDS_BYTES (RING * SLOT_BYTES + RED_BYTES)

enum { MODE_GATE_UP = 0, MODE_DOWN = 1 };

// ---- hand-issued memory operations --------------------------------------------
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(g), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void dma16_stream(const void *g, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
               :: "v"(g), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// The lookup tables are separate __restrict__ kernel parameters so that the
// compiler can prove them unclobbered and read them through the scalar unit: a
// vector load here would make it wait for the whole prefetch queue.
struct Tables {
  const int32_t *__restrict__ plan;
  const int32_t *__restrict__ offsets;
  const int32_t *__restrict__ row_token;
};

// ---- the tile line ----------------------------------------------------------------
// segment 0: shared expert, segment 1: big routed entries, segment 2: small routed
struct Line {
  int n[3];      // tiles per segment
  int cost[3];   // cost per tile, in quarter slot-times
  int tiles_r;   // row tiles per routed expert
  int tiles_s;   // row tiles of the shared expert
  int parts;     // k-parts of the shared down projection (1 for gate/up)
  bool shared_big;
};

__device__ __forceinline__ long line_cost(const Line &L) {
  return (long)L.n[0] * L.cost[0] + (long)L.n[1] * L.cost[1] + (long)L.n[2] * L.cost[2];
}

// first tile whose start cost is >= x
__device__ __forceinline__ int tile_at(const Line &L, long x) {
  int base = 0;
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const long span = (long)L.n[s] * L.cost[s];
    if (x <= span) return base + (L.cost[s] ? (int)((x + L.cost[s] - 1) / L.cost[s]) : 0);
    x -= span;
    base += L.n[s];
  }
  return base;
}

// One (group, token block): everything that is constant over its row tiles.
struct Entry {
  const uint16_t *a0, *a1;  // row 0 of the two operand halves at this entry's k origin
  long a_stride;
  int n_rows;               // rows of the weight matrix (for clamping the last tile)
  const uint16_t *b;        // token-row matrix at this entry's k origin
  long b_stride;
  bool use_map;             // token rows go through row_token
  int row0, m;              // first token row, number of token rows (1..64)
  int klen, nkb;
  bool big;
  void *out;
  int out_n;
  int tiles;                // row tiles in this entry
  int first_tile;           // line index of its row tile 0
};

template <int MODE>
__device__ __forceinline__ Entry load_entry(const StreamArgs &a, const Tables &tb_, const Line &L, int tile) {
  Entry en;
  if (tile < L.n[0]) {  // shared expert
    const int per = L.tiles_s;
    const int blk = tile / per;           // gate/up: token block; down: (token block, part)
    const int part = (MODE == MODE_DOWN) ? blk % L.parts : 0;
    const int tbk = (MODE == MODE_DOWN) ? blk / L.parts : blk;
    const int rows = L.shared_big ? BIG_TB : SMALL_M;
    en.big = L.shared_big;
    en.use_map = false;
    en.row0 = tbk * rows;
    en.m = min(a.T - en.row0, rows);
    en.tiles = per;
    en.first_tile = blk * per;
    if (MODE == MODE_GATE_UP) {
      en.a0 = a.ws_gate;
      en.a1 = a.ws_up;
      en.a_stride = a.d;
      en.n_rows = a.S;
      en.b = a.x;
      en.b_stride = a.d;
      en.klen = a.d;
      en.out = a.hs;
      en.out_n = a.S;
    } else {
      const int k0 = part * a.part_k;
      en.a0 = a.ws_down + k0;
      en.a1 = en.a0 + (size_t)16 * a.S;
      en.a_stride = a.S;
      en.n_rows = a.d;
      en.b = a.hs + k0;
      en.b_stride = a.S;
      en.klen = min(a.part_k, a.S - k0);
      en.out = a.ys + (size_t)part * a.T * a.d;
      en.out_n = a.d;
    }
  } else {
    int j = tile - L.n[0];
    int e, tbk = 0;
    en.big = j < L.n[1];
    if (en.big) {
      const int entry = j / L.tiles_r;
      e = tb_.plan[PLAN_HDR + a.E + 2 * entry];
      tbk = tb_.plan[PLAN_HDR + a.E + 2 * entry + 1];
      en.first_tile = L.n[0] + entry * L.tiles_r;
    } else {
      j -= L.n[1];
      const int entry = j / L.tiles_r;
      e = tb_.plan[PLAN_HDR + entry];
      en.first_tile = L.n[0] + L.n[1] + entry * L.tiles_r;
    }
    const int beg = tb_.offsets[e], end = tb_.offsets[e + 1];
    const int rows = en.big ? BIG_TB : SMALL_M;
    en.row0 = beg + tbk * rows;
    en.m = min(end - en.row0, rows);
    en.tiles = L.tiles_r;
    if (MODE == MODE_GATE_UP) {
      en.a0 = a.w_gate + (size_t)e * a.I * a.d;
      en.a1 = a.w_up + (size_t)e * a.I * a.d;
      en.a_stride = a.d;
      en.n_rows = a.I;
      en.b = a.x;
      en.b_stride = a.d;
      en.use_map = true;
      en.klen = a.d;
      en.out = a.h;
      en.out_n = a.I;
    } else {
      en.a0 = a.w_down + (size_t)e * a.d * a.I;
      en.a1 = en.a0 + (size_t)16 * a.I;
      en.a_stride = a.I;
      en.n_rows = a.d;
      en.b = a.h;
      en.b_stride = a.I;
      en.use_map = false;
      en.klen = a.I;
      en.out = a.y;
      en.out_n = a.d;
    }
  }
  en.nkb = (en.klen + KB - 1) / KB;
  return en;
}

// rows per tile in the weight matrix: gate/up 16 (of each matrix), down 32
template <int MODE>
__device__ __forceinline__ int tile_i0(int rt) { return MODE == MODE_GATE_UP ? rt * 16 : rt * 32; }

// Per-lane source pointers of the DMA instructions this wave issues.
struct LoadPtrs {
  const uint16_t *a[4];  // weight rows of the current tile
  const uint16_t *b[8];  // token rows: [0,1] first slot, [2..7] second slot of a big block
};

template <int MODE>
__device__ __forceinline__ void setup_b(LoadPtrs &lp, const Entry &en,
                                        const int32_t *__restrict__ row_token, int wave, int lane) {
  const int half = lane >> 5, slot = lane & 31;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (i >= 2 && !en.big) break;
    // instruction -> token row pair: first slot pairs 2w, 2w+1 (rows 0..15);
    // second slot pairs 8 + 6w + (i-2) (rows 16..63)
    const int pair = (i < 2) ? wave * 2 + i : 8 + wave * 6 + (i - 2);
    const int ra = min(2 * pair, en.m - 1), rb = min(2 * pair + 1, en.m - 1);
    int ta = en.row0 + ra, tb = en.row0 + rb;
    if (en.use_map) {
      ta = row_token[ta];
      tb = row_token[tb];
    }
    const int tok = half ? tb : ta;
    const int r = 2 * pair + half;
    lp.b[i] = en.b + (size_t)tok * en.b_stride + ((slot ^ (r & 7)) << 3);
  }
}

template <int MODE>
__device__ __forceinline__ void setup_a(LoadPtrs &lp, const Entry &en, int rt, int wave, int lane) {
  const int half = lane >> 5, slot = lane & 31;
  const int i0 = tile_i0<MODE>(rt);
  // valid rows in each 16-row half of this tile (at least 1 after clamping)
  const int rv0 = min(16, en.n_rows - i0);
  const int rv1 = (MODE == MODE_GATE_UP) ? rv0 : max(1, min(16, en.n_rows - i0 - 16));
  const bool second_ok = (MODE == MODE_GATE_UP) || (en.n_rows - i0 > 16);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = wave * 4 + i;  // 0..15: half = j >> 3, row pair = j & 7
    const int r = 2 * (j & 7) + half;
    const uint16_t *base = ((j >> 3) && second_ok) ? en.a1 : en.a0;
    const int rv = (j >> 3) ? rv1 : rv0;
    lp.a[i] = base + (size_t)(i0 + min(r, rv - 1)) * en.a_stride + ((slot ^ (r & 7)) << 3);
  }
}

// Issue one slot: exactly LW loads per wave.  second = second slot of a big block.
__device__ __forceinline__ void issue_slot(const LoadPtrs &lp, int klen, int kb, bool second,
                                           uint32_t slot_base, int wave, int lane) {
  const int k0 = kb * KB;
  const bool full = k0 + KB <= klen;
  // pieces past the end of a row are pulled back inside it; their products are masked
  const int sl = lane & 31, half = lane >> 5;
  auto koff = [&](int r) -> int {
    if (full) return k0;
    const int piece = sl ^ (r & 7);
    return min(k0 + piece * 8, klen - 8) - piece * 8;
  };
  if (!second) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = wave * 4 + i;
      dma16_stream(lp.a[i] + koff(2 * (j & 7) + half), slot_base + (uint32_t)j * 1024u);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int pair = wave * 2 + i;
      dma16(lp.b[i] + koff(2 * pair + half), slot_base + A_BYTES + (uint32_t)pair * 1024u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 6; ++i) {
      const int q2 = wave * 6 + i;  // token rows 16 + 2*q2, +1
      dma16(lp.b[2 + i] + koff(2 * (8 + q2) + half), slot_base + (uint32_t)q2 * 1024u);
    }
  }
}

template <int MODE>
__global__ __launch_bounds__(256) void expert_stream_kernel(StreamArgs a,
                                                            const int32_t *__restrict__ plan,
                                                            const int32_t *__restrict__ offsets,
                                                            const int32_t *__restrict__ row_token) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const Tables tb_{plan, offsets, row_token};
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uni(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  float *red = reinterpret_cast<float *>(smem + RING * SLOT_BYTES);

  // ---- the line and this workgroup's share of it --------------------------------
  Line L;
  {
    const int n_small = plan[0], n_big = plan[1];
    const bool has_shared = a.S > 0;
    L.shared_big = a.T > SMALL_M;
    L.parts = (MODE == MODE_DOWN && has_shared) ? (a.S + a.part_k - 1) / a.part_k : 1;
    L.tiles_r = (MODE == MODE_GATE_UP) ? (a.I + 15) / 16 : (a.d + 31) / 32;
    L.tiles_s = (MODE == MODE_GATE_UP) ? (a.S + 15) / 16 : (a.d + 31) / 32;
    const int n_tb = L.shared_big ? (a.T + BIG_TB - 1) / BIG_TB : 1;
    const int nkb_r = ((MODE == MODE_GATE_UP ? a.d : a.I) + KB - 1) / KB;
    const int nkb_s = ((MODE == MODE_GATE_UP ? a.d : min(a.part_k, a.S)) + KB - 1) / KB;
    L.n[0] = has_shared ? L.tiles_s * L.parts * n_tb : 0;
    L.n[1] = n_big * L.tiles_r;
    L.n[2] = n_small * L.tiles_r;
    // measured: a big block (two slots, four times the token bytes) takes about
    // 2.25 small-block times in gate/up and 2.75 in down
    const int big_q = (MODE == MODE_GATE_UP) ? 9 : 11;
    L.cost[0] = (L.shared_big ? big_q : 4) * nkb_s;
    L.cost[1] = big_q * nkb_r;
    L.cost[2] = 4 * nkb_r;
  }
  const long C = line_cost(L);
  const int G = gridDim.x, b = blockIdx.x;
  const int t_begin = tile_at(L, C * b / G);
  const int t_end = tile_at(L, C * (b + 1) / G);
  if (t_begin >= t_end) return;

  // ---- load cursor -------------------------------------------------------------------
  int l_tile = t_begin, l_kb = 0, l_slot = 0;
  bool l_second = false;
  Entry len = load_entry<MODE>(a, tb_, L, l_tile);
  LoadPtrs lp;
  setup_b<MODE>(lp, len, tb_.row_token, wave, lane);
  setup_a<MODE>(lp, len, l_tile - len.first_tile, wave, lane);
  bool l_live = true;

  auto advance_load = [&]() {
    issue_slot(lp, len.klen, l_kb, l_second, lds0 + (uint32_t)(l_slot % RING) * SLOT_BYTES, wave, lane);
    ++l_slot;
    if (len.big && !l_second) {
      l_second = true;
      return;
    }
    l_second = false;
    if (++l_kb == len.nkb) {
      l_kb = 0;
      if (++l_tile == t_end) {
        l_live = false;
        return;
      }
      if (l_tile - len.first_tile == len.tiles) {
        len = load_entry<MODE>(a, tb_, L, l_tile);
        setup_b<MODE>(lp, len, tb_.row_token, wave, lane);
      }
      setup_a<MODE>(lp, len, l_tile - len.first_tile, wave, lane);
    }
  };

  // ---- compute cursor -----------------------------------------------------------------
  int c_tile = t_begin, c_kb = 0, c_slot = 0;
  bool c_second = false;
  Entry cen = load_entry<MODE>(a, tb_, L, c_tile);
  f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  // a finished small tile whose partial sums wait in `red` for the next barrier
  bool pend = false;
  int pend_m = 0, pend_row0 = 0, pend_i0 = 0, pend_n = 0;
  void *pend_out = nullptr;

  auto store_out = [&](void *out, int out_n, size_t orow, int i0, int fi, float s0, float s1) {
    if (MODE == MODE_GATE_UP) {
      const int i = i0 + fi;
      if (i < out_n)
        reinterpret_cast<uint16_t *>(out)[orow * out_n + i] = (uint16_t)f32_to_bf16_bits(silu_f32(s0) * s1);
    } else {
      float *y = reinterpret_cast<float *>(out);
      const int i = i0 + fi;
      if (i < out_n) y[orow * out_n + i] = s0;
      if (i + 16 < out_n) y[orow * out_n + i + 16] = s1;
    }
  };
  auto flush_pending = [&]() {  // after a barrier: add the four waves' partial tiles
    const int l2 = tid & 63, rr = tid >> 6;
    const int j = l2 & 15, fi = 4 * (l2 >> 4) + rr;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      s0 += red[(w * 2 + 0) * 256 + tid];
      s1 += red[(w * 2 + 1) * 256 + tid];
    }
    if (j < pend_m) store_out(pend_out, pend_n, (size_t)(pend_row0 + j), pend_i0, fi, s0, s1);
    pend = false;
  };

  for (int i = 0; i < AHEAD && l_live; ++i) advance_load();

  while (true) {
    // slot c_slot must have landed: at most AHEAD-1 younger slots may be pending
    if (l_slot - c_slot == AHEAD) wait_vm<(AHEAD - 1) * LW>();
    else wait_vm<0>();
    wg_barrier();
    if (l_live) advance_load();
    if (pend) flush_pending();

    const char *sb = smem + (size_t)(c_slot % RING) * SLOT_BYTES;
    const int kbase = c_kb * KB;
    bool tile_done = false;
    if (!cen.big) {
      // waves split the 8 steps
      if (kbase + KB <= cen.klen) {  // whole block: no masks, reads issued back to back
        u32x4 fa0[2], fa1[2], fb[2];
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
          const int piece = 4 * (wave * 2 + ss) + q;
          const int off = r16 * ROW_BYTES + ((piece ^ (r16 & 7)) << 4);
          fa0[ss] = *reinterpret_cast<const u32x4 *>(sb + off);
          fa1[ss] = *reinterpret_cast<const u32x4 *>(sb + 8192 + off);
          fb[ss] = *reinterpret_cast<const u32x4 *>(sb + A_BYTES + off);
        }
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
          acc0 = mfma16(fa0[ss], fb[ss], acc0);
          acc1 = mfma16(fa1[ss], fb[ss], acc1);
        }
      } else {
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {
          const int s = wave * 2 + ss;
          if (kbase + s * 32 < cen.klen) {
            const int piece = 4 * s + q;
            const int off = r16 * ROW_BYTES + ((piece ^ (r16 & 7)) << 4);
            const u32x4 fa0 = *reinterpret_cast<const u32x4 *>(sb + off);
            const u32x4 fa1 = *reinterpret_cast<const u32x4 *>(sb + 8192 + off);
            u32x4 fb = *reinterpret_cast<const u32x4 *>(sb + A_BYTES + off);
            if (kbase + piece * 8 >= cen.klen) fb = (u32x4){0u, 0u, 0u, 0u};  // ragged last step
            acc0 = mfma16(fa0, fb, acc0);
            acc1 = mfma16(fa1, fb, acc1);
          }
        }
      }
      tile_done = (c_kb == cen.nkb - 1);
      ++c_kb;
    } else if (c_second) {
      // wave w owns token rows 16w..16w+15; weights sit in the previous slot
      const char *sa = smem + (size_t)((c_slot + RING - 1) % RING) * SLOT_BYTES;
      const char *sbt = (wave == 0) ? sa + A_BYTES : sb + (size_t)(wave - 1) * 16 * ROW_BYTES;
      if (wave * 16 < cen.m) {
        if (kbase + KB <= cen.klen) {  // whole block: two groups of four steps, reads ahead of the MFMAs
#pragma unroll
          for (int g4 = 0; g4 < 2; ++g4) {
            u32x4 fa0[4], fa1[4], fb[4];
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
              const int piece = 4 * (g4 * 4 + s4) + q;
              const int off = r16 * ROW_BYTES + ((piece ^ (r16 & 7)) << 4);
              fa0[s4] = *reinterpret_cast<const u32x4 *>(sa + off);
              fa1[s4] = *reinterpret_cast<const u32x4 *>(sa + 8192 + off);
              fb[s4] = *reinterpret_cast<const u32x4 *>(sbt + off);
            }
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
              acc0 = mfma16(fa0[s4], fb[s4], acc0);
              acc1 = mfma16(fa1[s4], fb[s4], acc1);
            }
          }
        } else {
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            if (kbase + s * 32 < cen.klen) {
              const int piece = 4 * s + q;
              const int off = r16 * ROW_BYTES + ((piece ^ (r16 & 7)) << 4);
              const u32x4 fa0 = *reinterpret_cast<const u32x4 *>(sa + off);
              const u32x4 fa1 = *reinterpret_cast<const u32x4 *>(sa + 8192 + off);
              u32x4 fb = *reinterpret_cast<const u32x4 *>(sbt + off);
              if (kbase + piece * 8 >= cen.klen) fb = (u32x4){0u, 0u, 0u, 0u};
              acc0 = mfma16(fa0, fb, acc0);
              acc1 = mfma16(fa1, fb, acc1);
            }
          }
        }
      }
      tile_done = (c_kb == cen.nkb - 1);
      ++c_kb;
      c_second = false;
    } else {
      c_second = true;  // first half of a big block: nothing to compute yet
    }
    ++c_slot;

    if (tile_done) {
      const int rt = c_tile - cen.first_tile;
      const int i0 = tile_i0<MODE>(rt);
      if (cen.big) {
        // straight from the accumulators: token row 16*wave + r16, features 4q..4q+3
        const int j = wave * 16 + r16;
        if (j < cen.m) {
#pragma unroll
          for (int rr = 0; rr < 4; ++rr)
            store_out(cen.out, cen.out_n, (size_t)(cen.row0 + j), i0, 4 * q + rr, acc0[rr], acc1[rr]);
        }
      } else {
        if (cen.nkb == 1) wg_barrier();  // the previous tile's sums may still be read from `red`
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          red[(wave * 2 + 0) * 256 + rr * 64 + lane] = acc0[rr];
          red[(wave * 2 + 1) * 256 + rr * 64 + lane] = acc1[rr];
        }
        pend = true;
        pend_m = cen.m;
        pend_row0 = cen.row0;
        pend_i0 = i0;
        pend_n = cen.out_n;
        pend_out = cen.out;
      }
      acc0 = (f32x4){0.f, 0.f, 0.f, 0.f};
      acc1 = (f32x4){0.f, 0.f, 0.f, 0.f};
      c_kb = 0;
      if (++c_tile == t_end) break;
      if (c_tile - cen.first_tile == cen.tiles) cen = load_entry<MODE>(a, tb_, L, c_tile);
    }
  }
  if (pend) {
    wg_barrier();
    flush_pending();
  }
}

static hipError_t launch_stream(int mode, const StreamArgs &a, hipStream_t s) {
  static int n_cu = 0;
  static bool attr_set[2] = {false, false};
  if (n_cu == 0) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return e;
    n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  const void *fn = mode == MODE_GATE_UP ? reinterpret_cast<const void *>(expert_stream_kernel<MODE_GATE_UP>)
                                        : reinterpret_cast<const void *>(expert_stream_kernel<MODE_DOWN>);
  if (!attr_set[mode]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, STREAM_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set[mode] = true;
  }
  if (mode == MODE_GATE_UP)
    hipLaunchKernelGGL(expert_stream_kernel<MODE_GATE_UP>, dim3(n_cu), dim3(256), STREAM_LDS_BYTES, s, a,
                       a.plan, a.offsets, a.row_token);
  else
    hipLaunchKernelGGL(expert_stream_kernel<MODE_DOWN>, dim3(n_cu), dim3(256), STREAM_LDS_BYTES, s, a,
                       a.plan, a.offsets, a.row_token);
  return hipGetLastError();
}

hipError_t launch_gate_up(const StreamArgs &a, hipStream_t s) { return launch_stream(MODE_GATE_UP, a, s); }
hipError_t launch_down(const StreamArgs &a, hipStream_t s) { return launch_stream(MODE_DOWN, a, s); }
