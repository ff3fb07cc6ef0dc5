// Expert FFN: persistent weight-streaming kernels (gate/up + SwiGLU, and down).
//
// While an expert sees few tokens the layer is bound by loading the activated
// experts' parameters (the k2*N term of the paper's Sec. 3.3 forward-time model;
// Sec. 3.2 shows that sparser models stay in this regime for longer).  These
// kernels are therefore built around the weight stream, not around the MFMA:
//
//  * One persistent workgroup of 8 waves per compute unit, one pair per SIMD: waves 4..7
//    only load (they issue every DMA instruction and wait for their own loads), waves 0..3
//    only multiply (LDS reads, MFMAs, epilogues).  Issuing a DMA instruction blocks while
//    the memory system's queues are full, which is most of the time here; in a wave that
//    also multiplies, the MFMAs would start only after that.  The two sides meet at one
//    s_barrier per slot: the loading waves arrive when slot k has landed, the multiplying
//    waves when they are done with slot k-1, whose ring position is then refilled.
//  * Three tile shapes, so that the token rows never cost more than the weight
//    bytes that travel with them and every expert's weights stream once:
//      small: an expert (or token block) with 1..16 rows.  32 weight rows (16 of
//             w_gate + the same 16 of w_up, or 32 rows of w_down), contraction
//             blocks of 512 elements; a block is one 48 KB slot: 32 KB of
//             weights + 16 KB of tokens.
//      wide:  17..64 rows.  128 weight rows (64 + 64, or 128 of w_down), contraction
//             blocks of 256 elements; a block is three 32 KB slots: the 64 token
//             rows, 64 rows of the first operand half, 64 of the second.
//      wide, 65..128 rows: the same with two token slots per block (four slots).
//    Experts beyond 128 rows belong to the MFMA-tiled kernel.
//  * Every slot is exactly twelve (wide: eight) global_load_lds_dwordx4 per loading wave, each
//    moving 1 KB (one 1 KB row piece, wide: two 512-byte pieces, contiguous in HBM:
//    256-byte pieces stream at three quarters of the rate, and the longer the blocks
//    the fewer steps a byte costs) straight into LDS; the weights carry the
//    non-temporal hint (each byte is read once).  So the hand-written s_waitcnt
//    counts are compile-time constants.  Loads run two slots ahead in a ring of three
//    (wide: three in a ring of four), across tile borders; the compiler sees no
//    vector memory load in the loop and cannot serialise the prefetch.
//  * Work split: wide tiles are dealt round-robin, then every workgroup gets a
//    contiguous run of small tiles sized so that all finish together.  When the line
//    of small tiles is long, that covers its first 60 % only and the rest is drawn from
//    a counter in units of a few tiles, which evens out the differences in speed
//    between workgroups that no fixed split can know.
//  * MFMA operands come from LDS.  The 16-byte pieces of a row are stored
//    XOR-swizzled by (row & 15): the 16 rows that one quarter-wave reads then
//    fall into 16 different 16-byte bank groups of the 64-bank LDS, while the DMA
//    writes stay linear.
//  * Small tiles: the four multiplying waves split the sixteen 32-element MFMA steps of a
//    block and add their partial 16x16 tiles through LDS in a fixed order.
//    Wide tiles: a wave multiplies 32 token rows, whose fragments of the whole block
//    it keeps in registers (a token slot is free as soon as it has been read), by 32
//    rows of every weight slot (64-row class: the waves form 2 x 2) or by all 64
//    (128-row class: one wave per 32 token rows); no reduction.
//    Results never depend on scheduling.
//
// MFMA operand use (v_mfma_f32_16x16x32_bf16): lane l = 16*q + r supplies 8
// consecutive contraction elements (piece 4*s + q of step s) of weight row r
// as A and of token row r as B; it receives, for token r, output features
// 4*q .. 4*q+3.
#include "common.h"
#include "stream_sched.h"

#define SLOT_BYTES 49152   // one ring slot
#define RING 3             // slots in the ring
#define AHEAD 2            // slots in flight
#define LW 12              // loads per wave per slot
#define RED_ROW 20         // floats per token row of a partial tile: 16 features + 4 of padding (bank spread)
#define RED_TILE (16 * RED_ROW)
#define RED_BYTES (8 * RED_TILE * 4)  // 4 waves x 2 halves x 16 rows
#define STREAM_LDS_BYTES (RING * SLOT_BYTES + RED_BYTES + 64)  // + the four words that carry drawn units
#define STREAM_THREADS 512  // waves 0..3 multiply, waves 4..7 load
// small tiles
#define SROW_BYTES 1024
#define A_BYTES 32768      // 2 halves x 16 rows x 1 KB
#define ROW_BYTES 512      // (wide tiles)
// wide tiles: 512-byte row pieces as well (256-byte pieces stream from HBM at about three quarters of
// the rate), three 32 KB slots per block: the 64 token rows, 64 rows of the first operand half, 64
// of the second
#define WSLOT_BYTES 32768
#define WRING 4            // every slot is consumed in the step it arrives in
#define WAHEAD 3
#define WLW 8              // loads per wave per slot
#ifndef W128_FRAG_DEPTH
#define W128_FRAG_DEPTH 2  // chunks of weight fragments in flight in the 128-row class
#endif
// The 128-row wide class comes in two widths (weight slots per block, stream_sched.h): class 3 is the one
// with WIDE_WN_MANY weight slots.
enum { CLS_W128X = 3 };
// token slots per block of a class (the small class keeps its tokens inside the one slot)
template <int CLS> struct ClsGeo {
  static constexpr bool WIDE = CLS != CLS_SMALL;
  static constexpr bool T128 = CLS == CLS_W128 || CLS == CLS_W128X;  // 128 token rows per tile
  static constexpr int NTS = T128 ? 2 : 1;
  static constexpr int WN = CLS == CLS_W128X ? WIDE_WN_MANY : WIDE_WN_FEW;  // weight slots per block
  static constexpr int WH = 32 * WN;                 // rows of each operand half in a tile (bf16)
  static constexpr int NSUB = WIDE ? NTS + WN : 1;  // slots per block
  static constexpr int ROWS = CLS == CLS_SMALL ? SMALL_M : (T128 ? W128_TB : W64_TB);
};


// ---- hand-issued memory operations --------------------------------------------
// lds_base is wave-uniform by construction; readfirstlane makes that explicit so the
// operand always lands in a scalar register.  The instruction takes its LDS address from m0,
// which the asm sets itself and names as clobbered (the compiler reserves m0 and warns about
// seeing it in a clobber list; the clobber is what keeps any value of its own out of m0 here).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void *g, uint32_t lds_base) {
  const uint32_t b = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(g), "s"(b) : "memory", "m0");
}
__device__ __forceinline__ void dma16_stream(const void *g, uint32_t lds_base) {
  const uint32_t b = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
               :: "v"(g), "s"(b) : "memory", "m0");
}
#pragma clang diagnostic pop
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Read one int32 of a lookup table through the scalar unit (read-only use of the
// scalar cache; the tables were written by an earlier kernel).  Spelled out by
// hand because a compiler-chosen vector load would count in vmcnt and make the
// compiler wait for the whole prefetch queue; the result is wave-uniform.
__device__ __forceinline__ int sload(const int32_t *p, int idx) {
  int v;
  const int off = uni(idx) * 4;
  asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p), "s"(off) : "memory");
  return v;
}

// the same for two and for four words, with one wait
__device__ __forceinline__ void sload2(const int32_t *p, int i0, int i1, int &v0, int &v1) {
  const int o0 = uni(i0) * 4, o1 = uni(i1) * 4;
  asm volatile("s_load_dword %0, %2, %3\n\ts_load_dword %1, %2, %4\n\ts_waitcnt lgkmcnt(0)"
               : "=&s"(v0), "=&s"(v1)
               : "s"(p), "s"(o0), "s"(o1)
               : "memory");
}
__device__ __forceinline__ void sload4(const int32_t *p, int i0, int i1, int i2, int i3, int &v0, int &v1,
                                       int &v2, int &v3) {
  const int o0 = uni(i0) * 4, o1 = uni(i1) * 4, o2 = uni(i2) * 4, o3 = uni(i3) * 4;
  asm volatile(
      "s_load_dword %0, %4, %5\n\ts_load_dword %1, %4, %6\n\ts_load_dword %2, %4, %7\n\t"
      "s_load_dword %3, %4, %8\n\ts_waitcnt lgkmcnt(0)"
      : "=&s"(v0), "=&s"(v1), "=&s"(v2), "=&s"(v3)
      : "s"(p), "s"(o0), "s"(o1), "s"(o2), "s"(o3)
      : "memory");
}

struct Tables {
  const int32_t *__restrict__ plan;
  const int32_t *__restrict__ offsets;
  const int32_t *__restrict__ row_token;
};

// One (group, token block): everything that is constant over its row tiles.
struct Entry {
  const char *a0, *a1;      // row 0 of the two operand halves at this entry's k origin (bytes)
  long a_stride;            // bytes per weight row
  int n_rows;               // rows of the weight matrix (for clamping the last tile)
  const uint16_t *b;        // token-row matrix at this entry's k origin
  long b_stride;
  bool use_map;             // token rows go through row_token
  int row0, m;              // first token row, number of token rows (1..128)
  int klen, nkb;            // contraction length, blocks (of KB or KBW)
  void *out;
  int out_n;
  int tiles;                // row tiles in this entry
  int first;                // id (in its class) of this entry's row tile 0
  const float *s0, *s1;     // 8-bit weights: the row scales of the two operand halves
};

template <int MODE, bool FP8>
__device__ __forceinline__ void fill_group(Entry &en, const StreamArgs &a, bool shared, int e, int part) {
  constexpr long esz = FP8 ? 1 : 2;  // bytes per weight
  if (shared) {
    en.use_map = false;
    if (MODE == MODE_GATE_UP) {
      en.a0 = reinterpret_cast<const char *>(a.ws_gate);
      en.a1 = reinterpret_cast<const char *>(a.ws_up);
      en.a_stride = a.d * esz;
      en.n_rows = a.S;
      en.b = a.x;
      en.b_stride = a.d;
      en.klen = a.d;
      en.out = a.hs;
      en.out_n = a.S;
      en.s0 = a.ss_gate;
      en.s1 = a.ss_up;
    } else {
      const int k0 = part * a.part_k;
      en.a0 = reinterpret_cast<const char *>(a.ws_down) + k0 * esz;
      en.a1 = en.a0;
      en.a_stride = a.S * esz;
      en.n_rows = a.d;
      en.b = a.hs + k0;
      en.b_stride = a.S;
      en.klen = min(a.part_k, a.S - k0);
      en.out = a.ys + (size_t)part * a.T * a.d;
      en.out_n = a.d;
      en.s0 = en.s1 = a.ss_down;
    }
  } else {
    if (MODE == MODE_GATE_UP) {
      en.a0 = reinterpret_cast<const char *>(a.w_gate) + (size_t)e * a.I * a.d * esz;
      en.a1 = reinterpret_cast<const char *>(a.w_up) + (size_t)e * a.I * a.d * esz;
      en.a_stride = a.d * esz;
      en.n_rows = a.I;
      en.b = a.x;
      en.b_stride = a.d;
      en.use_map = true;
      en.klen = a.d;
      en.out = a.h;
      en.out_n = a.I;
      en.s0 = a.s_gate + (size_t)e * a.I;
      en.s1 = a.s_up + (size_t)e * a.I;
    } else {
      en.a0 = reinterpret_cast<const char *>(a.w_down) + (size_t)e * a.d * a.I * esz;
      en.a1 = en.a0;
      en.a_stride = a.I * esz;
      en.n_rows = a.d;
      en.b = a.h;
      en.b_stride = a.I;
      en.use_map = false;
      en.klen = a.I;
      en.out = a.y;
      en.out_n = a.d;
      en.s0 = en.s1 = a.s_down + (size_t)e * a.d;
    }
  }
}

// entry that owns tile `id` of the class
template <int MODE, int CLS, bool FP8>
__device__ __forceinline__ Entry load_entry(const StreamArgs &a, const Tables &tb_, const ClassCfg &c,
                                            int id) {
  Entry en;
  constexpr bool WIDE = ClsGeo<CLS>::WIDE;
  constexpr int rows = ClsGeo<CLS>::ROWS;
  if (id < c.n_sh) {
    const int per = c.per_s;
    const int blk = id / per;  // gate/up: token block; down: (token block, part)
    const int part = (MODE == MODE_DOWN) ? blk % c.parts : 0;
    const int tbk = (MODE == MODE_DOWN) ? blk / c.parts : blk;
    en.row0 = tbk * rows;
    en.m = min(a.T - en.row0, rows);
    en.tiles = per;
    en.first = blk * per;
    fill_group<MODE, FP8>(en, a, true, 0, part);
  } else {
    const int per = c.per_r;
    const int entry = (id - c.n_sh) / per;
    // the class's list of expert ids in the plan; an expert is one block of its class
    const int list = CLS == CLS_SMALL ? PLAN_HDR : (ClsGeo<CLS>::T128 ? PLAN_BIG128_OFF(a.E) : PLAN_BIG64_OFF(a.E));
    const int e = sload(tb_.plan, list + entry);
    int beg, end;
    sload2(tb_.offsets, e, e + 1, beg, end);
    en.row0 = beg;
    en.m = min(end - beg, rows);
    en.tiles = per;
    en.first = c.n_sh + entry * per;
    fill_group<MODE, FP8>(en, a, false, e, 0);
  }
  en.nkb = WIDE ? (en.klen + KBW - 1) / KBW : (en.klen + KB - 1) / KB;
  return en;
}

// first weight row of row tile rt (small tiles: 16 + 16 or 32 rows of bf16, 32 + 32 or 64 rows of 8-bit codes)
template <int MODE, int CLS, bool FP8>
__device__ __forceinline__ int tile_i0(int rt) {
  constexpr bool WIDE = ClsGeo<CLS>::WIDE;
  constexpr int WH = ClsGeo<CLS>::WH;
  if (MODE == MODE_GATE_UP) return WIDE ? rt * (FP8 ? 2 : 1) * WH : rt * (FP8 ? 32 : 16);
  return WIDE ? rt * (FP8 ? 4 : 2) * WH : rt * (FP8 ? 64 : 32);
}

// Per-lane source pointers of the DMA instructions this wave issues.
//   small: a[0..7] weights, b[0..3] tokens (one 1 KB row per instruction)
//   wide:  b[0..8*NTS) tokens, eight per token slot; the weight rows' addresses are formed when a
//          slot is issued (i0: the tile's first weight row)
template <int CLS>
struct LoadPtrs {
  const char *a[ClsGeo<CLS>::WIDE ? 1 : 8];
  const uint16_t *b[ClsGeo<CLS>::WIDE ? 8 * ClsGeo<CLS>::NTS : 4];
  int i0;
};

template <int MODE, int CLS>
__device__ __forceinline__ void setup_b(LoadPtrs<CLS> &lp, const Entry &en,
                                        const int32_t *__restrict__ row_token, int wave, int lane) {
  if (!ClsGeo<CLS>::WIDE) {
    int tok[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) tok[i] = en.row0 + min(wave * 4 + i, en.m - 1);  // token rows of the tile
    if (en.use_map) sload4(row_token, tok[0], tok[1], tok[2], tok[3], tok[0], tok[1], tok[2], tok[3]);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = wave * 4 + i;
      lp.b[i] = en.b + (size_t)tok[i] * en.b_stride + ((lane ^ (r & 15)) << 3);
    }
  } else {
    const int half = lane >> 5, pos = lane & 31;
#pragma unroll
    for (int ts = 0; ts < ClsGeo<CLS>::NTS; ++ts) {  // token slot ts holds token rows 64 ts .. 64 ts + 63
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        const int pair = wave * 8 + i;  // rows 2*pair .. 2*pair+3 of the slot: this and the next instruction
        int t4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) t4[j] = en.row0 + min(64 * ts + 2 * pair + j, en.m - 1);
        if (en.use_map) sload4(row_token, t4[0], t4[1], t4[2], t4[3], t4[0], t4[1], t4[2], t4[3]);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int tok = half ? t4[2 * j + 1] : t4[2 * j];
          const int r = 2 * (pair + j) + half;
          lp.b[8 * ts + i + j] = en.b + (size_t)tok * en.b_stride + ((pos ^ (r & 15)) << 3);
        }
      }
    }
  }
}

template <int MODE, int CLS, bool FP8>
__device__ __forceinline__ void setup_a(LoadPtrs<CLS> &lp, const Entry &en, int rt, int wave, int lane) {
  constexpr bool WIDE = ClsGeo<CLS>::WIDE;
  const int i0 = tile_i0<MODE, CLS, FP8>(rt);
  if (!WIDE && !FP8) {
    // valid rows in each 16-row half of this tile (at least 1 after clamping)
    const int rv0 = min(16, en.n_rows - i0);
    const int rv1 = (MODE == MODE_GATE_UP) ? rv0 : max(1, min(16, en.n_rows - i0 - 16));
    const int off1 = (MODE == MODE_GATE_UP) ? 0 : ((en.n_rows - i0 > 16) ? 16 : 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = wave * 8 + i;  // 0..31: half = j >> 4, row = j & 15
      const int r = j & 15;
      const char *base = (j >> 4) ? en.a1 : en.a0;
      const int row = (j >> 4) ? i0 + off1 + min(r, rv1 - 1) : i0 + min(r, rv0 - 1);
      lp.a[i] = base + (size_t)row * en.a_stride + ((lane ^ r) << 4);
    }
  } else if (!WIDE) {
    // 8-bit codes: 64 slot rows of 512 bytes, two per instruction (lanes 0..31 row 2p, lanes 32..63 row
    // 2p + 1).  gate/up: slot rows 0..31 are w_gate rows i0.., slot rows 32..63 the same rows of w_up;
    // down: 64 consecutive rows.
    const int half = lane >> 5, pos = lane & 31;
    const int rv = min((MODE == MODE_GATE_UP) ? 32 : 64, en.n_rows - i0);  // valid rows (at least 1)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = 2 * (wave * 8 + i) + half;  // slot row 0..63
      const bool second = (MODE == MODE_GATE_UP) && r >= 32;
      const int row = i0 + min(second ? r - 32 : r, rv - 1);
      lp.a[i] = (second ? en.a1 : en.a0) + (size_t)row * en.a_stride + ((pos ^ (r & 15)) << 4);
    }
  } else {
    lp.i0 = i0;
  }
}

// Issue one slot: exactly LW loads per wave.  Pieces past the end of a row are
// pulled back inside it; their products are masked in the MFMA loop.
template <int MODE, int CLS, bool FP8>
__device__ __forceinline__ void issue_slot(const LoadPtrs<CLS> &lp, const Entry &en, int kb, int sub,
                                           uint32_t slot_base, int wave, int lane) {
  constexpr bool WIDE = ClsGeo<CLS>::WIDE;
  constexpr int NTS = ClsGeo<CLS>::NTS, WNW = ClsGeo<CLS>::WN, WHROWS = ClsGeo<CLS>::WH;
  const int klen = en.klen;
  if (!WIDE) {
    const int k0 = kb * KB;
    const bool full = k0 + KB <= klen;
    auto koff = [&](int r) __attribute__((always_inline)) -> int {
      if (full) return k0;
      const int piece = lane ^ (r & 15);
      return min(k0 + piece * 8, klen - 8) - piece * 8;
    };
    if (!FP8) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int j = wave * 8 + i;
        dma16_stream(lp.a[i] + 2 * koff(j & 15), slot_base + (uint32_t)j * 1024u);
      }
    } else {
      // 16-byte pieces of 16 codes; a piece past the end of the row is pulled back inside it
      const int pos = lane & 31, half = lane >> 5;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int pair = wave * 8 + i;
        const int piece = pos ^ ((2 * pair + half) & 15);
        const int ko = full ? k0 : min(k0 + piece * 16, klen - 16) - piece * 16;
        dma16_stream(lp.a[i] + ko, slot_base + (uint32_t)pair * 1024u);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = wave * 4 + i;
      dma16(lp.b[i] + koff(r), slot_base + A_BYTES + (uint32_t)r * 1024u);
    }
  } else {
    // sub 0 .. NTS-1: 64 token rows each; then WNW slots of 64 weight rows each (gate/up: the first
    // WNW/2 hold w_gate rows, the others the same rows of w_up; down: consecutive rows).
    // Wave w moves rows 16w .. 16w+15 of the slot, two per instruction.
    const int k0 = kb * KBW;
    const bool full = k0 + KBW <= klen;
    const int pos = lane & 31, half = lane >> 5;
    auto koff = [&](int r) __attribute__((always_inline)) -> int {
      if (full) return k0;
      const int piece = pos ^ (r & 15);
      return min(k0 + piece * 8, klen - 8) - piece * 8;
    };
    if (sub == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int pair = wave * 8 + i;
        dma16(lp.b[i] + koff(2 * pair + half), slot_base + (uint32_t)pair * 1024u);
      }
    } else if (NTS == 2 && sub == 1) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int pair = wave * 8 + i;
        dma16(lp.b[(NTS == 2 ? 8 : 0) + i] + koff(2 * pair + half), slot_base + (uint32_t)pair * 1024u);
      }
    } else {
      const int w = sub - NTS;
      const char *base = (MODE == MODE_GATE_UP && w >= WNW / 2) ? en.a1 : en.a0;
      if constexpr (!FP8) {
        const int first = (MODE == MODE_GATE_UP) ? 64 * (w % (WNW / 2)) : 64 * w;  // of the tile's rows in this matrix
        const int rv = min((MODE == MODE_GATE_UP) ? WHROWS : 2 * WHROWS, en.n_rows - lp.i0);  // valid ones
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int pair = wave * 8 + i;
          const int r = 2 * pair + half;
          const int row = lp.i0 + min(first + r, rv - 1);
          dma16_stream(base + (size_t)row * en.a_stride + 2 * (((pos ^ (r & 15)) << 3) + koff(r)),
                       slot_base + (uint32_t)pair * 1024u);
        }
      } else {
        // 8-bit codes: a weight slot is 128 rows of 256 bytes, four rows per instruction (lane l: row
        // l >> 4 of the four, LDS position l & 15 of the row, which receives the row's piece
        // (l & 15) ^ (row & 15) of 16 codes); wave w moves rows 32w .. 32w+31
        const int first = (MODE == MODE_GATE_UP) ? 128 * (w % (WNW / 2)) : 128 * w;
        const int rv = min((MODE == MODE_GATE_UP) ? 2 * WHROWS : 4 * WHROWS, en.n_rows - lp.i0);
        const int sub4 = lane >> 4, p16 = lane & 15;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int quad = wave * 8 + i;
          const int r = 4 * quad + sub4;
          const int row = lp.i0 + min(first + r, rv - 1);
          const int piece = p16 ^ (r & 15);
          const int ko = full ? k0 : min(k0 + piece * 16, klen - 16) - piece * 16;
          dma16_stream(base + (size_t)row * en.a_stride + (piece * 16 + ko), slot_base + (uint32_t)quad * 1024u);
        }
      }
    }
  }
}

template <int MODE>
__device__ __forceinline__ void store_out(void *out, int out_n, size_t orow, int i, int second_off,
                                          float s0, float s1) {
  // s0/s1: the two operand halves' results for one (token row, feature); second_off is
  // the feature distance between the halves in the down projection
  if (MODE == MODE_GATE_UP) {
    if (i < out_n)
      reinterpret_cast<uint16_t *>(out)[orow * out_n + i] = (uint16_t)f32_to_bf16_bits(silu_f32(s0) * s1);
  } else {
    float *y = reinterpret_cast<float *>(out);
    if (i < out_n) y[orow * out_n + i] = s0;
    if (i + second_off < out_n) y[orow * out_n + i + second_off] = s1;
  }
}

// the same for 4 neighbouring features i..i+3 (i and out_n are multiples of 4, so the four
// are inside the row together or not at all)
template <int MODE>
__device__ __forceinline__ void store_out4(void *out, int out_n, size_t orow, int i, int second_off, f32x4 s0,
                                           f32x4 s1) {
  if (MODE == MODE_GATE_UP) {
    if (i < out_n) {
      uint32_t hb[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) hb[c] = f32_to_bf16_bits(silu_f32(s0[c]) * s1[c]);
      u32x2 o;
      o[0] = hb[0] | (hb[1] << 16);
      o[1] = hb[2] | (hb[3] << 16);
      *reinterpret_cast<u32x2 *>(reinterpret_cast<uint16_t *>(out) + orow * out_n + i) = o;
    }
  } else {
    float *y = reinterpret_cast<float *>(out);
    if (i < out_n) *reinterpret_cast<f32x4 *>(y + orow * out_n + i) = s0;
    if (i + second_off < out_n) *reinterpret_cast<f32x4 *>(y + orow * out_n + i + second_off) = s1;
  }
}

// All tiles of one class for this workgroup: the software pipeline.
template <int MODE, int CLS, bool FP8>
__device__ __forceinline__ void run_class(const StreamArgs &a, const Tables &tb_, const ClassCfg &c,
                                          char *smem) {
  constexpr bool WIDE = ClsGeo<CLS>::WIDE, T128 = ClsGeo<CLS>::T128;
  constexpr int NTS = ClsGeo<CLS>::NTS, NSUB = ClsGeo<CLS>::NSUB;
  constexpr int WNW = ClsGeo<CLS>::WN, WHROWS = ClsGeo<CLS>::WH;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uni(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  float *red = reinterpret_cast<float *>(smem + RING * SLOT_BYTES);
  // Units drawn from the counter travel from the multiplying waves (wave 0 draws) to the loading
  // waves through four words of LDS: unit n of this workgroup in word n & 3.  (An LDS pointer by
  // type, so that the accesses are ds operations, which no vector-memory wait guards; the barriers
  // between a write and its reads are compiler memory fences as well.)
  typedef __attribute__((address_space(3))) int lds_int;
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wint-to-pointer-cast"
  lds_int *mbox = (lds_int *)(lds0 + (uint32_t)(RING * SLOT_BYTES + RED_BYTES));
#pragma clang diagnostic pop
  const bool dyn = !WIDE && c.dyn;
  // unit 0: the workgroup's own range; if that is empty and units can be drawn, the first drawn one
  int first_t0 = c.id0, first_t1 = c.id0 + c.n_mine;
  if (dyn && c.n_mine <= 0) {
    if (tid == 0) mbox[0] = (int)atomicAdd(c.ctr, 1);
    __syncthreads();
    unit_range(c, mbox[0], first_t0, first_t1);
    if (first_t0 >= first_t1) return;  // (the same for every wave)
  } else if (c.n_mine <= 0) {
    return;
  }
  constexpr int NACC = 1;  // (small tiles; the wide tiles keep theirs in accw)
  constexpr int RG = WIDE ? WRING : RING, AH = WIDE ? WAHEAD : AHEAD, LWN = WIDE ? WLW : LW;
  constexpr int SLOTB = WIDE ? WSLOT_BYTES : SLOT_BYTES;

  if (wave >= 4) {
    // ---- loading waves: the load cursor ----------------------------------------------
    const int lw = wave - 4;
    unsigned long long single = 0ull;  // bit s & 63: slot s is the only one of its tile
    int l_i = 0, l_kb = 0, l_slot = 0;
    int l_sub = 0;  // wide: 0 .. NTS-1 token slots, then the WNW weight slots
    int l_id = dyn ? first_t0 : c.id0, l_end = first_t1, l_n = 0;  // (dyn: tile, end of its unit, unit number)
    bool l_need = false;  // dyn: the unit is used up, the next one is fetched when its first slot is due
    Entry len = load_entry<MODE, CLS, FP8>(a, tb_, c, l_id);
    LoadPtrs<CLS> lp;
    setup_b<MODE, CLS>(lp, len, tb_.row_token, lw, lane);
    setup_a<MODE, CLS, FP8>(lp, len, l_id - len.first, lw, lane);
    bool l_live = true;

    auto open_tile = [&](int id) __attribute__((always_inline)) {
      if (id - len.first >= len.tiles || id < len.first) {
        len = load_entry<MODE, CLS, FP8>(a, tb_, c, id);
        setup_b<MODE, CLS>(lp, len, tb_.row_token, lw, lane);
      }
      setup_a<MODE, CLS, FP8>(lp, len, id - len.first, lw, lane);
    };
    auto advance_load = [&]() __attribute__((always_inline)) {
      if (dyn && l_need) {
        // Written by wave 0 during the first step of the unit just loaded, which lies at least one
        // barrier back: every unit has at least three slots and this slot is due two steps ahead.
        ++l_n;
        unit_range(c, mbox[l_n & 3], l_id, l_end);
        if (l_id >= l_end) {
          l_live = false;
          return;
        }
        l_need = false;
        open_tile(l_id);
      }
      issue_slot<MODE, CLS, FP8>(lp, len, l_kb, l_sub, lds0 + (uint32_t)(l_slot % RG) * SLOTB, lw, lane);
      // a tile of one slot: the multiplying waves put one more barrier into that slot's step
      if (!WIDE) single = (single & ~(1ull << (l_slot & 63))) | ((unsigned long long)(len.nkb == 1) << (l_slot & 63));
      ++l_slot;
      if (WIDE && l_sub < NSUB - 1) {
        ++l_sub;
        return;
      }
      l_sub = 0;
      if (++l_kb == len.nkb) {
        l_kb = 0;
        if (dyn) {
          if (++l_id == l_end) {
            l_need = true;
            return;
          }
        } else {
          if (++l_i == c.n_mine) {
            l_live = false;
            return;
          }
          l_id = c.id0 + l_i * c.stride;
        }
        open_tile(l_id);
      }
    };

    for (int i = 0; i < AH && l_live; ++i) advance_load();
    int k = 0;  // the slot whose step this is
    while (k < l_slot) {
      // slot k must have landed: at most AH-1 younger slots may be pending
      if (l_slot - k == AH) wait_vm<(AH - 1) * LWN>();
      else wait_vm<0>();
      wg_barrier();  // slot k is in LDS for the multiplying waves; they are done with slot k-1
      if (l_live) advance_load();
      if (!WIDE && ((single >> (k & 63)) & 1ull)) wg_barrier();
      ++k;
    }
    if (!WIDE) wg_barrier();  // the last tile's reduction
  } else {
    // ---- multiplying waves: the compute cursor -------------------------------------------
    int c_i = 0, c_kb = 0, c_slot = 0;
    int c_id = dyn ? first_t0 : c.id0, c_end = first_t1, c_n = 0;
    bool c_first = dyn;  // dyn: this is the first step of a unit
    Entry cen = load_entry<MODE, CLS, FP8>(a, tb_, c, c_id);
    f32x4 acc0[NACC], acc1[NACC];
#pragma unroll
    for (int nt = 0; nt < NACC; ++nt) {
      acc0[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      acc1[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    // a finished small tile whose partial sums wait in `red` for the next barrier
    bool pend = false;
    int pend_m = 0, pend_row0 = 0, pend_i0 = 0, pend_n = 0;
    void *pend_out = nullptr;
    // (8-bit weights: the row scales of this thread's four sums, fetched when the tile is finished so that
    // they have landed when the sums are added, a barrier later)
    float pend_c0[2] = {0.f, 0.f}, pend_c1[2] = {0.f, 0.f};

    // After a barrier: add the waves' partial tiles.  Thread t takes token row t >> 4 and feature
    // t & 15 (of both halves), so 16 neighbouring lanes store 16 neighbouring features of a row.
    auto flush_pending = [&]() __attribute__((always_inline)) {
      const int j = tid >> 4, fi = tid & 15;
      if (!FP8) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          s0 += red[(w * 2 + 0) * RED_TILE + j * RED_ROW + fi];
          s1 += red[(w * 2 + 1) * RED_TILE + j * RED_ROW + fi];
        }
        if (j < pend_m) store_out<MODE>(pend_out, pend_n, (size_t)(pend_row0 + j), pend_i0 + fi, 16, s0, s1);
      } else {
        // 8-bit weights: wave (h, kh) left the sums of rows 16h.. (tile 0) and 32 + 16h.. (tile 1) over
        // its half kh of the block's contraction; each sum is scaled by its weight row's scale
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int i = pend_i0 + 16 * hh + fi;  // feature (gate/up) or first of the two output rows (down)
          const float c0 = pend_c0[hh], c1 = pend_c1[hh];
          const float s0 = red[(0 * 4 + hh * 2 + 0) * RED_TILE + j * RED_ROW + fi] +
                           red[(1 * 4 + hh * 2 + 0) * RED_TILE + j * RED_ROW + fi];
          const float s1 = red[(0 * 4 + hh * 2 + 1) * RED_TILE + j * RED_ROW + fi] +
                           red[(1 * 4 + hh * 2 + 1) * RED_TILE + j * RED_ROW + fi];
          if (j < pend_m) store_out<MODE>(pend_out, pend_n, (size_t)(pend_row0 + j), i, 32, s0 * c0, s1 * c1);
        }
      }
      pend = false;
    };

    // Wide tiles: a wave keeps the fragments of its 2 x 16 token rows of the current block, all 8 steps,
    // in registers.  64-row class: the waves form 2 (row halves of a weight slot) x 2 (token halves) and a
    // wave multiplies 2 row tiles of every weight slot; 128-row class: wave w owns token rows 32w .. 32w+31
    // (token slot w >> 1) and multiplies all 4 row tiles of every weight slot.
    constexpr int NRT = (T128 ? 4 : 2) * (FP8 ? 2 : 1);  // row tiles of a weight slot per wave (8-bit codes: slots of 128 rows)
    u32x4 fbw[WIDE ? 2 : 1][WIDE ? 8 : 1];
    f32x4 accw[WIDE ? WNW : 1][WIDE ? NRT : 1][2];  // [weight slot][row tile of the wave][token tile of the wave]
#pragma unroll
    for (int w = 0; w < (WIDE ? WNW : 1); ++w)
#pragma unroll
      for (int i = 0; i < (WIDE ? NRT : 1) * 2; ++i) accw[w][i >> 1][i & 1] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int wr = T128 ? 0 : (wave & 1);           // first row tile of the wave: NRT * wr
    const int wt = T128 ? wave : (wave >> 1);       // token rows 32 wt .. 32 wt + 31 of the tile
    const int tok_sub = T128 ? (wave >> 1) : 0;     // the token slot they arrive in
    const int tok_row = T128 ? 32 * (wave & 1) : 32 * wt;  // their first row inside that slot

    while (true) {
      bool tile_done = false;
      if (!WIDE) {
        wg_barrier();  // slot c_slot has landed (the loading waves waited for it)
        if (pend) flush_pending();
        if (dyn && c_first) {
          // First step of a unit: wave 0 draws the unit after this one and waits for the answer
          // (the multiplying waves have time to spare: they wait for the loading waves at every
          // barrier).  Keeping the answer pending in a register instead makes the compiler guard
          // every later use of that register with a wait for all of the wave's stores.  The loading
          // waves ask for the unit when this unit's last slot has been issued, at least one barrier
          // later: a unit has three slots or more and slots are issued two steps ahead.
          if (wave == 0) {
            int u = 0;
            if (lane == 0) u = (int)atomicAdd(c.ctr, 1);
            if (lane == 0) mbox[(c_n + 1) & 3] = u;
          }
          c_first = false;
        }
        const char *sb = smem + (size_t)(c_slot % RG) * SLOTB;
        const int kbase = c_kb * KB;
        if constexpr (FP8) {
          // 64 rows of 8-bit codes per slot.  Wave (h, kh) = (wave & 1, wave >> 1) multiplies slot rows
          // 16h .. 16h+15 and 32 + 16h .. (the same rows of w_gate and w_up, or two groups of w_down rows)
          // over the half kh of the block's 512 contraction elements: 4 chunks of 64.  In a chunk lane
          // (r, q) holds the 16 codes k = 16q .. 16q+15 of its row: two MFMA operands after widening to
          // bf16 (exact), matched by the token pieces 2q and 2q + 1 of the chunk.
          const int h = wave & 1, kh = wave >> 1;
          const char *pa0 = sb + (size_t)(16 * h + r16) * 512;
          const char *pa1 = sb + (size_t)(32 + 16 * h + r16) * 512;
          const char *pb = sb + A_BYTES + (size_t)r16 * SROW_BYTES;
          auto widen = [&](u32x4 codes, u32x4 &lo, u32x4 &hi) __attribute__((always_inline)) {
#pragma unroll
            for (int dw = 0; dw < 2; ++dw) {
              lo[2 * dw] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[dw], 1.0f, false));
              lo[2 * dw + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[dw], 1.0f, true));
              hi[2 * dw] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[2 + dw], 1.0f, false));
              hi[2 * dw + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[2 + dw], 1.0f, true));
            }
          };
          const bool whole = kbase + KB <= cen.klen;
          u32x4 ra0[4], ra1[4], fb0[4], fb1[4];
#pragma unroll
          for (int cc = 0; cc < 4; ++cc) {
            const int ch = 4 * kh + cc;        // chunk of 64 contraction elements
            const int pc = 4 * ch + q;         // 16-byte piece of codes
            const int pt = 8 * ch + 2 * q;     // first of the two 16-byte pieces of tokens
            ra0[cc] = *reinterpret_cast<const u32x4 *>(pa0 + ((pc ^ r16) << 4));
            ra1[cc] = *reinterpret_cast<const u32x4 *>(pa1 + ((pc ^ r16) << 4));
            fb0[cc] = *reinterpret_cast<const u32x4 *>(pb + ((pt ^ r16) << 4));
            fb1[cc] = *reinterpret_cast<const u32x4 *>(pb + (((pt + 1) ^ r16) << 4));
            if (!whole) {  // ragged last block: pieces past the row's end hold bytes pulled back from inside it
              if (kbase + pt * 8 >= cen.klen) fb0[cc] = (u32x4){0u, 0u, 0u, 0u};
              if (kbase + (pt + 1) * 8 >= cen.klen) fb1[cc] = (u32x4){0u, 0u, 0u, 0u};
            }
          }
#pragma unroll
          for (int cc = 0; cc < 4; ++cc) {
            if (whole || kbase + 64 * (4 * kh + cc) < cen.klen) {
              u32x4 lo, hi;
              widen(ra0[cc], lo, hi);
              acc0[0] = mfma16(lo, fb0[cc], acc0[0]);
              acc0[0] = mfma16(hi, fb1[cc], acc0[0]);
              widen(ra1[cc], lo, hi);
              acc1[0] = mfma16(lo, fb0[cc], acc1[0]);
              acc1[0] = mfma16(hi, fb1[cc], acc1[0]);
            }
          }
        } else {
        // waves split the 16 steps
        if (kbase + KB <= cen.klen) {  // whole block: no masks, reads issued back to back
          u32x4 fa0[4], fa1[4], fb[4];
#pragma unroll
          for (int ss = 0; ss < 4; ++ss) {
            const int piece = 4 * (wave * 4 + ss) + q;
            const int off = r16 * SROW_BYTES + ((piece ^ r16) << 4);
            fa0[ss] = *reinterpret_cast<const u32x4 *>(sb + off);
            fa1[ss] = *reinterpret_cast<const u32x4 *>(sb + 16 * SROW_BYTES + off);
            fb[ss] = *reinterpret_cast<const u32x4 *>(sb + A_BYTES + off);
          }
#pragma unroll
          for (int ss = 0; ss < 4; ++ss) {
            acc0[0] = mfma16(fa0[ss], fb[ss], acc0[0]);
            acc1[0] = mfma16(fa1[ss], fb[ss], acc1[0]);
          }
        } else {
#pragma unroll
          for (int ss = 0; ss < 4; ++ss) {
            const int s = wave * 4 + ss;
            if (kbase + s * 32 < cen.klen) {
              const int piece = 4 * s + q;
              const int off = r16 * SROW_BYTES + ((piece ^ r16) << 4);
              const u32x4 fa0 = *reinterpret_cast<const u32x4 *>(sb + off);
              const u32x4 fa1 = *reinterpret_cast<const u32x4 *>(sb + 16 * SROW_BYTES + off);
              u32x4 fb = *reinterpret_cast<const u32x4 *>(sb + A_BYTES + off);
              if (kbase + piece * 8 >= cen.klen) fb = (u32x4){0u, 0u, 0u, 0u};  // ragged last step
              acc0[0] = mfma16(fa0, fb, acc0[0]);
              acc1[0] = mfma16(fa1, fb, acc1[0]);
            }
          }
        }
        }
        tile_done = (c_kb == cen.nkb - 1);
        ++c_kb;
        ++c_slot;
      } else {
        // One block per turn of the loop: its NTS token slots, then its WNW weight slots, one barrier
        // each (the slot has landed: the loading waves waited for it).  The token fragments of a block
        // stay in registers, so a token slot is free again as soon as it has been read, like every
        // weight slot; nothing is added across waves.
        const bool busy = 32 * wt < cen.m;  // (a wave without token rows only keeps the barriers)
        const int kbase = c_kb * KBW;
#pragma unroll
        for (int ts = 0; ts < NTS; ++ts) {
          wg_barrier();
          const char *sb = smem + (size_t)(c_slot % RG) * SLOTB;
          if (busy && ts == tok_sub) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
              const char *pb = sb + (size_t)(tok_row + 16 * tt + r16) * ROW_BYTES;
#pragma unroll
              for (int st = 0; st < 8; ++st) {
                // bf16 weights: step st takes the 8 elements 32 st + 8 q ..; 8-bit weights: lane (r, q) holds the
                // 16 codes 64 (st >> 1) + 16 q .. of its row per chunk, two operands once widened, which meet
                // the token pieces 8 (st >> 1) + 2 q and the next
                const int piece = FP8 ? 8 * (st >> 1) + 2 * q + (st & 1) : 4 * st + q;
                fbw[tt][st] = *reinterpret_cast<const u32x4 *>(pb + ((piece ^ r16) << 4));
                // ragged last block: pieces past the row's end hold bytes pulled back from inside it
                if (kbase + piece * 8 >= cen.klen) fbw[tt][st] = (u32x4){0u, 0u, 0u, 0u};
              }
            }
          }
          ++c_slot;
        }
#pragma unroll
        for (int w = 0; w < WNW; ++w) {
          wg_barrier();
          const char *sb = smem + (size_t)(c_slot % RG) * SLOTB;
          if (busy) {
            if constexpr (FP8) {
              // 128 rows of 256 codes: the wave's NRT row tiles (64-row class: its half of the slot; 128-row
              // class: all of it), 4 chunks of 64 contraction elements each
#pragma unroll
              for (int rtl = 0; rtl < NRT; ++rtl) {
                const char *pa = sb + (size_t)(16 * (NRT * wr + rtl) + r16) * 256;
                u32x4 codes[4];
#pragma unroll
                for (int ch = 0; ch < 4; ++ch)
                  codes[ch] = *reinterpret_cast<const u32x4 *>(pa + (((4 * ch + q) ^ r16) << 4));
#pragma unroll
                for (int ch = 0; ch < 4; ++ch) {
                  u32x4 lo, hi;
#pragma unroll
                  for (int dw = 0; dw < 2; ++dw) {
                    lo[2 * dw] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[ch][dw], 1.0f, false));
                    lo[2 * dw + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[ch][dw], 1.0f, true));
                    hi[2 * dw] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[ch][2 + dw], 1.0f, false));
                    hi[2 * dw + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(codes[ch][2 + dw], 1.0f, true));
                  }
#pragma unroll
                  for (int tt = 0; tt < 2; ++tt) {
                    accw[w][rtl][tt] = mfma16(lo, fbw[tt][2 * ch], accw[w][rtl][tt]);
                    accw[w][rtl][tt] = mfma16(hi, fbw[tt][2 * ch + 1], accw[w][rtl][tt]);
                  }
                }
              }
            } else if constexpr (T128) {
              // 8 chunks of (2 row tiles) x (2 steps): the fragments of the next chunks are read while this
              // one is multiplied, and consecutive MFMAs go to 4 different accumulators.  All 8 steps of 2
              // row tiles at once would not fit the registers beside 64 accumulator and 64 token-fragment
              // registers.
              constexpr int DEPTH = W128_FRAG_DEPTH;  // chunks in flight
              u32x4 fa[DEPTH][4];  // [buffer][2 * row tile + step]
              auto read_chunk = [&](int ch, u32x4 (&f)[4]) __attribute__((always_inline)) {
                // chunk ch: row tiles 2 (ch >> 2), +1; steps 2 (ch & 3), +1
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  const int rt = 2 * (ch >> 2) + (i >> 1), st = 2 * (ch & 3) + (i & 1);
                  f[i] = *reinterpret_cast<const u32x4 *>(sb + (size_t)(16 * rt + r16) * ROW_BYTES +
                                                         (((4 * st + q) ^ r16) << 4));
                }
              };
#pragma unroll
              for (int ch = 0; ch < DEPTH - 1; ++ch) read_chunk(ch, fa[ch]);
#pragma unroll
              for (int ch = 0; ch < 8; ++ch) {
                if (ch + DEPTH - 1 < 8) read_chunk(ch + DEPTH - 1, fa[(ch + DEPTH - 1) % DEPTH]);
#pragma unroll
                for (int si = 0; si < 2; ++si)
#pragma unroll
                  for (int ri = 0; ri < 2; ++ri) {
                    const int rt = 2 * (ch >> 2) + ri, st = 2 * (ch & 3) + si;
#pragma unroll
                    for (int tt = 0; tt < 2; ++tt)
                      accw[w][rt][tt] = mfma16(fa[ch % DEPTH][2 * ri + si], fbw[tt][st], accw[w][rt][tt]);
                  }
                __builtin_amdgcn_sched_barrier(0);  // keeps the reads DEPTH - 1 chunks ahead, not more
              }
            } else {
#pragma unroll
              for (int rtl = 0; rtl < NRT; ++rtl) {
                const char *pa = sb + (size_t)(16 * (NRT * wr + rtl) + r16) * ROW_BYTES;
                u32x4 fa[8];
#pragma unroll
                for (int st = 0; st < 8; ++st)
                  fa[st] = *reinterpret_cast<const u32x4 *>(pa + (((4 * st + q) ^ r16) << 4));
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                  for (int st = 0; st < 8; ++st) accw[w][rtl][tt] = mfma16(fa[st], fbw[tt][st], accw[w][rtl][tt]);
              }
            }
          }
          ++c_slot;
        }
        tile_done = (c_kb == cen.nkb - 1);
        ++c_kb;
      }

      if (tile_done) {
        const int id = c_id;
        const int i0 = tile_i0<MODE, CLS, FP8>(id - cen.first);
        if (WIDE) {
          // straight from the accumulators: token row 32wt + 16tt + r16; slot w < WNW/2 pairs with slot
          // w + WNW/2 (gate with up rows; down: WHROWS features further on)
          // (8-bit weights: one scale per weight row = per output feature, fetched once per row tile for both
          // token tiles, from clamped addresses: a feature past the end gets some other row's scale and its
          // store is skipped.  The registers are nearly all taken here, so no further ahead than that.)
#pragma unroll
          for (int w = 0; w < WNW / 2; ++w)
#pragma unroll
            for (int rtl = 0; rtl < NRT; ++rtl) {
              const int i = i0 + (FP8 ? 128 : 64) * w + 16 * (NRT * wr + rtl) + 4 * q;
              f32x4 c0 = {1.f, 1.f, 1.f, 1.f}, c1 = {1.f, 1.f, 1.f, 1.f};
              if constexpr (FP8) {
                const int i1 = (MODE == MODE_GATE_UP) ? i : i + 2 * WHROWS;
                c0 = *reinterpret_cast<const f32x4 *>(cen.s0 + min(i, cen.out_n - 4));
                c1 = *reinterpret_cast<const f32x4 *>(cen.s1 + min(i1, cen.out_n - 4));
              }
#pragma unroll
              for (int tt = 0; tt < 2; ++tt) {
                const int j = 32 * wt + 16 * tt + r16;
                if (j < cen.m) {
                  f32x4 v0 = accw[w][rtl][tt], v1 = accw[w + WNW / 2][rtl][tt];
                  if constexpr (FP8) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                      v0[c] *= c0[c];
                      v1[c] *= c1[c];
                    }
                  }
                  store_out4<MODE>(cen.out, cen.out_n, (size_t)(cen.row0 + j), i, FP8 ? 2 * WHROWS : WHROWS, v0, v1);
                }
              }
            }
#pragma unroll
          for (int w = 0; w < WNW; ++w)
#pragma unroll
            for (int i = 0; i < NRT * 2; ++i) accw[w][i >> 1][i & 1] = (f32x4){0.f, 0.f, 0.f, 0.f};
        } else {
          if (cen.nkb == 1) wg_barrier();  // the previous tile's sums may still be read from `red`
          // lane (q, r16) holds features 4q..4q+3 of token row r16: one 16-byte store per half
          // (8-bit weights: partial tile index (kh, h, tile) = 4 (wave >> 1) + 2 (wave & 1) + tile)
          const int slot2 = FP8 ? 4 * (wave >> 1) + 2 * (wave & 1) : wave * 2;
          *reinterpret_cast<f32x4 *>(red + (slot2 + 0) * RED_TILE + r16 * RED_ROW + 4 * q) = acc0[0];
          *reinterpret_cast<f32x4 *>(red + (slot2 + 1) * RED_TILE + r16 * RED_ROW + 4 * q) = acc1[0];
          if constexpr (FP8) {
            const int pj = tid >> 4, pf = tid & 15;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
              const int i = i0 + 16 * hh + pf;
              const int i1 = (MODE == MODE_GATE_UP) ? i : i + 32;
              pend_c0[hh] = (pj < cen.m && i < cen.out_n) ? cen.s0[i] : 0.f;
              pend_c1[hh] = (pj < cen.m && i1 < cen.out_n) ? cen.s1[i1] : 0.f;
            }
          }
          pend = true;
          pend_m = cen.m;
          pend_row0 = cen.row0;
          pend_i0 = i0;
          pend_n = cen.out_n;
          pend_out = cen.out;
          acc0[0] = (f32x4){0.f, 0.f, 0.f, 0.f};
          acc1[0] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        c_kb = 0;
        if (dyn) {
          if (++c_id == c_end) {
            ++c_n;
            unit_range(c, mbox[c_n & 3], c_id, c_end);  // written at least one barrier ago
            if (c_id >= c_end) break;
            c_first = true;
          }
        } else {
          if (++c_i == c.n_mine) break;
          c_id = c.id0 + c_i * c.stride;
        }
        const int nid = c_id;
        if (nid - cen.first >= cen.tiles || nid < cen.first) cen = load_entry<MODE, CLS, FP8>(a, tb_, c, nid);
      }
    }
    if (!WIDE && pend) {
      wg_barrier();
      flush_pending();
    }
  }
  // nothing pending, every wave done reading the ring: the next class may reuse it
  wait_vm<0>();
  wg_barrier();
}

// DYN: the variant that can draw units of small tiles from the counter (the host launches the
// other one, which is a little quicker to start, when the small line is certainly too short for it).
// FP8: expert weights are E4M3 codes with a scale per output row.
template <int MODE, bool DYN, bool FP8>
__global__ __launch_bounds__(STREAM_THREADS) void expert_stream_kernel(StreamArgs a,
                                                            const int32_t *__restrict__ plan,
                                                            const int32_t *__restrict__ offsets,
                                                            const int32_t *__restrict__ row_token) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const Tables tb_{plan, offsets, row_token};
  const int G = gridDim.x, bid = blockIdx.x;

  // ---- the schedule (stream_sched.h) -------------------------------------------------
  int n_small_e, n_b64_e, n_large_e, n_b128_e;
  sload4(plan, 0, 1, 2, 3, n_small_e, n_b64_e, n_large_e, n_b128_e);
  SchedIn in;
  in.mode = MODE;
  in.d = a.d; in.I = a.I; in.S = a.S; in.T = a.T; in.part_k = a.part_k;
  in.shared_stream = a.shared_stream;
  in.n_small_e = n_small_e; in.n_b64_e = n_b64_e; in.n_b128_e = n_b128_e;
  in.G = G; in.bid = bid;
  in.dyn_allowed = DYN ? 1 : 0;
  in.fp8 = FP8 ? 1 : 0;
  StreamSched sc;
  stream_schedule(in, const_cast<int32_t *>(plan) + PLAN_CTR + MODE, sc);
  if constexpr (!FP8) {
    if (sc.c128.wn == WIDE_WN_MANY) run_class<MODE, CLS_W128X, false>(a, tb_, sc.c128, smem);
    else run_class<MODE, CLS_W128, false>(a, tb_, sc.c128, smem);
    run_class<MODE, CLS_W64, false>(a, tb_, sc.c64, smem);
  } else {
    run_class<MODE, CLS_W128, true>(a, tb_, sc.c128, smem);
    run_class<MODE, CLS_W64, true>(a, tb_, sc.c64, smem);
  }
  run_class<MODE, CLS_SMALL, FP8>(a, tb_, sc.cs, smem);
}

static hipError_t launch_stream(int mode, const StreamArgs &a, hipStream_t s) {
  static LdsLimitOnce lds_once[8];
  int dev = 0, n_cu = 0;
  hipError_t e0 = current_device(&dev, &n_cu);
  if (e0 != hipSuccess) return e0;
  // Upper bound of the small tiles (the plan is on the device): experts with rows x row tiles, plus
  // the shared expert's when it has at most 16 rows.  Below the threshold the kernel would deal
  // everything in fixed ranges anyway.
  const long srows = a.fp8 ? 64 : 32;  // weight rows of a small tile
  const long kr = mode == MODE_GATE_UP ? a.d : a.I;
  const long nkb_s = (kr + KB - 1) / KB;
  const long per_r = mode == MODE_GATE_UP ? (a.I + srows / 2 - 1) / (srows / 2) : (a.d + srows - 1) / srows;
  const long per_s = mode == MODE_GATE_UP ? (a.S + srows / 2 - 1) / (srows / 2) : (a.d + srows - 1) / srows;
  const long parts = (mode == MODE_DOWN && a.S > 0) ? (a.S + a.part_k - 1) / a.part_k : 1;
  const long e_max = (long)a.T * a.K < a.E ? (long)a.T * a.K : a.E;
  const long small_max = e_max * per_r + ((a.S > 0 && a.T <= SMALL_M)
                                              ? per_s * parts * ((a.T + SMALL_M - 1) / SMALL_M) : 0);
  const bool dyn = DYN_STATIC_PCT < 100 && small_max * nkb_s >= (long)DYN_MIN_SLOTS * n_cu &&
                   small_max >= (long)DYN_MIN_TILES * n_cu;
  const int which = (a.fp8 ? 4 : 0) + mode * 2 + (dyn ? 1 : 0);
  typedef void (*kern_t)(StreamArgs, const int32_t *, const int32_t *, const int32_t *);
  static const kern_t fns[8] = {
      expert_stream_kernel<MODE_GATE_UP, false, false>, expert_stream_kernel<MODE_GATE_UP, true, false>,
      expert_stream_kernel<MODE_DOWN, false, false>,    expert_stream_kernel<MODE_DOWN, true, false>,
      expert_stream_kernel<MODE_GATE_UP, false, true>,  expert_stream_kernel<MODE_GATE_UP, true, true>,
      expert_stream_kernel<MODE_DOWN, false, true>,     expert_stream_kernel<MODE_DOWN, true, true>};
  e0 = raise_dynamic_lds_limit(lds_once[which], dev, reinterpret_cast<const void *>(fns[which]), STREAM_LDS_BYTES);
  if (e0 != hipSuccess) return e0;
  hipLaunchKernelGGL(fns[which], dim3(n_cu), dim3(STREAM_THREADS), STREAM_LDS_BYTES, s, a, a.plan, a.offsets,
                     a.row_token);
  return hipGetLastError();
}

hipError_t launch_gate_up(const StreamArgs &a, hipStream_t s) { return launch_stream(MODE_GATE_UP, a, s); }
hipError_t launch_down(const StreamArgs &a, hipStream_t s) { return launch_stream(MODE_DOWN, a, s); }
