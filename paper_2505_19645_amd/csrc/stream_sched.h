// Work split of the streaming expert kernels (expert_stream.hip): which tiles of each class a
// workgroup processes.  Plain integer / double arithmetic on launch-wide values, written so that
// the kernel (every workgroup for itself) and a host-side test compute it from the same code.
//
// While an expert sees few tokens the layer's time is the loading of the activated experts'
// weights (the k2*N term of the paper's Sec. 3.3); the split below is what keeps every compute
// unit loading until the last byte: tiles of the two wide classes are dealt round-robin, then the
// line of small tiles is cut so that every workgroup's estimated time is the same, and when that
// line is long its tail is handed out in units drawn from a counter.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define MOESD_SCHED_FN __host__ __device__ __forceinline__
#else
#define MOESD_SCHED_FN inline
#endif

enum { MODE_GATE_UP = 0, MODE_DOWN = 1 };
// tile classes: token rows per tile
enum { CLS_SMALL = 0, CLS_W64 = 1, CLS_W128 = 2 };
#define SMALL_M 16   // token rows of a small tile
#define W64_TB 64    // of a tile of the first wide class
#define W128_TB 128  // of the second
#define KB 512       // contraction elements per block, small tiles
#define KBW 256      // wide tiles
// Weight slots (of 64 rows of bf16) per block of a wide tile: a wide tile has 64 * wn weight rows, and its
// token rows are fetched once per that many.  Two; in the 128-row class four where the class then still
// has WIDE4_MIN_TILES_PER_WG tiles per workgroup (its two token slots are then a third instead of half of
// what the loading waves move: DeepSeek-V3-shaped layer at T = 2560 5.23 -> 4.87 ms).  With few tiles the
// longer ones leave compute units idle (Mixtral-shaped down projection at T = 64 when forced: 0.78 -> 0.57
// of the HBM peak), and in the 64-row class the wider tile measured slower in mixed launches.
#define WIDE_WN_FEW 2
#define WIDE_WN_MANY 4
#define WIDE4_MIN_TILES_PER_WG 2
// the schedule's cost model, in hundredths of a routed expert's small slot
#define COST_WIDE_SLOT 100
#define COST_CLASS_SWITCH 650
#define COST_DISTINCT_ROWS 15
#ifndef DYN_STATIC_PCT
#define DYN_STATIC_PCT 60  // share of a long small line that is dealt in fixed ranges (100: all of it)
#endif
#ifndef DYN_MIN_SLOTS
#define DYN_MIN_SLOTS 40   // slots of small tiles per workgroup from which units are drawn at all
#endif
#ifndef DYN_MIN_TILES
#define DYN_MIN_TILES 12   // and small tiles per workgroup (a few long tiles are better dealt evenly)
#endif

// The tiles of one class that a workgroup processes: ids id0, id0 + stride, ...  A class's tile
// ids run over [shared expert's tiles][routed entries x row tiles].
struct ClassCfg {
  int n_mine, id0, stride;
  int n_sh;    // shared-expert tiles at the head of the class
  int per_s;   // row tiles per shared entry
  int per_r;   // row tiles per routed entry
  int parts;   // k-parts of the shared down projection (1 for gate/up)
  int wn;      // wide classes: weight slots per block (WIDE_WN_FEW or WIDE_WN_MANY)
  // Small tiles only: after its own range (n_mine tiles from id0) the workgroup draws units of
  // further tiles from a counter shared by all workgroups.  Units u < n_double hold 2 * ut tiles,
  // the others ut, the last one also what is left of the line; all lie in [pool0, n_tiles).
  int dyn;
  int n_units, n_double, ut, pool0, n_tiles;
  int32_t *ctr;
};

// tiles [t0, t1) of drawn unit u; empty when the counter has run past the last unit
MOESD_SCHED_FN void unit_range(const ClassCfg &c, int u, int &t0, int &t1) {
  if (u < 0 || u >= c.n_units) {
    t0 = t1 = 0;
  } else if (u < c.n_double) {
    t0 = c.pool0 + u * 2 * c.ut;
    t1 = t0 + 2 * c.ut;
  } else {
    t0 = c.pool0 + c.n_double * 2 * c.ut + (u - c.n_double) * c.ut;
    t1 = (u == c.n_units - 1) ? c.n_tiles : t0 + c.ut;
  }
}

struct SchedIn {
  int mode;                  // MODE_GATE_UP or MODE_DOWN
  int d, I, S, T, part_k;    // layer shape, tokens, k-part length of the shared down projection
  int shared_stream;         // the streaming kernels take the shared expert also above 128 tokens
                             // (in token blocks of 128 through the second wide class)
  int n_small_e, n_b64_e, n_b128_e;  // experts with 1..16, 17..64, 65..128 rows
  int G, bid;                // workgroups, this workgroup
  int dyn_allowed;           // the launched kernel can draw units
  int fp8;                   // 8-bit weights: small tiles of 64 weight rows, wide slots of 128
};

struct StreamSched {
  ClassCfg c128, c64, cs;
};

// Where the shared expert runs: with at most 16 tokens in the small class, up to 64 in the first
// wide class (one token block), beyond that in the second (blocks of 128 tokens) if the streaming
// kernels keep it at all.  With 8-bit weights a wide weight slot holds 128 rows of codes instead of 64
// rows of bf16, so a wide tile has twice the weight rows.
MOESD_SCHED_FN void stream_schedule(const SchedIn &in, int32_t *ctr, StreamSched &out) {
  const bool gu = in.mode == MODE_GATE_UP;
  const bool has_shared = in.S > 0;
  const int G = in.G, bid = in.bid;
  const int parts = (!gu && has_shared) ? (in.S + in.part_k - 1) / in.part_k : 1;
  ClassCfg &c128 = out.c128, &c64 = out.c64, &cs = out.cs;
  c128.parts = c64.parts = cs.parts = parts;
  // a small tile is one 32 KB weight slot wide: 32 rows of bf16 (16 of w_gate + 16 of w_up, or 32 of
  // w_down) or 64 rows of 8-bit codes
  const int srows = in.fp8 ? 64 : 32;
  cs.per_r = gu ? (in.I + srows / 2 - 1) / (srows / 2) : (in.d + srows - 1) / srows;
  cs.per_s = gu ? (in.S + srows / 2 - 1) / (srows / 2) : (in.d + srows - 1) / srows;
  cs.n_sh = (has_shared && in.T <= SMALL_M) ? cs.per_s * parts : 0;
  cs.wn = 0;
  // the wide classes: the shared expert's token blocks, and the tile width each class gets
  const int sh64 = (has_shared && in.T > SMALL_M && in.T <= W64_TB) ? parts : 0;
  const int sh128 = (has_shared && in.T > W64_TB && in.shared_stream)
                        ? parts * ((in.T + W128_TB - 1) / W128_TB) : 0;
  auto wide_cfg = [&](ClassCfg &c, int n_sh_blocks, int n_e, bool may_widen) {
    int wn = (in.fp8 || !may_widen) ? WIDE_WN_FEW : WIDE_WN_MANY;
    for (;;) {
      const int wh = (in.fp8 ? 64 : 32) * wn;  // rows of each operand half in a wide tile (8-bit: slots of 128 rows)
      c.per_r = gu ? (in.I + wh - 1) / wh : (in.d + 2 * wh - 1) / (2 * wh);
      c.per_s = gu ? (in.S + wh - 1) / wh : (in.d + 2 * wh - 1) / (2 * wh);
      c.n_sh = n_sh_blocks * c.per_s;
      c.wn = wn;
      if (wn == WIDE_WN_FEW || (long)c.n_sh + (long)n_e * c.per_r >= (long)WIDE4_MIN_TILES_PER_WG * G) break;
      wn = WIDE_WN_FEW;
    }
  };
  wide_cfg(c64, sh64, in.n_b64_e, false);
  wide_cfg(c128, sh128, in.n_b128_e, true);
  const int n128 = c128.n_sh + in.n_b128_e * c128.per_r;
  const int n64 = c64.n_sh + in.n_b64_e * c64.per_r;
  const int n_small = cs.n_sh + in.n_small_e * cs.per_r;
  c128.dyn = c64.dyn = 0;
  c128.n_units = c128.n_double = c128.ut = c128.pool0 = c128.n_tiles = 0;
  c64.n_units = c64.n_double = c64.ut = c64.pool0 = c64.n_tiles = 0;
  c128.ctr = c64.ctr = ctr;

  // The wide tiles form one sequence, the 128-row class first, dealt round-robin: tile j of the
  // sequence goes to workgroup j mod G.
  const int k128 = n128 / G, r128 = n128 - k128 * G;
  const int k64 = n64 / G, r64 = n64 - k64 * G;
  c128.id0 = bid;
  c128.stride = G;
  c128.n_mine = k128 + (bid < r128 ? 1 : 0);
  const int j0 = bid >= r128 ? bid - r128 : bid - r128 + G;  // this workgroup's first tile of the 64-row class
  c64.id0 = j0;
  c64.stride = G;
  c64.n_mine = k64 + (j0 < r64 ? 1 : 0);

  // The small line is then cut so that every workgroup's estimated time is the same.  Costs in
  // hundredths of the time of one small slot of a routed expert, from per-workgroup timelines on the
  // MI355X: a byte of a wide slot takes as long as one of a small slot, moving from the wide to the
  // small class drains and refills the ring (about 6 slots), and a small slot whose 16 token rows are
  // all distinct (the shared expert at T = 16) takes 1.15x as long as one with a few.
  const int kr = gu ? in.d : in.I;
  const int nkb_s = (kr + KB - 1) / KB, nkb_w = (kr + KBW - 1) / KBW;
  const double c_w64 = (double)(nkb_w * (c64.wn + 1) * 2 * COST_WIDE_SLOT) / 3.0;  // a wide slot is 2/3 of a small one
  const double c_w128 = (double)(nkb_w * (c128.wn + 2) * 2 * COST_WIDE_SLOT) / 3.0;
  const double c_sh = (double)(nkb_s * (100 + COST_DISTINCT_ROWS * (in.T < SMALL_M ? in.T : SMALL_M) / SMALL_M));
  const double c_r = (double)(nkb_s * 100);
  const int n_shs = cs.n_sh, n_rs = n_small - cs.n_sh;
  const double S = n_shs * c_sh + n_rs * c_r;  // the small line
  const double sw = S > 0 ? (double)COST_CLASS_SWITCH : 0.0;
  // Workgroup b holds k128 (+1 if b < r128) tiles of the 128-row class and k64 (+1 if its first
  // 64-row tile j0(b) < r64) of the other, so the wide cost is constant on at most three ranges of b.
  const int x = r128 + r64;
  int bp[4];
  bool e128[3], e64[3];
  bp[0] = 0;
  bp[3] = G;
  if (x <= G) {
    bp[1] = r128; bp[2] = x;
    e128[0] = true;  e64[0] = false;
    e128[1] = false; e64[1] = true;
    e128[2] = false; e64[2] = false;
  } else {
    bp[1] = x - G; bp[2] = r128;
    e128[0] = true;  e64[0] = true;
    e128[1] = true;  e64[1] = false;
    e128[2] = false; e64[2] = true;
  }
  double wcost[3], C = S;
  for (int i = 0; i < 3; ++i) {
    const double wv = (k128 + (e128[i] ? 1 : 0)) * c_w128 + (k64 + (e64[i] ? 1 : 0)) * c_w64;
    wcost[i] = wv + (wv > 0 ? sw : 0.0);
    C += wcost[i] * (bp[i + 1] - bp[i]);
  }
  // what is left of a workgroup's equal share for small tiles (all quantities scaled by G)
  double left[3], p_tot = 0.0;
  for (int i = 0; i < 3; ++i) {
    left[i] = C - wcost[i] * G;
    if (left[i] < 0.0) left[i] = 0.0;
    p_tot += left[i] * (bp[i + 1] - bp[i]);
  }
  // A long small line is cut this way only over its first DYN_STATIC_PCT percent; the rest is
  // drawn from a counter in units of at least three slots (a workgroup learns its next unit one
  // unit ahead), two units' worth at a time until the last two per workgroup.  The workgroups'
  // speeds differ by a few percent from launch to launch and between XCDs, which no fixed
  // split can know; the ranges below then only set where each workgroup starts.
  const int ut = (3 + nkb_s - 1) / nkb_s > 1 ? (3 + nkb_s - 1) / nkb_s : 1;
  int n_stat = n_small;
  cs.dyn = 0;
  cs.n_units = cs.n_double = cs.pool0 = 0;
  cs.ut = ut;
  cs.n_tiles = n_small;
  cs.ctr = ctr;
  if (in.dyn_allowed && DYN_STATIC_PCT < 100 && p_tot > 0.0) {
    const int ns = (int)((long long)n_small * DYN_STATIC_PCT / 100) / ut * ut;
    const int nq = (n_small - ns) / ut;  // groups of ut tiles in the drawn part
    if (ns >= G * ut && nq >= G && (long long)n_small * nkb_s >= (long long)DYN_MIN_SLOTS * G &&
        n_small >= DYN_MIN_TILES * G) {
      int n_single = nq < 2 * G ? nq : 2 * G;
      if ((nq - n_single) & 1) ++n_single;
      n_stat = ns;
      cs.dyn = 1;
      cs.n_double = (nq - n_single) / 2;
      cs.n_units = cs.n_double + n_single;
      cs.pool0 = ns;
    }
  }
  const int n_shs_l = n_shs < n_stat ? n_shs : n_stat;
  const double S_l = n_shs_l * c_sh + (n_stat - n_shs_l) * c_r;  // the part of the line that is cut
  // first small tile of workgroup b: the tile at cost position S_l * p(b) / p_tot of that part
  int fs[2];
  for (int which = 0; which < 2; ++which) {
    const int b = bid + which;
    int ti;
    if (p_tot <= 0.0 || b <= 0) {
      ti = 0;
    } else if (b >= G) {
      ti = n_stat;
    } else {
      double pb = 0.0;
      for (int i = 0; i < 3; ++i) {
        int n = b - bp[i];
        if (n > bp[i + 1] - bp[i]) n = bp[i + 1] - bp[i];
        if (n > 0) pb += left[i] * n;
      }
      const double pos = S_l * pb / p_tot;
      const double head = n_shs_l * c_sh;
      const double t = pos <= head ? pos / c_sh : (double)n_shs_l + (pos - head) / c_r;
      ti = (int)t < n_stat ? (int)t : n_stat;
      if (cs.dyn) ti = ti / ut * ut;
    }
    fs[which] = ti;
  }
  if (p_tot <= 0.0) fs[0] = fs[1] = 0;
  cs.n_mine = fs[1] - fs[0];
  cs.id0 = fs[0];
  cs.stride = 1;
}
