// Host build of the streaming kernels' work split (csrc/stream_sched.h) for the CPU tests:
// the same header the kernels include, compiled with g++, one C entry point.
#include "../../paper_2505_19645_amd/csrc/stream_sched.h"

extern "C" {
// Fills, for workgroup `bid`, out[0..20]: per class (128-row, 64-row, small) n_mine, id0, stride, n_sh,
// per_s, per_r; then the small class's dyn, n_units, n_double, ut, pool0, n_tiles.
void moesd_test_stream_schedule(int mode, int d, int I, int S, int T, int part_k, int shared_stream,
                                int n_small_e, int n_b64_e, int n_b128_e, int G, int bid,
                                int dyn_allowed, int fp8, int *out) {
  SchedIn in;
  in.mode = mode; in.d = d; in.I = I; in.S = S; in.T = T; in.part_k = part_k;
  in.shared_stream = shared_stream;
  in.n_small_e = n_small_e; in.n_b64_e = n_b64_e; in.n_b128_e = n_b128_e;
  in.G = G; in.bid = bid; in.dyn_allowed = dyn_allowed; in.fp8 = fp8;
  StreamSched sc;
  stream_schedule(in, nullptr, sc);
  const ClassCfg *cs[3] = {&sc.c128, &sc.c64, &sc.cs};
  for (int i = 0; i < 3; ++i) {
    out[6 * i + 0] = cs[i]->n_mine; out[6 * i + 1] = cs[i]->id0; out[6 * i + 2] = cs[i]->stride;
    out[6 * i + 3] = cs[i]->n_sh;   out[6 * i + 4] = cs[i]->per_s; out[6 * i + 5] = cs[i]->per_r;
  }
  out[18] = sc.cs.dyn; out[19] = sc.cs.n_units; out[20] = sc.cs.n_double;
  out[21] = sc.cs.ut;  out[22] = sc.cs.pool0;   out[23] = sc.cs.n_tiles;
}
// tiles [t0, t1) of drawn unit u
void moesd_test_unit_range(int n_units, int n_double, int ut, int pool0, int n_tiles, int u, int *t01) {
  ClassCfg c{};
  c.n_units = n_units; c.n_double = n_double; c.ut = ut; c.pool0 = pool0; c.n_tiles = n_tiles;
  unit_range(c, u, t01[0], t01[1]);
}
}
