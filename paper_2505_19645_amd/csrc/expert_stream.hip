// Expert FFN for few rows per expert: persistent weight-streaming kernels.
//
// While an expert sees few tokens the layer is bound by loading the activated
// experts' parameters (the k2*N term of the paper's Sec. 3.3 forward-time model;
// Sec. 3.2 shows that sparser models stay in this regime for longer).  These
// kernels are therefore built around the weight stream, not around the MFMA:
//
//  * One persistent workgroup per compute unit walks a list of equal-cost tiles
//    (static round-robin, so all workgroups finish together).  A tile is 32
//    weight rows (16 of w_gate + the same 16 of w_up, or 32 rows of w_down)
//    against one block of at most 16*NT token rows of one expert.
//  * The contraction dimension is cut into 256-element blocks ("stages").  Each
//    stage is fetched with global_load_lds_dwordx4: every wave instruction moves
//    two whole 512-byte row pieces, contiguous in HBM, straight into LDS without
//    touching a register, the weights with the non-temporal hint (each byte is
//    read exactly once).  D stages are kept in an LDS ring, so D-1 stages of
//    loads are always in flight across tile boundaries.
//  * The loads are issued and awaited by hand (s_waitcnt vmcnt with a computed
//    count, one s_barrier per stage): the compiler never sees a vector memory
//    load in the loop, so it cannot serialise the prefetch.
//  * MFMA operands come from LDS.  The 16-byte pieces of a row are stored
//    XOR-swizzled by (row & 7) so the 16-rows-by-4-pieces operand read is free
//    of bank conflicts while the DMA writes stay linear.
//  * The four waves split the eight 32-element MFMA steps of a stage; their
//    partial 16x16 tiles are added through LDS in a fixed order at the end of a
//    tile, so results do not depend on scheduling.
//
// MFMA operand use (v_mfma_f32_16x16x32_bf16): lane l = 16*q + r supplies 8
// consecutive contraction elements (piece 4*s + q of step s) of weight row r
// as A and of token row r as B; it receives, for token r, output features
// 4*q .. 4*q+3.
#include "common.h"

#define KB 256            // contraction elements per stage
#define ROW_BYTES 512     // KB * 2
#define A_BYTES 16384     // 2 matrices x 16 rows x 512 B
#define SMALL_M 16        // experts with at most this many rows go through the NT=1 phase
#define BIG_TB 64         // token rows per pass in the NT=4 phase

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

// ---- tile description (wave-uniform) ---------------------------------------------
struct Tile {
  const uint16_t *a0, *a1;  // first row of the two 16-row operand halves, at this tile's k origin
  long a_stride;            // elements between weight rows
  int rv0, rv1;             // valid rows in each half (>= 1 after clamping)
  const uint16_t *b;        // token-row matrix at this tile's k origin
  long b_stride;
  bool use_map;             // token rows go through row_token (sorted row -> token)
  int row0, m;              // first token row of the block, rows in the block
  int klen;                 // contraction length
  int out_i0;               // first output feature
  int out_n;                // number of output features of this group
  void *out;                // output matrix of this group
  int out_row0;             // output row of token row 0
};

struct PhaseCfg {
  int n_tiles;
  int n_shared_tiles;  // leading tiles that belong to the shared expert (0 if not in this phase)
  int tiles_r;         // row tiles per routed expert
  int tiles_s;         // row tiles of the shared expert
  int parts;           // k-parts of the shared down projection
  int part_k;
  int tb_rows;         // token rows per block in this phase
};

// The three lookup tables are separate __restrict__ kernel parameters so that the
// compiler can prove them unclobbered and read them through the scalar unit: a
// vector load here would make it wait for the whole prefetch queue.
struct Tables {
  const int32_t *__restrict__ plan;
  const int32_t *__restrict__ offsets;
  const int32_t *__restrict__ row_token;
};

template <int MODE>
__device__ __forceinline__ Tile decode_tile(const StreamArgs &a, const Tables &tb_, const PhaseCfg &pc,
                                            int idx, bool big) {
  Tile t;
  if (idx < pc.n_shared_tiles) {
    int rt, tb, part = 0;
    if (MODE == MODE_GATE_UP) {
      rt = idx % pc.tiles_s;
      tb = idx / pc.tiles_s;
    } else {
      rt = idx % pc.tiles_s;
      const int rest = idx / pc.tiles_s;
      part = rest % pc.parts;
      tb = rest / pc.parts;
    }
    t.use_map = false;
    t.row0 = tb * pc.tb_rows;
    t.m = min(a.T - t.row0, pc.tb_rows);
    t.out_row0 = t.row0;
    if (MODE == MODE_GATE_UP) {
      const int i0 = rt * 16;
      t.a0 = a.ws_gate + (size_t)i0 * a.d;
      t.a1 = a.ws_up + (size_t)i0 * a.d;
      t.a_stride = a.d;
      t.rv0 = t.rv1 = min(16, a.S - i0);
      t.b = a.x;
      t.b_stride = a.d;
      t.klen = a.d;
      t.out_i0 = i0;
      t.out_n = a.S;
      t.out = a.hs;
    } else {
      const int i0 = rt * 32;
      const int k0 = part * pc.part_k;
      t.a0 = a.ws_down + (size_t)i0 * a.S + k0;
      t.a1 = t.a0 + (size_t)16 * a.S;
      t.a_stride = a.S;
      t.rv0 = min(16, a.d - i0);
      t.rv1 = max(1, min(16, a.d - i0 - 16));
      if (a.d - i0 <= 16) t.a1 = t.a0;
      t.b = a.hs + k0;
      t.b_stride = a.S;
      t.klen = min(pc.part_k, a.S - k0);
      t.out_i0 = i0;
      t.out_n = a.d;
      t.out = a.ys + (size_t)part * a.T * a.d;
    }
    return t;
  }
  const int j = idx - pc.n_shared_tiles;
  const int entry = j / pc.tiles_r;
  const int rt = j % pc.tiles_r;
  int e, tb = 0;
  if (!big) {
    e = tb_.plan[PLAN_HDR + entry];
  } else {
    e = tb_.plan[PLAN_HDR + a.E + 2 * entry];
    tb = tb_.plan[PLAN_HDR + a.E + 2 * entry + 1];
  }
  const int beg = tb_.offsets[e], end = tb_.offsets[e + 1];
  t.row0 = beg + tb * pc.tb_rows;
  t.m = min(end - t.row0, pc.tb_rows);
  t.out_row0 = t.row0;
  if (MODE == MODE_GATE_UP) {
    const int i0 = rt * 16;
    t.a0 = a.w_gate + ((size_t)e * a.I + i0) * a.d;
    t.a1 = a.w_up + ((size_t)e * a.I + i0) * a.d;
    t.a_stride = a.d;
    t.rv0 = t.rv1 = min(16, a.I - i0);
    t.b = a.x;
    t.b_stride = a.d;
    t.use_map = true;
    t.klen = a.d;
    t.out_i0 = i0;
    t.out_n = a.I;
    t.out = a.h;
  } else {
    const int i0 = rt * 32;
    t.a0 = a.w_down + ((size_t)e * a.d + i0) * a.I;
    t.a1 = t.a0 + (size_t)16 * a.I;
    t.a_stride = a.I;
    t.rv0 = min(16, a.d - i0);
    t.rv1 = max(1, min(16, a.d - i0 - 16));
    if (a.d - i0 <= 16) t.a1 = t.a0;
    t.b = a.h;
    t.b_stride = a.I;
    t.use_map = false;
    t.klen = a.I;
    t.out_i0 = i0;
    t.out_n = a.d;
    t.out = a.y;
  }
  return t;
}

// Per-lane source pointers of the DMA instructions this wave issues for a tile.
template <int NT>
struct LoadPtrs {
  const uint16_t *a[4];
  const uint16_t *b[2 * NT];
  int klen;
  int nkb;
};

template <int NT>
__device__ __forceinline__ void setup_loads(LoadPtrs<NT> &lp, const Tile &t,
                                            const int32_t *__restrict__ row_token, int wave, int lane) {
  const int half = lane >> 5, slot = lane & 31;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = wave * 4 + i;       // 0..15: matrix = j >> 3, row pair = j & 7
    const int pair = j & 7;
    const int r = 2 * pair + half;
    const int piece = slot ^ (r & 7);
    const uint16_t *base = (j >> 3) ? t.a1 : t.a0;
    const int rv = (j >> 3) ? t.rv1 : t.rv0;
    lp.a[i] = base + (size_t)min(r, rv - 1) * t.a_stride + piece * 8;
  }
#pragma unroll
  for (int i = 0; i < 2 * NT; ++i) {
    const int jp = wave * 2 * NT + i;  // 0..8NT-1: token rows 2jp, 2jp+1
    const int ra = min(2 * jp, t.m - 1), rb = min(2 * jp + 1, t.m - 1);
    int ta = t.row0 + ra, tb = t.row0 + rb;
    if (t.use_map) {
      ta = row_token[ta];
      tb = row_token[tb];
    }
    const int tok = half ? tb : ta;
    const int r = 2 * jp + half;
    const int piece = slot ^ (r & 7);
    lp.b[i] = t.b + (size_t)tok * t.b_stride + piece * 8;
  }
  lp.klen = t.klen;
  lp.nkb = (t.klen + KB - 1) / KB;
}

// Issue one stage: exactly 4 + 2*NT loads per wave, always (addresses of pieces
// past the end of a row are pulled back inside it; their products are masked).
template <int NT>
__device__ __forceinline__ void issue_stage(const LoadPtrs<NT> &lp, int kb, uint32_t slot_base,
                                            int wave, int lane) {
  const int slot = lane & 31;
  const int k0 = kb * KB;
  if (k0 + KB <= lp.klen) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16_stream(lp.a[i] + k0, slot_base + (uint32_t)(wave * 4 + i) * 1024u);
#pragma unroll
    for (int i = 0; i < 2 * NT; ++i)
      dma16(lp.b[i] + k0, slot_base + A_BYTES + (uint32_t)(wave * 2 * NT + i) * 1024u);
  } else {
    // last, partial block: lp pointers already hold (slot ^ swz) * 8; undo it to clamp
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = wave * 4 + i;
      const int r = 2 * (j & 7) + (lane >> 5);
      const int piece = slot ^ (r & 7);
      const int k = min(k0 + piece * 8, lp.klen - 8);
      dma16_stream(lp.a[i] - piece * 8 + k, slot_base + (uint32_t)j * 1024u);
    }
#pragma unroll
    for (int i = 0; i < 2 * NT; ++i) {
      const int jp = wave * 2 * NT + i;
      const int r = 2 * jp + (lane >> 5);
      const int piece = slot ^ (r & 7);
      const int k = min(k0 + piece * 8, lp.klen - 8);
      dma16(lp.b[i] - piece * 8 + k, slot_base + A_BYTES + (uint32_t)jp * 1024u);
    }
  }
}

template <int MODE, int NT, int D>
__device__ __forceinline__ void run_phase(const StreamArgs &a, const Tables &tb_, const PhaseCfg &pc,
                                          bool big, char *smem) {
  constexpr int STAGE_BYTES = A_BYTES + NT * 16 * ROW_BYTES;
  constexpr int LW = 4 + 2 * NT;  // loads per wave per stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = uni(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  const int G = gridDim.x;

  // load cursor
  int l_tile = blockIdx.x, l_kb = 0, l_stage = 0;
  LoadPtrs<NT> lp;
  bool l_live = l_tile < pc.n_tiles;
  if (l_live) {
    const Tile t = decode_tile<MODE>(a, tb_, pc, l_tile, big);
    setup_loads<NT>(lp, t, tb_.row_token, wave, lane);
  }
  // compute cursor
  int c_tile = blockIdx.x, c_kb = 0, c_stage = 0;
  if (c_tile >= pc.n_tiles) return;
  Tile ct = decode_tile<MODE>(a, tb_, pc, c_tile, big);
  int c_nkb = (ct.klen + KB - 1) / KB;

  f32x4 acc0[NT], acc1[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    acc0[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    acc1[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  auto advance_load = [&]() {
    issue_stage<NT>(lp, l_kb, lds0 + (uint32_t)(l_stage % D) * STAGE_BYTES, wave, lane);
    ++l_stage;
    if (++l_kb == lp.nkb) {
      l_kb = 0;
      l_tile += G;
      l_live = l_tile < pc.n_tiles;
      if (l_live) {
        const Tile t = decode_tile<MODE>(a, tb_, pc, l_tile, big);
        setup_loads<NT>(lp, t, tb_.row_token, wave, lane);
      }
    }
  };

  // prologue: D-1 stages in flight
  for (int i = 0; i < D - 1 && l_live; ++i) advance_load();

  while (true) {
    // stage c_stage must have landed: at most the D-2 younger stages may be pending
    if (l_stage - c_stage == D - 1) wait_vm<(D - 2) * LW>();
    else wait_vm<0>();
    wg_barrier();
    if (l_live) advance_load();

    const char *sb = smem + (size_t)(c_stage % D) * STAGE_BYTES;
    const int ntc = (ct.m + 15) >> 4;
    const int kbase = c_kb * KB;
#pragma unroll
    for (int ss = 0; ss < 2; ++ss) {
      const int s = wave * 2 + ss;
      if (kbase + s * 32 < ct.klen) {
        const int piece = 4 * s + q;
        const int off = r16 * ROW_BYTES + ((piece ^ (r16 & 7)) << 4);
        const u32x4 fa0 = *reinterpret_cast<const u32x4 *>(sb + off);
        const u32x4 fa1 = *reinterpret_cast<const u32x4 *>(sb + 8192 + off);
        const bool live = kbase + piece * 8 < ct.klen;  // false only inside a ragged last step
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          if (nt < ntc) {
            u32x4 fb = *reinterpret_cast<const u32x4 *>(sb + A_BYTES + nt * 16 * ROW_BYTES + off);
            if (!live) fb = (u32x4){0u, 0u, 0u, 0u};
            acc0[nt] = mfma16(fa0, fb, acc0[nt]);
            acc1[nt] = mfma16(fa1, fb, acc1[nt]);
          }
      }
    }

    if (c_kb == c_nkb - 1) {
      // tile done: fold the four waves' partial tiles through the slot just consumed
      wg_barrier();
      float *red = reinterpret_cast<float *>(smem + (size_t)(c_stage % D) * STAGE_BYTES);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if (nt < ntc) {
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            red[((wave * NT + nt) * 2 + 0) * 256 + rr * 64 + lane] = acc0[nt][rr];
            red[((wave * NT + nt) * 2 + 1) * 256 + rr * 64 + lane] = acc1[nt][rr];
          }
          acc0[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
          acc1[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
      wg_barrier();
      {
        const int l2 = tid & 63, rr = tid >> 6;
        const int j = l2 & 15, fi = 4 * (l2 >> 4) + rr;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          if (nt < ntc) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              s0 += red[((w * NT + nt) * 2 + 0) * 256 + tid];
              s1 += red[((w * NT + nt) * 2 + 1) * 256 + tid];
            }
            const int pr = nt * 16 + j;
            if (pr < ct.m) {
              const size_t orow = (size_t)(ct.out_row0 + pr);
              if (MODE == MODE_GATE_UP) {
                const int i = ct.out_i0 + fi;
                if (i < ct.out_n)
                  reinterpret_cast<uint16_t *>(ct.out)[orow * ct.out_n + i] =
                      (uint16_t)f32_to_bf16_bits(silu_f32(s0) * s1);
              } else {
                float *y = reinterpret_cast<float *>(ct.out);
                const int i = ct.out_i0 + fi;
                if (i < ct.out_n) y[orow * ct.out_n + i] = s0;
                if (i + 16 < ct.out_n) y[orow * ct.out_n + i + 16] = s1;
              }
            }
          }
      }
      c_kb = 0;
      c_tile += G;
      ++c_stage;
      if (c_tile >= pc.n_tiles) break;
      ct = decode_tile<MODE>(a, tb_, pc, c_tile, big);
      c_nkb = (ct.klen + KB - 1) / KB;
    } else {
      ++c_kb;
      ++c_stage;
    }
  }
  // leave with nothing pending and the ring free for the next phase
  wait_vm<0>();
  wg_barrier();
}

template <int MODE>
__global__ __launch_bounds__(256) void expert_stream_kernel(StreamArgs a,
                                                            const int32_t *__restrict__ plan,
                                                            const int32_t *__restrict__ offsets,
                                                            const int32_t *__restrict__ row_token) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  Tables tb_{plan, offsets, row_token};
  const int n_small = plan[0], n_big = plan[1];
  const bool has_shared = a.S > 0;
  const int parts = (MODE == MODE_DOWN && has_shared) ? (a.S + a.part_k - 1) / a.part_k : 1;
  PhaseCfg pc;
  pc.tiles_r = (MODE == MODE_GATE_UP) ? (a.I + 15) / 16 : (a.d + 31) / 32;
  pc.tiles_s = (MODE == MODE_GATE_UP) ? (a.S + 15) / 16 : (a.d + 31) / 32;
  pc.parts = parts;
  pc.part_k = a.part_k;
  const bool shared_small = has_shared && a.T <= SMALL_M;
  // phase 1: groups with at most 16 rows, one n-tile
  pc.tb_rows = SMALL_M;
  pc.n_shared_tiles = shared_small ? pc.tiles_s * parts : 0;
  pc.n_tiles = pc.n_shared_tiles + n_small * pc.tiles_r;
  run_phase<MODE, 1, 6>(a, tb_, pc, false, smem);
  // phase 2: groups with more rows, passes of up to 64 rows
  pc.tb_rows = BIG_TB;
  pc.n_shared_tiles = (has_shared && !shared_small) ? pc.tiles_s * parts * ((a.T + BIG_TB - 1) / BIG_TB) : 0;
  pc.n_tiles = pc.n_shared_tiles + n_big * pc.tiles_r;
  run_phase<MODE, 4, 3>(a, tb_, pc, true, smem);
}

#define STREAM_LDS_BYTES (144 * 1024)

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
