// Expert FFN for few rows per expert: weight-streaming skinny GEMMs on MFMA.
//
// While an expert sees few tokens the layer is bound by loading the activated
// experts' parameters (the k2*N term of the paper's Sec. 3.3 forward-time model;
// Sec. 3.2 shows that sparser models stay in this regime for longer).  So the
// kernels below are organised around the weight stream: each 16-byte piece of a
// weight matrix is fetched from HBM exactly once, straight into the registers
// of the one wave that needs it, and multiplied against up to 64 token rows with
// v_mfma_f32_16x16x32_bf16.  The token rows (a few KB) come through the caches.
//
// Work split: blockIdx.y picks the group (routed expert e < E, or the shared
// expert as group E), blockIdx.x a tile of 16 output features.  The four waves
// of a workgroup split the contraction dimension in 128-element chunks and add
// their partial 16x16 tiles through LDS in a fixed order, so results do not
// depend on scheduling.
//
// MFMA operand use (16x16x32, bf16): lane l = 16*q + r supplies, for the A
// operand, 8 consecutive contraction elements of weight row r, and for the B
// operand the same 8 elements of token row r; the result lane holds, for token
// r, output features 4*q .. 4*q+3.  Which 8 elements belong to (q, step j) is
// free as long as A and B agree: here q owns bytes [64q, 64q+64) of each 256-byte
// chunk, so a wave's loads cover 16 rows x 256 contiguous bytes.
#include "common.h"

#define ES_CHUNK 128  // contraction elements per wave step (256 bytes per row)

template <int NT>
struct Frag {
  u32x4 a1[4], a2[4];
  u32x4 b[NT][4];
};

// load one chunk's operands.  kq = element offset of this lane's 64-byte piece;
// pieces beyond the contraction length are zero (so are their B partners).
template <int NT, bool TWO>
__device__ __forceinline__ void load_frag(Frag<NT> &f, const uint16_t *pa1, const uint16_t *pa2,
                                          const uint16_t *const (&pb)[NT], int kq, int klen,
                                          int ntc) {
  const u32x4 zero = {0u, 0u, 0u, 0u};
  if (kq + 32 <= klen) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f.a1[j] = ld16_stream(pa1 + kq + j * 8);
      if (TWO) f.a2[j] = ld16_stream(pa2 + kq + j * 8);
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      if (nt < ntc) {
#pragma unroll
        for (int j = 0; j < 4; ++j) f.b[nt][j] = ld16(pb[nt] + kq + j * 8);
      }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool ok = kq + j * 8 < klen;  // klen is a multiple of 8
      f.a1[j] = ok ? ld16_stream(pa1 + kq + j * 8) : zero;
      if (TWO) f.a2[j] = ok ? ld16_stream(pa2 + kq + j * 8) : zero;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if (nt < ntc) f.b[nt][j] = ok ? ld16(pb[nt] + kq + j * 8) : zero;
    }
  }
}

// ---------------------------------------------------------------------------
// gate/up + SwiGLU:  h[p, i] = silu(x_p . wg[i,:]) * (x_p . wu[i,:])
// ---------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(256) void gate_up_stream_kernel(ExpertArgs a) {
  const int g = blockIdx.y;
  const bool shared = (g == a.E);
  int row0, m, N;
  const uint16_t *wg, *wu;
  uint16_t *h;
  if (!shared) {
    row0 = a.offsets[g];
    m = a.offsets[g + 1] - row0;
    N = a.I;
    wg = a.w_gate + (size_t)g * a.I * a.d;
    wu = a.w_up + (size_t)g * a.I * a.d;
    h = a.h;
  } else {
    row0 = 0;
    m = a.T;
    N = a.S;
    wg = a.ws_gate;
    wu = a.ws_up;
    h = a.hs;
  }
  const int i0 = blockIdx.x * 16;
  if (m <= 0 || i0 >= N) return;

  __shared__ float red[4][NT][2][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int d = a.d;
  const int arow = min(i0 + r, N - 1);
  const uint16_t *pg = wg + (size_t)arow * d;
  const uint16_t *pu = wu + (size_t)arow * d;
  const int nchunk = (d + ES_CHUNK - 1) / ES_CHUNK;

  for (int mb = 0; mb < m; mb += 16 * NT) {
    const int ntc = min(NT, (m - mb + 15) / 16);
    const uint16_t *pb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int p = row0 + min(mb + nt * 16 + r, m - 1);
      const int tok = shared ? p : a.perm[p] / a.K;
      pb[nt] = a.x + (size_t)tok * d;
    }
    f32x4 accg[NT], accu[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      accg[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      accu[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    Frag<NT> cur, nxt;
    int c = wave;
    if (c < nchunk) load_frag<NT, true>(cur, pg, pu, pb, c * ES_CHUNK + q * 32, d, ntc);
    for (; c < nchunk; c += 4) {
      const bool more = c + 4 < nchunk;
      if (more) load_frag<NT, true>(nxt, pg, pu, pb, (c + 4) * ES_CHUNK + q * 32, d, ntc);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if (nt < ntc) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            accg[nt] = mfma16(cur.a1[j], cur.b[nt][j], accg[nt]);
            accu[nt] = mfma16(cur.a2[j], cur.b[nt][j], accu[nt]);
          }
        }
      if (more) cur = nxt;
    }
    // fold the four waves' partial tiles (fixed order) and apply SwiGLU
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      if (nt < ntc) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          red[wave][nt][0][rr * 64 + lane] = accg[nt][rr];
          red[wave][nt][1][rr * 64 + lane] = accu[nt][rr];
        }
      }
    __syncthreads();
    {
      const int l2 = tid & 63, rr = tid >> 6;
      const int j = l2 & 15, i = i0 + 4 * (l2 >> 4) + rr;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if (nt < ntc) {
          const float gsum = ((red[0][nt][0][tid] + red[1][nt][0][tid]) + red[2][nt][0][tid]) +
                             red[3][nt][0][tid];
          const float usum = ((red[0][nt][1][tid] + red[1][nt][1][tid]) + red[2][nt][1][tid]) +
                             red[3][nt][1][tid];
          const int pr = mb + nt * 16 + j;
          if (pr < m && i < N)
            h[(size_t)(row0 + pr) * N + i] = (uint16_t)f32_to_bf16_bits(silu_f32(gsum) * usum);
        }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// down:  y[p, c] = sum_i h[p, i] * wd[c, i]
// ---------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(256) void down_stream_kernel(ExpertArgs a) {
  const int g = blockIdx.y;
  const bool shared = (g == a.E);
  int row0, m, Kc;
  const uint16_t *wd, *hb;
  float *y;
  if (!shared) {
    row0 = a.offsets[g];
    m = a.offsets[g + 1] - row0;
    Kc = a.I;
    wd = a.w_down + (size_t)g * a.d * a.I;
    hb = a.h;
    y = a.y;
  } else {
    row0 = 0;
    m = a.T;
    Kc = a.S;
    wd = a.ws_down;
    hb = a.hs;
    y = a.ys;
  }
  const int N = a.d;
  const int i0 = blockIdx.x * 16;
  if (m <= 0 || i0 >= N) return;

  __shared__ float red[4][NT][256];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, q = lane >> 4;
  const int arow = min(i0 + r, N - 1);
  const uint16_t *pa = wd + (size_t)arow * Kc;
  const int nchunk = (Kc + ES_CHUNK - 1) / ES_CHUNK;

  for (int mb = 0; mb < m; mb += 16 * NT) {
    const int ntc = min(NT, (m - mb + 15) / 16);
    const uint16_t *pb[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int p = row0 + min(mb + nt * 16 + r, m - 1);
      pb[nt] = hb + (size_t)p * Kc;
    }
    f32x4 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    Frag<NT> cur, nxt;
    int c = wave;
    if (c < nchunk) load_frag<NT, false>(cur, pa, pa, pb, c * ES_CHUNK + q * 32, Kc, ntc);
    for (; c < nchunk; c += 4) {
      const bool more = c + 4 < nchunk;
      if (more) load_frag<NT, false>(nxt, pa, pa, pb, (c + 4) * ES_CHUNK + q * 32, Kc, ntc);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if (nt < ntc) {
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[nt] = mfma16(cur.a1[j], cur.b[nt][j], acc[nt]);
        }
      if (more) cur = nxt;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      if (nt < ntc) {
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) red[wave][nt][rr * 64 + lane] = acc[nt][rr];
      }
    __syncthreads();
    {
      const int l2 = tid & 63, rr = tid >> 6;
      const int j = l2 & 15, i = i0 + 4 * (l2 >> 4) + rr;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        if (nt < ntc) {
          const float s = ((red[0][nt][tid] + red[1][nt][tid]) + red[2][nt][tid]) + red[3][nt][tid];
          const int pr = mb + nt * 16 + j;
          if (pr < m && i < N) y[(size_t)(row0 + pr) * N + i] = s;
        }
    }
    __syncthreads();
  }
}

static int pick_nt(int T) { return T <= 16 ? 1 : (T <= 32 ? 2 : 4); }

hipError_t launch_gate_up(const ExpertArgs &a, hipStream_t s) {
  const int nmax = a.I > a.S ? a.I : a.S;
  dim3 grid((nmax + 15) / 16, a.E + (a.S > 0 ? 1 : 0));
  switch (pick_nt(a.T)) {
    case 1: hipLaunchKernelGGL(gate_up_stream_kernel<1>, grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL(gate_up_stream_kernel<2>, grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL(gate_up_stream_kernel<4>, grid, dim3(256), 0, s, a); break;
  }
  return hipGetLastError();
}

hipError_t launch_down(const ExpertArgs &a, hipStream_t s) {
  dim3 grid((a.d + 15) / 16, a.E + (a.S > 0 ? 1 : 0));
  switch (pick_nt(a.T)) {
    case 1: hipLaunchKernelGGL(down_stream_kernel<1>, grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL(down_stream_kernel<2>, grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL(down_stream_kernel<4>, grid, dim3(256), 0, s, a); break;
  }
  return hipGetLastError();
}
