// Weighted scatter-combine: out[t,:] = sum_s w[t,s] * y[inv[t*K+s],:] + g_t * ys[t,:]
// summed in slot order s = 0..K-1, then the shared expert, in fp32, and rounded
// once to bf16.  The shared expert's down projection arrives as n_parts partial
// sums over slices of its intermediate dimension; they are added first, in
// order.  One thread produces four adjacent output features.
#include "common.h"

__global__ __launch_bounds__(256) void combine_kernel(
    const float *__restrict__ y, const float *__restrict__ ys, int n_parts, const float *__restrict__ w,
    const float *__restrict__ gate, const int32_t *__restrict__ inv, int T, int K, int d,
    uint16_t *__restrict__ out, float *__restrict__ out_f32) {
  const int t = blockIdx.x;
  const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (c >= d) return;  // d is a multiple of 8, so a thread's four features are all valid
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < K; ++s) {
    const int p = inv[(size_t)t * K + s];
    const float ws = w[(size_t)t * K + s];
    const f32x4 v = *reinterpret_cast<const f32x4 *>(y + (size_t)p * d + c);
    acc[0] = fmaf(ws, v[0], acc[0]);
    acc[1] = fmaf(ws, v[1], acc[1]);
    acc[2] = fmaf(ws, v[2], acc[2]);
    acc[3] = fmaf(ws, v[3], acc[3]);
  }
  if (n_parts > 0) {
    const float g = gate[t];
    f32x4 v = *reinterpret_cast<const f32x4 *>(ys + (size_t)t * d + c);
    for (int p = 1; p < n_parts; ++p) {
      const f32x4 u = *reinterpret_cast<const f32x4 *>(ys + ((size_t)p * T + t) * d + c);
      v[0] += u[0];
      v[1] += u[1];
      v[2] += u[2];
      v[3] += u[3];
    }
    acc[0] = fmaf(g, v[0], acc[0]);
    acc[1] = fmaf(g, v[1], acc[1]);
    acc[2] = fmaf(g, v[2], acc[2]);
    acc[3] = fmaf(g, v[3], acc[3]);
  }
  u32x2 o;
  o[0] = f32_to_bf16_bits(acc[0]) | (f32_to_bf16_bits(acc[1]) << 16);
  o[1] = f32_to_bf16_bits(acc[2]) | (f32_to_bf16_bits(acc[3]) << 16);
  *reinterpret_cast<u32x2 *>(out + (size_t)t * d + c) = o;
  if (out_f32) *reinterpret_cast<f32x4 *>(out_f32 + (size_t)t * d + c) = acc;
}

hipError_t launch_combine(const float *y, const float *ys, int n_parts, const float *w,
                          const float *gate, const int32_t *inv, int T, int K, int d, uint16_t *out,
                          float *out_f32, hipStream_t s) {
  dim3 grid(T, (d / 4 + 255) / 256);
  hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, s, y, ys, n_parts, w, gate, inv, T, K, d, out,
                     out_f32);
  return hipGetLastError();
}
