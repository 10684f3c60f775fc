// Offline fold of the 128-point Walsh-Hadamard rotation into projection weights (Section III-C.2 / Fig. 7 of
// arXiv 2501.15021: H is merged into W_V and W_O, so the value rotation and the output un-rotation cost nothing
// online; akvq_quantize_append then takes AKVQ_V_PREROTATED and akvq_decode_attention AKVQ_OUT_ROTATED).
// Arithmetic as for cached rows: binary16 in, fp32 butterfly with strides 1, 2, ..., 64 in this order, times 2^-3.5,
// rounded to binary16 (nearest even).
#include "akvq_device.h"
#include "akvq_kernels.h"

namespace akvq {

namespace {

// x * 2^-3.5 rounded to fp32, then to binary16: the register barrier keeps the two roundings apart (the compiler would
// otherwise fuse the multiply into a mixed-precision instruction that rounds the exact product once)
__device__ __forceinline__ uint16_t scale_to_half(float x) {
  float y = __fmul_rn(x, inv_sqrt128());
  asm volatile("" : "+v"(y));
  return (uint16_t)float_to_half_bits_rne(y);
}

// axis 1: one wavefront per run of 128 consecutive columns of a row; lane l holds elements l and l + 64, so strides
// 1..32 exchange lanes (the lower lane keeps a+b, the upper one a-b) and stride 64 stays inside the lane
__global__ __launch_bounds__(256) void fold_columns_kernel(const uint16_t *w, uint16_t *out, long n_runs) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long run = (long)blockIdx.x * 4 + wave;
  if (run >= n_runs) return;
  const uint16_t *src = w + run * kD;
  float x0 = half_bits_to_float(src[lane]), x1 = half_bits_to_float(src[lane + 64]);
#pragma unroll
  for (int h = 1; h < kWave; h *= 2) {
    const float p0 = __shfl_xor(x0, h, kWave), p1 = __shfl_xor(x1, h, kWave);
    x0 = (lane & h) ? p0 - x0 : x0 + p0;
    x1 = (lane & h) ? p1 - x1 : x1 + p1;
  }
  const float s = x0 + x1, d = x0 - x1;
  out[run * kD + lane] = scale_to_half(s);
  out[run * kD + lane + 64] = scale_to_half(d);
}

// axis 0: one thread per column of a run of 128 rows (neighbouring threads read neighbouring columns)
__global__ __launch_bounds__(64) void fold_rows_kernel(const uint16_t *w, uint16_t *out, int cols) {
  const int c = blockIdx.x * 64 + threadIdx.x;
  if (c >= cols) return;
  const size_t base = (size_t)blockIdx.y * kD * cols + c;
  float u[kD];
#pragma unroll
  for (int e = 0; e < kD; ++e) u[e] = half_bits_to_float(w[base + (size_t)e * cols]);
#pragma unroll
  for (int h = 1; h < kD; h *= 2)
#pragma unroll
    for (int i = 0; i < kD; ++i)
      if ((i & h) == 0) {
        const float a = u[i], b = u[i + h];
        u[i] = a + b;
        u[i + h] = a - b;
      }
#pragma unroll
  for (int e = 0; e < kD; ++e)
    out[base + (size_t)e * cols] = scale_to_half(u[e]);
}

}  // namespace

hipError_t launch_fold_hadamard(const uint16_t *w, uint16_t *out, int rows, int cols, int axis, hipStream_t stream) {
  if (axis == 1) {
    const long n_runs = (long)rows * (cols / kD);
    hipLaunchKernelGGL(fold_columns_kernel, dim3((unsigned)((n_runs + 3) / 4)), dim3(256), 0, stream, w, out, n_runs);
  } else {
    hipLaunchKernelGGL(fold_rows_kernel, dim3((cols + 63) / 64, rows / kD), dim3(64), 0, stream, w, out, cols);
  }
  return hipGetLastError();
}

}  // namespace akvq
