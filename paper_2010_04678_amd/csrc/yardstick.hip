// Practical-peak yardsticks: what the device sustains on the two resources the fused MTTKRP is bound by
// (fp64 matrix instructions, HBM reads), measured with the simplest possible kernels.
#include "cals_internal.h"

namespace cals {

typedef double double4_t __attribute__((ext_vector_type(4)));

// Every wavefront issues `iters` x 16 independent-accumulator fp64 MFMAs on register operands.
__global__ void __launch_bounds__(256) yardstick_mfma_kernel(double* __restrict__ sink, int iters) {
  double4_t acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = double4_t{0.0, 0.0, 0.0, 0.0};
  const double a = 1.0 + 1e-3 * threadIdx.x, b = 1.0 - 1e-3 * (threadIdx.x & 15);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[j], 0, 0, 0);
  }
  double s = 0.0;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
  if (s == 123.456) sink[0] = s;          // keeps the loop alive; never true
}

// Grid-stride streaming read of n16 16-byte pieces, summed.
__global__ void __launch_bounds__(256) yardstick_read_kernel(const double2* __restrict__ src, int64_t n16,
                                                             double* __restrict__ sink) {
  double s = 0.0;
  const int64_t stride = (int64_t)gridDim.x * 256;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const double2 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    s += (v0.x + v0.y) + (v1.x + v1.y) + (v2.x + v2.y) + (v3.x + v3.y);
  }
  for (; i < n16; i += stride) s += src[i].x + src[i].y;
  if (s == 123.456) sink[0] = s;
}

hipError_t launch_yardstick(int kind, const void* buf, int64_t bytes, int reps, int num_cus, double* sink,
                            hipStream_t stream, double* value) {
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
  const int iters = 20000;
  const int mfma_blocks = num_cus * 8;
  const int64_t n16 = bytes / 16;
  const int read_blocks = num_cus * 8;
  for (int r = -1; r < reps; ++r) {       // r = -1: warm-up
    if (r == 0) (void)hipEventRecord(e0, stream);
    if (kind == 0)
      hipLaunchKernelGGL(yardstick_mfma_kernel, dim3(mfma_blocks), dim3(256), 0, stream, sink, iters);
    else
      hipLaunchKernelGGL(yardstick_read_kernel, dim3(read_blocks), dim3(256), 0, stream,
                         static_cast<const double2*>(buf), n16, sink);
  }
  (void)hipEventRecord(e1, stream);
  e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return e;
  const double sec = (double)ms * 1e-3 / reps;
  if (kind == 0)   // 16x16x4 MFMA = 2*16*16*4 flop per wavefront instruction; 4 wavefronts per block
    *value = 2048.0 * 16.0 * iters * 4.0 * mfma_blocks / sec * 1e-12;
  else
    *value = (double)(n16 * 16) / sec * 1e-9;
  return hipGetLastError();
}

}  // namespace cals
