// Second step of the two-step sweep (reuse of a partial contraction across two mode updates; the scheme the
// paper's related-work section attributes to Phan et al., and names as compatible with CALS):
//   Y[(i2,i3), c] = sum_i1 T[i1,i2,i3] * U1[i1,c]            -- one GEMM-shaped pass over the tensor (the fused
//                                                               MTTKRP kernel with a row of ones as second factor)
//   M2[i2, c] = sum_i3 Y[(i2,i3), c] * U3[i3,c],   M3[i3, c] = sum_i2 Y[(i2,i3), c] * U2[i2,c]
// This file holds the column-wise contraction of Y with one factor (HBM-bound: Y is read once per use).
#include "cals_internal.h"

namespace cals {

// M[o, c] = sum_{s < ns} Y[(o*so + s*ss) * ld + c] * U[s * ld + c],  o < no, c < ncols.
// Workgroup = 64 column lanes x 4 groups of the s range; each group sums its quarter in ascending s, the four
// partial sums are added left to right (fixed order: bit-reproducible).
template <bool PAIR>
__global__ void __launch_bounds__(256) ttv_kernel(const double* __restrict__ Y, const double* __restrict__ U,
                                                  double* __restrict__ M, int no, int ns, int64_t so, int64_t ss, int ld,
                                                  int ncols, int ncb) {
  constexpr int PW = PAIR ? 2 : 1;
  __shared__ double part[4][64][PW];
  const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int o = blockIdx.x / ncb, cb = blockIdx.x % ncb;
  const int c = (cb * 64 + lane) * PW;
  const bool live = c < ncols;                   // PAIR: c + 1 < ld always (ld even), stored only when < ncols
  const int per = (ns + 3) / 4;
  const int s0 = g * per, s1 = (s0 + per < ns) ? (s0 + per) : ns;
  double acc[PW];
#pragma unroll
  for (int w = 0; w < PW; ++w) acc[w] = 0.0;
  if (live) {
    const double* y = Y + ((int64_t)o * so + (int64_t)s0 * ss) * ld + c;
    const double* u = U + (int64_t)s0 * ld + c;
    const int64_t ystep = ss * ld;
    int s = s0;
    for (; s + 4 <= s1; s += 4) {                // four rows in flight; added in ascending s
      double yv[4][PW], uv[4][PW];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (PAIR) {
          const double2 a = *reinterpret_cast<const double2*>(y + q * ystep);
          const double2 b = *reinterpret_cast<const double2*>(u + (int64_t)q * ld);
          yv[q][0] = a.x; yv[q][PW - 1] = a.y;
          uv[q][0] = b.x; uv[q][PW - 1] = b.y;
        } else {
          yv[q][0] = y[q * ystep];
          uv[q][0] = u[(int64_t)q * ld];
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int w = 0; w < PW; ++w) acc[w] += yv[q][w] * uv[q][w];
      y += 4 * ystep;
      u += 4 * (int64_t)ld;
    }
    for (; s < s1; ++s, y += ystep, u += ld)
#pragma unroll
      for (int w = 0; w < PW; ++w) acc[w] += y[w] * u[w];
  }
#pragma unroll
  for (int w = 0; w < PW; ++w) part[g][lane][w] = acc[w];
  __syncthreads();
  if (g == 0 && live) {
#pragma unroll
    for (int w = 0; w < PW; ++w) {
      if (c + w < ncols)
        M[(int64_t)o * ld + c + w] = ((part[0][lane][w] + part[1][lane][w]) + part[2][lane][w]) + part[3][lane][w];
    }
  }
}

hipError_t launch_ttv(const double* Y, const double* U, double* M, int no, int ns, int64_t so, int64_t ss, int ld,
                      int ncols, hipStream_t stream) {
  if (no < 1 || ns < 1 || ncols < 1 || ncols > ld) return hipErrorInvalidValue;
  const bool pair = (ld % 2 == 0) &&
                    ((reinterpret_cast<uintptr_t>(Y) | reinterpret_cast<uintptr_t>(U)) & 15) == 0;
  const int per_block = pair ? 128 : 64;
  const int ncb = (ncols + per_block - 1) / per_block;
  const int64_t nblocks = (int64_t)no * ncb;
  if (nblocks >= (1LL << 31)) return hipErrorInvalidValue;
  if (pair)
    hipLaunchKernelGGL(ttv_kernel<true>, dim3((unsigned)nblocks), dim3(256), 0, stream, Y, U, M, no, ns, so, ss, ld, ncols, ncb);
  else
    hipLaunchKernelGGL(ttv_kernel<false>, dim3((unsigned)nblocks), dim3(256), 0, stream, Y, U, M, no, ns, so, ss, ld, ncols, ncb);
  return hipGetLastError();
}

__global__ void __launch_bounds__(256) fill_kernel(double* __restrict__ p, int64_t n, double v) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

hipError_t launch_fill(double* p, int64_t n, double v, hipStream_t stream) {
  if (n < 1) return hipSuccess;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n, v);
  return hipGetLastError();
}

}  // namespace cals
