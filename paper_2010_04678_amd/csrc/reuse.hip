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

// Second step for tensors of order above 3: the intermediate Y has one row per index tuple (i2, ..., iN); for output
// mode n the other modes form a fast run L (modes 2..n-1, PL combined indices) and a slow run R (modes n+1..N, PR):
//   M[o, c] = sum_{r < PR} sum_{l < PL} Y[(l + PL * (o + no * r)) * ld + c] * KL[l * ld + c] * KR[r * ld + c],
// KL / KR being a factor multi-matrix, the explicit Khatri-Rao product of a run, or a single row of ones.
// Grid (output rows x column blocks, slices of the flattened (l, r) range): a workgroup = 64 column lanes (x 2
// columns) x 4 groups that cut its slice in four; every group sums in ascending order (four loads in flight along
// a run of l), the four partial sums are added left to right; with more than one slice the slices' results go to a
// workspace and are added in slice order by the split-K reduction kernel (fixed order: reproducible).
template <bool PAIR>
__global__ void __launch_bounds__(256) ttv2_kernel(const double* __restrict__ Y, const double* __restrict__ KL,
                                                   const double* __restrict__ KR, double* __restrict__ out, int no, int PL,
                                                   int PR, int ld, int ncols, int ncb, int64_t slice, int64_t ostride) {
  constexpr int PW = PAIR ? 2 : 1;
  __shared__ double part[4][64][PW];
  const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int o = blockIdx.x / ncb, cb = blockIdx.x % ncb;
  const int c = (cb * 64 + lane) * PW;
  const bool live = c < ncols;
  const int64_t total = (int64_t)PL * PR;
  const int64_t z0 = (int64_t)blockIdx.y * slice;
  const int64_t z1 = (z0 + slice < total) ? (z0 + slice) : total;
  const int64_t per = (z1 - z0 + 3) / 4;
  const int64_t s0 = z0 + g * per, s1 = (s0 + per < z1) ? (s0 + per) : z1;
  double acc[PW];
#pragma unroll
  for (int w = 0; w < PW; ++w) acc[w] = 0.0;
  if (live && s0 < s1) {
    int r = (int)(s0 / PL), l = (int)(s0 - (int64_t)r * PL);
    int64_t s = s0;
    while (s < s1) {
      // a run of consecutive l with the same r
      const int64_t left = s1 - s;
      const int nrun = (PL - l < left) ? (PL - l) : (int)left;
      const double* y = Y + ((int64_t)l + (int64_t)PL * ((int64_t)o + (int64_t)no * r)) * ld + c;
      const double* kl = KL + (int64_t)l * ld + c;
      double rv[PW];
#pragma unroll
      for (int w = 0; w < PW; ++w) rv[w] = KR[(int64_t)r * ld + c + w];
      int t = 0;
      for (; t + 4 <= nrun; t += 4) {
        double yv[4][PW], lv[4][PW];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (PAIR) {
            const double2 a = *reinterpret_cast<const double2*>(y + (int64_t)q * ld);
            const double2 b = *reinterpret_cast<const double2*>(kl + (int64_t)q * ld);
            yv[q][0] = a.x; yv[q][PW - 1] = a.y;
            lv[q][0] = b.x; lv[q][PW - 1] = b.y;
          } else {
            yv[q][0] = y[(int64_t)q * ld];
            lv[q][0] = kl[(int64_t)q * ld];
          }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int w = 0; w < PW; ++w) acc[w] += yv[q][w] * (lv[q][w] * rv[w]);
        y += 4 * (int64_t)ld;
        kl += 4 * (int64_t)ld;
      }
      for (; t < nrun; ++t, y += ld, kl += ld)
#pragma unroll
        for (int w = 0; w < PW; ++w) acc[w] += y[w] * (kl[w] * rv[w]);
      s += nrun;
      l += nrun;
      if (l == PL) { l = 0; ++r; }
    }
  }
#pragma unroll
  for (int w = 0; w < PW; ++w) part[g][lane][w] = acc[w];
  __syncthreads();
  if (g == 0 && live) {
    double* dst = out + (int64_t)blockIdx.y * ostride + (int64_t)o * ld + c;
#pragma unroll
    for (int w = 0; w < PW; ++w)
      if (c + w < ncols) dst[w] = ((part[0][lane][w] + part[1][lane][w]) + part[2][lane][w]) + part[3][lane][w];
  }
}

// Slices of the (l, r) range for launch_ttv2: enough workgroups to keep the memory system busy (about four per CU).
int ttv2_slices(int no, int PL, int PR, int ld, int ncols, int num_cus) {
  const int per_block = (ld % 2 == 0) ? 128 : 64;
  const int64_t base = (int64_t)no * ((ncols + per_block - 1) / per_block);
  const int64_t total = (int64_t)PL * PR;
  int64_t g = (4 * (int64_t)num_cus + base - 1) / base;
  const int64_t most = total / 64 > 1 ? total / 64 : 1;      // at least 64 steps per slice
  if (g > most) g = most;
  if (g > 64) g = 64;
  return (int)(g < 1 ? 1 : g);
}

hipError_t launch_ttv2(const double* Y, const double* KL, int PL, const double* KR, int PR, double* M, int no, int ld,
                       int ncols, int slices, double* workspace, hipStream_t stream) {
  if (no < 1 || PL < 1 || PR < 1 || ncols < 1 || ncols > ld || !Y || !KL || !KR || !M) return hipErrorInvalidValue;
  if (slices < 1 || slices > 65535 || (slices > 1 && !workspace)) return hipErrorInvalidValue;
  const bool pair = (ld % 2 == 0) && ((reinterpret_cast<uintptr_t>(Y) | reinterpret_cast<uintptr_t>(KL) |
                                       reinterpret_cast<uintptr_t>(KR)) & 15) == 0;
  const int per_block = pair ? 128 : 64;
  const int ncb = (ncols + per_block - 1) / per_block;
  const int64_t nblocks = (int64_t)no * ncb;
  if (nblocks >= (1LL << 31)) return hipErrorInvalidValue;
  const int64_t total = (int64_t)PL * PR;
  const int64_t slice = (total + slices - 1) / slices;
  const int64_t ostride = (int64_t)no * ld;
  double* out = slices > 1 ? workspace : M;
  const dim3 grid((unsigned)nblocks, (unsigned)slices);
  if (pair)
    hipLaunchKernelGGL(ttv2_kernel<true>, grid, dim3(256), 0, stream, Y, KL, KR, out, no, PL, PR, ld, ncols, ncb, slice, ostride);
  else
    hipLaunchKernelGGL(ttv2_kernel<false>, grid, dim3(256), 0, stream, Y, KL, KR, out, no, PL, PR, ld, ncols, ncb, slice, ostride);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || slices == 1) return e;
  return launch_splitk_reduce(workspace, M, ostride, ld, ncols, slices, stream);
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
