// Line search for CALS (Sec. 5 of the paper, "Line search"), applied to each model independently after a
// round's mode updates: P_new = P_prev + alpha (P_cur - P_prev); the extrapolated point replaces P_cur
// only if its error is lower.  The error of P_new comes from the fast formula of Alg. 1 with ONE extra fused
// MTTKRP over the extrapolated multi-matrices, so the central fused operation is preserved.  The inner product
// <T, model> is sum(A_n * M_n) for any mode n, so the host picks the mode whose MTTKRP runs best (the longest one;
// the last one when it comes from the two-step contraction).
// With two-step sweeps the tensor contracted with the mode-1 factors of the extrapolated point is the same
// combination of the contractions at P_prev and P_cur (the contraction is linear in those factors), so the extra
// MTTKRP needs no pass over the tensor.
#include "cals_internal.h"

namespace cals {

constexpr int kRows = 256;
constexpr int kXs = kRows + 1;

__device__ inline bool ls_takes_part(const ModelDesc& d, const ModelOut& o) {
  return (d.flags & 2u) && o.status == 0 && o.iters >= 2;
}

__device__ inline double ls_block_sum(double v, double* red) {
  const int tid = threadIdx.x;
  red[tid] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  const double r = red[0];
  __syncthreads();
  return r;
}

__global__ void __launch_bounds__(256) ls_extrapolate_kernel(LineSearchArgs a) {
  const int mode = blockIdx.y;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)a.In[mode] * a.ncols) return;
  const int i = (int)(idx / a.ncols), c = (int)(idx % a.ncols);
  const ModelDesc d = a.desc[a.colmodel[c]];
  const ModelOut o = a.out[d.sid];
  const int64_t e = (int64_t)i * a.ld + c;
  const double scale = (mode == a.nmodes - 1) ? a.lambda[d.sid * kMaxRank + (c - d.col)] : 1.0;
  const double cur = a.U[mode][e] * scale;
  double v = cur;
  if (ls_takes_part(d, o)) {
    const double prev = a.Uprev[mode][e];
    v = prev + d.alpha * (cur - prev);
    if ((d.flags & 1u) && !(v > 0.0)) v = 0.0;   // NONNEG models: projected back onto the feasible set
  }
  a.Unew[mode][e] = v;
}

// grid (n_models, modes, row blocks): partial Gramian of the extrapolated mode-`y` factor block over the block's rows;
// for the last mode also the partial sum(A_new * M).  Partials go to a.part; ls_decide_kernel adds them in block order.
__global__ void __launch_bounds__(256) ls_gram_kernel(LineSearchArgs a) {
  extern __shared__ double lds[];
  const ModelDesc d = a.desc[blockIdx.x];
  const ModelOut o = a.out[d.sid];
  if (!ls_takes_part(d, o)) return;
  const int mode = blockIdx.y, tid = threadIdx.x, R = d.rank, In = a.In[mode];
  const int nblk = gridDim.z;
  const int rpb = ((In + nblk - 1) / nblk + kRows - 1) / kRows * kRows;
  const int r0 = blockIdx.z * rpb;
  const int r1 = (r0 + rpb < In) ? (r0 + rpb) : In;
  double* xs = lds;                 // R x kXs staged rows
  double* red = xs + kMaxRank * kXs;
  const double* Ub = a.Unew[mode] + d.col;
  const int npairs = R * (R + 1) / 2;
  double gacc[3] = {0.0, 0.0, 0.0};
  double inner = 0.0;
  for (int base = r0; base < r1; base += kRows) {
    const int i = base + tid;
    const int nrows = (r1 - base < kRows) ? (r1 - base) : kRows;
    if (i < r1) {
      double part = 0.0;
      for (int r = 0; r < R; ++r) {
        const double x = Ub[(int64_t)i * a.ld + r];
        xs[r * kXs + tid] = x;
        if (mode == a.ls_mode) part += x * a.M3[(int64_t)i * a.ld + d.col + r];
      }
      inner += part;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const int p = tid + 256 * q;
      if (p < npairs) {
        int r = (int)((sqrt(8.0 * p + 1.0) - 1.0) * 0.5);
        while (r * (r + 1) / 2 > p) --r;
        while ((r + 1) * (r + 2) / 2 <= p) ++r;
        const int s = p - r * (r + 1) / 2;
        double acc = gacc[q];
        for (int j = 0; j < nrows; ++j) acc += xs[r * kXs + j] * xs[s * kXs + j];
        gacc[q] = acc;
      }
    }
    __syncthreads();
  }
  double* part = a.part + (((size_t)blockIdx.x * a.nmodes + mode) * nblk + blockIdx.z) * kUpdatePartStride;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const int p = tid + 256 * q;
    if (p < npairs) part[p] = gacc[q];
  }
  if (mode == a.ls_mode) {
    const double tot = ls_block_sum(inner, red);
    if (tid == 0) part[528] = tot;
  }
}

// grid (n_models): error of the extrapolated point and the decision.
__global__ void __launch_bounds__(256) ls_decide_kernel(LineSearchArgs a) {
  __shared__ double red[256];
  const ModelDesc d = a.desc[blockIdx.x];
  ModelOut* o = a.out + d.sid;
  const int tid = threadIdx.x;
  if (!ls_takes_part(d, *o)) {
    if (tid == 0) a.accept[blockIdx.x] = 0;
    return;
  }
  ModelState* st = a.state + d.sid;
  const int R = d.rank;
  // Gramians of the extrapolated point: the row blocks' partials, added in block order
  const int npairs = R * (R + 1) / 2;
  for (int mode = 0; mode < a.nmodes; ++mode) {
    const double* pm = a.part + ((size_t)blockIdx.x * a.nmodes + mode) * a.nblk * kUpdatePartStride;
    for (int p = tid; p < npairs; p += 256) {
      double g = 0.0;
      for (int b = 0; b < a.nblk; ++b) g += pm[(size_t)b * kUpdatePartStride + p];
      int r = (int)((sqrt(8.0 * p + 1.0) - 1.0) * 0.5);
      while (r * (r + 1) / 2 > p) --r;
      while ((r + 1) * (r + 2) / 2 <= p) ++r;
      const int c = p - r * (r + 1) / 2;
      st->Gls[mode][r * R + c] = g;
      st->Gls[mode][c * R + r] = g;
    }
  }
  if (tid == 0) {
    const double* pm = a.part + ((size_t)blockIdx.x * a.nmodes + a.ls_mode) * a.nblk * kUpdatePartStride;
    double in = 0.0;
    for (int b = 0; b < a.nblk; ++b) in += pm[(size_t)b * kUpdatePartStride + 528];
    st->inner_ls = in;
  }
  __syncthreads();
  double part = 0.0;
  for (int e = tid; e < R * R; e += 256) {
    double h = st->Gls[0][e];
    for (int k = 1; k < a.nmodes; ++k) h *= st->Gls[k][e];
    part += h;
  }
  const double normsq = ls_block_sum(part, red);
  const double err = a.normT2 + normsq - 2.0 * st->inner_ls;
  const bool take = err < o->err;             // uniform: every thread reads the same values
  __syncthreads();
  if (take) {
    for (int k = 0; k < a.nmodes; ++k)
      for (int e = tid; e < R * R; e += 256) st->G[k][e] = st->Gls[k][e];
    if (tid < R) a.lambda[d.sid * kMaxRank + tid] = 1.0;
  }
  __syncthreads();
  if (tid == 0) {
    a.accept[blockIdx.x] = take ? 1 : 0;
    if (take) {
      o->err = err;
      o->fit = 1.0 - sqrt(err > 0.0 ? err : 0.0) / sqrt(a.normT2);
      o->ls_accepted += 1;
    }
  }
}

__global__ void __launch_bounds__(256) ls_apply_kernel(LineSearchArgs a) {
  const int mode = blockIdx.y;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)a.In[mode] * a.ncols) return;
  const int i = (int)(idx / a.ncols), c = (int)(idx % a.ncols);
  const int k = a.colmodel[c];
  const ModelDesc d = a.desc[k];
  if (!(d.flags & 2u)) return;
  const ModelOut o = a.out[d.sid];
  if (o.status != 0) return;
  const int64_t e = (int64_t)i * a.ld + c;
  double v;
  if (a.accept[k]) {
    v = a.Unew[mode][e];
    a.U[mode][e] = v;                          // lambda of an accepted point is 1
  } else {
    v = a.U[mode][e];
    if (mode == a.nmodes - 1) v *= a.lambda[d.sid * kMaxRank + (c - d.col)];
  }
  a.Uprev[mode][e] = v;
}

// grid (column blocks of 256, row chunks): thread = one column over the chunk's rows (coalesced along the columns)
template <bool KEEP>
__global__ void __launch_bounds__(256) ls_y_kernel(LineSearchArgs a, int rows_per_block) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= a.ncols) return;
  const int k = a.colmodel[c];
  const ModelDesc d = a.desc[k];
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
  const int64_t r1 = (r0 + rows_per_block < a.yrows) ? (r0 + rows_per_block) : a.yrows;
  if (KEEP) {
    const double* src = a.accept[k] ? a.Ynew : a.Ycur;
    for (int64_t i = r0; i < r1; ++i) a.Yprev[i * a.ld + c] = src[i * a.ld + c];
  } else {
    const bool part = ls_takes_part(d, a.out[d.sid]);
    const double alpha = d.alpha;
    for (int64_t i = r0; i < r1; ++i) {
      const double cur = a.Ycur[i * a.ld + c];
      double v = cur;
      if (part) {
        const double prev = a.Yprev[i * a.ld + c];
        v = prev + alpha * (cur - prev);
      }
      a.Ynew[i * a.ld + c] = v;
    }
  }
}

template <bool KEEP>
static hipError_t launch_ls_y(const LineSearchArgs& a, hipStream_t stream) {
  if (a.n_models < 1 || a.ncols < 1 || a.yrows < 1) return hipSuccess;
  if (!a.Ycur || !a.Yprev || !a.Ynew) return hipErrorInvalidValue;
  int rows_per_block = 8;
  while ((a.yrows + rows_per_block - 1) / rows_per_block > 65535) rows_per_block *= 2;
  const dim3 grid((a.ncols + 255) / 256, (unsigned)((a.yrows + rows_per_block - 1) / rows_per_block));
  hipLaunchKernelGGL(ls_y_kernel<KEEP>, grid, dim3(256), 0, stream, a, rows_per_block);
  return hipGetLastError();
}
hipError_t launch_ls_y_combine(const LineSearchArgs& a, hipStream_t stream) { return launch_ls_y<false>(a, stream); }
hipError_t launch_ls_y_keep(const LineSearchArgs& a, hipStream_t stream) { return launch_ls_y<true>(a, stream); }

static dim3 elem_grid(const LineSearchArgs& a) {
  int imax = a.In[0];
  for (int k = 1; k < a.nmodes; ++k) imax = imax > a.In[k] ? imax : a.In[k];
  const int64_t total = (int64_t)imax * a.ncols;
  return dim3((unsigned)((total + 255) / 256), a.nmodes);
}

hipError_t launch_ls_extrapolate(const LineSearchArgs& a, hipStream_t stream) {
  if (a.n_models < 1 || a.ncols < 1) return hipSuccess;
  hipLaunchKernelGGL(ls_extrapolate_kernel, elem_grid(a), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_ls_decide(const LineSearchArgs& a, hipStream_t stream) {
  static std::atomic<unsigned long long> attr_seen{0};
  const size_t lds = sizeof(double) * (kMaxRank * kXs + 256);
  if (first_use_on_current_device(attr_seen)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ls_gram_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (a.n_models < 1) return hipSuccess;
  if (!a.part || a.nblk < 1 || a.nmodes < 1 || a.nmodes > kMaxModes) return hipErrorInvalidValue;
  hipLaunchKernelGGL(ls_gram_kernel, dim3(a.n_models, a.nmodes, a.nblk), dim3(256), lds, stream, a);
  hipLaunchKernelGGL(ls_decide_kernel, dim3(a.n_models), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_ls_apply(const LineSearchArgs& a, hipStream_t stream) {
  if (a.n_models < 1 || a.ncols < 1) return hipSuccess;
  hipLaunchKernelGGL(ls_apply_kernel, elem_grid(a), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace cals
