// Tensors of order above 3: the fused MTTKRP kernel contracts over two index groups (a fast one and a slow one).
// For N modes the N-1 contracted modes are split into two runs of consecutive modes; a run of more than one mode
// is represented by the explicit Khatri-Rao product of its factor multi-matrices (the paper's order-N fallback
// forms the whole Khatri-Rao product explicitly, Sec. 5 "MTTKRP"; here only the two partial products are formed,
// each far smaller than the tensor, and the kernel still generates their product on the fly).
#include "cals_internal.h"

namespace cals {

__global__ void __launch_bounds__(256) krp_kernel(KrpArgs a) {
  const int64_t total = a.rows * a.ncols;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    int64_t row = idx / a.ncols;
    const int c = (int)(idx - row * a.ncols);
    const int64_t out = row * a.ld + c;
    double k = 1.0;
    for (int q = 0; q < a.nrun; ++q) {
      const int64_t next = row / a.In[q];
      const int i = (int)(row - next * a.In[q]);
      const double u = a.U[q][(int64_t)i * a.ld + c];
      k = (q == 0) ? u : k * u;
      row = next;
    }
    a.K[out] = k;
  }
}

hipError_t launch_krp(const KrpArgs& a, hipStream_t stream) {
  if (a.nrun < 1 || a.nrun > kMaxModes || a.rows < 1 || a.ncols < 1 || a.ncols > a.ld || !a.K) return hipErrorInvalidValue;
  int64_t rows = 1;
  for (int q = 0; q < a.nrun; ++q) {
    if (a.In[q] < 1 || !a.U[q]) return hipErrorInvalidValue;
    rows *= a.In[q];
  }
  if (rows != a.rows) return hipErrorInvalidValue;
  const int64_t total = a.rows * a.ncols;
  const int64_t blocks = (total + 255) / 256;
  hipLaunchKernelGGL(krp_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace cals
