// Internal declarations shared by the HIP translation units of the CALS library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace cals {

// True the first time it is called with the given flag word while a given device is current (kernel attributes
// such as the dynamic LDS limit are per device); safe to call from several host threads.
inline bool first_use_on_current_device(std::atomic<unsigned long long>& seen) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return true;
  const unsigned long long bit = 1ull << dev;
  return (seen.fetch_or(bit) & bit) == 0;
}

#if defined(__HIPCC__)
// Broadcast of a double from one lane (wave-uniform index) to the whole wavefront through scalar registers.
__device__ inline double readlane_f64(double v, int src_lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src_lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src_lane);
  return __hiloint2double(hi, lo);
}
#endif

constexpr int kMaxRank = 32;       // largest rank of one model (CALS_MAX_RANK)
constexpr int kMaxModes = 6;       // largest tensor order (CALS_MAX_MODES)
constexpr int kGramStride = kMaxRank * kMaxRank;

// ---- fused MTTKRP (Eq. (2); Alg. 2 fused-MTTKRP line) ------------------------------------------
// GEMM view for output mode n:  M[In x ncols] = A[In x K] * KRP[K x ncols],  K = Ia*Ib, where
// `a` is the faster and `b` the slower of the two contracted tensor indices and
// A[m, (ia,ib)] = T[m*sm + ia*sa + ib*sb],  KRP[(ia,ib), c] = Ua[ia,c] * Ub[ib,c].
struct MttkrpProblem {
  const double* T;
  const double* Ua;   // row-major Ia x ld
  const double* Ub;   // row-major Ib x ld
  double* M;          // row-major In x ld, columns [0,ncols) written
  const double* zeros; // device buffer of at least 4 zero doubles, 16-byte aligned
  int64_t sm, sa, sb; // element strides in T
  int In, Ia, Ib;
  int ncols;          // fused width (total rank)
  int ld;             // leading dimension (doubles) of Ua, Ub, M
};

struct MttkrpPart {  // one kernel launch: `ny` column blocks of `wn` 16-column tiles each, starting at column col0
  int wn, ny, col0;
};

// Development overrides of the launch planner (zero / negative = let the planner decide).  A context reads them
// once, when it is created, from the environment variables CALS_MTTKRP_WNMAX, _WM, _PERCU, _SPLITS, _CONTIGU,
// _NOCONTIG, _NOROWPAIR, _NOPAIR; nothing on the launch path looks at the environment.
struct MttkrpTuning {
  int wn_max = 0;        // widest column block, in 16-column tiles
  int wm = 0;            // row tiles per wavefront (1, 2 or 4)
  int per_cu = 0;        // resident workgroups per compute unit assumed by the cost model
  int splits = 0;        // split-K factor
  int contig_u = -1;     // padded-run reads of unaligned tensors: 1 always, 0 never, -1 by width and size
  bool no_contig = false, no_rowpair = false, no_pair = false;   // switch off a read or production variant
  int kernel = 0;        // 1: the tile kernel only; 2: the rows kernel wherever it is eligible; 0: by modelled time
  int rows_wmb = 0, rows_wnb = 0, rows_nsb = 0;   // rows kernel: variant and workgroup-level split count
};
MttkrpTuning mttkrp_tuning_from_env();

struct MttkrpPlan {
  int wm;          // 16-row MFMA tiles per wavefront
  int ka;          // contraction rows per LDS stage
  int nparts;      // launches: column blocks of unequal width run as separate launches (no padded tile columns)
  MttkrpPart part[2];
  int splits;      // split-K factor (same for all parts)
  int64_t chunk;   // contraction indices per split
  int mtiles;      // row blocks of 64*wm rows
  size_t workspace_bytes;  // split-K partials: splits * In * ld doubles (0 when splits == 1)
  int read_mode;   // how the kernel reads the tensor along the contraction (kAffine ... kContig4U)
  int ia_counted;  // length of the fast contracted index as the kernel counts it (kContig4U: Ia rounded up to 4)
  int pair;        // factor rows 16-byte aligned: two columns per lane in the Khatri-Rao production
  // kind 1: the rows kernel (every wavefront holds all row tiles of a row block; see mttkrp_rows_kernel.h).  Then
  // `chunk` counts contraction indices per WAVEFRONT, `splits` the partial panels (workgroup-level splits), and
  // wm / ka / nparts / part / mtiles / read_mode / ia_counted / pair are unused.
  int kind;        // 0: tile kernel, 1: rows kernel
  int rows_wmb, rows_wnb;   // kernel variant: row tiles and column tiles per wavefront
  int rows_amode;           // kRowsContig / kRowsPair
  int rows_tpb;             // row tiles per row block (<= rows_wmb)
  int rows_nrb, rows_ncg;   // row blocks, column groups
  int rows_rem;             // column groups with rows_wnb tiles (the others have one fewer)
  double cost_us;           // modelled time
};

// Chooses tile shape, tensor read mode and split-K for a problem on a device with `num_cus` compute units.
MttkrpPlan mttkrp_plan(const MttkrpProblem& p, int num_cus, const MttkrpTuning& tune = MttkrpTuning());
// Enqueues contraction (+ ordered split-K reduction when plan.splits > 1) on `stream`.
// `workspace` must hold plan.workspace_bytes.  ev[0..3], when non-null, are recorded around the
// contraction kernel (ev[0], ev[1]) and around the reduction kernel (ev[2], ev[3]); *timed (when non-null) tells
// whether every record succeeded -- if not, the launch stands but its events must not be read.
hipError_t mttkrp_launch(const MttkrpProblem& p, const MttkrpPlan& plan, double* workspace, hipStream_t stream,
                         hipEvent_t* ev, bool* timed = nullptr);
// One-time per-process kernel attribute set-up (dynamic LDS sizes).
hipError_t mttkrp_init();

// ---- per-model steps (Alg. 2 inner loop: Hadamard of Gramians, update; Alg. 1 error line) -------
struct ModelDesc {   // one per active model, in slot order
  int32_t sid;       // index of the model's persistent per-model storage
  int32_t col;       // first column in the multi-matrices
  int32_t rank;
  uint32_t flags;
  double alpha;      // line-search step
};

struct ModelState {  // persistent per-model device storage, indexed by sid
  double G[kMaxModes][kGramStride];   // Gramians of the current factors (rank x rank, ld = rank)
  double inner, normsq;               // error terms of the last update of the last mode
  double Gls[kMaxModes][kGramStride]; // line search: Gramians of the extrapolated point
  double inner_ls;                    // line search: sum(A_N,new * M_N(A_new))
};

#if defined(__HIPCC__)
// Element e of the Hadamard product of the Gramians of all modes but `mode`, multiplied up in increasing mode
// order (Alg. 1, Hadamard line).
__device__ inline double hadamard_of_others(const ModelState* st, int nmodes, int mode, int e) {
  int k = (mode == 0) ? 1 : 0;
  double h = st->G[k][e];
  for (++k; k < nmodes; ++k)
    if (k != mode) h *= st->G[k][e];
  return h;
}
#endif

struct ModelOut {    // per-model scalars the host reads back once per round, indexed by sid
  double err, fit;            // after the last completed iteration
  int32_t status;             // CALS_RUNNING or CALS_NUMERICAL (set on device)
  int32_t iters;              // completed iterations
  int32_t ls_accepted;
  int32_t pad;
};

struct UpdateArgs {
  const ModelDesc* desc;
  ModelState* state;
  ModelOut* out;
  double* lambda;       // column norms, kMaxRank doubles per sid
  const double* M;      // MTTKRP result, row-major In x ld
  double* U;            // factor multi-matrix of the updated mode, row-major In x ld
  const double* X;      // NONNEG: rows already solved by the non-negative update (row-major In x ld), or null
  int32_t* nn_fail;     // NONNEG: per slot position, set when a row's sub-block could not be factorised (reset here)
  int In, ld, mode;     // mode = 0 .. nmodes-1
  int nmodes;           // tensor order
  int n_models;
  double normT2;
  double* part;         // tall modes: per (slot position, row block) partial Gramian and inner product
                        // (update_part_doubles(In) doubles per slot position); may be null when update_row_blocks(In) == 1
};

// Row blocks a mode of In rows is cut into for the update (1: one workgroup per model does everything).
constexpr int kUpdatePartStride = 536;   // 528 lower-triangle pairs + the inner-product term, padded
inline int update_row_blocks(int In) {
  const int b = (In + 255) / 256;
  return b < 1 ? 1 : (b > 32 ? 32 : b);
}
inline size_t update_part_doubles(int In) { return (size_t)update_row_blocks(In) * kUpdatePartStride; }

hipError_t launch_update(const UpdateArgs& a, hipStream_t stream);
// Gramians of all `nmodes` modes for models [first, first+count) of desc (used when a model is inserted).
// With reset_out, also puts the models' ModelOut back to {0, 0, RUNNING, 0, 0}.
// passive[nmodes] (may hold nulls): the NONNEG passive-set masks, cleared for the models' storage ids on reset.
hipError_t launch_gram_init(const ModelDesc* desc, ModelState* state, ModelOut* out, double* lambda, bool reset_out,
                            uint32_t* const* passive, int capacity, const double* const* U, const int* In, int nmodes,
                            int ld, int first, int count, hipStream_t stream);
// ||T||^2 with a fixed summation tree, and a finiteness check (flag[0] != 0 when a NaN/Inf was seen).
hipError_t launch_norm_sq(const double* T, int64_t n, double* partial /* >= 1024 doubles */, double* out, int* flag,
                          hipStream_t stream);
// Stable left-compaction / arbitrary column gather of a row-major multi-matrix:
// dst[i, c] = src[i, map[c]] for c < ncols, all rows.
hipError_t launch_gather_columns(const double* src, double* dst, const int32_t* map, int rows, int ncols, int ld,
                                 hipStream_t stream);

// Strided block copy on the device: dst[i*dst_ld + c] = src[i*src_ld + c], i < rows, c < cols.
hipError_t launch_copy_block(const double* src, int64_t src_ld, double* dst, int64_t dst_ld, int rows, int cols,
                             hipStream_t stream);
// dst[i*dst_ld + c] = src[i*src_ld + map[c]] (gather with separate leading dimensions).
hipError_t launch_gather_block(const double* src, int64_t src_ld, double* dst, int64_t dst_ld, const int32_t* map,
                               int rows, int cols, hipStream_t stream);

// ---- non-negative update (Sec. 5, "Non-negativity constraints") -------------------------------------
struct NnlsArgs {
  const ModelDesc* desc;
  const ModelState* state;
  const ModelOut* out;
  const double* M;      // MTTKRP result, row-major In x ld
  double* X;            // out: solved rows of the NONNEG models, row-major In x ld (other columns untouched)
  uint32_t* passive;    // per (row, sid) passive-set masks of this mode, In x capacity; read (warm start) and written
  int32_t* fail;        // per slot position; or-ed with 1 on failure
  const int32_t* order; // slot positions in the order the grid takes them (costliest models first), n_models entries
  int In, ld, mode, n_models, capacity;
  int nmodes;           // tensor order
  int max_rank;         // largest rank among the NONNEG models of this launch
  int rows_per_block;   // set by launch_nnls
};
hipError_t launch_nnls(const NnlsArgs& a, hipStream_t stream);

// ---- line search (Sec. 5, "Line search") -----------------------------------------------------------
// A point is held with lambda folded into the factor of the last mode.  A model takes part in a round's line search when
// it has the LINESEARCH flag, is still running and has completed at least two iterations.
struct LineSearchArgs {
  const ModelDesc* desc;
  ModelState* state;
  ModelOut* out;
  double* lambda;
  const int32_t* colmodel; // slot position of the model that owns each column
  int32_t* accept;         // per slot position: 1 when the extrapolated point was taken this round
  double* U[kMaxModes];     // current factors
  double* Uprev[kMaxModes]; // point after the previous iteration
  double* Unew[kMaxModes];  // extrapolated point
  const double* M3;        // MTTKRP of mode `ls_mode` at the extrapolated point, row-major I_mode x ld
  int ls_mode;             // 0-based mode whose MTTKRP gives the inner product <T, model> of the extrapolated point
  double* part;            // per (slot position, mode, row block): partial Gramian and inner product of the
                           // extrapolated point, kUpdatePartStride doubles each
  int nblk;                // row blocks (update_row_blocks of the longest mode)
  int In[kMaxModes];
  int nmodes;              // tensor order
  int ld, n_models, ncols;
  double normT2;
  // two-step sweeps only: the tensor contracted with the mode-1 factors of the current point (Ycur), of the point
  // kept after the previous round (Yprev) and of the extrapolated point (Ynew); yrows x ld each
  const double* Ycur;
  double* Yprev;
  double* Ynew;
  int64_t yrows;
};
// Unew = Uprev + alpha (A_cur - Uprev) for the models taking part, Unew = A_cur for all other columns.
hipError_t launch_ls_extrapolate(const LineSearchArgs& a, hipStream_t stream);
// Gramians of the extrapolated point and sum(A_N,new * M_N); then e_new = ||T||^2 + sum(G1*...*GN) - 2 inner and the
// decision (strictly lower error wins): accepted models get err/fit/Gramians of the new point and lambda = 1.
hipError_t launch_ls_decide(const LineSearchArgs& a, hipStream_t stream);
// U = Unew for accepted models; Uprev = the point kept (lambda folded into the last mode) for every line-search model.
hipError_t launch_ls_apply(const LineSearchArgs& a, hipStream_t stream);
// Two-step sweeps: the contraction with the mode-1 factors is linear in them, so for the extrapolated point it is
// Ynew = Yprev + alpha (Ycur - Yprev) column by column (Ynew = Ycur for the columns of models not taking part) ...
hipError_t launch_ls_y_combine(const LineSearchArgs& a, hipStream_t stream);
// ... and after the decision the contraction of the point each model keeps: Yprev = accepted ? Ynew : Ycur.
hipError_t launch_ls_y_keep(const LineSearchArgs& a, hipStream_t stream);

// ---- two-step sweep: contraction of the intermediate Y with one factor ---------------------------------------
// M[o, c] = sum_{s < ns} Y[(o*so + s*ss) * ld + c] * U[s * ld + c],  o < no, c < ncols (fixed summation order).
hipError_t launch_ttv(const double* Y, const double* U, double* M, int no, int ns, int64_t so, int64_t ss, int ld,
                      int ncols, hipStream_t stream);
hipError_t launch_fill(double* p, int64_t n, double v, hipStream_t stream);
// Order above 3:  M[o, c] = sum_{r < PR} sum_{l < PL} Y[(l + PL * (o + no * r)) * ld + c] * KL[l * ld + c] * KR[r * ld + c]
// (fixed summation order); KL / KR are row-major with leading dimension ld (a single row of ones when PL / PR = 1).
// `slices` (from ttv2_slices) cuts the (l, r) range over several workgroups; with more than one, `workspace` must hold
// slices * no * ld doubles.
int ttv2_slices(int no, int PL, int PR, int ld, int ncols, int num_cus);
hipError_t launch_ttv2(const double* Y, const double* KL, int PL, const double* KR, int PR, double* M, int no, int ld,
                       int ncols, int slices, double* workspace, hipStream_t stream);
// Adds `splits` partial panels P[z][n_rows_ld] into M in split order (columns >= ncols of a row are left alone).
hipError_t launch_splitk_reduce(const double* P, double* M, int64_t n_rows_ld, int ld, int ncols, int splits, hipStream_t stream);

// ---- tensors of order above 3: explicit Khatri-Rao product of a run of consecutive modes ----------------------
// K[row, c] = prod_{q < nrun} U[q][i_q * ld + c],  row = i_0 + In[0] * (i_1 + In[1] * (...)),  c < ncols; K and the
// U[q] are row-major with leading dimension ld.  The product is taken in increasing q.
struct KrpArgs {
  const double* U[kMaxModes];
  int In[kMaxModes];
  int nrun;
  double* K;
  int64_t rows;
  int ld, ncols;
};
hipError_t launch_krp(const KrpArgs& a, hipStream_t stream);

// ---- practical-peak yardsticks (kind 0: fp64 MFMA issue rate in TFLOP/s, kind 1: streaming read in GB/s) ----
hipError_t launch_yardstick(int kind, const void* buf, int64_t bytes, int reps, int num_cus, double* sink,
                            hipStream_t stream, double* value);

}  // namespace cals
