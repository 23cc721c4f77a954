// C boundary and host scheduler of the CALS library: the queue logic of the paper's full algorithm
// (Alg. 3) around the device kernels.  One round = fill the multi-matrices from the queue front,
// advance every active model one ALS iteration with one fused MTTKRP per mode, read back the per-model
// fits, retire in slot order, compact.  The only host-visible data dependency per round is the
// retire decision.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/cals.h"
#include "cals_internal.h"

using namespace cals;

#define HIP_TRY(expr)                         \
  do {                                        \
    hipError_t e__ = (expr);                  \
    if (e__ != hipSuccess) {                  \
      (void)hipGetLastError();                \
      return CALS_E_HIP;                      \
    }                                         \
  } while (0)
#define CALS_TRY(expr)            \
  do {                            \
    int rc__ = (expr);            \
    if (rc__ != CALS_OK) return rc__; \
  } while (0)

namespace {

struct PendingModel {
  int64_t id;
  int rank;
  double tol;
  int max_iters;
  uint32_t flags;
  double alpha;
  std::vector<double> init[kMaxModes];  // column-major I_n x rank, as given
};

struct ActiveModel {
  int64_t id;
  int sid, col, rank;
  double tol;
  int max_iters;
  uint32_t flags;
  double alpha;
  double fit_prev;
  int iters;        // completed iterations as of the last read-back
};

struct Leaving { ActiveModel m; int status; int64_t round; int slot; };

struct RetiredModel {
  cals_result res;
  std::vector<double> U[kMaxModes];     // column-major I_n x rank
  std::vector<double> lambda;
};

struct TimedLaunch { hipEvent_t ev[4]; int mode; bool reduced; };
struct TimedRound { hipEvent_t ev[2]; size_t index; };   // index into the round log

constexpr int kMaxDevices = 64;
constexpr size_t kScratchDoubles = CALS_NOALLOC_SCRATCH_BYTES / sizeof(double);

}  // namespace

// Fixed scratch of the entry point that allocates nothing (cals_mttkrp_noalloc): the split-K partial panels of one
// fused MTTKRP.  Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name below is only a handle: the device address comes from hipGetSymbolAddress,
// taken once per device in cals_create with that device current, and only that address is ever handed to kernels.
static __device__ __align__(256) double scratch[kScratchDoubles];

namespace {
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};   // per device: the device address of `scratch`

// The address of this device's copy of the scratch array (the device must be current).
int scratch_address(int device, double** out) {
  if (device < 0 || device >= kMaxDevices) return CALS_E_INVALID;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    double* ptr = nullptr;
    if (hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return CALS_E_HIP;
    }
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return CALS_OK;
}
}  // namespace

struct cals_ctx {
  cals_options opt;
  hipStream_t stream = nullptr;
  int num_cus = 0;
  MttkrpTuning tune;          // development overrides of the launch planner, read once at creation
  double* scratch_dev = nullptr;   // this device's copy of the fixed scratch array (cals_mttkrp_noalloc)
  bool has_tensor = false;
  int nmodes = 0;             // tensor order N (3 .. kMaxModes)
  int64_t dims[kMaxModes] = {0, 0, 0, 0, 0, 0};
  const double* T = nullptr;
  double* T_owned = nullptr;
  double normT2 = 0.0;
  int ld = 0;                 // leading dimension of every multi-matrix (R* rounded up to 16)
  int capacity = 0;           // slots with persistent storage
  double* U[kMaxModes] = {};
  double* Ualt[kMaxModes] = {};
  double* Uprev[kMaxModes] = {};   // line search only (allocated on first use)
  double* Unew[kMaxModes] = {};
  double* Kbuf[2] = {nullptr, nullptr};   // order > 3: explicit Khatri-Rao products of the fast and the slow run
  double* M = nullptr;        // MTTKRP result, max(I_n) x ld
  double* workspace = nullptr;
  size_t workspace_bytes = 0;
  ModelDesc* d_desc = nullptr;
  ModelDesc* h_desc = nullptr;   // pinned
  ModelState* d_state = nullptr;
  ModelOut* d_out = nullptr;
  ModelOut* h_out = nullptr;     // pinned
  int32_t* d_map = nullptr;
  int32_t* h_map = nullptr;      // pinned
  uint32_t* passive[kMaxModes] = {};  // NONNEG only
  double* d_scratch = nullptr;   // 1024 partial sums + result + flag
  double* Y = nullptr;           // two-step sweeps: the tensor contracted with the mode-1 multi-matrix, (I2*...*IN) x ld
  double* Yprev = nullptr;       // two-step sweeps with line search: Y at the point kept after the previous round ...
  double* Ynew = nullptr;        // ... and at the extrapolated point (both allocated with the line-search buffers)
  double* Ychain[kMaxModes] = {};  // order > 3: Y contracted further with modes 2, 3, ... (index = level, from 2)
  double* d_ones = nullptr;      // two-step sweeps: ld ones (the second "factor" of the first step)
  double* d_sink = nullptr;      // never-written target of the yardstick kernels
  double* d_zeros = nullptr;     // 8 zero doubles (what MTTKRP lanes past the end of a split load)
  double* d_lambda = nullptr;    // kMaxRank column norms per sid
  double* h_lambda = nullptr;    // pinned
  double* d_stage = nullptr;     // (I1+...+IN) x ld doubles: packed columns on their way in (fill) or out (retire)
  double* h_stage = nullptr;     // pinned, same size
  int32_t* d_rmap = nullptr;     // columns of the models being retired
  int32_t* h_rmap = nullptr;     // pinned
  int32_t* d_colmodel = nullptr; // line search: slot position owning each column
  int32_t* h_colmodel = nullptr; // pinned
  int32_t* d_accept = nullptr;   // line search: per slot position, extrapolated point taken this round
  double* d_lspart = nullptr;    // line search: per (slot position, mode, row block) partial sums
  double* d_updpart = nullptr;   // update of tall modes: per (slot position, row block) partial sums
  int32_t* d_nnfail = nullptr;   // non-negativity: per slot position, failure flag of the current mode update
  int32_t* d_nnorder = nullptr;  // slot positions sorted for the non-negative update (NONNEG first, high ranks first)
  int32_t* h_nnorder = nullptr;  // pinned
  std::deque<PendingModel> queue;
  std::vector<ActiveModel> active;
  std::vector<int> free_sids;
  std::map<int64_t, RetiredModel> retired;
  std::deque<int64_t> out_queue;
  int64_t next_id = 0;
  int total_rank = 0;
  bool desc_dirty = true;
  bool any_ls = false, any_nonneg = false;
  // statistics
  int64_t rounds = 0, n_retired = 0;
  int64_t rounds_unread = 0;     // rounds launched since the last read-back of the per-model records
  double mttkrp_flops = 0.0;
  double mttkrp_ms[kMaxModes] = {}, reduce_ms[kMaxModes] = {};
  int64_t mttkrp_launches[kMaxModes] = {};
  int64_t mttkrp_rows_launches = 0;
  std::vector<TimedLaunch> timed;
  std::vector<TimedRound> timed_rounds;
  std::vector<cals_round_record> round_log;   // one record per round (bounded)
  std::vector<hipEvent_t> event_pool;
};

namespace {

int set_device(cals_ctx* c) {
  HIP_TRY(hipSetDevice(c->opt.device));
  return CALS_OK;
}

bool all_finite(const double* p, int64_t n) {
  for (int64_t i = 0; i < n; ++i)
    if (!std::isfinite(p[i])) return false;
  return true;
}

int ensure_workspace(cals_ctx* c, size_t bytes) {
  if (bytes <= c->workspace_bytes) return CALS_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (c->workspace) HIP_TRY(hipFree(c->workspace));
  c->workspace = nullptr;
  c->workspace_bytes = 0;
  hipError_t e = hipMalloc(&c->workspace, bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); return CALS_E_NOMEM; }
  c->workspace_bytes = bytes;
  return CALS_OK;
}

// The contracted modes of output mode n, as a fast run A = [a0, a1) and a slow run B = [b0, b1) of consecutive
// modes (first index fastest).  For an inner mode the runs are the modes before and after it; for the first and the
// last mode the N-1 remaining modes are cut where the larger of the two run sizes is smallest (first such cut).
// For N = 3 every run is a single mode.
struct Runs { int a0, a1, b0, b1; int64_t Ia, Ib; };

Runs contraction_runs(const cals_ctx* c, int n) {
  const int N = c->nmodes;
  Runs r{};
  if (n > 0 && n < N - 1) {
    r.a0 = 0; r.a1 = n; r.b0 = n + 1; r.b1 = N;
  } else {
    const int lo = (n == 0) ? 1 : 0, hi = (n == 0) ? N : N - 1;
    int best_k = lo + 1;
    double best = 1e300;
    for (int k = lo + 1; k < hi; ++k) {
      double pa = 1.0, pb = 1.0;
      for (int m = lo; m < k; ++m) pa *= (double)c->dims[m];
      for (int m = k; m < hi; ++m) pb *= (double)c->dims[m];
      const double worst = pa > pb ? pa : pb;
      if (worst < best) { best = worst; best_k = k; }
    }
    r.a0 = lo; r.a1 = best_k; r.b0 = best_k; r.b1 = hi;
  }
  r.Ia = 1; r.Ib = 1;
  for (int m = r.a0; m < r.a1; ++m) r.Ia *= c->dims[m];
  for (int m = r.b0; m < r.b1; ++m) r.Ib *= c->dims[m];
  return r;
}

int64_t mode_stride(const cals_ctx* c, int m) {
  int64_t s = 1;
  for (int k = 0; k < m; ++k) s *= c->dims[k];
  return s;
}

// One contracted run as the kernel's factor operand: the factor multi-matrix itself for a run of one mode, else the
// explicit Khatri-Rao product of the run's multi-matrices, formed in `kbuf` (rows in memory order of the run).
int run_operand(cals_ctx* c, int m0, int m1, int64_t rows, const double* const* U, double* kbuf, int ncols, int ld,
                const double** out) {
  if (m1 - m0 == 1) { *out = U[m0]; return CALS_OK; }
  if (!kbuf || ld > c->ld) return CALS_E_INVALID;
  KrpArgs k{};
  k.nrun = m1 - m0;
  for (int q = 0; q < k.nrun; ++q) { k.U[q] = U[m0 + q]; k.In[q] = (int)c->dims[m0 + q]; }
  k.K = kbuf; k.rows = rows; k.ld = ld; k.ncols = ncols;
  HIP_TRY(launch_krp(k, c->stream));
  *out = kbuf;
  return CALS_OK;
}

int64_t rows_without_mode1(const cals_ctx* c);

// Shape of the fused MTTKRP for output mode `mode` (0-based): everything but the two factor operands.
int problem_shape(const cals_ctx* c, int mode, double* M, int ncols, int ld, MttkrpProblem* out, Runs* runs) {
  const Runs r = contraction_runs(c, mode);
  if (r.Ia >= (1LL << 31) || r.Ib >= (1LL << 31)) return CALS_E_UNSUPPORTED;
  MttkrpProblem p{};
  p.T = c->T;
  p.zeros = c->d_zeros;
  p.M = M;
  p.ncols = ncols;
  p.ld = ld;
  p.In = (int)c->dims[mode]; p.sm = mode_stride(c, mode);
  p.Ia = (int)r.Ia; p.sa = mode_stride(c, r.a0);
  p.Ib = (int)r.Ib; p.sb = mode_stride(c, r.b0);
  *out = p;
  *runs = r;
  return CALS_OK;
}

// Problem description of the fused MTTKRP for output mode `mode` (0-based) over given multi-matrices.  Enqueues the
// Khatri-Rao products of runs of more than one mode (tensors of order above 3).
int make_problem(cals_ctx* c, int mode, const double* const* U, double* M, int ncols, int ld, MttkrpProblem* out) {
  MttkrpProblem p{};
  Runs r{};
  CALS_TRY(problem_shape(c, mode, M, ncols, ld, &p, &r));
  CALS_TRY(run_operand(c, r.a0, r.a1, r.Ia, U, c->Kbuf[0], ncols, ld, &p.Ua));
  CALS_TRY(run_operand(c, r.b0, r.b1, r.Ib, U, c->Kbuf[1], ncols, ld, &p.Ub));
  *out = p;
  return CALS_OK;
}

// The largest split-K workspace any round of this context can ask for: every mode at every fused width (in steps of
// one 16-column tile up to R*), and the first contraction of two-step sweeps.  Allocated once when the tensor
// arrives, so that no round has to stop the stream and reallocate (ensure_workspace stays as the fallback for
// cals_mttkrp calls with a leading dimension of their own).
size_t largest_round_workspace(const cals_ctx* c) {
  size_t need = 0;
  for (int w = 16; w <= c->ld; w += 16) {
    const int ncols = w < (int)c->opt.max_total_rank ? w : (int)c->opt.max_total_rank;
    for (int mode = 0; mode < c->nmodes; ++mode) {
      MttkrpProblem p{};
      Runs r{};
      if (problem_shape(c, mode, c->M, ncols, c->ld, &p, &r) != CALS_OK) continue;
      p.Ua = c->U[0]; p.Ub = c->U[0];        // the planner looks at their alignment only
      need = std::max(need, mttkrp_plan(p, c->num_cus, c->tune).workspace_bytes);
    }
    if (c->Y && rows_without_mode1(c) < (1LL << 31)) {
      MttkrpProblem p{};
      p.T = c->T; p.zeros = c->d_zeros; p.M = c->Y; p.ncols = ncols; p.ld = c->ld;
      p.In = (int)rows_without_mode1(c); p.sm = c->dims[0];
      p.Ia = (int)c->dims[0]; p.sa = 1; p.Ua = c->U[0];
      p.Ib = 1; p.sb = c->dims[0]; p.Ub = c->U[0];
      need = std::max(need, mttkrp_plan(p, c->num_cus, c->tune).workspace_bytes);
    }
  }
  return need;
}

// Four events for one timed launch, or none (what was taken goes back to the pool).
bool take_events(cals_ctx* c, hipEvent_t (&ev)[4]);

hipEvent_t take_event(cals_ctx* c) {
  if (!c->event_pool.empty()) {
    hipEvent_t e = c->event_pool.back();
    c->event_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

bool take_events(cals_ctx* c, hipEvent_t (&ev)[4]) {
  for (int i = 0; i < 4; ++i) {
    ev[i] = take_event(c);
    if (!ev[i]) {
      (void)hipGetLastError();
      for (int k = 0; k < i; ++k) c->event_pool.push_back(ev[k]);
      return false;
    }
  }
  return true;
}

int drain_timings(cals_ctx* c) {
  if (c->timed.empty() && c->timed_rounds.empty()) return CALS_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (TimedLaunch& t : c->timed) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t.ev[0], t.ev[1]) == hipSuccess) c->mttkrp_ms[t.mode] += ms;
    if (t.reduced && hipEventElapsedTime(&ms, t.ev[2], t.ev[3]) == hipSuccess) c->reduce_ms[t.mode] += ms;
    for (int i = 0; i < 4; ++i) c->event_pool.push_back(t.ev[i]);
  }
  c->timed.clear();
  for (TimedRound& t : c->timed_rounds) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t.ev[0], t.ev[1]) == hipSuccess) c->round_log[t.index].ms = ms;
    c->event_pool.push_back(t.ev[0]);
    c->event_pool.push_back(t.ev[1]);
  }
  c->timed_rounds.clear();
  return CALS_OK;
}

// Returns the events of a timed launch that was not enqueued to the pool.
void give_back_events(cals_ctx* c, hipEvent_t (&ev)[4]) {
  for (int i = 0; i < 4; ++i) c->event_pool.push_back(ev[i]);
}

// no_alloc: the split-K partials go to the fixed scratch array instead of the context's workspace, nothing is
// allocated (no workspace growth, no events: such a launch is not timed), and a launch whose partials do not fit
// is refused.
int run_mttkrp(cals_ctx* c, int mode, const double* const* U, double* M, int ncols, int ld, bool no_alloc = false) {
  MttkrpProblem p{};
  CALS_TRY(make_problem(c, mode, U, M, ncols, ld, &p));
  // factor matrices are addressed with 32-bit byte offsets
  // (with room for the rows a workgroup requests past the end of its range)
  if ((int64_t)(p.Ia + 64) * ld * 8 >= (1LL << 32) || (int64_t)(p.Ib + 64) * ld * 8 >= (1LL << 32)) return CALS_E_UNSUPPORTED;
  MttkrpPlan pl = mttkrp_plan(p, c->num_cus, c->tune);
  if (pl.chunk >= (1LL << 31)) return CALS_E_UNSUPPORTED;
  double* partials = nullptr;
  if (no_alloc) {
    if (pl.workspace_bytes > CALS_NOALLOC_SCRATCH_BYTES) return CALS_E_TOOLARGE;
    if (!c->scratch_dev) return CALS_E_STATE;
    partials = c->scratch_dev;
  } else {
    CALS_TRY(ensure_workspace(c, pl.workspace_bytes));
    partials = c->workspace;
  }
  hipEvent_t* ev = nullptr;
  TimedLaunch t{};
  if ((c->opt.flags & CALS_CTX_TIMING) && !no_alloc) {
    if (!take_events(c, t.ev)) return CALS_E_HIP;
    t.mode = mode;
    t.reduced = pl.splits > 1;
    ev = t.ev;
  }
  bool timed = false;
  {
    const hipError_t e = mttkrp_launch(p, pl, partials, c->stream, ev, &timed);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (ev) give_back_events(c, t.ev);
      return CALS_E_HIP;
    }
  }
  if (ev && !timed) {        // an event could not be recorded: the launch stands, it is just not timed
    give_back_events(c, t.ev);
    ev = nullptr;
  }
  if (ev) {
    c->timed.push_back(t);
    if (c->timed.size() > 2048) CALS_TRY(drain_timings(c));
  }
  double elems = 1.0;
  for (int n = 0; n < c->nmodes; ++n) elems *= (double)c->dims[n];
  c->mttkrp_flops += 2.0 * ncols * elems;
  c->mttkrp_launches[mode] += 1;
  if (pl.kind == 1) c->mttkrp_rows_launches += 1;
  return CALS_OK;
}

// First step of a two-step sweep: Y[(i2,i3), c] = sum_i1 T[i1,i2,i3] * U1[i1,c], i.e. the fused MTTKRP kernel on the
// (I2*I3) x I1 unfolding with a single row of ones as the second factor.  Timed under mode index 1.
int64_t rows_without_mode1(const cals_ctx* c) {
  int64_t rows = 1;
  for (int n = 1; n < c->nmodes; ++n) rows *= c->dims[n];
  return rows;
}

int run_contract_mode1(cals_ctx* c, const double* U1, int ncols, int ld, double* Y = nullptr) {
  const int64_t rows = rows_without_mode1(c);
  if (!Y) Y = c->Y;
  if (rows >= (1LL << 31) || (int64_t)(c->dims[0] + 64) * ld * 8 >= (1LL << 32)) return CALS_E_UNSUPPORTED;
  MttkrpProblem p{};
  p.T = c->T; p.zeros = c->d_zeros; p.M = Y; p.ncols = ncols; p.ld = ld;
  p.In = (int)rows; p.sm = c->dims[0];
  p.Ia = (int)c->dims[0]; p.sa = 1; p.Ua = U1;
  p.Ib = 1; p.sb = c->dims[0]; p.Ub = c->d_ones;
  MttkrpPlan pl = mttkrp_plan(p, c->num_cus, c->tune);
  if (pl.chunk >= (1LL << 31)) return CALS_E_UNSUPPORTED;
  CALS_TRY(ensure_workspace(c, pl.workspace_bytes));
  hipEvent_t* ev = nullptr;
  TimedLaunch t{};
  if (c->opt.flags & CALS_CTX_TIMING) {
    if (!take_events(c, t.ev)) return CALS_E_HIP;
    t.mode = 1;
    t.reduced = pl.splits > 1;
    ev = t.ev;
  }
  bool timed = false;
  {
    const hipError_t e = mttkrp_launch(p, pl, c->workspace, c->stream, ev, &timed);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (ev) give_back_events(c, t.ev);
      return CALS_E_HIP;
    }
  }
  if (ev && !timed) {        // an event could not be recorded: the launch stands, it is just not timed
    give_back_events(c, t.ev);
    ev = nullptr;
  }
  if (ev) {
    c->timed.push_back(t);
    if (c->timed.size() > 2048) CALS_TRY(drain_timings(c));
  }
  return CALS_OK;
}

// Rows of the chain intermediate of level k (1-based mode k contracted last): one per index tuple (i_{k+1}, ..., i_N).
int64_t chain_rows(const cals_ctx* c, int level) {
  int64_t rows = 1;
  for (int n = level; n < c->nmodes; ++n) rows *= c->dims[n];
  return rows;
}

// Order above 3: Y_level = Y_{level-1} contracted with the multi-matrix of (0-based) mode level-1, column by column.
int advance_chain(cals_ctx* c, int level, const double* const* U, int ncols, int ld, const double* Y1) {
  const int64_t rows = chain_rows(c, level);
  if (rows >= (1LL << 31)) return CALS_E_UNSUPPORTED;
  const double* src = (level == 2) ? Y1 : c->Ychain[level - 1];
  HIP_TRY(launch_ttv2(src, U[level - 1], (int)c->dims[level - 1], c->d_ones, 1, c->Ychain[level], (int)rows, ld, ncols, 1,
                      nullptr, c->stream));
  return CALS_OK;
}

// Second step: the MTTKRP of mode `mode` (0-based, >= 1) from the contraction(s) and the factors of the remaining
// modes.  Order 3: Y and one remaining factor (ttv_kernel).  Higher orders: a chain Y_1 = Y (mode 1 contracted),
// Y_2 = Y_1 contracted with mode 2, ... -- level `mode` is formed here from level mode-1 and the mode just updated
// (sweeps call this in increasing mode order; `rebuild` forms every level from Y, for a call that starts at a later
// mode) -- and the MTTKRP is Y_mode contracted with the modes after `mode` (their explicit Khatri-Rao product when
// there are several).  Every level is 1/I_k of the previous one, so a sweep reads Y about twice.
int run_from_contraction(cals_ctx* c, int mode, const double* const* U, double* M, int ncols, int ld, bool rebuild = false,
                         const double* Y1 = nullptr /* the mode-1 contraction to start from; default: the context's */) {
  const int N = c->nmodes;
  if (!Y1) Y1 = c->Y;
  if (N == 3) {
    const int I2 = (int)c->dims[1], I3 = (int)c->dims[2];
    if (mode == 1) HIP_TRY(launch_ttv(Y1, U[2], M, I2, I3, 1, I2, ld, ncols, c->stream));
    else HIP_TRY(launch_ttv(Y1, U[1], M, I3, I2, I2, 1, ld, ncols, c->stream));
  } else {
    for (int level = rebuild ? 2 : mode; level <= mode; ++level)
      if (level >= 2) CALS_TRY(advance_chain(c, level, U, ncols, ld, Y1));
    const double* src = (mode == 1) ? Y1 : c->Ychain[mode];
    int64_t PR = 1;
    for (int m = mode + 1; m < N; ++m) PR *= c->dims[m];
    if (PR >= (1LL << 31)) return CALS_E_UNSUPPORTED;
    const double* KR = c->d_ones;
    if (mode < N - 1) CALS_TRY(run_operand(c, mode + 1, N, PR, U, c->Kbuf[1], ncols, ld, &KR));
    const int slices = ttv2_slices((int)c->dims[mode], 1, (int)PR, ld, ncols, c->num_cus);
    if (slices > 1) CALS_TRY(ensure_workspace(c, sizeof(double) * (size_t)slices * c->dims[mode] * ld));
    HIP_TRY(launch_ttv2(src, c->d_ones, 1, KR, (int)PR, M, (int)c->dims[mode], ld, ncols, slices, c->workspace, c->stream));
  }
  double elems = 1.0;
  for (int n = 0; n < N; ++n) elems *= (double)c->dims[n];
  c->mttkrp_flops += 2.0 * ncols * elems;
  c->mttkrp_launches[mode] += 1;
  return CALS_OK;
}

// Buffers only the non-negative update needs: per (row, storage id) passive-set masks, failure flags.
int ensure_nn_buffers(cals_ctx* c) {
  if (c->d_nnfail) return CALS_OK;
  HIP_TRY(hipSetDevice(c->opt.device));
  bool ok = true;
  for (int n = 0; n < c->nmodes; ++n) {
    const size_t bytes = sizeof(uint32_t) * (size_t)c->dims[n] * c->capacity;
    ok = ok && hipMalloc(&c->passive[n], bytes) == hipSuccess;
    if (ok) ok = hipMemsetAsync(c->passive[n], 0, bytes, c->stream) == hipSuccess;
  }
  ok = ok && hipMalloc(&c->d_nnfail, sizeof(int32_t) * c->capacity) == hipSuccess;
  if (ok) ok = hipMemsetAsync(c->d_nnfail, 0, sizeof(int32_t) * c->capacity, c->stream) == hipSuccess;
  ok = ok && hipMalloc(&c->d_nnorder, sizeof(int32_t) * c->capacity) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_nnorder, sizeof(int32_t) * c->capacity) == hipSuccess;
  if (ok) c->desc_dirty = true;      // the order travels with the descriptors
  if (!ok) {
    // nothing of a failed attempt stays behind: the next NONNEG model tries again from scratch
    (void)hipGetLastError();
    (void)hipStreamSynchronize(c->stream);
    for (int n = 0; n < c->nmodes; ++n) { (void)hipFree(c->passive[n]); c->passive[n] = nullptr; }
    (void)hipFree(c->d_nnfail); c->d_nnfail = nullptr;
    (void)hipFree(c->d_nnorder); c->d_nnorder = nullptr;
    (void)hipHostFree(c->h_nnorder); c->h_nnorder = nullptr;
    return CALS_E_NOMEM;
  }
  return CALS_OK;
}

// Buffers only line search needs: the previous and the extrapolated point, column ownership, decisions.
// Line search under two-step sweeps: the contraction at the extrapolated point is either a pass over the tensor or a
// combination of two stored contractions (about six passes over an array of the contraction's size per round, with
// the bookkeeping of the point kept).  Rough times at the context's full width decide which.
bool combination_beats_contraction(const cals_ctx* c) {
  const double rows = (double)rows_without_mode1(c), I1 = (double)c->dims[0], w = (double)c->ld;
  const double combine_s = 6.0 * rows * w * 8.0 / 4.0e12;
  const double contract_s = std::max(rows * I1 * 8.0 / 5.0e12, 2.0 * rows * I1 * w / 55.0e12);
  return combine_s < contract_s;
}

int ensure_ls_buffers(cals_ctx* c) {
  if (c->d_colmodel) return CALS_OK;
  HIP_TRY(hipSetDevice(c->opt.device));
  bool ok = true;
  for (int n = 0; n < c->nmodes; ++n) {
    const size_t bytes = sizeof(double) * (size_t)c->dims[n] * c->ld;
    ok = ok && hipMalloc(&c->Uprev[n], bytes) == hipSuccess && hipMalloc(&c->Unew[n], bytes) == hipSuccess;
    if (ok) ok = hipMemsetAsync(c->Uprev[n], 0, bytes, c->stream) == hipSuccess &&
                 hipMemsetAsync(c->Unew[n], 0, bytes, c->stream) == hipSuccess;
  }
  ok = ok && hipMalloc(&c->d_accept, sizeof(int32_t) * c->capacity) == hipSuccess;
  {
    const int64_t imax = *std::max_element(c->dims, c->dims + c->nmodes);
    ok = ok && hipMalloc(&c->d_lspart, sizeof(double) * c->nmodes * update_part_doubles((int)imax) * c->capacity) == hipSuccess;
  }
  ok = ok && hipHostMalloc(&c->h_colmodel, sizeof(int32_t) * c->ld) == hipSuccess;
  ok = ok && hipMalloc(&c->d_colmodel, sizeof(int32_t) * c->ld) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    (void)hipStreamSynchronize(c->stream);
    for (int n = 0; n < c->nmodes; ++n) {
      (void)hipFree(c->Uprev[n]); (void)hipFree(c->Unew[n]);
      c->Uprev[n] = c->Unew[n] = nullptr;
    }
    (void)hipFree(c->d_accept); (void)hipFree(c->d_lspart); (void)hipFree(c->d_colmodel); (void)hipHostFree(c->h_colmodel);
    c->d_accept = nullptr; c->d_lspart = nullptr; c->d_colmodel = nullptr; c->h_colmodel = nullptr;
    return CALS_E_NOMEM;
  }
  if (c->Y && combination_beats_contraction(c)) {
    // optional: without them the extrapolated point gets a contraction of its own
    const size_t bytes = sizeof(double) * (size_t)rows_without_mode1(c) * c->ld;
    if (hipMalloc(&c->Yprev, bytes) != hipSuccess || hipMalloc(&c->Ynew, bytes) != hipSuccess ||
        hipMemsetAsync(c->Yprev, 0, bytes, c->stream) != hipSuccess) {
      (void)hipGetLastError();
      (void)hipFree(c->Yprev); (void)hipFree(c->Ynew);
      c->Yprev = c->Ynew = nullptr;
    }
  }
  c->desc_dirty = true;
  return CALS_OK;
}

int upload_desc(cals_ctx* c) {
  if (!c->desc_dirty) return CALS_OK;
  const int n = (int)c->active.size();
  for (int k = 0; k < n; ++k) {
    const ActiveModel& m = c->active[k];
    ModelDesc d;
    d.sid = m.sid; d.col = m.col; d.rank = m.rank; d.flags = m.flags; d.alpha = m.alpha;
    c->h_desc[k] = d;
  }
  if (n > 0) HIP_TRY(hipMemcpyAsync(c->d_desc, c->h_desc, sizeof(ModelDesc) * n, hipMemcpyHostToDevice, c->stream));
  if (c->d_nnorder && n > 0) {
    // the non-negative update's grid order: NONNEG models first, highest rank first (a row's search costs about
    // rank^2 per solve), ties in slot order
    for (int k = 0; k < n; ++k) c->h_nnorder[k] = k;
    std::stable_sort(c->h_nnorder, c->h_nnorder + n, [c](int32_t x, int32_t y) {
      const ActiveModel& a = c->active[x];
      const ActiveModel& b = c->active[y];
      const int ka = (a.flags & CALS_MODEL_NONNEG) ? a.rank : 0, kb = (b.flags & CALS_MODEL_NONNEG) ? b.rank : 0;
      return ka > kb;
    });
    HIP_TRY(hipMemcpyAsync(c->d_nnorder, c->h_nnorder, sizeof(int32_t) * n, hipMemcpyHostToDevice, c->stream));
  }
  if (c->d_colmodel && n > 0) {
    for (int k = 0; k < n; ++k)
      for (int q = 0; q < c->active[k].rank; ++q) c->h_colmodel[c->active[k].col + q] = k;
    HIP_TRY(hipMemcpyAsync(c->d_colmodel, c->h_colmodel, sizeof(int32_t) * c->total_rank, hipMemcpyHostToDevice,
                           c->stream));
  }
  c->desc_dirty = false;
  return CALS_OK;
}

// Alg. 3, fill loop: take models from the queue front while they fit; stop at the first that does not.
// The new models' starting factors travel as ONE packed block per mode (pinned staging, one copy, one
// scatter kernel) and land in the columns right after the current ones.
int fill(cals_ctx* c) {
  const int first_new = (int)c->active.size();
  const int col0 = c->total_rank;
  std::vector<const PendingModel*> fresh;
  int newcols = 0;
  size_t n_take = 0;
  for (const PendingModel& pm : c->queue) {
    if (col0 + newcols + pm.rank > c->opt.max_total_rank) break;
    if ((int)c->active.size() + (int)fresh.size() >= c->capacity) break;
    fresh.push_back(&pm);
    newcols += pm.rank;
    ++n_take;
  }
  if (fresh.empty()) return CALS_OK;
  // pack: per mode a row-major I_n x newcols block
  size_t off = 0;
  size_t mode_off[kMaxModes];
  for (int n = 0; n < c->nmodes; ++n) {
    const int64_t In = c->dims[n];
    mode_off[n] = off;
    double* blk = c->h_stage + off;
    int cofs = 0;
    for (const PendingModel* pm : fresh) {
      const double* src = pm->init[n].data();
      for (int q = 0; q < pm->rank; ++q)
        for (int64_t i = 0; i < In; ++i) blk[(size_t)i * newcols + cofs + q] = src[(size_t)(i + In * q)];
      cofs += pm->rank;
    }
    off += (size_t)In * newcols;
  }
  HIP_TRY(hipMemcpyAsync(c->d_stage, c->h_stage, sizeof(double) * off, hipMemcpyHostToDevice, c->stream));
  for (int n = 0; n < c->nmodes; ++n)
    HIP_TRY(launch_copy_block(c->d_stage + mode_off[n], newcols, c->U[n] + col0, c->ld, (int)c->dims[n], newcols,
                              c->stream));
  int col = col0;
  for (const PendingModel* pm : fresh) {
    ActiveModel m;
    m.id = pm->id; m.rank = pm->rank; m.tol = pm->tol; m.max_iters = pm->max_iters; m.flags = pm->flags;
    m.alpha = pm->alpha; m.fit_prev = 0.0; m.iters = 0;
    m.sid = c->free_sids.back();
    c->free_sids.pop_back();
    m.col = col;
    col += m.rank;
    c->active.push_back(m);
  }
  c->total_rank = col;
  c->desc_dirty = true;
  CALS_TRY(upload_desc(c));
  int In[kMaxModes];
  for (int n = 0; n < c->nmodes; ++n) In[n] = (int)c->dims[n];
  HIP_TRY(launch_gram_init(c->d_desc, c->d_state, c->d_out, c->d_lambda, true, c->passive, c->capacity, c->U, In,
                           c->nmodes, c->ld, first_new, (int)fresh.size(), c->stream));
  // the staging buffer and the queue entries are free again once the copy has been consumed
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (size_t k = 0; k < n_take; ++k) c->queue.pop_front();
  return CALS_OK;
}

// Copies the factors and column norms of the models leaving this round to the host: one gather kernel and
// one contiguous copy per mode, then a host-side unpack into per-model column-major matrices.
int retire_models(cals_ctx* c, const std::vector<ActiveModel>& leaving, const std::vector<int>& statuses) {
  int outcols = 0;
  for (const ActiveModel& m : leaving) {
    for (int q = 0; q < m.rank; ++q) c->h_rmap[outcols + q] = m.col + q;
    outcols += m.rank;
  }
  HIP_TRY(hipMemcpyAsync(c->d_rmap, c->h_rmap, sizeof(int32_t) * outcols, hipMemcpyHostToDevice, c->stream));
  size_t off = 0;
  size_t mode_off[kMaxModes];
  for (int n = 0; n < c->nmodes; ++n) {
    mode_off[n] = off;
    HIP_TRY(launch_gather_block(c->U[n], c->ld, c->d_stage + off, outcols, c->d_rmap, (int)c->dims[n], outcols,
                                c->stream));
    off += (size_t)c->dims[n] * outcols;
  }
  HIP_TRY(hipMemcpyAsync(c->h_stage, c->d_stage, sizeof(double) * off, hipMemcpyDeviceToHost, c->stream));
  int max_sid = 0;
  for (const ActiveModel& m : leaving) max_sid = std::max(max_sid, m.sid);
  HIP_TRY(hipMemcpyAsync(c->h_lambda, c->d_lambda, sizeof(double) * kMaxRank * (max_sid + 1), hipMemcpyDeviceToHost,
                         c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  int cofs = 0;
  for (size_t k = 0; k < leaving.size(); ++k) {
    const ActiveModel& m = leaving[k];
    const ModelOut& o = c->h_out[m.sid];
    RetiredModel r;
    r.res.model_id = m.id;
    r.res.rank = m.rank;
    r.res.iters = o.iters;
    r.res.status = statuses[k];
    r.res.ls_accepted = o.ls_accepted;
    r.res.fit = o.fit;
    r.res.error = o.err;
    for (int n = 0; n < c->nmodes; ++n) {
      const int64_t In = c->dims[n];
      const double* blk = c->h_stage + mode_off[n];
      r.U[n].resize((size_t)In * m.rank);
      for (int q = 0; q < m.rank; ++q)
        for (int64_t i = 0; i < In; ++i) r.U[n][(size_t)(i + In * q)] = blk[(size_t)i * outcols + cofs + q];
    }
    r.lambda.assign(c->h_lambda + (size_t)m.sid * kMaxRank, c->h_lambda + (size_t)m.sid * kMaxRank + m.rank);
    cofs += m.rank;
    c->retired[m.id] = std::move(r);
    c->out_queue.push_back(m.id);
    c->free_sids.push_back(m.sid);
    c->n_retired += 1;
  }
  return CALS_OK;
}

// Stable left-compaction of the column blocks of the survivors (Sec. 4, "compression routine").
int compact(cals_ctx* c, const std::vector<ActiveModel>& survivors) {
  int col = 0;
  bool moved = false;
  std::vector<ActiveModel> out = survivors;
  for (ActiveModel& m : out) {
    for (int q = 0; q < m.rank; ++q) c->h_map[col + q] = m.col + q;
    if (m.col != col) moved = true;
    m.col = col;
    col += m.rank;
  }
  if (moved && col > 0) {
    HIP_TRY(hipMemcpyAsync(c->d_map, c->h_map, sizeof(int32_t) * col, hipMemcpyHostToDevice, c->stream));
    for (int n = 0; n < c->nmodes; ++n) {
      HIP_TRY(launch_gather_columns(c->U[n], c->Ualt[n], c->d_map, (int)c->dims[n], col, c->ld, c->stream));
      std::swap(c->U[n], c->Ualt[n]);
      if (c->Uprev[n]) {
        HIP_TRY(launch_gather_columns(c->Uprev[n], c->Ualt[n], c->d_map, (int)c->dims[n], col, c->ld, c->stream));
        std::swap(c->Uprev[n], c->Ualt[n]);
      }
    }
    if (c->Yprev) {
      HIP_TRY(launch_gather_columns(c->Yprev, c->Ynew, c->d_map, (int)rows_without_mode1(c), col, c->ld, c->stream));
      std::swap(c->Yprev, c->Ynew);
    }
    // h_map is reused next round: the copy above must have been consumed before it is rewritten
    HIP_TRY(hipStreamSynchronize(c->stream));
  }
  c->active.swap(out);
  c->total_rank = col;
  c->desc_dirty = true;
  return CALS_OK;
}

// A round's read-back can be postponed when no model can leave in it: nothing waits in the queue and every
// active model runs a fixed number of iterations that it has not reached yet.  (A model whose update fails
// numerically in such a round is noticed at the next read-back and then takes its place in the output queue
// by the round in which it failed, so the order is the same as with a read-back every round.)
bool round_may_retire(const cals_ctx* c) {
  if (!c->queue.empty()) return true;
  for (const ActiveModel& m : c->active)
    if (!(m.tol < 0.0) || m.iters + c->rounds_unread + 1 >= m.max_iters) return true;
  return false;
}

int one_round(cals_ctx* c, int* retired_now, bool last_of_call) {
  CALS_TRY(fill(c));
  const int n = (int)c->active.size();
  if (n == 0) return CALS_OK;
  CALS_TRY(upload_desc(c));
  const int N = c->nmodes;
  // one log record per round (the segments of the paper's efficiency measurement), timed by a pair of events
  constexpr size_t kMaxRoundLog = (size_t)1 << 20;
  const bool logged = c->round_log.size() < kMaxRoundLog;
  const double flops_before = c->mttkrp_flops;
  TimedRound tr{};
  bool round_timed = false;
  if (logged) {
    cals_round_record rec{};
    rec.round = c->rounds; rec.n_active = n; rec.total_rank = c->total_rank; rec.ms = 0.0; rec.mttkrp_flops = 0.0;
    c->round_log.push_back(rec);
    if (c->opt.flags & CALS_CTX_TIMING) {
      tr.ev[0] = take_event(c);
      tr.ev[1] = take_event(c);
      if (tr.ev[0] && tr.ev[1]) {
        tr.index = c->round_log.size() - 1;
        round_timed = hipEventRecord(tr.ev[0], c->stream) == hipSuccess;
      }
      if (!round_timed) {
        (void)hipGetLastError();
        if (tr.ev[0]) c->event_pool.push_back(tr.ev[0]);
        if (tr.ev[1]) c->event_pool.push_back(tr.ev[1]);
      }
    }
  }
  for (int mode = 0; mode < N; ++mode) {
    if (c->Y && mode > 0) {
      // two-step sweep: modes 2 and 3 come from the tensor contracted with the mode-1 factors just updated
      if (mode == 1) CALS_TRY(run_contract_mode1(c, c->U[0], c->total_rank, c->ld));
      CALS_TRY(run_from_contraction(c, mode, c->U, c->M, c->total_rank, c->ld));
    } else {
      CALS_TRY(run_mttkrp(c, mode, c->U, c->M, c->total_rank, c->ld));
    }
    bool round_has_nn = false;
    int nn_max_rank = 1;
    for (const ActiveModel& m : c->active)
      if (m.flags & CALS_MODEL_NONNEG) {
        round_has_nn = true;
        nn_max_rank = std::max(nn_max_rank, m.rank);
      }
    if (round_has_nn) {
      // rows of the NONNEG models, solved into the spare multi-matrix (free between compactions)
      NnlsArgs na{};
      na.desc = c->d_desc; na.state = c->d_state; na.out = c->d_out; na.M = c->M; na.X = c->Ualt[mode];
      na.passive = c->passive[mode]; na.fail = c->d_nnfail; na.order = c->d_nnorder;
      na.In = (int)c->dims[mode]; na.ld = c->ld; na.mode = mode; na.nmodes = N; na.n_models = n; na.capacity = c->capacity; na.max_rank = nn_max_rank;
      HIP_TRY(launch_nnls(na, c->stream));
    }
    UpdateArgs ua{};
    ua.desc = c->d_desc; ua.state = c->d_state; ua.out = c->d_out; ua.lambda = c->d_lambda;
    ua.M = c->M; ua.U = c->U[mode]; ua.X = c->Ualt[mode]; ua.nn_fail = c->d_nnfail;
    ua.In = (int)c->dims[mode]; ua.ld = c->ld; ua.mode = mode; ua.nmodes = N;
    ua.n_models = n; ua.normT2 = c->normT2; ua.part = c->d_updpart;
    HIP_TRY(launch_update(ua, c->stream));
  }
  // line search (Sec. 5): extrapolate, one extra fused MTTKRP of the last mode at the extrapolated point, decide, apply
  bool round_has_ls = false, ls_takes_part = false;
  for (const ActiveModel& m : c->active)
    if (m.flags & CALS_MODEL_LINESEARCH) {
      round_has_ls = true;
      if (m.iters + c->rounds_unread + 1 >= 2) ls_takes_part = true;
    }
  if (round_has_ls) {
    LineSearchArgs la{};
    la.desc = c->d_desc; la.state = c->d_state; la.out = c->d_out; la.lambda = c->d_lambda;
    la.colmodel = c->d_colmodel; la.accept = c->d_accept;
    la.nmodes = N;
    for (int k = 0; k < N; ++k) {
      la.U[k] = c->U[k]; la.Uprev[k] = c->Uprev[k]; la.Unew[k] = c->Unew[k]; la.In[k] = (int)c->dims[k];
    }
    // the extra MTTKRP: of the longest mode (best-shaped contraction: most rows, e.g. 4000 instead of 50), or of the
    // last mode when it comes from the contraction of a two-step sweep
    int ls_mode = N - 1;
    if (!c->Y) ls_mode = (int)(std::max_element(c->dims, c->dims + N) - c->dims);
    la.ls_mode = ls_mode;
    la.M3 = c->M; la.ld = c->ld; la.n_models = n; la.ncols = c->total_rank; la.normT2 = c->normT2;
    la.part = c->d_lspart;
    la.nblk = update_row_blocks((int)*std::max_element(c->dims, c->dims + N));
    la.Ycur = c->Y; la.Yprev = c->Yprev; la.Ynew = c->Ynew; la.yrows = c->Y ? rows_without_mode1(c) : 0;
    if (ls_takes_part) {
      HIP_TRY(launch_ls_extrapolate(la, c->stream));
      if (c->Y && c->Yprev) {
        // the extrapolated mode-1 factors are a linear combination unless a NONNEG model's were clipped
        bool linear = true;
        for (const ActiveModel& m : c->active)
          if ((m.flags & CALS_MODEL_LINESEARCH) && (m.flags & CALS_MODEL_NONNEG)) linear = false;
        if (linear) HIP_TRY(launch_ls_y_combine(la, c->stream));
        else CALS_TRY(run_contract_mode1(c, c->Unew[0], c->total_rank, c->ld, c->Ynew));
        CALS_TRY(run_from_contraction(c, N - 1, c->Unew, c->M, c->total_rank, c->ld, /*rebuild=*/true, c->Ynew));
      } else if (c->Y) {
        CALS_TRY(run_contract_mode1(c, c->Unew[0], c->total_rank, c->ld));
        CALS_TRY(run_from_contraction(c, N - 1, c->Unew, c->M, c->total_rank, c->ld, /*rebuild=*/true));
      } else {
        CALS_TRY(run_mttkrp(c, ls_mode, c->Unew, c->M, c->total_rank, c->ld));
      }
    }
    HIP_TRY(launch_ls_decide(la, c->stream));
    HIP_TRY(launch_ls_apply(la, c->stream));
    if (c->Yprev) HIP_TRY(launch_ls_y_keep(la, c->stream));   // no model took part: nothing accepted, Yprev = Y
  }
  if (logged) c->round_log.back().mttkrp_flops = c->mttkrp_flops - flops_before;
  if (round_timed) {
    (void)hipEventRecord(tr.ev[1], c->stream);
    c->timed_rounds.push_back(tr);
    if (c->timed_rounds.size() > 4096) CALS_TRY(drain_timings(c));
  }
  c->rounds += 1;
  if (!last_of_call && !round_may_retire(c)) {
    c->rounds_unread += 1;
    return CALS_OK;
  }
  // the only per-round readback: fit, error, status and iteration count of every slot in use
  int max_sid = 0;
  for (const ActiveModel& m : c->active) max_sid = std::max(max_sid, m.sid);
  HIP_TRY(hipMemcpyAsync(c->h_out, c->d_out, sizeof(ModelOut) * (max_sid + 1), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  const int64_t unread = c->rounds_unread;     // rounds before this one whose records were not read
  c->rounds_unread = 0;

  // Alg. 3, removal loop: slots in order; a model leaves when its fit changed by less than tol between two
  // consecutive iterations, when it reached its iteration cap, or when its update failed numerically.
  std::vector<ActiveModel> survivors;
  std::vector<Leaving> gone;
  survivors.reserve(c->active.size());
  int slot = 0;
  for (ActiveModel& m : c->active) {
    const ModelOut& o = c->h_out[m.sid];
    int status = CALS_RUNNING;
    int64_t round = c->rounds;
    if (o.status == CALS_NUMERICAL) {
      status = CALS_NUMERICAL;
      // it failed in the iteration after its last completed one; rounds since the previous read-back: unread + 1
      round = c->rounds - (unread + 1) + (o.iters - m.iters) + 1;
    } else if (o.iters >= 2 && std::fabs(o.fit - m.fit_prev) < m.tol) status = CALS_CONVERGED;
    else if (o.iters >= m.max_iters) status = CALS_MAX_ITERS;
    m.fit_prev = o.fit;
    m.iters = o.iters;
    if (status != CALS_RUNNING) {
      gone.push_back(Leaving{m, status, round, slot});
      *retired_now += 1;
    } else {
      survivors.push_back(m);
    }
    ++slot;
  }
  if (!gone.empty()) {
    std::stable_sort(gone.begin(), gone.end(), [](const Leaving& x, const Leaving& y) {
      return x.round != y.round ? x.round < y.round : x.slot < y.slot;
    });
    std::vector<ActiveModel> leaving;
    std::vector<int> statuses;
    for (const Leaving& g : gone) { leaving.push_back(g.m); statuses.push_back(g.status); }
    CALS_TRY(retire_models(c, leaving, statuses));
    CALS_TRY(compact(c, survivors));
  }
  return CALS_OK;
}

// No C++ exception leaves the library: the host containers' allocation failures become CALS_E_NOMEM.
template <class F>
int guarded(F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return CALS_E_NOMEM;
  } catch (...) {
    return CALS_E_STATE;
  }
}

}  // namespace

extern "C" {

int cals_create(cals_ctx** out, const cals_options* opt) {
  if (!out || !opt) return CALS_E_INVALID;
  *out = nullptr;
  if (opt->max_total_rank < 1 || opt->max_total_rank > (1 << 20) || opt->max_slots < 0) return CALS_E_INVALID;
  if (opt->device < 0 || opt->device >= kMaxDevices) return CALS_E_INVALID;
  cals_ctx* c = new (std::nothrow) cals_ctx();
  if (!c) return CALS_E_NOMEM;
  c->opt = *opt;
  c->stream = reinterpret_cast<hipStream_t>(opt->stream);
  int rc = CALS_OK;
  hipDeviceProp_t prop;
  if (hipSetDevice(opt->device) != hipSuccess || hipGetDeviceProperties(&prop, opt->device) != hipSuccess ||
      mttkrp_init() != hipSuccess) {
    (void)hipGetLastError();
    rc = CALS_E_HIP;
  }
  if (rc == CALS_OK) rc = scratch_address(opt->device, &c->scratch_dev);   // the device is current here
  if (rc != CALS_OK) { delete c; return rc; }
  c->tune = mttkrp_tuning_from_env();
  c->num_cus = prop.multiProcessorCount;
  c->ld = (int)((opt->max_total_rank + 15) / 16 * 16);
  c->capacity = opt->max_slots > 0 ? opt->max_slots : (int)std::min<int64_t>(opt->max_total_rank, 4096);
  *out = c;
  return CALS_OK;
}

int cals_destroy(cals_ctx* c) {
  if (!c) return CALS_E_INVALID;
  (void)hipSetDevice(c->opt.device);
  (void)hipStreamSynchronize(c->stream);
  for (TimedLaunch& t : c->timed)
    for (int i = 0; i < 4; ++i) (void)hipEventDestroy(t.ev[i]);
  for (TimedRound& t : c->timed_rounds)
    for (int i = 0; i < 2; ++i) (void)hipEventDestroy(t.ev[i]);
  for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
  for (int n = 0; n < kMaxModes; ++n) {
    (void)hipFree(c->U[n]); (void)hipFree(c->Ualt[n]); (void)hipFree(c->Uprev[n]); (void)hipFree(c->Unew[n]);
    (void)hipFree(c->passive[n]);
  }
  (void)hipFree(c->Kbuf[0]); (void)hipFree(c->Kbuf[1]);
  for (int n = 0; n < kMaxModes; ++n) (void)hipFree(c->Ychain[n]);
  (void)hipFree(c->M); (void)hipFree(c->workspace); (void)hipFree(c->d_desc); (void)hipFree(c->d_state);
  (void)hipFree(c->d_out); (void)hipFree(c->d_map); (void)hipFree(c->d_scratch); (void)hipFree(c->T_owned); (void)hipFree(c->d_updpart); (void)hipFree(c->d_lspart);
  (void)hipFree(c->d_nnfail); (void)hipFree(c->d_nnorder); (void)hipHostFree(c->h_nnorder); (void)hipFree(c->d_colmodel); (void)hipFree(c->d_accept); (void)hipHostFree(c->h_colmodel);
  (void)hipFree(c->d_sink); (void)hipFree(c->Y); (void)hipFree(c->Yprev); (void)hipFree(c->Ynew); (void)hipFree(c->d_ones);
  (void)hipFree(c->d_zeros); (void)hipFree(c->d_lambda); (void)hipFree(c->d_stage); (void)hipFree(c->d_rmap);
  (void)hipHostFree(c->h_desc); (void)hipHostFree(c->h_out); (void)hipHostFree(c->h_map);
  (void)hipHostFree(c->h_lambda); (void)hipHostFree(c->h_stage); (void)hipHostFree(c->h_rmap);
  delete c;
  return CALS_OK;
}

int cals_submit_tensor(cals_ctx* c, const double* data, const int64_t dims[3], int on_device) {
  return cals_submit_tensor_nd(c, data, 3, dims, on_device);
}

static int submit_tensor_nd(cals_ctx* c, const double* data, int32_t ndims, const int64_t* dims, int on_device) {
  if (!c || !data || !dims) return CALS_E_INVALID;
  if (ndims < 3 || ndims > CALS_MAX_MODES) return CALS_E_INVALID;
  if (c->has_tensor || c->nmodes != 0) return CALS_E_STATE;   // also after an attempt that failed half-way
  int64_t total = 1;
  for (int n = 0; n < ndims; ++n) {
    if (dims[n] < 1 || dims[n] >= (1LL << 31)) return CALS_E_INVALID;
    total *= dims[n];
    if (total >= (1LL << 40)) return CALS_E_INVALID;
  }
  CALS_TRY(set_device(c));
  c->nmodes = ndims;
  for (int n = 0; n < ndims; ++n) c->dims[n] = dims[n];
  if (on_device) {
    c->T = data;
  } else {
    if (hipMalloc(&c->T_owned, sizeof(double) * (size_t)total) != hipSuccess) { (void)hipGetLastError(); return CALS_E_NOMEM; }
    HIP_TRY(hipMemcpy(c->T_owned, data, sizeof(double) * (size_t)total, hipMemcpyHostToDevice));
    c->T = c->T_owned;
  }
  // buffers: one factor multi-matrix per mode (+ a spare set for compaction), the MTTKRP result, per-model storage
  const int64_t imax = *std::max_element(dims, dims + ndims);
  bool ok = true;
  for (int n = 0; n < ndims; ++n) {
    const size_t bytes = sizeof(double) * (size_t)dims[n] * c->ld;
    ok = ok && hipMalloc(&c->U[n], bytes) == hipSuccess && hipMalloc(&c->Ualt[n], bytes) == hipSuccess;
    if (ok) ok = hipMemsetAsync(c->U[n], 0, bytes, c->stream) == hipSuccess &&
                 hipMemsetAsync(c->Ualt[n], 0, bytes, c->stream) == hipSuccess;
  }
  ok = ok && hipMalloc(&c->M, sizeof(double) * (size_t)imax * c->ld) == hipSuccess;
  ok = ok && hipMalloc(&c->d_desc, sizeof(ModelDesc) * c->capacity) == hipSuccess;
  ok = ok && hipMalloc(&c->d_state, sizeof(ModelState) * (size_t)c->capacity) == hipSuccess;
  ok = ok && hipMalloc(&c->d_out, sizeof(ModelOut) * c->capacity) == hipSuccess;
  ok = ok && hipMalloc(&c->d_map, sizeof(int32_t) * c->ld) == hipSuccess;
  ok = ok && hipMalloc(&c->d_scratch, sizeof(double) * 1032) == hipSuccess;
  // order above 3: room for the explicit Khatri-Rao products of the contracted runs (largest over the modes)
  {
    int64_t need[2] = {0, 0};
    for (int n = 0; n < ndims; ++n) {
      const Runs r = contraction_runs(c, n);
      if (r.a1 - r.a0 > 1) need[0] = std::max(need[0], r.Ia);
      if (r.b1 - r.b0 > 1) need[1] = std::max(need[1], r.Ib);
      if ((c->opt.flags & CALS_CTX_REUSE) && ndims > 3 && n >= 1) {   // second step of two-step sweeps: runs 2..n-1, n+1..N
        int64_t pr = 1;
        for (int m = n + 1; m < ndims; ++m) pr *= dims[m];
        if (n < ndims - 2) need[1] = std::max(need[1], pr);
      }
    }
    for (int q = 0; q < 2; ++q)
      if (need[q] > 0) {
        const size_t bytes = sizeof(double) * (size_t)need[q] * c->ld;
        ok = ok && hipMalloc(&c->Kbuf[q], bytes) == hipSuccess;
        if (ok) ok = hipMemsetAsync(c->Kbuf[q], 0, bytes, c->stream) == hipSuccess;
      }
  }
  if ((c->opt.flags & CALS_CTX_REUSE) && rows_without_mode1(c) < (1LL << 31)) {
    ok = ok && hipMalloc(&c->Y, sizeof(double) * (size_t)rows_without_mode1(c) * c->ld) == hipSuccess;
    ok = ok && hipMalloc(&c->d_ones, sizeof(double) * c->ld) == hipSuccess;
    ok = ok && launch_fill(c->d_ones, c->ld, 1.0, c->stream) == hipSuccess;
    for (int level = 2; ndims > 3 && level < ndims; ++level)
      ok = ok && hipMalloc(&c->Ychain[level], sizeof(double) * (size_t)chain_rows(c, level) * c->ld) == hipSuccess;
  }
  if (update_row_blocks((int)imax) > 1)
    ok = ok && hipMalloc(&c->d_updpart, sizeof(double) * update_part_doubles((int)imax) * c->capacity) == hipSuccess;
  ok = ok && hipMalloc(&c->d_zeros, sizeof(double) * 8) == hipSuccess;
  ok = ok && hipMemsetAsync(c->d_zeros, 0, sizeof(double) * 8, c->stream) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_desc, sizeof(ModelDesc) * c->capacity) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_out, sizeof(ModelOut) * c->capacity) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_map, sizeof(int32_t) * c->ld) == hipSuccess;
  int64_t dim_sum = 0;
  for (int n = 0; n < ndims; ++n) dim_sum += dims[n];
  const size_t stage_doubles = (size_t)dim_sum * c->ld;
  ok = ok && hipMalloc(&c->d_lambda, sizeof(double) * kMaxRank * c->capacity) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_lambda, sizeof(double) * kMaxRank * c->capacity) == hipSuccess;
  ok = ok && hipMalloc(&c->d_stage, sizeof(double) * stage_doubles) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_stage, sizeof(double) * stage_doubles) == hipSuccess;
  ok = ok && hipMalloc(&c->d_rmap, sizeof(int32_t) * c->ld) == hipSuccess;
  ok = ok && hipHostMalloc(&c->h_rmap, sizeof(int32_t) * c->ld) == hipSuccess;
  if (!ok) { (void)hipGetLastError(); return CALS_E_NOMEM; }
  CALS_TRY(ensure_workspace(c, largest_round_workspace(c)));
  HIP_TRY(hipMemsetAsync(c->d_out, 0, sizeof(ModelOut) * c->capacity, c->stream));
  c->free_sids.clear();
  for (int s = c->capacity - 1; s >= 0; --s) c->free_sids.push_back(s);
  // ||T||^2 once (Alg. 1, error line: the tensor term is computed once at the start), and a NaN/Inf scan
  int* d_flag = reinterpret_cast<int*>(c->d_scratch + 1025);
  HIP_TRY(hipMemsetAsync(d_flag, 0, sizeof(int), c->stream));
  HIP_TRY(launch_norm_sq(c->T, total, c->d_scratch, c->d_scratch + 1024, d_flag, c->stream));
  double nrm = 0.0;
  int flag = 0;
  HIP_TRY(hipMemcpyAsync(&nrm, c->d_scratch + 1024, sizeof(double), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipMemcpyAsync(&flag, d_flag, sizeof(int), hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (flag != 0 || !std::isfinite(nrm)) return CALS_E_INVALID;
  c->normT2 = nrm;
  c->has_tensor = true;
  return CALS_OK;
}

int cals_submit_tensor_nd(cals_ctx* c, const double* data, int32_t ndims, const int64_t* dims, int on_device) {
  return guarded([&] { return submit_tensor_nd(c, data, ndims, dims, on_device); });
}

static int enqueue_model(cals_ctx* c, int32_t rank, const double* const* init, double tol, int32_t max_iters,
                         uint32_t flags, double ls_alpha, int64_t* model_id) {
  if (!c || !init) return CALS_E_INVALID;
  if (!c->has_tensor) return CALS_E_STATE;
  if (rank < 1 || rank > CALS_MAX_RANK || rank > c->opt.max_total_rank || max_iters < 1) return CALS_E_INVALID;
  if (std::isnan(tol)) return CALS_E_INVALID;
  if (flags & ~(CALS_MODEL_NONNEG | CALS_MODEL_LINESEARCH)) return CALS_E_INVALID;
  if ((flags & CALS_MODEL_LINESEARCH) && !std::isfinite(ls_alpha)) return CALS_E_INVALID;
  if (flags & CALS_MODEL_NONNEG) CALS_TRY(ensure_nn_buffers(c));
  if (flags & CALS_MODEL_LINESEARCH) CALS_TRY(ensure_ls_buffers(c));
  PendingModel pm;
  pm.id = c->next_id;
  pm.rank = rank; pm.tol = tol; pm.max_iters = max_iters; pm.flags = flags; pm.alpha = ls_alpha;
  for (int n = 0; n < c->nmodes; ++n) {
    if (!init[n]) return CALS_E_INVALID;
    const int64_t In = c->dims[n];
    if (!all_finite(init[n], In * rank)) return CALS_E_INVALID;
    pm.init[n].assign(init[n], init[n] + (size_t)In * rank);
  }
  c->queue.push_back(std::move(pm));
  if (model_id) *model_id = c->next_id;
  c->next_id += 1;
  return CALS_OK;
}

int cals_enqueue_model(cals_ctx* c, int32_t rank, const double* const* init, double tol, int32_t max_iters,
                       uint32_t flags, double ls_alpha, int64_t* model_id) {
  return guarded([&] { return enqueue_model(c, rank, init, tol, max_iters, flags, ls_alpha, model_id); });
}

static int iterate(cals_ctx* c, int32_t n_rounds, int32_t* n_retired) {
  if (!c || n_rounds < 0) return CALS_E_INVALID;
  if (!c->has_tensor) return CALS_E_STATE;
  CALS_TRY(set_device(c));
  int retired_now = 0;
  if (n_retired) *n_retired = 0;
  for (int r = 0; r < n_rounds; ++r) {
    if (c->queue.empty() && c->active.empty()) break;
    CALS_TRY(one_round(c, &retired_now, r + 1 == n_rounds));
    if (n_retired) *n_retired = retired_now;
  }
  return CALS_OK;
}

int cals_iterate(cals_ctx* c, int32_t n_rounds, int32_t* n_retired) {
  return guarded([&] { return iterate(c, n_rounds, n_retired); });
}

int cals_run(cals_ctx* c) {
  if (!c) return CALS_E_INVALID;
  if (!c->has_tensor) return CALS_E_STATE;
  while (!(c->queue.empty() && c->active.empty())) CALS_TRY(cals_iterate(c, 64, nullptr));
  return CALS_OK;
}

int cals_poll_retired(cals_ctx* c, cals_result* out, int32_t cap, int32_t* n) {
  if (!c || !n || cap < 0 || (cap > 0 && !out)) return CALS_E_INVALID;
  int k = 0;
  while (k < cap && !c->out_queue.empty()) {
    out[k++] = c->retired[c->out_queue.front()].res;
    c->out_queue.pop_front();
  }
  *n = k;
  return CALS_OK;
}

int cals_get_factors(cals_ctx* c, int64_t model_id, double* const* U, double* lambda) {
  if (!c) return CALS_E_INVALID;
  auto it = c->retired.find(model_id);
  if (it == c->retired.end()) return CALS_E_NOTFOUND;
  const RetiredModel& r = it->second;
  if (U)
    for (int n = 0; n < c->nmodes; ++n)
      if (U[n]) std::memcpy(U[n], r.U[n].data(), sizeof(double) * r.U[n].size());
  if (lambda) std::memcpy(lambda, r.lambda.data(), sizeof(double) * r.lambda.size());
  return CALS_OK;
}

int cals_mttkrp(cals_ctx* c, int32_t mode, int32_t total_rank, int64_t ld, const double* const* U_dev,
                double* M_dev) {
  if (!c || !U_dev || !M_dev) return CALS_E_INVALID;
  if (!c->has_tensor) return CALS_E_STATE;
  if (mode < 1 || mode > c->nmodes || total_rank < 1 || ld < total_rank || ld >= (1LL << 24)) return CALS_E_INVALID;
  if (c->nmodes > 3 && ld > c->ld) return CALS_E_INVALID;
  for (int n = 0; n < c->nmodes; ++n)
    if (n != mode - 1 && !U_dev[n]) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  return run_mttkrp(c, mode - 1, U_dev, M_dev, total_rank, (int)ld);
}

int cals_mttkrp_noalloc(cals_ctx* c, int32_t mode, int32_t total_rank, int64_t ld, const double* const* U_dev,
                        double* M_dev) {
  if (!c || !U_dev || !M_dev) return CALS_E_INVALID;
  if (!c->has_tensor) return CALS_E_STATE;
  if (mode < 1 || mode > c->nmodes || total_rank < 1 || ld < total_rank || ld >= (1LL << 24)) return CALS_E_INVALID;
  if (c->nmodes > 3 && ld > c->ld) return CALS_E_INVALID;
  for (int n = 0; n < c->nmodes; ++n)
    if (n != mode - 1 && !U_dev[n]) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  return run_mttkrp(c, mode - 1, U_dev, M_dev, total_rank, (int)ld, /*no_alloc=*/true);
}

int cals_mttkrp_reuse(cals_ctx* c, int32_t total_rank, int64_t ld, const double* const U_dev[3], double* M2_dev,
                      double* M3_dev) {
  if (!c || !U_dev || !M2_dev || !M3_dev) return CALS_E_INVALID;
  if (!c->T || !c->Y) return CALS_E_STATE;
  if (total_rank < 1 || ld < total_rank || ld > c->ld) return CALS_E_INVALID;
  for (int n = 0; n < 3; ++n)
    if (!U_dev[n]) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  if (c->nmodes != 3) return CALS_E_STATE;
  CALS_TRY(run_contract_mode1(c, U_dev[0], total_rank, (int)ld));
  CALS_TRY(run_from_contraction(c, 1, U_dev, M2_dev, total_rank, (int)ld));
  CALS_TRY(run_from_contraction(c, 2, U_dev, M3_dev, total_rank, (int)ld));
  return CALS_OK;
}

int cals_mttkrp_reuse_nd(cals_ctx* c, int32_t total_rank, int64_t ld, const double* const* U_dev, double* const* M_dev) {
  if (!c || !U_dev || !M_dev) return CALS_E_INVALID;
  if (!c->T || !c->Y) return CALS_E_STATE;
  if (total_rank < 1 || ld < total_rank || ld > c->ld) return CALS_E_INVALID;
  for (int n = 0; n < c->nmodes; ++n)
    if (!U_dev[n] || (n >= 1 && !M_dev[n])) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  CALS_TRY(run_contract_mode1(c, U_dev[0], total_rank, (int)ld));
  for (int n = 1; n < c->nmodes; ++n) CALS_TRY(run_from_contraction(c, n, U_dev, M_dev[n], total_rank, (int)ld));
  return CALS_OK;
}

int cals_get_round_log(cals_ctx* c, int64_t first_round, cals_round_record* out, int32_t cap, int32_t* n) {
  if (!c || !n || cap < 0 || first_round < 0 || (cap > 0 && !out)) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  CALS_TRY(drain_timings(c));
  int k = 0;
  for (size_t i = (size_t)first_round; i < c->round_log.size() && k < cap; ++i) out[k++] = c->round_log[i];
  *n = k;
  return CALS_OK;
}

int cals_get_stats(cals_ctx* c, cals_stats* s) {
  if (!c || !s) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  CALS_TRY(drain_timings(c));
  s->rounds = c->rounds;
  s->models_retired = c->n_retired;
  s->models_queued = (int64_t)c->queue.size();
  s->n_active = (int32_t)c->active.size();
  s->total_rank = c->total_rank;
  s->tensor_norm_sq = c->normT2;
  s->mttkrp_flops = c->mttkrp_flops;
  for (int n = 0; n < CALS_MAX_MODES; ++n) {
    s->mttkrp_ms[n] = c->mttkrp_ms[n];
    s->reduce_ms[n] = c->reduce_ms[n];
    s->mttkrp_launches[n] = c->mttkrp_launches[n];
  }
  s->mttkrp_rows_launches = c->mttkrp_rows_launches;
  return CALS_OK;
}

int cals_yardstick(cals_ctx* c, int32_t kind, const void* buf, int64_t bytes, int32_t reps, double* value) {
  if (!c || !value) return CALS_E_INVALID;
  if (kind == CALS_YARDSTICK_CLOCK_MHZ || kind == CALS_YARDSTICK_COMPUTE_UNITS) {
    int v = 0;
    HIP_TRY(hipDeviceGetAttribute(&v, kind == CALS_YARDSTICK_CLOCK_MHZ ? hipDeviceAttributeClockRate
                                                                         : hipDeviceAttributeMultiprocessorCount,
                                  c->opt.device));
    *value = (kind == CALS_YARDSTICK_CLOCK_MHZ) ? v * 1e-3 : (double)v;
    return CALS_OK;
  }
  if (reps < 1 || reps > 100) return CALS_E_INVALID;
  if (kind != CALS_YARDSTICK_MFMA && kind != CALS_YARDSTICK_READ) return CALS_E_INVALID;
  if (kind == CALS_YARDSTICK_READ && (!buf || bytes < (1 << 20) || (reinterpret_cast<uintptr_t>(buf) & 15))) return CALS_E_INVALID;
  CALS_TRY(set_device(c));
  if (!c->d_sink && hipMalloc(&c->d_sink, sizeof(double) * 8) != hipSuccess) { (void)hipGetLastError(); return CALS_E_NOMEM; }
  HIP_TRY(launch_yardstick(kind, buf, bytes, reps, c->num_cus, c->d_sink, c->stream, value));
  return CALS_OK;
}

const char* cals_strerror(int code) {
  switch (code) {
    case CALS_OK: return "ok";
    case CALS_E_INVALID: return "invalid argument";
    case CALS_E_STATE: return "call not allowed in this state";
    case CALS_E_NOMEM: return "out of memory";
    case CALS_E_HIP: return "HIP runtime error";
    case CALS_E_UNSUPPORTED: return "not supported";
    case CALS_E_NOTFOUND: return "model not found or not finished";
    case CALS_E_TOOLARGE: return "launch needs more scratch than the fixed buffer of the no-allocation entry point holds";
    default: return "unknown error code";
  }
}

}  // extern "C"
