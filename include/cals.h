/*
 * cals.h -- C boundary of the MI355X (gfx950) implementation of Concurrent ALS (CALS):
 * many CP-ALS instances on one dense fp64 tensor of order N = 3 (the paper's case) up to CALS_MAX_MODES,
 * advanced in lock-step so that the N MTTKRPs of an iteration are each ONE fused contraction over the
 * concatenated factor matrices.
 *
 * The update of a mode is U = M H^+ (Alg. 1): through a Cholesky factorisation while H is numerically positive
 * definite (every pivot above 1e-12 of its diagonal entry), else through the pseudo-inverse from an
 * eigen-decomposition (eigenvalues up to 1e-12 of the largest count as zero), so a model with dead or duplicated
 * components keeps running.
 *
 * The calls follow the problem statement of the paper's full algorithm (Alg. 3): a tensor, an
 * input queue of starting points, a main loop (fill, advance all active instances one iteration,
 * remove converged instances), and an output queue.
 *
 * Conventions
 *   - Every function returns CALS_OK (0) or a negative CALS_E_* code; nothing throws or aborts.
 *   - "host" / "device" on a pointer says where the memory lives.  The library never frees a
 *     caller pointer.
 *   - Tensor memory order: first index fastest, element (i1,i2,i3) at i1 + I1*(i2 + I2*i3); order N likewise.
 *   - Arrays indexed by mode (dims, init, U, U_dev) have one entry per mode of the tensor: N entries.
 *   - Per-model factor matrices cross the boundary column-major, I_n x rank, ld = I_n.
 *   - Device multi-matrices (cals_mttkrp) are ROW-major: row i of mode n holds the total_rank
 *     concatenated columns of all models, leading dimension `ld` doubles.
 *   - A context is not thread-safe.  All work is enqueued on the stream given at creation.
 *   - The library needs its HIP code object; there is no CPU fallback of any kind.
 */
#ifndef CALS_H
#define CALS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CALS_OK 0
#define CALS_E_INVALID (-1)     /* bad argument (null pointer, size, NaN/Inf, rank out of range) */
#define CALS_E_STATE (-2)       /* call not allowed in this state (e.g. no tensor yet)           */
#define CALS_E_NOMEM (-3)       /* host or device allocation failed                             */
#define CALS_E_HIP (-4)         /* a HIP runtime call failed                                    */
#define CALS_E_UNSUPPORTED (-5) /* valid request the library does not implement                 */
#define CALS_E_NOTFOUND (-6)    /* unknown model id / model not finished                        */
#define CALS_E_TOOLARGE (-7)    /* cals_mttkrp_noalloc: the launch needs more scratch than the fixed buffer holds */

/* model status (cals_result.status) */
#define CALS_RUNNING 0
#define CALS_CONVERGED 1   /* |fit - fit_prev| < tol at an iteration >= 2            */
#define CALS_MAX_ITERS 2   /* iteration cap reached                                   */
#define CALS_NUMERICAL 3   /* normal equations non-finite or without a positive eigenvalue (plain update), or a
                              singular block met by the non-negative search; factors of the last good point */

/* per-model flags (cals_enqueue_model) */
#define CALS_MODEL_NONNEG 1u     /* non-negative factors by an active-set method (Sec. 5)      */
#define CALS_MODEL_LINESEARCH 2u /* extrapolate after each iteration, keep if better (Sec. 5)  */

/* context flags (cals_options.flags) */
#define CALS_CTX_TIMING 1u /* bracket every MTTKRP launch with HIP events (read by cals_get_stats) */
#define CALS_CTX_REUSE 2u  /* two-step sweeps: after the mode-1 update, contract the tensor once with the new
                              mode-1 multi-matrix (Y[(i2,i3),c] = sum_i1 T * U1) and obtain the mode-2 and mode-3
                              MTTKRPs from Y instead of from the tensor (partial-contraction reuse, the scheme of
                              Phan et al. cited in Sec. 2; same results up to rounding order, one pass over the
                              tensor fewer per sweep).  Costs a device buffer of I2*I3*ld doubles.  Order N > 3
                              likewise: Y has one row per (i2,...,iN) -- I2*...*IN*ld doubles -- and is contracted
                              further with every updated mode in turn (each level 1/I_k of the one before), so a
                              sweep reads the tensor twice and Y twice instead of the tensor N times.
                              With line-search models in the queue, up to two more buffers of Y's size may be held
                              (Y at the point each model kept and at the extrapolated point, which is their
                              combination: Y is linear in the mode-1 factors); if they cannot be allocated, or would
                              cost more time than they save, the extrapolated point is contracted on its own. */

#define CALS_MAX_RANK 32 /* largest number of components of one model */
#define CALS_MAX_MODES 6 /* largest tensor order */

typedef struct cals_ctx cals_ctx; /* opaque; one per tensor */

typedef struct {
  int64_t max_total_rank; /* R*: width of the factor multi-matrix buffers (Sec. 4); >= largest rank */
  int32_t max_slots;      /* cap on simultaneously active models; 0 = limited by R* only            */
  int32_t device;         /* HIP device ordinal                                                     */
  void* stream;           /* hipStream_t to enqueue on (0 = the null stream); never created here    */
  uint32_t flags;         /* CALS_CTX_*                                                             */
} cals_options;

typedef struct {
  int64_t model_id; /* enqueue order: 0,1,2,... */
  int32_t rank;
  int32_t iters;  /* completed iterations */
  int32_t status; /* CALS_CONVERGED | CALS_MAX_ITERS | CALS_NUMERICAL */
  int32_t ls_accepted; /* accepted extrapolation steps */
  double fit;     /* 1 - ||T - model|| / ||T|| after the last completed iteration */
  double error;   /* ||T - model||^2 by the fast formula (Alg. 1, error line)     */
} cals_result;

typedef struct {
  int64_t rounds;            /* main-loop rounds executed (Alg. 3)                           */
  int64_t models_retired;
  int64_t models_queued;     /* still waiting in the input queue                             */
  int32_t n_active;
  int32_t total_rank;        /* fused width right now                                        */
  double tensor_norm_sq;     /* ||T||^2                                                      */
  double mttkrp_flops;       /* algorithmic: 2 * fused width * prod(I) per launch, summed    */
  double mttkrp_ms[CALS_MAX_MODES];  /* per mode, main contraction kernel only (needs CALS_CTX_TIMING) */
  double reduce_ms[CALS_MAX_MODES];  /* per mode, split-K reduction kernel (needs CALS_CTX_TIMING)     */
  int64_t mttkrp_launches[CALS_MAX_MODES];
  int64_t mttkrp_rows_launches;      /* of those, how many the planner gave to the rows kernel (short modes, few column
                                        groups) rather than the tile kernel                                         */
} cals_stats;

typedef struct {
  int64_t round;       /* 0-based index of the main-loop round (Alg. 3)                                        */
  int32_t n_active;    /* models advanced in this round                                                        */
  int32_t total_rank;  /* fused width of this round's MTTKRPs                                                  */
  double ms;           /* device time of the round's kernels (needs CALS_CTX_TIMING, else 0)                   */
  double mttkrp_flops; /* algorithmic flops of the round's fused MTTKRPs (2 * width * prod(I) each)            */
} cals_round_record;

/* Create / destroy a context.  `opt` is copied.  Errors: INVALID (null, R* < 1, slots < 0), HIP. */
int cals_create(cals_ctx** out, const cals_options* opt);
int cals_destroy(cals_ctx* c);

/* Hand over the tensor (Alg. 3 input T).  dims = {I1,I2,I3}, each >= 1, product < 2^40.
 * on_device = 1: `data` is a device pointer, BORROWED until cals_destroy (the caller keeps it
 * alive and unchanged); on_device = 0: `data` is a host pointer and is copied.  Computes ||T||^2
 * (needed once by the error formula of Alg. 1) and rejects a tensor with a NaN/Inf entry.
 * One tensor per context: a second call returns CALS_E_STATE, also when the first one failed after its
 * argument checks (destroy the context and start again). */
int cals_submit_tensor(cals_ctx* c, const double* data, const int64_t dims[3], int on_device);

/* The same for a tensor of order ndims (Alg. 1 and Alg. 3 are stated for N modes): 3 <= ndims <= CALS_MAX_MODES,
 * dims[0..ndims), first index fastest.  For output mode n the N-1 contracted modes form a fast and a slow run of
 * consecutive modes; a run of more than one mode enters the fused contraction as the explicit Khatri-Rao product of
 * its factor multi-matrices (device buffers of prod(run dims) x ld doubles, allocated here), so every product of
 * the dims of such a run must stay below 2^31.
 * Errors as cals_submit_tensor; INVALID also for ndims out of range. */
int cals_submit_tensor_nd(cals_ctx* c, const double* data, int32_t ndims, const int64_t* dims, int on_device);

/* Append a starting point to the input queue (Alg. 3, Q_in).  init[n] is a HOST pointer to the
 * column-major I_n x rank starting factor of mode n+1; it is copied.  tol < 0 means "never stop
 * by tolerance" (fixed iteration count).  ls_alpha is read only with CALS_MODEL_LINESEARCH.
 * Errors: STATE (no tensor), INVALID (rank < 1, > CALS_MAX_RANK or > R*; max_iters < 1; NaN
 * tol/alpha; NaN/Inf in init).  NONNEG and LINESEARCH may be combined: the extrapolated point is then clipped
 * at zero before its error is evaluated. */
int cals_enqueue_model(cals_ctx* c, int32_t rank, const double* const* init, double tol, int32_t max_iters,
                       uint32_t flags, double ls_alpha, int64_t* model_id);

/* Run up to n_rounds rounds of the main loop of Alg. 3 (fill from the queue front until the next
 * model does not fit; one fused ALS iteration of all active models; retire in slot order and
 * compact).  Stops early when the queue is empty and nothing is active.  *n_retired (may be
 * null) receives the number of models that left during this call.  Synchronises the stream. */
int cals_iterate(cals_ctx* c, int32_t n_rounds, int32_t* n_retired);

/* cals_iterate until the input queue is empty and no model is active. */
int cals_run(cals_ctx* c);

/* Pop finished models from the output queue (Alg. 3, Q_out) in retirement order: up to `cap`
 * results are written to `out` (host), *n receives how many. */
int cals_poll_retired(cals_ctx* c, cals_result* out, int32_t cap, int32_t* n);

/* Factors of a FINISHED model: U[n] (host, column-major I_n x rank, may be null to skip) and
 * lambda (host, rank doubles, may be null).  The model tensor is sum_r lambda[r] u1_r o u2_r o ... o uN_r.
 * Errors: NOTFOUND (unknown id or model not finished yet). */
int cals_get_factors(cals_ctx* c, int64_t model_id, double* const* U, double* lambda);

/* The fused MTTKRP alone (Eq. (2); Alg. 2, fused-MTTKRP line), for parity and roofline runs:
 *   M[i_mode, c] = sum over the other indices of T[i1,...,iN] * prod_{n != mode} U_n[i_n,c],  c < total_rank.
 * mode is 1 .. N.  U_dev[n] (device, row-major I_n x ld) for the modes != mode (the pointer of `mode` itself
 * is ignored and may be null); M_dev (device, row-major I_mode x ld) is overwritten in
 * columns [0, total_rank); ld >= total_rank (for N > 3 also ld <= max_total_rank rounded up to 16, the width of
 * the context's Khatri-Rao buffers).  Uses the context's tensor, stream and workspace. */
int cals_mttkrp(cals_ctx* c, int32_t mode, int32_t total_rank, int64_t ld, const double* const* U_dev,
                double* M_dev);

/* cals_mttkrp for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same launch plan and therefore bit-identical results; the
 * split-K partial panels go to a fixed device array of CALS_NOALLOC_SCRATCH_BYTES that every GPU the library runs
 * on holds from the first cals_create on it until the process ends (instead of the context's workspace, which
 * cals_mttkrp grows on demand).  The call allocates and frees nothing on host-visible HIP paths: no device memory,
 * no events (such a launch is never timed, whatever CALS_CTX_TIMING says).  A launch whose partials
 * (split count x I_mode x ld doubles, the split count chosen by the planner) exceed the array returns
 * CALS_E_TOOLARGE and enqueues nothing.  All calls on one GPU share that GPU's array: it keeps the previous call's
 * contents (every element a launch reads it has written first, so nothing needs clearing), and calls that overlap on
 * one GPU -- other streams, other contexts, other threads -- race; serialise them.
 * Other errors as cals_mttkrp. */
#define CALS_NOALLOC_SCRATCH_BYTES (256u << 20)
int cals_mttkrp_noalloc(cals_ctx* c, int32_t mode, int32_t total_rank, int64_t ld, const double* const* U_dev,
                        double* M_dev);

/* The two MTTKRPs of a two-step sweep alone, for parity runs (needs CALS_CTX_REUSE): Y from U_dev[0], then
 *   M2[i2,c] = sum_i3 Y[(i2,i3),c] * U3[i3,c]   and   M3[i3,c] = sum_i2 Y[(i2,i3),c] * U2[i2,c],   c < total_rank,
 * which equal the mode-2 and mode-3 MTTKRPs of (U1, U2, U3).  All three U_dev[n] are device, row-major I_n x ld,
 * ld <= the context's leading dimension (max_total_rank rounded up to 16); M2_dev (I2 x ld) and M3_dev (I3 x ld)
 * are overwritten in columns [0, total_rank).  Order-3 tensors only.  Errors: STATE (context without CALS_CTX_REUSE,
 * no tensor, or a tensor of higher order),
 * INVALID (arguments). */
int cals_mttkrp_reuse(cals_ctx* c, int32_t total_rank, int64_t ld, const double* const U_dev[3], double* M2_dev,
                      double* M3_dev);

/* The same for any order (needs CALS_CTX_REUSE): Y from U_dev[0], then for every mode n >= 2 the MTTKRP
 *   M_n[i_n,c] = sum over (i2..iN without i_n) of Y[(i2,..,iN),c] * prod_{m >= 2, m != n} U_m[i_m,c],   c < total_rank,
 * into M_dev[n-1] (device, row-major I_n x ld; M_dev[0] is ignored and may be null).  U_dev[n] for all N modes.
 * Errors: STATE (context without CALS_CTX_REUSE or no tensor), INVALID (arguments). */
int cals_mttkrp_reuse_nd(cals_ctx* c, int32_t total_rank, int64_t ld, const double* const* U_dev, double* const* M_dev);

/* One record per round of the main loop, in order: the segments of the paper's efficiency measurement (Sec. 6,
 * "Efficiency": time and flop count per CALS iteration).  Copies the records of rounds first_round, first_round+1, ...
 * (up to `cap`) to `out` (host); *n receives how many.  At most the first 2^20 rounds of a context are recorded.
 * Synchronises the stream when timing is on.  Errors: INVALID (arguments). */
int cals_get_round_log(cals_ctx* c, int64_t first_round, cals_round_record* out, int32_t cap, int32_t* n);

/* Counters and timings (see cals_stats).  Synchronises the stream when timing is on. */
int cals_get_stats(cals_ctx* c, cals_stats* s);

/* Practical peaks of the device the context runs on -- the yardsticks the MTTKRP rates are read against (the paper
 * does the same with a plain GEMM, Sec. 6, "experimental setup").  kind CALS_YARDSTICK_MFMA: every SIMD issues
 * back-to-back fp64 16x16x4 matrix instructions on register operands; *value = TFLOP/s.  kind CALS_YARDSTICK_READ:
 * a streaming read-and-sum of `bytes` bytes (rounded down to 16; at least 1 MiB) of the caller's device buffer `buf`
 * (pass the tensor); *value = GB/s.  Both run `reps` (1..100) timed launches after one warm-up on the context's stream
 * and return the average.  Synchronises the stream.  Errors: INVALID (arguments), HIP.
 * kinds CALS_YARDSTICK_CLOCK_MHZ and CALS_YARDSTICK_COMPUTE_UNITS return the device attributes the spec-sheet peaks
 * are derived from (buf, bytes, reps ignored). */
#define CALS_YARDSTICK_MFMA 0
#define CALS_YARDSTICK_READ 1
#define CALS_YARDSTICK_CLOCK_MHZ 2
#define CALS_YARDSTICK_COMPUTE_UNITS 3
int cals_yardstick(cals_ctx* c, int32_t kind, const void* buf, int64_t bytes, int32_t reps, double* value);

/* Static description of an error code. */
const char* cals_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CALS_H */
