/*
 * fsk.h -- C ABI of the MI355X (gfx950) Sinkhorn hot-path library.
 *
 * The library runs the Gibbs-kernel scaling iteration of entropic optimal
 * transport (paper: Sec. 1, Eq. 1 and the scaling form below it; Algorithm 1):
 *
 *     K = exp(-C/eps),   u <- a ./ (K v),   v <- b ./ (K^T u),
 *
 * one "iteration" being the u-update followed by the v-update, in its dense,
 * row-partitioned (Sec. 3.1, Proposition 1), log-domain (named in Sec. 1 and
 * Sec. 2.1; formulas are the logarithm of the iteration above) and multitarget
 * (Sec. 5.3.2) forms.
 *
 * Conventions common to every call
 *   - Every pointer documented "device" is GPU memory owned by the caller
 *     (e.g. a torch tensor); it must stay valid until the work enqueued on the
 *     stream has finished.  The library never allocates or frees device
 *     memory: scratch space comes in through the `workspace` argument, whose
 *     minimum size fsk_workspace_bytes() reports.  Pointers documented "host"
 *     are ordinary process memory.
 *   - Matrices are row-major with a leading dimension `ld` counted in
 *     elements.  K must be 16-byte aligned and ld*sizeof(element) must be a
 *     multiple of 16 (rows are read with 128-bit loads); entries in the padding
 *     columns [n, ld) are never used.  Full-length scaling vectors (u, v, v_full)
 *     must be 16-byte aligned as well; every other vector needs only its natural
 *     alignment.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     kernels are enqueued on it.  Calls that run a fixed number of iterations
 *     return as soon as the work is enqueued; calls in tolerance mode
 *     (opts->tol > 0) synchronise the stream at every poll and before they
 *     return.  A fixed-iteration call only enqueues kernels (the bounded-delay
 *     emulation also device-to-device copies): no allocation, no synchronisation,
 *     no memset, so a caller may record it into a HIP graph and replay it.
 *   - Return value: FSK_OK or a negative fsk_status.  fsk_last_error() gives a
 *     thread-local message for the last failure.  Arguments are validated on the
 *     host before anything is launched; a failed call launches nothing.
 *   - Not checked (assumptions A1-A2 of the paper's convergence section):
 *     K > 0, a, b > 0 with equal total mass.
 *   - Results are deterministic: no floating-point atomics; every reduction has a fixed order.
 *     For the dense flows FUSED, TWO_PASS and PAPER that order depends on (n, dtype, flow) only --
 *     not on the device, and not on the block count c (FUSED: as long as n/c is a multiple of the
 *     strip height, see fsk_flow) -- so c blocks reproduce the iterates of c = 1 bit for bit
 *     (Proposition 1).  FSK_FLOW_RESIDENT, the grid flow and the multitarget kernels group their
 *     sums by their own launch shapes (compute-unit count, workspace given): equal to rounding.
 */
#ifndef FSK_H
#define FSK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FSK_OK = 0,
  FSK_EINVAL = -1,       /* bad size, eps, c, ld, null pointer, unknown enum value            */
  FSK_EALIGN = -2,       /* K or ld not 16-byte aligned                                       */
  FSK_EDIV = -3,         /* c does not divide n (the paper takes n = c*m, Sec. 3.1)           */
  FSK_EWORKSPACE = -4,   /* workspace missing or smaller than fsk_workspace_bytes()           */
  FSK_ENONFINITE = -5,   /* a non-finite marginal error was read at a poll                    */
  FSK_EHIP = -6,         /* a HIP runtime call failed (message has the HIP error string)      */
  FSK_EUNSUPPORTED = -7  /* valid request outside what this build implements                  */
} fsk_status;

typedef enum { FSK_F32 = 0, FSK_F64 = 1 } fsk_dtype;

/* How one dense iteration moves through K.  All produce the iterates of
 * Algorithm 1; they differ in memory traffic and in summation order. */
typedef enum {
  FSK_FLOW_FUSED = 0,    /* one pass over K per iteration: a workgroup keeps rows in registers,
                            finishes u on them, and accumulates their contribution K_I^T u_I; a
                            second small kernel sums the contributions in fixed order and
                            divides.  Every row block I_j is cut into strips of h rows, one row
                            of partial column sums per strip (per workgroup of a strip); block
                            j's contribution s^(j) = K_{I_j,:}^T u_{I_j} -- what a worker holding
                            only its rows can form -- is the sum of its strips'.  h is
                            ceil(n / S) rounded up to the kernel's row group (S = 256 strips
                            for n >= 8192, 16 below), i.e. a function of n and dtype alone
                            whenever c divides S; if n/c is also a multiple of h the strips are
                            the same for every such c and the iterates equal those of c = 1
                            bit for bit, otherwise to rounding.                             */
  FSK_FLOW_TWO_PASS = 1, /* q = K v over all rows, then r = K^T u over all rows (two passes);
                            with c > 1 the c row slabs are one grid                          */
  FSK_FLOW_PAPER = 2,    /* Algorithm 1 as printed: block j forms u_{I_j} from its row slab,
                            then r_{I_j} = (K_{:,I_j})^T u from its column slab.  On one device
                            the c column slabs tile the column range and every column is summed
                            on its own over the same 128-row strips, so the slabs are served by
                            one launch over all columns: the enqueued kernels, and the bits,
                            are those of TWO_PASS.  What a client of this flow can see and
                            TWO_PASS's cannot -- vectors that differ from client to client --
                            is what fsk_sinkhorn_local_steps and
                            fsk_sinkhorn_async_emulated run on these slabs.                   */
  FSK_FLOW_RESIDENT = 3  /* small K only (n <= 1024 in fp32, n <= 512 in fp64): a
                            persistent grid of 8-32 workgroups holds K in registers and runs
                            all the iterations between two polls in ONE launch, exchanging the
                            workgroups' partial column sums across a grid-wide barrier.
                            opts->c is accepted and has no effect on the arithmetic (the row
                            blocks are the workgroups').  FSK_EUNSUPPORTED for a larger K.
                            If the barrier sees no progress for about a second the call
                            writes NaN into u and v instead of hanging.                      */
} fsk_flow;

typedef enum {
  FSK_DAMP_NONE = 0,
  FSK_DAMP_ARITHMETIC = 1, /* u <- (1-eta) u + eta a./(K v)            (Sec. 3.3)             */
  FSK_DAMP_GEOMETRIC = 2   /* u <- u^(1-eta) .* (a./(K v))^eta         (Remark in Sec. 3.3);
                              FSK_FLOW_FUSED carries it in fp32 and FSK_FLOW_RESIDENT in both
                              precisions as exp2 of the weighted log2's; an fp64 FUSED call
                              runs the two-pass kernels instead                                */
} fsk_damping;

typedef enum {
  FSK_NORM_L1 = 0,  /* ||P1 - a||_1, the default                                                  */
  FSK_NORM_L2 = 1   /* ||P1 - a||_2, the paper's own metric (Sec. 5.4, err_a; privacy appendix,
                       "Marginal error metric")                                                   */
} fsk_norm;

typedef struct {
  int32_t n;           /* problem size: K is n x n, a, b, u, v have n entries                  */
  int32_t m;           /* histograms per batch (multitarget form); 1 for the vector case       */
  int32_t c;           /* row blocks I_j = [j*n/c, (j+1)*n/c) emulating c workers; 1 =
                          centralised; must divide n                                           */
  int32_t max_iters;   /* IterMax of Algorithm 1                                               */
  double tol;          /* <= 0: run exactly max_iters iterations.  > 0: stop at the first poll
                          where ||P 1 - a|| < tol (norm: err_norm below), P = diag(u) K diag(v),
                          evaluated with the scalings as they stand after a v-update           */
  int32_t check_every; /* iterations between polls in tolerance mode (>= 1); the last
                          iteration is always polled                                           */
  int32_t dtype;       /* fsk_dtype of K, a, b, u, v (storage and arithmetic)                  */
  int32_t flow;        /* fsk_flow (dense calls only)                                          */
  int32_t damping;     /* fsk_damping (dense, log-domain and multitarget calls)                */
  double eta;          /* relaxation parameter in (0, 1]; ignored when damping = NONE          */
  int32_t err_norm;    /* fsk_norm of the marginal error that tolerance mode tests and reports
                          (dense, log-domain and multitarget calls; the multitarget call takes
                          the maximum over the targets of each target's norm)                  */
} fsk_opts;

typedef enum { FSK_MODE_DENSE = 0, FSK_MODE_LOG = 1, FSK_MODE_BATCHED = 2, FSK_MODE_SETUP = 3,
               FSK_MODE_PLAN = 4, FSK_MODE_RADIUS = 5 } fsk_mode;

/* Library version as major*10000 + minor*100 + patch. */
int fsk_version(void);

/* Message for the calling thread's last failed call ("" if none). Never NULL. */
const char* fsk_last_error(void);

/* Error trace (the paper logs the marginal error err_a against the iteration count, Sec. 5.4 and
 * the convergence plots): lends the calling thread a host buffer of 2*capacity doubles.  From
 * then on every tolerance-mode call of that thread (dense, log-domain, multitarget) restarts the
 * trace and appends, at each poll, the pair (iteration whose state was polled, that state's
 * error in opts->err_norm) -- no extra device work: these are the values the stop rule reads.
 * fsk_error_trace_count() = polls of the thread's last tolerance-mode call (it keeps counting
 * beyond the capacity, so a caller sees that the buffer was too small).  buf = NULL or
 * capacity <= 0 switches the trace off.  The buffer must stay valid while it is lent. */
void fsk_set_error_trace(double* buf, int32_t capacity);
int32_t fsk_error_trace_count(void);

/* Minimum workspace, in bytes, that a call of the given mode needs for these
 * options on the current device (0 on invalid options).  `d` is the point
 * dimension for FSK_MODE_LOG / FSK_MODE_SETUP and ignored otherwise. */
size_t fsk_workspace_bytes(const fsk_opts* opts, int mode, int d);

/* ---- setup: the Gibbs kernel K = exp(-C/eps) (Sec. 1) ----------------------------------
 * C, K: device, n x n, leading dimensions ldC, ldK.  K may alias C. */
int fsk_kernel_from_cost(const fsk_opts* opts, const void* C, int64_t ldC, double eps, void* K,
                         int64_t ldK, void* stream);

/* Same from two point clouds x, y (device, n x d row-major, dtype of opts) with the squared
 * Euclidean cost C_ij = ||x_i - y_j||^2 (Sec. 5.6).  normalise_by_max != 0 divides C by its
 * largest entry first (two passes over the pairs; needs the workspace).  If cmax_out (host)
 * is not NULL the call synchronises and stores max_ij C_ij there. */
int fsk_kernel_from_points(const fsk_opts* opts, const void* x, const void* y, int d, double eps,
                           int normalise_by_max, void* K, int64_t ldK, void* workspace,
                           size_t ws_bytes, double* cmax_out, void* stream);

/* ---- dense hot path (Algorithm 1; Sec. 4.1 for the per-iteration operations) ------------
 * K, a, b: device inputs.  u, v: device, IN/OUT -- the caller stores the starting scalings
 * (1 for a cold start, as in Algorithm 1, or a previous result to resume).  On return (after
 * the stream has drained) they hold the scalings after *iters_done iterations.
 * iters_done (host, may be NULL): iterations performed.  err (host, may be NULL): the last
 * polled ||P1 - a|| (in the norm opts->err_norm names) in tolerance mode, NaN in fixed-iteration
 * mode. */
int fsk_sinkhorn_dense(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                       const void* b, void* u, void* v, void* workspace, size_t ws_bytes,
                       int32_t* iters_done, double* err, void* stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: fsk_sinkhorn_dense without the workspace argument.
 * Same arguments, results and errors as fsk_sinkhorn_dense (it runs the same kernels); the scratch
 * that call takes from its workspace lives in a device array that is part of the library image,
 * FSK_STATIC_SCRATCH_BYTES per GPU, held by every GPU the library runs on until the process ends.
 * The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine).
 * Limit: fsk_workspace_bytes(opts, FSK_MODE_DENSE, 0) <= FSK_STATIC_SCRATCH_BYTES, which covers
 * every flow up to n = 32768 in fp32 and n = 16384 in fp64 on a 256-compute-unit device;
 * FSK_EWORKSPACE beyond it, with nothing launched.  The first call on a device looks the array's
 * address up (make that call outside a graph capture).  All calls on one GPU share that GPU's
 * array, which keeps the previous call's contents (the kernels overwrite what they read, and
 * clear the counters that must start at zero, themselves): two calls whose work overlaps in time
 * on one GPU -- different streams, or different host threads -- race on it and must be serialised
 * by the caller. */
#define FSK_STATIC_SCRATCH_BYTES (34u * 1024u * 1024u)
int fsk_sinkhorn_dense_static(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                              const void* b, void* u, void* v, int32_t* iters_done, double* err,
                              void* stream);

/* Poll budget of the grid barrier in FSK_FLOW_RESIDENT (process-wide; default 4000000, about a
 * second).  A waiter that exhausts it marks the launch failed: u and v come back NaN (and a
 * tolerance-mode call returns FSK_ENONFINITE) instead of the kernel waiting for ever.  For
 * callers that want a tighter bound, and for testing the failure path (0 = give up at the first
 * unsuccessful poll). */
void fsk_set_barrier_poll_limit(uint32_t polls);

/* Row and column marginals of P = diag(u) K diag(v) (device outputs of n entries each; either
 * may be NULL), and optionally the marginal error on a in two norms (host outputs, either may
 * be NULL; a non-NULL one makes the call synchronise): err_l1 = ||P1 - a||_1 and
 * err_l2 = ||P1 - a||_2, the one the paper's convergence plots and its privacy appendix report
 * (Sec. 5.4, "Marginal error metric").  Both come from one row pass; the sums are taken in fp64.
 * opts->err_norm plays no part here; err_l2 <= err_l1, so a run stopped at err_l1 < tol also
 * meets the 2-norm criterion at the same threshold. */
int fsk_marginals(const fsk_opts* opts, const void* K, int64_t ldK, const void* a, const void* u,
                  const void* v, void* row_marginal, void* col_marginal, void* workspace,
                  size_t ws_bytes, double* err_l1, double* err_l2, void* stream);

/* ---- objective of Eq. 1 at P = diag(u) K diag(v), without materialising P -----------------
 * One pass over K and the cost matrix C (device, n x n, same dtype, leading dimension ldC).
 * out (host, 5 doubles; the call synchronises):
 *   out[0] = <P, C>                  out[1] = sum_ij P_ij (log P_ij - 1)      (0 log 0 = 0)
 *   out[2] = out[0] + eps * out[1]   (the objective of Eq. 1)
 *   out[3] = sum_ij P_ij             out[4] = sum_ij P_ij l_j, l a device n-vector or NULL (0)
 * out[4] with l_j = l(x'_j) is the worst-case expected loss of the paper's finance example.
 * Workspace: fsk_workspace_bytes(opts, FSK_MODE_PLAN, 0). */
int fsk_plan_objective(const fsk_opts* opts, const void* K, int64_t ldK, const void* C, int64_t ldC,
                       double eps, const void* u, const void* v, const void* l, double* out,
                       void* workspace, size_t ws_bytes, void* stream);

/* ---- radius search of the robust-risk example (Sec. "Illustrative application"; appendix
 * "Enforcing the Wasserstein radius", steps 1-3) ------------------------------------------
 * The combined cost is C_lambda,ij = lambda c_ij - l_j with c the ground cost (device, n x n,
 * leading dimension ldc) and l_j the loss at target point j (device n-vector, or NULL for 0).
 *
 * fsk_kernel_from_cost_lambda: K_ij = exp(-(lambda c_ij - l_j)/eps), fp64 arithmetic with one
 * rounding to the storage type.  K must not alias c if c is needed again.  Enqueue only. */
int fsk_kernel_from_cost_lambda(const fsk_opts* opts, const void* c, int64_t ldc, double lambda,
                                const void* l, double eps, void* K, int64_t ldK, void* stream);

/* fsk_radius_search: bisection on [lambda_lo, lambda_hi] for <P(lambda), c> = delta.  Each
 * step: lambda = (lo + hi)/2; K as above; u = v = 1; the dense solve that fsk_sinkhorn_dense
 * would run with these opts (flow, c, max_iters, tol, check_every, err_norm, damping); g = <P, c> - delta
 * from the plan-sum kernel; stop if |g| <= gtol, else lo = lambda if g > 0 (transport too
 * large: raise its price) and hi = lambda otherwise.  At most max_steps (>= 1) solves; the
 * call synchronises once per step.
 * K (device, n x n, not aliasing c), u, v (device): OUT, as of the last solve.
 * out (host, 4 doubles): lambda, <P, c>, sum_ij P_ij l_j (the worst-case expected loss), solves.
 * Workspace: fsk_workspace_bytes(opts, FSK_MODE_RADIUS, 0).
 * Errors: FSK_EINVAL (sizes, eps, bracket, aliasing), FSK_EALIGN, FSK_EWORKSPACE,
 * FSK_ENONFINITE (a solve produced a non-finite cost: K under- or overflowed for this lambda). */
int fsk_radius_search(const fsk_opts* opts, const void* c, int64_t ldc, const void* l, const void* a,
                      const void* b, double eps, double delta, double lambda_lo, double lambda_hi,
                      int32_t max_steps, double gtol, void* K, int64_t ldK, void* u, void* v,
                      void* workspace, size_t ws_bytes, double* out, void* stream);

/* ---- bounded-delay emulation of the asynchronous schedule (Algorithm 3; assumption A3 of the
 * convergence section) on one device, with a deterministic delay.  Client j owns rows/columns
 * I_j (opts->c clients).  In iteration t it uses cached global vectors whose own slice is
 * current and whose remote slices are what the peers held at the end of iteration
 *     s(t) = floor((t-1-tau)/sync_every)*sync_every      (the initial vectors if <= 0):
 *   u_{I_j} <- (1-eta) u_{I_j} + eta a_j ./ (K_{I_j,:} v_cached),
 *   v_{I_j} <- (1-eta) v_{I_j} + eta b_j ./ ((K_{:,I_j})^T u_cached)   (u_cached has the new u_{I_j}).
 * eta = opts->eta if opts->damping == FSK_DAMP_ARITHMETIC, 1 for FSK_DAMP_NONE
 * (FSK_EUNSUPPORTED for the geometric relaxation: Algorithm 3 uses the arithmetic one).  Runs exactly
 * opts->max_iters iterations (FSK_EUNSUPPORTED for opts->tol > 0); u, v are IN/OUT as in
 * fsk_sinkhorn_dense.  tau >= 0, sync_every >= 1.  Workspace: fsk_async_workspace_bytes(). */
size_t fsk_async_workspace_bytes(const fsk_opts* opts, int32_t tau, int32_t sync_every);
int fsk_sinkhorn_async_emulated(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                                const void* b, void* u, void* v, int32_t tau, int32_t sync_every,
                                void* workspace, size_t ws_bytes, void* stream);

/* ---- synchronous iteration with w local steps between collectives (Sec. 3.1, Remark "Local
 * steps before communication"; appendix "Additional details on local steps"; the "optional"
 * collectives of Sec. 3.2.1) on one device.  Client j (opts->c clients) owns rows/columns I_j and
 * keeps its own view of u and v: its own slices as it last updated them, the peers' slices as of
 * the last collective.  Iteration k = 1, 2, ...: every client forms u_{I_j} = a_j ./ (K_{I_j,:} v_view);
 * if k is a multiple of w the slices of u are gathered; every client forms
 * v_{I_j} = b_j ./ ((K_{:,I_j})^T u_view); if k is a multiple of w the slices of v are gathered.
 * w = 1 is Algorithm 1 and gives the bits of FSK_FLOW_PAPER; c = 1 gives them for any w.
 * Runs exactly opts->max_iters iterations, undamped (FSK_EUNSUPPORTED for a tolerance or a
 * damping in opts); opts->flow is not used.  u, v are IN/OUT as in fsk_sinkhorn_dense and hold
 * every client's own slice on return; a resumed call starts with all views equal, so runs are
 * resumable at multiples of w.  Enqueue only (kernels and device-to-device copies).
 * Workspace: fsk_local_steps_workspace_bytes(). */
size_t fsk_local_steps_workspace_bytes(const fsk_opts* opts);
int fsk_sinkhorn_local_steps(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                             const void* b, void* u, void* v, int32_t w, void* workspace,
                             size_t ws_bytes, void* stream);

/* ---- 2D block distribution on one device (appendix "HPC baseline: 2D block distribution
 * with row/column Allreduce") --------------------------------------------------------------
 * K is cut into a p_r x p_c grid of blocks K_ij (block rows of n/p_r rows, block columns of
 * n/p_c columns).  An iteration forms the block products K_ij v_j, adds them along each block
 * row in the order j = 0, 1, ... (the row-wise reduction), u = a ./ q; then the block products
 * K_ij^T u_i, added along each block column in the order i = 0, 1, ... (the column-wise
 * reduction), v = b ./ r.  Same iterates as Algorithm 1 up to the grouping of the sums.
 * Runs exactly opts->max_iters iterations, undamped; u, v IN/OUT as in fsk_sinkhorn_dense;
 * opts->c and opts->flow are not used.  Enqueue only.
 * Errors: FSK_EDIV if p_r or p_c does not divide n; FSK_EALIGN if a block column does not start
 * on a 16-byte boundary (n/p_c must be a multiple of 4 entries in fp32, 2 in fp64);
 * FSK_EUNSUPPORTED for tolerance mode or damping.  Workspace: fsk_grid_workspace_bytes(). */
size_t fsk_grid_workspace_bytes(const fsk_opts* opts, int32_t p_r, int32_t p_c);
int fsk_sinkhorn_grid(const fsk_opts* opts, const void* K, int64_t ldK, const void* a, const void* b,
                      void* u, void* v, int32_t p_r, int32_t p_c, void* workspace, size_t ws_bytes,
                      void* stream);

/* ---- one worker's share (Sec. 3.1: client j holds rows I_j of K and slices a_j, b_j) -----
 * K_slab: device, `rows` x n, the rows [row0, row0+rows) of K (row0 is only used to index the
 * full-length vectors).  These are the per-worker operations of Algorithm 1 and Sec. 4.1 at
 * their real shape; a multi-GPU driver would put one exchange between them. */

/* u_slab = a_slab ./ (K_slab v_full): a_slab, u_slab have `rows` entries, v_full has n. */
int fsk_block_rowpass(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                      int32_t rows, const void* a_slab, const void* v_full, void* u_slab,
                      void* stream);

/* s = K_slab^T u_slab (n entries): the slab's contribution to K^T u. */
int fsk_block_colpartial(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                         int32_t rows, const void* u_slab, void* s_partial, void* workspace,
                         size_t ws_bytes, void* stream);

/* Both at once, reading the slab one time: u_slab = a_slab ./ (K_slab v_full) and
 * s = K_slab^T u_slab.  This is the kernel FSK_FLOW_FUSED runs, exposed on one slab. */
int fsk_block_fused(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                    int32_t rows, const void* a_slab, const void* v_full, void* u_slab,
                    void* s_partial, void* workspace, size_t ws_bytes, void* stream);

/* ---- log-domain hot path (stabilised form named in Sec. 1; implicit kernel, Sec. 4.1 Remark)
 * x, y: device, n x d point clouds; the cost ||x_i - y_j||^2 is evaluated on the fly and K is
 * never stored.  f, g: device, IN/OUT potentials (f = eps log u, g = eps log v; 0 for a cold
 * start).  Each iteration does
 *     f_i <- eps log a_i - eps LSE_j((g_j - C_ij)/eps),  g_j <- eps log b_j - eps LSE_i((f_i - C_ij)/eps).
 * With opts->damping the relaxed updates of Sec. 3.3 apply to both potentials: geometric is
 * f <- (1-eta) f + eta f_new, arithmetic is f <- eps log((1-eta) e^(f/eps) + eta e^(f_new/eps)).
 * FSK_F32: the cost term runs in fp64, exponentials and their sums in fp32.  FSK_F64: everything in
 * fp64.  1 <= d <= 4096 (FSK_EUNSUPPORTED outside); d <= 32 runs the kernel that keeps a row's
 * coordinates in registers, larger d a generic, slower one.  iters_done / err as in
 * fsk_sinkhorn_dense.  Within one call the potentials are carried in fp64 and f, g receive their
 * rounding to the interface type; a later call starts from those rounded values, so with FSK_F32
 * a run split into several calls agrees with the same run in one call to fp32 rounding of f, g
 * (about 1e-7 |f|, i.e. up to ~1e-5 in |f|/eps at eps = 0.01), not bit for bit. */
int fsk_sinkhorn_log_points(const fsk_opts* opts, const void* x, const void* y, int d, double eps,
                            const void* a, const void* b, void* f, void* g, void* workspace,
                            size_t ws_bytes, int32_t* iters_done, double* err, void* stream);

/* ---- multitarget hot path (Sec. 5.3.2) -------------------------------------------------
 * A, B (inputs), U, V (IN/OUT): device, n x m row-major with leading dimension m, one histogram
 * pair per column, K shared.  Q = K V and R = K^T U are matrix products (MFMA).  Runs exactly
 * opts->max_iters iterations (FSK_EUNSUPPORTED for opts->tol > 0: see the _tol call below).
 * FSK_F32 (fp32 MFMA) or FSK_F64 (fp64 MFMA; needs the whole workspace, FSK_EWORKSPACE
 * otherwise).  Any m >= 1: the columns go through the kernels in groups of up to 64, one pass
 * over K per group and product, so the time grows with ceil(m / 64).  ldK <= 2^22 elements and
 * m <= 2^20 (FSK_EUNSUPPORTED beyond: the kernels form 32-bit offsets).  Which kernel forms K V
 * (hence the order of its sums) depends on (n, m) and on whether the workspace has room for the
 * transposed copy, never on the iteration count: a run split into several calls with the same
 * workspace gives the bits of the run in one call.
 * Workspace: fsk_workspace_bytes(opts, FSK_MODE_BATCHED, 0) holds the partial products of all
 * groups and a transposed copy of K; with at least the partial products (the size the error
 * message of a too-small workspace states) an undamped call still runs, with a slower kernel
 * for K V.
 * opts->damping / opts->eta apply the relaxed updates of Sec. 3.3 to every target: each
 * half-step is written to a scratch n x m matrix and an elementwise kernel folds it into U or V
 * (arithmetic: (1 - eta) X + eta X_new; geometric: exp2((1 - eta) log2 X + eta log2 X_new) in
 * the call's precision).  A damped call needs the whole workspace of its opts (it holds that
 * scratch matrix too): FSK_EWORKSPACE otherwise. */
int fsk_sinkhorn_batched(const fsk_opts* opts, const void* K, int64_t ldK, const void* A,
                         const void* B, void* U, void* V, void* workspace, size_t ws_bytes,
                         void* stream);

/* The same with the stop rule of fsk_sinkhorn_dense applied to all targets at once (the
 * multitarget experiment of Sec. 5.3.2 iterates until every target meets the threshold):
 * opts->tol > 0 stops at the first poll (every opts->check_every iterations, and after
 * opts->max_iters) at which max over columns k of ||P_k 1 - a_k|| < tol (each target in the norm
 * opts->err_norm names), P_k = diag(u_k) K
 * diag(v_k), with the scalings as they stand after a V-update (damped or not: in a damped run
 * the error is read off the undamped U-update of that state before it is relaxed);
 * opts->tol <= 0 runs max_iters iterations and leaves *err NaN.  iters_done (host, required) and err (host, may be NULL)
 * receive the iteration count and that maximum; U, V hold the state they describe.  The call
 * synchronises at every poll.  Workspace: fsk_workspace_bytes(opts, FSK_MODE_BATCHED, 0) with
 * the same opts (in tolerance mode, as in a damped run, it also holds an n x m scratch matrix).  FSK_ENONFINITE as in the dense
 * call. */
int fsk_sinkhorn_batched_tol(const fsk_opts* opts, const void* K, int64_t ldK, const void* A,
                             const void* B, void* U, void* V, void* workspace, size_t ws_bytes,
                             int32_t* iters_done, double* err, void* stream);

/* ---- privacy layer (privacy appendix: "Gaussian noise on log-domain scalings", "RDP
 * accountant") ---------------------------------------------------------------------------
 * A release replaces an n x m scaling matrix X (device, row-major, leading dimension m, in
 * place) by exp(clip_S(log X) + sigma Z): clip_S scales every row of log X (the m targets of
 * one index) to l2 norm at most S; S <= 0 or +inf disables the clip (the Gaussian-only
 * ablation).  Z_ik is standard normal number i*m + k of the stream (seed, release): Philox4x32-10
 * with key = seed and counter = (call e/4, release) yields words x0..x3; with
 * u1 = (xa + 1/2) 2^-32, u2 = (xb + 1/2) 2^-32 the pair (x0, x1) gives numbers 0 and 1 of the
 * call as sqrt(-2 ln u1) cos(2 pi u2) and sqrt(-2 ln u1) sin(2 pi u2), the pair (x2, x3) numbers
 * 2 and 3.  The stream is a pure function of (seed, release, element): no state is kept. */
typedef struct {
  double clip_u, clip_v;   /* S_u, S_v */
  double sigma_u, sigma_v; /* noise scales, >= 0 */
  uint64_t seed;
  uint64_t release0;       /* index of the first release of the call (even); iteration t of the
                              call releases U as release0 + 2t and V as release0 + 2t + 1, so a
                              resumed run passes release0 + 2 * (iterations already done) */
} fsk_dp;

/* One release of X (n = opts->n rows, m = opts->m columns, dtype of opts).  Enqueue only. */
int fsk_dp_release(const fsk_opts* opts, void* X, double clip, double sigma, uint64_t seed,
                   uint64_t release, void* stream);

/* fsk_sinkhorn_batched with a release after every update (the noised scalings replace the held
 * ones, as in the appendix' experiments): U = A ./ (K V), release U, V = B ./ (K^T U), release V.
 * Undamped, fixed iteration count: FSK_EUNSUPPORTED for a damping or a tolerance in opts. */
int fsk_sinkhorn_batched_dp(const fsk_opts* opts, const void* K, int64_t ldK, const void* A,
                            const void* B, void* U, void* V, const fsk_dp* dp, void* workspace,
                            size_t ws_bytes, void* stream);

/* Host-only accountant: `releases` Gaussian releases with l2 sensitivity 2*clip and noise sigma
 * compose to eps_RDP(p) = releases * p (2 clip)^2 / (2 sigma^2); *eps_out = min over the given
 * orders p > 1 of eps_RDP(p) + log(1/delta)/(p - 1), *order_out (may be NULL) the minimiser.
 * The paper does not list its grid of orders: the caller supplies one. */
int fsk_rdp_epsilon(double clip, double sigma, int64_t releases, double delta, const double* orders,
                    int32_t n_orders, double* eps_out, double* order_out);

/* ---- measurement helpers -----------------------------------------------------------------
 * fsk_dense_profile times the launches of fsk_sinkhorn_dense's fixed-iteration mode (same
 * kernels, same launch shapes) with HIP events recorded on `stream`, in two back-to-back runs:
 * first `reps` + 1 times the K-streaming launches of an iteration alone (the first one untimed;
 * they recompute the u-update from the same v, or relax u further if opts asks for a damping),
 * then `reps` whole iterations (u and v advance as in the solver).  Outputs (host):
 * stream_ms = average time of the K-streaming (HBM-bound) launches of one iteration,
 * other_ms = whole iteration minus that: the small reduction kernels and the hand-overs between
 * launches, stream_launches = number of K-streaming launches per iteration.  Synchronises.
 * FSK_FLOW_RESIDENT: one launch runs all `reps` iterations; stream_ms is its time / reps.  */
int fsk_dense_profile(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                      const void* b, void* u, void* v, void* workspace, size_t ws_bytes, int reps,
                      double* stream_ms, double* other_ms, int32_t* stream_launches, void* stream);

/* A plain device copy dst <- src of `bytes` bytes (multiple of 16, both 16-byte aligned) with
 * the same 128-bit access pattern as the hot kernels; used to calibrate profiler byte counters
 * and to measure the achievable HBM rate next to the hot path. */
int fsk_bench_copy(void* dst, const void* src, size_t bytes, void* stream);
/* A plain streaming read of `bytes` bytes reduced to one float per workgroup in `sink`
 * (device, at least 4096 floats): the read-only counterpart of fsk_bench_copy. */
int fsk_bench_read(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FSK_H */
