// Host-side declarations shared by the translation units of libfsk.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/fsk.h"

namespace fsk {

// Records a thread-local message and returns `code`.
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

#define FSK_HIP(call)                                                                     \
  do {                                                                                    \
    hipError_t fsk_e_ = (call);                                                           \
    if (fsk_e_ != hipSuccess)                                                             \
      return ::fsk::set_error(FSK_EHIP, "%s failed: %s", #call, hipGetErrorString(fsk_e_)); \
  } while (0)

#define FSK_LAUNCH_CHECK(name)                                                            \
  do {                                                                                    \
    hipError_t fsk_e_ = hipGetLastError();                                                \
    if (fsk_e_ != hipSuccess)                                                             \
      return ::fsk::set_error(FSK_EHIP, "launch of %s failed: %s", name,                  \
                              hipGetErrorString(fsk_e_));                                 \
  } while (0)

#define FSK_TRY(expr)                       \
  do {                                      \
    int fsk_rc_ = (expr);                   \
    if (fsk_rc_ != FSK_OK) return fsk_rc_;  \
  } while (0)

inline size_t elem_size(int dtype) { return dtype == FSK_F64 ? 8 : 4; }
inline int pack_width(int dtype) { return dtype == FSK_F64 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Compute units of the current device (cached per device), 0 on failure.
int device_cu_count();

// The calling thread's error trace (fsk_set_error_trace): a tolerance-mode call resets it when it
// starts and records every poll -- the iteration whose state was polled and that state's error.
void trace_begin();
void trace_poll(int iteration, double err);

// ------------------------------------------------------------------ dense kernels
constexpr int kColStrip = 128;  // rows summed sequentially into one partial column sum

// Row strip count of the generic column pass over `rows` rows.
inline int col_strips(int rows) { return (rows + kColStrip - 1) / kColStrip; }

// out[i] = epilogue(marg[i], sum_j K[i][j] vin[j], old[i]) for the `rows` rows of K.
// err_out (optional, needs marg and old): also |old[i] * product_i - marg[i]|.
int launch_rowpass(int dtype, const void* K, int64_t ld, int n, int rows, const void* vin,
                   const void* marg, const void* old, void* out, int epi, double eta,
                   hipStream_t stream, void* err_out = nullptr);

// The same for `slabs` row slabs of `rows` rows each in ONE grid (slab y = rows [y*rows,
// (y+1)*rows) of K, marg, old, out, err_out): the row passes of the c clients of Sec. 3.1.
// vown != NULL: client y multiplies by its own view of the vector -- vown[j] on its own index
// range [y*rows, (y+1)*rows), vin[j] elsewhere (needs slabs * rows == n).
int launch_rowpass_slabs(int dtype, const void* K, int64_t ld, int n, int rows, int slabs,
                         const void* vin, const void* vown, const void* marg, const void* old,
                         void* out, int epi, double eta, hipStream_t stream,
                         void* err_out = nullptr);

// The column pass of all clients in one launch, each on its own view of u: column j is
// multiplied by uown[i] on the rows i of the index range of its owner (client j / um) and by
// u[i] elsewhere.  Covers all n rows and columns; partial has col_strips(n) rows.
int launch_colpartial_view(int dtype, const void* K, int64_t ld, int n, const void* u,
                           const void* uown, int um, void* partial, int64_t ld_ws,
                           hipStream_t stream);

// partial[s][j] = sum over rows of strip s of K[i][j] u[i], for the 16-byte column packs that
// intersect [c0, c1).  partial has col_strips(rows) rows of ld_ws elements.
int launch_colpartial(int dtype, const void* K, int64_t ld, int n, int rows, int c0, int c1,
                      const void* u, void* partial, int64_t ld_ws, hipStream_t stream);

// out[j] = epilogue(marg[j], sum_s partial[s][j], old[j]) for j in [c0, c1).
// groups > 0: the partial rows are summed in exactly that many contiguous groups (it must divide
// n_partials and be at most 256), each in index order, then the group sums in group order -- block
// products first, then the blocks; 0: a grouping chosen from the number of partials and the pitch.
int launch_colreduce(int dtype, const void* partial, int64_t ld_ws, int n_partials, int c0, int c1,
                     const void* marg, const void* old, void* out, int epi, double eta,
                     hipStream_t stream, int groups = 0);

// The block products K_{:,J_z} v_{J_z} of `blocks` column blocks of `ncols` columns each, over
// `rows` rows, in ONE grid: out + z*out_block_stride receives block z's `rows` products.
int launch_rowpass_colblocks(int dtype, const void* K, int64_t ld, int ncols, int rows, int blocks,
                             const void* vin, void* out, int64_t out_block_stride,
                             hipStream_t stream);

// Geometry of the fused one-pass kernel: every row block of m rows is cut into strips of h rows;
// a strip is streamed by gb workgroups, each of which leaves one row of partial column sums.
struct FusedPlan {
  bool ok;          // false: n exceeds what a workgroup can hold in registers
  int vpt;          // 16-byte packs per thread per row
  int r;            // rows processed together (one row group)
  int h;            // rows per strip (a multiple of r)
  int spb;          // strips per row block
  int nvb;          // strips in all (c * spb)
  int gb;           // workgroups per strip
  int rotmul;       // strip s starts its sweep at row group (s * rotmul) % groups
  size_t lds_bytes;
  int partial_rows() const { return nvb * gb; }
};
// `c` row blocks of `m` rows each.  When m is a multiple of the strip height that c = 1 gets for
// the same n, the strips (and so every partial sum) are the same for every c.
FusedPlan fused_plan(int dtype, int n, int m, int c);

// For each strip: u_out = epilogue(marg, K v, old_u) on its rows and
// partial[strip * gb + w][:] = contribution of the rows workgroup w handled to K^T u.
// K, marg, old_u, u_out start at the first row of block 0.
int launch_fused(int dtype, const FusedPlan& plan, const void* K, int64_t ld, int n, int m,
                 const void* marg, const void* vin, const void* old_u, void* u_out,
                 void* partial, int64_t ld_ws, int epi, double eta, hipStream_t stream,
                 void* err_out = nullptr);

// Per-row terms of the plan sums: with kv_ij = K_ij v_j,
//   rows[0][i] = u_i sum_j kv_ij            rows[1][i] = u_i sum_j kv_ij C_ij
//   rows[2][i] = u_i (sum_j kv_ij log kv_ij + log(u_i) sum_j kv_ij)
//   rows[3][i] = u_i sum_j kv_ij l_j        (0 if l is NULL);   rows: 4 arrays of `stride` elements.
int launch_plan_rows(int dtype, const void* K, int64_t ldK, const void* C, int64_t ldC, int n,
                     const void* u, const void* v, const void* l, void* rows, int64_t stride,
                     hipStream_t stream);

// out (one double) = sum of x[0..n) accumulated in fp64 in a fixed order.
int launch_sum_to_double(int dtype, const void* x, int n, double* out, hipStream_t stream,
                         bool square = false);

// ------------------------------------------------------------------ setup kernels
int launch_gibbs_from_cost(int dtype, const void* C, int64_t ldC, int n, double eps, void* K,
                           int64_t ldK, hipStream_t stream);
int launch_gibbs_lambda(int dtype, const void* c, int64_t ldc, int n, double lambda, const void* l,
                        double eps, void* K, int64_t ldK, hipStream_t stream);
int launch_fill(int dtype, void* x, int n, double value, hipStream_t stream);
// cmax_dev (one double, device) = max_ij ||x_i - y_j||^2; scratch holds one double per workgroup.
int launch_max_sqdist(int dtype, const void* x, const void* y, int n, int d, double* scratch,
                      size_t scratch_doubles, double* cmax_dev, hipStream_t stream);
// K_ij = exp(-(||x_i-y_j||^2 / cmax) / eps); cmax read from cmax_dev, or 1 if it is NULL.
int launch_gibbs_from_points(int dtype, const void* x, const void* y, int n, int d, double eps,
                             const double* cmax_dev, void* K, int64_t ldK, hipStream_t stream);
size_t max_sqdist_scratch_doubles(int n);

// ------------------------------------------------------------------ log-domain path
size_t log_workspace_bytes(int n, int d);  // 0 if the point dimension is not supported
int run_sinkhorn_log_points(const fsk_opts* o, const void* x, const void* y, int d, double eps,
                            const void* a, const void* b, void* f, void* g, void* workspace,
                            size_t ws_bytes, int32_t* iters_done, double* err_out,
                            hipStream_t st);

// ------------------------------------------------------------------ register-resident flow
struct ResidentPlan {
  bool ok;          // false: K does not fit the registers of 32 workgroups
  int wgs;          // workgroups of the persistent grid
  int rows_per_wg;  // rows of K a workgroup owns
  int p_pad;        // threads per row subgroup: 16-byte packs per row rounded up to whole waves
  int rpt;          // packs per thread the kernel variant holds (8 or 16)
  int64_t ld_ws;    // elements per partial row
};
ResidentPlan resident_plan(int dtype, int n);
size_t resident_workspace_bytes(int dtype, int n);
// `iters` iterations of Algorithm 1 (arithmetic relaxation if eta < 1) in one launch; u, v IN/OUT.
// `workspace` must hold resident_workspace_bytes().  A grid barrier that sees no progress for
// spin_limit polls makes the call write NaN results instead of hanging.
int launch_resident(int dtype, const void* K, int64_t ld, int n, int iters, const void* a,
                    const void* b, void* u, void* v, void* workspace, double eta,
                    unsigned spin_limit, hipStream_t st);

// ------------------------------------------------------------------ multitarget path
size_t batched_workspace_bytes(int n, int m);
// Tolerance mode of the multitarget iteration (may be null: fixed iteration count).  The error of
// the state after `it` iterations falls out of the U-update of iteration it + 1: with
// Q = K V of that state, |U_ik Q_ik - A_ik| = A_ik |U_ik / U_ik^new - 1|, so a poll costs a copy
// of U, one elementwise pass and a synchronisation; a state that met the tolerance is restored
// from the copy.  Only the state after max_iters needs one extra product.
struct BatchedPoll {
  double tol;
  int check_every;
  double* scratch;     // batched_poll_scratch_doubles(n, m) doubles; [0] receives the error
  int32_t* iters_done; // host
  double* err;         // host, may be null
};
size_t batched_poll_scratch_doubles(int n, int m);
// scratch[0] = max over columns k of sum_i A_ik |Uold_ik / Unew_ik - 1| (fp64, fixed order); with
// `l2` of sqrt(sum_i (A_ik |Uold_ik / Unew_ik - 1|)^2).
int launch_batched_poll_error(int dtype, const void* A, const void* Uold, const void* Unew, int n,
                              int m, double* scratch, hipStream_t st, bool l2 = false);
// X <- (1 - eta) X + eta Xnew, or X <- X^(1-eta) Xnew^eta (as exp2 of the weighted log2's), over
// `count` elements (Sec. 3.3 on every target).
int launch_batched_relax(int dtype, void* X, const void* Xnew, int64_t count, double eta, int geometric,
                         hipStream_t st);
// `dp` (may be null): release U after every U-update and V after every V-update.  `tmp`: n x m
// elements of scratch, needed when opts->damping != FSK_DAMP_NONE or `poll` asks for a tolerance.
int run_sinkhorn_batched(const fsk_opts* o, const void* K, int64_t ldK, const void* A, const void* B,
                         void* U, void* V, void* workspace, size_t ws_bytes, const fsk_dp* dp,
                         hipStream_t st, const BatchedPoll* poll = nullptr, void* tmp = nullptr);

// fp64 form (MFMA f64 16x16x4): needs the full workspace (partial products + K^T).
size_t batched_f64_workspace_bytes(int n, int m);
int run_sinkhorn_batched_f64(const fsk_opts* o, const void* K, int64_t ldK, const void* A, const void* B,
                             void* U, void* V, void* workspace, size_t ws_bytes, const fsk_dp* dp,
                             hipStream_t st, const BatchedPoll* poll = nullptr, void* tmp = nullptr);
// The loop both precisions share: `u_update(dst)` / `v_update(dst)` enqueue one half-step into dst
// (normally U or V itself), `release(it, is_v)` the privacy layer's step (may do nothing).
// `poll` null or with tol <= 0: exactly max_iters iterations, nothing synchronises.
// With a relaxation (Sec. 3.3) every half-step lands in `tmp` first and an elementwise kernel
// folds it into the scaling; the undamped U in `tmp` is also what a poll reads the error off.
template <class UUpdate, class VUpdate, class Release>
inline int batched_iterate(const fsk_opts* o, const void* A, void* U, void* V, const BatchedPoll* poll,
                           void* tmp, hipStream_t st, UUpdate u_update, VUpdate v_update,
                           Release release) {
  const int n = o->n, m = o->m;
  const int64_t count = (int64_t)n * m;
  const size_t bytes = (size_t)count * elem_size(o->dtype);
  const bool check = poll && poll->tol > 0.0;
  const bool damped = o->damping != FSK_DAMP_NONE && o->eta < 1.0;
  const int geometric = o->damping == FSK_DAMP_GEOMETRIC ? 1 : 0;
  if ((check || damped) && !tmp) return set_error(FSK_EWORKSPACE, "multitarget call: scratch for U is missing");
  int done = 0;
  double e = NAN;
  bool converged = false;
  auto read_error = [&](const void* u_old, const void* u_new) -> int {
    FSK_TRY(launch_batched_poll_error(o->dtype, A, u_old, u_new, n, m, poll->scratch, st,
                                      o->err_norm == FSK_NORM_L2));
    FSK_HIP(hipMemcpyAsync(&e, poll->scratch, sizeof(double), hipMemcpyDeviceToHost, st));
    FSK_HIP(hipStreamSynchronize(st));
    return FSK_OK;
  };
  if (check) trace_begin();
  auto nonfinite = [&](int at) {
    if (poll->iters_done) *poll->iters_done = at;
    if (poll->err) *poll->err = e;
    return set_error(FSK_ENONFINITE, "marginal error is not finite after %d iterations", at);
  };
  for (int it = 0; it < o->max_iters; ++it) {
    // the U-update forms K V of the state after `it` iterations: a poll reads its error there
    const bool p = check && it > 0 && it % poll->check_every == 0;
    if (damped) {
      FSK_TRY(u_update(tmp));
      if (p) {
        FSK_TRY(read_error(U, tmp));
        trace_poll(it, e);
        if (!(e == e) || e > 1.7e308) return nonfinite(it);
        if (e < poll->tol) {  // U has not been touched yet
          done = it;
          converged = true;
          break;
        }
      }
      FSK_TRY(launch_batched_relax(o->dtype, U, tmp, count, o->eta, geometric, st));
    } else {
      if (p) FSK_HIP(hipMemcpyAsync(tmp, U, bytes, hipMemcpyDeviceToDevice, st));
      FSK_TRY(u_update(U));
      if (p) {
        FSK_TRY(read_error(tmp, U));
        trace_poll(it, e);
        if (!(e == e) || e > 1.7e308) return nonfinite(it);
        if (e < poll->tol) {  // undo the update that revealed it
          FSK_HIP(hipMemcpyAsync(U, tmp, bytes, hipMemcpyDeviceToDevice, st));
          FSK_HIP(hipStreamSynchronize(st));
          done = it;
          converged = true;
          break;
        }
      }
    }
    FSK_TRY(release(it, false));
    if (damped) {
      FSK_TRY(v_update(tmp));
      FSK_TRY(launch_batched_relax(o->dtype, V, tmp, count, o->eta, geometric, st));
    } else {
      FSK_TRY(v_update(V));
    }
    FSK_TRY(release(it, true));
    done = it + 1;
  }
  if (check && !converged && done > 0) {  // the state after the last iteration is always polled
    FSK_TRY(u_update(tmp));                // its next (undamped) U, only to read the error off it
    FSK_TRY(read_error(U, tmp));
    trace_poll(done, e);
    if (!(e == e) || e > 1.7e308) return nonfinite(done);
  }
  if (poll) {
    if (poll->iters_done) *poll->iters_done = done;
    if (poll->err) *poll->err = e;
  }
  return FSK_OK;
}

// ------------------------------------------------------------------ privacy layer
// X (n x m, in place) <- exp(rowclip_S(log X) + sigma * normals of (seed, release)).
int launch_dp_release(int dtype, void* X, int n, int m, double S, double sigma, uint64_t seed,
                      uint64_t release, hipStream_t stream);

// ------------------------------------------------------------------ measurement helpers
int launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
int launch_read(const void* src, size_t bytes, float* sink, hipStream_t stream);

}  // namespace fsk
