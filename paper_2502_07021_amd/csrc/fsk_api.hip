// C ABI of libfsk: argument validation, workspace carving and the host loops that
// enqueue the kernels.  Declarations and the meaning of every argument are in
// include/fsk.h.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "fsk_device.h"
#include "fsk_internal.h"

#include <atomic>
#include <mutex>

namespace fsk {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = '\0'; }

// Error trace of the calling thread: (iteration, error) pairs of the polls of its last
// tolerance-mode call, in a buffer the caller lent with fsk_set_error_trace.
static thread_local double* g_trace = nullptr;
static thread_local int32_t g_trace_cap = 0, g_trace_len = 0;
void trace_begin() { g_trace_len = 0; }
void trace_poll(int iteration, double err) {
  if (g_trace && g_trace_len < g_trace_cap) {
    g_trace[2 * g_trace_len] = (double)iteration;
    g_trace[2 * g_trace_len + 1] = err;
  }
  if (g_trace) ++g_trace_len;  // counts the polls that did not fit as well
}

int device_cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (cached[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return 0;
    cached[dev] = cus;
  }
  return cached[dev];
}

// ------------------------------------------------------------------ validation
static int check_common(const fsk_opts* o) {
  if (!o) return set_error(FSK_EINVAL, "opts is NULL");
  if (o->n <= 0) return set_error(FSK_EINVAL, "n = %d must be positive", o->n);
  if (o->m < 1) return set_error(FSK_EINVAL, "m = %d must be >= 1", o->m);
  if (o->c < 1) return set_error(FSK_EINVAL, "c = %d must be >= 1", o->c);
  if (o->max_iters < 0) return set_error(FSK_EINVAL, "max_iters = %d must be >= 0", o->max_iters);
  if (o->dtype != FSK_F32 && o->dtype != FSK_F64)
    return set_error(FSK_EINVAL, "unknown dtype %d", o->dtype);
  if (o->flow < FSK_FLOW_FUSED || o->flow > FSK_FLOW_RESIDENT)
    return set_error(FSK_EINVAL, "unknown flow %d", o->flow);
  if (o->damping < FSK_DAMP_NONE || o->damping > FSK_DAMP_GEOMETRIC)
    return set_error(FSK_EINVAL, "unknown damping %d", o->damping);
  if (o->damping != FSK_DAMP_NONE && !(o->eta > 0.0 && o->eta <= 1.0))
    return set_error(FSK_EINVAL, "eta = %g must lie in (0, 1]", o->eta);
  if (o->tol > 0.0 && o->check_every < 1)
    return set_error(FSK_EINVAL, "check_every = %d must be >= 1 in tolerance mode", o->check_every);
  if (std::isnan(o->tol)) return set_error(FSK_EINVAL, "tol is NaN");
  if (o->err_norm != FSK_NORM_L1 && o->err_norm != FSK_NORM_L2)
    return set_error(FSK_EINVAL, "unknown err_norm %d", o->err_norm);
  if (o->n % o->c != 0)
    return set_error(FSK_EDIV, "c = %d does not divide n = %d (n = c*m is required)", o->c, o->n);
  return FSK_OK;
}

static int check_matrix(const char* name, const void* p, int64_t ld, int n, int dtype) {
  if (!p) return set_error(FSK_EINVAL, "%s is NULL", name);
  if (ld < n) return set_error(FSK_EINVAL, "leading dimension %lld of %s is below n = %d", (long long)ld, name, n);
  if (!aligned16(p)) return set_error(FSK_EALIGN, "%s is not 16-byte aligned", name);
  if ((ld * (int64_t)elem_size(dtype)) % 16 != 0)
    return set_error(FSK_EALIGN, "row pitch of %s (%lld bytes) is not a multiple of 16", name,
                     (long long)(ld * (int64_t)elem_size(dtype)));
  return FSK_OK;
}

static int check_vec(const char* name, const void* p, bool need16) {
  if (!p) return set_error(FSK_EINVAL, "%s is NULL", name);
  if (need16 && !aligned16(p)) return set_error(FSK_EALIGN, "%s is not 16-byte aligned", name);
  return FSK_OK;
}

// ------------------------------------------------------------------ workspace
struct DenseWs {
  int64_t ld_ws;        // elements per partial row
  size_t partial_rows;  // rows the partial area holds
  size_t partial_off, vec_off, scalar_off, save_off, resident_off, total;
};

static DenseWs dense_ws(const fsk_opts* o) {
  DenseWs w{};
  const size_t s = elem_size(o->dtype);
  w.ld_ws = (int64_t)align_up((size_t)o->n, 64);
  const int rows_blk = o->n / o->c;
  size_t rows = (size_t)col_strips(o->n);
  FusedPlan p = fused_plan(o->dtype, o->n, rows_blk, o->c);
  if (p.ok && (size_t)p.partial_rows() > rows) rows = (size_t)p.partial_rows();
  w.partial_rows = rows;
  w.partial_off = 0;
  w.vec_off = align_up(rows * (size_t)w.ld_ws * s, 256);
  w.scalar_off = w.vec_off + align_up((size_t)o->n * s, 256);
  w.save_off = w.scalar_off + 256;  // u and v as they stood at a polled state
  w.resident_off = w.save_off + 2 * align_up((size_t)o->n * s, 256);
  w.total = w.resident_off + (o->flow == FSK_FLOW_RESIDENT ? resident_workspace_bytes(o->dtype, o->n) : 0);
  return w;
}

static int epi_of(const fsk_opts* o) {
  return o->damping == FSK_DAMP_ARITHMETIC ? kEpiDampArith
         : o->damping == FSK_DAMP_GEOMETRIC ? kEpiDampGeom
                                            : kEpiDivide;
}

}  // namespace fsk

using namespace fsk;

extern "C" {

int fsk_version(void) { return 100; }

const char* fsk_last_error(void) { return g_err; }

void fsk_set_error_trace(double* buf, int32_t capacity) {
  g_trace = capacity > 0 ? buf : nullptr;
  g_trace_cap = g_trace ? capacity : 0;
  g_trace_len = 0;
}

int32_t fsk_error_trace_count(void) { return g_trace_len; }

static size_t plan_ws_bytes(const fsk_opts* opts);

// Multitarget workspace: [partial products | K^T]; behind them an n x m scratch matrix (tolerance
// mode: the copy of U a poll compares against; damped run: where every half-step lands before
// it is folded in) and, in tolerance mode, the error kernels' scratch.
static size_t batched_base_bytes(const fsk_opts* o) {
  return align_up(o->dtype == FSK_F64 ? batched_f64_workspace_bytes(o->n, o->m)
                                      : batched_workspace_bytes(o->n, o->m), 256);
}
static size_t batched_save_bytes(const fsk_opts* o) {
  return align_up((size_t)o->n * (size_t)o->m * elem_size(o->dtype), 256);
}
static bool batched_needs_tmp(const fsk_opts* o) { return o->tol > 0.0 || o->damping != FSK_DAMP_NONE; }
static size_t batched_total_bytes(const fsk_opts* o) {
  size_t total = batched_base_bytes(o);
  if (batched_needs_tmp(o)) total += batched_save_bytes(o);
  if (o->tol > 0.0) total += align_up(batched_poll_scratch_doubles(o->n, o->m) * 8, 256);
  return total;
}

size_t fsk_workspace_bytes(const fsk_opts* opts, int mode, int d) {
  if (check_common(opts) != FSK_OK) return 0;
  switch (mode) {
    case FSK_MODE_DENSE: return dense_ws(opts).total;
    case FSK_MODE_LOG: return log_workspace_bytes(opts->n, d);
    case FSK_MODE_PLAN: return plan_ws_bytes(opts);
    case FSK_MODE_RADIUS: return align_up(dense_ws(opts).total, 256) + plan_ws_bytes(opts);
    case FSK_MODE_BATCHED: return batched_total_bytes(opts);
    case FSK_MODE_SETUP: return align_up(max_sqdist_scratch_doubles(opts->n) * 8, 256) + 256;
    default: return 0;
  }
}

int fsk_kernel_from_cost(const fsk_opts* opts, const void* C, int64_t ldC, double eps, void* K,
                         int64_t ldK, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (!(eps > 0.0)) return set_error(FSK_EINVAL, "eps = %g must be positive", eps);
  if (!C || !K) return set_error(FSK_EINVAL, "C or K is NULL");
  if (ldC < opts->n || ldK < opts->n) return set_error(FSK_EINVAL, "leading dimension below n");
  return launch_gibbs_from_cost(opts->dtype, C, ldC, opts->n, eps, K, ldK, (hipStream_t)stream);
}

int fsk_kernel_from_points(const fsk_opts* opts, const void* x, const void* y, int d, double eps,
                           int normalise_by_max, void* K, int64_t ldK, void* workspace,
                           size_t ws_bytes, double* cmax_out, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (!(eps > 0.0)) return set_error(FSK_EINVAL, "eps = %g must be positive", eps);
  if (d < 1) return set_error(FSK_EINVAL, "d = %d must be >= 1", d);
  if (!x || !y || !K) return set_error(FSK_EINVAL, "x, y or K is NULL");
  if (ldK < opts->n) return set_error(FSK_EINVAL, "leading dimension below n");
  hipStream_t st = (hipStream_t)stream;
  const bool need_max = normalise_by_max || cmax_out;
  double* cmax_dev = nullptr;
  if (need_max) {
    const size_t need = fsk_workspace_bytes(opts, FSK_MODE_SETUP, d);
    if (!workspace || ws_bytes < need)
      return set_error(FSK_EWORKSPACE, "setup needs %zu workspace bytes, got %zu", need, ws_bytes);
    const size_t cnt = max_sqdist_scratch_doubles(opts->n);
    double* scratch = (double*)workspace;
    cmax_dev = (double*)((char*)workspace + align_up(cnt * 8, 256));
    FSK_TRY(launch_max_sqdist(opts->dtype, x, y, opts->n, d, scratch, cnt, cmax_dev, st));
  }
  FSK_TRY(launch_gibbs_from_points(opts->dtype, x, y, opts->n, d, eps,
                                   normalise_by_max ? cmax_dev : nullptr, K, ldK, st));
  if (cmax_out) {
    FSK_HIP(hipMemcpyAsync(cmax_out, cmax_dev, sizeof(double), hipMemcpyDeviceToHost, st));
    FSK_HIP(hipStreamSynchronize(st));
  }
  return FSK_OK;
}

// One dense iteration, enqueued.  `stream_only`: just its K-streaming launches (the reduction
// kernels that finish the v-update are left out: what the profile call times on its own).
// *stream_launches (if given) receives the number of K-streaming launches.
// `errvec` (n entries, optional): the u-update also leaves |u_i (K v)_i - a_i| there for the
// scalings as they stood BEFORE this iteration (the row-marginal error terms, for free).
static int dense_iteration(const fsk_opts* o, const DenseWs& w, const char* K, int64_t ld,
                           const char* a, const char* b, char* u, char* v, char* ws,
                           hipStream_t st, bool stream_only = false,
                           int32_t* stream_launches = nullptr, char* errvec = nullptr) {
  const int n = o->n, c = o->c, m = n / c, dt = o->dtype;
  const int epi = epi_of(o);
  void* partial = ws + w.partial_off;
  int flow = o->flow;
  FusedPlan plan{};
  if (flow == FSK_FLOW_FUSED) {
    plan = fused_plan(dt, n, m, c);
    // rows too long to hold in registers, or the geometric relaxation in fp64 (its log2 / exp2
    // do not fit the fused kernel's register budget)
    if (!plan.ok || (epi == kEpiDampGeom && dt == FSK_F64)) flow = FSK_FLOW_TWO_PASS;
  }
  if (flow == FSK_FLOW_FUSED) {
    FSK_TRY(launch_fused(dt, plan, K, ld, n, m, a, v, u, u, partial, w.ld_ws, epi, o->eta, st, errvec));
    if (!stream_only)
      FSK_TRY(launch_colreduce(dt, partial, w.ld_ws, plan.partial_rows(), 0, n, b, v, v, epi, o->eta, st));
    if (stream_launches) *stream_launches = 1;
    return FSK_OK;
  }
  // every worker j at once (one grid, slab j = its row block): u_{I_j} from K_{I_j,:} and the shared v
  FSK_TRY(launch_rowpass_slabs(dt, K, ld, n, m, c, v, nullptr, a, u, u, epi, o->eta, st, errvec));
  // TWO_PASS: r = K^T u over all rows.  PAPER: worker j forms r_{I_j} = (K_{:,I_j})^T u from its
  // column slab; on one device the c column slabs tile the whole column range and every column is
  // summed on its own over the same row strips, so one launch over all columns IS the c slab
  // products (launching them one by one gave the same bits at 16 KiB-wide, slower reads).
  FSK_TRY(launch_colpartial(dt, K, ld, n, n, 0, n, u, partial, w.ld_ws, st));
  if (!stream_only)
    FSK_TRY(launch_colreduce(dt, partial, w.ld_ws, col_strips(n), 0, n, b, v, v, epi, o->eta, st));
  if (stream_launches) *stream_launches = 2;
  return FSK_OK;
}

// err = ||diag(u) K v - a||_1, synchronising.
// ||P1 - a||_1 into *err (and, if asked for, ||P1 - a||_2 into *err_l2) from one row pass.
static int dense_error(const fsk_opts* o, const DenseWs& w, const void* K, int64_t ld,
                       const void* a, const void* u, const void* v, char* ws, double* err,
                       hipStream_t st, double* err_l2 = nullptr) {
  void* errvec = ws + w.vec_off;
  double* scalar = (double*)(ws + w.scalar_off);
  FSK_TRY(launch_rowpass(o->dtype, K, ld, o->n, o->n, v, a, u, errvec, kEpiAbsErr, 0.0, st));
  FSK_TRY(launch_sum_to_double(o->dtype, errvec, o->n, scalar, st));
  if (err) FSK_HIP(hipMemcpyAsync(err, scalar, sizeof(double), hipMemcpyDeviceToHost, st));
  if (err_l2) {
    FSK_HIP(hipStreamSynchronize(st));  // the scalar is reused
    FSK_TRY(launch_sum_to_double(o->dtype, errvec, o->n, scalar, st, true));
    FSK_HIP(hipMemcpyAsync(err_l2, scalar, sizeof(double), hipMemcpyDeviceToHost, st));
  }
  FSK_HIP(hipStreamSynchronize(st));
  if (err_l2) *err_l2 = sqrt(*err_l2);
  return FSK_OK;
}

// Polls a waiter of the register-resident flow's grid barrier makes before it gives up (each
// poll is an atomic load plus a short sleep: of the order of a second in all by default).
static std::atomic<unsigned> g_resident_spin_limit{4000000u};
#define kResidentSpinLimit (g_resident_spin_limit.load(std::memory_order_relaxed))

static int check_resident(const fsk_opts* o) {
  if (!resident_plan(o->dtype, o->n).ok)
    return set_error(FSK_EUNSUPPORTED, "n = %d: K does not fit the registers of the resident grid", o->n);
  return FSK_OK;
}
// The resident kernel's encoding: 1 = plain, (0, 1) arithmetic, negative = geometric with -eta.
static double resident_eta(const fsk_opts* o) {
  return o->damping == FSK_DAMP_ARITHMETIC ? o->eta : o->damping == FSK_DAMP_GEOMETRIC ? -o->eta : 1.0;
}

// Algorithm 1 on validated arguments: opts->max_iters iterations, or until a poll finds the
// marginal error below opts->tol.
static int dense_solve(const fsk_opts* opts, const DenseWs& w, const void* K, int64_t ldK,
                       const void* a, const void* b, void* u, void* v, char* workspace,
                       int32_t* iters_done, double* err, hipStream_t st) {
  int done = 0;
  double e = NAN;
  const bool resident = opts->flow == FSK_FLOW_RESIDENT;
  if (resident) FSK_TRY(check_resident(opts));
  const bool check = opts->tol > 0.0;
  if (check) trace_begin();
  auto nonfinite = [&](int at) {
    if (iters_done) *iters_done = at;
    if (err) *err = e;
    return set_error(FSK_ENONFINITE, "marginal error is not finite after %d iterations", at);
  };
  const bool l2 = opts->err_norm == FSK_NORM_L2;
  auto state_error = [&]() -> int {  // the chosen norm of P1 - a for the scalings as they stand
    return l2 ? dense_error(opts, w, K, ldK, a, u, v, workspace, nullptr, st, &e)
              : dense_error(opts, w, K, ldK, a, u, v, workspace, &e, st);
  };
  if (resident) {
    for (int it = 0; it < opts->max_iters;) {  // all the iterations up to the next poll in one launch
      int chunk = opts->max_iters - it;
      if (check && opts->check_every - it % opts->check_every < chunk)
        chunk = opts->check_every - it % opts->check_every;
      FSK_TRY(launch_resident(opts->dtype, K, ldK, opts->n, chunk, a, b, u, v,
                              workspace + w.resident_off, resident_eta(opts), kResidentSpinLimit, st));
      it += chunk;
      done = it;
      if (check && (done % opts->check_every == 0 || done == opts->max_iters)) {
        FSK_TRY(state_error());
        trace_poll(done, e);
        if (!std::isfinite(e)) return nonfinite(done);
        if (e < opts->tol) break;
      }
    }
  } else {
    // The error of the state after `it` iterations falls out of the u-update of iteration
    // it + 1 (its row products are K v of that state): a poll costs two n-vector copies, a
    // sum and a synchronisation, not a pass over K.  If the state turns out to have met the
    // tolerance, the iteration that revealed it is undone by restoring the saved vectors.
    const size_t vec_bytes = (size_t)opts->n * elem_size(opts->dtype);
    char* errvec = workspace + w.vec_off;
    char* save_u = workspace + w.save_off;
    char* save_v = save_u + align_up(vec_bytes, 256);
    double* scalar = (double*)(workspace + w.scalar_off);
    bool converged = false;
    for (int it = 0; it < opts->max_iters; ++it) {
      const bool poll = check && it > 0 && it % opts->check_every == 0;
      if (poll) {
        FSK_HIP(hipMemcpyAsync(save_u, u, vec_bytes, hipMemcpyDeviceToDevice, st));
        FSK_HIP(hipMemcpyAsync(save_v, v, vec_bytes, hipMemcpyDeviceToDevice, st));
      }
      FSK_TRY(dense_iteration(opts, w, (const char*)K, ldK, (const char*)a, (const char*)b, (char*)u,
                              (char*)v, workspace, st, false, nullptr, poll ? errvec : nullptr));
      if (poll) {
        FSK_TRY(launch_sum_to_double(opts->dtype, errvec, opts->n, scalar, st, l2));
        FSK_HIP(hipMemcpyAsync(&e, scalar, sizeof(double), hipMemcpyDeviceToHost, st));
        FSK_HIP(hipStreamSynchronize(st));
        if (l2) e = sqrt(e);
        trace_poll(it, e);
        if (!std::isfinite(e)) {  // hand back the polled state itself, not the one advanced past it
          FSK_HIP(hipMemcpyAsync(u, save_u, vec_bytes, hipMemcpyDeviceToDevice, st));
          FSK_HIP(hipMemcpyAsync(v, save_v, vec_bytes, hipMemcpyDeviceToDevice, st));
          FSK_HIP(hipStreamSynchronize(st));
          return nonfinite(it);
        }
        if (e < opts->tol) {
          FSK_HIP(hipMemcpyAsync(u, save_u, vec_bytes, hipMemcpyDeviceToDevice, st));
          FSK_HIP(hipMemcpyAsync(v, save_v, vec_bytes, hipMemcpyDeviceToDevice, st));
          FSK_HIP(hipStreamSynchronize(st));
          done = it;
          converged = true;
          break;
        }
      }
      done = it + 1;
    }
    if (check && !converged && done > 0) {  // the state after the last iteration is always polled
      FSK_TRY(state_error());
      trace_poll(done, e);
      if (!std::isfinite(e)) return nonfinite(done);
    }
  }
  if (iters_done) *iters_done = done;
  if (err) *err = e;
  return FSK_OK;
}

void fsk_set_barrier_poll_limit(uint32_t polls) {
  g_resident_spin_limit.store(polls, std::memory_order_relaxed);
}

int fsk_sinkhorn_dense(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                       const void* b, void* u, void* v, void* workspace, size_t ws_bytes,
                       int32_t* iters_done, double* err, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "dense call takes m = 1 (use fsk_sinkhorn_batched)");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const DenseWs w = dense_ws(opts);
  if (!workspace || ws_bytes < w.total)
    return set_error(FSK_EWORKSPACE, "dense call needs %zu workspace bytes, got %zu", w.total, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  return dense_solve(opts, w, K, ldK, a, b, u, v, (char*)workspace, iters_done, err,
                     (hipStream_t)stream);
}

// ---- the dense call for callers that cannot allocate: its scratch is part of the library image.
// In host code the array's name only stands for the symbol; the device address comes from
// hipGetSymbolAddress, once per device (every GPU holds its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[FSK_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {nullptr};

static int static_scratch(char** out) {
  int dev = 0;
  FSK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(FSK_EUNSUPPORTED, "device index %d outside [0, 64)", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    FSK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return set_error(FSK_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return FSK_OK;
}

int fsk_sinkhorn_dense_static(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                              const void* b, void* u, void* v, int32_t* iters_done, double* err,
                              void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "dense call takes m = 1 (use fsk_sinkhorn_batched)");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const DenseWs w = dense_ws(opts);
  if (w.total > (size_t)FSK_STATIC_SCRATCH_BYTES)
    return set_error(FSK_EWORKSPACE,
                     "this problem needs %zu bytes of scratch, the built-in array holds %zu: use "
                     "fsk_sinkhorn_dense with a workspace", w.total, (size_t)FSK_STATIC_SCRATCH_BYTES);
  char* ws = nullptr;
  FSK_TRY(static_scratch(&ws));
  return dense_solve(opts, w, K, ldK, a, b, u, v, ws, iters_done, err, (hipStream_t)stream);
}

int fsk_dense_profile(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                      const void* b, void* u, void* v, void* workspace, size_t ws_bytes, int reps,
                      double* stream_ms, double* other_ms, int32_t* stream_launches, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "dense call takes m = 1");
  if (reps < 1) return set_error(FSK_EINVAL, "reps = %d must be >= 1", reps);
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const DenseWs w = dense_ws(opts);
  if (!workspace || ws_bytes < w.total)
    return set_error(FSK_EWORKSPACE, "dense call needs %zu workspace bytes, got %zu", w.total, ws_bytes);
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t ev[3];
  for (int k = 0; k < 3; ++k) FSK_HIP(hipEventCreate(&ev[k]));
  double t_stream = 0.0, t_other = 0.0;
  int32_t launches = 0;
  int rc = FSK_OK;
  if (opts->flow == FSK_FLOW_RESIDENT) {  // one launch runs all `reps` iterations
    rc = check_resident(opts);
    if (rc == FSK_OK && hipEventRecord(ev[0], st) != hipSuccess) rc = set_error(FSK_EHIP, "hipEventRecord failed");
    if (rc == FSK_OK)
      rc = launch_resident(opts->dtype, K, ldK, opts->n, reps, a, b, u, v,
                           (char*)workspace + w.resident_off, resident_eta(opts), kResidentSpinLimit, st);
    if (rc == FSK_OK && (hipEventRecord(ev[1], st) != hipSuccess || hipEventSynchronize(ev[1]) != hipSuccess))
      rc = set_error(FSK_EHIP, "event timing of the resident launch failed");
    float ms = 0.f;
    if (rc == FSK_OK && hipEventElapsedTime(&ms, ev[0], ev[1]) != hipSuccess)
      rc = set_error(FSK_EHIP, "hipEventElapsedTime failed");
    for (int k = 0; k < 3; ++k) (void)hipEventDestroy(ev[k]);
    if (rc != FSK_OK) return rc;
    if (stream_ms) *stream_ms = ms / reps;
    if (other_ms) *other_ms = 0.0;
    if (stream_launches) *stream_launches = 1;
    return FSK_OK;
  }
  // Two back-to-back runs between three events: `reps` times the K-streaming launches alone
  // (nothing between two of them but the hand-over from one kernel to the next, well under a
  // microsecond of a 0.05-0.6 ms launch), then `reps` whole iterations; the reduction kernels'
  // share is the difference.  An event per launch would put a marker packet, and its few
  // microseconds, inside every span.
  rc = dense_iteration(opts, w, (const char*)K, ldK, (const char*)a, (const char*)b, (char*)u,
                       (char*)v, (char*)workspace, st, true, &launches);  // untimed: the queue is busy after it
  if (rc == FSK_OK && hipEventRecord(ev[0], st) != hipSuccess) rc = set_error(FSK_EHIP, "hipEventRecord failed");
  for (int it = 0; it < reps && rc == FSK_OK; ++it)
    rc = dense_iteration(opts, w, (const char*)K, ldK, (const char*)a, (const char*)b, (char*)u,
                         (char*)v, (char*)workspace, st, true, &launches);
  if (rc == FSK_OK && hipEventRecord(ev[1], st) != hipSuccess) rc = set_error(FSK_EHIP, "hipEventRecord failed");
  for (int it = 0; it < reps && rc == FSK_OK; ++it)
    rc = dense_iteration(opts, w, (const char*)K, ldK, (const char*)a, (const char*)b, (char*)u,
                         (char*)v, (char*)workspace, st, false, &launches);
  if (rc == FSK_OK && (hipEventRecord(ev[2], st) != hipSuccess || hipEventSynchronize(ev[2]) != hipSuccess))
    rc = set_error(FSK_EHIP, "event timing failed");
  float ms01 = 0.f, ms12 = 0.f;
  if (rc == FSK_OK && (hipEventElapsedTime(&ms01, ev[0], ev[1]) != hipSuccess ||
                       hipEventElapsedTime(&ms12, ev[1], ev[2]) != hipSuccess))
    rc = set_error(FSK_EHIP, "hipEventElapsedTime failed");
  for (int k = 0; k < 3; ++k) (void)hipEventDestroy(ev[k]);
  if (rc != FSK_OK) return rc;
  t_stream = ms01 / reps;
  t_other = ms12 / reps - t_stream;
  if (stream_ms) *stream_ms = t_stream;
  if (other_ms) *other_ms = t_other > 0.0 ? t_other : 0.0;
  if (stream_launches) *stream_launches = launches;
  return FSK_OK;
}

int fsk_marginals(const fsk_opts* opts, const void* K, int64_t ldK, const void* a, const void* u,
                  const void* v, void* row_marginal, void* col_marginal, void* workspace,
                  size_t ws_bytes, double* err_l1, double* err_l2, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const DenseWs w = dense_ws(opts);
  if (!workspace || ws_bytes < w.total)
    return set_error(FSK_EWORKSPACE, "marginals need %zu workspace bytes, got %zu", w.total, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int n = opts->n, dt = opts->dtype;
  char* ws = (char*)workspace;
  if (row_marginal)
    FSK_TRY(launch_rowpass(dt, K, ldK, n, n, v, nullptr, u, row_marginal, kEpiMarginal, 0.0, st));
  if (col_marginal) {
    FSK_TRY(launch_colpartial(dt, K, ldK, n, n, 0, n, u, ws + w.partial_off, w.ld_ws, st));
    FSK_TRY(launch_colreduce(dt, ws + w.partial_off, w.ld_ws, col_strips(n), 0, n, nullptr, v,
                             col_marginal, kEpiMarginal, 0.0, st));
  }
  if (err_l1 || err_l2) {
    FSK_TRY(check_vec("a", a, false));
    FSK_TRY(dense_error(opts, w, K, ldK, a, u, v, ws, err_l1, st, err_l2));
  }
  return FSK_OK;
}

// ------------------------------------------------------------- plan objective
static size_t plan_ws_bytes(const fsk_opts* opts) {
  return 4 * align_up((size_t)opts->n * elem_size(opts->dtype), 256) + 256;
}

// The five plan sums on validated arguments (synchronises).
static int plan_sums(const fsk_opts* opts, const void* K, int64_t ldK, const void* C, int64_t ldC,
                     double eps, const void* u, const void* v, const void* l, double* out, char* ws,
                     hipStream_t st) {
  const int n = opts->n, dt = opts->dtype;
  const size_t vec = align_up((size_t)n * elem_size(dt), 256);
  const int64_t stride = (int64_t)(vec / elem_size(dt));
  double* sums = (double*)(ws + 4 * vec);
  FSK_TRY(launch_plan_rows(dt, K, ldK, C, ldC, n, u, v, l, ws, stride, st));
  for (int q = 0; q < 4; ++q)
    FSK_TRY(launch_sum_to_double(dt, ws + (size_t)q * vec, n, sums + q, st));
  double h[4];
  FSK_HIP(hipMemcpyAsync(h, sums, sizeof(h), hipMemcpyDeviceToHost, st));
  FSK_HIP(hipStreamSynchronize(st));
  out[0] = h[1];
  out[1] = h[2] - h[0];
  out[2] = out[0] + eps * out[1];
  out[3] = h[0];
  out[4] = l ? h[3] : 0.0;
  return FSK_OK;
}

int fsk_plan_objective(const fsk_opts* opts, const void* K, int64_t ldK, const void* C, int64_t ldC,
                       double eps, const void* u, const void* v, const void* l, double* out,
                       void* workspace, size_t ws_bytes, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (!out) return set_error(FSK_EINVAL, "out is NULL");
  if (!(eps > 0.0)) return set_error(FSK_EINVAL, "eps = %g must be positive", eps);
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_matrix("C", C, ldC, opts->n, opts->dtype));
  FSK_TRY(check_vec("u", u, false));
  FSK_TRY(check_vec("v", v, true));
  if (l && !aligned16(l)) return set_error(FSK_EALIGN, "l is not 16-byte aligned");
  const size_t need = fsk_workspace_bytes(opts, FSK_MODE_PLAN, 0);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "plan objective needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  return plan_sums(opts, K, ldK, C, ldC, eps, u, v, l, out, (char*)workspace, (hipStream_t)stream);
}

// ------------------------------------------------------------- radius search
int fsk_kernel_from_cost_lambda(const fsk_opts* opts, const void* c, int64_t ldc, double lambda,
                                const void* l, double eps, void* K, int64_t ldK, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (!(eps > 0.0)) return set_error(FSK_EINVAL, "eps = %g must be positive", eps);
  if (!std::isfinite(lambda)) return set_error(FSK_EINVAL, "lambda is not finite");
  if (!c || !K) return set_error(FSK_EINVAL, "c or K is NULL");
  if (ldc < opts->n || ldK < opts->n) return set_error(FSK_EINVAL, "leading dimension below n");
  return launch_gibbs_lambda(opts->dtype, c, ldc, opts->n, lambda, l, eps, K, ldK, (hipStream_t)stream);
}

int fsk_radius_search(const fsk_opts* opts, const void* c, int64_t ldc, const void* l, const void* a,
                      const void* b, double eps, double delta, double lambda_lo, double lambda_hi,
                      int32_t max_steps, double gtol, void* K, int64_t ldK, void* u, void* v,
                      void* workspace, size_t ws_bytes, double* out, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "radius search takes m = 1");
  if (!out) return set_error(FSK_EINVAL, "out is NULL");
  if (!(eps > 0.0)) return set_error(FSK_EINVAL, "eps = %g must be positive", eps);
  if (!std::isfinite(delta) || !std::isfinite(lambda_lo) || !std::isfinite(lambda_hi) ||
      lambda_lo > lambda_hi)
    return set_error(FSK_EINVAL, "need finite delta and lambda_lo <= lambda_hi");
  if (max_steps < 1) return set_error(FSK_EINVAL, "max_steps = %d must be >= 1", max_steps);
  if (!(gtol >= 0.0)) return set_error(FSK_EINVAL, "gtol = %g must be >= 0", gtol);
  FSK_TRY(check_matrix("c", c, ldc, opts->n, opts->dtype));
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  if (K == c) return set_error(FSK_EINVAL, "K must not alias c: every step rebuilds K from c");
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  if (l && !aligned16(l)) return set_error(FSK_EALIGN, "l is not 16-byte aligned");
  const size_t need = fsk_workspace_bytes(opts, FSK_MODE_RADIUS, 0);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "radius search needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const DenseWs w = dense_ws(opts);
  char* ws_dense = (char*)workspace;
  char* ws_plan = ws_dense + align_up(w.total, 256);
  const int n = opts->n, dt = opts->dtype;
  double lo = lambda_lo, hi = lambda_hi, lambda = 0.5 * (lo + hi), sums[5] = {NAN, NAN, NAN, NAN, NAN};
  int steps = 0;
  while (steps < max_steps) {
    lambda = 0.5 * (lo + hi);
    FSK_TRY(launch_gibbs_lambda(dt, c, ldc, n, lambda, l, eps, K, ldK, st));
    FSK_TRY(launch_fill(dt, u, n, 1.0, st));
    FSK_TRY(launch_fill(dt, v, n, 1.0, st));
    FSK_TRY(dense_solve(opts, w, K, ldK, a, b, u, v, ws_dense, nullptr, nullptr, st));
    FSK_TRY(plan_sums(opts, K, ldK, c, ldc, eps, u, v, l, sums, ws_plan, st));
    ++steps;
    if (!std::isfinite(sums[0]))
      return set_error(FSK_ENONFINITE, "transport cost is not finite at lambda = %g", lambda);
    const double g = sums[0] - delta;
    if (std::fabs(g) <= gtol) break;
    if (g > 0.0) lo = lambda; else hi = lambda;
  }
  out[0] = lambda;
  out[1] = sums[0];
  out[2] = sums[4];
  out[3] = (double)steps;
  return FSK_OK;
}

// ------------------------------------------------------------- bounded-delay emulation
size_t fsk_async_workspace_bytes(const fsk_opts* opts, int32_t tau, int32_t sync_every) {
  if (check_common(opts) != FSK_OK || tau < 0 || sync_every < 1) return 0;
  const size_t vec = align_up((size_t)opts->n * elem_size(opts->dtype), 256);
  const size_t slots = (size_t)tau + (size_t)sync_every + 1;
  return dense_ws(opts).total + vec * (2 * slots + 1);
}

int fsk_sinkhorn_async_emulated(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                                const void* b, void* u, void* v, int32_t tau, int32_t sync_every,
                                void* workspace, size_t ws_bytes, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "dense call takes m = 1");
  if (tau < 0 || sync_every < 1)
    return set_error(FSK_EINVAL, "tau = %d must be >= 0 and sync_every = %d >= 1", tau, sync_every);
  if (opts->tol > 0.0) return set_error(FSK_EUNSUPPORTED, "the emulation runs a fixed number of iterations");
  if (opts->damping == FSK_DAMP_GEOMETRIC)
    return set_error(FSK_EUNSUPPORTED, "Algorithm 3 uses the arithmetic relaxation");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const size_t need = fsk_async_workspace_bytes(opts, tau, sync_every);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "emulation needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int n = opts->n, c = opts->c, m = n / c, dt = opts->dtype;
  const size_t s = elem_size(dt), vec = align_up((size_t)n * s, 256);
  const DenseWs w = dense_ws(opts);
  const int slots = tau + sync_every + 1;
  char* ws = (char*)workspace;
  char* ring = ws + w.total;  // slot k: u at ring + 2k*vec, v at ring + (2k+1)*vec
  auto U = [&](int it) { return ring + (size_t)2 * (it % slots) * vec; };
  auto V = [&](int it) { return ring + ((size_t)2 * (it % slots) + 1) * vec; };
  const int epi = opts->damping == FSK_DAMP_ARITHMETIC ? kEpiDampArith : kEpiDivide;
  const double eta = opts->damping == FSK_DAMP_ARITHMETIC ? opts->eta : 1.0;
  const char* Kc = (const char*)K;
  FSK_HIP(hipMemcpyAsync(U(0), u, (size_t)n * s, hipMemcpyDeviceToDevice, st));
  FSK_HIP(hipMemcpyAsync(V(0), v, (size_t)n * s, hipMemcpyDeviceToDevice, st));
  for (int t = 1; t <= opts->max_iters; ++t) {
    int sidx = t - 1 - tau;
    sidx = sidx <= 0 ? 0 : (sidx / sync_every) * sync_every;
    const char *su = U(sidx), *sv = V(sidx), *pu = U(t - 1), *pv = V(t - 1);
    char *nu = U(t), *nv = V(t);
    // all clients in one grid each: client j's row pass on its view of v (remote slices from the
    // snapshot sv, own slice from the previous iteration pv), then its column-slab pass on its
    // view of u (remote su, own slice just updated)
    FSK_TRY(launch_rowpass_slabs(dt, Kc, ldK, n, m, c, sv, pv, a, pu, nu, epi, eta, st));
    FSK_TRY(launch_colpartial_view(dt, Kc, ldK, n, su, nu, m, ws + w.partial_off, w.ld_ws, st));
    FSK_TRY(launch_colreduce(dt, ws + w.partial_off, w.ld_ws, col_strips(n), 0, n, b, pv, nv, epi, eta, st));
  }
  FSK_HIP(hipMemcpyAsync(u, U(opts->max_iters), (size_t)n * s, hipMemcpyDeviceToDevice, st));
  FSK_HIP(hipMemcpyAsync(v, V(opts->max_iters), (size_t)n * s, hipMemcpyDeviceToDevice, st));
  return FSK_OK;
}

// ------------------------------------------------------------- synchronous local steps
size_t fsk_local_steps_workspace_bytes(const fsk_opts* opts) {
  if (check_common(opts) != FSK_OK) return 0;
  return align_up(dense_ws(opts).total, 256) + 2 * align_up((size_t)opts->n * elem_size(opts->dtype), 256);
}

int fsk_sinkhorn_local_steps(const fsk_opts* opts, const void* K, int64_t ldK, const void* a,
                             const void* b, void* u, void* v, int32_t w_steps, void* workspace,
                             size_t ws_bytes, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "dense call takes m = 1");
  if (w_steps < 1) return set_error(FSK_EINVAL, "w = %d local steps must be >= 1", w_steps);
  if (opts->tol > 0.0) return set_error(FSK_EUNSUPPORTED, "the local-steps call runs a fixed number of iterations");
  if (opts->damping != FSK_DAMP_NONE) return set_error(FSK_EUNSUPPORTED, "the synchronous variants are undamped");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const size_t need = fsk_local_steps_workspace_bytes(opts);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "local-steps call needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int n = opts->n, c = opts->c, m = n / c, dt = opts->dtype;
  const size_t bytes = (size_t)n * elem_size(dt), vec = align_up(bytes, 256);
  const DenseWs w = dense_ws(opts);
  char* ws = (char*)workspace;
  char* u_seen = ws + align_up(w.total, 256);  // the peers' slices as of the last Allgather of u
  char* v_seen = u_seen + vec;                 // ... of v
  FSK_HIP(hipMemcpyAsync(u_seen, u, bytes, hipMemcpyDeviceToDevice, st));  // "identical at all clients"
  FSK_HIP(hipMemcpyAsync(v_seen, v, bytes, hipMemcpyDeviceToDevice, st));
  for (int k = 1; k <= opts->max_iters; ++k) {
    const bool collective = k % w_steps == 0;
    // client j: q = K_{I_j,:} (its view of v), u_{I_j} = a_j ./ q -- all clients in one grid
    FSK_TRY(launch_rowpass_slabs(dt, K, ldK, n, m, c, v_seen, v, a, nullptr, u, kEpiDivide, 1.0, st));
    if (collective) FSK_HIP(hipMemcpyAsync(u_seen, u, bytes, hipMemcpyDeviceToDevice, st));  // Allgather u
    // client j: r = (K_{:,I_j})^T (its view of u), v_{I_j} = b_j ./ r
    FSK_TRY(launch_colpartial_view(dt, K, ldK, n, u_seen, u, m, ws + w.partial_off, w.ld_ws, st));
    FSK_TRY(launch_colreduce(dt, ws + w.partial_off, w.ld_ws, col_strips(n), 0, n, b, nullptr, v,
                             kEpiDivide, 1.0, st));
    if (collective) FSK_HIP(hipMemcpyAsync(v_seen, v, bytes, hipMemcpyDeviceToDevice, st));  // Allgather v
  }
  return FSK_OK;
}

// ------------------------------------------------------------- 2D block grid
struct GridWs { size_t stride_bytes, row_off, strip_off, tile_off, total; int64_t stride; };
static GridWs grid_ws(const fsk_opts* o, int p_r, int p_c) {
  GridWs g{};
  g.stride_bytes = align_up((size_t)o->n * elem_size(o->dtype), 256);
  g.stride = (int64_t)(g.stride_bytes / elem_size(o->dtype));
  g.row_off = 0;                                                  // p_c block-row products
  g.strip_off = g.row_off + (size_t)p_c * g.stride_bytes;         // row strips of the column pass
  g.tile_off = g.strip_off + (size_t)col_strips(o->n) * g.stride_bytes;  // p_r block-column products
  g.total = g.tile_off + (size_t)p_r * g.stride_bytes;
  return g;
}

static int check_grid(const fsk_opts* opts, int32_t p_r, int32_t p_c) {
  FSK_TRY(check_common(opts));
  if (p_r < 1 || p_c < 1) return set_error(FSK_EINVAL, "grid %d x %d must be at least 1 x 1", p_r, p_c);
  if (opts->n % p_r != 0 || opts->n % p_c != 0)
    return set_error(FSK_EDIV, "grid %d x %d does not divide n = %d", p_r, p_c, opts->n);
  if (((size_t)(opts->n / p_c) * elem_size(opts->dtype)) % 16 != 0)
    return set_error(FSK_EALIGN, "block columns of %d entries do not start on 16-byte boundaries",
                     opts->n / p_c);
  return FSK_OK;
}

size_t fsk_grid_workspace_bytes(const fsk_opts* opts, int32_t p_r, int32_t p_c) {
  if (check_grid(opts, p_r, p_c) != FSK_OK) return 0;
  return grid_ws(opts, p_r, p_c).total;
}

int fsk_sinkhorn_grid(const fsk_opts* opts, const void* K, int64_t ldK, const void* a, const void* b,
                      void* u, void* v, int32_t p_r, int32_t p_c, void* workspace, size_t ws_bytes,
                      void* stream) {
  clear_error();
  FSK_TRY(check_grid(opts, p_r, p_c));
  if (opts->m != 1) return set_error(FSK_EINVAL, "dense call takes m = 1");
  if (opts->tol > 0.0) return set_error(FSK_EUNSUPPORTED, "the grid flow runs a fixed number of iterations");
  if (opts->damping != FSK_DAMP_NONE) return set_error(FSK_EUNSUPPORTED, "the grid flow is undamped");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("u", u, true));
  FSK_TRY(check_vec("v", v, true));
  const GridWs g = grid_ws(opts, p_r, p_c);
  if (!workspace || ws_bytes < g.total)
    return set_error(FSK_EWORKSPACE, "grid flow needs %zu workspace bytes, got %zu", g.total, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int n = opts->n, dt = opts->dtype, nr = n / p_r, nc = n / p_c;
  const size_t s = elem_size(dt);
  char* ws = (char*)workspace;
  const char* Kc = (const char*)K;
  for (int it = 0; it < opts->max_iters; ++it) {
    // block products K_ij v_j for every block row and block column; the row-wise reduction over j
    // then divides
    if (p_c == 1) {
      FSK_TRY(launch_rowpass(dt, K, ldK, n, n, v, a, nullptr, u, kEpiDivide, 1.0, st));
    } else {  // all block columns in one grid; then the p_c products of a row in the order j = 0, 1, ...
      FSK_TRY(launch_rowpass_colblocks(dt, K, ldK, nc, n, p_c, v, ws + g.row_off, g.stride, st));
      FSK_TRY(launch_colreduce(dt, ws + g.row_off, g.stride, p_c, 0, n, a, nullptr, u, kEpiDivide, 1.0, st, 1));
    }
    // block products K_ij^T u_i for every block column at once; the column-wise reduction over i
    // then divides
    if (nr % kColStrip == 0 && p_r <= 256) {
      // block rows are whole 128-row strips: one pass over all rows, then per column the strips of
      // a block row in order (= the block product) and the p_r block products in the order i = 0, 1, ...
      FSK_TRY(launch_colpartial(dt, K, ldK, n, n, 0, n, u, ws + g.strip_off, g.stride, st));
      FSK_TRY(launch_colreduce(dt, ws + g.strip_off, g.stride, col_strips(n), 0, n, b, nullptr, v, kEpiDivide,
                               1.0, st, p_r));
    } else {  // one block row i at a time
      for (int i = 0; i < p_r; ++i) {
        FSK_TRY(launch_colpartial(dt, Kc + (size_t)i * nr * (size_t)ldK * s, ldK, n, nr, 0, n,
                                  (const char*)u + (size_t)i * nr * s, ws + g.strip_off, g.stride, st));
        FSK_TRY(launch_colreduce(dt, ws + g.strip_off, g.stride, col_strips(nr), 0, n, nullptr, nullptr,
                                 ws + g.tile_off + (size_t)i * g.stride_bytes, kEpiProduct, 1.0, st));
      }
      FSK_TRY(launch_colreduce(dt, ws + g.tile_off, g.stride, p_r, 0, n, b, nullptr, v, kEpiDivide, 1.0, st, 1));
    }
  }
  return FSK_OK;
}

// ------------------------------------------------------------- one worker's share
static int check_block(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                       int32_t rows) {
  FSK_TRY(check_common(opts));
  FSK_TRY(check_matrix("K_slab", K_slab, ldK, opts->n, opts->dtype));
  if (rows < 1 || row0 < 0 || (int64_t)row0 + rows > opts->n)
    return set_error(FSK_EINVAL, "rows [%d, %d) are not inside [0, %d)", row0, row0 + rows, opts->n);
  return FSK_OK;
}

int fsk_block_rowpass(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                      int32_t rows, const void* a_slab, const void* v_full, void* u_slab,
                      void* stream) {
  clear_error();
  FSK_TRY(check_block(opts, K_slab, ldK, row0, rows));
  FSK_TRY(check_vec("a_slab", a_slab, false));
  FSK_TRY(check_vec("v_full", v_full, true));
  FSK_TRY(check_vec("u_slab", u_slab, false));
  return launch_rowpass(opts->dtype, K_slab, ldK, opts->n, rows, v_full, a_slab, u_slab, u_slab,
                        epi_of(opts), opts->eta, (hipStream_t)stream);
}

int fsk_block_colpartial(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                         int32_t rows, const void* u_slab, void* s_partial, void* workspace,
                         size_t ws_bytes, void* stream) {
  clear_error();
  FSK_TRY(check_block(opts, K_slab, ldK, row0, rows));
  FSK_TRY(check_vec("u_slab", u_slab, false));
  FSK_TRY(check_vec("s_partial", s_partial, false));
  const DenseWs w = dense_ws(opts);
  if (!workspace || ws_bytes < w.total)
    return set_error(FSK_EWORKSPACE, "block call needs %zu workspace bytes, got %zu", w.total, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  FSK_TRY(launch_colpartial(opts->dtype, K_slab, ldK, opts->n, rows, 0, opts->n, u_slab,
                            ws + w.partial_off, w.ld_ws, st));
  return launch_colreduce(opts->dtype, ws + w.partial_off, w.ld_ws, col_strips(rows), 0, opts->n,
                          nullptr, nullptr, s_partial, kEpiProduct, 0.0, st);
}

int fsk_block_fused(const fsk_opts* opts, const void* K_slab, int64_t ldK, int32_t row0,
                    int32_t rows, const void* a_slab, const void* v_full, void* u_slab,
                    void* s_partial, void* workspace, size_t ws_bytes, void* stream) {
  clear_error();
  FSK_TRY(check_block(opts, K_slab, ldK, row0, rows));
  FSK_TRY(check_vec("a_slab", a_slab, false));
  FSK_TRY(check_vec("v_full", v_full, true));
  FSK_TRY(check_vec("u_slab", u_slab, false));
  FSK_TRY(check_vec("s_partial", s_partial, false));
  const FusedPlan plan = fused_plan(opts->dtype, opts->n, rows, 1);
  if (!plan.ok)
    return set_error(FSK_EUNSUPPORTED, "n = %d is too long for the register-resident fused kernel",
                     opts->n);
  const size_t s = elem_size(opts->dtype);
  const int64_t ld_ws = (int64_t)align_up((size_t)opts->n, 64);
  const size_t need = (size_t)plan.partial_rows() * (size_t)ld_ws * s;
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "fused block call needs %zu workspace bytes, got %zu", need, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  FSK_TRY(launch_fused(opts->dtype, plan, K_slab, ldK, opts->n, rows, a_slab, v_full, u_slab,
                       u_slab, workspace, ld_ws, epi_of(opts), opts->eta, st));
  return launch_colreduce(opts->dtype, workspace, ld_ws, plan.partial_rows(), 0, opts->n, nullptr, nullptr,
                          s_partial, kEpiProduct, 0.0, st);
}

// ------------------------------------------------------------- log-domain and multitarget
int fsk_sinkhorn_log_points(const fsk_opts* opts, const void* x, const void* y, int d, double eps,
                            const void* a, const void* b, void* f, void* g, void* workspace,
                            size_t ws_bytes, int32_t* iters_done, double* err, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->m != 1) return set_error(FSK_EINVAL, "log-domain call takes m = 1");
  if (opts->c != 1) return set_error(FSK_EUNSUPPORTED, "log-domain call takes c = 1");
  if (!(eps > 0.0)) return set_error(FSK_EINVAL, "eps = %g must be positive", eps);
  if (d < 1) return set_error(FSK_EINVAL, "d = %d must be >= 1", d);
  FSK_TRY(check_vec("x", x, false));
  FSK_TRY(check_vec("y", y, false));
  FSK_TRY(check_vec("a", a, false));
  FSK_TRY(check_vec("b", b, false));
  FSK_TRY(check_vec("f", f, false));
  FSK_TRY(check_vec("g", g, false));
  if (workspace && !aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  return run_sinkhorn_log_points(opts, x, y, d, eps, a, b, f, g, workspace, ws_bytes, iters_done,
                                 err, (hipStream_t)stream);
}

int fsk_sinkhorn_batched(const fsk_opts* opts, const void* K, int64_t ldK, const void* A,
                         const void* B, void* U, void* V, void* workspace, size_t ws_bytes,
                         void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->c != 1) return set_error(FSK_EUNSUPPORTED, "batched call takes c = 1");
  if (opts->tol > 0.0)
    return set_error(FSK_EUNSUPPORTED, "this call runs a fixed number of iterations (fsk_sinkhorn_batched_tol polls)");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("A", A, false));
  FSK_TRY(check_vec("B", B, false));
  FSK_TRY(check_vec("U", U, false));
  FSK_TRY(check_vec("V", V, false));
  if (workspace && !aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  if (opts->damping == FSK_DAMP_NONE)
    return run_sinkhorn_batched(opts, K, ldK, A, B, U, V, workspace, ws_bytes, nullptr, (hipStream_t)stream);
  // relaxed updates: every half-step lands in a scratch matrix behind the usual workspace first
  const size_t need = batched_total_bytes(opts), base = batched_base_bytes(opts);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "damped batched call needs %zu workspace bytes, got %zu", need, ws_bytes);
  return run_sinkhorn_batched(opts, K, ldK, A, B, U, V, workspace, base, nullptr, (hipStream_t)stream,
                              nullptr, (char*)workspace + base);
}

int fsk_sinkhorn_batched_tol(const fsk_opts* opts, const void* K, int64_t ldK, const void* A,
                             const void* B, void* U, void* V, void* workspace, size_t ws_bytes,
                             int32_t* iters_done, double* err, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (opts->c != 1) return set_error(FSK_EUNSUPPORTED, "batched call takes c = 1");
  if (!iters_done) return set_error(FSK_EINVAL, "iters_done is NULL");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("A", A, false));
  FSK_TRY(check_vec("B", B, false));
  FSK_TRY(check_vec("U", U, false));
  FSK_TRY(check_vec("V", V, false));
  const size_t need = batched_total_bytes(opts);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "batched call in tolerance mode needs %zu workspace bytes, got %zu",
                     need, ws_bytes);
  if (!aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  const size_t base = batched_base_bytes(opts);
  BatchedPoll poll{};
  poll.tol = opts->tol;
  poll.check_every = opts->check_every;
  void* tmp = batched_needs_tmp(opts) ? (char*)workspace + base : nullptr;
  poll.scratch = (double*)((char*)workspace + base + (tmp ? batched_save_bytes(opts) : 0));
  poll.iters_done = iters_done;
  poll.err = err;
  if (err) *err = NAN;
  return run_sinkhorn_batched(opts, K, ldK, A, B, U, V, workspace, base, nullptr, (hipStream_t)stream,
                              &poll, tmp);
}

// ------------------------------------------------------------- privacy layer
static int check_dp(const fsk_dp* dp) {
  if (!dp) return set_error(FSK_EINVAL, "dp is NULL");
  if (!(dp->sigma_u >= 0.0) || !(dp->sigma_v >= 0.0) || !std::isfinite(dp->sigma_u) ||
      !std::isfinite(dp->sigma_v))
    return set_error(FSK_EINVAL, "noise scales must be finite and >= 0");
  if (std::isnan(dp->clip_u) || std::isnan(dp->clip_v)) return set_error(FSK_EINVAL, "clip radius is NaN");
  if (dp->release0 % 2 != 0) return set_error(FSK_EINVAL, "release0 must be even (a U release)");
  return FSK_OK;
}

int fsk_dp_release(const fsk_opts* opts, void* X, double clip, double sigma, uint64_t seed,
                   uint64_t release, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  if (!X) return set_error(FSK_EINVAL, "X is NULL");
  if (!(sigma >= 0.0) || !std::isfinite(sigma)) return set_error(FSK_EINVAL, "sigma must be finite and >= 0");
  if (std::isnan(clip)) return set_error(FSK_EINVAL, "clip radius is NaN");
  return launch_dp_release(opts->dtype, X, opts->n, opts->m, clip, sigma, seed, release, (hipStream_t)stream);
}

int fsk_sinkhorn_batched_dp(const fsk_opts* opts, const void* K, int64_t ldK, const void* A,
                            const void* B, void* U, void* V, const fsk_dp* dp, void* workspace,
                            size_t ws_bytes, void* stream) {
  clear_error();
  FSK_TRY(check_common(opts));
  FSK_TRY(check_dp(dp));
  if (opts->c != 1) return set_error(FSK_EUNSUPPORTED, "batched call takes c = 1");
  if (opts->damping != FSK_DAMP_NONE) return set_error(FSK_EUNSUPPORTED, "the multitarget iteration is undamped");
  if (opts->tol > 0.0) return set_error(FSK_EUNSUPPORTED, "batched call runs a fixed number of iterations");
  FSK_TRY(check_matrix("K", K, ldK, opts->n, opts->dtype));
  FSK_TRY(check_vec("A", A, false));
  FSK_TRY(check_vec("B", B, false));
  FSK_TRY(check_vec("U", U, false));
  FSK_TRY(check_vec("V", V, false));
  if (workspace && !aligned16(workspace)) return set_error(FSK_EALIGN, "workspace is not 16-byte aligned");
  return run_sinkhorn_batched(opts, K, ldK, A, B, U, V, workspace, ws_bytes, dp, (hipStream_t)stream);
}

int fsk_rdp_epsilon(double clip, double sigma, int64_t releases, double delta, const double* orders,
                    int32_t n_orders, double* eps_out, double* order_out) {
  clear_error();
  if (!(clip > 0.0) || !std::isfinite(clip) || !(sigma > 0.0) || !std::isfinite(sigma))
    return set_error(FSK_EINVAL, "the accountant needs a finite clip radius > 0 and sigma > 0");
  if (releases < 0 || !(delta > 0.0) || !(delta < 1.0))
    return set_error(FSK_EINVAL, "need releases >= 0 and 0 < delta < 1");
  if (!orders || n_orders < 1 || !eps_out) return set_error(FSK_EINVAL, "orders or eps_out is NULL/empty");
  const double sens = 2.0 * clip, per_order = (double)releases * sens * sens / (2.0 * sigma * sigma);
  double best = INFINITY, arg = NAN;
  for (int t = 0; t < n_orders; ++t) {
    const double p = orders[t];
    if (!(p > 1.0)) continue;
    const double eps = per_order * p + std::log(1.0 / delta) / (p - 1.0);
    if (eps < best) { best = eps; arg = p; }
  }
  if (!std::isfinite(best)) return set_error(FSK_EINVAL, "no order above 1 in the grid");
  *eps_out = best;
  if (order_out) *order_out = arg;
  return FSK_OK;
}

// ------------------------------------------------------------- measurement helpers
int fsk_bench_copy(void* dst, const void* src, size_t bytes, void* stream) {
  clear_error();
  if (!dst || !src) return set_error(FSK_EINVAL, "dst or src is NULL");
  if (bytes % 16 != 0 || !aligned16(dst) || !aligned16(src))
    return set_error(FSK_EALIGN, "copy needs 16-byte aligned pointers and size");
  return launch_copy(dst, src, bytes, (hipStream_t)stream);
}

int fsk_bench_read(const void* src, size_t bytes, void* sink, void* stream) {
  clear_error();
  if (!sink || !src) return set_error(FSK_EINVAL, "src or sink is NULL");
  if (bytes % 16 != 0 || !aligned16(src))
    return set_error(FSK_EALIGN, "read needs a 16-byte aligned pointer and size");
  return launch_read(src, bytes, (float*)sink, (hipStream_t)stream);
}

}  // extern "C"
