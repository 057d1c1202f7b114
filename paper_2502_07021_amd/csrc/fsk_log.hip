// Log-domain Sinkhorn on point clouds for gfx950, cost evaluated on the fly (the
// stabilised form the paper names in Sec. 1 / Sec. 2.1, with the kernel applied
// implicitly as in the Remark of Sec. 4.1).  One half-step is
//
//     f_i <- eps ln a_i - eps LSE_j((g_j - ||x_i - y_j||^2)/eps)
//
// and the g-update is the same operation with the two clouds' roles swapped.
//
// Arithmetic.  Everything is moved to base 2 with s = log2(e)/eps and both clouds
// are shifted by their common mean mu (distances do not change):
//
//     s (g_j - C_ij) = beta_j - s|x~_i|^2 + (2 s x~_i) . y~_j,   beta_j = s g_j - s|y~_j|^2
//
// so a pair costs d FMAs.  The expansion cancels badly in fp32 (terms of size
// ~10^3 for a result known to ~10^-5), so the dot product runs in fp64 -- on
// gfx950 a v_fma_f64 issues at the same rate as an unpacked v_fma_f32 -- and only
// the exponential and the running sum are fp32 (v_exp_f32).  The potentials are
// kept in fp64 shadow copies for the whole call; the caller's fp32 arrays are
// read once at the start and written after every update.
//
// Work split.  A workgroup of 256 threads owns 512 rows (two per lane, the rows'
// scaled coordinates live in registers) and one slice of the columns; all four
// waves walk the same columns, whose coordinates arrive through uniform (scalar)
// loads and feed the FMAs straight from scalar registers.  The scalar data cache is the
// scarce resource of this kernel (measured: 100 % busy with one row per lane), so every
// coordinate fetched is used for two rows.  Each lane keeps (reference exponent, sum of 2^(z - reference)); the
// reference is raised lazily, only when a chunk exceeds it by 2^16, so the
// common case has no rescaling and every term that matters is rounded to fp32 at a
// magnitude below 16.  A second kernel merges the column slices in
// fixed order and applies the update.
#include <cmath>
#include <type_traits>

#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

constexpr int kLogRowsPerLane = 2;
constexpr int kLogThreads = 256;
constexpr int kLogRowTile = kLogThreads * kLogRowsPerLane;
constexpr int kLogChunk = 4;          // columns reduced together
constexpr float kLogRaise = 16.0f;    // raise the reference when a chunk exceeds it by this much

// ---------------------------------------------------------------- preparation
// mu[k] = mean over both clouds of coordinate k (fp64, fixed order): every workgroup sums its
// points once for all coordinates (a point's d values are contiguous), a second launch adds
// the workgroups' sums in order.  Any mu would do -- it only centres the clouds -- but a fixed
// order keeps runs reproducible.
constexpr int kLogMeanGroups = 256;

template <typename T, int DP>
__global__ __launch_bounds__(256) void log_mean_partial_kernel(const T* __restrict__ x,
                                                               const T* __restrict__ y, int n, int d,
                                                               double* __restrict__ partial) {
  __shared__ double sm[4][DP];
  double s[DP];
#pragma unroll
  for (int k = 0; k < DP; ++k) s[k] = 0.0;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
#pragma unroll
    for (int k = 0; k < DP; ++k)
      if (k < d) s[k] += (double)x[(int64_t)i * d + k] + (double)y[(int64_t)i * d + k];
  }
#pragma unroll
  for (int k = 0; k < DP; ++k) {
    const double t = wave_sum(s[k]);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6][k] = t;
  }
  __syncthreads();
  if (threadIdx.x < DP)
    partial[(int64_t)blockIdx.x * DP + threadIdx.x] =
        ((sm[0][threadIdx.x] + sm[1][threadIdx.x]) + sm[2][threadIdx.x]) + sm[3][threadIdx.x];
}

// The same for any dp: thread k of a workgroup owns coordinates k, k + 256, ... and walks the
// workgroup's points (g, g + groups, ...) in order.
template <typename T>
__global__ __launch_bounds__(256) void log_mean_partial_generic_kernel(const T* __restrict__ x,
                                                                       const T* __restrict__ y, int n,
                                                                       int d, int dp,
                                                                       double* __restrict__ partial) {
  for (int k = threadIdx.x; k < dp; k += 256) {
    double s = 0.0;
    if (k < d)
      for (int i = blockIdx.x; i < n; i += gridDim.x)
        s += (double)x[(int64_t)i * d + k] + (double)y[(int64_t)i * d + k];
    partial[(int64_t)blockIdx.x * dp + k] = s;
  }
}

__global__ __launch_bounds__(64) void log_mean_final_kernel(const double* __restrict__ partial,
                                                            int groups, int dp, int n,
                                                            double* __restrict__ mu) {
  const int k = blockIdx.x * 64 + threadIdx.x;
  if (k >= dp) return;
  double t = 0.0;
  for (int g = 0; g < groups; ++g) t += partial[(int64_t)g * dp + k];
  mu[k] = t / (2.0 * n);
}

// Per point of one cloud: centred coordinates (column role), 2s-scaled centred
// coordinates (row role), s|p~|^2, ln w, the fp64 shadow potential and its beta.
template <typename T>
__global__ __launch_bounds__(256) void log_prep_kernel(const T* __restrict__ p,
                                                       const T* __restrict__ w,
                                                       const T* __restrict__ pot, int n, int d,
                                                       int dp, double s,
                                                       const double* __restrict__ mu,
                                                       double* __restrict__ pc,
                                                       double* __restrict__ ps,
                                                       double* __restrict__ norm2,
                                                       double* __restrict__ lnw,
                                                       double* __restrict__ potd,
                                                       double* __restrict__ beta) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  double nn = 0.0;
  for (int k = 0; k < dp; ++k) {
    const double c = k < d ? (double)p[(int64_t)i * d + k] - mu[k] : 0.0;
    pc[(int64_t)i * dp + k] = c;
    ps[(int64_t)i * dp + k] = 2.0 * s * c;
    nn += c * c;
  }
  norm2[i] = s * nn;
  lnw[i] = log((double)w[i]);
  const double f = (double)pot[i];
  potd[i] = f;
  beta[i] = s * f - s * nn;
}

// ------------------------------------------------------------------ main kernel
// z0 += sum_k x0[k] q[k], z1 += sum_k x1[k] q[k] for N coordinates, with q taken from scalar
// registers and both rows consuming each coordinate back to back.  Written as one asm block
// because the compiler, left alone, finishes row 0 first and parks the scalar values in
// vector lanes (v_writelane) until row 1 needs them -- more instructions than the FMAs.
template <int N>
__device__ __forceinline__ void fma_rows2(double& z0, double& z1, const double* __restrict__ q,
                                          const double* x0, const double* x1);

template <>
__device__ __forceinline__ void fma_rows2<4>(double& z0, double& z1, const double* __restrict__ q,
                                             const double* x0, const double* x1) {
  asm volatile(
      "v_fmac_f64 %0, %2, %6\n\tv_fmac_f64 %1, %2, %10\n\t"
      "v_fmac_f64 %0, %3, %7\n\tv_fmac_f64 %1, %3, %11\n\t"
      "v_fmac_f64 %0, %4, %8\n\tv_fmac_f64 %1, %4, %12\n\t"
      "v_fmac_f64 %0, %5, %9\n\tv_fmac_f64 %1, %5, %13"
      : "+v"(z0), "+v"(z1)
      : "s"(q[0]), "s"(q[1]), "s"(q[2]), "s"(q[3]), "v"(x0[0]), "v"(x0[1]), "v"(x0[2]), "v"(x0[3]),
        "v"(x1[0]), "v"(x1[1]), "v"(x1[2]), "v"(x1[3])
      : "memory");
}

template <>
__device__ __forceinline__ void fma_rows2<8>(double& z0, double& z1, const double* __restrict__ q,
                                             const double* x0, const double* x1) {
  asm volatile(
      "v_fmac_f64 %0, %2, %10\n\tv_fmac_f64 %1, %2, %18\n\t"
      "v_fmac_f64 %0, %3, %11\n\tv_fmac_f64 %1, %3, %19\n\t"
      "v_fmac_f64 %0, %4, %12\n\tv_fmac_f64 %1, %4, %20\n\t"
      "v_fmac_f64 %0, %5, %13\n\tv_fmac_f64 %1, %5, %21\n\t"
      "v_fmac_f64 %0, %6, %14\n\tv_fmac_f64 %1, %6, %22\n\t"
      "v_fmac_f64 %0, %7, %15\n\tv_fmac_f64 %1, %7, %23\n\t"
      "v_fmac_f64 %0, %8, %16\n\tv_fmac_f64 %1, %8, %24\n\t"
      "v_fmac_f64 %0, %9, %17\n\tv_fmac_f64 %1, %9, %25"
      : "+v"(z0), "+v"(z1)
      : "s"(q[0]), "s"(q[1]), "s"(q[2]), "s"(q[3]), "s"(q[4]), "s"(q[5]), "s"(q[6]), "s"(q[7]),
        "v"(x0[0]), "v"(x0[1]), "v"(x0[2]), "v"(x0[3]), "v"(x0[4]), "v"(x0[5]), "v"(x0[6]),
        "v"(x0[7]), "v"(x1[0]), "v"(x1[1]), "v"(x1[2]), "v"(x1[3]), "v"(x1[4]), "v"(x1[5]),
        "v"(x1[6]), "v"(x1[7])
      : "memory");
}

__device__ __forceinline__ float exp2_of(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ double exp2_of(double x) { return exp2(x); }
__device__ __forceinline__ float max_of(float x, float y) { return fmaxf(x, y); }
__device__ __forceinline__ double max_of(double x, double y) { return fmax(x, y); }

// Adds 2^(zd[t]) for JJ values zd[t] = z_t - mref to the running pair (mref, sum), sum being
// sum of 2^(z - mref).  The reference is raised lazily: only when a value exceeds it by
// kLogRaise, and then exactly (in fp64) to the largest of the JJ values, so that the terms near
// the new maximum are rounded at their final, small magnitude.
template <typename S, int JJ>
__device__ __forceinline__ void lse_fold(const double (&zd)[JJ], double& mref, S& sum) {
  S zf[JJ];
#pragma unroll
  for (int t = 0; t < JJ; ++t) zf[t] = (S)zd[t];
  S cm = zf[0];
#pragma unroll
  for (int t = 1; t < JJ; ++t) cm = max_of(cm, zf[t]);
  if (cm > (S)kLogRaise) {  // rare
    double zmax = zd[0];
#pragma unroll
    for (int t = 1; t < JJ; ++t) zmax = zd[t] > zmax ? zd[t] : zmax;
    mref += zmax;
    sum *= exp2_of(-(S)zmax);
#pragma unroll
    for (int t = 0; t < JJ; ++t) zf[t] = (S)(zd[t] - zmax);
  }
#pragma unroll
  for (int t = 0; t < JJ; ++t) sum += exp2_of(zf[t]);
}

// part_m[sl*n_rows + i], part_s[...]: reference exponent and sum of
// 2^(z_ij - reference) over the columns j of slice sl, z_ij = beta_j + ps_i . qc_j.
// S: type of the exponentials and of the running sum (float for the fp32 interface: one
// v_exp_f32 per pair; double for the fp64 interface).
template <int DP, typename S>
__global__ __launch_bounds__(kLogThreads) void log_lse_kernel(const double* __restrict__ ps,
                                                              const double* __restrict__ qc,
                                                              const double* __restrict__ beta,
                                                              int n_rows, int n_cols,
                                                              int cols_per_slice, int slices,
                                                              double* __restrict__ part_m,
                                                              S* __restrict__ part_s) {
  constexpr int RI = kLogRowsPerLane;
  constexpr int J = kLogChunk;
  const int tid = threadIdx.x;
  const int sl = blockIdx.y;
  const int jb = sl * cols_per_slice;
  const int je = jb + cols_per_slice < n_cols ? jb + cols_per_slice : n_cols;

  double xs[RI][DP];
  int row[RI];
#pragma unroll
  for (int r = 0; r < RI; ++r) {
    row[r] = blockIdx.x * kLogRowTile + r * kLogThreads + tid;
    const int rc = row[r] < n_rows ? row[r] : n_rows - 1;  // clamp; dropped at the store
#pragma unroll
    for (int k = 0; k < DP; ++k) xs[r][k] = ps[(int64_t)rc * DP + k];
  }

  // reference exponent = z of the slice's first column; sums start empty
  double mref[RI];
  S sum[RI];
  {
    const double b0 = beta[jb];
#pragma unroll
    for (int r = 0; r < RI; ++r) {
      double z = b0;
#pragma unroll
      for (int k = 0; k < DP; ++k) z = fma(xs[r][k], qc[(int64_t)jb * DP + k], z);
      mref[r] = z;
      sum[r] = S(0);
    }
  }

  // The column coordinates come through scalar loads, one fetch ahead of the FMAs that use
  // them.  Scalar loads complete out of order, so the only wait is "all of them":
  // the empty asm statement marks the place where the current column must have arrived; the
  // next column is requested right after it and travels while the current column's FMAs run.
  // In the main loop (PIPE) that holds across chunks too: the last column of a chunk requests
  // the first column of the next one (clamped to the last column of the matrix when there is
  // none: a redundant, in-bounds read).
  // A fetch brings at most 16 coordinates (32 scalar registers; two fetches are in flight), so a
  // column of 32 coordinates travels as two parts and its FMAs run part by part.
  constexpr int H = DP > 16 ? 2 : 1;     // fetches per column
  constexpr int QB = DP / H;             // coordinates per fetch: 4, 8, 12 or 16
  double qbuf[2][QB];
  double bj[2];
  auto fetch = [&](int col, int part, int slot) {
    const double* q = qc + (int64_t)col * DP + part * QB;
#pragma unroll
    for (int k = 0; k < QB; ++k) qbuf[slot][k] = q[k];
    bj[slot] = beta[col];
  };

  auto chunk = [&](int j0, auto jj_tag, auto pipe_tag) {
    constexpr int JJ = decltype(jj_tag)::value;
    constexpr bool PIPE = decltype(pipe_tag)::value;
    static_assert(RI == 2, "fma_rows2 carries exactly two rows per lane");
    static_assert(!PIPE || (JJ * H) % 2 == 0, "a pipelined chunk must hand slot 0 to its successor");
    double zd[RI][JJ];
    double z[RI];
    if (!PIPE) fetch(j0, 0, 0);
#pragma unroll
    for (int t = 0; t < JJ * H; ++t) {  // unit t: part t % H of column t / H
      const int slot = t & 1, col = t / H, part = t % H;
#pragma unroll
      for (int k0 = 0; k0 < QB; k0 += 4)  // "use" every scalar of this unit: forces the wait here
        asm volatile("" : : "s"(qbuf[slot][k0]), "s"(qbuf[slot][k0 + 1]), "s"(qbuf[slot][k0 + 2]),
                     "s"(qbuf[slot][k0 + 3]), "s"(bj[slot]) : "memory");
      if (t + 1 < JJ * H) {
        fetch(j0 + (t + 1) / H, (t + 1) % H, slot ^ 1);
      } else if (PIPE) {
        const int nxt = j0 + JJ < n_cols ? j0 + JJ : n_cols - 1;
        fetch(nxt, 0, slot ^ 1);
      }
      if (part == 0) {
#pragma unroll
        for (int r = 0; r < RI; ++r) z[r] = bj[slot] - mref[r];
      }
#pragma unroll
      for (int k0 = 0; k0 < QB; k0 += 8) {  // FMA blocks of 8 coordinates, a last one of 4
        if (QB - k0 >= 8)
          fma_rows2<8>(z[0], z[1], &qbuf[slot][k0], &xs[0][part * QB + k0], &xs[1][part * QB + k0]);
        else
          fma_rows2<4>(z[0], z[1], &qbuf[slot][k0], &xs[0][part * QB + k0], &xs[1][part * QB + k0]);
      }
      if (part == H - 1) {
#pragma unroll
        for (int r = 0; r < RI; ++r) zd[r][col] = z[r];
      }
    }
#pragma unroll
    for (int r = 0; r < RI; ++r) lse_fold<S, JJ>(zd[r], mref[r], sum[r]);
  };

  int j = jb;
  if (j + J <= je) fetch(j, 0, 0);
  for (; j + J <= je; j += J) chunk(j, std::integral_constant<int, J>{}, std::true_type{});
  for (; j < je; ++j) chunk(j, std::integral_constant<int, 1>{}, std::false_type{});

#pragma unroll
  for (int r = 0; r < RI; ++r) {
    if (row[r] < n_rows) {
      part_m[(int64_t)sl * n_rows + row[r]] = mref[r];
      part_s[(int64_t)sl * n_rows + row[r]] = sum[r];
    }
  }
}

// The same for any point dimension (dp a multiple of 8): the rows' coordinates do not stay in
// registers but are re-read (cache hits) block of 8 coordinates by block of 8 for every chunk
// of 8 columns, whose coordinates are uniform loads.  Far from the tuned kernel's rate; it
// exists so that the dimension is not a limit of the interface.
template <typename S>
__global__ __launch_bounds__(kLogThreads) void log_lse_generic_kernel(const double* __restrict__ ps,
                                                                      const double* __restrict__ qc,
                                                                      const double* __restrict__ beta,
                                                                      int n_rows, int n_cols, int dp,
                                                                      int cols_per_slice, int slices,
                                                                      double* __restrict__ part_m,
                                                                      S* __restrict__ part_s) {
  constexpr int RI = kLogRowsPerLane;
  constexpr int J = 8, KB = 8;
  const int tid = threadIdx.x;
  const int sl = blockIdx.y;
  const int jb = sl * cols_per_slice;
  const int je = jb + cols_per_slice < n_cols ? jb + cols_per_slice : n_cols;
  int row[RI];
  const double* xrow[RI];
#pragma unroll
  for (int r = 0; r < RI; ++r) {
    row[r] = blockIdx.x * kLogRowTile + r * kLogThreads + tid;
    const int rc = row[r] < n_rows ? row[r] : n_rows - 1;  // clamp; dropped at the store
    xrow[r] = ps + (int64_t)rc * dp;
  }
  // z of JJ columns starting at j0 for both rows, relative to each row's reference
  auto dots = [&](int j0, auto jj_tag, double (&zd)[RI][J], const double (&mref)[RI]) {
    constexpr int JJ = decltype(jj_tag)::value;
#pragma unroll
    for (int t = 0; t < JJ; ++t) {
      const double bj = beta[j0 + t];
#pragma unroll
      for (int r = 0; r < RI; ++r) zd[r][t] = bj - mref[r];
    }
    for (int k0 = 0; k0 < dp; k0 += KB) {
      double xs[RI][KB];
#pragma unroll
      for (int r = 0; r < RI; ++r)
#pragma unroll
        for (int k = 0; k < KB; ++k) xs[r][k] = xrow[r][k0 + k];
#pragma unroll
      for (int t = 0; t < JJ; ++t) {
        const double* q = qc + (int64_t)(j0 + t) * dp + k0;
#pragma unroll
        for (int k = 0; k < KB; ++k) {
          const double qk = q[k];
#pragma unroll
          for (int r = 0; r < RI; ++r) zd[r][t] = fma(xs[r][k], qk, zd[r][t]);
        }
      }
    }
  };

  double mref[RI] = {};
  S sum[RI];
  double zd[RI][J];
  dots(jb, std::integral_constant<int, 1>{}, zd, mref);  // reference = z of the slice's first column
#pragma unroll
  for (int r = 0; r < RI; ++r) {
    mref[r] = zd[r][0];
    sum[r] = S(0);
  }
  int j = jb;
  for (; j + J <= je; j += J) {
    dots(j, std::integral_constant<int, J>{}, zd, mref);
#pragma unroll
    for (int r = 0; r < RI; ++r) lse_fold<S, J>(zd[r], mref[r], sum[r]);
  }
  for (; j < je; ++j) {
    dots(j, std::integral_constant<int, 1>{}, zd, mref);
#pragma unroll
    for (int r = 0; r < RI; ++r) {
      const double one[1] = {zd[r][0]};
      lse_fold<S, 1>(one, mref[r], sum[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < RI; ++r) {
    if (row[r] < n_rows) {
      part_m[(int64_t)sl * n_rows + row[r]] = mref[r];
      part_s[(int64_t)sl * n_rows + row[r]] = sum[r];
    }
  }
}

// ------------------------------------------------------------------ merge + update
// L2_i = log2 sum_j 2^(z_ij) from the slices (merged in a fixed order), then
//   pot_new = eps (ln w_i - ln2 (L2_i - s|p~_i|^2)).
// mode 0: store pot_new (fp64 shadow, caller's array, beta for the column role).
// mode 1: store |w_i exp((pot_i - pot_new)/eps) - w_i| -- the row-marginal error of the
//         plan exp((f_i + g_j - C_ij)/eps) with the potentials as they stand.
// mode 2: both (the error terms of the state before this update come for free with it).
template <typename T, typename TS>
__global__ __launch_bounds__(256) void log_finalize_kernel(const double* __restrict__ part_m,
                                                           const TS* __restrict__ part_s,
                                                           int slices, int n,
                                                           const double* __restrict__ norm2,
                                                           const double* __restrict__ lnw, double eps,
                                                           double s, int mode, double eta, int geometric,
                                                           double* potd,
                                                           T* __restrict__ pot_out,
                                                           double* __restrict__ beta_out,
                                                           double* __restrict__ errvec) {
  // Four adjacent lanes share a row: lane g merges slices g, g + 4, ... (a thread alone would
  // walk all slices with nothing to hide the latency of its loads and fp64 exponentials: one wave
  // per SIMD), then the four agree on the largest reference and add their sums pairwise, in the
  // same order in every launch.
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int g = t & 3;
  const bool live = (t >> 2) < n;
  const int i = live ? t >> 2 : n - 1;  // lanes past the end stay in the exchanges, store nothing
  double M = -__builtin_huge_val();
  for (int k = g; k < slices; k += 4) {
    const double m = part_m[(int64_t)k * n + i];
    M = m > M ? m : M;
  }
  double other = lane_xor_dpp<1>(M);
  M = other > M ? other : M;
  other = lane_xor_dpp<2>(M);
  M = other > M ? other : M;
  double S = 0.0;
  for (int k = g; k < slices; k += 4)
    S += (double)part_s[(int64_t)k * n + i] * exp2(part_m[(int64_t)k * n + i] - M);
  S += lane_xor_dpp<1>(S);
  S += lane_xor_dpp<2>(S);
  if (!live || g != 0) return;
  const double L2 = M + log2(S);
  const double ln2 = 0.693147180559945309417;
  const double pot_new = eps * (lnw[i] - ln2 * (L2 - norm2[i]));
  if (mode != 0) {  // before potd is overwritten: the error term belongs to the potentials as they stand
    const double w = exp(lnw[i]);
    errvec[i] = fabs(w * exp((potd[i] - pot_new) / eps) - w);
  }
  if (mode != 1) {
    // relaxed updates of Sec. 3.3 (eta < 1): geometric = linear in the potential; arithmetic =
    // eps log((1 - eta) e^(old/eps) + eta e^(new/eps)) with the larger exponent taken out
    double keep = pot_new;
    if (eta < 1.0) {
      const double old = potd[i];
      if (geometric) {
        keep = (1.0 - eta) * old + eta * pot_new;
      } else {
        const double top = old > pot_new ? old : pot_new;
        keep = top + eps * log((1.0 - eta) * exp((old - top) / eps) + eta * exp((pot_new - top) / eps));
      }
    }
    potd[i] = keep;
    pot_out[i] = (T)keep;
    beta_out[i] = s * keep - norm2[i];
  }
}

// ------------------------------------------------------------------ host side
struct LogWs {
  int dp, slices, cols_per_slice;
  size_t mu, mpart, xc, xs, yc, ys, nx2, ny2, lna, lnb, fd, gd, bx, by, pm, psum, err, scalar, save, total;
};

constexpr int kLogMaxDim = 4096;
// Padded dimension: 4, 8, 12, 16, 24, 32 select the register-resident kernel, larger multiples of 8 the
// generic one; 0 = not supported.
static int log_pad_dim(int d) {
  if (d < 1 || d > kLogMaxDim) return 0;
  return d <= 4 ? 4 : d <= 8 ? 8 : d <= 12 ? 12 : d <= 16 ? 16 : d <= 24 ? 24 : d <= 32 ? 32 : (d + 7) / 8 * 8;
}

static LogWs log_ws(int n, int d) {
  LogWs w{};
  w.dp = log_pad_dim(d);
  // Column slices per row tile: 40, at least 256 columns each.  Measured on MI355X (ms per
  // half-step, d = 16): n = 65536: 2.87 / 2.85 / 2.78 / 2.72 / 2.73 / 2.75 / 2.84 with 16 / 20 / 30 /
  // 40 / 50 / 64 / 128 slices (3.14 with 10, which is one full round of resident workgroups);
  // n = 131072: 11.8 / 10.9 / 10.7 / 10.7 with 8 / 20 / 30 / 40; n = 32768: 0.766 / 0.756 / 0.768 with
  // 32 / 40 / 80; d = 8, 32 and 3 agree (40-48 best).  Many short workgroups that start at
  // different times keep the vector unit fed through each other's ramps and tails; beyond ~50
  // the per-slice ramp and the merge of the slices cost more than that gains.
  constexpr int kLogSlices = 40;
  const int max_by_cols = n / 256 > 0 ? n / 256 : 1;
  const int slices = kLogSlices < max_by_cols ? kLogSlices : max_by_cols;
  w.cols_per_slice = ((n + slices - 1) / slices + kLogChunk - 1) / kLogChunk * kLogChunk;
  w.slices = (n + w.cols_per_slice - 1) / w.cols_per_slice;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  const size_t nd = (size_t)n * (size_t)(w.dp ? w.dp : 1) * 8, nv = (size_t)n * 8;
  w.mu = take((size_t)(w.dp > 32 ? w.dp : 32) * 8);
  w.mpart = take((size_t)kLogMeanGroups * (size_t)(w.dp ? w.dp : 1) * 8);  // per-workgroup coordinate sums
  w.xc = take(nd); w.xs = take(nd); w.yc = take(nd); w.ys = take(nd);
  w.nx2 = take(nv); w.ny2 = take(nv); w.lna = take(nv); w.lnb = take(nv);
  w.fd = take(nv); w.gd = take(nv); w.bx = take(nv); w.by = take(nv);
  w.pm = take(nv * w.slices); w.psum = take(nv * w.slices);  // sums: fp32 or fp64
  w.err = take(nv); w.scalar = take(256);
  w.save = take(6 * align_up(nv, 256));  // f, g, their fp64 shadows and betas at a polled state
  w.total = off;
  return w;
}

size_t log_workspace_bytes(int n, int d) { return log_pad_dim(d) ? log_ws(n, d).total : 0; }

template <int DP, typename S>
static int launch_lse(const LogWs& w, int n, const double* ps, const double* qc, const double* beta,
                      double* pm, S* psum, hipStream_t st) {
  dim3 grid((n + kLogRowTile - 1) / kLogRowTile, w.slices), block(kLogThreads);
  hipLaunchKernelGGL((log_lse_kernel<DP, S>), grid, block, 0, st, ps, qc, beta, n, n,
                     w.cols_per_slice, w.slices, pm, psum);
  FSK_LAUNCH_CHECK("log_lse_kernel");
  return FSK_OK;
}

template <typename S>
static int lse_dispatch(const LogWs& w, int n, const double* ps, const double* qc,
                        const double* beta, double* pm, S* psum, hipStream_t st) {
  switch (w.dp) {
    case 4: return launch_lse<4, S>(w, n, ps, qc, beta, pm, psum, st);
    case 8: return launch_lse<8, S>(w, n, ps, qc, beta, pm, psum, st);
    case 12: return launch_lse<12, S>(w, n, ps, qc, beta, pm, psum, st);
    case 16: return launch_lse<16, S>(w, n, ps, qc, beta, pm, psum, st);
    case 24: return launch_lse<24, S>(w, n, ps, qc, beta, pm, psum, st);
    case 32: return launch_lse<32, S>(w, n, ps, qc, beta, pm, psum, st);
    default: {
      dim3 grid((n + kLogRowTile - 1) / kLogRowTile, w.slices), block(kLogThreads);
      hipLaunchKernelGGL((log_lse_generic_kernel<S>), grid, block, 0, st, ps, qc, beta, n, n, w.dp,
                         w.cols_per_slice, w.slices, pm, psum);
      FSK_LAUNCH_CHECK("log_lse_generic_kernel");
      return FSK_OK;
    }
  }
}

template <typename T>
static int run_log_typed(const fsk_opts* o, const void* x, const void* y, int d, double eps,
                         const void* a, const void* b, void* f, void* g, void* workspace,
                         size_t ws_bytes, int32_t* iters_done, double* err_out, hipStream_t st) {
  const int n = o->n;
  const LogWs w = log_ws(n, d);
  if (!workspace || ws_bytes < w.total)
    return set_error(FSK_EWORKSPACE, "log-domain call needs %zu workspace bytes, got %zu", w.total, ws_bytes);
  char* ws = (char*)workspace;
  auto D = [&](size_t off) { return (double*)(ws + off); };
  const double s = 1.4426950408889634074 / eps;
  const double eta = o->damping == FSK_DAMP_NONE ? 1.0 : o->eta;
  const int geometric = o->damping == FSK_DAMP_GEOMETRIC ? 1 : 0;
  const T *xf = (const T*)x, *yf = (const T*)y, *af = (const T*)a, *bf = (const T*)b;
  T *ff = (T*)f, *gf = (T*)g;
  const int nb = (n + 255) / 256;

  {
    int groups = (n + 255) / 256;
    if (groups > kLogMeanGroups) groups = kLogMeanGroups;
    double* part = D(w.mpart);
    switch (w.dp) {
      case 4: hipLaunchKernelGGL((log_mean_partial_kernel<T, 4>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, part); break;
      case 8: hipLaunchKernelGGL((log_mean_partial_kernel<T, 8>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, part); break;
      case 12: hipLaunchKernelGGL((log_mean_partial_kernel<T, 12>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, part); break;
      case 16: hipLaunchKernelGGL((log_mean_partial_kernel<T, 16>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, part); break;
      case 24: hipLaunchKernelGGL((log_mean_partial_kernel<T, 24>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, part); break;
      case 32: hipLaunchKernelGGL((log_mean_partial_kernel<T, 32>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, part); break;
      default: hipLaunchKernelGGL((log_mean_partial_generic_kernel<T>), dim3(groups), dim3(256), 0, st, xf, yf, n, d, w.dp, part); break;
    }
    FSK_LAUNCH_CHECK("log_mean_partial_kernel");
    hipLaunchKernelGGL(log_mean_final_kernel, dim3((w.dp + 63) / 64), dim3(64), 0, st, (const double*)part, groups, w.dp, n, D(w.mu));
    FSK_LAUNCH_CHECK("log_mean_final_kernel");
  }
  hipLaunchKernelGGL((log_prep_kernel<T>), dim3(nb), dim3(256), 0, st, xf, af, ff, n, d, w.dp, s,
                     D(w.mu), D(w.xc), D(w.xs), D(w.nx2), D(w.lna), D(w.fd), D(w.bx));
  FSK_LAUNCH_CHECK("log_prep_kernel");
  hipLaunchKernelGGL((log_prep_kernel<T>), dim3(nb), dim3(256), 0, st, yf, bf, gf, n, d, w.dp, s,
                     D(w.mu), D(w.yc), D(w.ys), D(w.ny2), D(w.lnb), D(w.gd), D(w.by));
  FSK_LAUNCH_CHECK("log_prep_kernel");

  T* psum = (T*)(ws + w.psum);  // the exponentials and their sums run in the interface type
  auto half_step = [&](bool f_side, int mode) -> int {
    // f-update: rows = x (scaled), columns = y with beta_y; g-update: the roles swapped
    FSK_TRY(lse_dispatch<T>(w, n, D(f_side ? w.xs : w.ys), D(f_side ? w.yc : w.xc),
                            D(f_side ? w.by : w.bx), D(w.pm), psum, st));
    hipLaunchKernelGGL((log_finalize_kernel<T, T>), dim3((n + 63) / 64), dim3(256), 0, st, D(w.pm), psum,
                       w.slices, n, D(f_side ? w.nx2 : w.ny2), D(f_side ? w.lna : w.lnb), eps, s,
                       mode, eta, geometric, D(f_side ? w.fd : w.gd), f_side ? ff : gf,
                       D(f_side ? w.bx : w.by),
                       D(w.err));
    FSK_LAUNCH_CHECK("log_finalize_kernel");
    return FSK_OK;
  };

  // Tolerance mode: the f-update of iteration it + 1 evaluates the LSE with the potentials of
  // the state after `it` iterations, so that state's error terms come with it (mode 2); a poll
  // costs a few n-vector copies, a sum and a synchronisation.  If the state met the tolerance
  // the iteration that revealed it is undone from the saved copies.
  const size_t tb = (size_t)n * sizeof(T), db = (size_t)n * 8;
  char* sv = ws + w.save;
  char* keep[6] = {(char*)ff, (char*)gf, (char*)D(w.fd), (char*)D(w.gd), (char*)D(w.bx), (char*)D(w.by)};
  const size_t keep_bytes[6] = {tb, tb, db, db, db, db};
  auto copy_state = [&](bool restore) -> int {
    size_t off = 0;
    for (int k = 0; k < 6; ++k) {
      FSK_HIP(hipMemcpyAsync(restore ? keep[k] : sv + off, restore ? sv + off : keep[k], keep_bytes[k],
                             hipMemcpyDeviceToDevice, st));
      off += align_up(db, 256);
    }
    return FSK_OK;
  };
  const bool l2 = o->err_norm == FSK_NORM_L2;  // ||P1 - a||_2 instead of the 1-norm
  auto read_error = [&](double* out) -> int {
    FSK_TRY(launch_sum_to_double(FSK_F64, D(w.err), n, D(w.scalar), st, l2));
    FSK_HIP(hipMemcpyAsync(out, D(w.scalar), sizeof(double), hipMemcpyDeviceToHost, st));
    FSK_HIP(hipStreamSynchronize(st));
    if (l2) *out = sqrt(*out);
    return FSK_OK;
  };
  auto nonfinite = [&](int at, double e) {
    if (iters_done) *iters_done = at;
    if (err_out) *err_out = e;
    return set_error(FSK_ENONFINITE, "marginal error is not finite after %d iterations", at);
  };

  int done = 0;
  double e = NAN;
  bool converged = false;
  if (o->tol > 0.0) trace_begin();
  for (int it = 0; it < o->max_iters; ++it) {
    const bool poll = o->tol > 0.0 && it > 0 && it % o->check_every == 0;
    if (poll) FSK_TRY(copy_state(false));
    FSK_TRY(half_step(true, poll ? 2 : 0));
    FSK_TRY(half_step(false, 0));
    if (poll) {
      FSK_TRY(read_error(&e));
      trace_poll(it, e);
      if (!std::isfinite(e)) {  // hand back the polled state itself, not the one advanced past it
        FSK_TRY(copy_state(true));
        FSK_HIP(hipStreamSynchronize(st));
        return nonfinite(it, e);
      }
      if (e < o->tol) {
        FSK_TRY(copy_state(true));
        FSK_HIP(hipStreamSynchronize(st));
        done = it;
        converged = true;
        break;
      }
    }
    done = it + 1;
  }
  if (o->tol > 0.0 && !converged && done > 0) {  // the state after the last iteration is always polled
    FSK_TRY(half_step(true, 1));
    FSK_TRY(read_error(&e));
    trace_poll(done, e);
    if (!std::isfinite(e)) return nonfinite(done, e);
  }
  if (iters_done) *iters_done = done;
  if (err_out) *err_out = e;
  return FSK_OK;
}

int run_sinkhorn_log_points(const fsk_opts* o, const void* x, const void* y, int d, double eps,
                            const void* a, const void* b, void* f, void* g, void* workspace,
                            size_t ws_bytes, int32_t* iters_done, double* err_out,
                            hipStream_t st) {
  if (log_pad_dim(d) == 0)
    return set_error(FSK_EUNSUPPORTED, "point dimension %d is outside 1..%d", d, kLogMaxDim);
  return o->dtype == FSK_F64
             ? run_log_typed<double>(o, x, y, d, eps, a, b, f, g, workspace, ws_bytes, iters_done, err_out, st)
             : run_log_typed<float>(o, x, y, d, eps, a, b, f, g, workspace, ws_bytes, iters_done, err_out, st);
}

}  // namespace fsk
