// Setup kernels (off the timed loop): the Gibbs kernel K = exp(-C/eps) of Sec. 1
// from a stored cost matrix or from two point clouds with the squared Euclidean
// cost of Sec. 5.6, plus the plain copy / read kernels used for measurement.
//
// The arithmetic is done in fp64 whatever the storage type and rounded once on
// the store, so an fp32 K holds (up to the last place of the fp64 exp) the
// rounded exact value: the iteration then starts from the same kernel a
// double-precision evaluation would give.
#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

template <typename T>
__global__ __launch_bounds__(256) void gibbs_from_cost_kernel(const T* C, int64_t ldC, int n,
                                                              double eps, T* K, int64_t ldK) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int i = blockIdx.y;
  if (j < n) K[(int64_t)i * ldK + j] = (T)exp(-(double)C[(int64_t)i * ldC + j] / eps);
}

int launch_gibbs_from_cost(int dtype, const void* C, int64_t ldC, int n, double eps, void* K,
                           int64_t ldK, hipStream_t stream) {
  dim3 grid((n + 255) / 256, n), block(256);
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((gibbs_from_cost_kernel<double>), grid, block, 0, stream, (const double*)C,
                       ldC, n, eps, (double*)K, ldK);
  else
    hipLaunchKernelGGL((gibbs_from_cost_kernel<float>), grid, block, 0, stream, (const float*)C,
                       ldC, n, eps, (float*)K, ldK);
  FSK_LAUNCH_CHECK("gibbs_from_cost_kernel");
  return FSK_OK;
}

// K_ij = exp(-(lambda c_ij - l_j)/eps): the kernel of the combined cost of the robust-risk
// example (paper: Sec. "Illustrative application").  l may be null (taken as zero).
template <typename T>
__global__ __launch_bounds__(256) void gibbs_lambda_kernel(const T* c, int64_t ldc, int n,
                                                           double lambda, const T* l, double eps,
                                                           T* K, int64_t ldK) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int i = blockIdx.y;
  if (j < n) {
    const double lj = l ? (double)l[j] : 0.0;
    K[(int64_t)i * ldK + j] = (T)exp(-(lambda * (double)c[(int64_t)i * ldc + j] - lj) / eps);
  }
}

int launch_gibbs_lambda(int dtype, const void* c, int64_t ldc, int n, double lambda, const void* l,
                        double eps, void* K, int64_t ldK, hipStream_t stream) {
  dim3 grid((n + 255) / 256, n), block(256);
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((gibbs_lambda_kernel<double>), grid, block, 0, stream, (const double*)c, ldc,
                       n, lambda, (const double*)l, eps, (double*)K, ldK);
  else
    hipLaunchKernelGGL((gibbs_lambda_kernel<float>), grid, block, 0, stream, (const float*)c, ldc, n,
                       lambda, (const float*)l, eps, (float*)K, ldK);
  FSK_LAUNCH_CHECK("gibbs_lambda_kernel");
  return FSK_OK;
}

template <typename T>
__global__ __launch_bounds__(256) void fill_kernel(T* x, int n, T value) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) x[i] = value;
}

int launch_fill(int dtype, void* x, int n, double value, hipStream_t stream) {
  dim3 grid((n + 255) / 256), block(256);
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((fill_kernel<double>), grid, block, 0, stream, (double*)x, n, value);
  else
    hipLaunchKernelGGL((fill_kernel<float>), grid, block, 0, stream, (float*)x, n, (float)value);
  FSK_LAUNCH_CHECK("fill_kernel");
  return FSK_OK;
}

// Tile of 16 rows x 256 columns per workgroup; thread t owns column j and keeps
// y_j in registers/cache while it walks the 16 rows (x_i entries are uniform
// loads).  MODE 0: running maximum of the cost; MODE 1: write K.
constexpr int kSetupRows = 16;

template <typename T>
__device__ __forceinline__ double sqdist(const T* __restrict__ xi, const T* __restrict__ yj, int d) {
  double s = 0.0;
  for (int k = 0; k < d; ++k) {
    const double t = (double)xi[k] - (double)yj[k];
    s += t * t;
  }
  return s;
}

// The same sum with y_j already in registers (DP >= d values, zero padded) and the terms in
// the same order, so that both forms round alike.
template <typename T, int DP>
__device__ __forceinline__ double sqdist_reg(const T* __restrict__ xi, const double (&yj)[DP], int d) {
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < DP; ++k)
    if (k < d) {
      const double t = (double)xi[k] - yj[k];
      s += t * t;
    }
  return s;
}

template <typename T, int DP>
__device__ __forceinline__ void load_point(const T* __restrict__ p, int d, double (&out)[DP]) {
#pragma unroll
  for (int k = 0; k < DP; ++k) out[k] = k < d ? (double)p[k] : 0.0;
}

// DP > 0: d <= DP and y_j is held in registers for the tile's 16 rows; DP == 0: any d, y_j
// re-read per row.
template <typename T, int DP>
__global__ __launch_bounds__(256) void max_sqdist_kernel(const T* __restrict__ x,
                                                         const T* __restrict__ y, int n, int d,
                                                         double* __restrict__ wg_max) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int i0 = blockIdx.y * kSetupRows;
  double m = 0.0;
  if (j < n) {
    double yj[DP > 0 ? DP : 1];
    if (DP > 0) load_point<T, (DP > 0 ? DP : 1)>(y + (int64_t)j * d, d, yj);
    for (int r = 0; r < kSetupRows; ++r) {
      const int i = i0 + r;
      if (i < n) {
        const double s = DP > 0 ? sqdist_reg<T, (DP > 0 ? DP : 1)>(x + (int64_t)i * d, yj, d)
                                : sqdist(x + (int64_t)i * d, y + (int64_t)j * d, d);
        m = s > m ? s : m;
      }
    }
  }
  m = wave_max(m);
  __shared__ double sm[4];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = sm[0];
    for (int k = 1; k < 4; ++k) t = sm[k] > t ? sm[k] : t;
    wg_max[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(1024) void max_reduce_kernel(const double* __restrict__ x, int64_t cnt,
                                                          double* out) {
  double m = 0.0;
  for (int64_t i = threadIdx.x; i < cnt; i += 1024) m = x[i] > m ? x[i] : m;
  m = wave_max(m);
  __shared__ double sm[16];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = sm[0];
    for (int k = 1; k < 16; ++k) t = sm[k] > t ? sm[k] : t;
    *out = t;
  }
}

size_t max_sqdist_scratch_doubles(int n) {
  return (size_t)((n + 255) / 256) * (size_t)((n + kSetupRows - 1) / kSetupRows);
}

int launch_max_sqdist(int dtype, const void* x, const void* y, int n, int d, double* scratch,
                      size_t scratch_doubles, double* cmax_dev, hipStream_t stream) {
  const size_t need = max_sqdist_scratch_doubles(n);
  if (scratch_doubles < need) return set_error(FSK_EWORKSPACE, "max-cost scratch too small");
  dim3 grid((n + 255) / 256, (n + kSetupRows - 1) / kSetupRows), block(256);
#define FSK_MAXSQ(TT, DPV)                                                                        \
  hipLaunchKernelGGL((max_sqdist_kernel<TT, DPV>), grid, block, 0, stream, (const TT*)x,         \
                     (const TT*)y, n, d, scratch)
  if (dtype == FSK_F64) {
    if (d <= 4) FSK_MAXSQ(double, 4); else if (d <= 8) FSK_MAXSQ(double, 8);
    else if (d <= 16) FSK_MAXSQ(double, 16); else if (d <= 32) FSK_MAXSQ(double, 32);
    else FSK_MAXSQ(double, 0);
  } else {
    if (d <= 4) FSK_MAXSQ(float, 4); else if (d <= 8) FSK_MAXSQ(float, 8);
    else if (d <= 16) FSK_MAXSQ(float, 16); else if (d <= 32) FSK_MAXSQ(float, 32);
    else FSK_MAXSQ(float, 0);
  }
#undef FSK_MAXSQ
  FSK_LAUNCH_CHECK("max_sqdist_kernel");
  hipLaunchKernelGGL(max_reduce_kernel, dim3(1), dim3(1024), 0, stream, scratch, (int64_t)need,
                     cmax_dev);
  FSK_LAUNCH_CHECK("max_reduce_kernel");
  return FSK_OK;
}

template <typename T, int DP>
__global__ __launch_bounds__(256) void gibbs_from_points_kernel(const T* __restrict__ x,
                                                                const T* __restrict__ y, int n,
                                                                int d, double eps,
                                                                const double* __restrict__ cmax_dev,
                                                                T* __restrict__ K, int64_t ldK) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int i0 = blockIdx.y * kSetupRows;
  const double cmax = cmax_dev ? *cmax_dev : 1.0;
  if (j >= n) return;
  double yj[DP > 0 ? DP : 1];
  if (DP > 0) load_point<T, (DP > 0 ? DP : 1)>(y + (int64_t)j * d, d, yj);
  for (int r = 0; r < kSetupRows; ++r) {
    const int i = i0 + r;
    if (i < n) {
      const double s = DP > 0 ? sqdist_reg<T, (DP > 0 ? DP : 1)>(x + (int64_t)i * d, yj, d)
                              : sqdist(x + (int64_t)i * d, y + (int64_t)j * d, d);
      K[(int64_t)i * ldK + j] = (T)exp(-(s / cmax) / eps);
    }
  }
}

int launch_gibbs_from_points(int dtype, const void* x, const void* y, int n, int d, double eps,
                             const double* cmax_dev, void* K, int64_t ldK, hipStream_t stream) {
  dim3 grid((n + 255) / 256, (n + kSetupRows - 1) / kSetupRows), block(256);
#define FSK_GIBBS(TT, DPV)                                                                        \
  hipLaunchKernelGGL((gibbs_from_points_kernel<TT, DPV>), grid, block, 0, stream, (const TT*)x,  \
                     (const TT*)y, n, d, eps, cmax_dev, (TT*)K, ldK)
  if (dtype == FSK_F64) {
    if (d <= 4) FSK_GIBBS(double, 4); else if (d <= 8) FSK_GIBBS(double, 8);
    else if (d <= 16) FSK_GIBBS(double, 16); else if (d <= 32) FSK_GIBBS(double, 32);
    else FSK_GIBBS(double, 0);
  } else {
    if (d <= 4) FSK_GIBBS(float, 4); else if (d <= 8) FSK_GIBBS(float, 8);
    else if (d <= 16) FSK_GIBBS(float, 16); else if (d <= 32) FSK_GIBBS(float, 32);
    else FSK_GIBBS(float, 0);
  }
#undef FSK_GIBBS
  FSK_LAUNCH_CHECK("gibbs_from_points_kernel");
  return FSK_OK;
}

// ------------------------------------------------------------ measurement helpers
// Grid-stride 128-bit copy: the reference stream for byte counters and for the
// achievable HBM rate.
__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src,
                                                   float4* __restrict__ dst, size_t nvec) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

int launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t nvec = bytes / 16;
  if (nvec == 0) return FSK_OK;
  size_t wgs = (nvec + 255) / 256;
  const size_t cap = (size_t)device_cu_count() * 32;
  if (wgs > cap) wgs = cap;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)wgs), dim3(256), 0, stream, (const float4*)src,
                     (float4*)dst, nvec);
  FSK_LAUNCH_CHECK("copy_kernel");
  return FSK_OK;
}

// Read-only stream: every workgroup sums what it reads and stores one float.
__global__ __launch_bounds__(256) void read_kernel(const float4* __restrict__ src, size_t nvec,
                                                   float* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  float s = 0.f;
#pragma unroll 4
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
    const float4 p = src[i];
    s += (p.x + p.y) + (p.z + p.w);
  }
  s = wave_sum(s);
  __shared__ float sm[4];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

int launch_read(const void* src, size_t bytes, float* sink, hipStream_t stream) {
  const size_t nvec = bytes / 16;
  if (nvec == 0) return FSK_OK;
  size_t wgs = (nvec + 255) / 256;
  size_t cap = (size_t)device_cu_count() * 16;
  if (cap > 4096) cap = 4096;
  if (wgs > cap) wgs = cap;
  hipLaunchKernelGGL(read_kernel, dim3((unsigned)wgs), dim3(256), 0, stream, (const float4*)src,
                     nvec, sink);
  FSK_LAUNCH_CHECK("read_kernel");
  return FSK_OK;
}

}  // namespace fsk
