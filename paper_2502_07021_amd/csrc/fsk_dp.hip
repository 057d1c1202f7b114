// Privacy layer for gfx950 (paper: privacy appendix, "Gaussian noise on log-domain scalings"):
// after an update the n x m scalings are released as exp(clip_S(log X) + sigma N(0, I)), the
// clip being a row-wise l2 clip across the m targets.
//
// The normal numbers come from a counter-based generator so that a release can be reproduced
// from (seed, release index, element index) alone, on any grid: Philox4x32-10 (Salmon et al.,
// SC'11) keyed by the seed, counter = (call index, release index), four 32-bit words per call,
// turned into four normals by two Box-Muller transforms in fp64.  Element e of a release uses
// word pair (e % 4) / 2 of call e / 4.
//
// A row is shared by up to 64 threads of one wave (4 elements, i.e. one generator call, per
// thread and step); the row's values are walked twice (norm of the log-scalings, reduced over
// the row's threads in a fixed butterfly, then the release), everything in fp64 with one
// rounding on the store.  The matrices are a few MiB; the kernel is a small fraction of an
// iteration.
#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

struct PhiloxBlock { uint32_t w[4]; };

__device__ __forceinline__ PhiloxBlock philox4x32_10(uint64_t call, uint64_t release, uint64_t seed) {
  uint32_t c[4] = {(uint32_t)call, (uint32_t)(call >> 32), (uint32_t)release, (uint32_t)(release >> 32)};
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t lo0 = 0xD2511F53u * c[0], hi0 = __umulhi(0xD2511F53u, c[0]);
    const uint32_t lo1 = 0xCD9E8D57u * c[2], hi1 = __umulhi(0xCD9E8D57u, c[2]);
    const uint32_t a = hi1 ^ c[1] ^ k0, b = hi0 ^ c[3] ^ k1;
    c[0] = a; c[1] = lo1; c[2] = b; c[3] = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  PhiloxBlock out;
#pragma unroll
  for (int t = 0; t < 4; ++t) out.w[t] = c[t];
  return out;
}

// Normal number (e % 4) of a call's block.
__device__ __forceinline__ double block_normal(const PhiloxBlock& blk, int which) {
  const int pair = which >> 1;
  const double u1 = ((double)blk.w[2 * pair] + 0.5) * 0x1p-32;
  const double u2 = ((double)blk.w[2 * pair + 1] + 0.5) * 0x1p-32;
  const double r = sqrt(-2.0 * log(u1)), phi = 6.283185307179586476925286766559 * u2;
  return (which & 1) ? r * sin(phi) : r * cos(phi);
}

// TPR threads per row (a power of two, <= 64, so a row's threads sit in one wave); thread t of
// a row owns the 4-element chunks t, t + TPR, ...
template <typename T>
__global__ __launch_bounds__(256) void dp_release_kernel(T* X, int n, int m, int tpr, double S,
                                                         double sigma, uint64_t seed, uint64_t release) {
  const int rows_per_wg = 256 / tpr;
  const int t = threadIdx.x % tpr;
  const int i_raw = blockIdx.x * rows_per_wg + threadIdx.x / tpr;
  const bool live = i_raw < n;
  const int i = live ? i_raw : n - 1;  // idle threads shadow the last row and store nothing
  T* row = X + (int64_t)i * m;
  double scale = 1.0;
  if (S > 0.0 && isfinite(S)) {  // uniform branch: the shuffles below are reached by every lane
    double sq = 0.0;
    for (int k0 = 4 * t; k0 < m; k0 += 4 * tpr)
      for (int k = k0; k < k0 + 4 && k < m; ++k) {
        const double l = log((double)row[k]);
        sq += l * l;
      }
    for (int off = tpr >> 1; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
    const double norm = sqrt(sq);
    if (norm > S) scale = S / norm;
  }
  if (!live) return;
  uint64_t cached = ~uint64_t(0);
  PhiloxBlock blk{};
  for (int k0 = 4 * t; k0 < m; k0 += 4 * tpr)
    for (int k = k0; k < k0 + 4 && k < m; ++k) {
      const uint64_t e = (uint64_t)i * (uint64_t)m + (uint64_t)k;
      double l = log((double)row[k]) * scale;
      if (sigma != 0.0) {
        if (e / 4 != cached) {
          cached = e / 4;
          blk = philox4x32_10(cached, release, seed);
        }
        l += sigma * block_normal(blk, (int)(e % 4));
      }
      row[k] = (T)exp(l);
    }
}

int launch_dp_release(int dtype, void* X, int n, int m, double S, double sigma, uint64_t seed,
                      uint64_t release, hipStream_t stream) {
  int tpr = 1;
  while (tpr < 64 && 4 * tpr < m) tpr *= 2;
  const int rows_per_wg = 256 / tpr;
  dim3 grid((n + rows_per_wg - 1) / rows_per_wg), block(256);
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((dp_release_kernel<double>), grid, block, 0, stream, (double*)X, n, m, tpr, S,
                       sigma, seed, release);
  else
    hipLaunchKernelGGL((dp_release_kernel<float>), grid, block, 0, stream, (float*)X, n, m, tpr, S,
                       sigma, seed, release);
  FSK_LAUNCH_CHECK("dp_release_kernel");
  return FSK_OK;
}

}  // namespace fsk
