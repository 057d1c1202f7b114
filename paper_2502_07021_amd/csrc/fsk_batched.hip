// Multitarget Sinkhorn for gfx950 (paper: Sec. 5.3.2): m histogram pairs share one
// kernel matrix, so the two products of an iteration are real matrix products
//
//     Q = K V   (n x n by n x m),   U = A ./ Q,      R = K^T U,   V = B ./ R
//
// and run on the matrix cores with v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate).
//
// Both products use the same plan.  A wave owns a 64 x 64 output tile (2 x 2 MFMA
// blocks, 64 accumulator registers) and a contiguous part of the contraction
// range; it feeds the MFMAs straight from registers loaded from global memory
// (K with streaming 128-/64-bit loads, the n x m operand with 32-bit loads that
// hit in cache) -- there is no LDS staging and no barrier in the main loop.  The
// four waves of a workgroup share the output tile and split the contraction
// range; their accumulators are added through LDS in a fixed order.  If the grid
// splits the range further, the workgroup partials go to the workspace and a
// reduction kernel adds them in order and applies the division.
//
// MFMA 32x32x2 operand layout (lane l of 64): A[i = l%32][k = l/32],
// B[k = l/32][j = l%32], D[i = 8(v/4) + 4(l/32) + v%4][j = l%32] for accumulator
// register v.  A contraction chunk of 32 indices is consumed by 16 MFMAs per
// block pair; MFMA e of a chunk contracts indices {e, 16 + e}, so lane (.., h)
// supplies index 16h + e: with K stored row-major this lets a lane fetch its 16
// values of a chunk as four 128-bit loads along its row.
#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kBtTile = 64;    // output tile edge per workgroup
constexpr int kBtChunk = 32;   // contraction indices per chunk
constexpr int kBtWaves = 4;

__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Adds the four waves' accumulators as (w0 + w2) + (w1 + w3); the result is valid in wave 0.
__device__ __forceinline__ void reduce_waves(floatx16 (&acc)[2][2], float* lds, int wave, int lane) {
  // lds: 2 slots of 64 registers x 64 lanes
  float* slot = lds + (wave & 1) * 64 * 64;
  if (wave >= 2) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) slot[((a * 2 + b) * 16 + v) * 64 + lane] = acc[a][b][v];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] += slot[((a * 2 + b) * 16 + v) * 64 + lane];
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) lds[((a * 2 + b) * 16 + v) * 64 + lane] = acc[a][b][v];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] += lds[((a * 2 + b) * 16 + v) * 64 + lane];
  }
}

// Contraction chunks [c0, c1) of this wave: the range of `nchunks` chunks is split evenly
// over gridDim.y * kBtWaves consecutive parts.
__device__ __forceinline__ void wave_chunk_range(int nchunks, int part, int parts, int& c0, int& c1) {
  const int per = (nchunks + parts - 1) / parts;
  c0 = part * per;
  c1 = c0 + per < nchunks ? c0 + per : nchunks;
  if (c0 > nchunks) c0 = nchunks;
}

// Writes wave 0's reduced tile.  rowmap(a, i) gives the output row of MFMA row i of block a.
// final != 0: out = marg ./ acc (the scaling update); else out = acc (a partial sum).
template <typename RowMap>
__device__ __forceinline__ void store_tile(const floatx16 (&acc)[2][2], int lane, int n, int m,
                                           RowMap rowmap, const float* __restrict__ marg,
                                           float* __restrict__ out, int final) {
  const int cl = lane & 31, hl = lane >> 5;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = rowmap(a, 8 * (v / 4) + 4 * hl + (v % 4));
      if (row < n) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int col = 32 * b + cl;
          if (col < m) {
            const int64_t idx = (int64_t)row * m + col;
            out[idx] = final ? marg[idx] / acc[a][b][v] : acc[a][b][v];
          }
        }
      }
    }
}

// ------------------------------------------------------------------ Q = K V
// Tile rows i0..i0+63 of K against all m <= 64 columns of V.
__global__ __launch_bounds__(256) void batched_rowprod_kernel(const float* __restrict__ K, int64_t ld,
                                                              int n, int m,
                                                              const float* __restrict__ V,
                                                              const float* __restrict__ marg,
                                                              float* __restrict__ out, int final) {
  __shared__ float lds[2 * 64 * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int i0 = blockIdx.x * kBtTile;
  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  int c0, c1;
  wave_chunk_range(nchunks, blockIdx.y * kBtWaves + wave, gridDim.y * kBtWaves, c0, c1);

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const float* krow[2];
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    int row = i0 + 32 * a + r;
    row = row < n ? row : n - 1;  // clamp; rows past the end are dropped at the store
    krow[a] = K + (int64_t)row * ld;
  }
  int vcol[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) vcol[b] = 32 * b + r < m ? 32 * b + r : m - 1;

  for (int c = c0; c < c1; ++c) {
    const int k0 = c * kBtChunk + 16 * h;  // this lane's 16 contraction indices: k0 .. k0+15
    float ka[2][16], vb[2][16];
    if (k0 + 16 <= n) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const Pack<float> p = load_pack_stream(krow[a] + k0 + 4 * t);
#pragma unroll
          for (int e = 0; e < 4; ++e) ka[a][4 * t + e] = p.e[e];
        }
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) vb[b][e] = V[(int64_t)(k0 + e) * m + vcol[b]];
    } else {  // ragged end of the contraction range: indices >= n contribute zero
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const bool ok = k0 + e < n;
        const int kk = ok ? k0 + e : n - 1;
#pragma unroll
        for (int a = 0; a < 2; ++a) ka[a][e] = ok ? krow[a][kk] : 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b) vb[b][e] = ok ? V[(int64_t)kk * m + vcol[b]] : 0.f;
      }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = mfma32(ka[a][e], vb[b][e], acc[a][b]);
  }

  reduce_waves(acc, lds, wave, lane);
  if (wave == 0) {
    float* dst = final ? out : out + (int64_t)blockIdx.y * n * m;
    store_tile(acc, lane, n, m, [&](int a, int i) { return i0 + 32 * a + i; }, marg, dst, final);
  }
}

// ------------------------------------------------------------------ R = K^T U
// Tile columns j0..j0+63 of K (rows of the result).  A lane fetches two adjacent columns
// with one 64-bit load, so MFMA row i of block a is column j0 + 2 i + a of K.
__global__ __launch_bounds__(256) void batched_colprod_kernel(const float* __restrict__ K, int64_t ld,
                                                              int n, int m,
                                                              const float* __restrict__ U,
                                                              const float* __restrict__ marg,
                                                              float* __restrict__ out, int final) {
  __shared__ float lds[2 * 64 * 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int j0 = blockIdx.x * kBtTile;
  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  int c0, c1;
  wave_chunk_range(nchunks, blockIdx.y * kBtWaves + wave, gridDim.y * kBtWaves, c0, c1);

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // column pair of this lane, clamped inside the row pitch (ld is a multiple of 4)
  int jc = j0 + 2 * r;
  const int jmax = (int)ld - 2;
  jc = jc < jmax ? jc : jmax;
  int ucol[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) ucol[b] = 32 * b + r < m ? 32 * b + r : m - 1;

  for (int c = c0; c < c1; ++c) {
    const int i_first = c * kBtChunk + 16 * h;  // this lane's 16 contraction indices (rows of K)
    float ka[2][16], ub[2][16];
    if (i_first + 16 <= n) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const floatx2 p = __builtin_nontemporal_load(
            reinterpret_cast<const floatx2*>(K + (int64_t)(i_first + e) * ld + jc));
        ka[0][e] = p[0];
        ka[1][e] = p[1];
      }
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) ub[b][e] = U[(int64_t)(i_first + e) * m + ucol[b]];
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const bool ok = i_first + e < n;
        const int ii = ok ? i_first + e : n - 1;
        const floatx2 p = *reinterpret_cast<const floatx2*>(K + (int64_t)ii * ld + jc);
        ka[0][e] = ok ? p[0] : 0.f;
        ka[1][e] = ok ? p[1] : 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b) ub[b][e] = ok ? U[(int64_t)ii * m + ucol[b]] : 0.f;
      }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e)
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = mfma32(ka[a][e], ub[b][e], acc[a][b]);
  }

  reduce_waves(acc, lds, wave, lane);
  if (wave == 0) {
    float* dst = final ? out : out + (int64_t)blockIdx.y * n * m;
    store_tile(acc, lane, n, m, [&](int a, int i) { return j0 + 2 * i + a; }, marg, dst, final);
  }
}

// ------------------------------------------------------------------ host side
static int batched_splits(int n) {
  int cus = device_cu_count();
  if (cus < 1) cus = 256;
  const int tiles = (n + kBtTile - 1) / kBtTile;
  int s = (4 * cus + tiles - 1) / tiles;
  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  const int max_s = nchunks / (2 * kBtWaves) > 0 ? nchunks / (2 * kBtWaves) : 1;  // >= 2 chunks per wave
  if (s > max_s) s = max_s;
  if (s > 16) s = 16;
  return s < 1 ? 1 : s;
}

size_t batched_workspace_bytes(int n, int m) {
  const int mg = m < 64 ? m : 64;
  return align_up((size_t)batched_splits(n) * (size_t)n * (size_t)mg * 4, 256) + 256;
}

int run_sinkhorn_batched(const fsk_opts* o, const void* K, int64_t ldK, const void* A, const void* B,
                         void* U, void* V, void* workspace, size_t ws_bytes, hipStream_t st) {
  if (o->dtype != FSK_F32) return set_error(FSK_EUNSUPPORTED, "batched path takes fp32");
  if (o->m > 64) return set_error(FSK_EUNSUPPORTED, "batched path is built for m <= 64 histograms per call");
  const int n = o->n, m = o->m;
  const size_t need = batched_workspace_bytes(n, m);
  const int S = batched_splits(n);
  if (S > 1 && (!workspace || ws_bytes < need))
    return set_error(FSK_EWORKSPACE, "batched call needs %zu workspace bytes, got %zu", need, ws_bytes);
  const float *Kf = (const float*)K, *Af = (const float*)A, *Bf = (const float*)B;
  float *Uf = (float*)U, *Vf = (float*)V, *part = (float*)workspace;
  dim3 grid((n + kBtTile - 1) / kBtTile, S), block(256);
  const int nm = n * m;
  for (int it = 0; it < o->max_iters; ++it) {
    hipLaunchKernelGGL(batched_rowprod_kernel, grid, block, 0, st, Kf, ldK, n, m, Vf, Af,
                       S == 1 ? Uf : part, S == 1 ? 1 : 0);
    FSK_LAUNCH_CHECK("batched_rowprod_kernel");
    if (S > 1)
      FSK_TRY(launch_colreduce(FSK_F32, part, nm, S, 0, nm, Af, nullptr, Uf, kEpiDivide, 1.0, st));
    hipLaunchKernelGGL(batched_colprod_kernel, grid, block, 0, st, Kf, ldK, n, m, Uf, Bf,
                       S == 1 ? Vf : part, S == 1 ? 1 : 0);
    FSK_LAUNCH_CHECK("batched_colprod_kernel");
    if (S > 1)
      FSK_TRY(launch_colreduce(FSK_F32, part, nm, S, 0, nm, Bf, nullptr, Vf, kEpiDivide, 1.0, st));
  }
  return FSK_OK;
}

}  // namespace fsk
