// Multitarget Sinkhorn for gfx950 (paper: Sec. 5.3.2): m histogram pairs share one
// kernel matrix, so the two products of an iteration are real matrix products
//
//     Q = K V   (n x n by n x m),   U = A ./ Q,      R = K^T U,   V = B ./ R
//
// and run on the matrix cores with v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate).
//
// Both products use the same plan.  A workgroup of 4 waves owns a 256 x 64 output tile
// (64 x 64 per wave: 2 x 2 MFMA blocks, 64 accumulator registers) and one part of the
// contraction range, walked in chunks of 32 indices.  K, the operand that streams from
// HBM, goes straight from global memory into registers (128-bit loads along a row for
// K V, 64-bit loads for K^T U, non-temporal, one chunk ahead of the MFMAs).  The chunk of
// the n x m operand (32 x 64 values) is shared by the four waves: it is staged in LDS,
// double buffered, one barrier per chunk.  The grid splits the contraction range S ways;
// the S partial tiles go to the workspace and a reduction kernel adds them in fixed order
// and applies the division (S = 1: the division is fused into the tile store).
//
// The row-major walk of K^T U (lanes along a row of K, 64-bit loads, 256 contiguous bytes
// per half-wave) costs the memory pipeline far fewer address operations than the walk of
// K V (every lane on a different row), and that, not HBM, is what limits these kernels.
// Since K is fixed over hundreds of iterations, the call therefore builds K^T once in the
// workspace and runs BOTH products as "transposed" products (Q = (K^T)^T V).  When the
// workspace has no room for K^T the direct row-product kernel is used instead.
//
// MFMA 32x32x2 operand layout (lane l of 64): A[i = l%32][k = l/32],
// B[k = l/32][j = l%32], D[i = 8(v/4) + 4(l/32) + v%4][j = l%32] for accumulator
// register v.  MFMA e of a chunk of C indices contracts the chunk's indices {e, C/2 + e},
// so lane (.., h = l/32) supplies index (C/2) h + e: with K row-major a lane fetches its
// C/2 values of a chunk as 128-bit loads along its row.
#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int kBtCols = 64;        // histogram columns per call (m <= 64)
constexpr int kBtWaveTile = 64;    // output rows per wave
constexpr int kBtWaves = 4;
constexpr int kBtTile = kBtWaveTile * kBtWaves;  // output rows per workgroup
constexpr int kBtChunk = 32;       // contraction indices per chunk
constexpr int kBtHalf = kBtChunk / 2;  // indices of a chunk supplied by one half-wave
constexpr int kBtStage = kBtChunk * kBtCols / 256;  // staged operand values per thread

__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// One product.  COLPROD == false: out rows are rows of K, contraction over columns
// (Q = K X).  COLPROD == true: out rows are columns of K, contraction over rows (R = K^T X).
// X is the n x m operand.  final != 0: out = marg ./ product; else the partial product of
// this grid slice goes to out + slice * n * m.
template <bool COLPROD>
__global__ __launch_bounds__(256) void batched_prod_kernel(const float* __restrict__ K, int64_t ld,
                                                           int n, int m,
                                                           const float* __restrict__ X,
                                                           const float* __restrict__ marg,
                                                           float* __restrict__ out, int final) {
  __shared__ float xs[2][kBtChunk][kBtCols];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  const int o0 = blockIdx.x * kBtTile + wave * kBtWaveTile;  // first output row of this wave

  // contraction chunks of this grid slice
  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  const int per = (nchunks + gridDim.y - 1) / gridDim.y;
  int c0 = blockIdx.y * per;
  int c1 = c0 + per < nchunks ? c0 + per : nchunks;
  if (c0 > c1) c0 = c1;
  int full_end = n / kBtChunk < c1 ? n / kBtChunk : c1;  // chunks [c0, full_end) are whole
  if (full_end < c0) full_end = c0;

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // --- K addressing of this lane
  const float* kbase[2];
  if (!COLPROD) {
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      int row = o0 + 32 * a + r;
      row = row < n ? row : n - 1;  // clamp; rows past the end are dropped at the store
      kbase[a] = K + (int64_t)row * ld;
    }
  } else {
    int jc = o0 + 2 * r;  // two adjacent columns of K per lane, clamped inside the row pitch
    const int jmax = (int)ld - 2;
    jc = jc < jmax ? jc : jmax;
    kbase[0] = kbase[1] = K + jc;
  }

  // ka[a][e]: the K value of MFMA row r of block a for contraction index 16h + e of a chunk
  auto load_k = [&](int c, float(&ka)[2][kBtHalf]) {
    const int first = c * kBtChunk + kBtHalf * h;
    if (!COLPROD) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int t = 0; t < kBtHalf / 4; ++t) {
          const Pack<float> p = load_pack_stream(kbase[a] + first + 4 * t);
#pragma unroll
          for (int e = 0; e < 4; ++e) ka[a][4 * t + e] = p.e[e];
        }
    } else {
#pragma unroll
      for (int e = 0; e < kBtHalf; ++e) {
        const floatx2 p = __builtin_nontemporal_load(
            reinterpret_cast<const floatx2*>(kbase[0] + (int64_t)(first + e) * ld));
        ka[0][e] = p[0];
        ka[1][e] = p[1];
      }
    }
  };
  // same with the contraction indices >= n masked to zero (ragged last chunk)
  auto load_k_masked = [&](int c, float(&ka)[2][kBtHalf]) {
    const int first = c * kBtChunk + kBtHalf * h;
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
      const bool ok = first + e < n;
      const int kk = ok ? first + e : n - 1;
      if (!COLPROD) {
#pragma unroll
        for (int a = 0; a < 2; ++a) ka[a][e] = ok ? kbase[a][kk] : 0.f;
      } else {
        const floatx2 p = *reinterpret_cast<const floatx2*>(kbase[0] + (int64_t)kk * ld);
        ka[0][e] = ok ? p[0] : 0.f;
        ka[1][e] = ok ? p[1] : 0.f;
      }
    }
  };

  // --- staging of the X chunk: kBtChunk x 64 values, kBtStage per thread.  Columns >= m are clamped
  // duplicates (they only feed output columns that are never stored).
  const int sc = tid & 63, sk = tid >> 6;  // column, first contraction row of this thread
  const float* xcol = X + (sc < m ? sc : m - 1);
  auto load_x = [&](int c, float(&st)[kBtStage]) {  // whole chunk: every contraction index < n
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) st[i] = xcol[(int64_t)(c * kBtChunk + sk + 4 * i) * m];
  };
  auto load_x_masked = [&](int c, float(&st)[kBtStage]) {  // ragged chunk: indices >= n give zero
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) {
      const int kk = c * kBtChunk + sk + 4 * i;
      const float val = xcol[(int64_t)(kk < n ? kk : n - 1) * m];
      st[i] = kk < n ? val : 0.f;
    }
  };
  auto store_x = [&](int buf, const float(&st)[kBtStage]) {
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) xs[buf][sk + 4 * i][sc] = st[i];
  };

  auto multiply = [&](int buf, const float(&ka)[2][kBtHalf]) {
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
      const float b0 = xs[buf][kBtHalf * h + e][r];
      const float b1 = xs[buf][kBtHalf * h + e][32 + r];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        acc[a][0] = mfma32(ka[a][e], b0, acc[a][0]);
        acc[a][1] = mfma32(ka[a][e], b1, acc[a][1]);
      }
    }
  };

  float kaA[2][kBtHalf], kaB[2][kBtHalf], st[kBtStage];
  if (c0 < full_end) {
    load_k(c0, kaA);
    load_x(c0, st);
    store_x(0, st);
  }
  __syncthreads();
  // Two chunks per trip: chunk c sits in kaA / xs[0], chunk c+1 goes through kaB / xs[1].
  // Loads for the chunk after next are issued before the MFMAs of the current one.
  int c = c0;
  for (; c + 2 <= full_end; c += 2) {
    load_k(c + 1, kaB);
    load_x(c + 1, st);
    multiply(0, kaA);
    store_x(1, st);
    __syncthreads();
    const bool more = c + 2 < full_end;
    if (more) {
      load_k(c + 2, kaA);
      load_x(c + 2, st);
    }
    multiply(1, kaB);
    if (more) store_x(0, st);
    __syncthreads();
  }
  if (c < full_end) {  // odd chunk left over: already in kaA / xs[0]
    multiply(0, kaA);
    __syncthreads();
  }
  if (full_end < c1) {  // the one ragged chunk at the end of the contraction range
    load_k_masked(full_end, kaA);
    load_x_masked(full_end, st);
    __syncthreads();
    store_x(0, st);
    __syncthreads();
    multiply(0, kaA);
  }

  // --- store the wave's 64 x 64 tile
  float* dst = final ? out : out + (int64_t)blockIdx.y * n * m;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = 8 * (v / 4) + 4 * h + (v % 4);  // MFMA row of accumulator register v
      const int row = COLPROD ? o0 + 2 * i + a : o0 + 32 * a + i;
      if (row < n) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int col = 32 * b + r;
          if (col < m) {
            const int64_t idx = (int64_t)row * m + col;
            dst[idx] = final ? marg[idx] / acc[a][b][v] : acc[a][b][v];
          }
        }
      }
    }
}

// ------------------------------------------------------------------ K^T (setup, once per call)
__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ K, int64_t ld, int n,
                                                        float* __restrict__ Kt, int64_t ldt) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
#pragma unroll 4
  for (int r = ty; r < 64; r += 4)
    if (i0 + r < n && j0 + tx < n) tile[r][tx] = K[(int64_t)(i0 + r) * ld + j0 + tx];
  __syncthreads();
#pragma unroll 4
  for (int r = ty; r < 64; r += 4)
    if (j0 + r < n && i0 + tx < n) Kt[(int64_t)(j0 + r) * ldt + i0 + tx] = tile[tx][r];
}

// ------------------------------------------------------------------ host side
static int batched_splits(int n) {
  int cus = device_cu_count();
  if (cus < 1) cus = 256;
  const int tiles = (n + kBtTile - 1) / kBtTile;
  int s = (4 * cus + tiles - 1) / tiles;
  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  const int max_s = nchunks / 4 > 0 ? nchunks / 4 : 1;  // at least 4 chunks per slice
  if (s > max_s) s = max_s;
  if (s > 32) s = 32;
  return s < 1 ? 1 : s;
}

static size_t batched_partial_bytes(int n, int m) {
  const int mg = m < kBtCols ? m : kBtCols;
  return align_up((size_t)batched_splits(n) * (size_t)n * (size_t)mg * 4, 256);
}
static int64_t batched_ldt(int n) { return (int64_t)align_up((size_t)n, 64); }

// partial products + room for K^T
size_t batched_workspace_bytes(int n, int m) {
  return batched_partial_bytes(n, m) + align_up((size_t)n * (size_t)batched_ldt(n) * 4, 256) + 256;
}

int run_sinkhorn_batched(const fsk_opts* o, const void* K, int64_t ldK, const void* A, const void* B,
                         void* U, void* V, void* workspace, size_t ws_bytes, hipStream_t st) {
  if (o->dtype != FSK_F32) return set_error(FSK_EUNSUPPORTED, "batched path takes fp32");
  if (o->m > kBtCols)
    return set_error(FSK_EUNSUPPORTED, "batched path is built for m <= 64 histograms per call");
  const int n = o->n, m = o->m;
  const int S = batched_splits(n);
  const size_t part_bytes = batched_partial_bytes(n, m);
  if (S > 1 && (!workspace || ws_bytes < part_bytes))
    return set_error(FSK_EWORKSPACE, "batched call needs at least %zu workspace bytes (%zu to run at "
                     "full speed), got %zu", part_bytes, batched_workspace_bytes(n, m), ws_bytes);
  const float *Kf = (const float*)K, *Af = (const float*)A, *Bf = (const float*)B;
  float *Uf = (float*)U, *Vf = (float*)V, *part = (float*)workspace;
  // K^T in the workspace if it fits and the run is long enough to pay for it
  const bool use_kt = workspace && ws_bytes >= batched_workspace_bytes(n, m) && o->max_iters >= 2;
  const int64_t ldt = batched_ldt(n);
  float* Kt = use_kt ? (float*)((char*)workspace + part_bytes) : nullptr;
  if (use_kt) {
    dim3 tg((n + 63) / 64, (n + 63) / 64);
    hipLaunchKernelGGL(transpose_kernel, tg, dim3(256), 0, st, Kf, ldK, n, Kt, ldt);
    FSK_LAUNCH_CHECK("transpose_kernel");
  }
  dim3 grid((n + kBtTile - 1) / kBtTile, S), block(256);
  const int nm = n * m;
  for (int it = 0; it < o->max_iters; ++it) {
    if (use_kt)  // Q = K V as the transposed product of K^T
      hipLaunchKernelGGL((batched_prod_kernel<true>), grid, block, 0, st, (const float*)Kt, ldt, n, m,
                         (const float*)Vf, Af, S == 1 ? Uf : part, S == 1 ? 1 : 0);
    else
      hipLaunchKernelGGL((batched_prod_kernel<false>), grid, block, 0, st, Kf, ldK, n, m,
                         (const float*)Vf, Af, S == 1 ? Uf : part, S == 1 ? 1 : 0);
    FSK_LAUNCH_CHECK("batched_prod_kernel (K V)");
    if (S > 1)
      FSK_TRY(launch_colreduce(FSK_F32, part, nm, S, 0, nm, Af, nullptr, Uf, kEpiDivide, 1.0, st));
    hipLaunchKernelGGL((batched_prod_kernel<true>), grid, block, 0, st, Kf, ldK, n, m,
                       (const float*)Uf, Bf, S == 1 ? Vf : part, S == 1 ? 1 : 0);
    FSK_LAUNCH_CHECK("batched_prod_kernel (K^T U)");
    if (S > 1)
      FSK_TRY(launch_colreduce(FSK_F32, part, nm, S, 0, nm, Bf, nullptr, Vf, kEpiDivide, 1.0, st));
  }
  return FSK_OK;
}

}  // namespace fsk
