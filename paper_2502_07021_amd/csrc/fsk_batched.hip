// Multitarget Sinkhorn for gfx950 (paper: Sec. 5.3.2): m histogram pairs share one
// kernel matrix, so the two products of an iteration are real matrix products
//
//     Q = K V   (n x n by n x m),   U = A ./ Q,      R = K^T U,   V = B ./ R
//
// and run on the matrix cores with v_mfma_f32_32x32x2_f32 (fp32 in, fp32 accumulate).
//
// A walk of K in which the lanes of a wave run along a row (R = K^T X: output rows are
// columns of K) costs the memory pipeline far fewer address operations than one in which
// every lane sits on its own row (Q = K X), and that, not HBM, limits these kernels.  K is
// fixed over hundreds of iterations, so the call builds K^T once in the workspace and runs
// BOTH products as transposed products (Q = (K^T)^T V) with batched_prod_wide_kernel: a
// wave owns a 128 x 64 output tile (4 x 2 MFMA blocks, 128 accumulator registers, one wave
// per SIMD), a workgroup of 4 waves 512 x 64 and one part of the contraction range, walked in
// chunks of 32 indices.  K goes straight from global memory into registers (128-bit
// non-temporal buffer loads, one chunk ahead of the MFMAs, addressed as scalar base + scalar
// row offset + a fixed lane offset so that no vector instruction stands between two MFMAs);
// the chunk of the n x m operand (32 x 64 values) is shared by the four waves through LDS,
// double buffered, one barrier per chunk.
// Wider problems (the paper stacks N = 500 targets and more) run as ceil(m / 64) column groups
// inside the same launch.  The 1-D grid is row tiles x column groups x S parts of the
// contraction range, S chosen so that the grid fills the compute units; for S > 1 the partial
// tiles go to the workspace in the order the wave's registers hold them (whole-KiB stores) and
// a reduction kernel adds them in fixed order and applies the division (S = 1: the division
// is fused into the tile store).  When the workspace has no room
// for K^T, Q = K V falls back to batched_rowprod_kernel, the direct walk with a 64 x 64 tile per
// wave, one column group per launch.
//
// MFMA 32x32x2 operand layout (lane l of 64): A[i = l%32][k = l/32],
// B[k = l/32][j = l%32], D[i = 8(v/4) + 4(l/32) + v%4][j = l%32] for accumulator
// register v.  MFMA e of a chunk of C indices contracts the chunk's indices {e, C/2 + e},
// so lane (.., h = l/32) supplies index (C/2) h + e.
#include "fsk_device.h"
#include "fsk_internal.h"

#include <type_traits>

namespace fsk {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kBtCols = 64;        // histogram columns per tile (wider problems go in groups)
constexpr int kBtWaveTile = 64;    // output rows per wave
constexpr int kBtWaves = 4;
constexpr int kBtTile = kBtWaveTile * kBtWaves;  // output rows per workgroup
constexpr int kBtChunk = 32;       // contraction indices per chunk
constexpr int kBtHalf = kBtChunk / 2;  // indices of a chunk supplied by one half-wave
constexpr int kBtStage = kBtChunk * kBtCols / 256;  // staged operand values per thread

__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Q = K X by the direct walk: out rows are rows of K, contraction over columns, a lane
// fetches its row's values of a chunk as 128-bit loads.  X holds the n x m operand (m <= 64
// columns of a wider matrix with row pitch ldm).  final != 0: out = marg ./ product, with marg
// and out laid out like X; else the partial product of this grid slice goes, densely packed
// (pitch m), to out + slice * n * m.
__global__ __launch_bounds__(256) void batched_rowprod_kernel(const float* __restrict__ K, int64_t ld,
                                                           int n, int m, int64_t ldm,
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
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    int row = o0 + 32 * a + r;
    row = row < n ? row : n - 1;  // clamp; rows past the end are dropped at the store
    kbase[a] = K + (int64_t)row * ld;
  }

  // ka[a][e]: the K value of MFMA row r of block a for contraction index 16h + e of a chunk
  auto load_k = [&](int c, float(&ka)[2][kBtHalf]) {
    const int first = c * kBtChunk + kBtHalf * h;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int t = 0; t < kBtHalf / 4; ++t) {
        const Pack<float> p = load_pack_stream(kbase[a] + first + 4 * t);
#pragma unroll
        for (int e = 0; e < 4; ++e) ka[a][4 * t + e] = p.e[e];
      }
  };
  // same with the contraction indices >= n masked to zero (ragged last chunk)
  auto load_k_masked = [&](int c, float(&ka)[2][kBtHalf]) {
    const int first = c * kBtChunk + kBtHalf * h;
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
      const bool ok = first + e < n;
      const int kk = ok ? first + e : n - 1;
#pragma unroll
      for (int a = 0; a < 2; ++a) ka[a][e] = ok ? kbase[a][kk] : 0.f;
    }
  };

  // --- staging of the X chunk: kBtChunk x 64 values, kBtStage per thread.  Columns >= m are clamped
  // duplicates (they only feed output columns that are never stored).
  const int sc = tid & 63, sk = tid >> 6;  // column, first contraction row of this thread
  const float* xcol = X + (sc < m ? sc : m - 1);
  auto load_x = [&](int c, float(&st)[kBtStage]) {  // whole chunk: every contraction index < n
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) st[i] = xcol[(int64_t)(c * kBtChunk + sk + 4 * i) * ldm];
  };
  auto load_x_masked = [&](int c, float(&st)[kBtStage]) {  // ragged chunk: indices >= n give zero
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) {
      const int kk = c * kBtChunk + sk + 4 * i;
      const float val = xcol[(int64_t)(kk < n ? kk : n - 1) * ldm];
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
    // keep the loads above the MFMAs: left alone the scheduler sinks them to the end of
    // the chunk to shorten register live ranges, which throws the prefetch away
    __builtin_amdgcn_sched_barrier(0);
    multiply(0, kaA);
    store_x(1, st);
    __syncthreads();
    const bool more = c + 2 < full_end;
    if (more) {
      load_k(c + 2, kaA);
      load_x(c + 2, st);
    }
    __builtin_amdgcn_sched_barrier(0);
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
      const int row = o0 + 32 * a + i;
      if (row < n) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
          const int col = 32 * b + r;
          if (col < m) {
            if (final) {
              const int64_t idx = (int64_t)row * ldm + col;
              dst[idx] = marg[idx] / acc[a][b][v];
            } else {
              dst[(int64_t)row * m + col] = acc[a][b][v];
            }
          }
        }
      }
    }
}

// ------------------------------------------------------------------ wide transposed product
// R = K^T X with a 128 x 64 output tile per wave (512 x 64 per workgroup): a lane fetches four
// adjacent columns of K with one 128-bit load (512 contiguous bytes per half-wave), so MFMA
// row i of block a is column o0 + 4 i + a of K; 4 x 2 MFMA blocks, 128 accumulator registers,
// one wave per SIMD.  Twice the flops per load instruction and per LDS read of the 64 x 64
// kernel above; the loads of the next chunk are in flight under the 128 MFMAs of this one.
constexpr int kBtWideWaveTile = 128;
constexpr int kBtWideTile = kBtWideWaveTile * kBtWaves;
constexpr int kBtWaveTileFloats = kBtWideWaveTile * kBtCols;  // one wave's partial tile

// A partial tile (the grid splits the contraction range) is stored in the order the wave holds it:
// [MFMA block a][block b][register quad vq][lane][4 registers], one 128-bit store per lane and
// quad, a whole KiB per instruction.  Element j of that pack is output row
// 128 wt + 4 (8 vq + 4 (lane / 32) + j) + a and column 32 b + lane % 32 of the wave's tile wt; the
// partial area of one (column group, slice) holds ceil(n / 128) such tiles.
__host__ __device__ inline int64_t bt_partial_area(int n) {
  return (int64_t)((n + kBtWideWaveTile - 1) / kBtWideWaveTile) * kBtWaveTileFloats;
}

// X, marg and out (final) are n x mtot with row pitch mtot; the grid covers `groups` column
// groups of up to 64 columns, `slices` contraction slices and the row tiles.  final == 0: the
// partial product of (group g, slice s) goes to out + (g * slices + s) * bt_partial_area(n) in
// the layout described above.  XVEC: mtot is a multiple of 4 and X is 16-byte aligned, so the
// X chunk is staged with 128-bit accesses.
template <bool XVEC>
__global__ __launch_bounds__(256) void batched_prod_wide_kernel(const float* __restrict__ K,
                                                                int64_t ld, int n, int mtot,
                                                                const float* __restrict__ X,
                                                                const float* __restrict__ marg,
                                                                float* __restrict__ out, int final,
                                                                int slices, int groups) {
  __shared__ __attribute__((aligned(16))) float xs[2][kBtChunk][kBtCols];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;
  // 1-D grid, slice fastest: workgroups are dealt to the 8 XCDs round-robin, so the workgroups
  // of one contraction slice -- the ones that read the same rows of X -- meet on the same XCDs
  // and share those rows in that XCD's L2 instead of every L2 holding all of X.
  const int slice = blockIdx.x % slices, grp = (blockIdx.x / slices) % groups;
  const int tile = blockIdx.x / (slices * groups);
  const int o0 = tile * kBtWideTile + wave * kBtWideWaveTile;
  const int col0 = grp * kBtCols;
  const int m = mtot - col0 < kBtCols ? mtot - col0 : kBtCols;  // columns of this group
  const int64_t ldm = mtot;
  X += col0;
  marg += col0;

  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  const int per = (nchunks + slices - 1) / slices;
  int c0 = slice * per;
  int c1 = c0 + per < nchunks ? c0 + per : nchunks;
  if (c0 > c1) c0 = c1;
  int full_end = n / kBtChunk < c1 ? n / kBtChunk : c1;
  if (full_end < c0) full_end = c0;

  floatx16 acc[4][2];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  int jc = o0 + 4 * r;  // four adjacent columns of K per lane, clamped inside the row pitch
  const int jmax = (int)ld - 4;
  jc = jc < jmax ? jc : jmax;
  const float* kcol = K + jc;
  // Addresses are split into a byte offset that belongs to the lane (its columns and its
  // half-wave's row inside a chunk; 32 bits, formed once) and a wave-uniform part: the chunk's
  // first row (the base of a buffer descriptor, advanced once per chunk on the scalar unit) plus
  // e row pitches for k-step e (a scalar offset).
  const uint32_t kb = (uint32_t)(((int64_t)(kBtHalf * h) * ld + jc) * 4);
  const uint32_t ldb = (uint32_t)(ld * 4), ldmb = (uint32_t)(ldm * 4);
  auto at = [&](const float* row, uint32_t lane_bytes) {
    return reinterpret_cast<const float*>(reinterpret_cast<const char*>(row) + lane_bytes);
  };
  auto load_k = [&](int c, Pack<float>(&ka)[kBtHalf]) {
    const float* row = K + (int64_t)c * kBtChunk * ld;
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e, row += ld) ka[e] = load_pack_stream(at(row, kb));
  };
  auto load_k_masked = [&](int c, Pack<float>(&ka)[kBtHalf]) {
    const int first = c * kBtChunk + kBtHalf * h;
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
      const bool ok = first + e < n;
      Pack<float> p = load_pack(kcol + (int64_t)(ok ? first + e : n - 1) * ld);
#pragma unroll
      for (int q = 0; q < 4; ++q) p.e[q] = ok ? p.e[q] : 0.f;
      ka[e] = p;
    }
  };

  // Staging of the X chunk (32 x 64 values) through registers into LDS.  Scalar form: thread =
  // (column sc, rows sk + 4 i), 8 values.  Vector form: thread = (four columns from 4 xq, rows xr
  // and xr + 16), two 128-bit packs.  Columns >= m are clamped duplicates (they only feed output
  // columns that are never stored).
  const int sc = tid & 63, sk = tid >> 6;
  const float* xcol = X + (sc < m ? sc : m - 1);
  const uint32_t xb = (uint32_t)(((int64_t)sk * ldm + (sc < m ? sc : m - 1)) * 4);  // lane's bytes
  const int xr = tid >> 4, xq = tid & 15;
  const int xc4 = 4 * xq + 3 < m ? 4 * xq : (m >= 4 ? m - 4 : 0);
  const uint32_t xvb = (uint32_t)(((int64_t)xr * ldm + xc4) * 4);
  auto load_x = [&](int c, float(&st)[kBtStage]) {
    const float* row = X + (int64_t)c * kBtChunk * ldm;
#pragma unroll
    for (int i = 0; i < kBtStage; ++i, row += 4 * ldm) st[i] = *at(row, xb);
  };
  auto load_x_masked = [&](int c, float(&st)[kBtStage]) {
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) {
      const int kk = c * kBtChunk + sk + 4 * i;
      const float val = xcol[(int64_t)(kk < n ? kk : n - 1) * ldm];
      st[i] = kk < n ? val : 0.f;
    }
  };
  auto store_x = [&](int buf, const float(&st)[kBtStage]) {
#pragma unroll
    for (int i = 0; i < kBtStage; ++i) xs[buf][sk + 4 * i][sc] = st[i];
  };
  auto store_xv = [&](int buf, const Pack<float>(&sv)[2]) {
    store_pack(&xs[buf][xr][4 * xq], sv[0]);
    store_pack(&xs[buf][xr + 16][4 * xq], sv[1]);
  };
  auto multiply = [&](int buf, const Pack<float>(&ka)[kBtHalf]) {
    float b0[kBtHalf], b1[kBtHalf];  // the chunk's B operands, fetched from LDS up front
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
      b0[e] = xs[buf][kBtHalf * h + e][r];
      b1[e] = xs[buf][kBtHalf * h + e][32 + r];
    }
    __builtin_amdgcn_sched_barrier(0);  // one LDS wait per chunk instead of one per k-step
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        acc[a][0] = mfma32(ka[e].e[a], b0[e], acc[a][0]);
        acc[a][1] = mfma32(ka[e].e[a], b1[e], acc[a][1]);
      }
    }
  };

  // One chunk of the steady state: the MFMAs of the chunk in `ka` / xs[buf], whose first two
  // k-steps' B operands arrive in `bcur`.  With NEXT, everything the following chunk needs is
  // spread between them: its X rows (from `xrow`) are requested first -- before any K load of
  // this chunk, so that waiting for them later does not also wait for K loads issued since (the
  // memory counter retires loads in order) --, one K load (rows from `krow` on) follows every
  // k-step, the X values go to xs[buf ^ 1] and the workgroup meets at a barrier after k-step
  // kBtHalf - 2, and the following chunk's first two B operands are read (into `bnext`) before the
  // last k-step.  A wave issues in order, so a burst of loads, a wait for memory or a barrier at
  // the chunk boundary would leave the matrix pipe without work; spread out like this, nothing
  // stands between the last MFMA of one chunk and the first of the next.  The scheduling
  // barriers pin the order (left alone the scheduler sinks the loads to the end of the chunk).
  // Two LDS buffers suffice: every read of xs[buf] has completed (the barrier's own wait) before
  // any wave passes the barrier after which xs[buf] is written again.
  auto chunk_step = [&](auto next_tag, int buf, const Pack<float>(&ka)[kBtHalf],
                        const float(&bcur)[2][2], const float* krow, const float* xrow,
                        Pack<float>(&kn)[kBtHalf], float(&bnext)[2][2]) {
    constexpr bool NEXT = decltype(next_tag)::value;
    static_assert(kBtStage <= kBtHalf - 2, "the X loads must be issued before they are staged");
    float b0[kBtHalf], b1[kBtHalf];  // B operands: two k-steps ahead of the MFMAs that use them
    float stn[kBtStage];
    Pack<float> svn[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) b0[e] = bcur[e][0], b1[e] = bcur[e][1];
    const __amdgpu_buffer_rsrc_t rk = buffer_over(krow), rx = buffer_over(xrow);
    if (NEXT && XVEC) {
      svn[0] = buffer_load_pack<float, false>(rx, xvb, 0);
      svn[1] = buffer_load_pack<float, false>(rx, xvb, 16 * ldmb);
    }
#pragma unroll
    for (int e = 0; e < kBtHalf; ++e) {
      if (NEXT && e == kBtHalf - 1) {  // after the barrier: the next chunk's first operands
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          bnext[t][0] = xs[buf ^ 1][kBtHalf * h + t][r];
          bnext[t][1] = xs[buf ^ 1][kBtHalf * h + t][32 + r];
        }
      }
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        acc[a][0] = mfma32(ka[e].e[a], b0[e], acc[a][0]);
        acc[a][1] = mfma32(ka[e].e[a], b1[e], acc[a][1]);
      }
      if (e + 2 < kBtHalf) {
        b0[e + 2] = xs[buf][kBtHalf * h + e + 2][r];
        b1[e + 2] = xs[buf][kBtHalf * h + e + 2][32 + r];
      }
      if (NEXT) {
        kn[e] = buffer_load_pack<float, true>(rk, kb, e * ldb);
        if (!XVEC && e < kBtStage) stn[e] = *at(xrow + (int64_t)4 * e * ldm, xb);
        if (e == kBtHalf - 2) {
          if (XVEC) store_xv(buf ^ 1, svn); else store_x(buf ^ 1, stn);
          __syncthreads();
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  const std::true_type with_next;
  const std::false_type last;

  Pack<float> kaA[kBtHalf], kaB[kBtHalf];
  float st[kBtStage];
  float bA[2][2], bB[2][2];
  int c = c0;
  if (c0 < full_end) {
    load_x(c0, st);   // asked for first: loads retire in order, and staging X must not wait for K
    load_k(c0, kaA);
    __builtin_amdgcn_sched_barrier(0);
    store_x(0, st);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      bA[t][0] = xs[0][kBtHalf * h + t][r];
      bA[t][1] = xs[0][kBtHalf * h + t][32 + r];
    }
    const int64_t kstep = (int64_t)kBtChunk * ld, xstep = (int64_t)kBtChunk * ldm;
    const float* kp = K + (int64_t)(c0 + 1) * kstep;  // first rows of the chunk prepared next
    const float* xp = X + (int64_t)(c0 + 1) * xstep;
    for (; c + 2 < full_end; c += 2) {  // chunks c and c + 1 both have a successor to prepare
      chunk_step(with_next, 0, kaA, bA, kp, xp, kaB, bB);
      chunk_step(with_next, 1, kaB, bB, kp + kstep, xp + xstep, kaA, bA);
      kp += 2 * kstep;
      xp += 2 * xstep;
    }
    if (c + 1 < full_end) {  // two whole chunks left
      chunk_step(with_next, 0, kaA, bA, kp, xp, kaB, bB);
      chunk_step(last, 1, kaB, bB, kp, xp, kaA, bA);
    } else {                 // one
      chunk_step(last, 0, kaA, bA, kp, xp, kaB, bB);
    }
    __syncthreads();
  }
  if (full_end < c1) {
    load_k_masked(full_end, kaA);
    load_x_masked(full_end, st);
    __syncthreads();
    store_x(0, st);
    __syncthreads();
    multiply(0, kaA);
  }

  if (final) {
    float* dst = out + col0;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = 8 * (v / 4) + 4 * h + (v % 4);
        const int row = o0 + 4 * i + a;
        if (row < n) {
#pragma unroll
          for (int b = 0; b < 2; ++b) {
            const int col = 32 * b + r;
            if (col < m) {
              const int64_t idx = (int64_t)row * ldm + col;
              dst[idx] = marg[idx] / acc[a][b][v];
            }
          }
        }
      }
  } else if (o0 < n) {
    float* dst = out + ((int64_t)grp * slices + slice) * bt_partial_area(n) +
                 (int64_t)(o0 / kBtWideWaveTile) * kBtWaveTileFloats + 4 * lane;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          Pack<float> p;
#pragma unroll
          for (int j = 0; j < 4; ++j) p.e[j] = acc[a][b][4 * vq + j];
          store_pack(dst + ((a * 2 + b) * 4 + vq) * 256, p);
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
// Grid slices of the contraction range.  The wide kernel keeps one workgroup per compute unit
// busy (one wave per SIMD), the 64 x 64 kernel two.
static int batched_splits_wide(int n, int groups) {
  int cus = device_cu_count();
  if (cus < 1) cus = 256;
  const int tiles = ((n + kBtWideTile - 1) / kBtWideTile) * groups;
  // One workgroup (one wave per SIMD) per compute unit.  The grid runs in rounds of `cus`
  // workgroups: take the slice count whose last round is fullest, a little in favour of fewer
  // slices (every slice writes and re-reads one partial tile).
  const int nchunks = (n + kBtChunk - 1) / kBtChunk;
  int max_s = nchunks / 4 > 0 ? nchunks / 4 : 1;  // at least 4 chunks per slice
  if (max_s > 32) max_s = 32;
  int s = 1;
  double best = -1.0;
  for (int q = 1; q <= max_s; ++q) {
    const int wgs = tiles * q, rounds = (wgs + cus - 1) / cus;
    const double score = (double)wgs / ((double)rounds * cus) - 0.02 * q;
    if (score > best) best = score, s = q;
  }
  return s;
}

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
  const int groups = (m + kBtCols - 1) / kBtCols;
  const size_t wide = (size_t)batched_splits_wide(n, groups) * groups * (size_t)bt_partial_area(n);
  const size_t direct = (size_t)batched_splits(n) * (size_t)n * kBtCols;  // one group at a time
  return align_up((wide > direct ? wide : direct) * 4, 256);
}
static int64_t batched_ldt(int n) { return (int64_t)align_up((size_t)n, 64); }

// partial products + room for K^T
size_t batched_workspace_bytes(int n, int m) {
  return batched_partial_bytes(n, m) + align_up((size_t)n * (size_t)batched_ldt(n) * 4, 256) + 256;
}

// out[row][col] = marg[row][col] / sum_s partial[g][s][row][col] for every column group g
// (blockIdx.y).  A thread fetches one 128-bit pack of the wide kernel's partial layout (four rows,
// 4 apart, of one column) and adds it over the slices in slice order; four adjacent lanes then
// transpose their 4 x 4 values, so that each ends with four adjacent columns of one row and (vec:
// mtot a multiple of 4, marg and out 16-byte aligned) reads marg and writes out 128 bits at a
// time.  marg and out are n x mtot.
__global__ __launch_bounds__(256) void batched_reduce_kernel(const float* __restrict__ partial,
                                                             int slices, int n, int mtot,
                                                             const float* __restrict__ marg,
                                                             float* __restrict__ out, int vec) {
  const int grp = blockIdx.y, col0 = grp * kBtCols;
  const int cols = mtot - col0 < kBtCols ? mtot - col0 : kBtCols;
  const int64_t area = bt_partial_area(n);  // a multiple of 8192: a workgroup is all in or all out
  const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (4 * f >= area) return;
  const int r = (int)(f & 31), b = (int)(f >> 5) & 1, h = (int)(f >> 6) & 1, vq = (int)(f >> 7) & 3;
  const int a = (int)(f >> 9) & 3, wt = (int)(f >> 11);
  const float* p = partial + (int64_t)grp * slices * area + (int64_t)wt * kBtWaveTileFloats +
                   4 * ((((a * 2 + b) * 4 + vq) * 2 + h) * 32 + r);
  Pack<float> s = load_pack(p);
  for (int k = 1; k < slices; ++k) {
    const Pack<float> y = load_pack(p + (int64_t)k * area);
#pragma unroll
    for (int e = 0; e < 4; ++e) s.e[e] += y.e[e];
  }
  lanes_transpose4(s.e, r);  // now: row index j = r % 4, columns 4 (r / 4) .. + 3 of block b
  const int row = wt * kBtWideWaveTile + 4 * (8 * vq + 4 * h + (r & 3)) + a;
  const int col = 32 * b + (r & ~3);
  if (row >= n || col >= cols) return;
  const int64_t o = (int64_t)row * mtot + col0 + col;
  if (vec) {  // cols is then a multiple of 4
    const Pack<float> mg = load_pack(marg + o);
#pragma unroll
    for (int e = 0; e < 4; ++e) s.e[e] = mg.e[e] / s.e[e];
    store_pack(out + o, s);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (col + e < cols) out[o + e] = marg[o + e] / s.e[e];
  }
}

// The same for one column group of the direct row kernel: dense partial tiles n * cols apart.
__global__ __launch_bounds__(256) void batched_rowreduce_kernel(const float* __restrict__ partial,
                                                                int slices, int n, int cols,
                                                                int64_t ldm,
                                                                const float* __restrict__ marg,
                                                                float* __restrict__ out) {
  const int64_t total = (int64_t)n * cols;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  float s = partial[idx];
  for (int k = 1; k < slices; ++k) s += partial[(int64_t)k * total + idx];
  const int64_t o = (idx / cols) * ldm + idx % cols;
  out[o] = marg[o] / s;
}

int run_sinkhorn_batched(const fsk_opts* o, const void* K, int64_t ldK, const void* A, const void* B,
                         void* U, void* V, void* workspace, size_t ws_bytes, const fsk_dp* dp,
                         hipStream_t st, const BatchedPoll* poll, void* tmp) {
  const int n = o->n, m = o->m;
  // the product kernels address K through 32-bit offsets from a per-chunk base (lane part + scalar
  // part span at most 32 rows of the chunk: 128 ldK bytes in fp32, 256 ldK in fp64, kept below 2^31
  // so that they also pass the descriptor's range field), and the n x m operand likewise
  if (ldK > (int64_t)1 << 22 || m > 1 << 20)
    return set_error(FSK_EUNSUPPORTED, "batched call takes a row pitch of K up to 2^22 elements and up to 2^20 "
                     "targets (got %lld, %d)", (long long)ldK, m);
  if (o->dtype == FSK_F64)
    return run_sinkhorn_batched_f64(o, K, ldK, A, B, U, V, workspace, ws_bytes, dp, st, poll, tmp);
  const int S = batched_splits(n);
  const size_t part_bytes = batched_partial_bytes(n, m);
  if (!workspace || ws_bytes < part_bytes)
    return set_error(FSK_EWORKSPACE, "batched call needs at least %zu workspace bytes (%zu to run at "
                     "full speed), got %zu", part_bytes, batched_workspace_bytes(n, m), ws_bytes);
  const float *Kf = (const float*)K, *Af = (const float*)A, *Bf = (const float*)B;
  float *Uf = (float*)U, *Vf = (float*)V, *part = (float*)workspace;
  // K^T in the workspace if it fits.  The choice rests on (n, m, workspace) alone -- not on the
  // iteration count -- so that a run split into several calls adds every sum in the same order
  // as the run done in one call (a one-iteration call pays the transpose: n^2 entries read and
  // written, about one extra product's time).
  const bool use_kt = workspace && ws_bytes >= batched_workspace_bytes(n, m) && o->max_iters >= 1;
  const int64_t ldt = batched_ldt(n);
  float* Kt = use_kt ? (float*)((char*)workspace + part_bytes) : nullptr;
  if (use_kt) {
    dim3 tg((n + 63) / 64, (n + 63) / 64);
    hipLaunchKernelGGL(transpose_kernel, tg, dim3(256), 0, st, Kf, ldK, n, Kt, ldt);
    FSK_LAUNCH_CHECK("transpose_kernel");
  }
  dim3 grid((n + kBtTile - 1) / kBtTile, S), block(256);
  // The m histogram columns go through the kernels in groups of up to 64 (the kernels' tile
  // width); a group costs one pass over K per product, so the time grows with ceil(m / 64).
  // The transposed-product kernel takes all groups in one launch and splits the contraction
  // range only as far as the grid still needs it (tiles x groups x slices ~ compute units).
  const int groups = (m + kBtCols - 1) / kBtCols;
  const int SW = batched_splits_wide(n, groups);
  dim3 gridw(((n + kBtWideTile - 1) / kBtWideTile) * SW * groups);
  auto reduce_all = [&](const float* marg, float* dst) -> int {
    const int64_t packs = bt_partial_area(n) / 4;
    const int vec = m % 4 == 0 && (uintptr_t)marg % 16 == 0 && (uintptr_t)dst % 16 == 0;
    hipLaunchKernelGGL(batched_reduce_kernel, dim3((unsigned)((packs + 255) / 256), groups), dim3(256), 0, st,
                       (const float*)part, SW, n, m, marg, dst, vec);
    FSK_LAUNCH_CHECK("batched_reduce_kernel");
    return FSK_OK;
  };
  auto wide = [&](const float* Km, int64_t ldm_k, const float* X, const float* marg, float* dst,
                  const char* what) -> int {
    const bool xvec = m % 4 == 0 && (uintptr_t)X % 16 == 0;  // 128-bit staging of the n x m operand
    if (xvec)
      hipLaunchKernelGGL(batched_prod_wide_kernel<true>, gridw, block, 0, st, Km, ldm_k, n, m, X, marg,
                         SW == 1 ? dst : part, SW == 1 ? 1 : 0, SW, groups);
    else
      hipLaunchKernelGGL(batched_prod_wide_kernel<false>, gridw, block, 0, st, Km, ldm_k, n, m, X, marg,
                         SW == 1 ? dst : part, SW == 1 ? 1 : 0, SW, groups);
    FSK_LAUNCH_CHECK(what);
    if (SW > 1) FSK_TRY(reduce_all(marg, dst));
    return FSK_OK;
  };
  auto u_update = [&](void* dst_v) -> int {
    float* dst = (float*)dst_v;
    if (use_kt) return wide(Kt, ldt, Vf, Af, dst, "batched_prod_wide_kernel (K V)");  // Q = K V on K^T
    for (int c0 = 0; c0 < m; c0 += kBtCols) {  // direct row walk, one column group per launch
      const int cols = m - c0 < kBtCols ? m - c0 : kBtCols;
      hipLaunchKernelGGL(batched_rowprod_kernel, grid, block, 0, st, Kf, ldK, n, cols, (int64_t)m,
                         (const float*)Vf + c0, Af + c0, S == 1 ? dst + c0 : part, S == 1 ? 1 : 0);
      FSK_LAUNCH_CHECK("batched_rowprod_kernel (K V)");
      if (S > 1) {
        const int64_t total = (int64_t)n * cols;
        hipLaunchKernelGGL(batched_rowreduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                           st, (const float*)part, S, n, cols, (int64_t)m, Af + c0, dst + c0);
        FSK_LAUNCH_CHECK("batched_rowreduce_kernel");
      }
    }
    return FSK_OK;
  };
  auto v_update = [&](void* dst) -> int {  // V = B ./ (K^T U)
    return wide(Kf, ldK, Uf, Bf, (float*)dst, "batched_prod_wide_kernel (K^T U)");
  };
  auto release = [&](int it, bool is_v) -> int {  // the release clips every row across ALL m targets
    if (!dp) return FSK_OK;
    return is_v ? launch_dp_release(FSK_F32, Vf, n, m, dp->clip_v, dp->sigma_v, dp->seed,
                                    dp->release0 + 2 * (uint64_t)it + 1, st)
                : launch_dp_release(FSK_F32, Uf, n, m, dp->clip_u, dp->sigma_u, dp->seed,
                                    dp->release0 + 2 * (uint64_t)it, st);
  };
  return batched_iterate(o, Af, Uf, Vf, poll, tmp, st, u_update, v_update, release);
}

// ------------------------------------------------------------------ error of a polled state
// partial[strip][k] = sum over the 256 rows i of the strip of A_ik |Uold_ik / Unew_ik - 1|, or of
// its square with `l2` (fp64, rows in increasing order per thread, then the four row lanes in order).
template <typename T>
__global__ __launch_bounds__(256) void batched_poll_partial_kernel(const T* __restrict__ A,
                                                                   const T* __restrict__ Uold,
                                                                   const T* __restrict__ Unew, int n,
                                                                   int m, double* __restrict__ partial,
                                                                   int l2) {
  __shared__ double sm[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int k = blockIdx.x * 64 + cl, strip = blockIdx.y;
  const int i1 = (strip + 1) * 256 < n ? (strip + 1) * 256 : n;
  double s = 0.0;
  if (k < m)
    for (int i = strip * 256 + rl; i < i1; i += 4) {
      const int64_t idx = (int64_t)i * m + k;
      const double term = (double)A[idx] * fabs((double)Uold[idx] / (double)Unew[idx] - 1.0);
      s += l2 ? term * term : term;
    }
  sm[rl][cl] = s;
  __syncthreads();
  if (rl == 0 && k < m) partial[(int64_t)strip * m + k] = ((sm[0][cl] + sm[1][cl]) + sm[2][cl]) + sm[3][cl];
}

// out[0] = max over columns of the strips' sum (strips in order), or of its square root with `l2`;
// NaN wins the maximum.
__global__ __launch_bounds__(256) void batched_poll_final_kernel(const double* __restrict__ partial,
                                                                 int strips, int m,
                                                                 double* __restrict__ out, int l2) {
  __shared__ double sm[256];
  double best = 0.0;
  bool bad = false;
  for (int k = threadIdx.x; k < m; k += 256) {
    double s = 0.0;
    for (int t = 0; t < strips; ++t) s += partial[(int64_t)t * m + k];
    if (l2) s = sqrt(s);
    if (!(s == s)) bad = true;
    best = s > best ? s : best;
  }
  sm[threadIdx.x] = bad ? NAN : best;
  __syncthreads();
  if (threadIdx.x == 0) {
    double r = 0.0;
    bool any_bad = false;
    for (int t = 0; t < 256; ++t) {
      if (!(sm[t] == sm[t])) any_bad = true;
      else r = sm[t] > r ? sm[t] : r;
    }
    out[0] = any_bad ? NAN : r;
  }
}

// ------------------------------------------------------------------ relaxed updates (Sec. 3.3)
__device__ __forceinline__ float relax_log2(float x) { return log2f(x); }
__device__ __forceinline__ double relax_log2(double x) { return log2(x); }
__device__ __forceinline__ float relax_exp2(float x) { return exp2f(x); }
__device__ __forceinline__ double relax_exp2(double x) { return exp2(x); }

template <typename T>
__global__ __launch_bounds__(256) void batched_relax_kernel(T* __restrict__ X, const T* __restrict__ Xnew,
                                                            int64_t count, T eta, int geometric) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= count) return;
  const T old = X[e], fresh = Xnew[e];
  X[e] = geometric ? relax_exp2(fma(T(1) - eta, relax_log2(old), eta * relax_log2(fresh)))
                   : (T(1) - eta) * old + eta * fresh;
}

int launch_batched_relax(int dtype, void* X, const void* Xnew, int64_t count, double eta, int geometric,
                         hipStream_t st) {
  const dim3 grid((unsigned)((count + 255) / 256));
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((batched_relax_kernel<double>), grid, dim3(256), 0, st, (double*)X, (const double*)Xnew,
                       count, eta, geometric);
  else
    hipLaunchKernelGGL((batched_relax_kernel<float>), grid, dim3(256), 0, st, (float*)X, (const float*)Xnew,
                       count, (float)eta, geometric);
  FSK_LAUNCH_CHECK("batched_relax_kernel");
  return FSK_OK;
}

size_t batched_poll_scratch_doubles(int n, int m) { return 8 + (size_t)((n + 255) / 256) * (size_t)m; }

int launch_batched_poll_error(int dtype, const void* A, const void* Uold, const void* Unew, int n,
                              int m, double* scratch, hipStream_t st, bool l2) {
  const int strips = (n + 255) / 256;
  dim3 grid((m + 63) / 64, strips);
  double* partial = scratch + 8;
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((batched_poll_partial_kernel<double>), grid, dim3(256), 0, st, (const double*)A,
                       (const double*)Uold, (const double*)Unew, n, m, partial, l2 ? 1 : 0);
  else
    hipLaunchKernelGGL((batched_poll_partial_kernel<float>), grid, dim3(256), 0, st, (const float*)A,
                       (const float*)Uold, (const float*)Unew, n, m, partial, l2 ? 1 : 0);
  FSK_LAUNCH_CHECK("batched_poll_partial_kernel");
  hipLaunchKernelGGL(batched_poll_final_kernel, dim3(1), dim3(256), 0, st, (const double*)partial, strips, m,
                     scratch, l2 ? 1 : 0);
  FSK_LAUNCH_CHECK("batched_poll_final_kernel");
  return FSK_OK;
}

}  // namespace fsk
