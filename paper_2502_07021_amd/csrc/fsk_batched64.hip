// Multitarget Sinkhorn in fp64 for gfx950 (paper: Sec. 5.3.2; the paper's own multitarget runs
// store everything in double precision): the same plan as the fp32 path -- both products run
// as transposed products R = K^T X, the second one on a copy of K^T built once per call -- on
// v_mfma_f64_16x16x4_f64.
//
// MFMA 16x16x4 f64 operand layout (lane l of 64, measured): A[i = l%16][k = l/16],
// B[k = l/16][j = l%16], D[i = 4 v + l/16][j = l%16] for accumulator element v of 4.
//
// A wave owns a 64 x 64 output tile: 4 x 4 MFMA blocks, 64 fp64 accumulators (128 registers).
// A lane fetches two pairs of adjacent columns of K with two 128-bit loads, each of which
// covers 256 contiguous bytes (two whole cache lines) per quarter-wave: MFMA row i of block a is
// column o0 + 32 (a / 2) + 2 i + a % 2 of K.  A chunk is 32
// contraction indices = 8 MFMA k-steps; quarter-wave q supplies indices 8 q + e of the chunk at
// k-step e.  The 32 x 64 chunk of the n x m operand is shared by the workgroup's four waves
// through LDS (double buffered, one barrier per chunk, placed inside the chunk so that the matrix
// pipe has work queued while the waves meet); the next chunk's loads are spread between the
// MFMAs of the current one (a wave issues in order: a burst of loads would starve the matrix
// pipe).  K and X loads go through buffer descriptors (scalar base, scalar row offset, fixed
// lane offset), so no vector instruction besides the MFMAs, the loads and the LDS accesses is
// issued in the steady state.  The contraction range is split over grid slices; partial tiles go
// to the workspace in the order the wave's registers hold them and a reduction kernel adds
// them in slice order and divides.
#include "fsk_device.h"
#include "fsk_internal.h"

#include <type_traits>

namespace fsk {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int kB64Cols = 64;       // histogram columns per launch
constexpr int kB64WaveTile = 64;   // output rows per wave
constexpr int kB64Tile = 4 * kB64WaveTile;
constexpr int kB64Chunk = 32;      // contraction indices per chunk
constexpr int kB64Steps = kB64Chunk / 4;  // MFMA k-steps per chunk
constexpr int kB64Stage = kB64Chunk * kB64Cols / 256;

struct K4 { Pack<double> lo, hi; };  // four adjacent columns of one row of K

constexpr int kB64WaveTileDoubles = kB64WaveTile * kB64Cols;  // one wave's partial tile

// A partial tile is stored in the order the wave holds it: [MFMA block a][block b][half hf][lane]
// [2 accumulator elements], one 128-bit store per lane, a whole KiB per instruction.  Element t
// of that pack is accumulator element v = 2 hf + t, i.e. output row
// 64 wt + 32 (a / 2) + 2 (4 v + lane / 16) + a % 2 and column 16 b + lane % 16 of the wave's tile
// wt; the partial area of one (column group, slice) holds ceil(n / 64) such tiles.
__host__ __device__ inline int64_t b64_partial_area(int n) {
  return (int64_t)((n + kB64WaveTile - 1) / kB64WaveTile) * kB64WaveTileDoubles;
}

// X, marg and out (final) are n x mtot with row pitch mtot; the grid covers `groups` column groups
// of up to 64 columns, `slices` contraction slices and the row tiles.  final == 0: the partial
// product of (group g, slice s) goes to out + (g * slices + s) * b64_partial_area(n) in the layout
// described above.  XVEC: mtot is even and X is 16-byte aligned, so the X chunk is staged with
// 128-bit accesses.
template <bool XVEC>
__global__ __launch_bounds__(256) void batched_prod_f64_kernel(const double* __restrict__ K, int64_t ld,
                                                               int n, int mtot,
                                                               const double* __restrict__ X,
                                                               const double* __restrict__ marg,
                                                               double* __restrict__ out, int final,
                                                               int slices, int groups) {
  __shared__ __attribute__((aligned(16))) double xs[2][kB64Chunk][kB64Cols];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, q = lane >> 4;
  // 1-D grid, slice fastest: the workgroups of one contraction slice share rows of X in an XCD's L2
  const int slice = blockIdx.x % slices, grp = (blockIdx.x / slices) % groups;
  const int tile = blockIdx.x / (slices * groups);
  const int o0 = tile * kB64Tile + wave * kB64WaveTile;
  const int col0 = grp * kB64Cols;
  const int m = mtot - col0 < kB64Cols ? mtot - col0 : kB64Cols;  // columns of this group
  const int64_t ldm = mtot;
  X += col0;
  marg += col0;

  const int nchunks = (n + kB64Chunk - 1) / kB64Chunk;
  const int per = (nchunks + slices - 1) / slices;
  int c0 = slice * per;
  int c1 = c0 + per < nchunks ? c0 + per : nchunks;
  if (c0 > c1) c0 = c1;
  int full_end = n / kB64Chunk < c1 ? n / kB64Chunk : c1;
  if (full_end < c0) full_end = c0;

  doublex4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[a][b][v] = 0.0;

  // two 16-byte column pairs per lane, each clamped inside the row pitch (clamped duplicates
  // only feed output rows >= n, which are never stored)
  const int jmax = (int)ld - 2;
  const int j0 = o0 + 2 * r < jmax ? o0 + 2 * r : jmax;
  const int j1 = o0 + 32 + 2 * r < jmax ? o0 + 32 + 2 * r : jmax;
  const double* kc0 = K + j0;
  const double* kc1 = K + j1;
  // Addresses are split into a byte offset that belongs to the lane (its columns and its
  // quarter-wave's row inside a chunk; 32 bits, formed once) and a wave-uniform part: the
  // chunk's first row (the base of a buffer descriptor, advanced once per chunk on the scalar
  // unit) plus e row pitches for k-step e (a scalar offset).
  const uint32_t ldb = (uint32_t)(ld * 8), ldmb = (uint32_t)(ldm * 8);
  const uint32_t kb0 = (uint32_t)(((int64_t)(kB64Steps * q) * ld + j0) * 8);
  const uint32_t kb1 = (uint32_t)(((int64_t)(kB64Steps * q) * ld + j1) * 8);
  auto k_at = [&](const double* row, uint32_t lane_bytes) {
    return reinterpret_cast<const double*>(reinterpret_cast<const char*>(row) + lane_bytes);
  };
  auto load_k = [&](int c, K4(&ka)[kB64Steps]) {
    const double* row = K + (int64_t)c * kB64Chunk * ld;
#pragma unroll
    for (int e = 0; e < kB64Steps; ++e, row += ld) {
      ka[e].lo = load_pack_stream(k_at(row, kb0));
      ka[e].hi = load_pack_stream(k_at(row, kb1));
    }
  };
  auto load_k_masked = [&](int c, K4(&ka)[kB64Steps]) {
    const int first = c * kB64Chunk + kB64Steps * q;
#pragma unroll
    for (int e = 0; e < kB64Steps; ++e) {
      const bool ok = first + e < n;
      const int64_t row = ok ? first + e : n - 1;
      Pack<double> lo = load_pack(kc0 + row * ld), hi = load_pack(kc1 + row * ld);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        lo.e[t] = ok ? lo.e[t] : 0.0;
        hi.e[t] = ok ? hi.e[t] : 0.0;
      }
      ka[e].lo = lo;
      ka[e].hi = hi;
    }
  };

  const int sc = tid & 63, sk = tid >> 6;
  const double* xcol = X + (sc < m ? sc : m - 1);
  const uint32_t xb = (uint32_t)(((int64_t)sk * ldm + (sc < m ? sc : m - 1)) * 8);  // lane's bytes
  auto load_x = [&](int c, double(&st)[kB64Stage]) {
    const double* row = X + (int64_t)c * kB64Chunk * ldm;
#pragma unroll
    for (int i = 0; i < kB64Stage; ++i, row += 4 * ldm) st[i] = *k_at(row, xb);
  };
  auto load_x_masked = [&](int c, double(&st)[kB64Stage]) {
#pragma unroll
    for (int i = 0; i < kB64Stage; ++i) {
      const int kk = c * kB64Chunk + sk + 4 * i;
      const double val = xcol[(int64_t)(kk < n ? kk : n - 1) * ldm];
      st[i] = kk < n ? val : 0.0;
    }
  };
  auto store_x = [&](int buf, const double(&st)[kB64Stage]) {
#pragma unroll
    for (int i = 0; i < kB64Stage; ++i) xs[buf][sk + 4 * i][sc] = st[i];
  };
  // vector form of the staging: thread = (two columns from 2 xq, rows xr + 8 i), four 128-bit packs
  const int xr = tid >> 5, xq = tid & 31;
  const int xc2 = 2 * xq + 1 < m ? 2 * xq : (m >= 2 ? m - 2 : 0);
  const uint32_t xvb = (uint32_t)(((int64_t)xr * ldm + xc2) * 8);
  auto store_xv = [&](int buf, const Pack<double>(&sv)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) store_pack(&xs[buf][xr + 8 * i][2 * xq], sv[i]);
  };

  // B operands of k-step e of the chunk in xs[buf]
  auto read_b = [&](int buf, int e, double(&bv)[4]) {
#pragma unroll
    for (int b = 0; b < 4; ++b) bv[b] = xs[buf][kB64Steps * q + e][16 * b + r];
  };
  auto mfma_step = [&](const K4& k4, const double(&bv)[4]) {
    const double av[4] = {k4.lo.e[0], k4.lo.e[1], k4.hi.e[0], k4.hi.e[1]};
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[a], bv[b], acc[a][b], 0, 0, 0);
  };
  auto multiply = [&](int buf, const K4(&ka)[kB64Steps]) {
    double bv[kB64Steps][4];
#pragma unroll
    for (int e = 0; e < kB64Steps; ++e) read_b(buf, e, bv[e]);
#pragma unroll
    for (int e = 0; e < kB64Steps; ++e) mfma_step(ka[e], bv[e]);
  };
  // One chunk of the steady state: the MFMAs of the chunk in `ka` / xs[buf], whose first two
  // k-steps' B operands arrive in `bcur`.  With NEXT, everything the following chunk needs is
  // spread between them: its X rows (from `xrow`) are requested first -- before any K load of
  // this chunk, so that waiting for them later does not also wait for K loads issued since (the
  // memory counter retires loads in order) --, two K loads (rows from `krow` on) follow every
  // k-step, the X values go to xs[buf ^ 1] and the workgroup meets at a barrier after k-step
  // kB64Steps - 2, and the following chunk's first two k-steps' B operands are read (into `bnext`)
  // before the last k-step.  The matrix pipe therefore never drains at a chunk boundary: no wait
  // for memory, for the barrier or for LDS stands between the last MFMA of one chunk and the first
  // of the next.  Two LDS buffers suffice: every read of xs[buf] has completed (the barrier's
  // own wait) before any wave passes the barrier after which xs[buf] is written again.
  auto chunk_step = [&](auto next_tag, int buf, const K4(&ka)[kB64Steps], const double(&bcur)[2][4],
                        const double* krow, const double* xrow, K4(&kn)[kB64Steps],
                        double(&bnext)[2][4]) {
    constexpr bool NEXT = decltype(next_tag)::value;
    static_assert(kB64Stage == kB64Steps, "two X loads on each of the first kB64Steps / 2 k-steps");
    double bv[kB64Steps][4];
    double stn[kB64Stage];
    Pack<double> svn[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) bv[0][b] = bcur[0][b], bv[1][b] = bcur[1][b];
    const __amdgpu_buffer_rsrc_t rk = buffer_over(krow), rx = buffer_over(xrow);
    if (NEXT && XVEC) {
#pragma unroll
      for (int i = 0; i < 4; ++i) svn[i] = buffer_load_pack<double, false>(rx, xvb, 8 * i * ldmb);
    }
#pragma unroll
    for (int e = 0; e < kB64Steps; ++e) {
      if (NEXT && e == kB64Steps - 1) {  // after the barrier: the next chunk's first operands
        read_b(buf ^ 1, 0, bnext[0]);
        read_b(buf ^ 1, 1, bnext[1]);
      }
      mfma_step(ka[e], bv[e]);
      if (e + 2 < kB64Steps) read_b(buf, e + 2, bv[e + 2]);
      if (NEXT) {
        kn[e].lo = buffer_load_pack<double, true>(rk, kb0, e * ldb);
        kn[e].hi = buffer_load_pack<double, true>(rk, kb1, e * ldb);
        if (!XVEC && e < kB64Steps / 2) {
          stn[2 * e] = *k_at(xrow + (int64_t)8 * e * ldm, xb);
          stn[2 * e + 1] = *k_at(xrow + (int64_t)(8 * e + 4) * ldm, xb);
        }
        if (e == kB64Steps - 2) {
          if (XVEC) store_xv(buf ^ 1, svn); else store_x(buf ^ 1, stn);
          __syncthreads();
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  const std::true_type with_next;
  const std::false_type last;

  // Empty statements that name the accumulators as accumulation registers: left alone, the
  // register allocator carries them across the loop's back edge in ordinary vector registers
  // and copies all 128 of them to the accumulation file and back on every trip.
  auto pin_acc = [&]() {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) asm volatile("" : "+a"(acc[a][b]));
  };

  K4 kaA[kB64Steps], kaB[kB64Steps];
  double st[kB64Stage];
  double bA[2][4], bB[2][4];
  int c = c0;
  if (c0 < full_end) {
    load_x(c0, st);   // asked for first: loads retire in order, and staging X must not wait for K
    load_k(c0, kaA);
    __builtin_amdgcn_sched_barrier(0);
    store_x(0, st);
    __syncthreads();
    read_b(0, 0, bA[0]);
    read_b(0, 1, bA[1]);
    pin_acc();
    const int64_t kstep = (int64_t)kB64Chunk * ld, xstep = (int64_t)kB64Chunk * ldm;
    const double* kp = K + (int64_t)(c0 + 1) * kstep;  // first rows of the chunk prepared next
    const double* xp = X + (int64_t)(c0 + 1) * xstep;
    for (; c + 2 < full_end; c += 2) {  // chunks c and c + 1 both have a successor to prepare
      pin_acc();
      chunk_step(with_next, 0, kaA, bA, kp, xp, kaB, bB);
      chunk_step(with_next, 1, kaB, bB, kp + kstep, xp + xstep, kaA, bA);
      kp += 2 * kstep;
      xp += 2 * xstep;
      pin_acc();
    }
    if (c + 1 < full_end) {  // two whole chunks left
      chunk_step(with_next, 0, kaA, bA, kp, xp, kaB, bB);
      chunk_step(last, 1, kaB, bB, kp, xp, kaA, bA);
    } else {                 // one
      chunk_step(last, 0, kaA, bA, kp, xp, kaB, bB);
    }
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

  if (final) {
    double* dst = out + col0;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int i = 4 * v + q;  // MFMA row of accumulator element v
        const int row = o0 + 32 * (a >> 1) + 2 * i + (a & 1);
        if (row < n) {
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const int col = 16 * b + r;
            if (col < m) {
              const int64_t idx = (int64_t)row * ldm + col;
              dst[idx] = marg[idx] / acc[a][b][v];
            }
          }
        }
      }
  } else if (o0 < n) {
    double* dst = out + ((int64_t)grp * slices + slice) * b64_partial_area(n) +
                  (int64_t)(o0 / kB64WaveTile) * kB64WaveTileDoubles + 2 * lane;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          Pack<double> p;
          p.e[0] = acc[a][b][2 * hf];
          p.e[1] = acc[a][b][2 * hf + 1];
          store_pack(dst + ((a * 4 + b) * 2 + hf) * 128, p);
        }
  }
}

__global__ __launch_bounds__(256) void transpose_f64_kernel(const double* __restrict__ K, int64_t ld,
                                                            int n, double* __restrict__ Kt, int64_t ldt) {
  __shared__ double tile[64][65];
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

// out[row][col] = marg[row][col] / sum_s partial[g][s][row][col] for every column group g
// (blockIdx.y), the slices added in slice order.  A thread fetches one 128-bit pack of the product
// kernel's partial layout (two rows, 8 apart, of one column); two adjacent lanes then exchange
// one value each, so that each ends with two adjacent columns of one row and (vec: mtot even,
// marg and out 16-byte aligned) reads marg and writes out 128 bits at a time.  marg and out
// are n x mtot.
__global__ __launch_bounds__(256) void batched_reduce_f64_kernel(const double* __restrict__ partial,
                                                                 int slices, int n, int mtot,
                                                                 const double* __restrict__ marg,
                                                                 double* __restrict__ out, int vec) {
  const int grp = blockIdx.y, col0 = grp * kB64Cols;
  const int cols = mtot - col0 < kB64Cols ? mtot - col0 : kB64Cols;
  const int64_t area = b64_partial_area(n);  // a multiple of 4096: a workgroup is all in or all out
  const int64_t f = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (2 * f >= area) return;
  const int r = (int)(f & 15), b = (int)(f >> 4) & 3, q = (int)(f >> 6) & 3, hf = (int)(f >> 8) & 1;
  const int a = (int)(f >> 9) & 3, wt = (int)(f >> 11);
  const double* p = partial + (int64_t)grp * slices * area + (int64_t)wt * kB64WaveTileDoubles +
                    2 * ((((a * 4 + b) * 2 + hf) * 4 + q) * 16 + r);
  Pack<double> s = load_pack(p);
  for (int k = 1; k < slices; ++k) {
    const Pack<double> y = load_pack(p + (int64_t)k * area);
    s.e[0] += y.e[0];
    s.e[1] += y.e[1];
  }
  lanes_transpose2(s.e, r);  // now: accumulator element v = 2 hf + r % 2, columns 2 (r / 2), + 1 of block b
  const int row = wt * kB64WaveTile + 32 * (a >> 1) + 2 * (4 * (2 * hf + (r & 1)) + q) + (a & 1);
  const int col = 16 * b + (r & ~1);
  if (row >= n || col >= cols) return;
  const int64_t o = (int64_t)row * mtot + col0 + col;
  if (vec) {  // cols is then even
    const Pack<double> mg = load_pack(marg + o);
    s.e[0] = mg.e[0] / s.e[0];
    s.e[1] = mg.e[1] / s.e[1];
    store_pack(out + o, s);
  } else {
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (col + e < cols) out[o + e] = marg[o + e] / s.e[e];
  }
}

static int b64_groups(int m) { return (m + kB64Cols - 1) / kB64Cols; }

static int b64_splits(int n, int groups) {
  int cus = device_cu_count();
  if (cus < 1) cus = 256;
  const int tiles = ((n + kB64Tile - 1) / kB64Tile) * groups;
  // One workgroup (one wave per SIMD) per compute unit.  The grid runs in rounds of `cus`
  // workgroups: take the slice count whose last round is fullest, a little in favour of fewer
  // slices (every slice writes and re-reads one partial tile).
  const int nchunks = (n + kB64Chunk - 1) / kB64Chunk;
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
static size_t b64_partial_bytes(int n, int m) {
  const int groups = b64_groups(m);
  return align_up((size_t)b64_splits(n, groups) * groups * (size_t)b64_partial_area(n) * 8, 256);
}
static int64_t b64_ldt(int n) { return (int64_t)align_up((size_t)n, 32); }

size_t batched_f64_workspace_bytes(int n, int m) {
  return b64_partial_bytes(n, m) + align_up((size_t)n * (size_t)b64_ldt(n) * 8, 256) + 256;
}

int run_sinkhorn_batched_f64(const fsk_opts* o, const void* K, int64_t ldK, const void* A, const void* B,
                             void* U, void* V, void* workspace, size_t ws_bytes, const fsk_dp* dp,
                             hipStream_t st, const BatchedPoll* poll, void* tmp) {
  const int n = o->n, m = o->m;
  const size_t need = batched_f64_workspace_bytes(n, m);
  if (!workspace || ws_bytes < need)
    return set_error(FSK_EWORKSPACE, "fp64 batched call needs %zu workspace bytes (partial products and a "
                     "transposed copy of K), got %zu", need, ws_bytes);
  const double *Kd = (const double*)K, *Ad = (const double*)A, *Bd = (const double*)B;
  double *Ud = (double*)U, *Vd = (double*)V, *part = (double*)workspace;
  const int64_t ldt = b64_ldt(n);
  double* Kt = (double*)((char*)workspace + b64_partial_bytes(n, m));
  if (o->max_iters > 0) {
    dim3 tg((n + 63) / 64, (n + 63) / 64);
    hipLaunchKernelGGL(transpose_f64_kernel, tg, dim3(256), 0, st, Kd, ldK, n, Kt, ldt);
    FSK_LAUNCH_CHECK("transpose_f64_kernel");
  }
  // all column groups of 64 in one launch; the contraction range is split only as far as the
  // grid still needs it (tiles x groups x slices ~ compute units)
  const int groups = b64_groups(m), S = b64_splits(n, groups);
  dim3 grid(((n + kB64Tile - 1) / kB64Tile) * S * groups), block(256);
  auto product = [&](const double* Km, int64_t ldm_k, const double* X, const double* marg,
                     double* dst) -> int {
    const bool xvec = m % 2 == 0 && (uintptr_t)X % 16 == 0;  // 128-bit staging of the n x m operand
    if (xvec)
      hipLaunchKernelGGL(batched_prod_f64_kernel<true>, grid, block, 0, st, Km, ldm_k, n, m, X, marg,
                         S == 1 ? dst : part, S == 1 ? 1 : 0, S, groups);
    else
      hipLaunchKernelGGL(batched_prod_f64_kernel<false>, grid, block, 0, st, Km, ldm_k, n, m, X, marg,
                         S == 1 ? dst : part, S == 1 ? 1 : 0, S, groups);
    FSK_LAUNCH_CHECK("batched_prod_f64_kernel");
    if (S > 1) {
      const int64_t packs = b64_partial_area(n) / 2;
      const int vec = m % 2 == 0 && (uintptr_t)marg % 16 == 0 && (uintptr_t)dst % 16 == 0;
      hipLaunchKernelGGL(batched_reduce_f64_kernel, dim3((unsigned)((packs + 255) / 256), groups),
                         dim3(256), 0, st, (const double*)part, S, n, m, marg, dst, vec);
      FSK_LAUNCH_CHECK("batched_reduce_f64_kernel");
    }
    return FSK_OK;
  };
  auto u_update = [&](void* dst) -> int {  // U = A ./ (K V) as the transposed product of K^T
    return product(Kt, ldt, Vd, Ad, (double*)dst);
  };
  auto v_update = [&](void* dst) -> int { return product(Kd, ldK, Ud, Bd, (double*)dst); };  // V = B ./ (K^T U)
  auto release = [&](int it, bool is_v) -> int {
    if (!dp) return FSK_OK;
    return is_v ? launch_dp_release(FSK_F64, Vd, n, m, dp->clip_v, dp->sigma_v, dp->seed,
                                    dp->release0 + 2 * (uint64_t)it + 1, st)
                : launch_dp_release(FSK_F64, Ud, n, m, dp->clip_u, dp->sigma_u, dp->seed,
                                    dp->release0 + 2 * (uint64_t)it, st);
  };
  return batched_iterate(o, Ad, Ud, Vd, poll, tmp, st, u_update, v_update, release);
}

}  // namespace fsk
