// Dense Sinkhorn kernels for gfx950: the two kernel products of one iteration
// (paper: Sec. 1 scaling form, Algorithm 1 loop body, Sec. 4.1 local operations)
//
//     q = K v,  u = a ./ q            (row pass)
//     r = K^T u, v = b ./ r           (column pass)
//
// as (1) a generic two-pass pair that works for any n and any row / column range
// (one worker's slab, Sec. 3.1), and (2) a fused one-pass kernel that reads K
// once per iteration: a workgroup keeps whole rows in registers, finishes u on
// them and immediately accumulates their contribution to K^T u.
//
// All of them are HBM-bound streams over K with 128-bit loads; sums use a fixed
// order (per-thread sequential, wave butterfly, per-wave slots added in index
// order), no atomics.
#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

// ============================================================== row pass (generic)
// One workgroup of 256 threads takes ROWS consecutive rows (2 or 4: see the launcher); thread t
// walks the 16-byte packs t, t+256, ... of each row, so a wave reads 1 KiB contiguous per
// load and v is fetched once for all ROWS rows.
// blockIdx.y = slab: the launch covers gridDim.y row slabs of `rows` rows each, slab y being
// rows [y*rows, (y+1)*rows) of K, marg, old, out and err_out -- the row blocks of the c clients
// (Sec. 3.1) in one grid.
// blockIdx.z = column block (2D block grid): block z multiplies columns [z*n, (z+1)*n) of K by
// entries [z*n, (z+1)*n) of vin and writes its products to out + z*out_block_stride.
// VIEW: slab y is client y working on ITS view of the vector (Sec. 3.2.1, "a current global view
// ... obtained from the previous collective"; Algorithm 3's cached slices): entry j comes from
// `vown` inside the client's own index range [y*rows, (y+1)*rows) and from `vin` elsewhere.
template <typename T, int ROWS, bool VIEW>
__global__ __launch_bounds__(256) void rowpass_kernel(const T* __restrict__ K, int64_t ld, int n,
                                                      int rows, const T* __restrict__ vin,
                                                      const T* __restrict__ vown, const T* marg,
                                                      const T* old, T* out, int epi, T eta,
                                                      T* err_out, int64_t out_block_stride) {
  // err_out (may be null): |old_i * product_i - marg_i|, the row-marginal error term of the
  // scalings as they stood before this update (old is read before out is written: out may
  // alias old).
  constexpr int W = Pack<T>::W;
  constexpr int NT = 256, NW = NT / kWave;
  const int tid = threadIdx.x;
  const int r_base = blockIdx.x * ROWS;
  const int nvec_full = n / W;
  const int64_t slab0 = (int64_t)blockIdx.y * rows;  // first row of this slab
  const int own_lo = (int)slab0, own_hi = own_lo + rows;
  K += slab0 * ld + (int64_t)blockIdx.z * n;
  vin += (int64_t)blockIdx.z * n;
  out += (int64_t)blockIdx.z * out_block_stride;

  const T* rowp[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    int row = r_base + r;
    row = row < rows ? row : rows - 1;  // clamp: duplicates are computed and dropped
    rowp[r] = K + (int64_t)row * ld;
  }
  T acc[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) acc[r] = T(0);

  // two trips in flight in the plain pass, one where the view doubles the loads of v (local steps
  // at n = 32768, c = 8: 1251 against 1268 us per iteration; the plain pass loses 0.7 % with one)
  constexpr int kTrips = VIEW ? 1 : 2;
#pragma unroll kTrips
  for (int c = tid; c < nvec_full; c += NT) {
    Pack<T> vv = load_pack(vin + (int64_t)c * W);
    if (VIEW) {
      const Pack<T> vo = load_pack(vown + (int64_t)c * W);
#pragma unroll
      for (int e = 0; e < W; ++e) {
        const int j = c * W + e;
        vv.e[e] = (j >= own_lo && j < own_hi) ? vo.e[e] : vv.e[e];
      }
    }
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const Pack<T> kk = load_pack_stream(rowp[r] + (int64_t)c * W);
#pragma unroll
      for (int e = 0; e < W; ++e) acc[r] = fma(kk.e[e], vv.e[e], acc[r]);
    }
  }
  if (tid == 0) {  // ragged tail of fewer than W columns
    for (int j = nvec_full * W; j < n; ++j) {
      const T vj = (VIEW && j >= own_lo && j < own_hi) ? vown[j] : vin[j];
#pragma unroll
      for (int r = 0; r < ROWS; ++r) acc[r] = fma(rowp[r][j], vj, acc[r]);
    }
  }

  __shared__ T red[ROWS][NW];
  const int lane = tid & (kWave - 1), wave = tid / kWave;
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    const T s = wave_sum(acc[r]);
    if (lane == 0) red[r][wave] = s;
  }
  __syncthreads();
  if (tid < ROWS) {
    const int row = r_base + tid;
    if (row < rows) {
      const int64_t g = slab0 + row;
      T q = T(0);
#pragma unroll
      for (int k = 0; k < NW; ++k) q += red[tid][k];
      const T mg = epi_needs_marg(epi) ? marg[g] : T(0);
      const T od = (epi_needs_old(epi) || err_out) ? old[g] : T(0);
      if (err_out) err_out[g] = fsk_abs(od * q - marg[g]);
      out[g] = apply_epilogue(epi, mg, q, od, eta);
    }
  }
}

template <typename T>
static int rowpass_typed(const void* K, int64_t ld, int n, int rows, int slabs, const void* vin,
                         const void* vown, const void* marg, const void* old, void* out, int epi,
                         double eta, void* err_out, hipStream_t stream, int col_blocks = 1,
                         int64_t out_block_stride = 0) {
  if (rows <= 0 || slabs <= 0 || col_blocks <= 0) return FSK_OK;
  // Rows per workgroup (the sums are per row, so the choice changes no bit): two for the plain
  // pass (n = 16384: 348 us per iteration of the two-pass flow against 356 with four, fp64 629
  // against 645; n = 32768: 1235 against 1249), four where every entry of v is picked from one
  // of two vectors first (with two that variant loses 4 % at n = 32768).
  constexpr int kRowsPlain = 2, kRowsView = 4;
  dim3 block(256);
  if (vown) {
    dim3 grid((rows + kRowsView - 1) / kRowsView, slabs, col_blocks);
    hipLaunchKernelGGL((rowpass_kernel<T, kRowsView, true>), grid, block, 0, stream, (const T*)K, ld, n,
                       rows, (const T*)vin, (const T*)vown, (const T*)marg, (const T*)old, (T*)out,
                       epi, (T)eta, (T*)err_out, out_block_stride);
  } else {
    dim3 grid((rows + kRowsPlain - 1) / kRowsPlain, slabs, col_blocks);
    hipLaunchKernelGGL((rowpass_kernel<T, kRowsPlain, false>), grid, block, 0, stream, (const T*)K, ld, n,
                       rows, (const T*)vin, (const T*)nullptr, (const T*)marg, (const T*)old,
                       (T*)out, epi, (T)eta, (T*)err_out, out_block_stride);
  }
  FSK_LAUNCH_CHECK("rowpass_kernel");
  return FSK_OK;
}

int launch_rowpass(int dtype, const void* K, int64_t ld, int n, int rows, const void* vin,
                   const void* marg, const void* old, void* out, int epi, double eta,
                   hipStream_t stream, void* err_out) {
  return dtype == FSK_F64 ? rowpass_typed<double>(K, ld, n, rows, 1, vin, nullptr, marg, old, out,
                                                  epi, eta, err_out, stream)
                          : rowpass_typed<float>(K, ld, n, rows, 1, vin, nullptr, marg, old, out, epi,
                                                 eta, err_out, stream);
}

int launch_rowpass_colblocks(int dtype, const void* K, int64_t ld, int ncols, int rows, int blocks,
                             const void* vin, void* out, int64_t out_block_stride,
                             hipStream_t stream) {
  if (blocks > 65535) return set_error(FSK_EUNSUPPORTED, "more than 65535 column blocks in one launch");
  return dtype == FSK_F64
             ? rowpass_typed<double>(K, ld, ncols, rows, 1, vin, nullptr, nullptr, nullptr, out,
                                     kEpiProduct, 1.0, nullptr, stream, blocks, out_block_stride)
             : rowpass_typed<float>(K, ld, ncols, rows, 1, vin, nullptr, nullptr, nullptr, out,
                                    kEpiProduct, 1.0, nullptr, stream, blocks, out_block_stride);
}

int launch_rowpass_slabs(int dtype, const void* K, int64_t ld, int n, int rows, int slabs,
                         const void* vin, const void* vown, const void* marg, const void* old,
                         void* out, int epi, double eta, hipStream_t stream, void* err_out) {
  if (slabs > 65535) return set_error(FSK_EUNSUPPORTED, "more than 65535 row slabs in one launch");
  return dtype == FSK_F64 ? rowpass_typed<double>(K, ld, n, rows, slabs, vin, vown, marg, old, out,
                                                  epi, eta, err_out, stream)
                          : rowpass_typed<float>(K, ld, n, rows, slabs, vin, vown, marg, old, out,
                                                 epi, eta, err_out, stream);
}

// ========================================================== column pass (generic)
// Grid (column tiles, row strips).  A thread owns PPT 16-byte packs of columns (256 packs
// apart, so a workgroup reads PPT x 4 KiB contiguous bytes of every row) and adds
// K[i][cols] * u[i] over the rows of its strip in increasing i; the strip partition depends
// only on the row count and every column is summed on its own, so a column-restricted launch
// (and either PPT) sums every column exactly like an unrestricted one.
// VIEW != 0: column j belongs to client j / um, who multiplies by ITS view of u: uown[i] for the
// rows i of its own index range, u[i] elsewhere (the transpose action of Algorithm 1 / 3 on a
// client's cached vector).  One launch then serves the column slabs of all clients.
// VIEW == 1: um is a multiple of the pack width, so the columns of a pack have one owner and the
// choice is made once per pack and row; VIEW == 2: any um, chosen per column.  Either way the
// kernel must keep the 8 waves per SIMD of the plain one: the grid is one full round of
// workgroups at that occupancy and a second, nearly empty round costs 25 % (792 against 622 us
// at n = 32768 when the view variant needed 71 registers).
template <typename T, int PPT, int VIEW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8))) void colpartial_kernel(const T* __restrict__ K, int64_t ld,
                                                         int rows, int vec_lo, int vec_hi,
                                                         const T* __restrict__ u,
                                                         const T* __restrict__ uown, int um,
                                                         T* __restrict__ partial, int64_t ld_ws) {
  constexpr int W = Pack<T>::W;
  const int vc0 = vec_lo + blockIdx.x * 256 * PPT + threadIdx.x;
  const int s = blockIdx.y;
  const int i0 = s * kColStrip;
  const int i1 = i0 + kColStrip < rows ? i0 + kColStrip : rows;
  if (vc0 >= vec_hi) return;  // no barrier below
  // packs past the end of the range are clamped to the thread's first pack: read again, not stored
  int64_t off[PPT];
#pragma unroll
  for (int k = 0; k < PPT; ++k) off[k] = (int64_t)(vc0 + k * 256 < vec_hi ? vc0 + k * 256 : vc0) * W;
  Pack<T> acc[PPT];
#pragma unroll
  for (int k = 0; k < PPT; ++k)
#pragma unroll
    for (int e = 0; e < W; ++e) acc[k].e[e] = T(0);
  const T* kp = K + (int64_t)i0 * ld;
  // [row_lo, row_lo + um): the index range of the client that owns row i (the same for the whole
  // workgroup, kept on the scalar unit); a column inside it is one of that client's own
  int row_lo = VIEW ? (i0 / um) * um : 0;
#pragma unroll 4
  for (int i = i0; i < i1; ++i) {
    const T ui = u[i];
    const T uo = VIEW ? uown[i] : T(0);
    if (VIEW && i >= row_lo + um) row_lo += um;
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      const Pack<T> kk = load_pack_stream(kp + off[k]);
      const T uk = (VIEW == 1 && (unsigned)((int)off[k] - row_lo) < (unsigned)um) ? uo : ui;
#pragma unroll
      for (int e = 0; e < W; ++e) {
        const T ue = (VIEW == 2 && (unsigned)((int)off[k] + e - row_lo) < (unsigned)um) ? uo : uk;
        acc[k].e[e] = fma(kk.e[e], ue, acc[k].e[e]);
      }
    }
    kp += ld;
  }
#pragma unroll
  for (int k = 0; k < PPT; ++k)
    if (vc0 + k * 256 < vec_hi) store_pack(partial + (int64_t)s * ld_ws + off[k], acc[k]);
}

template <typename T, int VIEW>
static int colpartial_typed(const void* K, int64_t ld, int n, int rows, int c0, int c1,
                            const void* u, const void* uown, int um, void* partial, int64_t ld_ws,
                            hipStream_t stream) {
  constexpr int W = Pack<T>::W;
  if (rows <= 0 || c1 <= c0) return FSK_OK;
  const int vec_lo = c0 / W, vec_hi = (c1 + W - 1) / W;
  (void)n;
  const int nvec = vec_hi - vec_lo;
  dim3 block(256);
  // wide and tall enough for >= 1024 workgroups of the wide shape: 16 KiB of every row per workgroup
  if (nvec >= 4096 && (int64_t)((nvec + 1023) / 1024) * col_strips(rows) >= 1024) {
    dim3 grid((nvec + 1023) / 1024, col_strips(rows));
    hipLaunchKernelGGL((colpartial_kernel<T, 4, VIEW>), grid, block, 0, stream, (const T*)K, ld, rows,
                       vec_lo, vec_hi, (const T*)u, (const T*)uown, um, (T*)partial, ld_ws);
  } else {
    dim3 grid((nvec + 255) / 256, col_strips(rows));
    hipLaunchKernelGGL((colpartial_kernel<T, 1, VIEW>), grid, block, 0, stream, (const T*)K, ld, rows,
                       vec_lo, vec_hi, (const T*)u, (const T*)uown, um, (T*)partial, ld_ws);
  }
  FSK_LAUNCH_CHECK("colpartial_kernel");
  return FSK_OK;
}

int launch_colpartial(int dtype, const void* K, int64_t ld, int n, int rows, int c0, int c1,
                      const void* u, void* partial, int64_t ld_ws, hipStream_t stream) {
  return dtype == FSK_F64
             ? colpartial_typed<double, 0>(K, ld, n, rows, c0, c1, u, nullptr, 1, partial, ld_ws, stream)
             : colpartial_typed<float, 0>(K, ld, n, rows, c0, c1, u, nullptr, 1, partial, ld_ws, stream);
}

int launch_colpartial_view(int dtype, const void* K, int64_t ld, int n, const void* u,
                           const void* uown, int um, void* partial, int64_t ld_ws,
                           hipStream_t stream) {
  if (um < 1) return set_error(FSK_EINVAL, "client block of %d columns", um);
  const bool whole_packs = um % pack_width(dtype) == 0;  // a pack of columns has one owner
  if (dtype == FSK_F64)
    return whole_packs ? colpartial_typed<double, 1>(K, ld, n, n, 0, n, u, uown, um, partial, ld_ws, stream)
                       : colpartial_typed<double, 2>(K, ld, n, n, 0, n, u, uown, um, partial, ld_ws, stream);
  return whole_packs ? colpartial_typed<float, 1>(K, ld, n, n, 0, n, u, uown, um, partial, ld_ws, stream)
                     : colpartial_typed<float, 2>(K, ld, n, n, 0, n, u, uown, um, partial, ld_ws, stream);
}

// ======================================================= partial sums -> result
// The partial rows are split into G contiguous groups (G = 4..32), each summed in increasing
// index, then the G group sums are added in group order.  G is a function of the number of
// partials and of the row pitch of the partial area alone, so the result does not depend on
// the column range, the alignment or the grid.  A workgroup is G x Q threads (Q = 256 / G);
// thread (g, q) sums group g for one 16-byte pack of columns, so a group row is read as Q
// contiguous packs and every thread has its whole group in flight at once.  Wide problems
// get few groups (long contiguous reads), narrow ones many (enough threads).
__host__ __device__ inline int colreduce_groups(int n_partials, int64_t pitch_packs) {
  int g = 4;
  while (g < 32 && pitch_packs * g < 65536 && 4 * g <= n_partials) g *= 2;
  return g;
}

template <typename T>
__global__ __launch_bounds__(256) void colreduce_kernel(const T* __restrict__ partial,
                                                        int64_t ld_ws, int n_partials, int c0,
                                                        int c1, const T* marg, const T* old, T* out,
                                                        int epi, T eta, int aligned, int groups) {
  // groups > 0: exactly that many groups (it divides n_partials): the sums of the 2D block grid,
  // block products first, then the blocks in block order
  constexpr int W = Pack<T>::W;
  const int G = groups > 0 ? groups : colreduce_groups(n_partials, ld_ws / W), Q = 256 / G;
  const int q = threadIdx.x % Q, g = threadIdx.x / Q;
  const int j = c0 + (blockIdx.x * Q + q) * W;  // first column of this thread's pack
  const int per = (n_partials + G - 1) / G;
  const int s0 = g * per;
  const int s1 = s0 + per < n_partials ? s0 + per : n_partials;
  const bool whole = aligned && j + W <= c1;  // the pack lies inside the range and is aligned
  Pack<T> acc;
#pragma unroll
  for (int e = 0; e < W; ++e) acc.e[e] = T(0);
  if (j < c1 && g < G) {
    const T* p = partial + (int64_t)s0 * ld_ws + j;
    if (whole) {
#pragma unroll 8
      for (int s = s0; s < s1; ++s) {
        const Pack<T> x = load_pack(p);
#pragma unroll
        for (int e = 0; e < W; ++e) acc.e[e] += x.e[e];
        p += ld_ws;
      }
    } else {
#pragma unroll 4
      for (int s = s0; s < s1; ++s) {
#pragma unroll
        for (int e = 0; e < W; ++e)
          if (j + e < c1) acc.e[e] += p[e];
        p += ld_ws;
      }
    }
  }
  __shared__ __align__(16) T sm[256 * W];
  store_pack(sm + threadIdx.x * W, acc);
  __syncthreads();
  if (g == 0 && j < c1) {
    Pack<T> r = load_pack(sm + q * W);
    for (int k = 1; k < G; ++k) {
      const Pack<T> x = load_pack(sm + (k * Q + q) * W);
#pragma unroll
      for (int e = 0; e < W; ++e) r.e[e] += x.e[e];
    }
#pragma unroll
    for (int e = 0; e < W; ++e)
      if (j + e < c1) {
        const T mg = epi_needs_marg(epi) ? marg[j + e] : T(0);
        const T od = epi_needs_old(epi) ? old[j + e] : T(0);
        out[j + e] = apply_epilogue(epi, mg, r.e[e], od, eta);
      }
  }
}

template <typename T>
static int colreduce_typed(const void* partial, int64_t ld_ws, int n_partials, int c0, int c1,
                           const void* marg, const void* old, void* out, int epi, double eta,
                           hipStream_t stream, int groups) {
  if (c1 <= c0) return FSK_OK;
  constexpr int W = Pack<T>::W;
  if (groups > 0 && (groups > 256 || n_partials % groups != 0))
    return set_error(FSK_EINVAL, "%d groups do not divide %d partial sums", groups, n_partials);
  const int G = groups > 0 ? groups : colreduce_groups(n_partials, ld_ws / W);
  const int cols_per_wg = 256 / G * W;
  const int aligned = ld_ws % W == 0 && ((uintptr_t)((const T*)partial + c0)) % 16 == 0;
  dim3 grid((c1 - c0 + cols_per_wg - 1) / cols_per_wg), block(256);
  hipLaunchKernelGGL((colreduce_kernel<T>), grid, block, 0, stream, (const T*)partial, ld_ws,
                     n_partials, c0, c1, (const T*)marg, (const T*)old, (T*)out, epi, (T)eta, aligned,
                     groups);
  FSK_LAUNCH_CHECK("colreduce_kernel");
  return FSK_OK;
}

int launch_colreduce(int dtype, const void* partial, int64_t ld_ws, int n_partials, int c0, int c1,
                     const void* marg, const void* old, void* out, int epi, double eta,
                     hipStream_t stream, int groups) {
  return dtype == FSK_F64
             ? colreduce_typed<double>(partial, ld_ws, n_partials, c0, c1, marg, old, out, epi, eta, stream, groups)
             : colreduce_typed<float>(partial, ld_ws, n_partials, c0, c1, marg, old, out, epi, eta, stream, groups);
}

__device__ __forceinline__ float fsk_log2(float x) { return log2f(x); }
__device__ __forceinline__ double fsk_log2(double x) { return (double)log2f((float)x); }  // never reached
__device__ __forceinline__ float fsk_exp2(float x) { return exp2f(x); }
__device__ __forceinline__ double fsk_exp2(double x) { return (double)exp2f((float)x); }  // never reached

// ============================================================ fused one-pass kernel
// One workgroup of 512 threads (8 waves, 2 per SIMD, up to 256 VGPRs each) per
// compute unit.  Thread t owns the packs t, t+512, ... of every row: VPT packs
// per row, R rows at a time, so a group of R rows (R*VPT = 16 packs = 64 VGPRs)
// sits in registers while the next group is in flight into a second register
// set.  v lives in LDS (up to 128 KiB of the 160 KiB), the thread's slice of the
// column accumulator in registers.  Per group: partial dot products, butterfly
// wave sums, one barrier, u = a ./ q, then acc += K_row * u from the same
// registers.  K is read exactly once.
//
// Rows are handed out in STRIPS: row block j (rows [j*m, (j+1)*m), Sec. 3.1) is cut into
// strips of h rows (the last one shorter if h does not divide m); a strip is streamed by
// `gb` workgroups (1 in production) which each leave one row of partial column sums for it.
// h is a function of (n, dtype) alone when the block height m is a multiple of it, so the
// strips -- hence every partial sum and the order the reduction adds them in -- are the
// same for every block count c: the iterates of c blocks equal those of c = 1 bit for bit
// (Proposition 1 holds in floating point too, not only in exact arithmetic).
constexpr int kFusedWindow = 5;

template <typename T, int VPT, int R, bool EXACT>
__global__ __launch_bounds__(512) void fused_kernel(const T* __restrict__ K, int64_t ld, int n,
                                                    int m, int h, int spb, int nvb, int gb,
                                                    int rotmul, const T* marg,
                                                    const T* __restrict__ vin, const T* old_u,
                                                    T* u_out, T* __restrict__ partial,
                                                    int64_t ld_ws, T eta, T* err_out) {
  // m: rows per row block; h: rows per strip; spb: strips per block; nvb: strips in all.
  // err_out (may be null): |old_u_i (K v)_i - marg_i| per row, the row-marginal error term of
  // the scalings as they stood before this update (free: the product is at hand).
  // VPT = ceil(packs per row / 512), so the packs of slots i < VPT - 1 are whole and inside the
  // row for every thread and only the last slot can hold a partial pack or none.
  // EXACT: n == VPT*512*W, the last slot is whole too and nothing is masked.
  // |eta| < 1 selects a relaxation (Sec. 3.3): eta > 0 the arithmetic one,
  // u <- (1-eta) u + eta a./(K v); eta < 0 the geometric one with parameter -eta,
  // u <- u^(1+eta) (a./(K v))^(-eta), evaluated as exp2 of the weighted log2's (a general pow
  // would not fit the kernel's register budget); fp32 only, the launcher refuses it in fp64.
  constexpr int W = Pack<T>::W;
  constexpr int NT = 512, NW = NT / kWave;
  extern __shared__ __align__(16) unsigned char fsk_smem[];
  T* v_lds = reinterpret_cast<T*>(fsk_smem);  // VPT*NT*W entries, zero beyond n
  T* red = v_lds + VPT * NT * W;              // [2][R][NW]

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  // The grid is `nb` teams of `gb` workgroups.  Team `team` owns the strips team, team + nb,
  // ...; inside a strip its row groups are dealt round-robin to the team's workgroups.
  const int G = gb, w = blockIdx.x % gb, team = blockIdx.x / gb, nb = gridDim.x / gb;
  const int nvec = (n + W - 1) / W, nvec_full = n / W;
  const int spv = ((h + R - 1) / R + G - 1) / G;          // steps this workgroup spends on one strip
  const int total = ((nvb - team + nb - 1) / nb) * spv;   // steps over all strips of the team
  const bool geom = eta < T(0);
  const T et = geom ? -eta : eta;
  const bool damped = et < T(1);

  // v is fetched here and goes to LDS further down, after the first K request has been issued
  Pack<T> vreg[VPT];
#pragma unroll
  for (int i = 0; i < VPT; ++i) {
    const int vi = i * NT + tid;
    Pack<T> p;
#pragma unroll
    for (int e = 0; e < W; ++e) p.e[e] = T(0);
    if (EXACT || i < VPT - 1 || vi < nvec_full) {
      p = load_pack(vin + (int64_t)vi * W);
    } else if (vi < nvec) {
#pragma unroll
      for (int e = 0; e < W; ++e)
        if (vi * W + e < n) p.e[e] = vin[vi * W + e];
    }
    vreg[i] = p;
  }

  Pack<T> bufA[R][VPT], bufB[R][VPT], acc[VPT];
  T mgA[R], mgB[R], odA[R], odB[R];

  // The last slot of a thread: its pack index clamped into the row (a redundant, in-bounds read
  // for threads past the end) and which of its elements are columns of K.
  const int tail_vi = (VPT - 1) * NT + tid;
  const int tail_back = tail_vi < nvec ? 0 : (tail_vi - (nvec - 1)) * W;
  bool tail_ok[W];
#pragma unroll
  for (int e = 0; e < W; ++e) tail_ok[e] = tail_vi * W + e < n;

  // Strip vb: rows [rbase, rbase + rows) of K.  Its `groups` row groups are walked from a start
  // that differs from strip to strip (a rotation of the group index by a multiple of the strip
  // index), which keeps the concurrent streams from marching through DRAM in lock step; the
  // rotation is a function of the strip alone, so it does not disturb the equality over c.
  auto strip_rows = [&](int vb, int64_t& rbase) {
    const int j = vb / spb, ls = vb - j * spb;
    rbase = (int64_t)j * m + (int64_t)ls * h;
    const int left = m - ls * h;
    return left < h ? left : h;
  };
  // Step t of this workgroup is row group w + (t % spv)*G of strip team + (t / spv)*nb.  Steps
  // and rows past the end (of a short strip) are clamped to the last valid one (a redundant,
  // in-bounds read) and contribute nothing because their u is forced to 0 in process().
  // The usual case -- the workgroup walks ONE strip -- is located without any division.
  const bool one_strip = total == spv;
  int64_t rbase1;
  const int rows1 = strip_rows(team, rbase1);
  const int groups1 = (rows1 + R - 1) / R;
  const int rot1 = (int)(((unsigned)team * (unsigned)rotmul) % (unsigned)groups1);
  auto locate = [&](int t, int& vb, int64_t& rbase, int& rows, int& g) {
    if (one_strip) {
      vb = team;
      rbase = rbase1;
      rows = rows1;
      g = w + t * G;
      if (g < groups1) {
        g += rot1;
        g = g >= groups1 ? g - groups1 : g;
      }
    } else {
      vb = team + (t / spv) * nb;
      rows = strip_rows(vb, rbase);
      const int groups = (rows + R - 1) / R;
      g = w + (t % spv) * G;
      if (g < groups) g = (int)(((unsigned)g + (unsigned)vb * (unsigned)rotmul) % (unsigned)groups);
    }
  };

  auto load_group = [&](Pack<T>(&buf)[R][VPT], T(&mg)[R], T(&od)[R], int t) {
    t = t < total ? t : total - 1;
    int vb, rows, g;
    int64_t rbase;
    locate(t, vb, rbase, rows, g);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      int row = g * R + r;
      row = row < rows ? row : rows - 1;
      const T* kp = K + (rbase + row) * ld + (int64_t)tid * W;
      mg[r] = marg[rbase + row];
      od[r] = (damped || err_out) ? old_u[rbase + row] : T(0);
#pragma unroll
      for (int i = 0; i < VPT; ++i) {
        if (EXACT || i < VPT - 1) {
          buf[r][i] = load_pack_stream(kp + i * NT * W);
          // Long rows: a thread keeps at most kFusedWindow K loads in flight.  The memory system
          // delivers a little more when the 256 streams ask for ~40 KiB at a time than when each
          // posts a whole 128 KiB row at once (measured: 607 against 618 us per launch at
          // n = 32768, 349 against 360 at 24576, 162.1 against 163.8 at 16384; shorter rows and
          // the 9-11 packs per thread around n = 20000 lose from it).
          if (VPT == 8 || VPT >= 12) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kFusedWindow - 1) : "memory");
        } else {
          Pack<T> p = load_pack_stream(kp + i * NT * W - tail_back);
#pragma unroll
          for (int e = 0; e < W; ++e)
            if (!tail_ok[e]) p.e[e] = T(0);  // padding columns and clamped duplicates
          buf[r][i] = p;
        }
      }
    }
  };

  auto process = [&](Pack<T>(&buf)[R][VPT], T(&mg)[R], T(&od)[R], int t, int parity) {
    int vb, rows, g;
    int64_t rbase;
    locate(t, vb, rbase, rows, g);
    T d[R];
#pragma unroll
    for (int r = 0; r < R; ++r) d[r] = T(0);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const Pack<T> vv = load_pack(v_lds + (int64_t)(i * NT + tid) * W);
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < W; ++e) d[r] = fma(buf[r][i].e[e], vv.e[e], d[r]);
    }
    T* slot = red + parity * R * NW;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const T s = wave_sum(d[r]);
      if (lane == 0) slot[r * NW + wave] = s;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
      T q = T(0);
#pragma unroll
      for (int k = 0; k < NW; ++k) q += slot[r * NW + k];
      const int row = g * R + r;
      T ur = T(0);
      if (row < rows) {
        ur = mg[r] / q;
        if (damped) {
          if (sizeof(T) == 4 && geom)  // fp32 only: the fp64 log2 / exp2 would spill
            ur = fsk_exp2(fma(T(1) - et, fsk_log2(od[r]), et * fsk_log2(ur)));
          else
            ur = (T(1) - et) * od[r] + et * ur;
        }
        if (tid == 0) {
          if (err_out) err_out[rbase + row] = fsk_abs(od[r] * q - mg[r]);
          u_out[rbase + row] = ur;
        }
      }
#pragma unroll
      for (int i = 0; i < VPT; ++i)
#pragma unroll
        for (int e = 0; e < W; ++e) acc[i].e[e] = fma(buf[r][i].e[e], ur, acc[i].e[e]);
    }
    if (one_strip ? t == spv - 1 : t % spv == spv - 1) {  // last step of a strip: hand over its contribution
      T* prow = partial + ((int64_t)vb * G + w) * ld_ws;
#pragma unroll
      for (int i = 0; i < VPT; ++i) {
        const int vi = i * NT + tid;
        if (EXACT || i < VPT - 1 || vi < nvec) store_pack(prow + (int64_t)vi * W, acc[i]);
#pragma unroll
        for (int e = 0; e < W; ++e) acc[i].e[e] = T(0);
      }
    }
  };

  // Two register sets alternate: while one group is being reduced the next one is
  // already in flight, across strip boundaries too.
  // The step after the last one is not fetched: at 8 steps per workgroup (n = 8192) a redundant
  // group would be an eighth of the kernel's reads.
  // Short rows (up to 8 packs per thread): the first group is requested BEFORE v is staged.  The
  // loads retire in order and v was asked for first, so the wait for v does not wait for K, and
  // K's first trip to HBM runs under the staging and its barrier.  (Long rows have no registers
  // to hold v and a group at once, and gain nothing measurable.)
  // n = 8192: 49.0 -> 48.6 us per iteration, 12288: 100.1 -> 99.1, 2048: 10.07 -> 9.97.
  constexpr bool kEarlyK = VPT <= 8;
  if (kEarlyK) {
    load_group(bufA, mgA, odA, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int i = 0; i < VPT; ++i) store_pack(v_lds + (int64_t)(i * NT + tid) * W, vreg[i]);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < VPT; ++i)
#pragma unroll
    for (int e = 0; e < W; ++e) acc[i].e[e] = T(0);
  if (!kEarlyK) load_group(bufA, mgA, odA, 0);
  for (int t = 0; t < total; t += 2) {
    if (t + 1 < total) load_group(bufB, mgB, odB, t + 1);
    process(bufA, mgA, odA, t, 0);
    if (t + 1 >= total) break;
    if (t + 2 < total) load_group(bufA, mgA, odA, t + 2);
    process(bufB, mgB, odB, t + 1, 1);
  }
}

// Rows held in one register set: 16 packs (64 VGPRs) per thread, at most 8 rows.
constexpr int fused_rows_per_group(int vpt) { return 16 / vpt < 8 ? 16 / vpt : 8; }

// Workgroups the kernel is planned for, and the strips a row block is cut into when it has the
// device to itself.  Constants, not the device's compute-unit count, so that the partial sums
// (and the iterates) do not depend on the device either.  Large K: one workgroup per strip, 256
// strips.  Below n = 8192 a strip per workgroup loses to fewer, taller strips shared by 16
// workgroups each, which keep the concurrent reads in fewer, wider windows (n = 4096: 22.0 us
// per iteration with 256 strips, 19.5 with 16; n = 3072: 17.6 against 16.6; n = 8192: 51.6
// against 52.9); the iterates are then the same for every c that divides 16.
constexpr int kFusedWorkgroups = 256;
inline int fused_strips(int n) { return n >= 8192 ? 256 : 16; }

FusedPlan fused_plan(int dtype, int n, int m, int c) {
  FusedPlan p{};
  const int W = pack_width(dtype);
  const int nvec = (n + W - 1) / W;
  const int vpt = (nvec + 511) / 512;
  p.ok = vpt >= 1 && vpt <= 16 && m > 0 && n > 0 && c >= 1;
  if (!p.ok) return p;
  p.vpt = vpt;
  p.r = fused_rows_per_group(vpt);
  const int strips = fused_strips(n);
  // strip height: the block's share of the strips, in whole row groups.  With c | strips this
  // is ceil(n / strips) rounded up to row groups, whatever c is.
  const int share = strips / c > 1 ? strips / c : 1;
  p.h = ((m + share - 1) / share + p.r - 1) / p.r * p.r;
  p.spb = (m + p.h - 1) / p.h;
  p.nvb = c * p.spb;
  const int groups = (p.h + p.r - 1) / p.r;
  const int gb = kFusedWorkgroups / strips;
  p.gb = gb < groups ? gb : groups;
  // Staggered starts (strip s begins at row group 21 s mod groups) pay in the middle of the size
  // range once a strip has enough row groups to spread over -- n = 24576: 353 against 380 us per
  // iteration, 16384: 163.0 against 163.4 -- and cost a little where a row is a whole 120-128 KiB
  // (n = 32768: 609.3 against 605.6-607, 30000: 547 against 544) and at n = 8192 (8 groups per
  // strip: 53.3 against 52.3).  Measured on the kernel as it stands; an earlier loop structure
  // preferred them at every large size.
  p.rotmul = (groups >= 16 && vpt < 15) ? 21 : 0;
  p.lds_bytes = (size_t)vpt * 512 * 16 + (size_t)2 * p.r * 8 * elem_size(dtype);
  return p;
}

// Teams launched: one per strip while the compute units last, else the teams take strips in turn.
static int fused_teams(const FusedPlan& plan) {
  int cus = device_cu_count();
  if (cus < 1) cus = 1;
  int teams = cus / plan.gb;
  if (teams < 1) teams = 1;
  return teams < plan.nvb ? teams : plan.nvb;
}

template <typename T, int VPT, bool EXACT>
static int fused_typed(const FusedPlan& plan, const void* K, int64_t ld, int n, int m,
                       const void* marg, const void* vin, const void* old_u, void* u_out,
                       void* partial, int64_t ld_ws, double eta, void* err_out, hipStream_t stream) {
  constexpr int R = fused_rows_per_group(VPT);
  auto kern = fused_kernel<T, VPT, R, EXACT>;
  // the attribute belongs to the kernel's code object on ONE device: kept per device
  // (benign race: setting it twice is harmless)
  static bool attr_set[64] = {false};
  int dev = 0;
  FSK_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64 || !attr_set[dev]) {
    FSK_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    if (dev >= 0 && dev < 64) attr_set[dev] = true;
  }
  dim3 grid(plan.gb * fused_teams(plan)), block(512);
  hipLaunchKernelGGL(kern, grid, block, plan.lds_bytes, stream, (const T*)K, ld, n, m, plan.h,
                     plan.spb, plan.nvb, plan.gb, plan.rotmul, (const T*)marg, (const T*)vin, (const T*)old_u, (T*)u_out, (T*)partial, ld_ws,
                     (T)eta, (T*)err_out);
  FSK_LAUNCH_CHECK("fused_kernel");
  return FSK_OK;
}

template <typename T>
static int fused_dispatch(const FusedPlan& plan, const void* K, int64_t ld, int n, int m,
                          const void* marg, const void* vin, const void* old_u, void* u_out,
                          void* partial, int64_t ld_ws, double eta, void* err_out,
                          hipStream_t stream) {
  const bool exact = n == plan.vpt * 512 * Pack<T>::W;
#define FSK_FUSED_CASE(V)                                                                         \
  case V:                                                                                         \
    return exact ? fused_typed<T, V, true>(plan, K, ld, n, m, marg, vin, old_u, u_out,            \
                                           partial, ld_ws, eta, err_out, stream)                  \
                 : fused_typed<T, V, false>(plan, K, ld, n, m, marg, vin, old_u, u_out,           \
                                            partial, ld_ws, eta, err_out, stream)
  switch (plan.vpt) {
    FSK_FUSED_CASE(1);
    FSK_FUSED_CASE(2);
    FSK_FUSED_CASE(3);
    FSK_FUSED_CASE(4);
    FSK_FUSED_CASE(5);
    FSK_FUSED_CASE(6);
    FSK_FUSED_CASE(7);
    FSK_FUSED_CASE(8);
    FSK_FUSED_CASE(9);
    FSK_FUSED_CASE(10);
    FSK_FUSED_CASE(11);
    FSK_FUSED_CASE(12);
    FSK_FUSED_CASE(13);
    FSK_FUSED_CASE(14);
    FSK_FUSED_CASE(15);
    FSK_FUSED_CASE(16);
    default: return set_error(FSK_EUNSUPPORTED, "fused kernel: n = %d does not fit in registers", n);
  }
#undef FSK_FUSED_CASE
}

int launch_fused(int dtype, const FusedPlan& plan, const void* K, int64_t ld, int n, int m,
                 const void* marg, const void* vin, const void* old_u, void* u_out,
                 void* partial, int64_t ld_ws, int epi, double eta, hipStream_t stream,
                 void* err_out) {
  if (!plan.ok) return set_error(FSK_EUNSUPPORTED, "fused kernel: n = %d does not fit in registers", n);
  if (epi != kEpiDivide && epi != kEpiDampArith && epi != kEpiDampGeom)
    return set_error(FSK_EUNSUPPORTED, "fused kernel: only the plain and the damped updates");
  if (epi == kEpiDivide) eta = 1.0;
  if (epi == kEpiDampGeom) {
    if (dtype == FSK_F64)
      return set_error(FSK_EUNSUPPORTED, "fused kernel: the geometric relaxation exists in fp32 only");
    eta = -eta;  // the kernel's encoding of the geometric relaxation
  }
  return dtype == FSK_F64
             ? fused_dispatch<double>(plan, K, ld, n, m, marg, vin, old_u, u_out, partial, ld_ws,
                                      eta, err_out, stream)
             : fused_dispatch<float>(plan, K, ld, n, m, marg, vin, old_u, u_out, partial, ld_ws,
                                     eta, err_out, stream);
}

// ================================================================= plan sums (Eq. 1)
// Same walk as the row pass, over two matrices at once (K and the cost C); four running sums
// per row.  HBM bound: 2 n^2 s bytes.
__device__ __forceinline__ float fsk_log(float x) { return logf(x); }
__device__ __forceinline__ double fsk_log(double x) { return log(x); }

template <typename T, int ROWS>
__global__ __launch_bounds__(256) void plan_rows_kernel(const T* __restrict__ K, int64_t ldK,
                                                        const T* __restrict__ C, int64_t ldC, int n,
                                                        const T* __restrict__ u,
                                                        const T* __restrict__ v,
                                                        const T* __restrict__ l,
                                                        T* __restrict__ rows, int64_t stride) {
  constexpr int W = Pack<T>::W;
  constexpr int NT = 256, NW = NT / kWave;
  const int tid = threadIdx.x;
  const int r_base = blockIdx.x * ROWS;
  const int nvec_full = n / W;
  const T* kp[ROWS];
  const T* cp[ROWS];
#pragma unroll
  for (int r = 0; r < ROWS; ++r) {
    int row = r_base + r;
    row = row < n ? row : n - 1;
    kp[r] = K + (int64_t)row * ldK;
    cp[r] = C + (int64_t)row * ldC;
  }
  T acc[ROWS][4];
#pragma unroll
  for (int r = 0; r < ROWS; ++r)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[r][q] = T(0);
  auto term = [&](int r, T k, T c, T vj, T lj) {
    const T kv = k * vj;
    acc[r][0] += kv;
    acc[r][1] = fma(kv, c, acc[r][1]);
    if (kv > T(0)) acc[r][2] = fma(kv, fsk_log(kv), acc[r][2]);
    acc[r][3] = fma(kv, lj, acc[r][3]);
  };
  for (int cidx = tid; cidx < nvec_full; cidx += NT) {
    const Pack<T> vv = load_pack(v + (int64_t)cidx * W);
    Pack<T> ll;
#pragma unroll
    for (int e = 0; e < W; ++e) ll.e[e] = T(0);
    if (l) ll = load_pack(l + (int64_t)cidx * W);
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
      const Pack<T> kk = load_pack_stream(kp[r] + (int64_t)cidx * W);
      const Pack<T> cc = load_pack_stream(cp[r] + (int64_t)cidx * W);
#pragma unroll
      for (int e = 0; e < W; ++e) term(r, kk.e[e], cc.e[e], vv.e[e], ll.e[e]);
    }
  }
  if (tid == 0) {
    for (int j = nvec_full * W; j < n; ++j)
#pragma unroll
      for (int r = 0; r < ROWS; ++r) term(r, kp[r][j], cp[r][j], v[j], l ? l[j] : T(0));
  }
  __shared__ T red[ROWS][4][NW];
  const int lane = tid & (kWave - 1), wave = tid / kWave;
#pragma unroll
  for (int r = 0; r < ROWS; ++r)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const T s = wave_sum(acc[r][q]);
      if (lane == 0) red[r][q][wave] = s;
    }
  __syncthreads();
  if (tid < ROWS) {
    const int row = r_base + tid;
    if (row < n) {
      T s[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        s[q] = T(0);
#pragma unroll
        for (int k = 0; k < NW; ++k) s[q] += red[tid][q][k];
      }
      const T ui = u[row];
      rows[row] = ui * s[0];
      rows[stride + row] = ui * s[1];
      rows[2 * stride + row] = ui > T(0) ? ui * (s[2] + fsk_log(ui) * s[0]) : T(0);
      rows[3 * stride + row] = ui * s[3];
    }
  }
}

int launch_plan_rows(int dtype, const void* K, int64_t ldK, const void* C, int64_t ldC, int n,
                     const void* u, const void* v, const void* l, void* rows, int64_t stride,
                     hipStream_t stream) {
  constexpr int ROWS = 2;
  dim3 grid((n + ROWS - 1) / ROWS), block(256);
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((plan_rows_kernel<double, ROWS>), grid, block, 0, stream, (const double*)K,
                       ldK, (const double*)C, ldC, n, (const double*)u, (const double*)v,
                       (const double*)l, (double*)rows, stride);
  else
    hipLaunchKernelGGL((plan_rows_kernel<float, ROWS>), grid, block, 0, stream, (const float*)K, ldK,
                       (const float*)C, ldC, n, (const float*)u, (const float*)v, (const float*)l,
                       (float*)rows, stride);
  FSK_LAUNCH_CHECK("plan_rows_kernel");
  return FSK_OK;
}

// ================================================================= fp64 sum of a vector
// *out = sum_i x_i, or sum_i x_i^2 with `square`, accumulated in fp64 in a fixed order.
template <typename T>
__global__ __launch_bounds__(1024) void sum_to_double_kernel(const T* __restrict__ x, int n,
                                                             double* out, int square) {
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += 1024) {
    const double t = (double)x[i];
    s += square ? t * t : t;
  }
  s = wave_sum(s);
  __shared__ double sm[16];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int k = 0; k < 16; ++k) t += sm[k];
    *out = t;
  }
}

int launch_sum_to_double(int dtype, const void* x, int n, double* out, hipStream_t stream, bool square) {
  if (dtype == FSK_F64)
    hipLaunchKernelGGL((sum_to_double_kernel<double>), dim3(1), dim3(1024), 0, stream,
                       (const double*)x, n, out, square ? 1 : 0);
  else
    hipLaunchKernelGGL((sum_to_double_kernel<float>), dim3(1), dim3(1024), 0, stream,
                       (const float*)x, n, out, square ? 1 : 0);
  FSK_LAUNCH_CHECK("sum_to_double_kernel");
  return FSK_OK;
}

}  // namespace fsk
