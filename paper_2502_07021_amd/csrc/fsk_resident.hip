// Small problems (paper: Algorithm 1 on a kernel of a few MiB): K is read from memory once per
// CALL, not once per iteration.  A persistent grid of G <= 32 workgroups keeps the whole matrix
// in registers -- workgroup w owns a contiguous block of rows, thread (rs, cp) of it the 16-byte
// column pack cp of the rows rs, rs + RS, ... of that block -- and iterates
//
//     q = K v (registers x registers, wave butterflies + LDS across waves),  u = a ./ q,
//     s^(w) = K_w^T u_w (registers),  one grid-wide barrier,  v = b ./ sum_w s^(w)
//
// exchanging only the G partial column sums (n values each) through global memory.  An
// iteration costs one barrier round trip instead of two kernel launches.
//
// Grid barrier: a monotone counter in the workspace (zeroed by a fill kernel before the
// launch).  Every thread waits for its own partial stores to complete, the workgroup
// synchronises, one thread arrives with an agent-scope release add and polls with atomic loads
// (sleeping in between), then acquires; the partials themselves are agent-scope atomic stores
// and loads (measured: 1.9 / 2.4 / 4.1 us per round for 8 / 16 / 32 workgroups, against 7-8 us
// when every wave issues full fences around plain stores and loads).  The G workgroups are far
// fewer than the compute units, so they are co-resident as soon as the device has room for
// them; a waiter nevertheless gives up after `spin_limit` polls, marks the call failed, and its
// workgroup writes NaN results and leaves: the grid always drains.
// The partial area is double buffered by iteration parity: a workgroup can be at most one
// barrier ahead of the slowest one.
#include <type_traits>

#include "fsk_device.h"
#include "fsk_internal.h"

namespace fsk {

constexpr int kResThreads = 512;

__global__ void resident_reset_kernel(unsigned* state) {
  if (threadIdx.x < 2) state[threadIdx.x] = 0u;  // [0] barrier counter, [1] failure flag
}

// The partial sums cross compute units (and their separate L2 slices) as agent-scope atomic
// 64-bit stores and loads, which travel through the coherent levels without whole-cache
// write-backs or invalidations.
template <typename T>
__device__ __forceinline__ void store_agent(T* p, const Pack<T>& v) {
  static_assert(sizeof(Pack<T>) == 16, "a pack is 16 bytes");
  unsigned long long w[2];
  __builtin_memcpy(w, &v, 16);
  unsigned long long* q = reinterpret_cast<unsigned long long*>(p);
  __hip_atomic_store(q, w[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 1, w[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ Pack<T> load_agent(const T* p) {
  const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
  unsigned long long w[2];
  w[0] = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  w[1] = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  Pack<T> v;
  __builtin_memcpy(&v, w, 16);
  return v;
}

__device__ __forceinline__ float res_log2(float x) { return log2f(x); }
__device__ __forceinline__ double res_log2(double x) { return log2(x); }
__device__ __forceinline__ float res_exp2(float x) { return exp2f(x); }
__device__ __forceinline__ double res_exp2(double x) { return exp2(x); }
// (1 - et) old + et fresh, or old^(1 - et) fresh^et
template <typename T>
__device__ __forceinline__ T relax(T old, T fresh, T et, bool geom) {
  return geom ? res_exp2(fma(T(1) - et, res_log2(old), et * res_log2(fresh)))
              : (T(1) - et) * old + et * fresh;
}

// RPT: rows per thread (register-resident packs per thread).
template <typename T, int RPT>
__global__ __launch_bounds__(kResThreads) void resident_kernel(
    const T* __restrict__ K, int64_t ld, int n, int iters, int rows_per_wg, int p_pad,
    const T* __restrict__ a, const T* __restrict__ b, T* u, T* v, T* partial, int64_t ld_ws,
    unsigned* state, unsigned spin_limit, T eta) {
  constexpr int W = Pack<T>::W;
  constexpr int NW = kResThreads / kWave;
  constexpr int kMaxRows = RPT * NW;       // rows a workgroup can own
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int G = gridDim.x, w = blockIdx.x;
  const int RS = kResThreads / p_pad;      // row subgroups: threads sharing a column pack
  const int wps = p_pad / kWave;           // waves per row subgroup
  const int cp = tid % p_pad, rs = tid / p_pad;
  const int col = cp * W;
  const bool active = rs < RS && col < n;  // threads past the row end or past the subgroups idle
  const int row_lo = w * rows_per_wg;
  const int row_hi = row_lo + rows_per_wg < n ? row_lo + rows_per_wg : n;
  const int my_rows = row_hi > row_lo ? row_hi - row_lo : 0;
  // |eta| < 1 selects a relaxation (Sec. 3.3): eta > 0 the arithmetic one, eta < 0 the geometric
  // one with parameter -eta, x <- x^(1+eta) (new)^(-eta), as exp2 of the weighted log2's.
  const bool geom = eta < T(0);
  const T et = geom ? -eta : eta;
  const bool damped = et < T(1);

  __shared__ T red[kMaxRows][NW];  // [row of the workgroup][wave of its subgroup]
  __shared__ __align__(16) T colred[kResThreads * W];
  __shared__ T a_s[kMaxRows], u_s[2][kMaxRows];  // per row: marginal, scaling (by iteration parity)
  __shared__ int dead;
  if (tid == 0) dead = 0;
  for (int local = tid; local < kMaxRows; local += kResThreads) {
    a_s[local] = local < my_rows ? a[row_lo + local] : T(1);
    u_s[0][local] = local < my_rows ? u[row_lo + local] : T(0);
    u_s[1][local] = T(0);
  }

  // K of this thread's rows (row rs + k RS of the workgroup); b and the starting v of its pack
  Pack<T> kreg[RPT];
  Pack<T> v_p, b_p;
#pragma unroll
  for (int e = 0; e < W; ++e) { v_p.e[e] = T(0); b_p.e[e] = T(0); }
  if (active) {
#pragma unroll
    for (int e = 0; e < W; ++e)
      if (col + e < n) { v_p.e[e] = v[col + e]; b_p.e[e] = b[col + e]; }
  }
#pragma unroll
  for (int k = 0; k < RPT; ++k) {
    const int row = row_lo + rs + k * RS;
#pragma unroll
    for (int e = 0; e < W; ++e) kreg[k].e[e] = T(0);
    if (active && row < row_hi) {
      const T* kp = K + (int64_t)row * ld + col;
      if (col + W <= n) {
        kreg[k] = load_pack(kp);
      } else {
#pragma unroll
        for (int e = 0; e < W; ++e)
          if (col + e < n) kreg[k].e[e] = kp[e];
      }
    }
  }
  __syncthreads();

  for (int it = 0; it < iters; ++it) {
    // ---- q = K v for the rows of this workgroup: per-thread partial dots, summed over the wave
    T d[RPT];
#pragma unroll
    for (int k = 0; k < RPT; ++k) {
      d[k] = T(0);
#pragma unroll
      for (int e = 0; e < W; ++e) d[k] = fma(kreg[k].e[e], v_p.e[e], d[k]);
    }
    const int k_mine = wave_sum_rows<T, RPT>(d, lane);
    if ((lane & (kWave / RPT - 1)) == 0 && rs < RS) red[rs + k_mine * RS][wave % wps] = d[0];
    __syncthreads();
    // ---- u = a ./ q, one thread per row
    if (tid < kMaxRows) {
      T un = T(0);
      if (tid < my_rows) {
        T q = T(0);
        for (int x = 0; x < wps; ++x) q += red[tid][x];
        un = a_s[tid] / q;
        if (damped) un = relax(u_s[it & 1][tid], un, et, geom);
      }
      u_s[(it + 1) & 1][tid] = un;
    }
    __syncthreads();
    // ---- s^(w) = K_w^T u_w: per-thread sums over its rows, then across the row subgroups
    Pack<T> acc;
#pragma unroll
    for (int e = 0; e < W; ++e) acc.e[e] = T(0);
    if (rs < RS) {
#pragma unroll
      for (int k = 0; k < RPT; ++k) {
        const T un = u_s[(it + 1) & 1][rs + k * RS];
#pragma unroll
        for (int e = 0; e < W; ++e) acc.e[e] = fma(kreg[k].e[e], un, acc.e[e]);
      }
    }
    T* mine = partial + ((int64_t)(it & 1) * G + w) * ld_ws;
    if (RS > 1) {
      store_pack(colred + (int64_t)tid * W, acc);
      __syncthreads();
      if (rs == 0 && col < n) {
        for (int x = 1; x < RS; ++x) {
          const Pack<T> y = load_pack(colred + (int64_t)(x * p_pad + cp) * W);
#pragma unroll
          for (int e = 0; e < W; ++e) acc.e[e] += y.e[e];
        }
      }
    }
    if (rs == 0 && col < n) store_agent(mine + col, acc);  // whole packs: ld_ws covers the padding
    // ---- grid-wide barrier: own stores done, then one arrival per workgroup
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add(&state[0], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned target = (unsigned)(it + 1) * (unsigned)G;
      unsigned polls = 0;
      while (__hip_atomic_load(&state[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        if (++polls > spin_limit ||
            ((polls & 1023u) == 0u &&
             __hip_atomic_load(&state[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
          __hip_atomic_store(&state[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          dead = 1;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
    if (dead) break;  // uniform: read after the barrier by every thread
    // ---- v = b ./ sum_w s^(w), every workgroup for itself, in workgroup order
    if (active) {
      const T* base = partial + (int64_t)(it & 1) * G * ld_ws + col;
      Pack<T> r;
#pragma unroll
      for (int e = 0; e < W; ++e) r.e[e] = T(0);
      // G is 8, 16 or 32.  Every load is a round trip beyond the XCD's L2 (~1 us), so as many
      // as the registers hold are in flight at once: all 8, or 16 at a time.  Added in workgroup
      // order either way.
      auto gather = [&](auto batch_tag, int g0) {
        constexpr int B = decltype(batch_tag)::value;
        Pack<T> y[B];
#pragma unroll
        for (int g = 0; g < B; ++g) y[g] = load_agent(base + (int64_t)(g0 + g) * ld_ws);
#pragma unroll
        for (int g = 0; g < B; ++g)
#pragma unroll
          for (int e = 0; e < W; ++e) r.e[e] += y[g].e[e];
      };
      if (G == 8) {
        gather(std::integral_constant<int, 8>{}, 0);
      } else {
        for (int g0 = 0; g0 < G; g0 += 16) gather(std::integral_constant<int, 16>{}, g0);
      }
#pragma unroll
      for (int e = 0; e < W; ++e) {
        T vn = T(0);
        if (col + e < n) {
          vn = b_p.e[e] / r.e[e];
          if (damped) vn = relax(v_p.e[e], vn, et, geom);
        }
        v_p.e[e] = vn;
      }
    }
  }

  // ---- results (NaN if the barrier gave up)
  __syncthreads();
  const T poison = dead ? T(NAN) : T(0);
  for (int local = tid; local < my_rows; local += kResThreads)
    u[row_lo + local] = u_s[iters & 1][local] + poison;
  if ((w == 0 || dead) && active && rs == 0) {
#pragma unroll
    for (int e = 0; e < W; ++e)
      if (col + e < n) v[col + e] = v_p.e[e] + poison;
  }
}

// Geometry: the smallest grid of 8, 16 or 32 workgroups whose threads hold at most 16 packs
// each (n <= 1024 in fp32, 512 in fp64); a variant with 32 packs per thread would spill.
ResidentPlan resident_plan(int dtype, int n) {
  ResidentPlan p{};
  const int W = pack_width(dtype);
  const int packs = (n + W - 1) / W;
  p.p_pad = (packs + kWave - 1) / kWave * kWave;
  if (n < 1 || p.p_pad > kResThreads) return p;
  const int RS = kResThreads / p.p_pad;
  for (int G : {8, 16, 32}) {
    const int rows = (n + G - 1) / G;
    const int rpt = (rows + RS - 1) / RS;
    if (rpt <= 16) {
      p.ok = true;
      p.wgs = G;
      p.rows_per_wg = rows;
      p.rpt = rpt <= 8 ? 8 : 16;
      p.ld_ws = (int64_t)p.p_pad * W;
      return p;
    }
  }
  return p;
}

size_t resident_workspace_bytes(int dtype, int n) {
  const ResidentPlan p = resident_plan(dtype, n);
  if (!p.ok) return 0;
  return align_up((size_t)2 * p.wgs * (size_t)p.ld_ws * elem_size(dtype), 256) + 256;
}

template <typename T, int RPT>
static void resident_launch(const ResidentPlan& p, const void* K, int64_t ld, int n, int iters,
                            const void* a, const void* b, void* u, void* v, void* partial,
                            unsigned* state, unsigned spin_limit, double eta, hipStream_t st) {
  hipLaunchKernelGGL((resident_kernel<T, RPT>), dim3(p.wgs), dim3(kResThreads), 0, st, (const T*)K,
                     ld, n, iters, p.rows_per_wg, p.p_pad, (const T*)a, (const T*)b, (T*)u, (T*)v,
                     (T*)partial, p.ld_ws, state, spin_limit, (T)eta);
}

int launch_resident(int dtype, const void* K, int64_t ld, int n, int iters, const void* a,
                    const void* b, void* u, void* v, void* workspace, double eta,
                    unsigned spin_limit, hipStream_t st) {
  const ResidentPlan p = resident_plan(dtype, n);
  if (!p.ok) return set_error(FSK_EUNSUPPORTED, "n = %d does not fit the register-resident flow", n);
  if (iters < 1) return FSK_OK;
  if ((int64_t)iters * p.wgs > 0x7fffffffLL)
    return set_error(FSK_EINVAL, "too many iterations for one register-resident launch");
  const size_t part_bytes = align_up((size_t)2 * p.wgs * (size_t)p.ld_ws * elem_size(dtype), 256);
  unsigned* state = (unsigned*)((char*)workspace + part_bytes);
  hipLaunchKernelGGL(resident_reset_kernel, dim3(1), dim3(64), 0, st, state);
  FSK_LAUNCH_CHECK("resident_reset_kernel");
#define FSK_RES_CASE(TT, R)                                                                        \
  resident_launch<TT, R>(p, K, ld, n, iters, a, b, u, v, workspace, state, spin_limit, eta, st)
  if (dtype == FSK_F64) {
    if (p.rpt == 8) FSK_RES_CASE(double, 8);
    else FSK_RES_CASE(double, 16);
  } else {
    if (p.rpt == 8) FSK_RES_CASE(float, 8);
    else FSK_RES_CASE(float, 16);
  }
#undef FSK_RES_CASE
  FSK_LAUNCH_CHECK("resident_kernel");
  return FSK_OK;
}

}  // namespace fsk
