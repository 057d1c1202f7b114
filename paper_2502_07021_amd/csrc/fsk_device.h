// Device-side helpers shared by the gfx950 kernels: 128-bit packs, wave64 and
// workgroup reductions with a fixed summation order, and the elementwise
// epilogues of the scaling updates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fsk {

constexpr int kWave = 64;

// 16-byte pack of T: 4 floats or 2 doubles, loaded and stored with one 128-bit access.
template <typename T>
struct alignas(16) Pack {
  static constexpr int W = 16 / sizeof(T);
  T e[W];
};

template <typename T>
__device__ __forceinline__ Pack<T> load_pack(const T* p) {
  return *reinterpret_cast<const Pack<T>*>(p);
}

template <typename T>
__device__ __forceinline__ void store_pack(T* p, const Pack<T>& v) {
  *reinterpret_cast<Pack<T>*>(p) = v;
}

// Streaming variants: the access carries the non-temporal hint, so a matrix that is read
// once per pass does not displace the small reused vectors in L2 (measured on MI355X: a
// 4 GiB read stream runs at ~7.1 TB/s with the hint against ~6.3 TB/s without).
template <typename T>
struct NativeVec;
template <>
struct NativeVec<float> {
  typedef float type __attribute__((ext_vector_type(4)));
};
template <>
struct NativeVec<double> {
  typedef double type __attribute__((ext_vector_type(2)));
};

template <typename T>
__device__ __forceinline__ Pack<T> load_pack_stream(const T* p) {
  using V = typename NativeVec<T>::type;
  const V t = __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
  Pack<T> r;
#pragma unroll
  for (int e = 0; e < Pack<T>::W; ++e) r.e[e] = t[e];
  return r;
}

// Buffer descriptor (raw, untyped, 32-bit elements) over the memory from `base` on; `base` must
// be the same for every lane of the wave.  A load through it takes a 32-bit lane offset and a
// 32-bit wave-uniform offset, both in bytes: a loop that walks rows of a matrix then forms each
// address on the scalar unit (with 64-bit flat addresses every load costs 64-bit vector
// additions, which the matrix-core kernels cannot hide between two MFMAs).  The range field is
// set wide, so the hardware range check never fires: the caller keeps every offset inside the
// operand, exactly as it would with a pointer.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_over(const void* base) {
  const uint64_t bits = (uint64_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)bits);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(bits >> 32));
  return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, 0x7ffffff0, 0x00020000);
}

template <typename T, bool STREAM>  // STREAM: with the non-temporal hint
__device__ __forceinline__ Pack<T> buffer_load_pack(__amdgpu_buffer_rsrc_t rs, uint32_t lane_bytes,
                                                    uint32_t wave_bytes) {
  using V = typename NativeVec<T>::type;
  // (the whole vector is re-typed at once: re-typing its elements one by one through
  // __builtin_bit_cast made the compiler fetch a single element)
  const V t = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_bytes, wave_bytes,
                                                                          STREAM ? 2 : 0));
  Pack<T> r;
#pragma unroll
  for (int e = 0; e < Pack<T>::W; ++e) r.e[e] = t[e];
  return r;
}

template <typename T>
__device__ __forceinline__ void store_pack_stream(T* p, const Pack<T>& v) {
  using V = typename NativeVec<T>::type;
  V t;
#pragma unroll
  for (int e = 0; e < Pack<T>::W; ++e) t[e] = v.e[e];
  __builtin_nontemporal_store(t, reinterpret_cast<V*>(p));
}

// Butterfly sum over the 64 lanes; every lane ends with the same total and the
// order of additions is the same in every launch.
// ---- lane exchanges on the vector ALU (no LDS crossbar): gfx950's v_permlane32_swap and
// v_permlane16_swap across halves / rows of a wave, DPP controls inside a row of 16 lanes.
// Measured layouts: permlane32_swap(a, b) returns {a with lanes 32-63 replaced by b's lanes 0-31,
// b with lanes 0-31 replaced by a's lanes 32-63}; permlane16_swap does the same per pair of rows;
// row_ror:8, row_half_mirror, quad_perm [3,2,1,0] and [1,0,3,2] read lane l ^ 8, ^ 7, ^ 3, ^ 1.
typedef unsigned fsk_uint2 __attribute__((ext_vector_type(2)));
template <typename T>
struct LaneWords {
  static constexpr int N = sizeof(T) / 4;
  unsigned w[N];
  __device__ __forceinline__ explicit LaneWords(T x) { __builtin_memcpy(w, &x, sizeof(T)); }
  __device__ __forceinline__ T value() const { T x; __builtin_memcpy(&x, w, sizeof(T)); return x; }
};

// a <- {a on the lower class, b of the partner on the upper class}, b <- the converse, for the
// lane pairing l <-> l ^ 32 (HALF = 32) or l ^ 16 (HALF = 16); then a + b is, on the lower class,
// the pair's sum of a and, on the upper class, the pair's sum of b.
template <int HALF, typename T>
__device__ __forceinline__ T pair_sum_swap(T a, T b) {
  LaneWords<T> x(a), y(b);
#pragma unroll
  for (int i = 0; i < LaneWords<T>::N; ++i) {
    const fsk_uint2 r = HALF == 32 ? __builtin_amdgcn_permlane32_swap(x.w[i], y.w[i], false, false)
                                   : __builtin_amdgcn_permlane16_swap(x.w[i], y.w[i], false, false);
    x.w[i] = r[0];
    y.w[i] = r[1];
  }
  return x.value() + y.value();
}

// The value of lane l ^ MASK for MASK in {8, 7, 3, 2, 1} (DPP inside a row of 16 lanes).
template <int MASK, typename T>
__device__ __forceinline__ T lane_xor_dpp(T v) {
  constexpr int ctrl = MASK == 8 ? 0x128 : MASK == 7 ? 0x141 : MASK == 3 ? 0x1B : MASK == 2 ? 0x4E : 0xB1;
  static_assert(MASK == 8 || MASK == 7 || MASK == 3 || MASK == 2 || MASK == 1,
                "no DPP control for this mask");
  LaneWords<T> x(v);
#pragma unroll
  for (int i = 0; i < LaneWords<T>::N; ++i)
    x.w[i] = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x.w[i], ctrl, 0xf, 0xf, false);
  return x.value();
}

// Transpose of the W x W block that W adjacent lanes (lane % W = c) hold as s[j] = M[c][j]:
// afterwards lane c holds s[i] = M[i][c].  W = 4 (two exchange stages) or 2 (one).  Every lane of
// the group must be active.
template <typename T>
__device__ __forceinline__ void lanes_transpose4(T (&s)[4], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2;
#pragma unroll
  for (int j = 0; j < 4; j += 2) {
    const T got = lane_xor_dpp<1>(b0 ? s[j] : s[j + 1]);
    if (b0) s[j] = got; else s[j + 1] = got;
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const T got = lane_xor_dpp<2>(b1 ? s[j] : s[j + 2]);
    if (b1) s[j] = got; else s[j + 2] = got;
  }
}
template <typename T>
__device__ __forceinline__ void lanes_transpose2(T (&s)[2], int lane) {
  const bool b0 = lane & 1;
  const T got = lane_xor_dpp<1>(b0 ? s[0] : s[1]);
  if (b0) s[0] = got; else s[1] = got;
}

// All-lanes sum of a wave: the pairings ^32, ^16, ^8, ^7, ^3, ^1 span the 64 lanes; every
// lane ends with the same value, formed in the same order in every launch.
template <typename T>
__device__ __forceinline__ T wave_sum(T x) {
  x = pair_sum_swap<32>(x, x);
  x = pair_sum_swap<16>(x, x);
  x += lane_xor_dpp<8>(x);
  x += lane_xor_dpp<7>(x);
  x += lane_xor_dpp<3>(x);
  x += lane_xor_dpp<1>(x);
  return x;
}

// Sums RPT (8 or 16) values per lane over the wave with RPT - 1 + log2(64 / RPT) exchanges
// instead of 6 RPT: each of the first log2(RPT) steps pairs the lanes by one lane bit (5, 4,
// 3, 2 in turn); the lane whose bit is clear completes the lower half of its values with the
// partner's, the other lane the upper half.  On return val[0] of lane l is the wave's sum of
// value number `which`, shared by the 64 / RPT lanes that differ in the low lane bits only.
template <typename T, int RPT>
__device__ __forceinline__ int wave_sum_rows(T (&val)[RPT], int lane) {
  static_assert(RPT == 8 || RPT == 16, "8 or 16 values per lane");
#pragma unroll
  for (int i = 0; i < RPT / 2; ++i) val[i] = pair_sum_swap<32>(val[i], val[i + RPT / 2]);
#pragma unroll
  for (int i = 0; i < RPT / 4; ++i) val[i] = pair_sum_swap<16>(val[i], val[i + RPT / 4]);
  int which = ((lane >> 5) & 1) * (RPT / 2) + ((lane >> 4) & 1) * (RPT / 4);
  {
    const bool upper = (lane & 8) != 0;
#pragma unroll
    for (int i = 0; i < RPT / 8; ++i) {
      const T send = upper ? val[i] : val[i + RPT / 8];
      const T keep = upper ? val[i + RPT / 8] : val[i];
      val[i] = keep + lane_xor_dpp<8>(send);
    }
    which += upper ? RPT / 8 : 0;
  }
  if (RPT == 16) {
    const bool upper = (lane & 4) != 0;
    const T send = upper ? val[0] : val[1];
    const T keep = upper ? val[1] : val[0];
    val[0] = keep + lane_xor_dpp<7>(send);
    which += upper ? 1 : 0;
  } else {
    val[0] += lane_xor_dpp<7>(val[0]);
  }
  val[0] += lane_xor_dpp<3>(val[0]);
  val[0] += lane_xor_dpp<1>(val[0]);
  return which;
}

template <typename T>
__device__ __forceinline__ T wave_max(T x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    T y = __shfl_xor(x, o, kWave);
    x = y > x ? y : x;
  }
  return x;
}

// Elementwise update applied to a finished kernel product (Sec. 1 scaling form;
// Sec. 3.3 for the relaxed forms).  `marg` is the prescribed marginal entry,
// `prod` the product (K v)_i or (K^T u)_j, `old` the scaling before the update.
enum Epilogue : int {
  kEpiDivide = 0,     // marg / prod
  kEpiDampArith = 1,  // (1-eta) old + eta marg/prod
  kEpiDampGeom = 2,   // old^(1-eta) (marg/prod)^eta
  kEpiMarginal = 3,   // old * prod          (row/column marginal of diag(u) K diag(v))
  kEpiAbsErr = 4,     // |old * prod - marg|
  kEpiProduct = 5     // prod itself
};

__device__ __forceinline__ float fsk_pow(float x, float y) { return powf(x, y); }
__device__ __forceinline__ double fsk_pow(double x, double y) { return pow(x, y); }
__device__ __forceinline__ float fsk_abs(float x) { return fabsf(x); }
__device__ __forceinline__ double fsk_abs(double x) { return fabs(x); }

template <typename T>
__device__ __forceinline__ T apply_epilogue(int epi, T marg, T prod, T old, T eta) {
  switch (epi) {
    case kEpiDivide: return marg / prod;
    case kEpiDampArith: return (T(1) - eta) * old + eta * (marg / prod);
    case kEpiDampGeom: return fsk_pow(old, T(1) - eta) * fsk_pow(marg / prod, eta);
    case kEpiMarginal: return old * prod;
    case kEpiAbsErr: return fsk_abs(old * prod - marg);
    default: return prod;
  }
}

__host__ __device__ constexpr bool epi_needs_marg(int epi) {
  return epi == kEpiDivide || epi == kEpiDampArith || epi == kEpiDampGeom || epi == kEpiAbsErr;
}
__host__ __device__ constexpr bool epi_needs_old(int epi) {
  return epi == kEpiDampArith || epi == kEpiDampGeom || epi == kEpiMarginal || epi == kEpiAbsErr;
}

}  // namespace fsk
