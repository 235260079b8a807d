// Device-side building blocks shared by the tc355 kernels (gfx950 only).
//
// Arithmetic model of the library (the int8 grouped convolution in gconv_i8.hpp
// states its own): fp32 inputs are widened exactly to
// fp64, multiplied and summed by the fp64 matrix-core instruction
// v_mfma_f64_16x16x4_f64, and rounded to fp32 once when a declared output is
// written.  An fp32 accumulator (vector or matrix) cannot meet the parity bar
// of 2e-5 relative to |ref| + 1e-3*max|ref|: near-zero outputs leave room for
// about 2e-8*max|ref| of absolute error, less than one fp32 rounding of a
// typical partial sum.
//
// Operand layout of one 16x16x4 fp64 MFMA on a 64-lane wavefront, with
// r16 = lane % 16 and q = lane / 16 (measured on MI355X with a one-hot probe):
//   A (16 x 4):  lane supplies A[row = r16][k = q]
//   B (4 x 16):  lane supplies B[k = q][col = r16]
//   D (16 x 16): lane holds 4 values, D[row = 4*v + q][col = r16], v = 0..3
// The order in which the reduction index is consumed is free, so kernels feed
// "k slot q" with whatever element is convenient as long as A and B agree.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tc355 {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef double dbl2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;
constexpr int WG_THREADS = 256;
constexpr int WAVES_PER_WG = WG_THREADS / WAVE;

__device__ __forceinline__ d4 mfma_f64(double a, double b, d4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ d4 d4_zero() {
  d4 z = {0.0, 0.0, 0.0, 0.0};
  return z;
}

__device__ __forceinline__ d4 d4_splat(double x) {
  d4 z = {x, x, x, x};
  return z;
}

// Row of the 16x16 result tile held in element v of a lane's accumulator.
__device__ __forceinline__ int d_row(int q, int v) { return 4 * v + q; }

// fmaxf(x, 0) semantics in fp64: NaN and -0 become +0.
__device__ __forceinline__ double relu64(double x) { return x > 0.0 ? x : 0.0; }

// Streaming store of an output element that the kernel never reads again: it does not displace the inputs that
// neighbouring tiles or bands re-read from L2 (2-3 % on the fp64 convolution kernels, 10 % on the int8 one).
template <typename T>
__device__ __forceinline__ void store_stream(T* p, T v) {
  __builtin_nontemporal_store(v, p);
}

// Vector of V elements of T, loaded with one instruction when V is 1, 2 or 4.
template <typename T, int V>
struct Vec {
  T e[V];
};

template <typename T, int V>
__device__ __forceinline__ Vec<T, V> load_vec(const T* p) {
  Vec<T, V> r;
  if constexpr (V == 1) {
    r.e[0] = *p;
  } else if constexpr (sizeof(T) == 4 && V == 2) {
    f2 t = *reinterpret_cast<const f2*>(p);
    r.e[0] = t[0];
    r.e[1] = t[1];
  } else if constexpr (sizeof(T) == 4 && V == 4) {
    f4 t = *reinterpret_cast<const f4*>(p);
    r.e[0] = t[0];
    r.e[1] = t[1];
    r.e[2] = t[2];
    r.e[3] = t[3];
  } else if constexpr (sizeof(T) == 8 && V == 2) {
    dbl2 t = *reinterpret_cast<const dbl2*>(p);
    r.e[0] = t[0];
    r.e[1] = t[1];
  } else if constexpr (sizeof(T) == 8 && V == 4) {
    d4 t = *reinterpret_cast<const d4*>(p);
    r.e[0] = t[0];
    r.e[1] = t[1];
    r.e[2] = t[2];
    r.e[3] = t[3];
  } else {
    static_assert(V == 1, "unsupported vector width");
  }
  return r;
}

}  // namespace tc355
