// Shared device-side helpers for the fused dense-layer kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fdl {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) double f64x4;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

constexpr int kWave = 64;

// Storage type -> arithmetic type: one level above the storage precision.
template <class T> struct ComputeOf;
template <> struct ComputeOf<float> { typedef double type; };
template <> struct ComputeOf<bf16_t> { typedef float type; };

template <class T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }

// Round a value of the arithmetic type to the storage type (nearest, ties to even).
template <class T, class C> __device__ __forceinline__ T to_storage(C v);
template <> __device__ __forceinline__ float to_storage<float, double>(double v) { return (float)v; }
template <> __device__ __forceinline__ float to_storage<float, float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t to_storage<bf16_t, float>(float v) { return (bf16_t)v; }
template <> __device__ __forceinline__ bf16_t to_storage<bf16_t, double>(double v) { return (bf16_t)(float)v; }

// ---------------------------------------------------------------------------------------------
// Standard normal CDF Phi and density phi, the two pieces of GELU_erf and its derivative:
//   GELU(z) = z Phi(z),   GELU'(z) = Phi(z) + z phi(z).
// double: library erfc/exp (erfc form keeps relative accuracy for z << 0).
// float : used with bf16 storage only.  Phi(z) = 1/2 + zc P(zc^2/16) with zc = clamp(z, -4, 4) and P a degree-8
//         minimax polynomial: no division, no exponential, |error| <= 2.7e-5 (the tail beyond |z| = 4 included),
//         two orders below what bf16 storage resolves.  GELU multiplies Phi by max(z, -4) instead of z so that
//         the polynomial's residual at the left clamp (2.5e-5) is not scaled by an arbitrarily large |z|: the
//         absolute error of GELU is <= 1.1e-4 for z < 0 and its relative error <= 2.6e-5 for z > 0.
//         phi needs one hardware exp2.  Within one forward/backward pair every kernel evaluates GELU the same
//         way - through these functions, or all of them through the table below (GaussTable) - so the row
//         statistics of the forward pass, the values normalised later and the backward pass agree exactly.
template <class C> struct Gauss;

template <> struct Gauss<double> {
  static __device__ __forceinline__ void eval(double z, double& Phi, double& phi) {
    Phi = 0.5 * erfc(-z * 0.70710678118654752440);
    phi = exp(-0.5 * z * z) * 0.39894228040143267794;
  }
  static __device__ __forceinline__ double cdf(double z) { return 0.5 * erfc(-z * 0.70710678118654752440); }
  static __device__ __forceinline__ double gelu_of(double z, double Phi) { return z * Phi; }
};

template <> struct Gauss<float> {
  static __device__ __forceinline__ float cdf(float z) {
    const float zc = __builtin_amdgcn_fmed3f(z, -4.0f, 4.0f);
    // P is fitted in (zc/4)^2; its coefficients are scaled by exact powers of two so that Horner runs on zc^2
    const float u = zc * zc;
    float p = 3.463215330e-01f * 0x1p-32f;
    p = __builtin_fmaf(p, u, -1.879980461e+00f * 0x1p-28f);
    p = __builtin_fmaf(p, u, 4.556957157e+00f * 0x1p-24f);
    p = __builtin_fmaf(p, u, -6.600788584e+00f * 0x1p-20f);
    p = __builtin_fmaf(p, u, 6.482041631e+00f * 0x1p-16f);
    p = __builtin_fmaf(p, u, -4.644545581e+00f * 0x1p-12f);
    p = __builtin_fmaf(p, u, 2.528634197e+00f * 0x1p-8f);
    p = __builtin_fmaf(p, u, -1.062569532e+00f * 0x1p-4f);
    p = __builtin_fmaf(p, u, 3.989227098e-01f);
    return __builtin_fmaf(zc, p, 0.5f);
  }
  // max(z, -4) written as the median of (z, -4, largest finite float): one instruction, where a plain maximum
  // first canonicalises its input (the two agree for every finite z)
  static __device__ __forceinline__ float gelu_of(float z, float Phi) {
    return __builtin_amdgcn_fmed3f(z, -4.0f, 3.402823466e+38f) * Phi;
  }
  static __device__ __forceinline__ void eval(float z, float& Phi, float& phi) {
    Phi = cdf(z);
    phi = __builtin_amdgcn_exp2f(-0.72134752044448170368f * z * z) * 0.39894228040143267794f;   // exp(-z^2/2)/sqrt(2 pi)
  }
};

template <class C> __device__ __forceinline__ C gelu(C z) { return Gauss<C>::gelu_of(z, Gauss<C>::cdf(z)); }

// ---------------------------------------------------------------------------------------------
// Compile-time evaluation of the normal distribution in double precision (for the table below: its entries are
// constants, so the compiler computes them once instead of every workgroup at every launch).
namespace ctmath {
constexpr double kLn2 = 0.69314718055994530941723212145818;
constexpr double kInvSqrtPi = 0.56418958354775628694807945156077;
// exp(-t), t >= 0: -t = -k ln 2 - r with |r| <= ln2 / 2, a 24-term series for exp(-r), then k halvings
constexpr double exp_neg(double t) {
  if (t > 700.0) return 0.0;
  const long k = (long)(t / kLn2 + 0.5);
  const double r = t - (double)k * kLn2;
  double term = 1.0, sum = 1.0;
  for (int n = 1; n <= 24; n++) { term *= -r / (double)n; sum += term; }
  for (long i = 0; i < k; i++) sum *= 0.5;
  return sum;
}
// erf(x), x >= 0: the Maclaurin series below 2.5 (its largest term is about e^6, so cancellation costs 3 of 16 digits),
// 1 - erfc(x) from the continued fraction erfc(x) = exp(-x^2) / sqrt(pi) / (x + (1/2)/(x + 1/(x + (3/2)/(x + ...)))) above
constexpr double erf_pos(double x) {
  if (x < 2.5) {
    const double x2 = x * x;
    double term = x, sum = x;
    for (int n = 1; n <= 90; n++) {
      term *= -x2 / (double)n;
      sum += term / (double)(2 * n + 1);
    }
    return 2.0 * kInvSqrtPi * sum;
  }
  double f = x;
  for (int n = 120; n >= 1; n--) f = x + 0.5 * (double)n / f;
  return 1.0 - exp_neg(x * x) * kInvSqrtPi / f;
}
}  // namespace ctmath

// ---------------------------------------------------------------------------------------------
// Exact Phi for bf16 arguments, from a table in LDS.  A bf16 number has 8 significant bits, so the magnitudes in
// [2^-14, 16) are only 18 binades x 128 = 2304 values; for each of them the table holds
//   H = Phi(|z|) - 1/2      and (kPair) Q = |z| phi(|z|),
// both odd in z, as fp32 roundings of an fp64 evaluation.  Smaller magnitudes use the first entry (H, Q < 2.5e-5)
// and larger ones the last (H = 1/2, Q = 0 to fp32).  A lookup is: clamp the magnitude bits, one LDS read, copy
// the sign of z onto the entries - five integer instructions instead of the eleven of the polynomial, and
// GELU(z) = z (1/2 + sign(z) H) carries no approximation error beyond fp32 rounding.  The entries are compile-time
// constants in device memory; every workgroup copies them into its LDS (coalesced, a few KB from the L2).
constexpr uint32_t kGaussLo = 0x3880u;          // bf16 bits of 2^-14
constexpr uint32_t kGaussHi = 0x417fu;          // bf16 bits of the largest bf16 number below 16
constexpr int kGaussEntries = (int)(kGaussHi - kGaussLo) + 1;
struct GaussTableData { float h[kGaussEntries]; float pair[2 * kGaussEntries]; };
constexpr GaussTableData make_gauss_table() {
  GaussTableData t = {};
  for (int i = 0; i < kGaussEntries; i++) {
    const double z = (double)__builtin_bit_cast(float, (kGaussLo + (uint32_t)i) << 16);
    const double H = 0.5 * ctmath::erf_pos(z * 0.70710678118654752440);
    const double Q = z * ctmath::exp_neg(0.5 * z * z) * 0.39894228040143267794;
    t.h[i] = (float)H;
    t.pair[2 * i] = (float)H;
    t.pair[2 * i + 1] = (float)Q;
  }
  return t;
}
__device__ const GaussTableData g_gauss_table = make_gauss_table();

template <bool kPair> struct GaussTable {
  static constexpr uint32_t kLo = kGaussLo;
  static constexpr uint32_t kHi = kGaussHi;
  static constexpr int kEntries = kGaussEntries;
  static constexpr int kEntryBytes = kPair ? 8 : 4;
  static constexpr int kBytes = kEntries * kEntryBytes;

  // tbl: LDS; every thread of the workgroup calls this (followed by a barrier at the caller)
  static __device__ __forceinline__ void build(float* tbl, int tid, int nthreads) {
    const float* src = kPair ? g_gauss_table.pair : g_gauss_table.h;
    for (int i = tid; i < (kPair ? 2 : 1) * kEntries; i += nthreads) tbl[i] = src[i];
  }
  // LDS address of the entry for the bf16 number whose bits (sign included or not) are in the low 16 bits of
  // `bits`: clamped magnitude bits times the entry size plus origin(table address), in three instructions
  static __device__ __forceinline__ uint32_t origin(uint32_t table_lds_address) {
    return table_lds_address - kLo * (uint32_t)kEntryBytes;     // wraps; the sum below is the true address again
  }
  static __device__ __forceinline__ uint32_t address_of(uint32_t bits, uint32_t org) {
    uint32_t mag = bits & 0x7fffu;
    mag = mag < kLo ? kLo : mag;
    mag = mag > kHi ? kHi : mag;
    return mag * (uint32_t)kEntryBytes + org;
  }
  // sign(z) |h|: magnitude bits of h, sign bit of z
  static __device__ __forceinline__ float with_sign_of(float h, float z) {
    return __builtin_bit_cast(float, (__builtin_bit_cast(uint32_t, h) & 0x7fffffffu) |
                                         (__builtin_bit_cast(uint32_t, z) & 0x80000000u));
  }
};

// ---------------------------------------------------------------------------------------------
// Vector access helpers: V consecutive storage elements <-> V values of the arithmetic type.
template <class T, int V> struct VecIO;

template <> struct VecIO<float, 4> {
  template <class C> static __device__ __forceinline__ void load(const float* p, C (&v)[4]) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(p);
    v[0] = (C)t[0]; v[1] = (C)t[1]; v[2] = (C)t[2]; v[3] = (C)t[3];
  }
  template <class C> static __device__ __forceinline__ void store(float* p, const C (&v)[4]) {
    f32x4 t; t[0] = (float)v[0]; t[1] = (float)v[1]; t[2] = (float)v[2]; t[3] = (float)v[3];
    *reinterpret_cast<f32x4*>(p) = t;
  }
};
template <> struct VecIO<float, 1> {
  template <class C> static __device__ __forceinline__ void load(const float* p, C (&v)[1]) { v[0] = (C)p[0]; }
  template <class C> static __device__ __forceinline__ void store(float* p, const C (&v)[1]) { p[0] = (float)v[0]; }
};
template <> struct VecIO<bf16_t, 8> {
  template <class C> static __device__ __forceinline__ void load(const bf16_t* p, C (&v)[8]) {
    const bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (C)(float)t[i];
  }
  template <class C> static __device__ __forceinline__ void store(bf16_t* p, const C (&v)[8]) {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; i++) t[i] = (bf16_t)(float)v[i];
    *reinterpret_cast<bf16x8*>(p) = t;
  }
};
template <> struct VecIO<bf16_t, 1> {
  template <class C> static __device__ __forceinline__ void load(const bf16_t* p, C (&v)[1]) { v[0] = (C)(float)p[0]; }
  template <class C> static __device__ __forceinline__ void store(bf16_t* p, const C (&v)[1]) { p[0] = (bf16_t)(float)v[0]; }
};

// Sum over the 64 lanes of a wavefront; every lane receives the total.
template <class C> __device__ __forceinline__ C wave_sum(C v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

// fp32: data-parallel-primitive lane moves folded into the adds instead of LDS permutes.
// dpp_f<CTRL, ROW_MASK>(x): the value of the lane CTRL selects; lanes in rows outside ROW_MASK read 0.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_f(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false));
}
// sum inside each row of 16 lanes; every lane of a row receives its row's sum
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]: lane ^ 1
  v += dpp_f<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]: lane ^ 2
  v += dpp_f<0x141, 0xF>(v);   // row_half_mirror: the other quad of each 8
  v += dpp_f<0x140, 0xF>(v);   // row_mirror: the other half of the row
  return v;
}
template <> __device__ __forceinline__ float wave_sum<float>(float v) {
  v = row16_sum(v);
  v += dpp_f<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3: rows 0+1, rows 2+3
  v += dpp_f<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3: row 3 now holds the total
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

}  // namespace fdl
