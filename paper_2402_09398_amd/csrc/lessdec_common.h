// Shared device helpers of the lessdec kernels (gfx950, wave64).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

namespace lessdec {

constexpr int kWave = 64;

// ---- 16-byte vector access to the storage type --------------------------------------
template <typename T> struct Store;
template <> struct Store<float> {
  static constexpr int kPerVec = 4;
  struct Vec { float4 raw; };
  __device__ static inline float get(const Vec &v, int i) { return (&v.raw.x)[i]; }
  __device__ static inline float from_float(float x) { return x; }
  __device__ static inline float to_float(float x) { return x; }
};
template <> struct Store<__half> {
  static constexpr int kPerVec = 8;
  struct Vec { uint4 raw; };
  __device__ static inline float get(const Vec &v, int i)
  {
    const __half *h = reinterpret_cast<const __half *>(&v.raw);
    return __half2float(h[i]);
  }
  __device__ static inline __half from_float(float x) { return __float2half_rn(x); }
  __device__ static inline float to_float(__half x) { return __half2float(x); }
};

template <typename T>
__device__ inline typename Store<T>::Vec load_vec(const T *p)
{
  typename Store<T>::Vec v;
  v.raw = *reinterpret_cast<const decltype(v.raw) *>(p);
  return v;
}

// Eviction candidate: smaller accumulated score first, then the older token.
struct Cand {
  double acc;
  int pos;
  int slot;
};
__device__ inline bool cand_less(const Cand &a, const Cand &b)
{
  return a.acc < b.acc || (a.acc == b.acc && a.pos < b.pos);
}
__device__ inline Cand cand_none() { return Cand{__builtin_inf(), INT_MAX, -1}; }

// e^x in fp64 for the softmax weights of the prompt phase, where x = s - max <= 0 up to
// rounding: x = n ln 2 + r with |r| <= ln 2 / 2, Taylor polynomial of degree 10 in r
// (truncation 2e-13 relative), scaled by 2^n; 0 below the underflow threshold and for -inf.
// Half the instructions of the library routine; its error is far inside the 1e-6 margin by
// which accumulated probabilities may differ before an eviction is called a tie.
__device__ inline double exp_softmax_f64(double x)
{
  const double n = __builtin_rint(x * 1.44269504088896338700e+00);
  double r = fma(n, -6.93147180369123816490e-01, x);
  r = fma(n, -1.90821492927058770002e-10, r);
  double p = 2.75573192239858906526e-07;                   // 1 / 10!
  p = fma(p, r, 2.75573192239858906526e-06);
  p = fma(p, r, 2.48015873015873015873e-05);
  p = fma(p, r, 1.98412698412698412698e-04);
  p = fma(p, r, 1.38888888888888888889e-03);
  p = fma(p, r, 8.33333333333333333333e-03);
  p = fma(p, r, 4.16666666666666666667e-02);
  p = fma(p, r, 1.66666666666666666667e-01);
  p = fma(p, r, 0.5);
  p = fma(p, r, 1.0);
  p = fma(p, r, 1.0);
  return x > -708.0 ? __builtin_ldexp(p, (int)n) : 0.0;
}

// GELU, x * Phi(x) (Sec. 3.2 names GELU as the activation of both feature maps).
__device__ inline double gelu_f64(double x) { return 0.5 * x * erfc(-x * 0.70710678118654752440); }

// Branch-free fp32 GELU for the matrix-core feature maps.  With t = |x| the upper normal
// tail is Q(t) = exp(-t^2/2) * (c1 u + ... + c7 u^7), u = 1 / (1 + 0.24 t) (polynomial error
// 1e-9; constants from fit_gelu_poly.py), and gelu(x) = x - t Q(t) for x >= 0, -t Q(t) else.
// Absolute error in fp32: 2.5e-7 on [-4, 4], one ulp of x beyond.
__device__ inline float gelu_fast_f32(float x)
{
  const float t = fabsf(x);
  const float u = __builtin_amdgcn_rcpf(fmaf(0.24f, t, 1.0f));
  float a = -1.2459717568e-01f;
  a = fmaf(a, u, 5.5222350684e-01f);
  a = fmaf(a, u, -6.4138824846e-01f);
  a = fmaf(a, u, 6.2064721284e-01f);
  a = fmaf(a, u, -1.5113306584e-01f);
  a = fmaf(a, u, 1.5460257740e-01f);
  a = fmaf(a, u, 8.9645194151e-02f);
  a *= u;
  const float e = __builtin_amdgcn_exp2f(t * t * -0.72134752044448170368f);   // exp(-t^2/2)
  const float tq = t * (a * e);
  return x >= 0.f ? x - tq : -tq;
}

// The same approximation evaluated in fp64 (absolute error 1e-9): for the handful of
// layer-2 activations per row, whose inputs already carry the fp32 rounding of layer 1.
// Much lighter on registers than the library erfc.
__device__ inline double gelu_poly_f64(double x)
{
  const double t = fabs(x);
  const double u = 1.0 / fma(0.24, t, 1.0);
  double a = -1.2459717568e-01;
  a = fma(a, u, 5.5222350684e-01);
  a = fma(a, u, -6.4138824846e-01);
  a = fma(a, u, 6.2064721284e-01);
  a = fma(a, u, -1.5113306584e-01);
  a = fma(a, u, 1.5460257740e-01);
  a = fma(a, u, 8.9645194151e-02);
  a *= u;
  const double tq = t * (a * exp(-0.5 * t * t));
  return x >= 0.0 ? x - tq : -tq;
}

}  // namespace lessdec
