// Device helpers: sine/cosine of a double-precision argument, row copies.
#pragma once
#include <hip/hip_runtime.h>

namespace tgnn {

// sin and cos of `arg`.  The argument of the time encoding, w * dt + b, reaches ~1e6 rad, where one float
// ulp is a quarter of a radian; so the argument is formed and reduced to [-pi/4, pi/4] in double, and only
// the polynomial is evaluated in float (absolute error ~1e-7).
__device__ __forceinline__ void sincos_reduced(double arg, float& s, float& c) {
  // j = arg * 2/pi rounded to the nearest integer, by adding and taking off 1.5 * 2^52 (round-to-nearest mode): the
  // sum's low mantissa bits then are j's low bits in two's complement, which gives the quadrant j mod 4 without a
  // double -> integer conversion (the 64-bit one is a dozen double-precision instructions).  |arg| < 2^51.
  const double magic = 6755399441055744.0;
  const double t = fma(arg, 0.63661977236758134308, magic);     // 2/pi
  const int q = __double2loint(t) & 3;
  const double j = t - magic;
  double r = fma(-j, 1.57079632679489655800e+00, arg);          // pi/2 high part
  r = fma(-j, 6.12323399573676603587e-17, r);                   // pi/2 low part
  const float x = (float)r, x2 = x * x;
  const float sp = x + x * x2 * (-1.6666654611e-1f + x2 * (8.3321608736e-3f + x2 * (-1.9515295891e-4f)));
  const float cp = 1.0f - 0.5f * x2 +
                   x2 * x2 * (4.166664568298827e-2f + x2 * (-1.388731625493765e-3f + x2 * 2.443315711809948e-5f));
  s = (q & 1) ? cp : sp;
  c = (q & 1) ? sp : cp;
  if (q & 2) s = -s;
  if ((q + 1) & 2) c = -c;
}

__device__ __forceinline__ float time_enc(double delta, float w, float b) {
  float s, c;
  sincos_reduced(fma((double)w, delta, (double)b), s, c);
  return c;
}

// One wavefront copies n floats (dst, src aligned to VEC floats, n % VEC == 0) and appends nz zeros.
template <int VEC>
__device__ __forceinline__ void wave_copy(float* __restrict__ dst, const float* __restrict__ src, int n, int nz,
                                          int lane) {
  if (VEC == 4) {
    for (int i = lane; i < n / 4; i += 64)
      reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
  } else if (VEC == 2) {
    for (int i = lane; i < n / 2; i += 64)
      reinterpret_cast<float2*>(dst)[i] = reinterpret_cast<const float2*>(src)[i];
  } else {
    for (int i = lane; i < n; i += 64) dst[i] = src[i];
  }
  for (int i = lane; i < nz; i += 64) dst[n + i] = 0.f;
}

__device__ __forceinline__ void wave_zero(float* __restrict__ dst, int n, int lane) {
  for (int i = lane; i < n; i += 64) dst[i] = 0.f;
}

}  // namespace tgnn
