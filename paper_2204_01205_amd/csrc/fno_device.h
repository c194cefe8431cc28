// Device helpers shared by the kernel translation units of libfno (gfx950, wave64).
#pragma once
#include "fno_kernels.h"
#include <cmath>
#include "fft_reg.h"

namespace fno {

namespace {

constexpr int kThreads = 256;
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int kfreq(int j, int L, int npos) { return j < npos ? j : j - L; }
__device__ __forceinline__ int posmod(int a, int m) { int r = a % m; return r < 0 ? r + m : r; }

__device__ __forceinline__ float gelu_f(float z) {
  return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f));
}
// GELU for the forward epilogue without branches or erff: with x = |z|/sqrt(2),
//   erf(x) = 1 - (1 + a1 x + ... + a6 x^6)^-16   (Abramowitz & Stegun 7.1.28, |error| <= 3e-7)
// and z Phi(z) = (z + |z| erf(x)) / 2.  The error it adds to the output is below 2e-7 |z|.
__device__ __forceinline__ float gelu_fast_f(float z) {
  const float az = fabsf(z);
  const float x = az * 0.70710678118654752440f;
  float p = fmaf(x, 0.0000430638f, 0.0002765672f);
  p = fmaf(x, p, 0.0001520143f);
  p = fmaf(x, p, 0.0092705272f);
  p = fmaf(x, p, 0.0422820123f);
  p = fmaf(x, p, 0.0705230784f);
  p = fmaf(x, p, 1.0f);
  p = p * p; p = p * p; p = p * p; p = p * p;
  const float erfx = 1.0f - __builtin_amdgcn_rcpf(p);   // v_rcp_f32, 1 ulp
  return 0.5f * fmaf(az, erfx, z);
}
__device__ __forceinline__ float gelu_prime_f(float z) {
  const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * expf(-0.5f * z * z);
  return fmaf(z, pdf, cdf);
}

inline int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

#define FNO_DISPATCH_M(Mval, CALL)                \
  switch (Mval) {                                 \
    case 1: { constexpr int MM = 1; CALL; } break;   \
    case 2: { constexpr int MM = 2; CALL; } break;   \
    case 4: { constexpr int MM = 4; CALL; } break;   \
    case 8: { constexpr int MM = 8; CALL; } break;   \
    case 16: { constexpr int MM = 16; CALL; } break; \
    case 32: { constexpr int MM = 32; CALL; } break; \
    default: return hipErrorInvalidValue;         \
  }

}  // namespace

}  // namespace fno
