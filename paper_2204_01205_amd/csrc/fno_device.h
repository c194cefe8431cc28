// Device helpers shared by the kernel translation units of libfno (gfx950, wave64).
#pragma once
#include "fno_kernels.h"
#include <cmath>
#include "fft_reg.h"

namespace fno {

namespace {

constexpr int kThreads = 256;
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int kfreq(int j, int L, int npos) { return j < npos ? j : j - L; }
__device__ __forceinline__ int posmod(int a, int m) { int r = a % m; return r < 0 ? r + m : r; }

__device__ __forceinline__ float gelu_f(float z) {
  return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f));
}
// GELU for the forward epilogue without branches or erff.  With a = |z| and
//   erf(x) = 1 - (1 + a1 x + ... + a6 x^6)^-16          (Abramowitz & Stegun 7.1.28, |error| <= 3e-7)
// the upper tail is T(a) = (1 - erf(a / sqrt 2)) / 2 = q(a)^-16 with q(a) = 2^(1/16) (1 + sum_i a_i (a / sqrt 2)^i),
// and z Phi(z) = max(z, 0) - a T(a).  The constants below are q's coefficients 2^(1/16) a_i 2^(-i/2).
// 16 issue slots per value (the reciprocal counts four).  Error against the float64 definition,
// evaluated in float32: at most 7.1e-7 absolute.
__device__ __forceinline__ float gelu_fast_f(float z) {
  const float a = fabsf(z);
  float q = fmaf(a, 5.6212996640e-06f, 5.1055209009e-05f);
  q = fmaf(a, q, 3.9686137011e-05f);
  q = fmaf(a, q, 3.4227392389e-03f);
  q = fmaf(a, q, 2.2076998457e-02f);
  q = fmaf(a, q, 5.2075163037e-02f);
  q = fmaf(a, q, 1.0442737824f);
  q = q * q; q = q * q; q = q * q; q = q * q;
  const float t = __builtin_amdgcn_rcpf(q);             // v_rcp_f32, 1 ulp
  // max(z, 0) as a median of three (one instruction; fmaxf would first quiet a signalling NaN)
  return fmaf(-a, t, __builtin_amdgcn_fmed3f(z, 0.0f, __builtin_inff()));
}
__device__ __forceinline__ float gelu_prime_f(float z) {
  const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * expf(-0.5f * z * z);
  return fmaf(z, pdf, cdf);
}

// Loads and stores of data that a kernel touches once.  STREAM: with the nontemporal hint, so that
// a stream much larger than the caches does not displace what other kernels and blocks reuse.  The
// launchers set it for tensors above kStreamBytes; below that the whole working set can live in the
// 256 MB memory-side cache from one kernel to the next, and the hint would throw that away
// (measured: +16 % on a block forward whose tensors are 84 MB, -4..-5 % from 335 MB up).
constexpr long long kStreamBytes = 256ll << 20;
template <bool STREAM, class T>
__device__ __forceinline__ T ld_once(const T* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool STREAM, class T>
__device__ __forceinline__ void st_once(T* p, T v) {
  if constexpr (STREAM) __builtin_nontemporal_store(v, p);
  else *p = v;
}
template <bool STREAM>
__device__ __forceinline__ float2 ld_once2(const float2* p) {
  const v2f v = ld_once<STREAM>(reinterpret_cast<const v2f*>(p));
  return make_float2(v[0], v[1]);
}
template <bool STREAM>
__device__ __forceinline__ void st_once2(float2* p, float2 v) {
  st_once<STREAM>(reinterpret_cast<v2f*>(p), v2f{v.x, v.y});
}

// Thread blocks are dealt to the chip's eight XCDs round robin.  For a grid padded to a multiple of
// eight blocks this is the work item of block `bid` under which every XCD walks a contiguous eighth
// of the items, so that the memory it has in flight at one time spans an eighth of the pages
// (measured on the forward (t, z) kernel: 6 % faster, and less spread between allocations).  The
// caller drops items past the end.
__device__ __forceinline__ long long xcd_contiguous_item(unsigned bid, unsigned nblocks) {
  return (long long)(bid & 7) * (nblocks >> 3) + (bid >> 3);
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
