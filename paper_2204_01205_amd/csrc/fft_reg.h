// In-register radix-2 FFT of compile-time length M (power of two, 1..64) for one thread.
//
// Every index is a template constant, so the data array lives in VGPRs and the twiddles are
// immediate operands.  Decimation in frequency: natural-order input, bit-reversed output;
// out(k) of a length-M transform sits at a[bitrev<M>(k)].
//
// SIGN = -1 gives sum_n a[n] exp(-2 pi i k n / M) (the forward transform F of eq. (3) of the
// paper along one axis), SIGN = +1 the unnormalised inverse.
#pragma once
#include <hip/hip_runtime.h>
#include <utility>

namespace fno {

// ---- compile-time cos/sin of 2*pi*k/M ----------------------------------------------------
constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double ct_sin_series(double x) {   // |x| <= pi/4
  double term = x, sum = x;
  for (int n = 1; n < 12; ++n) { term *= -x * x / double((2 * n) * (2 * n + 1)); sum += term; }
  return sum;
}
constexpr double ct_cos_series(double x) {   // |x| <= pi/4
  double term = 1.0, sum = 1.0;
  for (int n = 1; n < 12; ++n) { term *= -x * x / double((2 * n - 1) * (2 * n)); sum += term; }
  return sum;
}
// cos(2 pi k / M), sin(2 pi k / M) for 0 <= k < M, reduced to the first octant exactly.
constexpr double ct_cos_frac(int k, int M) {
  k %= M; if (k < 0) k += M;
  if (2 * k > M) return ct_cos_frac(M - k, M);                 // cos(2pi - a) = cos a
  if (4 * k > M) return -ct_cos_frac(M - 2 * k, 2 * M) ;       // cos(pi - a): a = 2pi(M-2k)/(2M)
  if (8 * k > M) {                                             // cos(a) = sin(pi/2 - a)
    return ct_sin_series(2.0 * kPi * double(M - 4 * k) / double(4 * M));
  }
  return ct_cos_series(2.0 * kPi * double(k) / double(M));
}
constexpr double ct_sin_frac(int k, int M) {
  k %= M; if (k < 0) k += M;
  if (2 * k > M) return -ct_sin_frac(M - k, M);
  if (4 * k > M) return ct_sin_frac(M - 2 * k, 2 * M);
  if (8 * k > M) return ct_cos_series(2.0 * kPi * double(M - 4 * k) / double(4 * M));
  return ct_sin_series(2.0 * kPi * double(k) / double(M));
}

template <int M> constexpr int ct_log2() { int l = 0; for (int m = M; m > 1; m >>= 1) ++l; return l; }

template <int M> constexpr int bitrev(int k) {
  int r = 0;
  for (int b = 0; b < ct_log2<M>(); ++b) { r = (r << 1) | ((k >> b) & 1); }
  return r;
}

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
  return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
// a * conj(b)
__device__ __forceinline__ float2 cmulc(float2 a, float2 b) {
  return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}
__device__ __forceinline__ float2 cfma(float2 a, float2 b, float2 acc) {
  acc.x = fmaf(a.x, b.x, acc.x); acc.x = fmaf(-a.y, b.y, acc.x);
  acc.y = fmaf(a.x, b.y, acc.y); acc.y = fmaf(a.y, b.x, acc.y);
  return acc;
}
// acc += a * conj(b)
__device__ __forceinline__ float2 cfmac(float2 a, float2 b, float2 acc) {
  acc.x = fmaf(a.x, b.x, acc.x); acc.x = fmaf(a.y, b.y, acc.x);
  acc.y = fmaf(a.y, b.x, acc.y); acc.y = fmaf(-a.x, b.y, acc.y);
  return acc;
}

// v * exp(SIGN * 2 pi i * IDX / M) with the trivial cases written out.
template <int M, int IDX, int SIGN>
__device__ __forceinline__ float2 mul_root(float2 v) {
  constexpr int idx = ((IDX % M) + M) % M;
  if constexpr (idx == 0) {
    return v;
  } else if constexpr (2 * idx == M) {
    return make_float2(-v.x, -v.y);
  } else if constexpr (4 * idx == M) {           // * (SIGN) i
    return SIGN > 0 ? make_float2(-v.y, v.x) : make_float2(v.y, -v.x);
  } else if constexpr (4 * idx == 3 * M) {       // * (-SIGN) i
    return SIGN > 0 ? make_float2(v.y, -v.x) : make_float2(-v.y, v.x);
  } else {
    constexpr float c = float(ct_cos_frac(idx, M));
    constexpr float s = float(SIGN > 0 ? ct_sin_frac(idx, M) : -ct_sin_frac(idx, M));
    return make_float2(v.x * c - v.y * s, v.x * s + v.y * c);
  }
}

template <int M, int SIGN, int S, int I>
__device__ __forceinline__ void dif_butterfly(float2 (&a)[M]) {
  constexpr int len = M >> S;
  constexpr int half = len / 2;
  constexpr int blk = I / half;
  constexpr int j = I % half;
  constexpr int i0 = blk * len + j;
  constexpr int i1 = i0 + half;
  float2 u = a[i0], v = a[i1];
  a[i0] = cadd(u, v);
  a[i1] = mul_root<M, (j << S), SIGN>(csub(u, v));
}

template <int M, int SIGN, int S, int... Is>
__device__ __forceinline__ void dif_stage(float2 (&a)[M], std::integer_sequence<int, Is...>) {
  (dif_butterfly<M, SIGN, S, Is>(a), ...);
}

template <int M, int SIGN, int... Ss>
__device__ __forceinline__ void dif_all(float2 (&a)[M], std::integer_sequence<int, Ss...>) {
  (dif_stage<M, SIGN, Ss>(a, std::make_integer_sequence<int, M / 2>{}), ...);
}

// In-place transform; result k is at a[bitrev<M>(k)].
template <int M, int SIGN>
__device__ __forceinline__ void fft_reg(float2 (&a)[M]) {
  if constexpr (M > 1) {
    dif_all<M, SIGN>(a, std::make_integer_sequence<int, ct_log2<M>()>{});
  }
}

}  // namespace fno
