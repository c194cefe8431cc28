// HIP kernels of libfno for gfx950 (wave64).  What they compute, in the paper's terms
// (arXiv 2204.01205): the transform F of eq. (3) restricted to the kept low-frequency modes,
// applied axis by axis (separability, Sec. 2.3); the per-mode weight multiplication of R_phi;
// the inverse transform; and the pointwise part of the block update of eq. (2) / Sec. 2.4,
// sigma(W x + b + K x), fused into the last inverse stage.  The adjoint kernels implement the
// transposed chain (eq. (7)) and the sum-reductions that are the adjoint of broadcasting W
// and b (Sec. 2.1).
//
// Every axis of length N is split N = P * M: M-point FFTs held in registers (fft_reg.h) over
// the residue classes n = P*n1 + n2, then a P-term twiddle combine evaluated only at the kept
// frequencies.  M = 1 degenerates to a dense truncated DFT and covers any axis length.
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

// ------------------------------------------------------------------------------------------
// Twiddle tables (double-precision sincospi, rounded once to float)
// ------------------------------------------------------------------------------------------
__global__ void axis_table_kernel(float2* tw, int N, int L, int npos, int P) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= L * P) return;
  const int j = idx / P, n2 = idx % P;
  const long long k = kfreq(j, L, npos);
  long long r = (k * n2) % N;
  if (r < 0) r += N;
  double s, c;
  sincospi(-2.0 * double(r) / double(N), &s, &c);
  tw[idx] = make_float2(float(c), float(s));
}

__global__ void t_table_kernel(float2* tw, int Nt, int mt) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= Nt * mt) return;
  const int kt = idx / Nt, n = idx % Nt;
  const long long r = ((long long)kt * n) % Nt;
  double s, c;
  sincospi(-2.0 * double(r) / double(Nt), &s, &c);
  tw[idx] = make_float2(float(c), float(s));
}

// ------------------------------------------------------------------------------------------
// Forward (t, z): one block transforms `ppb` contiguous (b,c,nx,ny) planes of Nz x Nt reals
// ------------------------------------------------------------------------------------------
// sum_i w[i] * x[i * xs] over n terms, eight at a time so that their reads are issued together
// (a term-by-term loop waits for every read before the next one goes out)
__device__ __forceinline__ float2 combine_terms(const float2* w, const float2* x, int xs, int n) {
  float2 acc0 = make_float2(0.f, 0.f), acc1 = make_float2(0.f, 0.f);
  int i = 0;
  for (; i + 8 <= n; i += 8) {
    float2 wv[8], xv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      wv[u] = w[i + u];
      xv[u] = x[(i + u) * xs];
    }
#pragma unroll
    for (int u = 0; u < 8; u += 2) {
      acc0 = cfma(wv[u], xv[u], acc0);
      acc1 = cfma(wv[u + 1], xv[u + 1], acc1);
    }
  }
  for (; i < n; ++i) acc0 = cfma(w[i], x[i * xs], acc0);
  return make_float2(acc0.x + acc1.x, acc0.y + acc1.y);
}

// Row stride of the z-rows in LDS, in complex values: 1 mod 16, so that the rows of the kt bins
// that adjacent lanes combine start 2 banks apart.
__host__ __device__ inline int tz_row_stride(int Nz) { return Nz + ((17 - (Nz & 15)) & 15); }

template <int MZ>
__global__ __launch_bounds__(kThreads) void tz_fwd_kernel(
    const float* __restrict__ x, float2* __restrict__ out, const float2* __restrict__ twt,
    const float2* __restrict__ twz, long long planes, int Nz, int Nt, int Lz, int nposz, int mt,
    int ppb) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int Pz = Nz / MZ;
  const int sS = Nt + 1;                       // row stride of S in floats
  const int sT = tz_row_stride(Nz);            // row stride of T in float2
  float* S = smem;                             // [ppb][Nz][sS]
  int s_floats = ppb * Nz * sS;
  s_floats += (s_floats & 1);
  float2* T = reinterpret_cast<float2*>(smem + s_floats);   // [ppb][mt][sT]
  const int tid = threadIdx.x;
  const long long plane0 = (long long)blockIdx.x * ppb;
  const int np = (int)min((long long)ppb, planes - plane0);
  const int plane_elems = Nz * Nt;

  // 1. coalesced load of the planes
  const float* src = x + plane0 * plane_elems;
  const int nelem = np * plane_elems;
  for (int i0 = tid; i0 < nelem; i0 += 8 * kThreads) {     // eight loads in flight per thread
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = i0 + u * kThreads;
      v[u] = idx < nelem ? src[idx] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = i0 + u * kThreads;
      if (idx < nelem) {
        const int row = idx / Nt, t = idx - row * Nt;
        S[row * sS + t] = v[u];
      }
    }
  }
  __syncthreads();

  // 2. real-to-complex transform over t, kept bins only: one thread per z-row
  for (int row = tid; row < np * Nz; row += kThreads) {
    const int p = row / Nz, z = row - p * Nz;
    const float* srow = S + row * sS;
    for (int kt0 = 0; kt0 < mt; kt0 += 4) {
      float2 acc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = make_float2(0.f, 0.f);
      int n = 0;
      for (; n + 4 <= Nt; n += 4) {         // four points per pass: their reads go out together
        float v[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) v[h] = srow[n + h];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (kt0 + u < mt) {
            float2 w[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) w[h] = twt[(kt0 + u) * Nt + n + h];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
              acc[u].x = fmaf(v[h], w[h].x, acc[u].x);
              acc[u].y = fmaf(v[h], w[h].y, acc[u].y);
            }
          }
        }
      }
      for (; n < Nt; ++n) {
        const float v = srow[n];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (kt0 + u < mt) {
            const float2 w = twt[(kt0 + u) * Nt + n];
            acc[u].x = fmaf(v, w.x, acc[u].x);
            acc[u].y = fmaf(v, w.y, acc[u].y);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (kt0 + u < mt) T[(p * mt + kt0 + u) * sT + z] = acc[u];
    }
  }
  __syncthreads();

  // 3. MZ-point FFTs over the residue classes of z, in place
  if constexpr (MZ > 1) {
    for (int idx = tid; idx < np * mt * Pz; idx += kThreads) {
      const int n2 = idx % Pz, col = idx / Pz;          // col = p*mt + kt
      float2* base = T + col * sT + n2;
      float2 a[MZ];
#pragma unroll
      for (int n1 = 0; n1 < MZ; ++n1) a[n1] = base[Pz * n1];
      fft_reg<MZ, -1>(a);
#pragma unroll
      for (int m = 0; m < MZ; ++m) base[Pz * m] = a[bitrev<MZ>(m)];
    }
    __syncthreads();
  }

  // 4. twiddle combine at the kept z-frequencies
  for (int idx = tid; idx < np * Lz * mt; idx += kThreads) {
    const int kt = idx % mt;
    const int jz = (idx / mt) % Lz;
    const int p = idx / (mt * Lz);
    const int mj = posmod(kfreq(jz, Lz, nposz), MZ);
    const float2* base = T + (p * mt + kt) * sT + Pz * mj;
    const float2* w = twz + jz * Pz;
    out[((plane0 + p) * Lz + jz) * mt + kt] = combine_terms(w, base, 1, Pz);
  }
}

// ------------------------------------------------------------------------------------------
// Forward (t, z) for a z axis with no power of two in its length (the z transform is a dense
// truncated DFT) and Nt a multiple of 4.  Rows are read straight from memory (one float4 run per
// thread) for the real-to-complex t stage; the z stage, out[jz][(p,kt)] = sum_n w[jz][n]
// T[(p,kt)][n], is a matrix product on 16x16x4 fp32 MFMA tiles (lane l supplies A[l%16][l/16] and
// B[l/16][l%16], holds rows 4 (l/16) + v of column l%16): the 16 columns are the kt bins of
// 16/mt planes, the z rows (K) are dealt to the four waves, whose partial sums meet in LDS.
// ------------------------------------------------------------------------------------------
constexpr int kDenseMT = 3;     // row tiles (16 kept z-frequencies each) per sweep
// row stride in complex values, 4 mod 16: the 16 lanes of a K step read 4 columns x 4 rows that
// fall on distinct banks
__host__ __device__ inline int tzd_row_stride(int Nz) { return Nz + ((20 - (Nz & 15)) & 15); }

__global__ __launch_bounds__(kThreads) void tz_fwd_dense_kernel(
    const float* __restrict__ x, float2* __restrict__ out, const float2* __restrict__ twt,
    const float2* __restrict__ twz, long long planes, int Nz, int Nt, int Lz, int mt, int ppb, int alias) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int sT = tzd_row_stride(Nz);
  float2* T = reinterpret_cast<float2*>(smem);                 // [16][sT]
  // [4][kDenseMT * 16][16] partial sums; when one sweep covers all kept z-frequencies they take
  // T's place once the sweep has read it (alias = 1), which halves the block's LDS
  float2* P = alias ? T : T + 16 * sT;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, lr = lane & 15, lk = lane >> 4;
  const long long plane0 = (long long)blockIdx.x * ppb;
  const int np = (int)min((long long)ppb, planes - plane0);
  const int ncol = np * mt;

  // t stage: one thread per z-row, every kept bin
  for (int row = tid; row < np * Nz; row += kThreads) {
    const int p = row / Nz, z = row - p * Nz;
    const float4* xr = reinterpret_cast<const float4*>(x + ((plane0 + p) * Nz + z) * (long long)Nt);
    float2 acc[16];
#pragma unroll
    for (int kt = 0; kt < 16; ++kt) acc[kt] = make_float2(0.f, 0.f);
    for (int n = 0; n < Nt; n += 4) {
      const float4 v = xr[n >> 2];
#pragma unroll
      for (int kt = 0; kt < 16; ++kt) {
        if (kt < mt) {
          const float2* wp = twt + kt * Nt + n;
          const float2 w0 = wp[0], w1 = wp[1], w2 = wp[2], w3 = wp[3];
          acc[kt].x = fmaf(v.x, w0.x, acc[kt].x); acc[kt].y = fmaf(v.x, w0.y, acc[kt].y);
          acc[kt].x = fmaf(v.y, w1.x, acc[kt].x); acc[kt].y = fmaf(v.y, w1.y, acc[kt].y);
          acc[kt].x = fmaf(v.z, w2.x, acc[kt].x); acc[kt].y = fmaf(v.z, w2.y, acc[kt].y);
          acc[kt].x = fmaf(v.w, w3.x, acc[kt].x); acc[kt].y = fmaf(v.w, w3.y, acc[kt].y);
        }
      }
    }
#pragma unroll
    for (int kt = 0; kt < 16; ++kt)
      if (kt < mt) T[(p * mt + kt) * sT + z] = acc[kt];
  }
  __syncthreads();

  // z stage
  const int nmt = (Lz + 15) >> 4, ksteps = (Nz + 3) >> 2;
  for (int mg = 0; mg < nmt; mg += kDenseMT) {
    v4f re[kDenseMT], im[kDenseMT];
#pragma unroll
    for (int m = 0; m < kDenseMT; ++m) {
      re[m] = v4f{0.f, 0.f, 0.f, 0.f};
      im[m] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    for (int s0 = w; s0 < ksteps; s0 += 8) {           // two K steps per pass: their loads go out together
      float2 bv[2], av[2][kDenseMT];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int n = 4 * (s0 + 4 * u) + lk;
        const bool nok = n < Nz;
        bv[u] = (nok && lr < ncol) ? T[lr * sT + n] : make_float2(0.f, 0.f);
#pragma unroll
        for (int m = 0; m < kDenseMT; ++m) {
          const int jz = (mg + m) * 16 + lr;
          av[u][m] = (nok && jz < Lz) ? twz[jz * Nz + n] : make_float2(0.f, 0.f);
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int m = 0; m < kDenseMT; ++m) {
          re[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][m].x, bv[u].x, re[m], 0, 0, 0);
          re[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(-av[u][m].y, bv[u].y, re[m], 0, 0, 0);
          im[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][m].x, bv[u].y, im[m], 0, 0, 0);
          im[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u][m].y, bv[u].x, im[m], 0, 0, 0);
        }
    }
    if (alias) __syncthreads();                          // every wave is done reading T
#pragma unroll
    for (int m = 0; m < kDenseMT; ++m)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        P[(w * (kDenseMT * 16) + m * 16 + 4 * lk + v) * 16 + lr] = make_float2(re[m][v], im[m][v]);
    __syncthreads();
    for (int idx = tid; idx < np * (kDenseMT * 16) * mt; idx += kThreads) {
      const int kt = idx % mt;
      const int jzl = (idx / mt) % (kDenseMT * 16);
      const int p = idx / (mt * kDenseMT * 16);
      const int jz = mg * 16 + jzl;
      if (jz < Lz) {
        const int col = p * mt + kt;
        float2 sum = make_float2(0.f, 0.f);
#pragma unroll
        for (int ww = 0; ww < kThreads / 64; ++ww) {
          const float2 v = P[(ww * (kDenseMT * 16) + jzl) * 16 + col];
          sum.x += v.x; sum.y += v.y;
        }
        out[((plane0 + p) * Lz + jz) * mt + kt] = sum;
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// Forward (t, z) for power-of-two Nt (16, 32, 64): float4 loads issued up front, the t stage as
// a real-input FFT of one z-row per thread (an NT/2-point complex FFT of the even/odd samples
// plus the split step), z twiddles in LDS.
// ------------------------------------------------------------------------------------------
// X[K] = E[K] + w^K O[K],  E = (Z[K] + conj Z[H-K]) / 2,  O = (Z[K] - conj Z[H-K]) / (2i)
template <int NT, int K>
__device__ __forceinline__ void rfft_bin(const float2 (&zc)[NT / 2], int mt, float2 (&X)[NT / 2 + 1]) {
  constexpr int H = NT / 2;
  if (K < mt) {
    const float2 zk = zc[bitrev<H>(K % H)];
    const float2 zm = zc[bitrev<H>((H - K) % H)];
    const float2 e = make_float2(0.5f * (zk.x + zm.x), 0.5f * (zk.y - zm.y));
    const float2 od = make_float2(0.5f * (zk.y + zm.y), -0.5f * (zk.x - zm.x));
    X[K] = cadd(e, mul_root<NT, K, -1>(od));
  }
}

template <int NT, int... Ks>
__device__ __forceinline__ void rfft_bins(const float2 (&zc)[NT / 2], int mt, float2 (&X)[NT / 2 + 1],
                                          std::integer_sequence<int, Ks...>) {
  (rfft_bin<NT, Ks>(zc, mt, X), ...);
}

// Bins 0..mt-1 of the real-input transform of one row of NT floats held as NT/4 float4 quads.
template <int NT>
__device__ __forceinline__ void rfft_row_bins(const float4 (&quads)[NT / 4], int mt, float2 (&X)[NT / 2 + 1]) {
  constexpr int H = NT / 2;
  float2 zc[H];
#pragma unroll
  for (int m4 = 0; m4 < NT / 4; ++m4) {
    zc[2 * m4] = make_float2(quads[m4].x, quads[m4].y);
    zc[2 * m4 + 1] = make_float2(quads[m4].z, quads[m4].w);
  }
  fft_reg<H, -1>(zc);
  rfft_bins<NT>(zc, mt, X, std::make_integer_sequence<int, H + 1>{});
}

// One thread per z-row (blockDim.x >= ppb * Nz).  The planes and the z twiddles go straight to
// LDS (16 bytes per lane, 1 KiB per wave instruction, nothing staged in registers).  Inside a
// row the quads are stored rotated by the row number so that the row-per-thread reads of the
// t stage spread over all banks; a wave's load still covers whole 128-byte lines.  The t-stage
// results wait in registers over a barrier so the complex tile T can reuse the LDS of S.
// Pz is a power of two and inv_mt = ceil(2^16 / mt) (shifts and a multiply instead of divisions).
template <int NT, int MZ>
__global__ __launch_bounds__(kThreads) void tz_fwd_fast_kernel(
    const float* __restrict__ x, float2* __restrict__ out, const float2* __restrict__ twz,
    long long planes, int Nz, int Lz, int nposz, int mt, int ppb, int region_floats, int pzshift,
    int inv_mt) {
  HIP_DYNAMIC_SHARED(float, smem)
  constexpr int QPR = NT / 4;                  // quads per row
  constexpr int ROT = 16 / QPR > 0 ? 16 / QPR : 1;   // rows that share a rotation
  constexpr int H = NT / 2;
  const int Pz = 1 << pzshift;
  const int sT = tz_row_stride(Nz);            // row stride of T in float2
  float* S = smem;                             // [ppb * Nz] rows of QPR rotated quads
  float2* T = reinterpret_cast<float2*>(smem); // [ppb][mt][sT], same memory, later
  float2* TW = reinterpret_cast<float2*>(smem + region_floats);   // [Lz][Pz]
  const int tid = threadIdx.x;
  const int nthr = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6;
  const long long plane0 = (long long)blockIdx.x * ppb;
  const int np = (int)min((long long)ppb, planes - plane0);

  {
    const float4* src = reinterpret_cast<const float4*>(x + plane0 * Nz * NT);
    const int tot4 = np * Nz * QPR;            // a multiple of 64 (checked on the host)
    for (int c0 = wave * 64; c0 < tot4; c0 += nthr) {
      const int p4 = c0 + lane;
      const int zl = p4 / QPR, sl = p4 - zl * QPR;
      const int q = (sl - zl / ROT) & (QPR - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + zl * QPR + q),
                                       (__attribute__((address_space(3))) void*)(S + 4 * c0), 16, 0, 0);
    }
    const float4* tsrc = reinterpret_cast<const float4*>(twz);
    const int tw4 = (Lz << pzshift) >> 1;      // float4 pieces of the twiddle table (Lz * Pz even)
    for (int c0 = wave * 64; c0 < tw4; c0 += nthr) {
      int f = c0 + lane;
      f = f < tw4 ? f : tw4 - 1;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(tsrc + f),
                                       (__attribute__((address_space(3))) void*)(smem + region_floats + 4 * c0),
                                       16, 0, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  __syncthreads();

  const bool live = tid < np * Nz;
  float2 X[H + 1];
  if (live) {
    float4 quads[QPR];
#pragma unroll
    for (int q = 0; q < QPR; ++q)
      quads[q] = *reinterpret_cast<const float4*>(S + 4 * (tid * QPR + ((q + tid / ROT) & (QPR - 1))));
    rfft_row_bins<NT>(quads, mt, X);
  }
  __syncthreads();
  if (live) {
    const int p = tid / Nz, z = tid - p * Nz;
#pragma unroll
    for (int k = 0; k <= H; ++k)
      if (k < mt) T[(p * mt + k) * sT + z] = X[k];
  }
  __syncthreads();

  if constexpr (MZ > 1) {
    for (int idx = tid; idx < ((np * mt) << pzshift); idx += nthr) {
      const int n2 = idx & (Pz - 1), col = idx >> pzshift;
      float2* base = T + col * sT + n2;
      float2 a[MZ];
#pragma unroll
      for (int n1 = 0; n1 < MZ; ++n1) a[n1] = base[n1 << pzshift];
      fft_reg<MZ, -1>(a);
#pragma unroll
      for (int m = 0; m < MZ; ++m) base[m << pzshift] = a[bitrev<MZ>(m)];
    }
    __syncthreads();
  }

  for (int p = 0; p < np; ++p) {
    float2* dst = out + (plane0 + p) * (long long)(Lz * mt);
    for (int idx = tid; idx < Lz * mt; idx += nthr) {
      const int jz = (idx * inv_mt) >> 16;
      const int kt = idx - jz * mt;
      const int mj = posmod(kfreq(jz, Lz, nposz), MZ);
      const float2* base = T + (p * mt + kt) * sT + (mj << pzshift);
      const float2* w = TW + (jz << pzshift);
      float2 acc = make_float2(0.f, 0.f);
      for (int n2 = 0; n2 < Pz; ++n2) acc = cfma(w[n2], base[n2], acc);
      dst[idx] = acc;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Complex pruned transform along the middle axis of [outer][N][inner] -> [outer][L][inner]
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kThreads) void axis_fwd_kernel(
    const float2* __restrict__ in, float2* __restrict__ out, const float2* __restrict__ tw, int N,
    int L, int npos, long long inner, int W, int ncb, int tw_lds) {
  HIP_DYNAMIC_SHARED(float, smem)
  float2* F = reinterpret_cast<float2*>(smem);          // [N][W]
  float2* TWs = F + N * W;                              // [L][P], only when tw_lds
  const int P = N / M;
  const int tid = threadIdx.x;
  const int nthr = blockDim.x;
  const long long o = blockIdx.x / ncb;
  const long long c0 = (long long)(blockIdx.x % ncb) * W;
  const int wc = (int)min((long long)W, inner - c0);

  if (tw_lds)
    for (int idx = tid; idx < L * P; idx += nthr) TWs[idx] = tw[idx];
  for (int idx = tid; idx < P * W; idx += nthr) {
    const int col = idx % W, n2 = idx / W;
    if (col < wc) {
      const float2* src = in + (o * N + n2) * inner + c0 + col;
      float2 a[M];
#pragma unroll
      for (int n1 = 0; n1 < M; ++n1) a[n1] = src[(long long)(P * n1) * inner];
      fft_reg<M, -1>(a);
#pragma unroll
      for (int m = 0; m < M; ++m) F[(P * m + n2) * W + col] = a[bitrev<M>(m)];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < L * W; idx += nthr) {
    const int col = idx % W, j = idx / W;
    if (col < wc) {
      const int mj = posmod(kfreq(j, L, npos), M);
      const float2* base = F + (P * mj) * W + col;
      const float2* w = (tw_lds ? TWs : tw) + j * P;
      out[(o * L + j) * inner + c0 + col] = combine_terms(w, base, W, P);
    }
  }
}

// [outer][L][inner] (kept frequencies, zero elsewhere) -> [outer][N][inner], exp(+i...)
template <int M>
__global__ __launch_bounds__(kThreads) void axis_inv_kernel(
    const float2* __restrict__ in, float2* __restrict__ out, const float2* __restrict__ tw, int N,
    int L, int npos, long long inner, int W, int ncb, int tw_lds) {
  HIP_DYNAMIC_SHARED(float, smem)
  float2* Y = reinterpret_cast<float2*>(smem);          // [L][W]
  float2* TWs = Y + L * W;                              // [L][P], only when tw_lds
  const float2* twp = tw_lds ? TWs : tw;
  const int P = N / M;
  const int tid = threadIdx.x;
  const int nthr = blockDim.x;
  const long long o = blockIdx.x / ncb;
  const long long c0 = (long long)(blockIdx.x % ncb) * W;
  const int wc = (int)min((long long)W, inner - c0);
  const int kmin = npos - L, kmax = npos - 1;

  if (tw_lds)
    for (int idx = tid; idx < L * P; idx += nthr) TWs[idx] = tw[idx];
  for (int i0 = tid; i0 < L * W; i0 += 8 * nthr) {         // eight loads in flight per thread
    float2 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = i0 + u * nthr;
      const int col = idx % W, j = idx / W;
      v[u] = (idx < L * W && col < wc) ? in[(o * L + j) * inner + c0 + col] : make_float2(0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = i0 + u * nthr;
      if (idx < L * W && idx % W < wc) Y[idx] = v[u];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < P * W; idx += nthr) {
    const int col = idx % W, n2 = idx / W;
    if (col < wc) {
      float2 g[M];
#pragma unroll
      for (int m = 0; m < M; ++m) {
        float2 acc = make_float2(0.f, 0.f);
        for (int k = kmin + posmod(m - kmin, M); k <= kmax; k += M) {
          const int j = k >= 0 ? k : k + L;
          acc = cfmac(Y[j * W + col], twp[j * P + n2], acc);
        }
        g[m] = acc;
      }
      fft_reg<M, +1>(g);
      float2* dst = out + (o * N + n2) * inner + c0 + col;
#pragma unroll
      for (int n1 = 0; n1 < M; ++n1) dst[(long long)(P * n1) * inner] = g[bitrev<M>(n1)];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Per-mode channel mix (the learned weight multiplication inside R_phi)
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float mode_scale(long long k, int mt, int Nt, float invN) {
  const int kt = (int)(k % mt);
  const bool single = (kt == 0) || ((Nt % 2 == 0) && (kt == Nt / 2));
  return single ? invN : 2.0f * invN;
}

constexpr int kMixB = 4;   // batch entries held per pass
constexpr int kMixO = 4;   // output channels per thread in the forward mix

__global__ __launch_bounds__(kThreads) void mix_fwd_kernel(
    const float2* __restrict__ xh, const float2* __restrict__ R, float2* __restrict__ yh, int B,
    int Ci, int Co, long long K, int mt, int Nt, float invN) {
  // one thread: one mode, kMixO output channels, kMixB batch entries; R is read exactly once
  const long long k = (long long)blockIdx.x * kThreads + threadIdx.x;
  const int o0 = blockIdx.y * kMixO;
  if (k >= K) return;
  const float sc = mode_scale(k, mt, Nt, invN);
  for (int b0 = 0; b0 < B; b0 += kMixB) {
    float2 acc[kMixB][kMixO];
#pragma unroll
    for (int u = 0; u < kMixB; ++u)
#pragma unroll
      for (int v = 0; v < kMixO; ++v) acc[u][v] = make_float2(0.f, 0.f);
    for (int i = 0; i < Ci; ++i) {
      float2 xv[kMixB];
#pragma unroll
      for (int u = 0; u < kMixB; ++u)
        xv[u] = (b0 + u < B) ? xh[((long long)(b0 + u) * Ci + i) * K + k] : make_float2(0.f, 0.f);
#pragma unroll
      for (int v = 0; v < kMixO; ++v) {
        if (o0 + v < Co) {
          const float2 r = R[((long long)i * Co + o0 + v) * K + k];
#pragma unroll
          for (int u = 0; u < kMixB; ++u) acc[u][v] = cfma(xv[u], r, acc[u][v]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kMixB; ++u)
#pragma unroll
      for (int v = 0; v < kMixO; ++v)
        if (b0 + u < B && o0 + v < Co)
          yh[((long long)(b0 + u) * Co + o0 + v) * K + k] = make_float2(acc[u][v].x * sc, acc[u][v].y * sc);
  }
}

// One thread: one mode k, kMixI input channels, the batch in chunks of kMixB; the gradient
// spectrum gh is then read once per kMixI input channels.
constexpr int kMixI = 4;
__global__ __launch_bounds__(kThreads) void mix_bwd_kernel(
    const float2* __restrict__ xh, const float2* __restrict__ R, const float2* __restrict__ gh,
    float2* __restrict__ gR, float2* __restrict__ gxh, int B, int Ci, int Co, long long K, int mt,
    int Nt, float invN) {
  const long long k = (long long)blockIdx.x * kThreads + threadIdx.x;
  const int i0 = blockIdx.y * kMixI;
  if (k >= K) return;
  const float sc = mode_scale(k, mt, Nt, invN);
  for (int b0 = 0; b0 < B; b0 += kMixB) {
    float2 xv[kMixB][kMixI], gx[kMixB][kMixI];
#pragma unroll
    for (int u = 0; u < kMixB; ++u)
#pragma unroll
      for (int v = 0; v < kMixI; ++v) {
        gx[u][v] = make_float2(0.f, 0.f);
        xv[u][v] = (b0 + u < B && i0 + v < Ci) ? xh[((long long)(b0 + u) * Ci + i0 + v) * K + k]
                                               : make_float2(0.f, 0.f);
      }
    for (int o = 0; o < Co; ++o) {
      float2 r[kMixI], gr[kMixI], gy[kMixB];
#pragma unroll
      for (int v = 0; v < kMixI; ++v) {
        const long long ridx = ((long long)(i0 + v) * Co + o) * K + k;
        r[v] = i0 + v < Ci ? R[ridx] : make_float2(0.f, 0.f);
        gr[v] = (gR != nullptr && b0 > 0 && i0 + v < Ci) ? gR[ridx] : make_float2(0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < kMixB; ++u) {
        gy[u] = b0 + u < B ? gh[((long long)(b0 + u) * Co + o) * K + k] : make_float2(0.f, 0.f);
        gy[u].x *= sc; gy[u].y *= sc;
      }
#pragma unroll
      for (int u = 0; u < kMixB; ++u)
#pragma unroll
        for (int v = 0; v < kMixI; ++v) {
          gr[v] = cfmac(gy[u], xv[u][v], gr[v]);        // conj(xh) * gy
          gx[u][v] = cfmac(gy[u], r[v], gx[u][v]);      // conj(R) * gy
        }
      if (gR != nullptr) {
#pragma unroll
        for (int v = 0; v < kMixI; ++v)
          if (i0 + v < Ci) gR[((long long)(i0 + v) * Co + o) * K + k] = gr[v];
      }
    }
    if (gxh != nullptr) {
#pragma unroll
      for (int u = 0; u < kMixB; ++u)
#pragma unroll
        for (int v = 0; v < kMixI; ++v)
          if (b0 + u < B && i0 + v < Ci) gxh[((long long)(b0 + u) * Ci + i0 + v) * K + k] = gx[u][v];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Inverse (z, t) with the block epilogue.  One block: all output channels of one (b,nx,ny)
// column, for the z rows of Q consecutive residue classes (z = Pz*n1 + n2).
// ------------------------------------------------------------------------------------------
struct EpiArgs {
  const float* u; int Cu; const float* W; int w_so, w_si; const float* bias; float* zsave; int act;
};

// The epilogue of one grid point: all output channels.  EXACT: the channel counts fill the
// register tile, so no per-channel guards (they cost scalar registers the compiler then spills).
template <int CO, bool EXACT>
__device__ __forceinline__ void zt_epilogue_point(const EpiArgs& ep, int Co, const float* WS, const float* Y,
                                                  int Rz, int sY, int r, int t, long long b, long long off,
                                                  long long Npts, float* __restrict__ out) {
  float acc[CO];
#pragma unroll
  for (int o = 0; o < CO; ++o) acc[o] = (ep.bias != nullptr && (EXACT || o < Co)) ? ep.bias[o] : 0.f;
  if (ep.u != nullptr) {
    const float* up = ep.u + (b * ep.Cu) * Npts + off;
    int i = 0;
    if (EXACT || ep.Cu <= CO) {              // every input channel of the point at once: one round trip
      float xv[CO];
#pragma unroll
      for (int h = 0; h < CO; ++h) xv[h] = (EXACT || h < ep.Cu) ? up[h * Npts] : 0.f;
#pragma unroll
      for (int h = 0; h < CO; ++h)
        if (EXACT || h < ep.Cu) {
#pragma unroll
          for (int o = 0; o < CO; ++o) acc[o] = fmaf(WS[h * CO + o], xv[h], acc[o]);
        }
      i = ep.Cu;
    }
    for (; i < ep.Cu; ++i) {                 // more input channels than the register tile: one at a time
      const float xv = up[i * Npts];
#pragma unroll
      for (int o = 0; o < CO; ++o)
        if (o < Co) acc[o] = fmaf(ep.W[o * ep.w_so + i * ep.w_si], xv, acc[o]);
    }
  }
#pragma unroll
  for (int o = 0; o < CO; ++o) {
    if (EXACT || o < Co) {
      const float zv = acc[o] + Y[(o * Rz + r) * sY + t];
      const long long oidx = (b * Co + o) * Npts + off;
      if (ep.zsave != nullptr) ep.zsave[oidx] = zv;
      out[oidx] = ep.act ? gelu_fast_f(zv) : zv;
    }
  }
}

// The t stage can hold a block's results in registers (eight 16-row tiles per wave, one 16-wide
// tile of t) until every wave has read V, and then write Y over V: one LDS buffer instead of two.
__host__ __device__ inline bool zt_y_over_v(int Nt, int rows, int mt) {
  return Nt <= 16 && rows <= 512 && 2 * mt <= 36;
}

template <int MZ, int CO, bool EXACT>
__global__ __launch_bounds__(kThreads) void zt_inv_kernel(
    const float2* __restrict__ a, float* __restrict__ out, const float2* __restrict__ twt,
    const float2* __restrict__ twz, int Co, int NxNy, int Nz, int Nt, int Lz, int nposz, int mt,
    int Q, EpiArgs ep) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int Pz = Nz / MZ;
  const int G = (Pz + Q - 1) / Q;             // the last group of residue classes may be ragged
  const int Rz = Q * MZ;
  const int sY = Nt + 1;
  float2* V = reinterpret_cast<float2*>(smem);                 // [Co][Rz][mt]
  const bool y_over_v = zt_y_over_v(Nt, Co * Rz, mt);
  float* Y = y_over_v ? smem : smem + 2 * Co * Rz * mt;        // [Co][Rz][sY]
  const int vy_floats = y_over_v ? max(2 * Co * Rz * mt, Co * Rz * sY) : 2 * Co * Rz * mt + Co * Rz * sY;
  float* WS = smem + ((vy_floats + 3) & ~3);                   // [Cu][CO]: W of the epilogue, zero past Co
  const int tid = threadIdx.x;
  if (ep.u != nullptr && ep.Cu <= CO)
    for (int idx = tid; idx < ep.Cu * CO; idx += kThreads) {
      const int i = idx / CO, o = idx - i * CO;
      WS[idx] = o < Co ? ep.W[o * ep.w_so + i * ep.w_si] : 0.f;
    }
  const long long bxy = blockIdx.x / G;
  const int g = blockIdx.x % G;
  const long long b = bxy / NxNy;
  const long long xy = bxy % NxNy;
  const int kmin = nposz - Lz, kmax = nposz - 1;

  // Z, dense (no power of two in Nz): V[q][(o,kt)] = sum_j conj(tw[j][n2]) a[j][(o,kt)] is a
  // matrix product; 16x16x4 fp32 MFMA tiles (lane l supplies A[l%16][l/16] and B[l/16][l%16] and
  // holds rows 4 (l/16) + v of column l%16), real and imaginary part as two accumulators.
  if constexpr (MZ == 1) {
    const int wv_id = tid >> 6, lane = tid & 63, lr = lane & 15, lk = lane >> 4;
    const int ncol = Co * mt;
    const int nct = (ncol + 15) >> 4, nrt = (Q + 15) >> 4;
    const int ksteps = (Lz + 3) >> 2;
    const float2* abase = a + ((b * Co) * NxNy + xy) * (long long)Lz * mt;
    for (int pair = wv_id; pair < nrt * nct; pair += kThreads / 64) {
      const int rt = pair / nct, ct = pair - rt * nct;
      const int q = rt * 16 + lr, n2 = g * Q + q;
      const bool rowok = q < Q && n2 < Pz;
      const int n = ct * 16 + lr;
      const bool colok = n < ncol;
      const int o = colok ? n / mt : 0, kt = colok ? n - o * mt : 0;
      const float2* src = abase + (long long)o * NxNy * Lz * mt + kt;
      v4f re = {0.f, 0.f, 0.f, 0.f}, im = {0.f, 0.f, 0.f, 0.f};
      for (int s0 = 0; s0 < ksteps; s0 += 8) {       // eight K steps per pass: 16 loads in flight per lane
        float2 wv[8], av[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int j = 4 * (s0 + u) + lk;
          const bool ok = j < Lz;
          wv[u] = (ok && rowok) ? twz[j * Pz + n2] : make_float2(0.f, 0.f);
          av[u] = (ok && colok) ? src[j * mt] : make_float2(0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          re = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[u].x, av[u].x, re, 0, 0, 0);
          re = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[u].y, av[u].y, re, 0, 0, 0);
          im = __builtin_amdgcn_mfma_f32_16x16x4f32(wv[u].x, av[u].y, im, 0, 0, 0);
          im = __builtin_amdgcn_mfma_f32_16x16x4f32(-wv[u].y, av[u].x, im, 0, 0, 0);
        }
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int qq = rt * 16 + 4 * lk + v;
        if (qq < Q && colok) V[((o * Rz) + qq) * mt + kt] = make_float2(re[v], im[v]);
      }
    }
  } else
  // Z: gather the kept z-frequencies with their twiddle into MZ bins, inverse FFT over n1
  for (int idx = tid; idx < Co * mt * Q; idx += kThreads) {
    const int q = idx % Q;
    const int kt = (idx / Q) % mt;
    const int o = idx / (Q * mt);
    const int n2 = g * Q + q;
    if (n2 >= Pz) continue;
    const float2* src = a + (((b * Co + o) * NxNy + xy) * Lz) * mt + kt;
    float2 gbin[MZ];
#pragma unroll
    for (int m = 0; m < MZ; ++m) {
      float2 acc = make_float2(0.f, 0.f);
      int k = kmin + posmod(m - kmin, MZ);
      // several terms at a time: their loads (global memory, served by L2) go out together;
      // more of them where the bins leave the registers free (dense or nearly dense z)
      constexpr int UB = MZ <= 2 ? 16 : 4;
      for (; k + (UB - 1) * MZ <= kmax; k += UB * MZ) {
        float2 av[UB], wv[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          const int kk = k + u * MZ;
          const int j = kk >= 0 ? kk : kk + Lz;
          av[u] = src[j * mt];
          wv[u] = twz[j * Pz + n2];
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) acc = cfmac(av[u], wv[u], acc);
      }
      for (; k <= kmax; k += MZ) {
        const int j = k >= 0 ? k : k + Lz;
        acc = cfmac(src[j * mt], twz[j * Pz + n2], acc);
      }
      gbin[m] = acc;
    }
    fft_reg<MZ, +1>(gbin);
#pragma unroll
    for (int n1 = 0; n1 < MZ; ++n1) V[((o * Rz) + n1 * Q + q) * mt + kt] = gbin[bitrev<MZ>(n1)];
  }
  __syncthreads();

  // T: complex-to-real over t.  Y[row][t] = sum_kk Vf[row][kk] Wf[kk][t] over the 2 mt real and
  // imaginary parts of a row: 16x16x4 MFMA tiles, the table operand held in registers.
  constexpr int kTSteps = 9;
  if (2 * mt <= 4 * kTSteps) {
    const int wv_id = tid >> 6, lane = tid & 63, lr = lane & 15, lk = lane >> 4;
    const float* Vf = reinterpret_cast<const float*>(V);
    const float* twf = reinterpret_cast<const float*>(twt);
    const int K2 = 2 * mt, kst = (K2 + 3) >> 2;
    const int nrows = Co * Rz;
    const int nrt = (nrows + 15) >> 4, ntt = (Nt + 15) >> 4;
    if (y_over_v) {
      const int t = lr;
      float bt[kTSteps];
#pragma unroll
      for (int s = 0; s < kTSteps; ++s) {
        const int kk = 4 * s + lk;
        bt[s] = (kk < K2 && t < Nt) ? twf[((kk >> 1) * Nt + t) * 2 + (kk & 1)] : 0.f;
      }
      v4f accs[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int rt = wv_id + (kThreads / 64) * k;
        accs[k] = v4f{0.f, 0.f, 0.f, 0.f};
        if (rt < nrt) {
          const int row = rt * 16 + lr;
#pragma unroll
          for (int s = 0; s < kTSteps; ++s) {
            if (s < kst) {
              const int kk = 4 * s + lk;
              const float av = (row < nrows && kk < K2) ? Vf[row * K2 + kk] : 0.f;
              accs[k] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bt[s], accs[k], 0, 0, 0);
            }
          }
        }
      }
      __syncthreads();                           // every wave has read its rows of V
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int rt = wv_id + (kThreads / 64) * k;
        if (rt < nrt) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int r2 = rt * 16 + 4 * lk + v;
            if (r2 < nrows && t < Nt) Y[r2 * sY + t] = accs[k][v];
          }
        }
      }
    } else
    for (int tt = 0; tt < ntt; ++tt) {
      const int t = tt * 16 + lr;
      float bt[kTSteps];
#pragma unroll
      for (int s = 0; s < kTSteps; ++s) {
        const int kk = 4 * s + lk;
        bt[s] = (kk < K2 && t < Nt) ? twf[((kk >> 1) * Nt + t) * 2 + (kk & 1)] : 0.f;
      }
      for (int rt = wv_id; rt < nrt; rt += kThreads / 64) {
        const int row = rt * 16 + lr;
        v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kTSteps; ++s) {
          if (s < kst) {
            const int kk = 4 * s + lk;
            const float av = (row < nrows && kk < K2) ? Vf[row * K2 + kk] : 0.f;
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bt[s], acc, 0, 0, 0);
          }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r2 = rt * 16 + 4 * lk + v;
          if (r2 < nrows && t < Nt) Y[r2 * sY + t] = acc[v];
        }
      }
    }
  } else
  for (int idx = tid; idx < Co * Rz; idx += kThreads) {
    const float2* vrow = V + idx * mt;
    float* yrow = Y + idx * sY;
    for (int n0 = 0; n0 < Nt; n0 += 4) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      for (int kt = 0; kt < mt; ++kt) {
        const float2 v = vrow[kt];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (n0 + u < Nt) {
            const float2 w = twt[kt * Nt + n0 + u];
            acc[u] = fmaf(v.x, w.x, acc[u]);
            acc[u] = fmaf(v.y, w.y, acc[u]);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (n0 + u < Nt) yrow[n0 + u] = acc[u];
    }
  }
  __syncthreads();

  // E: out = act(ys + W u + bias), one thread per point, all channels
  const long long Npts = (long long)NxNy * Nz * Nt;
  for (int idx = tid; idx < Rz * Nt; idx += kThreads) {
    const int t = idx % Nt, r = idx / Nt;
    if (g * Q + (r % Q) >= Pz) continue;
    const int z = Pz * (r / Q) + g * Q + (r % Q);
    const long long off = (xy * Nz + z) * Nt + t;
    zt_epilogue_point<CO, EXACT>(ep, Co, WS, Y, Rz, sY, r, t, b, off, Npts, out);
  }
}

// ------------------------------------------------------------------------------------------
// The same stage for t-lengths 16 and 32, with the two dense contractions on the matrix cores.
// Per grid point the pre-activation is one inner product of length Cu + 2 mt:
//     z[o] = b[o] + sum_i W[o][i] u[i]  +  sum_kt ( Re V[o][kt] cos(th) - Im V[o][kt] sin(th) )
// i.e. the channel-linear term of eq. (2) and the complex-to-real step over t share the
// accumulator.  v_mfma_f32_4x4x1 (16 independent 4x4 outer products per wave, full fp32) fits
// it without padding.  An MFMA block is 4 consecutive t of one z-row ("quad") times 4
// channels: lane 4b+i supplies the A value at t = 4 quad + i (u of the current input channel,
// or the twiddle), lane 4b+j supplies the B value of channel 4T+j (W[4T+j][i] or V[4T+j][row][kt]),
// and lane 4b+j receives, in its four result registers, channel 4T+j at the quad's four t:
// one float4 of the output.  A lane serves two quads (slots).
// Blocks that share a (b,nx,ny) column are placed on one XCD so the column's spectrum tile
// is fetched into that XCD's L2 once.
// ------------------------------------------------------------------------------------------



// Tables of the matrix-core inverse kernel, one blob per residue group g in the kernel's LDS
// layout: cos / -sin rows [2 mt][NT], W transposed and padded [Cu][CP], z twiddles [Q][Lz],
// bias padded [CP].
__global__ void zt_tables_kernel(float* __restrict__ blob, const float2* __restrict__ twt,
                                 const float2* __restrict__ twz, const float* __restrict__ W, int w_so,
                                 int w_si, const float* __restrict__ bias, int Co, int Cu, int CP, int mt,
                                 int NT, int nt_act, int Lz, int Pz, int Q, int blob_floats) {
  const int g = blockIdx.x;
  float* dst = blob + (long long)g * blob_floats;
  const int n_cs = 2 * mt * NT, n_wt = (W != nullptr) ? Cu * CP : 0, n_tw = 2 * Q * Lz;
  for (int idx = threadIdx.x; idx < blob_floats; idx += blockDim.x) {
    float v = 0.f;
    if (idx < n_cs) {
      // rows padded from the axis length nt_act to the tile width NT with zeros
      const int k = idx / NT, t = idx - k * NT;
      const float2 w = t < nt_act ? twt[(k >> 1) * nt_act + t] : make_float2(0.f, 0.f);
      v = (k & 1) ? w.y : w.x;
    } else if (idx < n_cs + n_wt) {
      const int e = idx - n_cs;
      const int i = e / CP, o = e - i * CP;
      v = o < Co ? W[o * w_so + i * w_si] : 0.f;
    } else if (idx < n_cs + n_wt + n_tw) {
      const int e = idx - n_cs - n_wt;
      const int c = e >> 1, q = c / Lz, j = c - q * Lz;
      const float2 w = twz[j * Pz + g * Q + q];
      v = (e & 1) ? w.y : w.x;
    } else if (idx < n_cs + n_wt + n_tw + CP) {
      const int o = idx - n_cs - n_wt - n_tw;
      v = (bias != nullptr && o < Co) ? bias[o] : 0.f;
    }
    dst[idx] = v;
  }
}

// Launch: grid (8 * G * ceil(NxNy / 8), B), 64 NW threads (a tile of NW * 128 / NT rows).  Q and G are powers of two (shifts
// instead of divisions); inv_mt = ceil(2^16 / mt) turns the division by mt into a multiply.
// FULL means Co == 4 CT and (no linear term or Cu == 4 CT): channel guards vanish at compile time.
// Four consecutive t of one channel: one 16-byte store, or, for a row length that is only even,
// the pairs of the quad that exist.
template <bool TPAD>
__device__ __forceinline__ void store_quad(float* dst, int valid, float4 v) {
  if constexpr (!TPAD) {
    *reinterpret_cast<float4*>(dst) = v;
  } else {
    if (valid >= 2) *reinterpret_cast<float2*>(dst) = make_float2(v.x, v.y);
    if (valid >= 4) *reinterpret_cast<float2*>(dst + 2) = make_float2(v.z, v.w);
  }
}

// TPAD: the t axis is shorter than the tile (nt_act < NT, nt_act even): rows of nt_act floats in
// memory, the tile's last quads partly or wholly outside (their u values read as zero, their
// table columns are zero, their results are not stored; stores go as float2 pairs, which the
// even row length keeps 8-byte aligned).
template <int NT, int MZ, int CT, bool FULL, int NW, bool TPAD>
__global__ __launch_bounds__(64 * NW, NW == 8 ? 4 : (CT >= 8 ? 2 : 3)) void zt_inv_mfma_kernel(
    const float2* __restrict__ a, float* __restrict__ out, const float2* __restrict__ twt,
    const float2* __restrict__ twz, int Co_rt, int NxNy, int Nz, int nt_act, int Lz, int nposz, int mt,
    int qshift, int gshift, int inv_mt, int region_floats, int a_stride4, int v_stride, const float* __restrict__ blob, int blob_floats, EpiArgs ep) {
  HIP_DYNAMIC_SHARED(float, smem)
  constexpr int CP = 4 * CT;                 // channels padded to whole MFMA tiles
  constexpr int CI = CP;                     // bound of the input-channel loop
  constexpr int QPR = NT / 4;                // quads per row
  constexpr int RPW = 32 / QPR;              // rows per wave: 16 MFMA blocks x 2 slots = 32 quads
  constexpr int Rz = NW * RPW;               // rows per tile (NW waves)
  const int Co = FULL ? CP : Co_rt;
  const int Cu = FULL ? CI : ep.Cu;
  const int Q = 1 << qshift;
  const int Pz = Nz / MZ;
  constexpr int nthr = 64 * NW;
  // LDS: the column's spectrum tile A [Co][Lz][mt] (complex), staged by LDS-direct loads; once
  // every z-stage item has read it, the same memory holds V [CP][Rz][mt].  Both with padded
  // channel strides.  Then the tables.
  float2* A = reinterpret_cast<float2*>(smem);
  float2* V = reinterpret_cast<float2*>(smem);
  float* CS = smem + region_floats;                     // [2 mt][NT]: cos rows and -sin rows
  float* Wt = CS + 2 * mt * NT;                         // [Cu][CP]
  const bool lin = ep.u != nullptr;
  float2* TWQ = reinterpret_cast<float2*>(Wt + (lin ? Cu * CP : 0));   // [Q][Lz]
  const int tid = threadIdx.x;
  const int xcd = blockIdx.x & 7;
  const int slot_id = blockIdx.x >> 3;
  const int xy = ((slot_id >> gshift) << 3) + xcd;
  const int g = slot_id & ((1 << gshift) - 1);
  if (xy >= NxNy) return;
  const long long b = blockIdx.y;
  const int lane = tid & 63, wave = tid >> 6;
  const int j4 = lane & 3;                    // t within the quad (A side) / channel within the tile (B, D side)
  const int blk = lane >> 2;
  const int quad = blk % QPR;                 // same for both slots because 16 % QPR == 0
  int rowt[2];                                // tile row of each slot
  long long poff[2];                          // offset of the quad's first point inside a channel slab
#pragma unroll
  for (int sl = 0; sl < 2; ++sl) {
    rowt[sl] = wave * RPW + (sl * 16 + blk) / QPR;
    const int z = Pz * (rowt[sl] >> qshift) + (g << qshift) + (rowt[sl] & (Q - 1));
    poff[sl] = ((long long)xy * Nz + z) * (TPAD ? nt_act : NT) + 4 * quad;
  }
  const long long Npts = (long long)NxNy * Nz * (TPAD ? nt_act : NT);
  const bool t_in = !TPAD || 4 * quad + j4 < nt_act;        // this lane's t of the quad exists
  const int quad_valid = TPAD ? nt_act - 4 * quad : 4;       // points of the quad that exist (<= 0, 2 or >= 4)
  const int kmin = nposz - Lz, kmax = nposz - 1;
  const int mbase = posmod(-kmin, MZ);
  const int nitems = (Co * mt) << qshift;

  // tables: one contiguous blob per residue group, prepared by zt_tables_kernel in the LDS layout
  {
    const float* bsrc = blob + (long long)g * blob_floats;
    for (int c0 = wave * 256; c0 < blob_floats; c0 += 256 * NW)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(bsrc + c0 + 4 * lane),
                                       (__attribute__((address_space(3))) void*)(CS + c0), 16, 0, 0);
  }
  asm volatile("" ::: "memory");    // keep the issue order: tables, tile, u (the wait below counts on it)
  // the spectrum tile goes straight to LDS, 16 bytes per lane, channel by channel: the channel
  // stride in LDS (a_stride4 float4) is padded so that the z-stage reads, whose lanes differ in
  // (channel, kt), spread over the banks
  {
    const int per_ch4 = (Lz * mt) >> 1;                  // float4 pieces per channel
    const float2* abase = a + ((b * Co) * NxNy + xy) * (long long)(Lz * mt);
    const long long astride = (long long)NxNy * Lz * mt; // float2 between channels
    for (int o = wave; o < Co; o += NW) {
      for (int c0 = 0; c0 < per_ch4; c0 += 64) {
        const int f = c0 + lane;
        if (f < per_ch4)
          __builtin_amdgcn_global_load_lds(
              (const __attribute__((address_space(1))) void*)(abase + o * astride + 2 * f),
              (__attribute__((address_space(3))) void*)(smem + 4 * (o * a_stride4 + c0)), 16, 0, 0);
      }
    }
  }
  asm volatile("" ::: "memory");
  // u loads last so they stay in flight during the z stage: lane 4b+i takes t = 4 quad + i
  float xv[CI][2];
  if (lin) {
    const float* up = ep.u + (b * Cu) * Npts + j4;
#pragma unroll
    for (int i = 0; i < CI; ++i) {
      if (FULL || i < Cu) {
        xv[i][0] = t_in ? up[i * Npts + poff[0]] : 0.f;
        xv[i][1] = t_in ? up[i * Npts + poff[1]] : 0.f;
      }
    }
  }
  asm volatile("" ::: "memory");
  // wait for the table blob and the tile, not for the u loads (they were issued after them;
  // the counter retires in order).  vmcnt sits in bits 3:0 and 15:14 of the immediate.
  if constexpr (FULL && 2 * CI < 64) {
    constexpr int n = 2 * CI;
    if (lin) __builtin_amdgcn_s_waitcnt(((n >> 4) << 14) | 0x0F70 | (n & 15));
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  } else {
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  __syncthreads();

  // z stage: item (o, kt, q) collects the kept z-frequencies of one (channel, kt) column with
  // their twiddles into MZ bins; an inverse FFT over n1 gives the rows z = Pz n1 + n2.  At most
  // kZItems items per thread; their results wait in registers until every item has read A.
  constexpr int kZItems = NW == 8 ? 1 : 2;      // z-stage items per thread (checked on the host)
  float2 gres[kZItems][MZ];
#pragma unroll
  for (int it = 0; it < kZItems; ++it) {
    const int item = tid + it * nthr;
    if (item < nitems) {
      const int q = item & (Q - 1);
      const int r = item >> qshift;
      const int o = (r * inv_mt) >> 16;
      const int kt = r - o * mt;
      const float2* asrc = A + o * (2 * a_stride4) + kt;
      const float2* twq = TWQ + q * Lz;
#pragma unroll
      for (int m = 0; m < MZ; ++m) {
        float2 accb = make_float2(0.f, 0.f);
        for (int k = kmin + ((m + mbase) & (MZ - 1)); k <= kmax; k += MZ) {
          const int j = k >= 0 ? k : k + Lz;
          accb = cfmac(asrc[j * mt], twq[j], accb);
        }
        gres[it][m] = accb;
      }
      fft_reg<MZ, +1>(gres[it]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kZItems; ++it) {
    const int item = tid + it * nthr;
    if (item < nitems) {
      const int q = item & (Q - 1);
      const int r = item >> qshift;
      const int o = (r * inv_mt) >> 16;
      const int kt = r - o * mt;
      float2* vdst = V + o * v_stride + q * mt + kt;
      const int vstep = mt << qshift;
#pragma unroll
      for (int n1 = 0; n1 < MZ; ++n1) vdst[n1 * vstep] = gres[it][bitrev<MZ>(n1)];
    }
  }
  if (!FULL) {
    // channels of the padding tiles: finite values so the unused MFMA columns stay harmless
    for (int idx = tid; idx < (CP - Co) * v_stride; idx += nthr) V[Co * v_stride + idx] = make_float2(0.f, 0.f);
  }
  __syncthreads();

  v4f acc[CT][2];
#pragma unroll
  for (int T = 0; T < CT; ++T) {
    const float bv = (ep.bias != nullptr && (FULL || 4 * T + j4 < Co)) ? ep.bias[4 * T + j4] : 0.f;
    const v4f init = {bv, bv, bv, bv};
    acc[T][0] = init;
    acc[T][1] = init;
  }
  if (lin) {
    constexpr int IB = 4;                       // input channels per batch of LDS reads
#pragma unroll
    for (int i0 = 0; i0 < CI; i0 += IB) {
      float wv[IB][CT];
#pragma unroll
      for (int ii = 0; ii < IB; ++ii)
#pragma unroll
        for (int T = 0; T < CT; ++T)
          wv[ii][T] = (FULL || i0 + ii < Cu) ? Wt[(i0 + ii) * CP + 4 * T + j4] : 0.f;
#pragma unroll
      for (int ii = 0; ii < IB; ++ii) {
        if (FULL || i0 + ii < Cu) {
#pragma unroll
          for (int T = 0; T < CT; ++T) {
            acc[T][0] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv[i0 + ii][0], wv[ii][T], acc[T][0], 0, 0, 0);
            acc[T][1] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv[i0 + ii][1], wv[ii][T], acc[T][1], 0, 0, 0);
          }
        }
      }
    }
  }
  const float* cs_lane = CS + 4 * quad + j4;
  const float2* v0 = V + j4 * v_stride + rowt[0] * mt;     // channel stride padded against bank conflicts
  const float2* v1 = V + j4 * v_stride + rowt[1] * mt;
  for (int kt = 0; kt < mt; ++kt) {
    const float c = cs_lane[(2 * kt) * NT];
    const float sn = cs_lane[(2 * kt + 1) * NT];
    float2 va[CT], vb[CT];
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      va[T] = v0[4 * T * v_stride + kt];
      vb[T] = v1[4 * T * v_stride + kt];
    }
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      acc[T][0] = __builtin_amdgcn_mfma_f32_4x4x1f32(c, va[T].x, acc[T][0], 0, 0, 0);
      acc[T][1] = __builtin_amdgcn_mfma_f32_4x4x1f32(c, vb[T].x, acc[T][1], 0, 0, 0);
      acc[T][0] = __builtin_amdgcn_mfma_f32_4x4x1f32(sn, va[T].y, acc[T][0], 0, 0, 0);
      acc[T][1] = __builtin_amdgcn_mfma_f32_4x4x1f32(sn, vb[T].y, acc[T][1], 0, 0, 0);
    }
  }
  // lane 4b+j now holds channel 4T+j at the four t of each of its two quads
  float* op = out + (b * Co + j4) * Npts;
  if (ep.zsave != nullptr) {
    float* zp = ep.zsave + (b * Co + j4) * Npts;
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      if (FULL || 4 * T + j4 < Co) {
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
          store_quad<TPAD>(zp + (4 * T) * Npts + poff[sl], quad_valid,
                           make_float4(acc[T][sl][0], acc[T][sl][1], acc[T][sl][2], acc[T][sl][3]));
      }
    }
  }
  if (ep.act) {
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      if (FULL || 4 * T + j4 < Co) {
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
          store_quad<TPAD>(op + (4 * T) * Npts + poff[sl], quad_valid,
                           make_float4(gelu_fast_f(acc[T][sl][0]), gelu_fast_f(acc[T][sl][1]),
                                       gelu_fast_f(acc[T][sl][2]), gelu_fast_f(acc[T][sl][3])));
      }
    }
  } else {
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      if (FULL || 4 * T + j4 < Co) {
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
          store_quad<TPAD>(op + (4 * T) * Npts + poff[sl], quad_valid,
                           make_float4(acc[T][sl][0], acc[T][sl][1], acc[T][sl][2], acc[T][sl][3]));
      }
    }
  }
}

// Column variant of the matrix-core inverse kernel for NT = 32, MZ = 16: one block of eight waves
// owns a whole (b,nx,ny) column, stages the column's spectrum once and walks the residue classes
// of z two at a time (a tile of 32 rows x 32 t per step, Pz / 2 steps).  The spectrum A stays in
// LDS for all steps; V holds one residue class (16 rows) at a time, so a step is two half steps
// (z stage, t stage, W part, epilogue), one per slot of u registers.  Slot s of lane block (wave, blk) is the quad
// blk % 8 of row z = Pz (2 wave + blk / 8) + 2 step + s.  Launch: grid (NxNy, B), 512 threads.
// The table blob is the one of zt_tables_kernel with Q = Pz (all twiddles, [Pz][Lz]).
template <int CT, bool FULL>
__global__ __launch_bounds__(512, 4) void zt_inv_col_kernel(
    const float2* __restrict__ a, float* __restrict__ out, int Co_rt, int NxNy, int Nz, int Lz,
    int nposz, int mt, int inv_mt, int a_floats, int a_stride4, int v_stride,
    const float* __restrict__ blob, int blob_floats, EpiArgs ep) {
  HIP_DYNAMIC_SHARED(float, smem)
  constexpr int NT = 32, MZ = 16, NW = 8;
  constexpr int CP = 4 * CT;
  constexpr int CI = CP;
  constexpr int nthr = 64 * NW;
  const int Co = FULL ? CP : Co_rt;
  const int Cu = FULL ? CI : ep.Cu;
  const int Pz = Nz / MZ;
  const float2* A = reinterpret_cast<const float2*>(smem);      // [Co][Lz][mt], padded channel stride
  float2* V = reinterpret_cast<float2*>(smem + a_floats);       // [CP][MZ][mt], padded channel stride
  float* CS = smem + a_floats + 2 * CP * v_stride;              // [2 mt][NT]: cos rows and -sin rows
  float* Wt = CS + 2 * mt * NT;                                 // [Cu][CP]
  const bool lin = ep.u != nullptr;
  const float2* TW = reinterpret_cast<const float2*>(Wt + (lin ? Cu * CP : 0));   // [Pz][Lz]
  const int tid = threadIdx.x;
  const int xy = blockIdx.x;
  const long long b = blockIdx.y;
  const int lane = tid & 63, wave = tid >> 6;
  const int j4 = lane & 3;                    // t within the quad (A side) / channel within the tile (B, D side)
  const int blk = lane >> 2;
  const int quad = blk & 7;
  const int n1 = 2 * wave + (blk >> 3);       // row of this lane block inside a residue class
  const long long Npts = (long long)NxNy * Nz * NT;
  const long long pbase = ((long long)xy * Nz + Pz * n1) * NT + 4 * quad;   // + (2 step + slot) * NT
  const int kmin = nposz - Lz, kmax = nposz - 1;
  const int mbase = posmod(-kmin, MZ);
  const int nitems = Co * mt;                 // z-stage items of one residue class: (channel, kt)

  for (int c0 = wave * 256; c0 < blob_floats; c0 += 256 * NW)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(blob + c0 + 4 * lane),
                                     (__attribute__((address_space(3))) void*)(CS + c0), 16, 0, 0);
  {
    const int per_ch4 = (Lz * mt) >> 1;                  // float4 pieces per channel
    const float2* abase = a + ((b * Co) * NxNy + xy) * (long long)(Lz * mt);
    const long long astride = (long long)NxNy * Lz * mt; // float2 between channels
    for (int o = wave; o < Co; o += NW) {
      for (int c0 = 0; c0 < per_ch4; c0 += 64) {
        const int f = c0 + lane;
        if (f < per_ch4)
          __builtin_amdgcn_global_load_lds(
              (const __attribute__((address_space(1))) void*)(abase + o * astride + 2 * f),
              (__attribute__((address_space(3))) void*)(smem + 4 * (o * a_stride4 + c0)), 16, 0, 0);
      }
    }
  }
  // this thread's z-stage item
  const int zo = (tid * inv_mt) >> 16;
  const int zkt = tid - zo * mt;
  const float2* asrc = A + zo * (2 * a_stride4) + zkt;
  float2* vdst = V + zo * v_stride + zkt;
  if (!FULL) {
    // channels of the padding tiles: finite values so the unused MFMA columns stay harmless
    for (int idx = tid; idx < (CP - Co) * v_stride; idx += nthr) V[Co * v_stride + idx] = make_float2(0.f, 0.f);
  }
  const float* BI = reinterpret_cast<const float*>(TW + Pz * Lz);      // bias, padded to CP
  // u values of the two slots (lane 4b+i takes t = 4 quad + i): loaded one step ahead, each
  // slot's registers refilled as soon as its W part has used them
  float xv[CI][2];
  const float* ubase = lin ? ep.u + (b * Cu) * Npts + j4 + pbase : nullptr;
  asm volatile("" ::: "memory");    // keep the issue order: tables, spectrum, u
  if (lin) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int i = 0; i < CI; ++i)
        if (FULL || i < Cu) xv[i][sl] = ubase[i * Npts + sl * NT];
  }
  asm volatile("" ::: "memory");
  // tables and spectrum have landed once at most the u loads, issued after them, are
  // outstanding (the counter retires in order; vmcnt sits in bits 3:0 and 15:14)
  if constexpr (FULL && 2 * CI < 64) {
    constexpr int n = 2 * CI;
    if (lin) __builtin_amdgcn_s_waitcnt(((n >> 4) << 14) | 0x0F70 | (n & 15));
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  } else {
    __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  __syncthreads();

  const int nsteps = Pz >> 1;
  for (int step = 0; step < nsteps; ++step) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
      const int n2 = 2 * step + sl;                       // residue class of this half step
      const long long poff = pbase + (long long)n2 * NT;  // this lane block's quad in a channel
      // z stage: item (o, kt) collects the kept z-frequencies with their twiddles into MZ bins;
      // an inverse FFT over n1 gives the rows z = Pz n1 + n2
      if (tid < nitems) {
        // The kept frequency k_j goes to bin k_j mod MZ.  When Lz is a multiple of MZ that is
        // j mod MZ for the stored order j as well (k_j = j or j - Lz), every bin gets Lz / MZ
        // terms, and a round of MZ consecutive j needs no index arithmetic: its reads go out
        // together.  Other Lz take one term at a time.
        const float2* twq = TW + n2 * Lz;
        float2 gres[MZ];
#pragma unroll
        for (int m = 0; m < MZ; ++m) gres[m] = make_float2(0.f, 0.f);
        if ((Lz & (MZ - 1)) == 0) {
          for (int r0 = 0; r0 < Lz; r0 += MZ) {
            const float2* ar = asrc + r0 * mt;
            const float2* tr = twq + r0;
#pragma unroll
            for (int mb = 0; mb < MZ; mb += 8) {
              float2 av[8], wv8[8];
#pragma unroll
              for (int u = 0; u < 8; ++u) {
                av[u] = ar[(mb + u) * mt];
                wv8[u] = tr[mb + u];
              }
#pragma unroll
              for (int u = 0; u < 8; ++u) gres[mb + u] = cfmac(av[u], wv8[u], gres[mb + u]);
            }
          }
        } else {
#pragma unroll
          for (int m = 0; m < MZ; ++m) {
            for (int k = kmin + ((m + mbase) & (MZ - 1)); k <= kmax; k += MZ) {
              const int j = k >= 0 ? k : k + Lz;
              gres[m] = cfmac(asrc[j * mt], twq[j], gres[m]);
            }
          }
        }
        fft_reg<MZ, +1>(gres);
#pragma unroll
        for (int r = 0; r < MZ; ++r) vdst[r * mt] = gres[bitrev<MZ>(r)];
      }
      __syncthreads();
      // t stage: complex-to-real step over kt on the matrix cores
      v4f acc[CT];
#pragma unroll
      for (int T = 0; T < CT; ++T) {
        const float bv = BI[4 * T + j4];
        acc[T] = v4f{bv, bv, bv, bv};
      }
      const float* cs_lane = CS + 4 * quad + j4;
      const float2* v0 = V + j4 * v_stride + n1 * mt;
      int kt = 0;
      constexpr int KB = 3;                       // kt per pass: their reads go out together
      for (; kt + KB <= mt; kt += KB) {
        float cs4[2 * KB];
        float2 va[KB][CT];
#pragma unroll
        for (int h = 0; h < KB; ++h) {
          cs4[2 * h] = cs_lane[(2 * (kt + h)) * NT];
          cs4[2 * h + 1] = cs_lane[(2 * (kt + h) + 1) * NT];
#pragma unroll
          for (int T = 0; T < CT; ++T) va[h][T] = v0[4 * T * v_stride + kt + h];
        }
#pragma unroll
        for (int h = 0; h < KB; ++h)
#pragma unroll
          for (int T = 0; T < CT; ++T) {
            acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(cs4[2 * h], va[h][T].x, acc[T], 0, 0, 0);
            acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(cs4[2 * h + 1], va[h][T].y, acc[T], 0, 0, 0);
          }
      }
      for (; kt < mt; ++kt) {
        const float c = cs_lane[(2 * kt) * NT];
        const float sn = cs_lane[(2 * kt + 1) * NT];
        float2 va[CT];
#pragma unroll
        for (int T = 0; T < CT; ++T) va[T] = v0[4 * T * v_stride + kt];
#pragma unroll
        for (int T = 0; T < CT; ++T) {
          acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(c, va[T].x, acc[T], 0, 0, 0);
          acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(sn, va[T].y, acc[T], 0, 0, 0);
        }
      }
      __syncthreads();      // V is rewritten by the next z stage
      if (lin) {
        constexpr int IB = 4;                       // input channels per batch of LDS reads
#pragma unroll
        for (int i0 = 0; i0 < CI; i0 += IB) {
          float wv[IB][CT];
#pragma unroll
          for (int ii = 0; ii < IB; ++ii)
#pragma unroll
            for (int T = 0; T < CT; ++T)
              wv[ii][T] = (FULL || i0 + ii < Cu) ? Wt[(i0 + ii) * CP + 4 * T + j4] : 0.f;
#pragma unroll
          for (int ii = 0; ii < IB; ++ii) {
            if (FULL || i0 + ii < Cu) {
#pragma unroll
              for (int T = 0; T < CT; ++T)
                acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv[i0 + ii][sl], wv[ii][T], acc[T], 0, 0, 0);
            }
          }
        }
        // this slot's u values of the next step
        asm volatile("" ::: "memory");
        if (step + 1 < nsteps) {
#pragma unroll
          for (int i = 0; i < CI; ++i)
            if (FULL || i < Cu) xv[i][sl] = ubase[i * Npts + (n2 + 2) * NT];
        }
        asm volatile("" ::: "memory");
      }
      // lane 4b+j now holds channel 4T+j at the four t of its quad
      float* op = out + (b * Co + j4) * Npts + poff;
      if (ep.zsave != nullptr) {
        float* zp = ep.zsave + (b * Co + j4) * Npts + poff;
#pragma unroll
        for (int T = 0; T < CT; ++T)
          if (FULL || 4 * T + j4 < Co)
            *reinterpret_cast<float4*>(zp + (4 * T) * Npts) = make_float4(acc[T][0], acc[T][1], acc[T][2], acc[T][3]);
      }
      if (ep.act) {
#pragma unroll
        for (int T = 0; T < CT; ++T)
          if (FULL || 4 * T + j4 < Co)
            *reinterpret_cast<float4*>(op + (4 * T) * Npts) =
                make_float4(gelu_fast_f(acc[T][0]), gelu_fast_f(acc[T][1]), gelu_fast_f(acc[T][2]),
                            gelu_fast_f(acc[T][3]));
      } else {
#pragma unroll
        for (int T = 0; T < CT; ++T)
          if (FULL || 4 * T + j4 < Co)
            *reinterpret_cast<float4*>(op + (4 * T) * Npts) = make_float4(acc[T][0], acc[T][1], acc[T][2], acc[T][3]);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Backward pointwise: gz = g * act'(z); partial sums for gb and gW
// ------------------------------------------------------------------------------------------
constexpr int kBwdTile = 256;      // points per tile (= threads)
constexpr int kBwdPairs = 5;       // sums per thread: covers Cout*(Cin+1) up to 1280

__global__ __launch_bounds__(kThreads) void bwd_pointwise_kernel(
    const float* __restrict__ z, const float* __restrict__ gout, const float* __restrict__ x,
    float* __restrict__ gz_out, double* __restrict__ part, int B, int Ci, int Co, long long N,
    int act, int mse_target, float mse_scale) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int sR = kBwdTile + 1;
  float* Gs = smem;                 // [Co][sR]
  float* Xs = smem + Co * sR;       // [Ci][sR]
  const int tid = threadIdx.x;
  const long long tiles_per_b = (N + kBwdTile - 1) / kBwdTile;
  const long long ntiles = tiles_per_b * B;
  const int npairs = Co * Ci + Co;
  // each thread owns up to kBwdPairs of the Co*Ci + Co sums (checked on the host)
  double acc[kBwdPairs];
#pragma unroll
  for (int h = 0; h < kBwdPairs; ++h) acc[h] = 0.0;
  for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const long long b = tile / tiles_per_b;
    const long long p = (tile % tiles_per_b) * kBwdTile + tid;
    const bool live = p < N;
    for (int o0 = 0; o0 < Co; o0 += 8) {          // eight channels per pass: their loads go out together
      float zv[8], g[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool on = live && o0 + u < Co;
        const long long e = (b * Co + o0 + u) * N + p;
        zv[u] = (on && (act || mse_target)) ? z[e] : 0.f;
        g[u] = on ? gout[e] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (o0 + u < Co) {
          float gv = 0.f;
          if (live) {
            float gg = g[u];
            if (mse_target) gg = mse_scale * ((act ? gelu_f(zv[u]) : zv[u]) - gg);
            gv = act ? gg * gelu_prime_f(zv[u]) : gg;
            if (gz_out != nullptr) gz_out[(b * Co + o0 + u) * N + p] = gv;
          }
          Gs[(o0 + u) * sR + tid] = gv;
        }
      }
    }
    for (int i0 = 0; i0 < Ci; i0 += 8) {
      float xv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) xv[u] = (live && i0 + u < Ci) ? x[(b * Ci + i0 + u) * N + p] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (i0 + u < Ci) Xs[(i0 + u) * sR + tid] = xv[u];
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < kBwdPairs; ++h) {
      const int q = tid + h * kThreads;
      if (q < npairs) {
        float s = 0.f;
        if (q < Co * Ci) {
          const float* gr = Gs + (q / Ci) * sR;
          const float* xr = Xs + (q % Ci) * sR;
          float s1 = 0.f;
          for (int t = 0; t < kBwdTile; t += 8) {    // eight terms per pass: their LDS reads go out together
            float gq[8], xq[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) { gq[u] = gr[t + u]; xq[u] = xr[t + u]; }
#pragma unroll
            for (int u = 0; u < 8; u += 2) { s = fmaf(gq[u], xq[u], s); s1 = fmaf(gq[u + 1], xq[u + 1], s1); }
          }
          s += s1;
        } else {
          const float* gr = Gs + (q - Co * Ci) * sR;
          float s1 = 0.f;
          for (int t = 0; t < kBwdTile; t += 8) {
            float gq[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) gq[u] = gr[t + u];
#pragma unroll
            for (int u = 0; u < 8; u += 2) { s += gq[u]; s1 += gq[u + 1]; }
          }
          s += s1;
        }
        acc[h] += double(s);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int h = 0; h < kBwdPairs; ++h)
    if (tid + h * kThreads < npairs) part[(long long)blockIdx.x * npairs + tid + h * kThreads] = acc[h];
}

// Same step for widths that are a multiple of 4 (up to 20) and N a multiple of 64, streaming
// and without LDS: lane (blk, j) of a wave owns channels j, 4+j, ... at the four consecutive
// points 4*blk .. 4*blk+3 of a 64-point step, so every z / g / x access is a float4 and gz is
// computed exactly once per element.  gW[o][i] = sum_p gz[o][p] x[i][p] is a dense contraction
// over points and runs on the matrix cores: v_mfma_f32_4x4x1 block blk adds the outer product
// gz[4To..4To+3][p] x[4Ti..4Ti+3][p] of its point p to its own 4x4 partial tile; the 16 blocks,
// the waves and the thread blocks are summed at the end (per-wave partials in double, fixed order).
__device__ __forceinline__ void gelu_and_grad_f(float z, float& val, float& grad) {
  const float az = fabsf(z);
  const float x = az * 0.70710678118654752440f;
  float p = fmaf(x, 0.0000430638f, 0.0002765672f);
  p = fmaf(x, p, 0.0001520143f);
  p = fmaf(x, p, 0.0092705272f);
  p = fmaf(x, p, 0.0422820123f);
  p = fmaf(x, p, 0.0705230784f);
  p = fmaf(x, p, 1.0f);
  p = p * p; p = p * p; p = p * p; p = p * p;
  const float erfx = 1.0f - __builtin_amdgcn_rcpf(p);              // erf(|z|/sqrt2), A&S 7.1.28
  const float cdf = 0.5f + 0.5f * copysignf(erfx, z);
  const float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
  val = z * cdf;
  grad = fmaf(z, pdf, cdf);
}

template <int CT>
__global__ __launch_bounds__(kThreads) void bwd_pointwise_mfma_kernel(
    const float* __restrict__ z, const float* __restrict__ gout, const float* __restrict__ x,
    float* __restrict__ gz_out, double* __restrict__ part, int B, long long N, int act, int mse_target,
    float mse_scale) {
  constexpr int C = 4 * CT;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int j4 = lane & 3, blk = lane >> 2;
  v4f acc[CT][CT];
#pragma unroll
  for (int a = 0; a < CT; ++a)
#pragma unroll
    for (int c = 0; c < CT; ++c) acc[a][c] = v4f{0.f, 0.f, 0.f, 0.f};
  float gbacc[CT];
#pragma unroll
  for (int a = 0; a < CT; ++a) gbacc[a] = 0.f;

  const long long steps_per_b = N >> 6;
  const long long steps = steps_per_b * B;
  const long long wave_id = (long long)blockIdx.x * (kThreads / 64) + wave;
  const long long nwaves = (long long)gridDim.x * (kThreads / 64);
  for (long long s = wave_id; s < steps; s += nwaves) {
    const long long bb = s / steps_per_b;
    const long long p0 = (s - bb * steps_per_b) * 64 + 4 * blk;
    float4 gzv[CT], xv[CT];
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      const long long e = (bb * C + 4 * T + j4) * N + p0;
      const float4 zv = *reinterpret_cast<const float4*>(z + e);
      float4 g = *reinterpret_cast<const float4*>(gout + e);
      xv[T] = *reinterpret_cast<const float4*>(x + e);
      if (act) {
        float v0, v1, v2, v3, d0, d1, d2, d3;
        gelu_and_grad_f(zv.x, v0, d0); gelu_and_grad_f(zv.y, v1, d1);
        gelu_and_grad_f(zv.z, v2, d2); gelu_and_grad_f(zv.w, v3, d3);
        if (mse_target) g = make_float4(mse_scale * (v0 - g.x), mse_scale * (v1 - g.y),
                                        mse_scale * (v2 - g.z), mse_scale * (v3 - g.w));
        g = make_float4(g.x * d0, g.y * d1, g.z * d2, g.w * d3);
      } else if (mse_target) {
        g = make_float4(mse_scale * (zv.x - g.x), mse_scale * (zv.y - g.y), mse_scale * (zv.z - g.z),
                        mse_scale * (zv.w - g.w));
      }
      *reinterpret_cast<float4*>(gz_out + e) = g;
      gbacc[T] += (g.x + g.y) + (g.z + g.w);
      gzv[T] = g;
    }
#pragma unroll
    for (int a = 0; a < CT; ++a) {
#pragma unroll
      for (int c = 0; c < CT; ++c) {
        acc[a][c] = __builtin_amdgcn_mfma_f32_4x4x1f32(gzv[a].x, xv[c].x, acc[a][c], 0, 0, 0);
        acc[a][c] = __builtin_amdgcn_mfma_f32_4x4x1f32(gzv[a].y, xv[c].y, acc[a][c], 0, 0, 0);
        acc[a][c] = __builtin_amdgcn_mfma_f32_4x4x1f32(gzv[a].z, xv[c].z, acc[a][c], 0, 0, 0);
        acc[a][c] = __builtin_amdgcn_mfma_f32_4x4x1f32(gzv[a].w, xv[c].w, acc[a][c], 0, 0, 0);
      }
    }
  }
  // sum the 16 blocks of the wave (lanes with equal j4), then lanes 0..3 write the wave's partial
  const int npairs = C * C + C;
  double* dst = part + wave_id * npairs;
#pragma unroll
  for (int a = 0; a < CT; ++a) {
#pragma unroll
    for (int c = 0; c < CT; ++c) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float v = acc[a][c][i];
        v += __shfl_xor(v, 4); v += __shfl_xor(v, 8); v += __shfl_xor(v, 16); v += __shfl_xor(v, 32);
        if (blk == 0) dst[(4 * a + i) * C + 4 * c + j4] = double(v);
      }
    }
    float gsum = gbacc[a];
    gsum += __shfl_xor(gsum, 4); gsum += __shfl_xor(gsum, 8); gsum += __shfl_xor(gsum, 16); gsum += __shfl_xor(gsum, 32);
    if (blk == 0) dst[C * C + 4 * a + j4] = double(gsum);
  }
}

// Sum of the partial slots in a fixed order (same bits on every run): 64 pairs per block, the
// slots dealt round-robin to kRedGroups threads per pair, whose sums are added in group order.
constexpr int kRedGroups = 16;
__global__ __launch_bounds__(64 * kRedGroups) void reduce_partials_kernel(
    const double* __restrict__ part, int nblk, int Co, int Ci, float* __restrict__ gW,
    float* __restrict__ gb) {
  __shared__ double sums[kRedGroups][64];
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int q = blockIdx.x * 64 + lane;
  const int npairs = Co * Ci + Co;
  double s = 0.0;
  if (q < npairs) {
    const double* p = part + q;
    int blk = grp;
    for (; blk + 7 * kRedGroups < nblk; blk += 8 * kRedGroups) {
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[(long long)(blk + u * kRedGroups) * npairs];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; blk < nblk; blk += kRedGroups) s += p[(long long)blk * npairs];
  }
  sums[grp][lane] = s;
  __syncthreads();
  if (grp == 0 && q < npairs) {
    double t = 0.0;
#pragma unroll
    for (int g = 0; g < kRedGroups; ++g) t += sums[g][lane];
    if (q < Co * Ci) { if (gW != nullptr) gW[q] = float(t); }
    else if (gb != nullptr) gb[q - Co * Ci] = float(t);
  }
}

// ------------------------------------------------------------------------------------------
// Pointwise lift and projection (Sec. 2.4)
// ------------------------------------------------------------------------------------------
template <int CO>
__global__ __launch_bounds__(kThreads) void pointwise_linear_kernel(
    int Ci, int Co, long long np, const float* __restrict__ x, const float* __restrict__ W,
    const float* __restrict__ bias, float* __restrict__ y) {
  const long long p = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long b = blockIdx.y;
  if (p >= np) return;
  float acc[CO];
#pragma unroll
  for (int o = 0; o < CO; ++o) acc[o] = (bias != nullptr && o < Co) ? bias[o] : 0.f;
  for (int i = 0; i < Ci; ++i) {
    const float xv = x[(b * Ci + i) * np + p];
#pragma unroll
    for (int o = 0; o < CO; ++o)
      if (o < Co) acc[o] = fmaf(W[o * Ci + i], xv, acc[o]);
  }
#pragma unroll
  for (int o = 0; o < CO; ++o)
    if (o < Co) y[(b * Co + o) * np + p] = acc[o];
}

// ------------------------------------------------------------------------------------------
// Adjoints of the lift and of the projection (what a whole-network backward needs around the
// blocks): sums over all points in a fixed order, per-block partials in double
// ------------------------------------------------------------------------------------------
__global__ void transpose_kernel(const float* __restrict__ w, float* __restrict__ wt, int rows, int cols) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < rows * cols) wt[(idx % cols) * rows + idx / cols] = w[idx];
}

// out[q] = sum over blocks of part[blk][q], blocks in order (same bits on every run); the result
// goes to four destinations by ranges of q (any of them may be null)
__global__ __launch_bounds__(kThreads) void reduce_ranges_kernel(
    const double* __restrict__ part, int nblk, int n0, int n1, int n2, int n3, float* __restrict__ d0,
    float* __restrict__ d1, float* __restrict__ d2, float* __restrict__ d3) {
  const int q = blockIdx.x * kThreads + threadIdx.x;
  const int npairs = n0 + n1 + n2 + n3;
  if (q >= npairs) return;
  double s = 0.0;
  for (int b = 0; b < nblk; ++b) s += part[(long long)b * npairs + q];
  if (q < n0) { if (d0 != nullptr) d0[q] = (float)s; }
  else if (q < n0 + n1) { if (d1 != nullptr) d1[q - n0] = (float)s; }
  else if (q < n0 + n1 + n2) { if (d2 != nullptr) d2[q - n0 - n1] = (float)s; }
  else if (d3 != nullptr) d3[q - n0 - n1 - n2] = (float)s;
}

// Adjoint of u = W2 gelu(W1 x + b1) + b2 per point.  One block: tiles of 256 points.  The hidden
// units are taken kMlpChunk at a time: every thread computes, for its point, h, a = gelu(h) and
// gh = (W2^T g) gelu'(h) of the chunk into LDS and adds W1^T gh to its gx; then the threads take
// one (row, row) pair each of the chunk's sums -- gW1[k][i] = sum gh_k x_i, gb1[k] = sum gh_k,
// gW2[o][k] = sum g_o a_k -- as a 256-term inner product in float, added to the block's double
// accumulator of that pair in LDS (one owner per pair: no atomics, fixed order).
constexpr int kMlpChunk = 8;
constexpr int kMlpBlocks = 512;     // blocks (= partial-sum slots) of the projection's backward
template <int CI>
__global__ __launch_bounds__(kThreads) void mlp2_bwd_kernel(
    int B, int Ci, int H, int Co, long long N, const float* __restrict__ x, const float* __restrict__ W1,
    const float* __restrict__ b1, const float* __restrict__ W2, const float* __restrict__ g,
    float* __restrict__ gx, double* __restrict__ part) {
  HIP_DYNAMIC_SHARED(float, smem)
  constexpr int sR = kThreads + 1;
  float* XS = smem;                          // [Ci][sR]
  float* GS = XS + Ci * sR;                  // [Co][sR]
  float* GH = GS + Co * sR;                  // [kMlpChunk][sR]
  float* AA = GH + kMlpChunk * sR;           // [kMlpChunk][sR]
  const int nsum = H * (Ci + 1) + Co * H + Co;       // gW1 | gb1 | gW2 | gb2
  int acc_off = (Ci + Co + 2 * kMlpChunk) * sR;
  acc_off += acc_off & 1;
  double* ACC = reinterpret_cast<double*>(smem + acc_off);   // [nsum]
  const int tid = threadIdx.x;
  for (int q = tid; q < nsum; q += kThreads) ACC[q] = 0.0;
  const long long tiles_per_b = (N + kThreads - 1) / kThreads;
  const long long ntiles = tiles_per_b * B;
  const int per_k = Ci + 1 + Co;             // sums per hidden unit
  for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const long long b = tile / tiles_per_b;
    const long long p = (tile % tiles_per_b) * kThreads + tid;
    const bool live = p < N;
    float xr[CI], gxr[CI], gr[4];
#pragma unroll
    for (int i = 0; i < CI; ++i) {
      xr[i] = (live && i < Ci) ? x[(b * Ci + i) * N + p] : 0.f;
      gxr[i] = 0.f;
      if (i < Ci) XS[i * sR + tid] = xr[i];
    }
#pragma unroll
    for (int o = 0; o < 4; ++o) {
      gr[o] = (live && o < Co) ? g[(b * Co + o) * N + p] : 0.f;
      if (o < Co) GS[o * sR + tid] = gr[o];
    }
    for (int k0 = 0; k0 < H; k0 += kMlpChunk) {
      __syncthreads();                         // the previous chunk's pair sums have read GH, AA
      for (int kk = 0; kk < kMlpChunk; ++kk) {
        const int k = k0 + kk;
        float ghv = 0.f, av = 0.f;
        if (k < H) {
          float h = b1 != nullptr ? b1[k] : 0.f;
#pragma unroll
          for (int i = 0; i < CI; ++i)
            if (i < Ci) h = fmaf(W1[k * Ci + i], xr[i], h);
          float t = 0.f;
#pragma unroll
          for (int o = 0; o < 4; ++o)
            if (o < Co) t = fmaf(W2[o * H + k], gr[o], t);
          av = gelu_f(h);
          ghv = t * gelu_prime_f(h);
#pragma unroll
          for (int i = 0; i < CI; ++i)
            if (i < Ci) gxr[i] = fmaf(W1[k * Ci + i], ghv, gxr[i]);
        }
        GH[kk * sR + tid] = ghv;
        AA[kk * sR + tid] = av;
      }
      __syncthreads();
      for (int q = tid; q < kMlpChunk * per_k; q += kThreads) {
        const int kk = q / per_k, r = q - kk * per_k;
        const int k = k0 + kk;
        if (k >= H) continue;
        const float* u = r <= Ci ? GH + kk * sR : GS + (r - Ci - 1) * sR;
        float sum = 0.f;
        int dst;
        if (r < Ci) {
          const float* w = XS + r * sR;
          for (int t = 0; t < kThreads; ++t) sum = fmaf(u[t], w[t], sum);
          dst = k * Ci + r;
        } else if (r == Ci) {
          for (int t = 0; t < kThreads; ++t) sum += u[t];
          dst = H * Ci + k;
        } else {
          const float* w = AA + kk * sR;
          for (int t = 0; t < kThreads; ++t) sum = fmaf(u[t], w[t], sum);
          dst = H * (Ci + 1) + (r - Ci - 1) * H + k;
        }
        ACC[dst] += (double)sum;
      }
    }
    // gb2[o] = sum g_o
    if (tid < Co) {
      const float* u = GS + tid * sR;
      float sum = 0.f;
      for (int t = 0; t < kThreads; ++t) sum += u[t];
      ACC[H * (Ci + 1) + Co * H + tid] += (double)sum;
    }
    if (gx != nullptr && live) {
#pragma unroll
      for (int i = 0; i < CI; ++i)
        if (i < Ci) gx[(b * Ci + i) * N + p] = gxr[i];
    }
    __syncthreads();                           // XS, GS are rewritten by the next tile
  }
  __syncthreads();
  for (int q = tid; q < nsum; q += kThreads) part[(long long)blockIdx.x * nsum + q] = ACC[q];
}

// ------------------------------------------------------------------------------------------
// The two-layer projection and its adjoint on the matrix cores
// ------------------------------------------------------------------------------------------
// v_mfma_f32_32x32x2 adds A (32x2) times B (2x32) to a 32x32 accumulator in full fp32.  Lane l
// supplies A[l%32][l/32] and B[l/32][l%32]; register v of its accumulator holds the element in
// row mfma_row(v, l/32), column l%32.
//
// A block of H/32 waves walks over tiles of 64 points (two column blocks of 32); wave w owns the
// hidden units 32w .. 32w+31 and keeps their weights in registers, already in operand order.
//   h   = [W1 | b1] [x ; 1]      K runs over the input channels and a row of ones
//   gx  = W1^T gh                K runs over the wave's hidden units in accumulator order, so
//                                the registers that hold gh are the B operand as they stand
//   gW1 | gb1 = gh [x ; 1]^T     K runs over the points; gh goes through LDS to turn it
// The activation, its slope and the products with W2 are the vector units' share.
typedef float v16f __attribute__((ext_vector_type(16)));
__device__ __forceinline__ int mfma_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

constexpr int kMlpTile = 64;             // points per pass of a block
constexpr int kMlpStage = 6;             // values a thread stages per pass
constexpr int kMlpXS = kMlpTile + 1;     // row stride of the staged tile (odd: column reads spread over the banks)
constexpr int kMlpTS = 33;               // row stride of a wave's 32x32 turn buffer
constexpr int kMlpFlush = 16;            // passes between flushes of the fp32 weight-gradient accumulator

template <int KS, int CO>
__global__ __launch_bounds__(512) void mlp2_fwd_mfma_kernel(
    int B, int Ci, int H, int Co, long long N, const float* __restrict__ x, const float* __restrict__ W1,
    const float* __restrict__ b1, const float* __restrict__ W2, const float* __restrict__ b2,
    float* __restrict__ y) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int nthreads = blockDim.x, nw = nthreads >> 6;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, half = lane >> 5, c = lane & 31;
  float* XS = smem;                          // [32][kMlpXS]: rows < Ci the tile, row Ci ones, the rest zero
  float* YP = XS + 32 * kMlpXS;              // [nw][CO][kMlpTile] partial outputs of the waves
  for (int e = tid; e < (32 - Ci) * kMlpXS; e += nthreads) XS[Ci * kMlpXS + e] = e < kMlpXS ? 1.f : 0.f;
  float A1[KS], W2r[CO][16];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    const int i = 2 * s + half, k = w * 32 + c;
    A1[s] = i < Ci ? W1[k * Ci + i] : ((i == Ci && b1 != nullptr) ? b1[k] : 0.f);
  }
#pragma unroll
  for (int o = 0; o < CO; ++o)
#pragma unroll
    for (int v = 0; v < 16; ++v) W2r[o][v] = o < Co ? W2[o * H + w * 32 + mfma_row(v, half)] : 0.f;
  const long long tiles_per_b = (N + kMlpTile - 1) / kMlpTile;
  const long long ntiles = tiles_per_b * B;
  const int nstage = Ci * kMlpTile;
  float pf[kMlpStage];
  {
    const long long t = blockIdx.x;
    const long long b = t / tiles_per_b, p0 = (t - b * tiles_per_b) * kMlpTile;
#pragma unroll
    for (int r = 0; r < kMlpStage; ++r) {
      const int e = tid + r * nthreads, row = e >> 6, col = e & 63;
      pf[r] = (t < ntiles && e < nstage && p0 + col < N) ? x[(b * Ci + row) * N + p0 + col] : 0.f;
    }
  }
  for (long long t = blockIdx.x; t < ntiles; t += gridDim.x) {
#pragma unroll
    for (int r = 0; r < kMlpStage; ++r) {
      const int e = tid + r * nthreads, row = e >> 6, col = e & 63;
      if (e < nstage) XS[row * kMlpXS + col] = pf[r];
    }
    __syncthreads();
    {
      const long long tn = t + gridDim.x;
      const long long b = tn / tiles_per_b, p0 = (tn - b * tiles_per_b) * kMlpTile;
#pragma unroll
      for (int r = 0; r < kMlpStage; ++r) {
        const int e = tid + r * nthreads, row = e >> 6, col = e & 63;
        pf[r] = (tn < ntiles && e < nstage && p0 + col < N) ? x[(b * Ci + row) * N + p0 + col] : 0.f;
      }
    }
    const long long b = t / tiles_per_b, p0 = (t - b * tiles_per_b) * kMlpTile;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int pc = nb * 32 + c;
      v16f hacc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s)
        hacc = __builtin_amdgcn_mfma_f32_32x32x2f32(A1[s], XS[(2 * s + half) * kMlpXS + pc], hacc, 0, 0, 0);
      float yp[CO];
#pragma unroll
      for (int o = 0; o < CO; ++o) yp[o] = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float a = gelu_fast_f(hacc[v]);
#pragma unroll
        for (int o = 0; o < CO; ++o) yp[o] = fmaf(W2r[o][v], a, yp[o]);
      }
#pragma unroll
      for (int o = 0; o < CO; ++o) {
        yp[o] += __shfl_xor(yp[o], 32);
        if (half == 0) YP[(w * CO + o) * kMlpTile + pc] = yp[o];
      }
    }
    __syncthreads();
    for (int e = tid; e < Co * kMlpTile; e += nthreads) {
      const int o = e >> 6, col = e & 63;
      float sum = b2 != nullptr ? b2[o] : 0.f;
      for (int ww = 0; ww < nw; ++ww) sum += YP[(ww * CO + o) * kMlpTile + col];
      if (p0 + col < N) y[(b * Co + o) * N + p0 + col] = sum;
    }
  }
}

template <int KS, int CO>
__global__ __launch_bounds__(512) void mlp2_bwd_mfma_kernel(
    int B, int Ci, int H, int Co, long long N, const float* __restrict__ x, const float* __restrict__ W1,
    const float* __restrict__ b1, const float* __restrict__ W2, const float* __restrict__ g,
    float* __restrict__ gx, double* __restrict__ part) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int nthreads = blockDim.x, nw = nthreads >> 6;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, half = lane >> 5, c = lane & 31;
  float* XS = smem;                                      // [32][kMlpXS]: tile, ones, zeros as above
  float* GS = XS + 32 * kMlpXS;                          // [CO][kMlpTile] upstream gradient of the tile
  float* T = GS + CO * kMlpTile + w * (32 * kMlpTS);     // this wave's [32][kMlpTS] turn buffer
  float* GXP = GS + CO * kMlpTile + nw * (32 * kMlpTS);  // [nw][Ci][kMlpXS] partial gx of the waves
  float* W2S = GXP + nw * Ci * kMlpXS;                   // [CO][H], only when CO > 1 (else W2 sits in registers)
  int acc_off = 32 * kMlpXS + CO * kMlpTile + nw * (32 * kMlpTS) + nw * Ci * kMlpXS + (CO > 1 ? CO * H : 0);
  acc_off += acc_off & 1;
  double* ACC = reinterpret_cast<double*>(smem + acc_off);   // [nsum] gW1 | gb1 | gW2 | gb2
  const int nsum = H * (Ci + 1) + Co * H + Co;
  for (int q = tid; q < nsum; q += nthreads) ACC[q] = 0.0;
  for (int e = tid; e < (32 - Ci) * kMlpXS; e += nthreads) XS[Ci * kMlpXS + e] = e < kMlpXS ? 1.f : 0.f;
  if constexpr (CO > 1)
    for (int e = tid; e < CO * H; e += nthreads) W2S[e] = e < Co * H ? W2[e] : 0.f;
  float A1[KS], A2[16], W2r[1][16];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    const int i = 2 * s + half, k = w * 32 + c;
    A1[s] = i < Ci ? W1[k * Ci + i] : ((i == Ci && b1 != nullptr) ? b1[k] : 0.f);
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int k = w * 32 + mfma_row(v, half);
    A2[v] = c < Ci ? W1[k * Ci + c] : 0.f;
    if constexpr (CO == 1) W2r[0][v] = W2[k];
  }
  const long long tiles_per_b = (N + kMlpTile - 1) / kMlpTile;
  const long long ntiles = tiles_per_b * B;
  const int nstage = (Ci + Co) * kMlpTile;
  v16f accw = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float acc2[CO][16], accg[CO];
#pragma unroll
  for (int o = 0; o < CO; ++o) {
    accg[o] = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc2[o][v] = 0.f;
  }
  float pf[kMlpStage];
  {
    const long long t = blockIdx.x;
    const long long b = t / tiles_per_b, p0 = (t - b * tiles_per_b) * kMlpTile;
#pragma unroll
    for (int r = 0; r < kMlpStage; ++r) {
      const int e = tid + r * nthreads, row = e >> 6, col = e & 63;
      float val = 0.f;
      if (t < ntiles && e < nstage && p0 + col < N)
        val = row < Ci ? x[(b * Ci + row) * N + p0 + col] : g[(b * Co + (row - Ci)) * N + p0 + col];
      pf[r] = val;
    }
  }
  int pass = 0;
  for (long long t = blockIdx.x; t < ntiles; t += gridDim.x) {
#pragma unroll
    for (int r = 0; r < kMlpStage; ++r) {
      const int e = tid + r * nthreads, row = e >> 6, col = e & 63;
      if (e < nstage) {
        if (row < Ci) XS[row * kMlpXS + col] = pf[r];
        else GS[(row - Ci) * kMlpTile + col] = pf[r];
      }
    }
    __syncthreads();
    {
      const long long tn = t + gridDim.x;
      const long long b = tn / tiles_per_b, p0 = (tn - b * tiles_per_b) * kMlpTile;
#pragma unroll
      for (int r = 0; r < kMlpStage; ++r) {
        const int e = tid + r * nthreads, row = e >> 6, col = e & 63;
        float val = 0.f;
        if (tn < ntiles && e < nstage && p0 + col < N)
          val = row < Ci ? x[(b * Ci + row) * N + p0 + col] : g[(b * Co + (row - Ci)) * N + p0 + col];
        pf[r] = val;
      }
    }
    const long long b = t / tiles_per_b, p0 = (t - b * tiles_per_b) * kMlpTile;
#pragma unroll 1
    for (int nb = 0; nb < 2; ++nb) {
      const int pc = nb * 32 + c;
      v16f hacc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < KS; ++s)
        hacc = __builtin_amdgcn_mfma_f32_32x32x2f32(A1[s], XS[(2 * s + half) * kMlpXS + pc], hacc, 0, 0, 0);
      float gl[CO];
#pragma unroll
      for (int o = 0; o < CO; ++o) {
        gl[o] = o < Co ? GS[o * kMlpTile + pc] : 0.f;
        if (half == 0) accg[o] += gl[o];
      }
      float gh[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float a, d;
        gelu_and_grad_f(hacc[v], a, d);
        float tt = 0.f;
#pragma unroll
        for (int o = 0; o < CO; ++o) {
          const float w2v = CO == 1 ? W2r[0][v] : W2S[o * H + w * 32 + mfma_row(v, half)];
          tt = fmaf(w2v, gl[o], tt);
          acc2[o][v] = fmaf(gl[o], a, acc2[o][v]);
        }
        gh[v] = tt * d;
        T[mfma_row(v, half) * kMlpTS + c] = gh[v];
      }
      v16f gacc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int v = 0; v < 16; ++v) gacc = __builtin_amdgcn_mfma_f32_32x32x2f32(A2[v], gh[v], gacc, 0, 0, 0);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = mfma_row(v, half);
        if (row < Ci) GXP[(w * Ci + row) * kMlpXS + pc] = gacc[v];
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int s = 0; s < 16; ++s)
        accw = __builtin_amdgcn_mfma_f32_32x32x2f32(T[c * kMlpTS + 2 * s + half],
                                                    XS[c * kMlpXS + nb * 32 + 2 * s + half], accw, 0, 0, 0);
      __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    if (gx != nullptr) {
      for (int e = tid; e < Ci * kMlpTile; e += nthreads) {
        const int i = e >> 6, col = e & 63;
        float sum = 0.f;
        for (int ww = 0; ww < nw; ++ww) sum += GXP[(ww * Ci + i) * kMlpXS + col];
        if (p0 + col < N) gx[(b * Ci + i) * N + p0 + col] = sum;
      }
    }
    if (++pass == kMlpFlush) {
      pass = 0;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int k = w * 32 + mfma_row(v, half);
        if (c < Ci) ACC[k * Ci + c] += (double)accw[v];
        else if (c == Ci) ACC[H * Ci + k] += (double)accw[v];
        accw[v] = 0.f;
      }
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int k = w * 32 + mfma_row(v, half);
    if (c < Ci) ACC[k * Ci + c] += (double)accw[v];
    else if (c == Ci) ACC[H * Ci + k] += (double)accw[v];
  }
  // gW2[o][k]: the lanes' sums over their points, added over the 32 lanes of a row through T
#pragma unroll
  for (int o = 0; o < CO; ++o) {
    if (o < Co) {
      __syncthreads();
#pragma unroll
      for (int v = 0; v < 16; ++v) T[mfma_row(v, half) * kMlpTS + c] = acc2[o][v];
      __syncthreads();
      if (half == 0) {
        double sum = 0.0;
        for (int cc = 0; cc < 32; ++cc) sum += (double)T[c * kMlpTS + cc];
        ACC[H * (Ci + 1) + o * H + w * 32 + c] = sum;
      }
      float sg = accg[o];
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) sg += __shfl_xor(sg, m);
      if (tid == 0) ACC[H * (Ci + 1) + Co * H + o] = (double)sg;
    }
  }
  __syncthreads();
  for (int q = tid; q < nsum; q += nthreads) part[(long long)blockIdx.x * nsum + q] = ACC[q];
}

// ------------------------------------------------------------------------------------------
// Training pieces outside the block (Sec. 4): relative L2 misfit and the Adam update
// ------------------------------------------------------------------------------------------
constexpr int kLossBlocks = 1024;      // partial sums of the loss (two doubles each)

// part[blk] = (sum (pred - target)^2, sum target^2) over the block's strided share, in double,
// combined in a fixed order (lane tree, then waves in order): same bits on every run.
__global__ __launch_bounds__(kThreads) void rel_l2_partial_kernel(
    long long n, const float* __restrict__ pred, const float* __restrict__ target, double* __restrict__ part) {
  __shared__ double sd[kThreads / 64], sy[kThreads / 64];
  double d2 = 0.0, y2 = 0.0;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kThreads) {
    const double y = target[i];
    const double d = (double)pred[i] - y;
    d2 += d * d;
    y2 += y * y;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    d2 += __shfl_xor(d2, off);
    y2 += __shfl_xor(y2, off);
  }
  if ((threadIdx.x & 63) == 0) { sd[threadIdx.x >> 6] = d2; sy[threadIdx.x >> 6] = y2; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double a = 0.0, b = 0.0;
    for (int w = 0; w < kThreads / 64; ++w) { a += sd[w]; b += sy[w]; }
    part[2 * blockIdx.x] = a;
    part[2 * blockIdx.x + 1] = b;
  }
}

// loss = sqrt(Sd) / sqrt(Sy); scale = 1 / (sqrt(Sd) sqrt(Sy)) for the gradient (0 when Sd = 0)
__global__ void rel_l2_final_kernel(const double* __restrict__ part, int nblk, float* __restrict__ loss,
                                    double* __restrict__ scale) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double a = 0.0, b = 0.0;
  for (int i = 0; i < nblk; ++i) { a += part[2 * i]; b += part[2 * i + 1]; }
  const double nd = sqrt(a), ny = sqrt(b);
  if (loss != nullptr) *loss = (float)(nd / ny);
  *scale = nd > 0.0 ? 1.0 / (nd * ny) : 0.0;
}

__global__ __launch_bounds__(kThreads) void rel_l2_grad_kernel(
    long long n, const float* __restrict__ pred, const float* __restrict__ target,
    const double* __restrict__ scale, float* __restrict__ grad) {
  const float sc = (float)*scale;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kThreads)
    grad[i] = (pred[i] - target[i]) * sc;
}

// Adam (Kingma & Ba, Algorithm 1), one step in place; c1 = 1 / (1 - beta1^t), c2 = 1 / (1 - beta2^t)
__global__ __launch_bounds__(kThreads) void adam_kernel(
    long long n, float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m,
    float* __restrict__ v, float lr, float beta1, float omb1, float beta2, float omb2, float eps, float c1,
    float c2) {
  // omb = 1 - beta, rounded from double on the host (1 - beta in float would lose five digits)
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kThreads) {
    const float gi = g[i];
    const float mi = fmaf(beta1, m[i], omb1 * gi);
    const float vi = fmaf(beta2, v[i], omb2 * gi * gi);
    m[i] = mi;
    v[i] = vi;
    p[i] -= lr * (mi * c1) / (sqrtf(vi * c2) + eps);
  }
}

// Input lifts of Sec. 2.4 (eqs. (8)-(9)) in one sweep: a_1 = W_t a + b_t along a time axis of
// length one, then nu = W_c a_1 + b_c along the channels, i.e.
//   nu[b][c][p][t] = W_t[t] s_c(p) + b_t[t] r_c + b_c[c],  s_c(p) = sum_j W_c[c][j] a[b][j][p],
//   r_c = sum_j W_c[c][j].
// One thread: one spatial point and four consecutive t; the output (the only large tensor) is
// written once, a is read through the cache by the threads that share a point.
template <int CO>
__global__ __launch_bounds__(kThreads) void time_lift_kernel(
    int Ci, int Co, long long np, int Nt, const float* __restrict__ a, const float* __restrict__ wt,
    const float* __restrict__ bt, const float* __restrict__ wc, const float* __restrict__ bc,
    float* __restrict__ out) {
  const int nt4 = (Nt + 3) >> 2;
  const long long e = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long b = blockIdx.y;
  if (e >= np * nt4) return;
  const long long p = e / nt4;
  const int t0 = 4 * (int)(e - p * nt4);
  float sc[CO], rc[CO];
#pragma unroll
  for (int c = 0; c < CO; ++c) { sc[c] = 0.f; rc[c] = 0.f; }
  for (int j = 0; j < Ci; ++j) {
    const float av = a[(b * Ci + j) * np + p];
#pragma unroll
    for (int c = 0; c < CO; ++c) {
      if (c < Co) {
        const float w = wc[c * Ci + j];
        sc[c] = fmaf(w, av, sc[c]);
        rc[c] += w;
      }
    }
  }
  float w4[4], b4[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    w4[u] = t0 + u < Nt ? wt[t0 + u] : 0.f;
    b4[u] = (bt != nullptr && t0 + u < Nt) ? bt[t0 + u] : 0.f;
  }
  const bool vec = (Nt & 3) == 0;      // rows of whole float4s (the base pointer is checked on the host)
#pragma unroll
  for (int c = 0; c < CO; ++c) {
    if (c < Co) {
      const float bias = bc != nullptr ? bc[c] : 0.f;
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = fmaf(w4[u], sc[c], fmaf(b4[u], rc[c], bias));
      float* dst = out + ((b * Co + c) * np + p) * Nt + t0;
      if (vec) {
        *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (t0 + u < Nt) dst[u] = v[u];
      }
    }
  }
}

// Adjoint of the fused lifts (eqs. (8)-(9)) with respect to their parameters.  With
//   G0[o][t] = sum_{b,s} g[b][o][s][t]   and   G1[i][o][t] = sum_{b,s} g[b][o][s][t] a[b][i][s]
// every gradient is a small contraction:  gbc[o] = sum_t G0,  gWc[o][i] = sum_t (Wt[t] G1 + bt[t] G0),
// gWt[t] = sum_{o,i} Wc[o][i] G1,  gbt[t] = sum_{o,i} Wc[o][i] G0.  The sweep over g (the only large
// tensor) keeps one (o, t) pair per thread, so a wave reads whole 128-byte runs of t and the input
// value a[b][i][s] is the same for all its lanes; a chunk of space positions per block row, fp32
// sums of 64 terms added into doubles, one partial per (chunk, pair) in a fixed order.
constexpr int kLiftChunks = 1024;      // partial-sum slots of the sweep
template <int CI>
__global__ __launch_bounds__(kThreads) void time_lift_bwd_kernel(
    int Ci, int Co, long long S, int Nt, int cpb, const float* __restrict__ a, const float* __restrict__ g,
    double* __restrict__ part) {
  const int pair = blockIdx.x * kThreads + threadIdx.x;
  const int npair = Co * Nt;
  const long long b = blockIdx.y / cpb;
  const int c = blockIdx.y - (int)b * cpb;
  const long long len = (S + cpb - 1) / cpb;
  const long long s0 = c * len, s1 = min(S, s0 + len);
  const bool live = pair < npair;
  const int o = live ? pair / Nt : 0, t = live ? pair - o * Nt : 0;
  const float* gp = g + ((b * Co + o) * S) * Nt + t;
  const float* ap = a + (b * Ci) * S;
  double d0 = 0.0, d1[CI];
#pragma unroll
  for (int i = 0; i < CI; ++i) d1[i] = 0.0;
  for (long long sb = s0; sb < s1; sb += 64) {
    float f0 = 0.f, f1[CI];
#pragma unroll
    for (int i = 0; i < CI; ++i) f1[i] = 0.f;
    const long long se = min(s1, sb + 64);
    long long sp = sb;
    for (; sp + 8 <= se; sp += 8) {              // eight positions per pass: their loads go out together
      float gv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) gv[u] = live ? gp[(sp + u) * Nt] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        f0 += gv[u];
#pragma unroll
        for (int i = 0; i < CI; ++i)
          if (i < Ci) f1[i] = fmaf(gv[u], ap[i * S + sp + u], f1[i]);
      }
    }
    for (; sp < se; ++sp) {
      const float gv = live ? gp[sp * Nt] : 0.f;
      f0 += gv;
#pragma unroll
      for (int i = 0; i < CI; ++i)
        if (i < Ci) f1[i] = fmaf(gv, ap[i * S + sp], f1[i]);
    }
    d0 += (double)f0;
#pragma unroll
    for (int i = 0; i < CI; ++i) d1[i] += (double)f1[i];
  }
  if (live) {
    double* dst = part + ((long long)blockIdx.y * (Ci + 1)) * npair + pair;
    dst[0] = d0;
#pragma unroll
    for (int i = 0; i < CI; ++i)
      if (i < Ci) dst[(long long)(i + 1) * npair] = d1[i];
  }
}

// G[k][pair] = sum over the chunks: 32 entries per block, the chunks dealt to 8 thread groups whose
// sums are added in a fixed order
__global__ __launch_bounds__(kThreads) void time_lift_bwd_reduce_kernel(const double* __restrict__ part, int nchunk,
                                                                        int nent, double* __restrict__ G) {
  __shared__ double P[8][32];
  const int el = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int e = blockIdx.x * 32 + el;
  double sum = 0.0;
  if (e < nent)
    for (int c = grp; c < nchunk; c += 8) sum += part[(long long)c * nent + e];
  P[grp][el] = sum;
  __syncthreads();
  if (grp == 0 && e < nent) {
    double tot = 0.0;
#pragma unroll
    for (int k = 0; k < 8; ++k) tot += P[k][el];
    G[e] = tot;
  }
}

// the four small contractions, one output per thread
__global__ __launch_bounds__(kThreads) void time_lift_bwd_final_kernel(
    int Ci, int Co, int Nt, const double* __restrict__ G, const float* __restrict__ wt,
    const float* __restrict__ bt, const float* __restrict__ wc, float* __restrict__ gwt,
    float* __restrict__ gbt, float* __restrict__ gwc, float* __restrict__ gbc) {
  const int npair = Co * Nt;
  const int nout = 2 * Nt + Co * Ci + Co;
  for (int q = threadIdx.x; q < nout; q += kThreads) {
    double sum = 0.0;
    if (q < 2 * Nt) {                            // gWt[t] (q < Nt) or gbt[t]
      const int t = q < Nt ? q : q - Nt;
      for (int o = 0; o < Co; ++o)
        for (int i = 0; i < Ci; ++i)
          sum += (double)wc[o * Ci + i] * (q < Nt ? G[(long long)(i + 1) * npair + o * Nt + t] : G[o * Nt + t]);
      float* dst = q < Nt ? gwt : gbt;
      if (dst != nullptr) dst[t] = (float)sum;
    } else if (q < 2 * Nt + Co * Ci) {           // gWc[o][i]
      const int oi = q - 2 * Nt, o = oi / Ci, i = oi - o * Ci;
      for (int t = 0; t < Nt; ++t)
        sum += (double)wt[t] * G[(long long)(i + 1) * npair + o * Nt + t] +
               (bt != nullptr ? (double)bt[t] * G[o * Nt + t] : 0.0);
      if (gwc != nullptr) gwc[oi] = (float)sum;
    } else {                                     // gbc[o]
      const int o = q - 2 * Nt - Co * Ci;
      for (int t = 0; t < Nt; ++t) sum += G[o * Nt + t];
      if (gbc != nullptr) gbc[o] = (float)sum;
    }
  }
}

template <int CI>
__global__ __launch_bounds__(kThreads) void pointwise_mlp2_kernel(
    int Ci, int H, int Co, long long np, const float* __restrict__ x, const float* __restrict__ W1,
    const float* __restrict__ b1, const float* __restrict__ W2, const float* __restrict__ b2,
    float* __restrict__ y) {
  const long long p = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long b = blockIdx.y;
  if (p >= np) return;
  float xv[CI];
#pragma unroll
  for (int i = 0; i < CI; ++i) xv[i] = (i < Ci) ? x[(b * Ci + i) * np + p] : 0.f;
  float acc[4];
#pragma unroll
  for (int o = 0; o < 4; ++o) acc[o] = (b2 != nullptr && o < Co) ? b2[o] : 0.f;
  for (int h = 0; h < H; ++h) {
    float s = (b1 != nullptr) ? b1[h] : 0.f;
#pragma unroll
    for (int i = 0; i < CI; ++i)
      if (i < Ci) s = fmaf(W1[h * Ci + i], xv[i], s);
    const float gh = gelu_f(s);
#pragma unroll
    for (int o = 0; o < 4; ++o)
      if (o < Co) acc[o] = fmaf(W2[o * H + h], gh, acc[o]);
  }
#pragma unroll
  for (int o = 0; o < 4; ++o)
    if (o < Co) y[(b * Co + o) * np + p] = acc[o];
}

int pick_q(AxisPlan az, int Nt) {
  // smallest divisor Q of Pz whose Q adjacent rows span at least 128 bytes; when that would make
  // the tile taller than 64 rows (Pz prime or nearly so): a Q that
  // need not divide Pz (the kernel skips the classes past the end of the last group), sized
  // for about one grid point per thread
  for (int q = 1; q <= az.P; ++q)
    if (az.P % q == 0 && q * Nt >= 32 && q * az.M <= 64) return q;
  int q = 256 / (Nt * az.M);        // about one point per thread
  if (q < 1) q = 1;
  if (q > az.P) q = az.P;
  while (q > 1 && q * az.M > 64) --q;
  return q;
}

size_t tz_fwd_lds(AxisPlan az, int Nt, int mt, int ppb) {
  size_t s_floats = (size_t)ppb * az.N * (Nt + 1);
  s_floats += (s_floats & 1);
  return s_floats * 4 + (size_t)ppb * mt * tz_row_stride(az.N) * 8;
}

size_t zt_inv_lds(AxisPlan az, int Nt, int mt, int Co) {
  const int Rz = pick_q(az, Nt) * az.M;
  // V and Y (one buffer where Y may take V's place), rounded up to 16 bytes, and the epilogue's
  // weights for up to kMaxCo x kMaxCo channels
  const size_t v_floats = (size_t)2 * Co * Rz * mt, y_floats = (size_t)Co * Rz * (Nt + 1);
  const size_t vy = zt_y_over_v(Nt, Co * Rz, mt) ? (v_floats > y_floats ? v_floats : y_floats) : v_floats + y_floats;
  return ((vy + 3) & ~(size_t)3) * 4 + (size_t)kMaxCo * kMaxCo * 4;
}

int axis_cols(AxisPlan ax, int64_t inner, int rows, int wmax) {
  // widest column tile whose [rows][w] complex tile stays within 32 KiB of LDS
  int w = wmax;
  while (w > 1 && (size_t)rows * w * 8 > (size_t)(32 * 1024)) w >>= 1;
  while (w > 1 && (w >> 1) >= inner) w >>= 1;
  return w;
}

int axis_threads(int items) {
  int t = ((items + 63) / 64) * 64;
  return t < 64 ? 64 : (t > kThreads ? kThreads : t);
}


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

bool tz_fwd_fits(AxisPlan az, int Nt, int mt) { return tz_fwd_lds(az, Nt, mt, 1) <= (size_t)kLdsBudget; }
bool zt_inv_fits(AxisPlan az, int Nt, int mt, int Co) {
  return Co <= kMaxCo && zt_inv_lds(az, Nt, mt, Co) <= (size_t)(68 * 1024);
}
bool axis_fits(AxisPlan ax) { return (size_t)ax.N * 8 <= (size_t)(32 * 1024); }
int mfma_q_nw(AxisPlan az, int Nt, int nw);
int mfma_nw(AxisPlan az, int Nt, int mt, int Co, int Cu);
size_t zt_mfma_lds(AxisPlan az, int Nt, int mt, int Co, int Cu, int q);
bool mfma_cfg_ok(AxisPlan az, int Nt, int mt, int Co, int Cu, int nw, size_t lds_cap) {
  const int q = mfma_q_nw(az, Nt, nw);
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  // the tile is staged in 16-byte pieces (L * mt even) and a thread owns at most two z-stage items
  return q > 0 && (az.L * mt) % 2 == 0 && Co * mt * q <= (nw == 8 ? 512 : 512) && Co <= kMaxCo && Cu <= 4 * CT &&
         (nw == 4 || CT <= 5) && zt_mfma_lds(az, Nt, mt, Co, Cu, q) <= lds_cap;
}
int mfma_tile_nt(int Nt);
bool zt_mfma_fits(AxisPlan az, int Nt, int mt, int Co, int Cu) {
  const int ntt = mfma_tile_nt(Nt);
  return ntt > 0 && mfma_nw(az, ntt, mt, Co, Cu) > 0;
}

hipError_t launch_axis_table(float2* tw, AxisPlan ax, hipStream_t s) {
  const int n = ax.L * ax.P;
  hipLaunchKernelGGL(axis_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, tw, ax.N, ax.L,
                     ax.npos, ax.P);
  return hipGetLastError();
}

hipError_t launch_t_table(float2* twt, int Nt, int mt, hipStream_t s) {
  const int n = Nt * mt;
  hipLaunchKernelGGL(t_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, twt, Nt, mt);
  return hipGetLastError();
}

int ilog2(int v);
int tz_fast_region(AxisPlan az, int Nt, int mt, int ppb) {
  const int s_floats = ppb * az.N * Nt;
  const int t_floats = 2 * ppb * mt * (az.N + 1);
  const int r = s_floats > t_floats ? s_floats : t_floats;
  return (r + 255) & ~255;
}

size_t tz_fast_lds(AxisPlan az, int Nt, int mt, int ppb) {
  const size_t tw_floats = ((size_t)az.L * az.P * 2 + 255) & ~size_t(255);      // whole 1 KiB loads
  return ((size_t)tz_fast_region(az, Nt, mt, ppb) + tw_floats) * 4;
}

hipError_t launch_tz_fwd(const float* x, float2* out, const float2* twt, const float2* twz,
                         int64_t planes, AxisPlan az, int Nt, int mt, hipStream_t s) {
  if (planes <= 0) return hipSuccess;
  const bool fast = (Nt == 16 || Nt == 32 || Nt == 64) && (az.M == 8 || az.M == 16) &&
                    (az.P & (az.P - 1)) == 0 && (az.N * Nt) % 256 == 0 && (az.L * az.P) % 2 == 0 &&
                    az.L * mt < 7000 && az.N <= kThreads &&
                    ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(twz)) & 15) == 0 &&
                    tz_fast_lds(az, Nt, mt, 1) <= (size_t)kLdsBudget;
  if (fast) {
    int ppb = 1;
    while (ppb * 2 * az.N <= 256 && tz_fast_lds(az, Nt, mt, ppb * 2) <= (size_t)kLdsBudget) ppb *= 2;
    const int thr = ((ppb * az.N + 63) / 64) * 64;
    const size_t lds = tz_fast_lds(az, Nt, mt, ppb);
    const int region = tz_fast_region(az, Nt, mt, ppb);
    const int64_t nblk = (planes + ppb - 1) / ppb;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    const int inv_mt = (65536 + mt - 1) / mt;
#define FNO_TZF(NTV, MZV)                                                                     \
  hipLaunchKernelGGL((tz_fwd_fast_kernel<NTV, MZV>), dim3((unsigned)nblk), dim3(thr), lds, s, \
                     x, out, twz, (long long)planes, az.N, az.L, az.npos, mt, ppb, region,    \
                     ilog2(az.P), inv_mt)
#define FNO_TZF_M(NTV)                     \
  do {                                     \
    if (az.M == 8) FNO_TZF(NTV, 8);        \
    else FNO_TZF(NTV, 16);                 \
  } while (0)
    if (Nt == 16) FNO_TZF_M(16); else if (Nt == 32) FNO_TZF_M(32); else FNO_TZF_M(64);
#undef FNO_TZF_M
#undef FNO_TZF
    return hipGetLastError();
  }
  if (az.M == 1 && Nt % 4 == 0 && mt <= 16 && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
    const int ppb = 16 / mt;
    const size_t t_bytes = (size_t)16 * tzd_row_stride(az.N) * 8;
    const size_t p_bytes = (size_t)(kThreads / 64) * kDenseMT * 16 * 16 * 8;
    const int alias = az.L <= kDenseMT * 16;      // one sweep: the partial sums reuse the rows' LDS
    const size_t lds = alias ? (t_bytes > p_bytes ? t_bytes : p_bytes) : t_bytes + p_bytes;
    const int64_t nblk = (planes + ppb - 1) / ppb;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    if (lds <= (size_t)(150 * 1024)) {
      hipLaunchKernelGGL(tz_fwd_dense_kernel, dim3((unsigned)nblk), dim3(kThreads), lds, s, x, out, twt, twz,
                         (long long)planes, az.N, Nt, az.L, mt, ppb, alias);
      return hipGetLastError();
    }
  }
  int ppb = 1;
  // enough rows to occupy the block, within an LDS share that keeps several blocks per CU
  while (ppb * 2 * az.N <= 2 * kThreads && tz_fwd_lds(az, Nt, mt, ppb * 2) <= (size_t)(32 * 1024)) ppb *= 2;
  const size_t lds = tz_fwd_lds(az, Nt, mt, ppb);
  const int64_t nblk = (planes + ppb - 1) / ppb;
  if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
  FNO_DISPATCH_M(az.M, hipLaunchKernelGGL((tz_fwd_kernel<MM>), dim3((unsigned)nblk), dim3(kThreads),
                                          lds, s, x, out, twt, twz, (long long)planes, az.N, Nt,
                                          az.L, az.npos, mt, ppb));
  return hipGetLastError();
}

hipError_t launch_axis_fwd(const float2* in, float2* out, const float2* tw, int64_t outer,
                           AxisPlan ax, int64_t inner, hipStream_t s) {
  if (outer <= 0 || inner <= 0) return hipSuccess;
  const int W = axis_cols(ax, inner, ax.N, 16);
  const int64_t ncb = (inner + W - 1) / W;
  const int64_t nblk = outer * ncb;
  if (nblk > 0x7fffffffLL || ncb > 0x7fffffffLL) return hipErrorInvalidValue;
  // the twiddles go to LDS only when that does not cost a resident block
  const int tw_lds = (size_t)ax.L * ax.P * 8 <= (size_t)(8 * 1024) && (size_t)ax.N * W * 8 <= (size_t)(16 * 1024);
  const size_t lds = (size_t)ax.N * W * 8 + (tw_lds ? (size_t)ax.L * ax.P * 8 : 0);
  FNO_DISPATCH_M(ax.M, hipLaunchKernelGGL((axis_fwd_kernel<MM>), dim3((unsigned)nblk),
                                          dim3(kThreads), lds, s, in, out, tw, ax.N, ax.L, ax.npos,
                                          (long long)inner, W, (int)ncb, tw_lds));
  return hipGetLastError();
}

hipError_t launch_axis_inv(const float2* in, float2* out, const float2* tw, int64_t outer,
                           AxisPlan ax, int64_t inner, hipStream_t s) {
  if (outer <= 0 || inner <= 0) return hipSuccess;
  const int W = axis_cols(ax, inner, ax.L, 32);
  const int64_t ncb = (inner + W - 1) / W;
  const int64_t nblk = outer * ncb;
  if (nblk > 0x7fffffffLL || ncb > 0x7fffffffLL) return hipErrorInvalidValue;
  const int tw_lds = (size_t)ax.L * ax.P * 8 <= (size_t)(8 * 1024);
  const size_t lds = (size_t)ax.L * W * 8 + (tw_lds ? (size_t)ax.L * ax.P * 8 : 0);
  const int thr = axis_threads(ax.P * W);
  FNO_DISPATCH_M(ax.M, hipLaunchKernelGGL((axis_inv_kernel<MM>), dim3((unsigned)nblk),
                                          dim3(thr), lds, s, in, out, tw, ax.N, ax.L, ax.npos,
                                          (long long)inner, W, (int)ncb, tw_lds));
  return hipGetLastError();
}

hipError_t launch_mix_fwd(const float2* xh, const float2* R, float2* yh, int B, int Ci, int Co,
                          int64_t K, int mt, int Nt, double invN, hipStream_t s) {
  const int64_t nb = (K + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || Co > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mix_fwd_kernel, dim3((unsigned)nb, (unsigned)((Co + kMixO - 1) / kMixO)), dim3(kThreads), 0, s, xh, R,
                     yh, B, Ci, Co, (long long)K, mt, Nt, (float)invN);
  return hipGetLastError();
}

hipError_t launch_mix_bwd(const float2* xh, const float2* R, const float2* gh, float2* gR,
                          float2* gxh, int B, int Ci, int Co, int64_t K, int mt, int Nt,
                          double invN, hipStream_t s) {
  const int64_t nb = (K + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || Ci > 4 * 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mix_bwd_kernel, dim3((unsigned)nb, (unsigned)((Ci + kMixI - 1) / kMixI)), dim3(kThreads), 0, s, xh, R,
                     gh, gR, gxh, B, Ci, Co, (long long)K, mt, Nt, (float)invN);
  return hipGetLastError();
}

// Tile of the matrix-core kernel: Q residue classes whose Rz = Q*M rows times Nt points make
// 128..512 points (64..256 threads, two points each) and whose Q adjacent rows span at least 128 bytes.
// Rows per tile for NW waves: each wave covers 128 points.  Returns Q = rows / M, or 0.
// t-tile of the matrix-core kernels for an axis of length Nt: 16 or 32 points, the axis itself or
// the next tile width above an even length; 0 when neither fits
int mfma_tile_nt(int Nt) {
  if (Nt == 16 || Nt == 32) return Nt;
  if (Nt % 2 != 0 || Nt < 10 || Nt > 32) return 0;
  return Nt < 16 ? 16 : 32;
}

int mfma_q_nw(AxisPlan az, int Nt, int nw) {
  if (Nt != 16 && Nt != 32) return 0;
  if (az.M != 8 && az.M != 16) return 0;
  if (az.P & (az.P - 1)) return 0;                 // residue-class count must be a power of two
  const int rz = nw * (128 / Nt);
  if (rz % az.M) return 0;
  const int q = rz / az.M;
  if (q > az.P) return 0;
  return q;
}

bool mfma_cfg_ok(AxisPlan az, int Nt, int mt, int Co, int Cu, int nw, size_t lds_cap);

// Eight waves (two blocks per CU) when the tile then still fits half a CU's LDS, else four.
int mfma_nw(AxisPlan az, int Nt, int mt, int Co, int Cu) {
  if (mfma_cfg_ok(az, Nt, mt, Co, Cu, 8, 78 * 1024)) return 8;
  if (mfma_cfg_ok(az, Nt, mt, Co, Cu, 4, 80 * 1024)) return 4;
  return 0;
}

int mfma_q(AxisPlan az, int Nt) { return mfma_q_nw(az, Nt, 4); }

int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

// LDS channel stride of the spectrum tile in float4: padded so that consecutive channels start
// 2 mt .. 64 - 2 mt floats apart modulo the 64 banks
int zt_mfma_astride4(AxisPlan az, int mt) {
  const int per_ch4 = (az.L * mt) / 2;
  for (int pad = 0; pad < 16; ++pad) {
    const int r = (4 * (per_ch4 + pad)) % 64;
    if (r >= 2 * mt && r <= 64 - 2 * mt) return per_ch4 + pad;
  }
  return per_ch4 + 1;
}

// channel stride of V in float2: rows * mt padded to 2 modulo 32, so that the four channels an
// MFMA block reads together fall into different banks
int zt_mfma_vstride(AxisPlan az, int mt, int q) {
  const int base = q * az.M * mt;
  return base + ((2 - base) % 32 + 32) % 32;
}

// floats of the region shared by the spectrum tile and V
int zt_mfma_region(AxisPlan az, int mt, int Co, int q) {
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  const int a_floats = Co * zt_mfma_astride4(az, mt) * 4 + 256;   // the last wave load may run 63 lanes past
  const int v_floats = 2 * 4 * CT * zt_mfma_vstride(az, mt, q);
  const int r = a_floats > v_floats ? a_floats : v_floats;
  return (r + 255) & ~255;
}

int zt_mfma_blob(AxisPlan az, int Nt, int mt, int Co, int Cu, int q) {
  const int CP = 4 * ((Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8));
  return ((2 * mt * Nt + Cu * CP + 2 * q * az.L + CP + 255) / 256) * 256;      // whole 1 KiB wave loads
}

size_t zt_mfma_lds(AxisPlan az, int Nt, int mt, int Co, int Cu, int q) {
  return ((size_t)zt_mfma_region(az, mt, Co, q) + (size_t)zt_mfma_blob(az, Nt, mt, Co, Cu, q)) * 4;
}

hipError_t launch_zt_inv(const float2* a, float* out, const float2* twt, const float2* twz, int B,
                         int Co, int Nx, int Ny, AxisPlan az, int Nt, int mt, Epilogue ep,
                         float* tables, hipStream_t s) {
  const int64_t ncols = (int64_t)B * Nx * Ny;
  if (ncols <= 0) return hipSuccess;
  if (Co > kMaxCo) return hipErrorInvalidValue;
  EpiArgs e{ep.u, ep.Cu, ep.W, ep.w_so, ep.w_si, ep.bias, ep.zsave, ep.act};
  const int NxNy = Nx * Ny;
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  const int ntt = mfma_tile_nt(Nt);           // t-tile of the matrix-core kernels (0: none)
  const bool tpad = ntt != Nt;
  const int nw = ntt > 0 ? mfma_nw(az, ntt, mt, Co, ep.u ? ep.Cu : 0) : 0;
  const int qf = nw > 0 ? mfma_q_nw(az, ntt, nw) : 0;
  const bool aligned = ((reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(ep.u) |
                         reinterpret_cast<uintptr_t>(ep.zsave) | reinterpret_cast<uintptr_t>(a) |
                         reinterpret_cast<uintptr_t>(tables)) & 15) == 0;
  // Column kernel (Nt = 32, 16-point z FFT): the spectrum of a column is staged once instead of
  // once per tile.  Taken when two blocks fit a CU's LDS, else the per-tile kernel below.
  if (aligned && tables != nullptr && Nt == 32 && az.M == 16 && az.P >= 2 && az.P % 2 == 0 &&
      (az.P & (az.P - 1)) == 0 && CT <= 5 && Co * mt <= 512 && (az.L * mt) % 2 == 0 && B <= 65535) {
    const int Cu = ep.u ? ep.Cu : 0;
    const int a_stride4 = zt_mfma_astride4(az, mt);
    const int a_floats = (Co * a_stride4 * 4 + 255) & ~255;
    const int v_stride = zt_mfma_vstride(az, mt, 1);
    const int blob_floats = zt_mfma_blob(az, Nt, mt, Co, Cu, az.P);
    const size_t lds = ((size_t)a_floats + 2 * 4 * CT * v_stride + blob_floats) * 4;
    if (Cu <= 4 * CT && lds <= (size_t)(79 * 1024) && (size_t)blob_floats * 4 <= kZtTablesBytes) {
      const bool full = (Co == 4 * CT) && (ep.u == nullptr || ep.Cu == 4 * CT);
      const int inv_mt = (65536 + mt - 1) / mt;
      hipLaunchKernelGGL(zt_tables_kernel, dim3(1), dim3(256), 0, s, tables, twt, twz, ep.u ? ep.W : nullptr,
                         ep.w_so, ep.w_si, ep.bias, Co, Cu, 4 * CT, mt, Nt, Nt, az.L, az.P, az.P, blob_floats);
      const dim3 grid((unsigned)NxNy, (unsigned)B);
#define FNO_ZTC(CTV, FULLV)                                                                        \
  hipLaunchKernelGGL((zt_inv_col_kernel<CTV, FULLV>), grid, dim3(512), lds, s, a, out, Co, NxNy,   \
                     az.N, az.L, az.npos, mt, inv_mt, a_floats, a_stride4, v_stride, tables,       \
                     blob_floats, e)
      if (CT == 2) { if (full) FNO_ZTC(2, true); else FNO_ZTC(2, false); }
      else { if (full) FNO_ZTC(5, true); else FNO_ZTC(5, false); }
#undef FNO_ZTC
      return hipGetLastError();
    }
  }
  if (qf > 0 && aligned) {
    const int G = az.P / qf;
    const int64_t gx = (int64_t)((NxNy + 7) / 8) * 8 * G;
    if (gx > 0x7fffffffLL || B > 65535 || Co * mt > 7000) return hipErrorInvalidValue;
    const int thr = 64 * nw;
    const size_t lds = zt_mfma_lds(az, ntt, mt, Co, ep.u ? ep.Cu : 0, qf);
    const int inv_mt = (65536 + mt - 1) / mt;
    const bool full = !tpad && (Co == 4 * CT) && (ep.u == nullptr || ep.Cu == 4 * CT);
    const dim3 grid((unsigned)gx, (unsigned)B);
    const int blob_floats = zt_mfma_blob(az, ntt, mt, Co, ep.u ? ep.Cu : 0, qf);
    if (tables == nullptr || (size_t)G * blob_floats * 4 > kZtTablesBytes) return hipErrorInvalidValue;
    hipLaunchKernelGGL(zt_tables_kernel, dim3(G), dim3(256), 0, s, tables, twt, twz, ep.u ? ep.W : nullptr,
                       ep.w_so, ep.w_si, ep.bias, Co, ep.u ? ep.Cu : 0, 4 * CT, mt, ntt, Nt, az.L, az.P, qf,
                       blob_floats);
#define FNO_ZTM(NTV, MZV, CTV, FULLV, NWV, TPADV)                                                     \
  hipLaunchKernelGGL((zt_inv_mfma_kernel<NTV, MZV, CTV, FULLV, NWV, TPADV>), grid, dim3(thr), lds, s, \
                     a, out, twt, twz, Co, NxNy, az.N, Nt, az.L, az.npos, mt, ilog2(qf), ilog2(G),    \
                     inv_mt, zt_mfma_region(az, mt, Co, qf), zt_mfma_astride4(az, mt),                \
                     zt_mfma_vstride(az, mt, qf), tables, blob_floats, e)
#define FNO_ZTM_F(NTV, MZV, CTV)                                         \
  do {                                                                   \
    if (tpad && nw == 8) FNO_ZTM(NTV, MZV, CTV, false, 8, true);         \
    else if (tpad) FNO_ZTM(NTV, MZV, CTV, false, 4, true);               \
    else if (nw == 8 && full) FNO_ZTM(NTV, MZV, CTV, true, 8, false);    \
    else if (nw == 8) FNO_ZTM(NTV, MZV, CTV, false, 8, false);           \
    else if (full) FNO_ZTM(NTV, MZV, CTV, true, 4, false);               \
    else FNO_ZTM(NTV, MZV, CTV, false, 4, false);                        \
  } while (0)
#define FNO_ZTM_CT(NTV, MZV)                                        \
  do {                                                              \
    if (CT == 2) FNO_ZTM_F(NTV, MZV, 2);                            \
    else if (CT == 5) FNO_ZTM_F(NTV, MZV, 5);                       \
    else if (tpad) FNO_ZTM(NTV, MZV, 8, false, 4, true);            \
    else FNO_ZTM(NTV, MZV, 8, false, 4, false);                     \
  } while (0)
#define FNO_ZTM_M(NTV)                                  \
  do {                                                  \
    if (az.M == 8) FNO_ZTM_CT(NTV, 8);                  \
    else FNO_ZTM_CT(NTV, 16);                           \
  } while (0)
    if (ntt == 16) FNO_ZTM_M(16); else FNO_ZTM_M(32);
#undef FNO_ZTM_M
#undef FNO_ZTM_CT
#undef FNO_ZTM_F
#undef FNO_ZTM
    return hipGetLastError();
  }
  const int Q = pick_q(az, Nt);
  const int G = (az.P + Q - 1) / Q;
  const int64_t nblk = ncols * G;
  if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
  const size_t lds = zt_inv_lds(az, Nt, mt, Co);
  // the channel counts fill the kernel's register tile exactly: the variant without per-channel guards
#define FNO_ZT_CALL(COV)                                                                              \
  do {                                                                                                \
    if (Co == COV && (e.u == nullptr || e.Cu == COV)) {                                               \
      FNO_DISPATCH_M(az.M, hipLaunchKernelGGL((zt_inv_kernel<MM, COV, true>), dim3((unsigned)nblk),   \
                                              dim3(kThreads), lds, s, a, out, twt, twz, Co, NxNy,     \
                                              az.N, Nt, az.L, az.npos, mt, Q, e));                    \
    } else {                                                                                          \
      FNO_DISPATCH_M(az.M, hipLaunchKernelGGL((zt_inv_kernel<MM, COV, false>), dim3((unsigned)nblk),  \
                                              dim3(kThreads), lds, s, a, out, twt, twz, Co, NxNy,     \
                                              az.N, Nt, az.L, az.npos, mt, Q, e));                    \
    }                                                                                                 \
  } while (0)
  if (Co <= 8) { FNO_ZT_CALL(8); }
  else if (Co <= 20) { FNO_ZT_CALL(20); }
  else { FNO_ZT_CALL(32); }
#undef FNO_ZT_CALL
  return hipGetLastError();
}

// number of partial-sum slots the workspace must hold (one per wave of the streaming kernel)
int bwd_pointwise_blocks(int B, int64_t N) {
  (void)B; (void)N;
  return 4096;
}

hipError_t launch_bwd_pointwise(const float* z, const float* gout, const float* x, float* gz_out,
                                double* part, int* nslots, int B, int Ci, int Co, int64_t N, int act,
                                int mse_target, double mse_scale, hipStream_t s) {
  if (Co * Ci + Co > kBwdPairs * kThreads) return hipErrorInvalidValue;
  const bool aligned = ((reinterpret_cast<uintptr_t>(z) | reinterpret_cast<uintptr_t>(gout) |
                         reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(gz_out)) & 15) == 0;
  if (Ci == Co && Co % 4 == 0 && Co <= 20 && N % 64 == 0 && aligned) {
    const int64_t steps = (N / 64) * B;
    int64_t nb = (steps + 3) / 4;
    if (nb > 1024) nb = 1024;
    *nslots = (int)nb * 4;
    const dim3 grid((unsigned)nb);
    switch (Co / 4) {
#define FNO_BPW(CTV)                                                                               \
  case CTV:                                                                                        \
    hipLaunchKernelGGL((bwd_pointwise_mfma_kernel<CTV>), grid, dim3(kThreads), 0, s, z, gout, x,   \
                       gz_out, part, B, (long long)N, act, mse_target, (float)mse_scale);          \
    break;
      FNO_BPW(1) FNO_BPW(2) FNO_BPW(3) FNO_BPW(4) FNO_BPW(5)
#undef FNO_BPW
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  const int64_t tiles = (int64_t)B * ((N + kBwdTile - 1) / kBwdTile);
  const int nblk = (int)(tiles < 2048 ? tiles : 2048);
  *nslots = nblk;
  const size_t lds = (size_t)(Co + Ci) * (kBwdTile + 1) * 4;
  hipLaunchKernelGGL(bwd_pointwise_kernel, dim3((unsigned)nblk), dim3(kThreads), lds, s, z, gout,
                     x, gz_out, part, B, Ci, Co, (long long)N, act, mse_target, (float)mse_scale);
  return hipGetLastError();
}

hipError_t launch_reduce_partials(const double* part, int nblk, int Co, int Ci, float* gW,
                                  float* gb, hipStream_t s) {
  const int npairs = Co * Ci + Co;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((npairs + 63) / 64), dim3(64 * kRedGroups), 0, s, part,
                     nblk, Co, Ci, gW, gb);
  return hipGetLastError();
}

hipError_t launch_pointwise_linear(int B, int Ci, int Co, int64_t np, const float* x, const float* W,
                                   const float* bias, float* y, hipStream_t s) {
  const int64_t nb = (np + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || B > 65535 || Co > 32) return hipErrorInvalidValue;
  if (nb == 0 || B == 0) return hipSuccess;
  dim3 grid((unsigned)nb, (unsigned)B);
  if (Co <= 8)
    hipLaunchKernelGGL((pointwise_linear_kernel<8>), grid, dim3(kThreads), 0, s, Ci, Co,
                       (long long)np, x, W, bias, y);
  else if (Co <= 20)
    hipLaunchKernelGGL((pointwise_linear_kernel<20>), grid, dim3(kThreads), 0, s, Ci, Co,
                       (long long)np, x, W, bias, y);
  else
    hipLaunchKernelGGL((pointwise_linear_kernel<32>), grid, dim3(kThreads), 0, s, Ci, Co,
                       (long long)np, x, W, bias, y);
  return hipGetLastError();
}

// The matrix-core projection kernels take hidden widths that are whole 32-row blocks, one wave
// each, and tiles whose (c_in + c_out) x 64 values the block's threads stage in kMlpStage loads.
bool mlp2_mfma_fits(int Ci, int H, int Co) {
  if (H % 32 != 0 || H < 32 || H > 256 || Ci > 31 || Co > 4 || Ci < 1 || Co < 1) return false;
  return Ci + Co <= kMlpStage * (H / 32);
}

size_t mlp2_bwd_mfma_lds(int Ci, int H, int Co) {
  const int nw = H / 32, co = Co == 1 ? 1 : 4;
  size_t floats = (size_t)32 * kMlpXS + (size_t)co * kMlpTile + (size_t)nw * 32 * kMlpTS + (size_t)nw * Ci * kMlpXS;
  if (co > 1) floats += (size_t)co * H;
  floats += floats & 1;
  return floats * 4 + ((size_t)H * (Ci + 1) + (size_t)Co * H + Co) * 8;
}

hipError_t launch_pointwise_mlp2(int B, int Ci, int H, int Co, int64_t np, const float* x,
                                 const float* W1, const float* b1, const float* W2,
                                 const float* b2, float* y, hipStream_t s) {
  const int64_t nb = (np + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || B > 65535 || Co > 4 || Ci > 32) return hipErrorInvalidValue;
  if (nb == 0 || B == 0) return hipSuccess;
  if (mlp2_mfma_fits(Ci, H, Co)) {
    const int nw = H / 32;
    const int64_t tiles = (int64_t)B * ((np + kMlpTile - 1) / kMlpTile);
    const unsigned nblk = (unsigned)(tiles < 2048 ? tiles : 2048);
    const int co = Co == 1 ? 1 : 4;
    const size_t lds = (size_t)(32 * kMlpXS + nw * co * kMlpTile) * 4;
#define FNO_MLPF(KSV, COV)                                                                              \
  hipLaunchKernelGGL((mlp2_fwd_mfma_kernel<KSV, COV>), dim3(nblk), dim3(64 * nw), lds, s, B, Ci, H, Co, \
                     (long long)np, x, W1, b1, W2, b2, y)
    if (Ci <= 21) { if (co == 1) FNO_MLPF(11, 1); else FNO_MLPF(11, 4); }
    else { if (co == 1) FNO_MLPF(16, 1); else FNO_MLPF(16, 4); }
#undef FNO_MLPF
    return hipGetLastError();
  }
  dim3 grid((unsigned)nb, (unsigned)B);
  if (Ci <= 20)
    hipLaunchKernelGGL((pointwise_mlp2_kernel<20>), grid, dim3(kThreads), 0, s, Ci, H, Co,
                       (long long)np, x, W1, b1, W2, b2, y);
  else
    hipLaunchKernelGGL((pointwise_mlp2_kernel<32>), grid, dim3(kThreads), 0, s, Ci, H, Co,
                       (long long)np, x, W1, b1, W2, b2, y);
  return hipGetLastError();
}

hipError_t launch_time_lift(int B, int Ci, int Co, int64_t np, int Nt, const float* a, const float* wt,
                            const float* bt, const float* wc, const float* bc, float* out, hipStream_t s) {
  const int nt4 = (Nt + 3) / 4;
  const int64_t nb = (np * nt4 + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || B > 65535 || Co > 32) return hipErrorInvalidValue;
  if (nb == 0 || B == 0) return hipSuccess;
  // float4 stores need whole quads per row and an aligned tensor
  if ((Nt & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) != 0) return hipErrorInvalidValue;
  dim3 grid((unsigned)nb, (unsigned)B);
  if (Co <= 8)
    hipLaunchKernelGGL((time_lift_kernel<8>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)np, Nt, a, wt,
                       bt, wc, bc, out);
  else if (Co <= 20)
    hipLaunchKernelGGL((time_lift_kernel<20>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)np, Nt, a, wt,
                       bt, wc, bc, out);
  else
    hipLaunchKernelGGL((time_lift_kernel<32>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)np, Nt, a, wt,
                       bt, wc, bc, out);
  return hipGetLastError();
}

size_t time_lift_bwd_workspace_bytes(int Ci, int Co, int Nt) {
  return ((size_t)kLiftChunks + 1) * (size_t)(Ci + 1) * Co * Nt * sizeof(double);
}

hipError_t launch_time_lift_bwd(int B, int Ci, int Co, int64_t S, int Nt, const float* a, const float* wt,
                                const float* bt, const float* wc, const float* g, float* gwt, float* gbt,
                                float* gwc, float* gbc, void* ws, hipStream_t s) {
  if (Ci > 8 || B > kLiftChunks || S <= 0) return hipErrorInvalidValue;
  const int npair = Co * Nt, nent = (Ci + 1) * npair;
  int cpb = (int)((S + 511) / 512);               // chunks per batch entry: at least 512 positions each
  if (cpb > kLiftChunks / B) cpb = kLiftChunks / B;
  if (cpb < 1) cpb = 1;
  const int nchunk = B * cpb;
  double* part = static_cast<double*>(ws);
  double* G = part + (size_t)kLiftChunks * nent;
  const dim3 grid((unsigned)((npair + kThreads - 1) / kThreads), (unsigned)nchunk);
#define FNO_TLB(CIV)                                                                                        \
  hipLaunchKernelGGL((time_lift_bwd_kernel<CIV>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)S, Nt, cpb, \
                     a, g, part)
  if (Ci == 1) FNO_TLB(1); else if (Ci == 2) FNO_TLB(2); else if (Ci <= 4) FNO_TLB(4); else FNO_TLB(8);
#undef FNO_TLB
  hipLaunchKernelGGL(time_lift_bwd_reduce_kernel, dim3((nent + 31) / 32), dim3(kThreads), 0, s, part, nchunk,
                     nent, G);
  hipLaunchKernelGGL(time_lift_bwd_final_kernel, dim3(1), dim3(kThreads), 0, s, Ci, Co, Nt, G, wt, bt, wc, gwt,
                     gbt, gwc, gbc);
  return hipGetLastError();
}

size_t rel_l2_workspace_bytes() { return (size_t)(2 * kLossBlocks + 1) * sizeof(double); }

hipError_t launch_rel_l2(int64_t n, const float* pred, const float* target, float* loss, float* grad,
                         double* ws, hipStream_t s) {
  if (n <= 0) return hipErrorInvalidValue;
  int nblk = (int)((n + kThreads - 1) / kThreads);
  if (nblk > kLossBlocks) nblk = kLossBlocks;
  double* scale = ws + 2 * kLossBlocks;
  hipLaunchKernelGGL(rel_l2_partial_kernel, dim3(nblk), dim3(kThreads), 0, s, (long long)n, pred, target, ws);
  hipLaunchKernelGGL(rel_l2_final_kernel, dim3(1), dim3(64), 0, s, ws, nblk, loss, scale);
  if (grad != nullptr) {
    int64_t gb = (n + kThreads - 1) / kThreads;
    if (gb > 65536) gb = 65536;
    hipLaunchKernelGGL(rel_l2_grad_kernel, dim3((unsigned)gb), dim3(kThreads), 0, s, (long long)n, pred, target,
                       scale, grad);
  }
  return hipGetLastError();
}

hipError_t launch_adam(int64_t n, float* p, const float* g, float* m, float* v, double lr, double beta1,
                       double beta2, double eps, int step, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const float c1 = (float)(1.0 / (1.0 - pow(beta1, (double)step)));
  const float c2 = (float)(1.0 / (1.0 - pow(beta2, (double)step)));
  int64_t nb = (n + kThreads - 1) / kThreads;
  if (nb > 65536) nb = 65536;
  hipLaunchKernelGGL(adam_kernel, dim3((unsigned)nb), dim3(kThreads), 0, s, (long long)n, p, g, m, v, (float)lr,
                     (float)beta1, (float)(1.0 - beta1), (float)beta2, (float)(1.0 - beta2), (float)eps, c1, c2);
  return hipGetLastError();
}

// doubles of partial sums + floats of a transposed weight
size_t pointwise_bwd_workspace_bytes(int Ci, int H, int Co) {
  const size_t lin = (size_t)2048 * ((size_t)Co * Ci + Co) * 8 + (size_t)Co * Ci * 4 + 64;
  const size_t mlp = (size_t)kMlpBlocks * ((size_t)H * (Ci + 1) + (size_t)Co * H + Co) * 8 + 64;
  return lin > mlp ? lin : mlp;
}

hipError_t launch_pointwise_linear_bwd(int B, int Ci, int Co, int64_t N, const float* x, const float* W,
                                       const float* g, float* gx, float* gW, float* gb, void* ws,
                                       hipStream_t s) {
  if (Co * Ci + Co > kBwdPairs * kThreads || Ci > 32) return hipErrorInvalidValue;
  if (N <= 0) return hipErrorInvalidValue;
  double* part = static_cast<double*>(ws);
  const int64_t tiles = (int64_t)B * ((N + kBwdTile - 1) / kBwdTile);
  const int nblk = (int)(tiles < 2048 ? tiles : 2048);
  if (gW != nullptr || gb != nullptr) {
    const size_t lds = (size_t)(Co + Ci) * (kBwdTile + 1) * 4;
    hipLaunchKernelGGL(bwd_pointwise_kernel, dim3((unsigned)nblk), dim3(kThreads), lds, s, g, g, x,
                       (float*)nullptr, part, B, Ci, Co, (long long)N, 0, 0, 0.f);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((Co * Ci + Co + 63) / 64), dim3(64 * kRedGroups), 0, s,
                       part, nblk, Co, Ci, gW, gb);
  }
  if (gx != nullptr) {
    float* wt = reinterpret_cast<float*>(part + (size_t)2048 * (Co * Ci + Co));
    hipLaunchKernelGGL(transpose_kernel, dim3((Co * Ci + 255) / 256), dim3(256), 0, s, W, wt, Co, Ci);
    const hipError_t e = launch_pointwise_linear(B, Co, Ci, N, g, wt, nullptr, gx, s);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

hipError_t launch_pointwise_mlp2_bwd(int B, int Ci, int H, int Co, int64_t N, const float* x, const float* W1,
                                     const float* b1, const float* W2, const float* g, float* gx, float* gW1,
                                     float* gb1, float* gW2, float* gb2, void* ws, hipStream_t s) {
  if (Ci > 32 || Co > 4 || N <= 0) return hipErrorInvalidValue;
  const int nsum = H * (Ci + 1) + Co * H + Co;
  if (mlp2_mfma_fits(Ci, H, Co) && mlp2_bwd_mfma_lds(Ci, H, Co) <= (size_t)(150 * 1024)) {
    const int nw = H / 32, co = Co == 1 ? 1 : 4;
    const size_t lds = mlp2_bwd_mfma_lds(Ci, H, Co);
    const int64_t tiles = (int64_t)B * ((N + kMlpTile - 1) / kMlpTile);
    const int nblk = (int)(tiles < kMlpBlocks ? tiles : kMlpBlocks);
    double* part = static_cast<double*>(ws);
#define FNO_MLPB(KSV, COV)                                                                                 \
  hipLaunchKernelGGL((mlp2_bwd_mfma_kernel<KSV, COV>), dim3((unsigned)nblk), dim3(64 * nw), lds, s, B, Ci, \
                     H, Co, (long long)N, x, W1, b1, W2, g, gx, part)
    if (Ci <= 21) { if (co == 1) FNO_MLPB(11, 1); else FNO_MLPB(11, 4); }
    else { if (co == 1) FNO_MLPB(16, 1); else FNO_MLPB(16, 4); }
#undef FNO_MLPB
    hipLaunchKernelGGL(reduce_ranges_kernel, dim3((nsum + kThreads - 1) / kThreads), dim3(kThreads), 0, s, part,
                       nblk, H * Ci, H, Co * H, Co, gW1, gb1, gW2, gb2);
    return hipGetLastError();
  }
  size_t lds_floats = (size_t)(Ci + Co + 2 * kMlpChunk) * (kThreads + 1);
  lds_floats += lds_floats & 1;
  const size_t lds = lds_floats * 4 + (size_t)nsum * 8;
  if (lds > (size_t)(150 * 1024)) return hipErrorInvalidValue;
  const int64_t tiles = (int64_t)B * ((N + kThreads - 1) / kThreads);
  const int nblk = (int)(tiles < kMlpBlocks ? tiles : kMlpBlocks);
  double* part = static_cast<double*>(ws);
  if (Ci <= 20)
    hipLaunchKernelGGL((mlp2_bwd_kernel<20>), dim3((unsigned)nblk), dim3(kThreads), lds, s, B, Ci, H, Co,
                       (long long)N, x, W1, b1, W2, g, gx, part);
  else
    hipLaunchKernelGGL((mlp2_bwd_kernel<32>), dim3((unsigned)nblk), dim3(kThreads), lds, s, B, Ci, H, Co,
                       (long long)N, x, W1, b1, W2, g, gx, part);
  hipLaunchKernelGGL(reduce_ranges_kernel, dim3((nsum + kThreads - 1) / kThreads), dim3(kThreads), 0, s, part,
                     nblk, H * Ci, H, Co * H, Co, gW1, gb1, gW2, gb2);
  return hipGetLastError();
}

}  // namespace fno
