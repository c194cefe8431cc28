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
//
// This file: twiddle tables, the forward (t, z) kernels, the pruned transforms along y and x,
// and the per-mode channel mix with its adjoint.
#include "fno_device.h"

namespace fno {

namespace {

// ------------------------------------------------------------------------------------------
// Twiddle tables (double-precision sincospi, rounded once to float)
// ------------------------------------------------------------------------------------------
// All tables of a plan in one launch: blockIdx.y picks the table.  An axis table holds
// w_N^(k_j n2) for the kept frequencies k_j and the residue classes n2 < P; the t table (L = 0)
// holds w_Nt^(kt n) for kt < npos (= mt), n < N (= Nt).
__global__ void plan_tables_kernel(TableSet ts) {
  const TableDesc t = ts.t[blockIdx.y];
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (t.L > 0) {
    if (idx >= t.L * t.P) return;
    const int j = idx / t.P, n2 = idx % t.P;
    const long long k = kfreq(j, t.L, t.npos);
    long long r = (k * n2) % t.N;
    if (r < 0) r += t.N;
    double s, c;
    sincospi(-2.0 * double(r) / double(t.N), &s, &c);
    t.tw[idx] = make_float2(float(c), float(s));
  } else {
    if (idx >= t.N * t.npos) return;
    const int kt = idx / t.N, n = idx % t.N;
    const long long r = ((long long)kt * n) % t.N;
    double s, c;
    sincospi(-2.0 * double(r) / double(t.N), &s, &c);
    t.tw[idx] = make_float2(float(c), float(s));
  }
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
  const long long plane0 = xcd_contiguous_item(blockIdx.x, gridDim.x) * ppb;   // grid: a multiple of 8
  if (plane0 >= planes) return;
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
  const long long plane0 = xcd_contiguous_item(blockIdx.x, gridDim.x) * ppb;   // grid: a multiple of 8
  if (plane0 >= planes) return;
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

// The same bins by a radix-4 split in time, for NT = 16 and 32: with n = 4 m + p,
//   X[K] = sum_{p<4} w_NT^{pK} D_p[K mod R],   D_p[q] = sum_{m<R} x[4m+p] w_R^{qm},  R = NT / 4,
// where each D_p is the transform of R real samples (the p-th component of the row's quads): only
// its bins 0..R/2 are computed, the others are their conjugates, and bins 0 and R/2 are real.
// About half the arithmetic of the packed complex transform above when few bins are kept.
// Forward transform of 4 / 8 real samples, bins 0..R/2 (w = exp(-2 pi i / R)).
__device__ __forceinline__ void real_dft(const float (&a)[4], float2 (&D)[3]) {
  const float s02 = a[0] + a[2], d02 = a[0] - a[2], s13 = a[1] + a[3], d13 = a[1] - a[3];
  D[0] = make_float2(s02 + s13, 0.f);
  D[1] = make_float2(d02, -d13);
  D[2] = make_float2(s02 - s13, 0.f);
}
__device__ __forceinline__ void real_dft(const float (&a)[8], float2 (&D)[5]) {
  constexpr float r = 0.70710678118654752440f;
  const float s04 = a[0] + a[4], d04 = a[0] - a[4], s26 = a[2] + a[6], d26 = a[2] - a[6];
  const float s15 = a[1] + a[5], d15 = a[1] - a[5], s37 = a[3] + a[7], d37 = a[3] - a[7];
  const float e0 = s04 + s26, e1 = s04 - s26, o0 = s15 + s37, o1 = s15 - s37;
  const float u = (d15 - d37) * r, v = (d15 + d37) * r;
  D[0] = make_float2(e0 + o0, 0.f);
  D[1] = make_float2(d04 + u, -d26 - v);
  D[2] = make_float2(e1, -o1);
  D[3] = make_float2(d04 - u, d26 - v);
  D[4] = make_float2(e0 - o0, 0.f);
}

// acc += exp(-2 pi i IDX / NT) * v, v complex or (REAL) real-valued
template <int NT, int IDX, bool REAL>
__device__ __forceinline__ float2 add_rooted(float2 acc, float2 v) {
  constexpr int idx = ((IDX % NT) + NT) % NT;
  constexpr float c = float(ct_cos_frac(idx, NT));
  constexpr float s = float(-ct_sin_frac(idx, NT));
  if constexpr (idx == 0) {
    acc.x += v.x;
    if constexpr (!REAL) acc.y += v.y;
  } else if constexpr (2 * idx == NT) {
    acc.x -= v.x;
    if constexpr (!REAL) acc.y -= v.y;
  } else if constexpr (4 * idx == NT) {            // * (-i)
    if constexpr (!REAL) acc.x += v.y;
    acc.y -= v.x;
  } else if constexpr (4 * idx == 3 * NT) {        // * (+i)
    if constexpr (!REAL) acc.x -= v.y;
    acc.y += v.x;
  } else {
    acc.x = fmaf(c, v.x, acc.x);
    acc.y = fmaf(s, v.x, acc.y);
    if constexpr (!REAL) {
      acc.x = fmaf(-s, v.y, acc.x);
      acc.y = fmaf(c, v.y, acc.y);
    }
  }
  return acc;
}

template <int NT, int K>
__device__ __forceinline__ void rfft4_bin(const float2 (&D)[4][NT / 8 + 1], int mt, float2 (&X)[NT / 2 + 1]) {
  constexpr int R = NT / 4;
  constexpr int q = K % R;
  constexpr bool real_bin = (q == 0) || (2 * q == R);
  constexpr bool conj_bin = 2 * q > R;
  constexpr int qi = conj_bin ? R - q : q;
  if (K < mt) {
    float2 acc = make_float2(D[0][qi].x, real_bin ? 0.f : (conj_bin ? -D[0][qi].y : D[0][qi].y));
    acc = add_rooted<NT, 1 * K, real_bin>(acc, make_float2(D[1][qi].x, conj_bin ? -D[1][qi].y : D[1][qi].y));
    acc = add_rooted<NT, 2 * K, real_bin>(acc, make_float2(D[2][qi].x, conj_bin ? -D[2][qi].y : D[2][qi].y));
    acc = add_rooted<NT, 3 * K, real_bin>(acc, make_float2(D[3][qi].x, conj_bin ? -D[3][qi].y : D[3][qi].y));
    X[K] = acc;
  }
}

template <int NT, int... Ks>
__device__ __forceinline__ void rfft4_bins(const float2 (&D)[4][NT / 8 + 1], int mt, float2 (&X)[NT / 2 + 1],
                                           std::integer_sequence<int, Ks...>) {
  (rfft4_bin<NT, Ks>(D, mt, X), ...);
}

template <int NT>
__device__ __forceinline__ void rfft_row_bins_r4(const float4 (&quads)[NT / 4], int mt, float2 (&X)[NT / 2 + 1]) {
  constexpr int R = NT / 4;
  float2 D[4][R / 2 + 1];
  float a[R];
#pragma unroll
  for (int m = 0; m < R; ++m) a[m] = quads[m].x;
  real_dft(a, D[0]);
#pragma unroll
  for (int m = 0; m < R; ++m) a[m] = quads[m].y;
  real_dft(a, D[1]);
#pragma unroll
  for (int m = 0; m < R; ++m) a[m] = quads[m].z;
  real_dft(a, D[2]);
#pragma unroll
  for (int m = 0; m < R; ++m) a[m] = quads[m].w;
  real_dft(a, D[3]);
  rfft4_bins<NT>(D, mt, X, std::make_integer_sequence<int, NT / 2 + 1>{});
}

// Bins 0..mt-1 of the real-input transform of one row of NT floats for an even NT that is no
// power of two: the plain sums, with x[n] and x[NT-n] folded (cos is even, sin odd in n), all
// twiddles compile-time constants.
//   Re X[k] = x[0] + (-1)^k x[NT/2] + sum_{0<n<NT/2} (x[n] + x[NT-n]) cos(2 pi k n / NT)
//   Im X[k] =                       - sum_{0<n<NT/2} (x[n] - x[NT-n]) sin(2 pi k n / NT)
template <int NT, int IDX> constexpr float kCosFrac = float(ct_cos_frac(IDX, NT));      // cos(2 pi IDX / NT)
template <int NT, int IDX> constexpr float kNegSinFrac = float(-ct_sin_frac(IDX, NT)); // -sin(2 pi IDX / NT)

template <int NT, int K, int... Ns>
__device__ __forceinline__ float2 dense_bin(const float (&sm)[NT / 2], const float (&df)[NT / 2], float x0, float xh,
                                            std::integer_sequence<int, Ns...>) {
  float re = (K % 2 == 0) ? x0 + xh : x0 - xh, im = 0.f;
  ((Ns > 0 ? (void)(re = fmaf(kCosFrac<NT, (K * Ns) % NT>, sm[Ns], re),
                    im = fmaf(kNegSinFrac<NT, (K * Ns) % NT>, df[Ns], im))
           : (void)0),
   ...);
  return make_float2(re, im);
}

template <int NT, int... Ks>
__device__ __forceinline__ void dense_bins(const float (&sm)[NT / 2], const float (&df)[NT / 2], float x0, float xh, int mt,
                                           float2 (&X)[NT / 2 + 1], std::integer_sequence<int, Ks...>) {
  ((Ks < mt ? (void)(X[Ks] = dense_bin<NT, Ks>(sm, df, x0, xh, std::make_integer_sequence<int, NT / 2>{})) : (void)0), ...);
}

template <int NT>
__device__ __forceinline__ void rdft_row_bins_dense(const float (&x)[NT], int mt, float2 (&X)[NT / 2 + 1]) {
  constexpr int H = NT / 2;
  float sm[H], df[H];
  sm[0] = 0.f; df[0] = 0.f;
#pragma unroll
  for (int n = 1; n < H; ++n) { sm[n] = x[n] + x[NT - n]; df[n] = x[n] - x[NT - n]; }
  dense_bins<NT>(sm, df, x[0], x[H], mt, X, std::make_integer_sequence<int, H + 1>{});
}

// One thread per z-row (blockDim.x >= ppb * Nz).  The planes and the z twiddles go straight to
// LDS (16 bytes per lane, 1 KiB per wave instruction, nothing staged in registers).  Inside a
// row the quads are stored rotated by the row number so that the row-per-thread reads of the
// t stage spread over all banks; a wave's load still covers whole 128-byte lines.  The t-stage
// results wait in registers over a barrier so the complex tile T can reuse the LDS of S.
// Pz is a power of two and inv_mt = ceil(2^16 / mt) (shifts and a multiply instead of divisions).
// MTC, LZC, NPC, PZC, NTHR: the kept counts on t and z (and how many of the latter are
// non-negative frequencies), log2 Pz and the block size as compile-time constants (0, or -1 for
// PZC: taken from the arguments).  With them the per-bin guards of the t stage vanish and the
// combine unrolls, its LDS reads going out together.
template <int NT, int MZ, int MTC, int LZC, int NPC, int PZC, int NTHR, bool STREAM>
__global__ __launch_bounds__(kThreads) void tz_fwd_fast_kernel(
    const float* __restrict__ x, float2* __restrict__ out, const float2* __restrict__ twz,
    long long planes, int Nz, int Lz_rt, int nposz_rt, int mt_rt, int ppb, int region_floats, int pzshift_rt,
    int inv_mt) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int mt = MTC ? MTC : mt_rt;
  const int Lz = LZC ? LZC : Lz_rt;
  const int nposz = LZC ? NPC : nposz_rt;
  const int pzshift = PZC >= 0 ? PZC : pzshift_rt;
  constexpr bool POW2 = (NT & (NT - 1)) == 0;  // else: an even length, rows unrotated, t stage as plain sums
  constexpr int QPR = POW2 ? NT / 4 : 1;       // quads per row
  constexpr int ROT = 16 / QPR > 0 ? 16 / QPR : 1;   // rows that share a rotation
  constexpr int H = NT / 2;
  const int Pz = 1 << pzshift;
  const int sT = tz_row_stride(Nz);            // row stride of T in float2
  float* S = smem;                             // [ppb * Nz] rows of QPR rotated quads
  float2* T = reinterpret_cast<float2*>(smem); // [ppb][mt][sT], same memory, later
  float2* TW = reinterpret_cast<float2*>(smem + region_floats);   // [Lz][Pz]
  const int tid = threadIdx.x;
  const int nthr = NTHR ? NTHR : (int)blockDim.x;
  const int lane = tid & 63, wave = tid >> 6;
  const long long plane0 = xcd_contiguous_item(blockIdx.x, gridDim.x) * ppb;   // grid: a multiple of 8
  if (plane0 >= planes) return;
  const int np = (int)min((long long)ppb, planes - plane0);

  {
    const float4* src = reinterpret_cast<const float4*>(x + plane0 * Nz * NT);
    if constexpr (POW2) {
      const int tot4 = np * Nz * QPR;            // a multiple of 64 (checked on the host)
      for (int c0 = wave * 64; c0 < tot4; c0 += nthr) {
        const int p4 = c0 + lane;
        const int zl = p4 / QPR, sl = p4 - zl * QPR;
        const int q = (sl - zl / ROT) & (QPR - 1);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + zl * QPR + q),
                                         (__attribute__((address_space(3))) void*)(S + 4 * c0), 16, 0, STREAM ? 2 : 0);   // aux 2: nontemporal
      }
    } else {
      const int tot4 = (np * Nz * NT) >> 2;      // whole 16-byte pieces (Nz NT is a multiple of 4, checked on the host)
      for (int c0 = wave * 64; c0 < tot4; c0 += nthr) {
        const int p4 = c0 + lane;
        if (p4 < tot4)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + p4),
                                           (__attribute__((address_space(3))) void*)(S + 4 * c0), 16, 0, STREAM ? 2 : 0);
      }
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
    if constexpr (POW2) {
      float4 quads[QPR];
#pragma unroll
      for (int q = 0; q < QPR; ++q)
        quads[q] = *reinterpret_cast<const float4*>(S + 4 * (tid * QPR + ((q + tid / ROT) & (QPR - 1))));
      if constexpr (NT == 16 || NT == 32) rfft_row_bins_r4<NT>(quads, mt, X);
      else rfft_row_bins<NT>(quads, mt, X);
    } else {
      // rows of NT floats start 8-byte aligned (NT even); 30 floats apart they spread over all banks
      float xr[NT];
#pragma unroll
      for (int n = 0; n < NT; n += 2) {
        const float2 v = *reinterpret_cast<const float2*>(S + tid * NT + n);
        xr[n] = v.x; xr[n + 1] = v.y;
      }
      rdft_row_bins_dense<NT>(xr, mt, X);
    }
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
    if constexpr (MTC > 0 && LZC > 0 && PZC >= 0 && NTHR > 0) {
      constexpr int PZ = 1 << PZC;
#pragma unroll
      for (int i0 = 0; i0 < LZC * MTC; i0 += NTHR) {
        const int idx = i0 + tid;
        if (i0 + NTHR <= LZC * MTC || idx < LZC * MTC) {
          const int jz = idx / MTC;
          const int kt = idx - jz * MTC;
          const int mj = posmod(kfreq(jz, LZC, NPC), MZ);
          const float2* base = T + (p * MTC + kt) * sT + (mj << PZC);
          const float2* w = TW + (jz << PZC);
          float2 wv[PZ], bv[PZ];
#pragma unroll
          for (int n2 = 0; n2 < PZ; ++n2) { wv[n2] = w[n2]; bv[n2] = base[n2]; }
          float2 acc = make_float2(0.f, 0.f);
#pragma unroll
          for (int n2 = 0; n2 < PZ; ++n2) acc = cfma(wv[n2], bv[n2], acc);
          st_once2<STREAM>(&dst[idx], acc);
        }
      }
    } else {
      for (int idx = tid; idx < Lz * mt; idx += nthr) {
        const int jz = (idx * inv_mt) >> 16;
        const int kt = idx - jz * mt;
        const int mj = posmod(kfreq(jz, Lz, nposz), MZ);
        const float2* base = T + (p * mt + kt) * sT + (mj << pzshift);
        const float2* w = TW + (jz << pzshift);
        float2 acc = make_float2(0.f, 0.f);
        for (int n2 = 0; n2 < Pz; ++n2) acc = cfma(w[n2], base[n2], acc);
        st_once2<STREAM>(&dst[idx], acc);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Complex pruned transform along the middle axis of [outer][N][inner] -> [outer][L][inner]
// ------------------------------------------------------------------------------------------
template <int M, bool STREAM>
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
      for (int n1 = 0; n1 < M; ++n1) a[n1] = ld_once2<STREAM>(&src[(long long)(P * n1) * inner]);
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
template <int M, bool STREAM>
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
      for (int n1 = 0; n1 < M; ++n1) st_once2<STREAM>(&dst[(long long)(P * n1) * inner], g[bitrev<M>(n1)]);
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

constexpr int kMixB = 4;   // batch entries held per pass (backward mix)

// One thread: one mode, KO output channels, KB batch entries per pass; R is read exactly once,
// the input spectrum once per group of KO output channels (launch: grid.y = ceil(Co / KO)).
template <int KB, int KO, bool STREAM>
__global__ __launch_bounds__(kThreads) void mix_fwd_kernel(
    const float2* __restrict__ xh, const float2* __restrict__ R, float2* __restrict__ yh, int B,
    int Ci, int Co, long long K, int mt, int Nt, float invN) {
  const long long k = (long long)blockIdx.x * kThreads + threadIdx.x;
  const int o0 = blockIdx.y * KO;
  if (k >= K) return;
  const float sc = mode_scale(k, mt, Nt, invN);
  for (int b0 = 0; b0 < B; b0 += KB) {
    float2 acc[KB][KO];
#pragma unroll
    for (int u = 0; u < KB; ++u)
#pragma unroll
      for (int v = 0; v < KO; ++v) acc[u][v] = make_float2(0.f, 0.f);
    for (int i = 0; i < Ci; ++i) {
      float2 xv[KB];
#pragma unroll
      for (int u = 0; u < KB; ++u)
        xv[u] = (b0 + u < B) ? xh[((long long)(b0 + u) * Ci + i) * K + k] : make_float2(0.f, 0.f);
#pragma unroll
      for (int v = 0; v < KO; ++v) {
        if (o0 + v < Co) {
          const float2 r = ld_once2<STREAM>(&R[((long long)i * Co + o0 + v) * K + k]);
#pragma unroll
          for (int u = 0; u < KB; ++u) acc[u][v] = cfma(xv[u], r, acc[u][v]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < KB; ++u)
#pragma unroll
      for (int v = 0; v < KO; ++v)
        if (b0 + u < B && o0 + v < Co)
          yh[((long long)(b0 + u) * Co + o0 + v) * K + k] = make_float2(acc[u][v].x * sc, acc[u][v].y * sc);
  }
}

// One thread: one mode k, kMixI input channels, the batch in chunks of kMixB; the gradient
// spectrum gh is then read once per kMixI input channels.
constexpr int kMixI = 4;
template <bool STREAM>
__global__ __launch_bounds__(kThreads) void mix_bwd_kernel(
    const float2* __restrict__ xh, const float2* __restrict__ R, const float2* __restrict__ gh,
    float2* __restrict__ gR, float2* __restrict__ gxh, int B, int Ci, int Co, long long K, int mt,
    int Nt, float invN, int accumulate) {
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
        r[v] = i0 + v < Ci ? ld_once2<STREAM>(&R[ridx]) : make_float2(0.f, 0.f);
        gr[v] = (gR != nullptr && (b0 > 0 || accumulate) && i0 + v < Ci) ? gR[ridx] : make_float2(0.f, 0.f);
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
          if (i0 + v < Ci) st_once2<STREAM>(&gR[((long long)(i0 + v) * Co + o) * K + k], gr[v]);
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

size_t tz_fwd_lds(AxisPlan az, int Nt, int mt, int ppb) {
  size_t s_floats = (size_t)ppb * az.N * (Nt + 1);
  s_floats += (s_floats & 1);
  return s_floats * 4 + (size_t)ppb * mt * tz_row_stride(az.N) * 8;
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

}  // namespace

bool tz_fwd_fits(AxisPlan az, int Nt, int mt) { return tz_fwd_lds(az, Nt, mt, 1) <= (size_t)kLdsBudget; }
bool axis_fits(AxisPlan ax) { return (size_t)ax.N * 8 <= (size_t)(32 * 1024); }

hipError_t launch_plan_tables(const TableSet& ts, hipStream_t s) {
  if (ts.n <= 0) return hipSuccess;
  int most = 1;
  for (int i = 0; i < ts.n; ++i) {
    const int n = ts.t[i].L > 0 ? ts.t[i].L * ts.t[i].P : ts.t[i].N * ts.t[i].npos;
    if (n > most) most = n;
  }
  hipLaunchKernelGGL(plan_tables_kernel, dim3((most + 255) / 256, ts.n), dim3(256), 0, s, ts);
  return hipGetLastError();
}

int tz_fast_region(AxisPlan az, int Nt, int mt, int ppb) {
  const int s_floats = ppb * az.N * Nt;
  const int t_floats = 2 * ppb * mt * tz_row_stride(az.N);
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
  // in-register t stage: the power-of-two lengths, and 30 (the time steps of the paper's training samples)
  // as plain sums with compile-time twiddles
  const bool pow2_t = Nt == 16 || Nt == 32 || Nt == 64;
  const bool fast = (pow2_t ? (az.N * Nt) % 256 == 0 : (Nt == 30 && (az.N * Nt) % 4 == 0 && mt <= 16)) &&
                    (az.M == 8 || az.M == 16) && (az.P & (az.P - 1)) == 0 && (az.L * az.P) % 2 == 0 &&
                    (int64_t)az.L * mt * mt < 65536 && az.N <= kThreads &&   // the kernel's multiply-shift division by mt is exact below that
                    ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(twz)) & 15) == 0 &&
                    tz_fast_lds(az, Nt, mt, 1) <= (size_t)kLdsBudget;
  if (fast) {
    int ppb = 1;
    // about 16 KB of input per block (one plane of 128 x 32, two of 128 x 16): the smaller LDS share
    // keeps more blocks resident, which hides the compute phases behind other blocks' loads a little
    // better than twice that, while smaller blocks than this lose to their fixed costs
    while (ppb * 2 * az.N <= 256 && ppb * 2 * az.N * Nt <= 4096 && tz_fast_lds(az, Nt, mt, ppb * 2) <= (size_t)kLdsBudget) ppb *= 2;
    const int thr = ((ppb * az.N + 63) / 64) * 64;
    const size_t lds = tz_fast_lds(az, Nt, mt, ppb);
    const int region = tz_fast_region(az, Nt, mt, ppb);
    const int64_t nblk = (((planes + ppb - 1) / ppb + 7) / 8) * 8;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    const int inv_mt = (65536 + mt - 1) / mt;
    const bool stream = planes * (int64_t)az.N * Nt * 4 >= kStreamBytes;
#define FNO_TZF_S(NTV, MZV, MTV, LZV, NPV, PZV, THRV, STRV)                                                   \
  hipLaunchKernelGGL((tz_fwd_fast_kernel<NTV, MZV, MTV, LZV, NPV, PZV, THRV, STRV>), dim3((unsigned)nblk),      \
                     dim3(thr), lds, s, x, out, twz, (long long)planes, az.N, az.L, az.npos, mt, ppb, region, \
                     ilog2(az.P), inv_mt)
#define FNO_TZF_C(NTV, MZV, MTV, LZV, NPV, PZV, THRV)                \
  do {                                                               \
    if (stream) FNO_TZF_S(NTV, MZV, MTV, LZV, NPV, PZV, THRV, true); \
    else FNO_TZF_S(NTV, MZV, MTV, LZV, NPV, PZV, THRV, false);       \
  } while (0)
#define FNO_TZF(NTV, MZV) FNO_TZF_C(NTV, MZV, 0, 0, 0, -1, 0)
#define FNO_TZF_M(NTV)                     \
  do {                                     \
    if (az.M == 8) FNO_TZF(NTV, 8);        \
    else FNO_TZF(NTV, 16);                 \
  } while (0)
    // the shapes of the named workloads as compile-time constants: 9 kept t bins with 32 kept z
    // frequencies in 8 residue classes (z of 128 points), or 9 / 8 t bins with 24 in 4 classes (64)
    const bool z128 = az.M == 16 && az.P == 8 && az.L == 32 && az.npos == 16 && mt == 9;
    const bool z64 = az.M == 16 && az.P == 4 && az.L == 24 && az.npos == 12;
    if (Nt == 32 && z128 && thr == 128) FNO_TZF_C(32, 16, 9, 32, 16, 3, 128);
    else if (Nt == 16 && z128 && thr == 256) FNO_TZF_C(16, 16, 9, 32, 16, 3, 256);
    else if (Nt == 32 && z64 && mt == 9 && thr == 128) FNO_TZF_C(32, 16, 9, 24, 12, 2, 128);
    else if (Nt == 16 && z64 && mt == 8 && thr == 256) FNO_TZF_C(16, 16, 8, 24, 12, 2, 256);
    else if (Nt == 16) FNO_TZF_M(16); else if (Nt == 32) FNO_TZF_M(32); else if (Nt == 64) FNO_TZF_M(64);
    else FNO_TZF_M(30);
#undef FNO_TZF_M
#undef FNO_TZF
#undef FNO_TZF_C
#undef FNO_TZF_S
    return hipGetLastError();
  }
  if (az.M == 1 && Nt % 4 == 0 && mt <= 16 && (reinterpret_cast<uintptr_t>(x) & 15) == 0) {
    const int ppb = 16 / mt;
    const size_t t_bytes = (size_t)16 * tzd_row_stride(az.N) * 8;
    const size_t p_bytes = (size_t)(kThreads / 64) * kDenseMT * 16 * 16 * 8;
    const int alias = az.L <= kDenseMT * 16;      // one sweep: the partial sums reuse the rows' LDS
    const size_t lds = alias ? (t_bytes > p_bytes ? t_bytes : p_bytes) : t_bytes + p_bytes;
    const int64_t nblk = (((planes + ppb - 1) / ppb + 7) / 8) * 8;
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
  const int64_t nblk = (((planes + ppb - 1) / ppb + 7) / 8) * 8;
  if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
  FNO_DISPATCH_M(az.M, hipLaunchKernelGGL((tz_fwd_kernel<MM>), dim3((unsigned)nblk), dim3(kThreads),
                                          lds, s, x, out, twt, twz, (long long)planes, az.N, Nt,
                                          az.L, az.npos, mt, ppb));
  return hipGetLastError();
}

hipError_t launch_axis_fwd(const float2* in, float2* out, const float2* tw, int64_t outer,
                           AxisPlan ax, int64_t inner, hipStream_t s) {
  if (outer <= 0 || inner <= 0) return hipSuccess;
  // the widest column tile the 32 KiB cap allows, up to 64 columns (16 for 256-point axes, 32 for
  // 128, 64 below): more threads share the first, FFT phase, whose items are P x W
  const int W = axis_cols(ax, inner, ax.N, 64);
  const int64_t ncb = (inner + W - 1) / W;
  const int64_t nblk = outer * ncb;
  if (nblk > 0x7fffffffLL || ncb > 0x7fffffffLL) return hipErrorInvalidValue;
  // the twiddles go to LDS only when that does not cost a resident block
  const int tw_lds = (size_t)ax.L * ax.P * 8 <= (size_t)(8 * 1024) && (size_t)ax.N * W * 8 <= (size_t)(16 * 1024);
  const size_t lds = (size_t)ax.N * W * 8 + (tw_lds ? (size_t)ax.L * ax.P * 8 : 0);
  // the input is read once: as a stream when it is larger than the caches
  if (outer * ax.N * inner * 8 >= kStreamBytes) {
    FNO_DISPATCH_M(ax.M, hipLaunchKernelGGL((axis_fwd_kernel<MM, true>), dim3((unsigned)nblk),
                                            dim3(kThreads), lds, s, in, out, tw, ax.N, ax.L, ax.npos,
                                            (long long)inner, W, (int)ncb, tw_lds));
  } else {
    FNO_DISPATCH_M(ax.M, hipLaunchKernelGGL((axis_fwd_kernel<MM, false>), dim3((unsigned)nblk),
                                            dim3(kThreads), lds, s, in, out, tw, ax.N, ax.L, ax.npos,
                                            (long long)inner, W, (int)ncb, tw_lds));
  }
  return hipGetLastError();
}

hipError_t launch_axis_inv(const float2* in, float2* out, const float2* tw, int64_t outer,
                           AxisPlan ax, int64_t inner, hipStream_t s) {
  if (outer <= 0 || inner <= 0) return hipSuccess;
  const int W = axis_cols(ax, inner, ax.L, 32);          // 16 and 64 columns both measured slower
  const int64_t ncb = (inner + W - 1) / W;
  const int64_t nblk = outer * ncb;
  if (nblk > 0x7fffffffLL || ncb > 0x7fffffffLL) return hipErrorInvalidValue;
  const int tw_lds = (size_t)ax.L * ax.P * 8 <= (size_t)(8 * 1024);
  const size_t lds = (size_t)ax.L * W * 8 + (tw_lds ? (size_t)ax.L * ax.P * 8 : 0);
  const int thr = axis_threads(ax.P * W);
  // the output is written once: as a stream when it is larger than the caches
  if (outer * ax.N * inner * 8 >= kStreamBytes) {
    FNO_DISPATCH_M(ax.M, hipLaunchKernelGGL((axis_inv_kernel<MM, true>), dim3((unsigned)nblk),
                                            dim3(thr), lds, s, in, out, tw, ax.N, ax.L, ax.npos,
                                            (long long)inner, W, (int)ncb, tw_lds));
  } else {
    FNO_DISPATCH_M(ax.M, hipLaunchKernelGGL((axis_inv_kernel<MM, false>), dim3((unsigned)nblk),
                                            dim3(thr), lds, s, in, out, tw, ax.N, ax.L, ax.npos,
                                            (long long)inner, W, (int)ncb, tw_lds));
  }
  return hipGetLastError();
}

hipError_t launch_mix_fwd(const float2* xh, const float2* R, float2* yh, int B, int Ci, int Co,
                          int64_t K, int mt, int Nt, double invN, hipStream_t s) {
  const int64_t nb = (K + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || Co > 65535) return hipErrorInvalidValue;
  // four output channels and up to four batch entries per thread (a tile of one or two entries for
  // batches that small: 3 % faster than four with unused rows); wider output tiles (10 or 20
  // channels for a single batch entry, which would read the input spectrum less often) measured slower.
  // R is read once per call: as a stream when it is larger than the caches
  const bool stream = (int64_t)Ci * Co * K * 8 >= kStreamBytes;
#define FNO_MIX(KBV, STRV)                                                                                  \
  hipLaunchKernelGGL((mix_fwd_kernel<KBV, 4, STRV>), dim3((unsigned)nb, (unsigned)((Co + 3) / 4)), dim3(kThreads), \
                     0, s, xh, R, yh, B, Ci, Co, (long long)K, mt, Nt, (float)invN)
#define FNO_MIX_B(STRV)                                                                      \
  do {                                                                                       \
    if (B == 1) FNO_MIX(1, STRV); else if (B == 2) FNO_MIX(2, STRV); else FNO_MIX(4, STRV);  \
  } while (0)
  if (stream) FNO_MIX_B(true); else FNO_MIX_B(false);
#undef FNO_MIX_B
#undef FNO_MIX
  return hipGetLastError();
}

hipError_t launch_mix_bwd(const float2* xh, const float2* R, const float2* gh, float2* gR,
                          float2* gxh, int B, int Ci, int Co, int64_t K, int mt, int Nt,
                          double invN, int accumulate, hipStream_t s) {
  const int64_t nb = (K + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || Ci > 4 * 65535) return hipErrorInvalidValue;
  if ((int64_t)Ci * Co * K * 8 >= kStreamBytes)
    hipLaunchKernelGGL(mix_bwd_kernel<true>, dim3((unsigned)nb, (unsigned)((Ci + kMixI - 1) / kMixI)), dim3(kThreads), 0,
                       s, xh, R, gh, gR, gxh, B, Ci, Co, (long long)K, mt, Nt, (float)invN, accumulate);
  else
    hipLaunchKernelGGL(mix_bwd_kernel<false>, dim3((unsigned)nb, (unsigned)((Ci + kMixI - 1) / kMixI)), dim3(kThreads), 0,
                       s, xh, R, gh, gR, gxh, B, Ci, Co, (long long)K, mt, Nt, (float)invN, accumulate);
  return hipGetLastError();
}

}  // namespace fno
