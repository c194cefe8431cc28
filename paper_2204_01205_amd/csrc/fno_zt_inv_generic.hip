// Inverse (z, t) + block epilogue, generic kernel: any axis lengths and channel counts up to 32
// (see fno_zt_inv.hip for what the stage computes).  One block: all output channels of one
// (b,nx,ny) column, for the z rows of Q consecutive residue classes (z = Pz*n1 + n2).
#include "fno_zt_inv.h"

namespace fno {

namespace {

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

}  // namespace

hipError_t launch_zt_inv_generic(const float2* a, float* out, const float2* twt, const float2* twz, int64_t ncols,
                                 int Co, int NxNy, AxisPlan az, int Nt, int mt, EpiArgs e, hipStream_t s) {
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

}  // namespace fno
