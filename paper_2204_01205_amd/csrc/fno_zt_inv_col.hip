// Inverse (z, t) + block epilogue, column variant on the matrix cores (see fno_zt_inv.hip for
// what the stage computes and fno_zt_inv_mfma.hip for the lane layout of the 4x4x1 MFMA blocks).
#include "fno_zt_inv.h"
#include <type_traits>

namespace fno {

namespace {

// Column variant of the matrix-core inverse kernel for NT = 32, MZ = 16: one block of eight waves
// owns a whole (b,nx,ny) column, stages the column's spectrum once and walks the residue classes
// of z two at a time (a tile of 32 rows x 32 t per step, Pz / 2 steps).  The spectrum A stays in
// LDS for all steps; V holds one residue class (16 rows) at a time, so a step is two half steps
// (z stage, t stage, W part, epilogue), one per slot of u registers.  Slot s of lane block (wave, blk) is the quad
// blk % 8 of row z = Pz (2 wave + blk / 8) + 2 step + s.  Launch: grid (NxNy, B), 512 threads.
// The table blob is the one of zt_tables_kernel with Q = Pz (all twiddles, [Pz][Lz]).
// MTC, LZC, NPC: the kept counts on t and z (and how many of the latter are non-negative
// frequencies) as compile-time constants (0: taken from the arguments), so
// that the loops over them unroll; EPI >= 0 fixes the epilogue at compile time (bit 0: GELU, bit 1:
// the pre-activation is stored as well), EPI = -1 reads it from the arguments.  With a fixed
// epilogue every half step issues the same number of loads and stores on every path, which the
// compiler's wait counts for the prefetched u values rely on.
template <int CT, bool FULL, int MTC, int LZC, int NPC, int EPI, bool STREAM>
__global__ __launch_bounds__(512, 4) void zt_inv_col_kernel(
    const float2* __restrict__ a, float* __restrict__ out, int Co_rt, int NxNy, int Nz, int Lz_rt,
    int nposz_rt, int mt_rt, int inv_mt, int a_floats, int a_stride4, int v_stride,
    const float* __restrict__ blob, int blob_floats, EpiArgs ep) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int mt = MTC ? MTC : mt_rt;
  const int Lz = LZC ? LZC : Lz_rt;
  const int nposz = LZC ? NPC : nposz_rt;      // first nposz stored frequencies are 0..nposz-1, the rest negative
  const bool act = EPI >= 0 ? (EPI & 1) != 0 : ep.act != 0;
  const bool zsave = EPI >= 0 ? (EPI & 2) != 0 : ep.zsave != nullptr;
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
  const bool lin = EPI >= 0 ? true : ep.u != nullptr;      // a fixed epilogue always has the linear term
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
        if (FULL || i < Cu) xv[i][sl] = ld_once<STREAM>(&ubase[i * Npts + sl * NT]);
  }
  asm volatile("" ::: "memory");
  // everything issued so far has landed (the first u values too: the bias step below reads LDS that
  // the LDS-direct loads write, and the compiler drains every load before such a read anyway)
  __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  __syncthreads();
  // The bias rides on the spectrum: adding b[o] to the entry (kz = 0, kt = 0) of channel o (stored
  // first: j = 0, kt = 0) adds b[o] to every point of the channel (that entry's z twiddle and its
  // cos row are 1), so the accumulators below start from zero.
  if (tid < Co) smem[tid * (4 * a_stride4)] += BI[tid];
  __syncthreads();

  const int nsteps = Pz >> 1;
  // One step = two half steps.  PREFETCH: the step also loads the u values of the next step.  The
  // last step of a column has no next step; it runs as a copy of the body without those loads, so
  // that inside the loop every half step issues the same number of loads on every path and the
  // compiler can count how many later memory operations may still be in flight when a u value is used.
  auto run_step = [&](const int step, auto prefetch_tag) {
    constexpr bool PREFETCH = decltype(prefetch_tag)::value;
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
        if ((Lz & (MZ - 1)) == 0) {
#pragma unroll
          for (int m = 0; m < MZ; ++m) gres[m] = make_float2(0.f, 0.f);
#pragma unroll
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
          for (int m = 0; m < MZ; ++m) gres[m] = make_float2(0.f, 0.f);
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
      for (int T = 0; T < CT; ++T) acc[T] = v4f{0.f, 0.f, 0.f, 0.f};
      const float* cs_lane = CS + 4 * quad + j4;
      const float2* v0 = V + j4 * v_stride + n1 * mt;
      int kt = 0;
      constexpr int KB = 3;                       // kt per pass: their reads go out together
#pragma unroll 1
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
#pragma unroll
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
        if constexpr (PREFETCH) {
#pragma unroll
          for (int i = 0; i < CI; ++i)
            if (FULL || i < Cu) xv[i][sl] = ld_once<STREAM>(&ubase[i * Npts + (n2 + 2) * NT]);
        }
        asm volatile("" ::: "memory");
      }
      // lane 4b+j now holds channel 4T+j at the four t of its quad
      float* op = out + (b * Co + j4) * Npts + poff;
      if (zsave) {
        float* zp = ep.zsave + (b * Co + j4) * Npts + poff;
#pragma unroll
        for (int T = 0; T < CT; ++T)
          if (FULL || 4 * T + j4 < Co)
            st_once<STREAM>(reinterpret_cast<v4f*>(zp + (4 * T) * Npts), acc[T]);
      }
      if (act) {
#pragma unroll
        for (int T = 0; T < CT; ++T)
          if (FULL || 4 * T + j4 < Co)
            st_once<STREAM>(reinterpret_cast<v4f*>(op + (4 * T) * Npts),
                            v4f{gelu_fast_f(acc[T][0]), gelu_fast_f(acc[T][1]), gelu_fast_f(acc[T][2]),
                                gelu_fast_f(acc[T][3])});
      } else {
#pragma unroll
        for (int T = 0; T < CT; ++T)
          if (FULL || 4 * T + j4 < Co)
            st_once<STREAM>(reinterpret_cast<v4f*>(op + (4 * T) * Npts), acc[T]);
      }
    }
  };
  for (int step = 0; step + 1 < nsteps; ++step) run_step(step, std::true_type{});
  run_step(nsteps - 1, std::false_type{});
}

}  // namespace

hipError_t launch_zt_inv_col(const float2* a, float* out, const float2* twt, const float2* twz, int B, int Co,
                             int NxNy, AxisPlan az, int Nt, int mt, EpiArgs ep, float* tables, hipStream_t s,
                             bool* taken) {
  *taken = false;
  const EpiArgs& e = ep;
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  // Column kernel (Nt = 32, 16-point z FFT): the spectrum of a column is staged once instead of
  // once per tile.  Taken when two blocks fit a CU's LDS, else the per-tile kernel below.
  if (Nt == 32 && az.M == 16 && az.P >= 2 && az.P % 2 == 0 &&
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
      hipError_t terr = launch_zt_tables(tables, 1, twt, twz, ep.u ? ep.W : nullptr, ep.w_so, ep.w_si, ep.bias, Co,
                                         Cu, 4 * CT, mt, Nt, Nt, az.L, az.P, az.P, blob_floats, s);
      if (terr != hipSuccess) return terr;
      const dim3 grid((unsigned)NxNy, (unsigned)B);
#define FNO_ZTC_S(CTV, FULLV, MTV, LZV, NPV, EPIV, STRV)                                                     \
  hipLaunchKernelGGL((zt_inv_col_kernel<CTV, FULLV, MTV, LZV, NPV, EPIV, STRV>), grid, dim3(512), lds, s, a, out, \
                     Co, NxNy, az.N, az.L, az.npos, mt, inv_mt, a_floats, a_stride4, v_stride, tables,       \
                     blob_floats, e)
      // u is read once and the results are written once: as streams when they are larger than the caches
      const bool stream = (int64_t)B * Co * NxNy * az.N * Nt * 4 >= kStreamBytes;
#define FNO_ZTC(CTV, FULLV, MTV, LZV, NPV, EPIV)                  \
  do {                                                            \
    if (stream) FNO_ZTC_S(CTV, FULLV, MTV, LZV, NPV, EPIV, true); \
    else FNO_ZTC_S(CTV, FULLV, MTV, LZV, NPV, EPIV, false);       \
  } while (0)
      // the shape of the large workloads (width 20, 9 kept t bins, 32 kept z frequencies) with its three
      // epilogues: forward, forward that keeps the pre-activation, and the adjoint's linear one
      const int epi = (e.act ? 1 : 0) | (e.zsave != nullptr ? 2 : 0);
      if (CT == 5 && full && mt == 9 && az.L == 32 && az.npos == 16 && e.u != nullptr && epi != 2) {
        if (epi == 1) FNO_ZTC(5, true, 9, 32, 16, 1);
        else if (epi == 3) FNO_ZTC(5, true, 9, 32, 16, 3);
        else FNO_ZTC(5, true, 9, 32, 16, 0);
      } else if (CT == 5 && full && mt == 9 && az.L == 24 && az.npos == 12 && e.u != nullptr && epi != 2) {
        if (epi == 1) FNO_ZTC(5, true, 9, 24, 12, 1);
        else if (epi == 3) FNO_ZTC(5, true, 9, 24, 12, 3);
        else FNO_ZTC(5, true, 9, 24, 12, 0);
      } else if (CT == 2) { if (full) FNO_ZTC(2, true, 0, 0, 0, -1); else FNO_ZTC(2, false, 0, 0, 0, -1); }
      else { if (full) FNO_ZTC(5, true, 0, 0, 0, -1); else FNO_ZTC(5, false, 0, 0, 0, -1); }
#undef FNO_ZTC
#undef FNO_ZTC_S
      *taken = true;
      return hipGetLastError();
    }
  }
  return hipSuccess;
}

}  // namespace fno
