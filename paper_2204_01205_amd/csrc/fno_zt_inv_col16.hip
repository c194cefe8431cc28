// Inverse (z, t) + block epilogue, column variant on the matrix cores for a t axis of 16 points
// (see fno_zt_inv.hip for what the stage computes, fno_zt_inv_mfma.hip for the lane layout of the
// 4x4x1 MFMA blocks and fno_zt_inv_col.hip for the 32-point column variant this one follows).
#include "fno_zt_inv.h"
#include <type_traits>

namespace fno {

namespace {

// One block of eight waves owns a whole (b,nx,ny) column and keeps the column's spectrum A in LDS.
// With NT = 16 a wave's 16 MFMA blocks are four rows of four quads, so the eight waves cover 32
// rows: two residue classes of z (a "pair") at a time.  V for two classes of all channels would
// not leave room for two blocks per CU, so a pair is worked in passes over the channel tiles (three
// tiles, then two, for five tiles): z stage of the pass's channels for both classes, t stage, W
// part and epilogue of those channels.  The u values of a pair serve all its passes and are
// loaded one step (two pairs, one per register set) ahead.
// Lane block (wave, blk): quad blk % 4, class (blk / 4) % 2 of the pair, n1 = 2 wave + blk / 8,
// z = Pz n1 + 2 pair + class.  Launch: grid (NxNy, B), 512 threads; Pz a multiple of 4.
// The table blob is the one of zt_tables_kernel with Q = Pz.  MTC, LZC, NPC, EPI as in the
// 32-point variant.
template <int CT, bool FULL, int MTC, int LZC, int NPC, int EPI, bool STREAM>
__global__ __launch_bounds__(512, 4) void zt_inv_col16_kernel(
    const float2* __restrict__ a, float* __restrict__ out, int Co_rt, int NxNy, int Nz, int Lz_rt,
    int nposz_rt, int mt_rt, int inv_mt, int a_floats, int a_stride4, int v_stride,
    const float* __restrict__ blob, int blob_floats, EpiArgs ep) {
  HIP_DYNAMIC_SHARED(float, smem)
  const int mt = MTC ? MTC : mt_rt;
  const int Lz = LZC ? LZC : Lz_rt;
  const int nposz = LZC ? NPC : nposz_rt;
  const bool act = EPI >= 0 ? (EPI & 1) != 0 : ep.act != 0;
  const bool zsave = EPI >= 0 ? (EPI & 2) != 0 : ep.zsave != nullptr;
  constexpr int NT = 16, MZ = 16, NW = 8;
  constexpr int CP = 4 * CT;
  constexpr int CI = CP;
  constexpr int TS = CT == 5 ? 3 : CT;              // channel tiles per pass
  constexpr int NSUB = (CT + TS - 1) / TS;          // passes per pair
  constexpr int nthr = 64 * NW;
  constexpr int ZB = 4;                             // z-stage terms whose LDS reads go out together
  const int Co = FULL ? CP : Co_rt;
  const int Cu = FULL ? CI : ep.Cu;
  const int Pz = Nz / MZ;
  const float2* A = reinterpret_cast<const float2*>(smem);      // [Co][Lz][mt], padded channel stride
  float2* V = reinterpret_cast<float2*>(smem + a_floats);       // [4 TS][2 MZ][mt], padded channel stride
  float* CS = smem + a_floats + 2 * (4 * TS) * v_stride;        // [2 mt][NT]: cos rows and -sin rows
  float* Wt = CS + 2 * mt * NT;                                 // [Cu][CP]
  const bool lin = EPI >= 0 ? true : ep.u != nullptr;
  const float2* TW = reinterpret_cast<const float2*>(Wt + (lin ? Cu * CP : 0));   // [Pz][Lz]
  const int tid = threadIdx.x;
  const int xy = blockIdx.x;
  const long long b = blockIdx.y;
  const int lane = tid & 63, wave = tid >> 6;
  const int j4 = lane & 3;
  const int blk = lane >> 2;
  const int quad = blk & 3;
  // a wave takes both classes of two n1: its rows z = Pz n1 + 2 pair + {0, 1} are adjacent in
  // memory, so each of its loads and stores covers whole 128-byte lines
  const int cls = (blk >> 2) & 1, n1 = 2 * wave + (blk >> 3);
  const int row = cls * MZ + n1;              // row of this lane block in V
  const long long Npts = (long long)NxNy * Nz * NT;
  const long long pbase = ((long long)xy * Nz + Pz * n1 + cls) * NT + 4 * quad;   // + 2 pair * NT
  const int kmin = nposz - Lz, kmax = nposz - 1;
  const int mbase = posmod(-kmin, MZ);

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
  if (!FULL) {
    // channel slots of V that no z stage writes feed unused MFMA columns: give them finite values
    for (int idx = tid; idx < 4 * TS * v_stride; idx += nthr) V[idx] = make_float2(0.f, 0.f);
  }
  const float* BI = reinterpret_cast<const float*>(TW + Pz * Lz);      // bias, padded to CP
  // u values of a pair (lane 4b+i takes t = 4 quad + i), two register sets: even and odd pairs
  float xv[CI][2];
  const float* ubase = lin ? ep.u + (b * Cu) * Npts + j4 + pbase : nullptr;
  asm volatile("" ::: "memory");    // keep the issue order: tables, spectrum, u
  if (lin) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl)
#pragma unroll
      for (int i = 0; i < CI; ++i)
        if (FULL || i < Cu) xv[i][sl] = ld_once<STREAM>(&ubase[i * Npts + (2 * sl) * NT]);
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
  __syncthreads();
  // the bias rides on the spectrum entry (kz = 0, kt = 0) of every channel
  if (tid < Co) smem[tid * (4 * a_stride4)] += BI[tid];
  __syncthreads();

  const int nsteps = Pz >> 2;                  // two pairs per step
  auto run_pass = [&](const int pair, const int sl, auto sub_tag, auto prefetch_tag) {
    constexpr int SUB = decltype(sub_tag)::value;
    constexpr bool PREFETCH = decltype(prefetch_tag)::value;
    constexpr int T0 = SUB * TS;                                    // first channel tile of the pass
    constexpr int NTL = (SUB == NSUB - 1) ? CT - T0 : TS;           // its channel tiles
    const int nch = FULL ? 4 * NTL : min(4 * NTL, Co - 4 * T0);     // channels that exist in the pass
    // z stage: item (class, channel, kt) collects the kept z-frequencies with their twiddles into
    // MZ bins; an inverse FFT over n1 gives the rows z = Pz n1 + 2 pair + class
    {
      const int per_cls = nch * mt;
      if (tid < 2 * per_cls) {
        const int zc = tid >= per_cls ? 1 : 0;
        const int rem = tid - zc * per_cls;
        const int zo = (rem * inv_mt) >> 16;
        const int zkt = rem - zo * mt;
        const float2* asrc = A + (4 * T0 + zo) * (2 * a_stride4) + zkt;
        float2* vdst = V + zo * v_stride + (zc * MZ) * mt + zkt;
        const float2* twq = TW + (2 * pair + zc) * Lz;
        float2 gres[MZ];
#pragma unroll
        for (int m = 0; m < MZ; ++m) gres[m] = make_float2(0.f, 0.f);
        if constexpr (LZC > 0) {
          // compile-time counts: the stored order j in rounds of ZB, each term to its bin k_j mod MZ
#pragma unroll
          for (int j0 = 0; j0 < LZC; j0 += ZB) {
            float2 av[ZB], wv8[ZB];
#pragma unroll
            for (int u = 0; u < ZB; ++u)
              if (j0 + u < LZC) {
                av[u] = asrc[(j0 + u) * mt];
                wv8[u] = twq[j0 + u];
              }
#pragma unroll
            for (int u = 0; u < ZB; ++u)
              if (j0 + u < LZC) {
                const int k = j0 + u < NPC ? j0 + u : j0 + u - LZC;
                const int m = ((k % MZ) + MZ) % MZ;
                gres[m] = cfmac(av[u], wv8[u], gres[m]);
              }
          }
        } else if ((Lz & (MZ - 1)) == 0) {
#pragma unroll
          for (int r0 = 0; r0 < Lz; r0 += MZ) {
            const float2* ar = asrc + r0 * mt;
            const float2* tr = twq + r0;
#pragma unroll
            for (int mb = 0; mb < MZ; mb += ZB) {
              float2 av[ZB], wv8[ZB];
#pragma unroll
              for (int u = 0; u < ZB; ++u) {
                av[u] = ar[(mb + u) * mt];
                wv8[u] = tr[mb + u];
              }
#pragma unroll
              for (int u = 0; u < ZB; ++u) gres[mb + u] = cfmac(av[u], wv8[u], gres[mb + u]);
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
    }
    __syncthreads();
    // t stage: complex-to-real step over kt on the matrix cores
    v4f acc[NTL];
#pragma unroll
    for (int T = 0; T < NTL; ++T) acc[T] = v4f{0.f, 0.f, 0.f, 0.f};
    const float* cs_lane = CS + 4 * quad + j4;
    const float2* v0 = V + j4 * v_stride + row * mt;
    int kt = 0;
    constexpr int KB = (MTC > 0 && MTC % 4 == 0) ? 4 : 3;   // kt per round: their reads go out together
#pragma unroll 1
    for (; kt + KB <= mt; kt += KB) {
      float cs4[2 * KB];
      float2 va[KB][NTL];
#pragma unroll
      for (int h = 0; h < KB; ++h) {
        cs4[2 * h] = cs_lane[(2 * (kt + h)) * NT];
        cs4[2 * h + 1] = cs_lane[(2 * (kt + h) + 1) * NT];
#pragma unroll
        for (int T = 0; T < NTL; ++T) va[h][T] = v0[4 * T * v_stride + kt + h];
      }
#pragma unroll
      for (int h = 0; h < KB; ++h)
#pragma unroll
        for (int T = 0; T < NTL; ++T) {
          acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(cs4[2 * h], va[h][T].x, acc[T], 0, 0, 0);
          acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(cs4[2 * h + 1], va[h][T].y, acc[T], 0, 0, 0);
        }
    }
#pragma unroll
    for (; kt < mt; ++kt) {
      const float c = cs_lane[(2 * kt) * NT];
      const float sn = cs_lane[(2 * kt + 1) * NT];
      float2 va[NTL];
#pragma unroll
      for (int T = 0; T < NTL; ++T) va[T] = v0[4 * T * v_stride + kt];
#pragma unroll
      for (int T = 0; T < NTL; ++T) {
        acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(c, va[T].x, acc[T], 0, 0, 0);
        acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(sn, va[T].y, acc[T], 0, 0, 0);
      }
    }
    __syncthreads();      // V is rewritten by the next z stage
    if (lin) {
      constexpr int IB = 4;                       // input channels per batch of LDS reads
#pragma unroll
      for (int i0 = 0; i0 < CI; i0 += IB) {
        float wv[IB][NTL];
#pragma unroll
        for (int ii = 0; ii < IB; ++ii)
#pragma unroll
          for (int T = 0; T < NTL; ++T)
            wv[ii][T] = (FULL || i0 + ii < Cu) ? Wt[(i0 + ii) * CP + 4 * (T0 + T) + j4] : 0.f;
#pragma unroll
        for (int ii = 0; ii < IB; ++ii) {
          if (FULL || i0 + ii < Cu) {
#pragma unroll
            for (int T = 0; T < NTL; ++T)
              acc[T] = __builtin_amdgcn_mfma_f32_4x4x1f32(xv[i0 + ii][sl], wv[ii][T], acc[T], 0, 0, 0);
          }
        }
      }
      if constexpr (SUB == NSUB - 1) {
        // the pair's last pass has used this register set: refill it for the pair two ahead
        asm volatile("" ::: "memory");
        if constexpr (PREFETCH) {
#pragma unroll
          for (int i = 0; i < CI; ++i)
            if (FULL || i < Cu) xv[i][sl] = ld_once<STREAM>(&ubase[i * Npts + (2 * (pair + 2)) * NT]);
        }
        asm volatile("" ::: "memory");
      }
    }
    // lane 4b+j now holds channel 4(T0+T)+j at the four t of its quad
    const long long poff = pbase + (long long)(2 * pair) * NT;
    float* op = out + (b * Co + 4 * T0 + j4) * Npts + poff;
    if (zsave) {
      float* zp = ep.zsave + (b * Co + 4 * T0 + j4) * Npts + poff;
#pragma unroll
      for (int T = 0; T < NTL; ++T)
        if (FULL || 4 * (T0 + T) + j4 < Co)
          st_once<STREAM>(reinterpret_cast<v4f*>(zp + (4 * T) * Npts), acc[T]);
    }
    if (act) {
#pragma unroll
      for (int T = 0; T < NTL; ++T)
        if (FULL || 4 * (T0 + T) + j4 < Co)
          st_once<STREAM>(reinterpret_cast<v4f*>(op + (4 * T) * Npts),
                          v4f{gelu_fast_f(acc[T][0]), gelu_fast_f(acc[T][1]), gelu_fast_f(acc[T][2]),
                              gelu_fast_f(acc[T][3])});
    } else {
#pragma unroll
      for (int T = 0; T < NTL; ++T)
        if (FULL || 4 * (T0 + T) + j4 < Co)
          st_once<STREAM>(reinterpret_cast<v4f*>(op + (4 * T) * Npts), acc[T]);
    }
  };
  // One step = two pairs, one per register set.  The last step of a column has no next step; it
  // runs as a copy of the body without the u loads, so that inside the loop every pass issues the
  // same number of loads on every path.
  auto run_step = [&](const int step, auto prefetch_tag) {
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {
      const int pair = 2 * step + sl;
      run_pass(pair, sl, std::integral_constant<int, 0>{}, prefetch_tag);
      if constexpr (NSUB > 1) run_pass(pair, sl, std::integral_constant<int, 1>{}, prefetch_tag);
    }
  };
  for (int step = 0; step + 1 < nsteps; ++step) run_step(step, std::true_type{});
  run_step(nsteps - 1, std::false_type{});
}

}  // namespace

hipError_t launch_zt_inv_col16(const float2* a, float* out, const float2* twt, const float2* twz, int B, int Co,
                               int NxNy, AxisPlan az, int Nt, int mt, EpiArgs ep, float* tables, hipStream_t s,
                               bool* taken) {
  *taken = false;
  const EpiArgs& e = ep;
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  if (Nt != 16 || az.M != 16 || az.P < 4 || az.P % 4 != 0 || (az.P & (az.P - 1)) != 0 || CT > 5 ||
      (az.L * mt) % 2 != 0 || B > 65535)
    return hipSuccess;
  const int TS = CT == 5 ? 3 : CT;
  if (2 * 4 * TS * mt > 512) return hipSuccess;         // one z-stage item per thread
  const int Cu = ep.u ? ep.Cu : 0;
  const int a_stride4 = zt_mfma_astride4(az, mt);
  const int a_floats = (Co * a_stride4 * 4 + 255) & ~255;
  const int v_stride = zt_mfma_vstride(az, mt, 2);
  const int blob_floats = zt_mfma_blob(az, Nt, mt, Co, Cu, az.P);
  const size_t lds = ((size_t)a_floats + 2 * 4 * TS * v_stride + blob_floats) * 4;
  // two blocks per CU
  if (Cu > 4 * CT || lds > (size_t)(80 * 1024 - 512) || (size_t)blob_floats * 4 > kZtTablesBytes) return hipSuccess;
  const bool full = (Co == 4 * CT) && (ep.u == nullptr || ep.Cu == 4 * CT);
  const int inv_mt = (65536 + mt - 1) / mt;
  // the shapes of the named workloads (width 20; 9 kept t bins and 32 kept z frequencies, or 8 and 24)
  // with their three epilogues: forward, forward that keeps the pre-activation, the adjoint's linear one
  const int epi = (e.act ? 1 : 0) | (e.zsave != nullptr ? 2 : 0);
  const bool named = CT == 5 && full && e.u != nullptr && epi != 2;
  const bool shape_a = named && mt == 9 && az.L == 32 && az.npos == 16;
  const bool shape_b = named && mt == 8 && az.L == 24 && az.npos == 12;
  // other widths above 8, with run-time counts, do not fit the register budget of two blocks per
  // CU: the per-tile kernel takes them
  if (!(shape_a || shape_b || CT == 2)) return hipSuccess;
  hipError_t terr = launch_zt_tables(tables, 1, twt, twz, ep.u ? ep.W : nullptr, ep.w_so, ep.w_si, ep.bias, Co,
                                     Cu, 4 * CT, mt, Nt, Nt, az.L, az.P, az.P, blob_floats, s);
  if (terr != hipSuccess) return terr;
  const dim3 grid((unsigned)NxNy, (unsigned)B);
#define FNO_ZTC16_S(CTV, FULLV, MTV, LZV, NPV, EPIV, STRV)                                                     \
  hipLaunchKernelGGL((zt_inv_col16_kernel<CTV, FULLV, MTV, LZV, NPV, EPIV, STRV>), grid, dim3(512), lds, s, a,   \
                     out, Co, NxNy, az.N, az.L, az.npos, mt, inv_mt, a_floats, a_stride4, v_stride, tables,  \
                     blob_floats, e)
  // u and the result as streams when they are larger than the caches, except in the launch that also
  // stores the pre-activation: with three streams per point it measured 4 % slower with the hint,
  // the other two epilogues 2-5 % faster
  const bool stream = e.zsave == nullptr && (int64_t)B * Co * NxNy * az.N * Nt * 4 >= kStreamBytes;
#define FNO_ZTC16(CTV, FULLV, MTV, LZV, NPV, EPIV)                  \
  do {                                                              \
    if (stream) FNO_ZTC16_S(CTV, FULLV, MTV, LZV, NPV, EPIV, true); \
    else FNO_ZTC16_S(CTV, FULLV, MTV, LZV, NPV, EPIV, false);       \
  } while (0)
  if (shape_a) {
    if (epi == 1) FNO_ZTC16(5, true, 9, 32, 16, 1);
    else if (epi == 3) FNO_ZTC16(5, true, 9, 32, 16, 3);
    else FNO_ZTC16(5, true, 9, 32, 16, 0);
  } else if (shape_b) {
    if (epi == 1) FNO_ZTC16(5, true, 8, 24, 12, 1);
    else if (epi == 3) FNO_ZTC16(5, true, 8, 24, 12, 3);
    else FNO_ZTC16(5, true, 8, 24, 12, 0);
  } else {
    if (full) FNO_ZTC16(2, true, 0, 0, 0, -1); else FNO_ZTC16(2, false, 0, 0, 0, -1);
  }
#undef FNO_ZTC16
#undef FNO_ZTC16_S
  *taken = true;
  return hipGetLastError();
}

}  // namespace fno
