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
#include "fno_zt_inv.h"

namespace fno {

namespace {

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
  asm volatile("" ::: "memory");    // keep the issue order: tables, tile, u
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
  // everything issued so far has landed.  (Waiting only for the tables and the tile, with the u
  // loads still in flight over the z stage, needs a hand-counted vmcnt that depends on how many
  // instructions the compiler emits for the u loads; it measured no faster, so the plain wait stays.)
  __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
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

}  // namespace

hipError_t launch_zt_inv_mfma(const float2* a, float* out, const float2* twt, const float2* twz, int B, int Co,
                              int NxNy, AxisPlan az, int Nt, int mt, EpiArgs ep, float* tables, hipStream_t s,
                              bool* taken) {
  *taken = false;
  const EpiArgs& e = ep;
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  const int ntt = mfma_tile_nt(Nt);           // t-tile of the matrix-core kernels (0: none)
  const bool tpad = ntt != Nt;
  const int nw = ntt > 0 ? mfma_nw(az, ntt, mt, Co, ep.u ? ep.Cu : 0) : 0;
  const int qf = nw > 0 ? mfma_q_nw(az, ntt, nw) : 0;
  if (qf > 0) {
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
    hipError_t terr = launch_zt_tables(tables, G, twt, twz, ep.u ? ep.W : nullptr, ep.w_so, ep.w_si, ep.bias, Co,
                                       ep.u ? ep.Cu : 0, 4 * CT, mt, ntt, Nt, az.L, az.P, qf, blob_floats, s);
    if (terr != hipSuccess) return terr;
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
    *taken = true;
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace fno
