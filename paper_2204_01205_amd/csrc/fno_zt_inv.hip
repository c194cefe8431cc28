// Inverse (z, t) stage of the transform chain (F^-1 of eq. (3) of arXiv 2204.01205 along the last
// two axes, complex-to-real over t) fused with the pointwise part of the block update of eq. (2) /
// Sec. 2.4, sigma(W x + b + K x).  Four kernels cover it, each in a translation unit of its own:
// per column on the matrix cores (fno_zt_inv_col.hip for 32 points of t, fno_zt_inv_col16.hip for
// 16), per tile on the matrix cores
// (fno_zt_inv_mfma.hip) and the generic one (fno_zt_inv_generic.hip).  This file: the table blobs
// the matrix-core kernels read and the choice between them.
#include "fno_zt_inv.h"

namespace fno {

namespace {

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

}  // namespace

hipError_t launch_zt_tables(float* blob, int groups, const float2* twt, const float2* twz, const float* W,
                            int w_so, int w_si, const float* bias, int Co, int Cu, int CP, int mt, int NT,
                            int nt_act, int Lz, int Pz, int Q, int blob_floats, hipStream_t s) {
  hipLaunchKernelGGL(zt_tables_kernel, dim3(groups), dim3(256), 0, s, blob, twt, twz, W, w_so, w_si, bias, Co,
                     Cu, CP, mt, NT, nt_act, Lz, Pz, Q, blob_floats);
  return hipGetLastError();
}

bool zt_inv_fits(AxisPlan az, int Nt, int mt, int Co) {
  return Co <= kMaxCo && zt_inv_lds(az, Nt, mt, Co) <= (size_t)(68 * 1024);
}

bool zt_mfma_fits(AxisPlan az, int Nt, int mt, int Co, int Cu) {
  const int ntt = mfma_tile_nt(Nt);
  return ntt > 0 && mfma_nw(az, ntt, mt, Co, Cu) > 0;
}

hipError_t launch_zt_inv(const float2* a, float* out, const float2* twt, const float2* twz, int B,
                         int Co, int Nx, int Ny, AxisPlan az, int Nt, int mt, Epilogue ep,
                         float* tables, hipStream_t s) {
  const int64_t ncols = (int64_t)B * Nx * Ny;
  if (ncols <= 0) return hipSuccess;
  if (Co > kMaxCo) return hipErrorInvalidValue;
  EpiArgs e{ep.u, ep.Cu, ep.W, ep.w_so, ep.w_si, ep.bias, ep.zsave, ep.act};
  const int NxNy = Nx * Ny;
  const bool aligned = ((reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(ep.u) |
                         reinterpret_cast<uintptr_t>(ep.zsave) | reinterpret_cast<uintptr_t>(a) |
                         reinterpret_cast<uintptr_t>(tables)) & 15) == 0;
  if (aligned && tables != nullptr) {
    bool taken = false;
    hipError_t err = launch_zt_inv_col(a, out, twt, twz, B, Co, NxNy, az, Nt, mt, e, tables, s, &taken);
    if (err != hipSuccess || taken) return err;
    err = launch_zt_inv_col16(a, out, twt, twz, B, Co, NxNy, az, Nt, mt, e, tables, s, &taken);
    if (err != hipSuccess || taken) return err;
    err = launch_zt_inv_mfma(a, out, twt, twz, B, Co, NxNy, az, Nt, mt, e, tables, s, &taken);
    if (err != hipSuccess || taken) return err;
  }
  return launch_zt_inv_generic(a, out, twt, twz, ncols, Co, NxNy, az, Nt, mt, e, s);
}

}  // namespace fno
