// Internal to libfno: what the three inverse (z, t) kernels share -- the epilogue arguments, the
// host-side sizing rules of their LDS tiles, and the entry points of their translation units.
#pragma once
#include "fno_device.h"

namespace fno {

// Pointwise part of the block update fused into the stage:  out = act(ys + W u + bias).
struct EpiArgs {
  const float* u; int Cu; const float* W; int w_so, w_si; const float* bias; float* zsave; int act;
};

// The t stage of the generic kernel can hold a block's results in registers (eight 16-row tiles
// per wave, one 16-wide tile of t) until every wave has read V, and then write Y over V: one LDS
// buffer instead of two.
__host__ __device__ inline bool zt_y_over_v(int Nt, int rows, int mt) {
  return Nt <= 16 && rows <= 512 && 2 * mt <= 36;
}

inline int pick_q(AxisPlan az, int Nt) {
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

inline size_t zt_inv_lds(AxisPlan az, int Nt, int mt, int Co) {
  const int Rz = pick_q(az, Nt) * az.M;
  // V and Y (one buffer where Y may take V's place), rounded up to 16 bytes, and the epilogue's
  // weights for up to kMaxCo x kMaxCo channels
  const size_t v_floats = (size_t)2 * Co * Rz * mt, y_floats = (size_t)Co * Rz * (Nt + 1);
  const size_t vy = zt_y_over_v(Nt, Co * Rz, mt) ? (v_floats > y_floats ? v_floats : y_floats) : v_floats + y_floats;
  return ((vy + 3) & ~(size_t)3) * 4 + (size_t)kMaxCo * kMaxCo * 4;
}

// Tile of the matrix-core kernel: Q residue classes whose Rz = Q*M rows times Nt points make
// 128..512 points (64..256 threads, two points each) and whose Q adjacent rows span at least 128 bytes.
// Rows per tile for NW waves: each wave covers 128 points.  Returns Q = rows / M, or 0.
// t-tile of the matrix-core kernels for an axis of length Nt: 16 or 32 points, the axis itself or
// the next tile width above an even length; 0 when neither fits
inline int mfma_tile_nt(int Nt) {
  if (Nt == 16 || Nt == 32) return Nt;
  if (Nt % 2 != 0 || Nt < 10 || Nt > 32) return 0;
  return Nt < 16 ? 16 : 32;
}

inline int mfma_q_nw(AxisPlan az, int Nt, int nw) {
  if (Nt != 16 && Nt != 32) return 0;
  if (az.M != 8 && az.M != 16) return 0;
  if (az.P & (az.P - 1)) return 0;                 // residue-class count must be a power of two
  const int rz = nw * (128 / Nt);
  if (rz % az.M) return 0;
  const int q = rz / az.M;
  if (q > az.P) return 0;
  return q;
}

// LDS channel stride of the spectrum tile in float4: padded so that consecutive channels start
// 2 mt .. 64 - 2 mt floats apart modulo the 64 banks
inline int zt_mfma_astride4(AxisPlan az, int mt) {
  const int per_ch4 = (az.L * mt) / 2;
  for (int pad = 0; pad < 16; ++pad) {
    const int r = (4 * (per_ch4 + pad)) % 64;
    if (r >= 2 * mt && r <= 64 - 2 * mt) return per_ch4 + pad;
  }
  return per_ch4 + 1;
}

// channel stride of V in float2: rows * mt padded to 2 modulo 32, so that the four channels an
// MFMA block reads together fall into different banks
inline int zt_mfma_vstride(AxisPlan az, int mt, int q) {
  const int base = q * az.M * mt;
  return base + ((2 - base) % 32 + 32) % 32;
}

// floats of the region shared by the spectrum tile and V
inline int zt_mfma_region(AxisPlan az, int mt, int Co, int q) {
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  const int a_floats = Co * zt_mfma_astride4(az, mt) * 4 + 256;   // the last wave load may run 63 lanes past
  const int v_floats = 2 * 4 * CT * zt_mfma_vstride(az, mt, q);
  const int r = a_floats > v_floats ? a_floats : v_floats;
  return (r + 255) & ~255;
}

inline int zt_mfma_blob(AxisPlan az, int Nt, int mt, int Co, int Cu, int q) {
  const int CP = 4 * ((Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8));
  return ((2 * mt * Nt + Cu * CP + 2 * q * az.L + CP + 255) / 256) * 256;      // whole 1 KiB wave loads
}

inline size_t zt_mfma_lds(AxisPlan az, int Nt, int mt, int Co, int Cu, int q) {
  return ((size_t)zt_mfma_region(az, mt, Co, q) + (size_t)zt_mfma_blob(az, Nt, mt, Co, Cu, q)) * 4;
}

inline bool mfma_cfg_ok(AxisPlan az, int Nt, int mt, int Co, int Cu, int nw, size_t lds_cap) {
  const int q = mfma_q_nw(az, Nt, nw);
  const int CT = (Co + 3) / 4 <= 2 ? 2 : ((Co + 3) / 4 <= 5 ? 5 : 8);
  // the tile is staged in 16-byte pieces (L * mt even) and a thread owns at most two z-stage items
  return q > 0 && (az.L * mt) % 2 == 0 && Co * mt * q <= (nw == 8 ? 512 : 512) && Co <= kMaxCo && Cu <= 4 * CT &&
         (nw == 4 || CT <= 5) && zt_mfma_lds(az, Nt, mt, Co, Cu, q) <= lds_cap;
}

// Eight waves (two blocks per CU) when the tile then still fits half a CU's LDS, else four.
inline int mfma_nw(AxisPlan az, int Nt, int mt, int Co, int Cu) {
  if (mfma_cfg_ok(az, Nt, mt, Co, Cu, 8, 78 * 1024)) return 8;
  if (mfma_cfg_ok(az, Nt, mt, Co, Cu, 4, 80 * 1024)) return 4;
  return 0;
}

// Table blobs of the matrix-core kernels, one per residue group, in the kernels' LDS layout
// (defined in fno_zt_inv.hip).
hipError_t launch_zt_tables(float* blob, int groups, const float2* twt, const float2* twz, const float* W,
                            int w_so, int w_si, const float* bias, int Co, int Cu, int CP, int mt, int NT,
                            int nt_act, int Lz, int Pz, int Q, int blob_floats, hipStream_t s);

// Each launcher sets *taken when its kernel covers the shape and has been launched.
hipError_t launch_zt_inv_col(const float2* a, float* out, const float2* twt, const float2* twz, int B, int Co,
                             int NxNy, AxisPlan az, int Nt, int mt, EpiArgs e, float* tables, hipStream_t s,
                             bool* taken);
hipError_t launch_zt_inv_col16(const float2* a, float* out, const float2* twt, const float2* twz, int B, int Co,
                               int NxNy, AxisPlan az, int Nt, int mt, EpiArgs e, float* tables, hipStream_t s,
                               bool* taken);
hipError_t launch_zt_inv_mfma(const float2* a, float* out, const float2* twt, const float2* twz, int B, int Co,
                              int NxNy, AxisPlan az, int Nt, int mt, EpiArgs e, float* tables, hipStream_t s,
                              bool* taken);
hipError_t launch_zt_inv_generic(const float2* a, float* out, const float2* twt, const float2* twz, int64_t ncols,
                                 int Co, int NxNy, AxisPlan az, int Nt, int mt, EpiArgs e, hipStream_t s);

}  // namespace fno
