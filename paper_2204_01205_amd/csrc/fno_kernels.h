// Host-side launchers of the HIP kernels (internal to libfno; not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fno {

// One transform axis split as N = P * M: M-point in-register FFTs over the residue classes
// n = P*n1 + n2 and a dense P-term twiddle combine over the kept frequencies.
struct AxisPlan {
  int N;      // axis length
  int L;      // kept frequencies
  int npos;   // first npos entries are k = 0..npos-1, the rest k = -(L-npos)..-1
  int M;      // in-register FFT length (power of two dividing N, 1 = dense)
  int P;      // N / M
};

// Fill the twiddle tables:  tw[j*P + n2] = exp(-2 pi i k_j n2 / N)  for an AxisPlan, and
// twt[kt*Nt + n] = exp(-2 pi i kt n / Nt) for the real axis.
// Twiddle tables of a plan, written by one launch.  Axis table: L > 0, [L][P] entries
// w_N^(k_j n2); t table: L = 0, [npos][N] entries w_N^(kt n).
struct TableDesc { float2* tw; int N, L, npos, P; };
struct TableSet { TableDesc t[6]; int n; };
hipError_t launch_plan_tables(const TableSet& ts, hipStream_t s);

// Forward (t, z): x[planes][Nz][Nt] real  ->  out[planes][Lz][mt] complex.
hipError_t launch_tz_fwd(const float* x, float2* out, const float2* twt, const float2* twz,
                         int64_t planes, AxisPlan az, int Nt, int mt, hipStream_t s);

// Complex pruned transform along the middle axis of [outer][N|L][inner].
hipError_t launch_axis_fwd(const float2* in, float2* out, const float2* tw, int64_t outer,
                           AxisPlan ax, int64_t inner, hipStream_t s);
hipError_t launch_axis_inv(const float2* in, float2* out, const float2* tw, int64_t outer,
                           AxisPlan ax, int64_t inner, hipStream_t s);

// Per-mode channel mix.  scale_t[kt] = c_kt / N is applied to the result.
hipError_t launch_mix_fwd(const float2* xh, const float2* R, float2* yh, int B, int Ci, int Co,
                          int64_t K, int mt, int Nt, double invN, hipStream_t s);
// gR[i][o][k] = sum_b conj(xh[b][i][k]) gy[b][o][k],  gxh[b][i][k] = sum_o conj(R[i][o][k]) gy[b][o][k]
// with gy = (c_kt / N) gh.  gR and gxh nullable; accumulate: the sum over b is added to what gR holds.
hipError_t launch_mix_bwd(const float2* xh, const float2* R, const float2* gh, float2* gR,
                          float2* gxh, int B, int Ci, int Co, int64_t K, int mt, int Nt,
                          double invN, int accumulate, hipStream_t s);

struct Epilogue {
  const float* u;      // [B][Cu][grid] tensor the channel-linear term acts on, or nullptr
  int Cu;              // its channel count
  const float* W;      // element (o, i) at W[o*w_so + i*w_si]
  int w_so, w_si;
  const float* bias;   // [Co] or nullptr
  float* zsave;        // [B][Co][grid] pre-activation copy, or nullptr
  int act;             // 0 identity, 1 GELU
};

// Inverse (z, t) of a[B*Co planes][Lz][mt] plus epilogue  out = act(ys + W u + bias).
// `tables` is kZtTablesBytes of scratch (16-byte aligned) for the kernel's per-call tables.
hipError_t launch_zt_inv(const float2* a, float* out, const float2* twt, const float2* twz,
                         int B, int Co, int Nx, int Ny, AxisPlan az, int Nt, int mt,
                         Epilogue ep, float* tables, hipStream_t s);

// gz = g * act'(z) (g = gout or the MSE gradient against a target), written to gz_out;
// partial sums of gb[o] and gW[o][i] into part[*nslots][Co*Ci + Co] (double); *nslots (at most
// bwd_pointwise_blocks()) is what launch_reduce_partials must be given.
hipError_t launch_bwd_pointwise(const float* z, const float* gout, const float* x, float* gz_out,
                                double* part, int* nslots, int B, int Ci, int Co, int64_t N, int act,
                                int mse_target, double mse_scale, hipStream_t s);
hipError_t launch_reduce_partials(const double* part, int nblk, int Co, int Ci, float* gW,
                                  float* gb, int accumulate, hipStream_t s);
int bwd_pointwise_blocks(int B, int64_t N);

hipError_t launch_pointwise_linear(int B, int Ci, int Co, int64_t np, const float* x, const float* W,
                                   const float* bias, float* y, hipStream_t s);
hipError_t launch_pointwise_mlp2(int B, int Ci, int H, int Co, int64_t np, const float* x,
                                 const float* W1, const float* b1, const float* W2,
                                 const float* b2, float* y, hipStream_t s);

// Input lifts: a [B][Ci][np] (time axis of length one) -> out [B][Co][np][Nt].
hipError_t launch_time_lift(int B, int Ci, int Co, int64_t np, int Nt, const float* a, const float* wt,
                            const float* bt, const float* wc, const float* bc, float* out, hipStream_t s);

// Adjoint of the fused lifts with respect to Wt, bt, Wc, bc (each output nullable).  ws: device
// scratch of time_lift_bwd_workspace_bytes(Ci, Co, Nt) bytes.  Ci <= 8, B <= 1024.
size_t time_lift_bwd_workspace_bytes(int Ci, int Co, int Nt);
hipError_t launch_time_lift_bwd(int B, int Ci, int Co, int64_t S, int Nt, const float* a, const float* wt,
                                const float* bt, const float* wc, const float* g, float* gwt, float* gbt,
                                float* gwc, float* gbc, void* ws, hipStream_t s);

// Relative L2 misfit ||pred - target|| / ||target|| (device scalar `loss`, nullable) and its
// gradient with respect to pred (nullable); ws: rel_l2_workspace_bytes() of scratch.
size_t rel_l2_workspace_bytes();
hipError_t launch_rel_l2(int64_t n, const float* pred, const float* target, float* loss, float* grad,
                         double* ws, hipStream_t s);
// One Adam step in place on n floats (complex parameters as pairs of floats); step counts from 1.
hipError_t launch_adam(int64_t n, float* p, const float* g, float* m, float* v, double lr, double beta1,
                       double beta2, double eps, int step, hipStream_t s);

// Adjoints of the channel lift and of the two-layer projection.  ws: pointwise_bwd_workspace_bytes()
// of scratch, 8-byte aligned.  Outputs nullable.
size_t pointwise_bwd_workspace_bytes(int Ci, int H, int Co);
hipError_t launch_pointwise_linear_bwd(int B, int Ci, int Co, int64_t N, const float* x, const float* W,
                                       const float* g, float* gx, float* gW, float* gb, void* ws,
                                       hipStream_t s);
hipError_t launch_pointwise_mlp2_bwd(int B, int Ci, int H, int Co, int64_t N, const float* x, const float* W1,
                                     const float* b1, const float* W2, const float* g, float* gx, float* gW1,
                                     float* gb1, float* gW2, float* gb2, void* ws, hipStream_t s);

// Limits of the kernels (checked by the API before any launch).
constexpr int kMaxFftM = 32;        // largest in-register FFT
constexpr int kMaxCo = 32;          // accumulator file of the epilogue
constexpr int kLdsBudget = 60 * 1024;
constexpr size_t kZtTablesBytes = 512 * 1024;
bool tz_fwd_fits(AxisPlan az, int Nt, int mt);
bool zt_inv_fits(AxisPlan az, int Nt, int mt, int Co);
bool axis_fits(AxisPlan ax);
bool zt_mfma_fits(AxisPlan az, int Nt, int mt, int Co, int Cu);

}  // namespace fno
