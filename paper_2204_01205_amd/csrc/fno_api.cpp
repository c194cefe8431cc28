// C ABI of libfno: argument checks, the per-call plan (how each axis is split, how the
// workspace is carved up) and the kernel sequence.  See include/fno.h for the contract.
#include "../../include/fno.h"
#include "fno_kernels.h"

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

namespace {

using fno::AxisPlan;

thread_local char g_detail[256] = "";

void set_detail(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  std::vsnprintf(g_detail, sizeof(g_detail), fmt, ap);
  va_end(ap);
}

struct Plan {
  int B, Ci, Co;
  int N[4], L[4], npos[4];
  AxisPlan ax[3];        // x, y, z
  AxisPlan axf[2];       // x, y of the forward transforms (see fwd_fft_len)
  int mt, Nt;
  int64_t K;             // kept modes per (batch, channel)
  int64_t Npts;          // grid points per (batch, channel)
  // workspace offsets in bytes
  size_t off_ztab, off_twt, off_tw[3], off_twf[2], off_a1, off_a2, off_s1, off_s2, off_s3, off_gz, off_part, total;
  int part_blocks;
};

size_t align_up(size_t v) { return (v + 255) & ~size_t(255); }

// FFT length of the forward x and y transforms.  The forward stage is an M-point FFT per residue
// class followed by a P-term combine at the kept frequencies only; measured on 64-, 128- and
// 256-point axes it runs fastest with P = 8 classes (128 points: M = 16 is 13 % faster than 32, and
// 8 is slower again), while the inverse stage (gather of the kept frequencies + FFT) wants the
// longest FFT.  Lengths without that split keep the inverse's M.
int fwd_fft_len(int n, int m_inv) {
  if (n % 8 != 0) return m_inv;
  const int cand = n / 8;
  const bool pow2 = (cand & (cand - 1)) == 0;
  return (pow2 && cand >= 8 && cand <= m_inv) ? cand : m_inv;
}

int largest_pow2_divisor(int n, int cap) {
  int m = 1;
  while (m * 2 <= cap && n % (m * 2) == 0) m *= 2;
  return m;
}

// Validates the descriptor and builds the plan.  need_block: Cin == Cout and Cout <= 32.
int make_plan(const fno_desc* d, bool need_block, bool need_bwd_block, Plan* p) {
  if (d == nullptr) { set_detail("descriptor is null"); return FNO_EINVAL; }
  if (d->batch < 1 || d->c_in < 1 || d->c_out < 1) { set_detail("batch and channel widths must be >= 1"); return FNO_EINVAL; }
  if (d->mode_rule != 0 && d->mode_rule != 1) { set_detail("mode_rule must be 0 or 1"); return FNO_EINVAL; }
  if (d->activation != FNO_ACT_IDENTITY && d->activation != FNO_ACT_GELU) { set_detail("unknown activation"); return FNO_EINVAL; }
  if (d->flags & ~(FNO_FLAG_MSE_TARGET | FNO_FLAG_ACCUMULATE_GRADS | FNO_FLAG_TABLES_READY)) { set_detail("unknown flag bits"); return FNO_EINVAL; }
  for (int a = 0; a < 4; ++a) {
    if (d->grid[a] < 1) { set_detail("grid sizes must be >= 1"); return FNO_EINVAL; }
    if (d->modes[a] < (a == 3 ? 1 : 0)) { set_detail("mode counts must be non-negative (mt >= 1)"); return FNO_EINVAL; }
  }
  p->B = d->batch; p->Ci = d->c_in; p->Co = d->c_out;
  for (int a = 0; a < 3; ++a) {
    const int m = d->modes[a];
    const long long L = d->mode_rule == 0 ? 2LL * m : 2LL * m + 1;
    if (L < 1 || L > d->grid[a]) { set_detail("kept modes on a spatial axis must satisfy 1 <= L <= N (axis %d)", a); return FNO_EINVAL; }
    p->N[a] = d->grid[a]; p->L[a] = (int)L;
    p->npos[a] = d->mode_rule == 0 ? m : m + 1;
  }
  if (d->modes[3] > d->grid[3] / 2 + 1) { set_detail("mt must be <= Nt/2 + 1"); return FNO_EINVAL; }
  p->N[3] = d->grid[3]; p->L[3] = d->modes[3]; p->npos[3] = d->modes[3];
  p->Nt = d->grid[3]; p->mt = d->modes[3];
  if (need_block && d->c_in != d->c_out) { set_detail("block calls need c_in == c_out"); return FNO_EINVAL; }

  p->K = (int64_t)p->L[0] * p->L[1] * p->L[2] * p->L[3];
  p->Npts = (int64_t)p->N[0] * p->N[1] * p->N[2] * p->N[3];
  const int Cm = p->Ci > p->Co ? p->Ci : p->Co;
  if (Cm > fno::kMaxCo) { set_detail("channel width above %d is not covered", fno::kMaxCo); return FNO_EUNSUPPORTED; }

  for (int a = 0; a < 2; ++a) {
    AxisPlan ap{p->N[a], p->L[a], p->npos[a], 1, p->N[a]};
    ap.M = largest_pow2_divisor(p->N[a], fno::kMaxFftM);
    ap.P = p->N[a] / ap.M;
    if (!fno::axis_fits(ap)) { set_detail("spatial axis too long for the LDS tile (axis %d)", a); return FNO_EUNSUPPORTED; }
    p->ax[a] = ap;
    AxisPlan af = ap;
    af.M = fwd_fft_len(p->N[a], ap.M);
    af.P = p->N[a] / af.M;
    p->axf[a] = af;
  }
  {
    AxisPlan az{p->N[2], p->L[2], p->npos[2], 1, p->N[2]};
    bool ok = false;
    // 16 suits the tile of the matrix-core inverse kernel best; then larger, then smaller splits
    const int order[6] = {16, 32, 8, 4, 2, 1};
    for (int c = 0; c < 6 && !ok; ++c) {
      const int m = order[c];
      if (m > fno::kMaxFftM || p->N[2] % m) continue;
      az.M = m; az.P = p->N[2] / m;
      ok = fno::tz_fwd_fits(az, p->Nt, p->mt) &&
           (fno::zt_mfma_fits(az, p->Nt, p->mt, Cm, Cm) || fno::zt_inv_fits(az, p->Nt, p->mt, Cm));
    }
    if (!ok) { set_detail("an Nz x Nt plane with this many channels does not fit the LDS tiles"); return FNO_EUNSUPPORTED; }
    p->ax[2] = az;
  }

  // workspace
  size_t off = 0;
  p->off_ztab = off; off = align_up(off + fno::kZtTablesBytes);
  p->off_twt = off; off = align_up(off + (size_t)p->mt * p->Nt * 8);
  for (int a = 0; a < 3; ++a) { p->off_tw[a] = off; off = align_up(off + (size_t)p->ax[a].L * p->ax[a].P * 8); }
  for (int a = 0; a < 2; ++a) {
    p->off_twf[a] = p->off_tw[a];
    if (p->axf[a].P != p->ax[a].P) { p->off_twf[a] = off; off = align_up(off + (size_t)p->axf[a].L * p->axf[a].P * 8); }
  }
  const size_t bc = (size_t)p->B * Cm;
  p->off_a1 = off; off = align_up(off + bc * p->N[0] * p->N[1] * p->L[2] * p->mt * 8);
  p->off_a2 = off; off = align_up(off + bc * p->N[0] * p->L[1] * p->L[2] * p->mt * 8);
  p->off_s1 = off; off = align_up(off + bc * (size_t)p->K * 8);
  p->off_s2 = off; off = align_up(off + bc * (size_t)p->K * 8);
  p->off_s3 = off; off = align_up(off + bc * (size_t)p->K * 8);
  p->off_gz = off;
  p->off_part = off;
  p->part_blocks = 0;
  if (need_bwd_block) {
    off = align_up(off + (size_t)p->B * p->Co * (size_t)p->Npts * 4);
    p->off_part = off;
    p->part_blocks = fno::bwd_pointwise_blocks(p->B, p->Npts);
    off = align_up(off + (size_t)p->part_blocks * (p->Co * p->Ci + p->Co) * 8);
  }
  p->total = off;
  return FNO_OK;
}

bool misaligned16(const void* a, const void* b = nullptr, const void* c = nullptr, const void* d = nullptr,
                  const void* e = nullptr, const void* f = nullptr) {
  const uintptr_t bits = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
                         reinterpret_cast<uintptr_t>(c) | reinterpret_cast<uintptr_t>(d) |
                         reinterpret_cast<uintptr_t>(e) | reinterpret_cast<uintptr_t>(f);
  if (bits & 15) { set_detail("tensor pointers must be 16-byte aligned"); return true; }
  return false;
}

int check_ws(const Plan& p, void* ws, size_t ws_bytes) {
  if (ws == nullptr) { set_detail("workspace is null"); return FNO_EINVAL; }
  if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0) { set_detail("workspace must be 256-byte aligned"); return FNO_ENOSPC; }
  if (ws_bytes < p.total) { set_detail("workspace too small: need %lld bytes", (long long)p.total); return FNO_ENOSPC; }
  return FNO_OK;
}

#define FNO_HIP(expr)                                                       \
  do {                                                                      \
    hipError_t e_ = (expr);                                                 \
    if (e_ != hipSuccess) {                                                 \
      set_detail("HIP error: %s", hipGetErrorString(e_));          \
      return FNO_EHIP;                                                      \
    }                                                                       \
  } while (0)

// ---- optional per-stage timing (benchmarks only) ------------------------------------------
struct TimingRecord { int stage; hipEvent_t start, stop; };
constexpr int kMaxTimingRecords = 8192;
int g_timing_mask = 0;        // bit per FNO_STAGE_*
int g_timing_used = 0;
std::vector<TimingRecord> g_timing;     // events are created once and reused

bool timing_begin(int stage, hipStream_t s) {
  if (((g_timing_mask >> stage) & 1) == 0 || g_timing_used >= kMaxTimingRecords) return false;
  if (g_timing_used == (int)g_timing.size()) {
    TimingRecord r{stage, nullptr, nullptr};
    if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return false;
    g_timing.push_back(r);
  }
  g_timing[g_timing_used].stage = stage;
  return hipEventRecord(g_timing[g_timing_used].start, s) == hipSuccess;
}
void timing_end(hipStream_t s) {
  hipEventRecord(g_timing[g_timing_used].stop, s);
  ++g_timing_used;
}

#define FNO_STAGE(stage, s, expr)                 \
  do {                                            \
    const bool timed_ = timing_begin((stage), (s)); \
    hipError_t e_ = (expr);                       \
    if (timed_) timing_end((s));                  \
    if (e_ != hipSuccess) {                       \
      set_detail("HIP error: %s", hipGetErrorString(e_)); \
      return FNO_EHIP;                            \
    }                                             \
  } while (0)

template <class T> T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

// The twiddle tables depend on the descriptor only (grid, kept modes, mode rule).  tables_ready: the
// caller states that fno_plan_tables wrote them into this workspace and nothing overwrote them.
int build_tables(const Plan& p, void* ws, hipStream_t s, bool tables_ready = false) {
  if (tables_ready) return FNO_OK;
  fno::TableSet ts{};
  ts.t[ts.n++] = fno::TableDesc{at<float2>(ws, p.off_twt), p.Nt, 0, p.mt, 1};
  for (int a = 0; a < 3; ++a)
    ts.t[ts.n++] = fno::TableDesc{at<float2>(ws, p.off_tw[a]), p.ax[a].N, p.ax[a].L, p.ax[a].npos, p.ax[a].P};
  for (int a = 0; a < 2; ++a)
    if (p.off_twf[a] != p.off_tw[a])
      ts.t[ts.n++] = fno::TableDesc{at<float2>(ws, p.off_twf[a]), p.axf[a].N, p.axf[a].L, p.axf[a].npos, p.axf[a].P};
  FNO_HIP(fno::launch_plan_tables(ts, s));
  return FNO_OK;
}

// real field [B*C][grid] -> kept spectrum [B*C][K]
int forward_chain(const Plan& p, void* ws, const float* field, int C, float2* spec, hipStream_t s) {
  const int64_t bc = (int64_t)p.B * C;
  float2* a1 = at<float2>(ws, p.off_a1);
  float2* a2 = at<float2>(ws, p.off_a2);
  FNO_STAGE(FNO_STAGE_TZ_FWD, s, fno::launch_tz_fwd(field, a1, at<float2>(ws, p.off_twt), at<float2>(ws, p.off_tw[2]),
                             bc * p.N[0] * p.N[1], p.ax[2], p.Nt, p.mt, s));
  const int64_t in_y = (int64_t)p.L[2] * p.mt;
  FNO_STAGE(FNO_STAGE_Y_FWD, s, fno::launch_axis_fwd(a1, a2, at<float2>(ws, p.off_twf[1]), bc * p.N[0], p.axf[1], in_y, s));
  const int64_t in_x = in_y * p.L[1];
  FNO_STAGE(FNO_STAGE_X_FWD, s, fno::launch_axis_fwd(a2, spec, at<float2>(ws, p.off_twf[0]), bc, p.axf[0], in_x, s));
  return FNO_OK;
}

// scaled spectrum [B*C][K] -> real field through the epilogue
int inverse_chain(const Plan& p, void* ws, const float2* spec, int C, float* out, fno::Epilogue ep,
                  hipStream_t s) {
  const int64_t bc = (int64_t)p.B * C;
  float2* a1 = at<float2>(ws, p.off_a1);
  float2* a2 = at<float2>(ws, p.off_a2);
  const int64_t in_y = (int64_t)p.L[2] * p.mt;
  const int64_t in_x = in_y * p.L[1];
  FNO_STAGE(FNO_STAGE_X_INV, s, fno::launch_axis_inv(spec, a2, at<float2>(ws, p.off_tw[0]), bc, p.ax[0], in_x, s));
  FNO_STAGE(FNO_STAGE_Y_INV, s, fno::launch_axis_inv(a2, a1, at<float2>(ws, p.off_tw[1]), bc * p.N[0], p.ax[1], in_y, s));
  FNO_STAGE(FNO_STAGE_ZT_INV, s, fno::launch_zt_inv(a1, out, at<float2>(ws, p.off_twt), at<float2>(ws, p.off_tw[2]), p.B, C,
                             p.N[0], p.N[1], p.ax[2], p.Nt, p.mt, ep, at<float>(ws, p.off_ztab), s));
  return FNO_OK;
}

int conv_fwd_common(const Plan& p, const float* x, const float* R, float* out, float* xhat_save,
                    void* ws, fno::Epilogue ep, bool tables_ready, hipStream_t s) {
  int rc = build_tables(p, ws, s, tables_ready);
  if (rc != FNO_OK) return rc;
  float2* xh = xhat_save != nullptr ? reinterpret_cast<float2*>(xhat_save) : at<float2>(ws, p.off_s1);
  rc = forward_chain(p, ws, x, p.Ci, xh, s);
  if (rc != FNO_OK) return rc;
  float2* yh = at<float2>(ws, p.off_s2);
  FNO_STAGE(FNO_STAGE_MIX, s, fno::launch_mix_fwd(xh, reinterpret_cast<const float2*>(R), yh, p.B, p.Ci, p.Co, p.K, p.mt,
                              p.Nt, 1.0 / double(p.Npts), s));
  return inverse_chain(p, ws, yh, p.Co, out, ep, s);
}

// shared by the two backward calls; gz is dL/d(pre-activation) [B][Co][grid]
int conv_bwd_common(const Plan& p, const float* x, const float* xhat_saved, const float* R,
                    const float* gz, float* gx, float* gR, void* ws, fno::Epilogue ep, int accumulate,
                    hipStream_t s) {
  int rc;
  const float2* xh = reinterpret_cast<const float2*>(xhat_saved);
  if (gR != nullptr && xh == nullptr) {
    float2* s3 = at<float2>(ws, p.off_s3);
    rc = forward_chain(p, ws, x, p.Ci, s3, s);
    if (rc != FNO_OK) return rc;
    xh = s3;
  }
  if (xh == nullptr) xh = at<float2>(ws, p.off_s3);   // unread when gR is null
  float2* gh = at<float2>(ws, p.off_s1);
  rc = forward_chain(p, ws, gz, p.Co, gh, s);
  if (rc != FNO_OK) return rc;
  float2* gxh = gx != nullptr ? at<float2>(ws, p.off_s2) : nullptr;
  FNO_STAGE(FNO_STAGE_MIX_BWD, s, fno::launch_mix_bwd(xh, reinterpret_cast<const float2*>(R), gh,
                              reinterpret_cast<float2*>(gR), gxh, p.B, p.Ci, p.Co, p.K, p.mt, p.Nt,
                              1.0 / double(p.Npts), accumulate, s));
  if (gx != nullptr) return inverse_chain(p, ws, gxh, p.Ci, gx, ep, s);
  return FNO_OK;
}

}  // namespace

namespace fno {
// for the library's other translation units: sets the text fno_status_string returns
void set_status_detail(const char* text) { set_detail("%s", text); }
}  // namespace fno

extern "C" {

int fno_workspace_bytes(const fno_desc* desc, int op, size_t* bytes) {
  if (bytes == nullptr) { set_detail("bytes is null"); return FNO_EINVAL; }
  if (op < FNO_OP_SPECTRAL_CONV_FWD || op > FNO_OP_BLOCK_BWD) { set_detail("unknown op"); return FNO_EINVAL; }
  Plan p;
  const bool blk = (op == FNO_OP_BLOCK_FWD || op == FNO_OP_BLOCK_BWD);
  const int rc = make_plan(desc, blk, op == FNO_OP_BLOCK_BWD, &p);
  if (rc != FNO_OK) return rc;
  *bytes = p.total;
  return FNO_OK;
}

int fno_plan_tables(const fno_desc* desc, int op, void* ws, size_t ws_bytes, void* stream) {
  if (op < FNO_OP_SPECTRAL_CONV_FWD || op > FNO_OP_BLOCK_BWD) { set_detail("unknown op"); return FNO_EINVAL; }
  Plan p;
  const bool blk = (op == FNO_OP_BLOCK_FWD || op == FNO_OP_BLOCK_BWD);
  int rc = make_plan(desc, blk, op == FNO_OP_BLOCK_BWD, &p);
  if (rc != FNO_OK) return rc;
  rc = check_ws(p, ws, ws_bytes);
  if (rc != FNO_OK) return rc;
  return build_tables(p, ws, static_cast<hipStream_t>(stream));
}

int fno_mode_indices(const fno_desc* desc, int axis, int32_t* out_k, int32_t* out_n) {
  if (out_n == nullptr) { set_detail("out_n is null"); return FNO_EINVAL; }
  if (axis < 0 || axis > 3) { set_detail("axis must be 0..3"); return FNO_EINVAL; }
  Plan p;
  const int rc = make_plan(desc, false, false, &p);
  if (rc != FNO_OK && rc != FNO_EUNSUPPORTED) return rc;
  const int L = p.L[axis], np = p.npos[axis];
  *out_n = L;
  if (out_k != nullptr)
    for (int j = 0; j < L; ++j) out_k[j] = j < np ? j : j - L;
  return FNO_OK;
}

int fno_spectral_conv_fwd(const fno_desc* desc, const float* x, const float* R, float* y,
                          float* xhat_save, void* ws, size_t ws_bytes, void* stream) {
  Plan p;
  int rc = make_plan(desc, false, false, &p);
  if (rc != FNO_OK) return rc;
  if (x == nullptr || R == nullptr || y == nullptr) { set_detail("x, R and y are required"); return FNO_EINVAL; }
  if (misaligned16(x, R, y, xhat_save)) return FNO_EINVAL;
  rc = check_ws(p, ws, ws_bytes);
  if (rc != FNO_OK) return rc;
  fno::Epilogue ep{nullptr, 0, nullptr, 0, 0, nullptr, nullptr, 0};
  return conv_fwd_common(p, x, R, y, xhat_save, ws, ep, (desc->flags & FNO_FLAG_TABLES_READY) != 0,
                         static_cast<hipStream_t>(stream));
}

int fno_spectral_conv_bwd(const fno_desc* desc, const float* x, const float* xhat_saved,
                          const float* R, const float* gy, float* gx, float* gR, void* ws,
                          size_t ws_bytes, void* stream) {
  Plan p;
  int rc = make_plan(desc, false, false, &p);
  if (rc != FNO_OK) return rc;
  if (R == nullptr || gy == nullptr) { set_detail("R and gy are required"); return FNO_EINVAL; }
  if (gR != nullptr && x == nullptr && xhat_saved == nullptr) { set_detail("gR needs x or xhat_saved"); return FNO_EINVAL; }
  if (misaligned16(x, xhat_saved, R, gy, gx, gR)) return FNO_EINVAL;
  rc = check_ws(p, ws, ws_bytes);
  if (rc != FNO_OK) return rc;
  if (gx == nullptr && gR == nullptr) return FNO_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = build_tables(p, ws, s, (desc->flags & FNO_FLAG_TABLES_READY) != 0);
  if (rc != FNO_OK) return rc;
  fno::Epilogue ep{nullptr, 0, nullptr, 0, 0, nullptr, nullptr, 0};
  return conv_bwd_common(p, x, xhat_saved, R, gy, gx, gR, ws, ep, (desc->flags & FNO_FLAG_ACCUMULATE_GRADS) ? 1 : 0, s);
}

int fno_block_fwd(const fno_desc* desc, const float* x, const float* R, const float* W,
                  const float* b, float* out, float* z_save, float* xhat_save, void* ws,
                  size_t ws_bytes, void* stream) {
  Plan p;
  int rc = make_plan(desc, true, false, &p);
  if (rc != FNO_OK) return rc;
  if (x == nullptr || R == nullptr || W == nullptr || out == nullptr) { set_detail("x, R, W and out are required"); return FNO_EINVAL; }
  if (misaligned16(x, R, out, z_save, xhat_save)) return FNO_EINVAL;
  rc = check_ws(p, ws, ws_bytes);
  if (rc != FNO_OK) return rc;
  fno::Epilogue ep{x, p.Ci, W, p.Ci, 1, b, z_save, desc->activation};
  return conv_fwd_common(p, x, R, out, xhat_save, ws, ep, (desc->flags & FNO_FLAG_TABLES_READY) != 0,
                         static_cast<hipStream_t>(stream));
}

int fno_block_bwd(const fno_desc* desc, const float* x, const float* R, const float* W,
                  const float* z_saved, const float* xhat_saved, const float* gout, float* gx,
                  float* gR, float* gW, float* gb, void* ws, size_t ws_bytes, void* stream) {
  Plan p;
  int rc = make_plan(desc, true, true, &p);
  if (rc != FNO_OK) return rc;
  if (x == nullptr || R == nullptr || W == nullptr || z_saved == nullptr || gout == nullptr) {
    set_detail("x, R, W, z_saved and gout are required");
    return FNO_EINVAL;
  }
  if (misaligned16(x, R, z_saved, xhat_saved, gout, gx) || misaligned16(gR)) return FNO_EINVAL;
  rc = check_ws(p, ws, ws_bytes);
  if (rc != FNO_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = build_tables(p, ws, s, (desc->flags & FNO_FLAG_TABLES_READY) != 0);
  if (rc != FNO_OK) return rc;
  float* gz = at<float>(ws, p.off_gz);
  double* part = at<double>(ws, p.off_part);
  const int mse = (desc->flags & FNO_FLAG_MSE_TARGET) ? 1 : 0;
  const int accumulate = (desc->flags & FNO_FLAG_ACCUMULATE_GRADS) ? 1 : 0;
  const double mse_scale = 2.0 / (double(p.B) * double(p.Co) * double(p.Npts));
  int nslots = 0;
  FNO_STAGE(FNO_STAGE_BWD_POINTWISE, s, fno::launch_bwd_pointwise(z_saved, gout, x, gz, part, &nslots, p.B, p.Ci, p.Co,
                                    p.Npts, desc->activation, mse, mse_scale, s));
  if (gW != nullptr || gb != nullptr)
    FNO_HIP(fno::launch_reduce_partials(part, nslots, p.Co, p.Ci, gW, gb, accumulate, s));
  if (gx == nullptr && gR == nullptr) return FNO_OK;
  // gx = K(R^H) gz + W^T gz : the epilogue applies W transposed to gz, no bias, no activation
  fno::Epilogue ep{gz, p.Co, W, 1, p.Ci, nullptr, nullptr, 0};
  return conv_bwd_common(p, x, xhat_saved, R, gz, gx, gR, ws, ep, accumulate, s);
}

int fno_pointwise_linear(int32_t batch, int32_t c_in, int32_t c_out, int64_t npoints, const float* x,
                         const float* W, const float* bias, float* y, void* stream) {
  if (batch < 1 || c_in < 1 || c_out < 1 || npoints < 0) { set_detail("sizes must be positive"); return FNO_EINVAL; }
  if (x == nullptr || W == nullptr || y == nullptr) { set_detail("x, W and y are required"); return FNO_EINVAL; }
  if (c_out > 32 || batch > 65535) { set_detail("pointwise_linear covers c_out <= 32, batch <= 65535"); return FNO_EUNSUPPORTED; }
  FNO_HIP(fno::launch_pointwise_linear(batch, c_in, c_out, npoints, x, W, bias, y,
                                       static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_pointwise_mlp2(int32_t batch, int32_t c_in, int32_t hidden, int32_t c_out, int64_t npoints,
                       const float* x, const float* W1, const float* b1, const float* W2,
                       const float* b2, float* y, void* stream) {
  if (batch < 1 || c_in < 1 || hidden < 1 || c_out < 1 || npoints < 0) { set_detail("sizes must be positive"); return FNO_EINVAL; }
  if (x == nullptr || W1 == nullptr || W2 == nullptr || y == nullptr) { set_detail("x, W1, W2 and y are required"); return FNO_EINVAL; }
  if (c_in > 32 || c_out > 4 || batch > 65535) { set_detail("pointwise_mlp2 covers c_in <= 32, c_out <= 4, batch <= 65535"); return FNO_EUNSUPPORTED; }
  FNO_HIP(fno::launch_pointwise_mlp2(batch, c_in, hidden, c_out, npoints, x, W1, b1, W2, b2, y,
                                     static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_time_lift(int32_t batch, int32_t c_in, int32_t c_out, int64_t nspace, int32_t nt, const float* a,
                  const float* Wt, const float* bt, const float* Wc, const float* bc, float* out,
                  void* stream) {
  if (batch < 1 || c_in < 1 || c_out < 1 || nspace < 0 || nt < 1) { set_detail("sizes must be positive"); return FNO_EINVAL; }
  if (a == nullptr || Wt == nullptr || Wc == nullptr || out == nullptr) { set_detail("a, Wt, Wc and out are required"); return FNO_EINVAL; }
  if (c_out > 32 || batch > 65535) { set_detail("time_lift covers c_out <= 32, batch <= 65535"); return FNO_EUNSUPPORTED; }
  if (nt % 4 == 0 && misaligned16(out)) { set_detail("out must be 16-byte aligned"); return FNO_EINVAL; }
  FNO_HIP(fno::launch_time_lift(batch, c_in, c_out, nspace, nt, a, Wt, bt, Wc, bc, out,
                                static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_time_lift_bwd_workspace_bytes(int32_t c_in, int32_t c_out, int32_t nt, size_t* bytes) {
  if (bytes == nullptr || c_in < 1 || c_out < 1 || nt < 1) { set_detail("positive sizes and bytes are required"); return FNO_EINVAL; }
  *bytes = fno::time_lift_bwd_workspace_bytes(c_in, c_out, nt);
  return FNO_OK;
}

int fno_time_lift_bwd(int32_t batch, int32_t c_in, int32_t c_out, int64_t nspace, int32_t nt, const float* a,
                      const float* Wt, const float* bt, const float* Wc, const float* g, float* gWt,
                      float* gbt, float* gWc, float* gbc, void* ws, size_t ws_bytes, void* stream) {
  if (batch < 1 || c_in < 1 || c_out < 1 || nspace < 1 || nt < 1) { set_detail("sizes must be positive"); return FNO_EINVAL; }
  if (a == nullptr || Wt == nullptr || Wc == nullptr || g == nullptr || ws == nullptr) { set_detail("a, Wt, Wc, g and ws are required"); return FNO_EINVAL; }
  if (c_in > 8 || batch > 1024 || (int64_t)c_out * nt > (int64_t)1 << 20) { set_detail("time_lift_bwd covers c_in <= 8, batch <= 1024, c_out * nt <= 2^20"); return FNO_EUNSUPPORTED; }
  if (ws_bytes < fno::time_lift_bwd_workspace_bytes(c_in, c_out, nt)) { set_detail("workspace too small"); return FNO_ENOSPC; }
  if (reinterpret_cast<uintptr_t>(ws) % 8 != 0) { set_detail("ws must be 8-byte aligned"); return FNO_EINVAL; }
  FNO_HIP(fno::launch_time_lift_bwd(batch, c_in, c_out, nspace, nt, a, Wt, bt, Wc, g, gWt, gbt, gWc, gbc, ws,
                                    static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_pointwise_bwd_workspace_bytes(int32_t c_in, int32_t hidden, int32_t c_out, size_t* bytes) {
  if (bytes == nullptr || c_in < 1 || hidden < 0 || c_out < 1) { set_detail("positive widths and bytes are required"); return FNO_EINVAL; }
  *bytes = fno::pointwise_bwd_workspace_bytes(c_in, hidden, c_out);
  return FNO_OK;
}

int fno_pointwise_linear_bwd(int32_t batch, int32_t c_in, int32_t c_out, int64_t npoints, const float* x,
                             const float* W, const float* g, float* gx, float* gW, float* gb, void* ws,
                             size_t ws_bytes, void* stream) {
  if (batch < 1 || c_in < 1 || c_out < 1 || npoints < 1) { set_detail("sizes must be positive"); return FNO_EINVAL; }
  if (x == nullptr || W == nullptr || g == nullptr || ws == nullptr) { set_detail("x, W, g and ws are required"); return FNO_EINVAL; }
  if (c_in > 32 || c_out > 32 || batch > 65535) { set_detail("pointwise_linear_bwd covers widths <= 32, batch <= 65535"); return FNO_EUNSUPPORTED; }
  if (ws_bytes < fno::pointwise_bwd_workspace_bytes(c_in, 0, c_out)) { set_detail("workspace too small"); return FNO_ENOSPC; }
  if (reinterpret_cast<uintptr_t>(ws) % 8 != 0) { set_detail("ws must be 8-byte aligned"); return FNO_EINVAL; }
  FNO_HIP(fno::launch_pointwise_linear_bwd(batch, c_in, c_out, npoints, x, W, g, gx, gW, gb, ws,
                                           static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_pointwise_mlp2_bwd(int32_t batch, int32_t c_in, int32_t hidden, int32_t c_out, int64_t npoints,
                           const float* x, const float* W1, const float* b1, const float* W2, const float* g,
                           float* gx, float* gW1, float* gb1, float* gW2, float* gb2, void* ws,
                           size_t ws_bytes, void* stream) {
  if (batch < 1 || c_in < 1 || hidden < 1 || c_out < 1 || npoints < 1) { set_detail("sizes must be positive"); return FNO_EINVAL; }
  if (x == nullptr || W1 == nullptr || W2 == nullptr || g == nullptr || ws == nullptr) { set_detail("x, W1, W2, g and ws are required"); return FNO_EINVAL; }
  if (c_in > 32 || c_out > 4 || hidden > 1024) { set_detail("pointwise_mlp2_bwd covers c_in <= 32, c_out <= 4, hidden <= 1024"); return FNO_EUNSUPPORTED; }
  if (ws_bytes < fno::pointwise_bwd_workspace_bytes(c_in, hidden, c_out)) { set_detail("workspace too small"); return FNO_ENOSPC; }
  if (reinterpret_cast<uintptr_t>(ws) % 8 != 0) { set_detail("ws must be 8-byte aligned"); return FNO_EINVAL; }
  FNO_HIP(fno::launch_pointwise_mlp2_bwd(batch, c_in, hidden, c_out, npoints, x, W1, b1, W2, g, gx, gW1, gb1, gW2,
                                         gb2, ws, static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_rel_l2_workspace_bytes(size_t* bytes) {
  if (bytes == nullptr) { set_detail("bytes is required"); return FNO_EINVAL; }
  *bytes = fno::rel_l2_workspace_bytes();
  return FNO_OK;
}

int fno_rel_l2_loss(int64_t n, const float* pred, const float* target, float* loss, float* grad,
                    void* ws, size_t ws_bytes, void* stream) {
  if (n < 1) { set_detail("n must be positive"); return FNO_EINVAL; }
  if (pred == nullptr || target == nullptr || ws == nullptr) { set_detail("pred, target and ws are required"); return FNO_EINVAL; }
  if (loss == nullptr && grad == nullptr) { set_detail("one of loss and grad is required"); return FNO_EINVAL; }
  if (ws_bytes < fno::rel_l2_workspace_bytes()) { set_detail("workspace too small"); return FNO_ENOSPC; }
  if (reinterpret_cast<uintptr_t>(ws) % 8 != 0) { set_detail("ws must be 8-byte aligned"); return FNO_EINVAL; }
  FNO_HIP(fno::launch_rel_l2(n, pred, target, loss, grad, static_cast<double*>(ws),
                             static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_adam_step(int64_t n, float* param, const float* grad, float* m, float* v, double lr, double beta1,
                  double beta2, double eps, int32_t step, void* stream) {
  if (n < 0 || step < 1) { set_detail("n must be non-negative and step at least 1"); return FNO_EINVAL; }
  if (n > 0 && (param == nullptr || grad == nullptr || m == nullptr || v == nullptr)) { set_detail("param, grad, m and v are required"); return FNO_EINVAL; }
  if (!(beta1 >= 0.0 && beta1 < 1.0 && beta2 >= 0.0 && beta2 < 1.0)) { set_detail("beta1 and beta2 must lie in [0, 1)"); return FNO_EINVAL; }
  FNO_HIP(fno::launch_adam(n, param, grad, m, v, lr, beta1, beta2, eps, step, static_cast<hipStream_t>(stream)));
  return FNO_OK;
}

int fno_timing_enable(int stage_mask) {
  g_timing_mask = stage_mask;
  g_timing_used = 0;
  return FNO_OK;
}

int fno_timing_read(int32_t* stages, float* ms, int32_t capacity, int32_t* count) {
  if (count == nullptr || capacity < 0 || (capacity > 0 && (stages == nullptr || ms == nullptr))) {
    set_detail("timing_read needs count, and stages/ms when capacity > 0");
    return FNO_EINVAL;
  }
  int n = 0;
  for (int r = 0; r < g_timing_used && n < capacity; ++r) {
    FNO_HIP(hipEventSynchronize(g_timing[r].stop));
    float t = 0.f;
    FNO_HIP(hipEventElapsedTime(&t, g_timing[r].start, g_timing[r].stop));
    stages[n] = g_timing[r].stage;
    ms[n] = t;
    ++n;
  }
  *count = n;
  g_timing_used = 0;
  return FNO_OK;
}

const char* fno_status_string(int status) {
  switch (status) {
    case FNO_OK: return "ok";
    case FNO_EINVAL: return g_detail[0] ? g_detail : "invalid argument";
    case FNO_EUNSUPPORTED: return g_detail[0] ? g_detail : "request outside what the kernels cover";
    case FNO_ENOSPC: return g_detail[0] ? g_detail : "workspace too small or misaligned";
    case FNO_EHIP: return g_detail[0] ? g_detail : "HIP runtime error";
    default: return "unknown status";
  }
}

}  // extern "C"
