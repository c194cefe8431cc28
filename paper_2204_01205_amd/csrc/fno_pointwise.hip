// Kernels of libfno for gfx950 that act point by point over the grid (arXiv 2204.01205): the
// activation/loss gradient with the sum-reductions that are the adjoint of broadcasting W and b
// (Sec. 2.1), the channel lift and the projection of Sec. 2.4 with their adjoints, the time lift
// (eqs. (8)-(9)) with its adjoint, the relative L2 misfit and the Adam update of Sec. 4.
#include "fno_device.h"

namespace fno {

namespace {

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
  // Phi and phi from one exponential: with x = |z| / sqrt 2 and t = 1 / (1 + p x),
  //   erfc(x) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-x^2)    (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7)
  // and exp(-x^2) = exp(-z^2 / 2) is phi(z) up to its constant.  The a_i below are halved, so the
  // polynomial times the exponential is the upper tail 1 - Phi(|z|).  23 issue slots (the reciprocal
  // and the exponential count four each); against float64: at most 4.3e-7 absolute on z Phi(z), 3.0e-7 on the slope.
  const float t = __builtin_amdgcn_rcpf(fmaf(fabsf(z), 0.23164190f, 1.0f));
  float q = fmaf(t, 0.5307027145f, -0.7265760135f);
  q = fmaf(t, q, 0.7107068705f);
  q = fmaf(t, q, -0.1422483680f);
  q = fmaf(t, q, 0.1274147960f);
  q *= t;
  const float e = __builtin_amdgcn_exp2f((z * z) * -0.72134752044f);    // exp(-z^2 / 2)
  const float tail = q * e;
  const float cdf = z < 0.f ? tail : 1.0f - tail;
  val = z * cdf;
  grad = fmaf(z, 0.39894228040143267794f * e, cdf);
}

template <int CT, bool STREAM>
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
  // Thread blocks are dealt to the eight XCDs round robin (the grid is a multiple of 8 blocks): each
  // XCD walks a contiguous eighth of the steps, its waves interleaved inside it (1-6 % faster than
  // all waves interleaved over the whole range, measured on the same allocations)
  const long long per_x = (steps + 7) >> 3;
  const long long xs = (long long)(blockIdx.x & 7) * per_x;
  const long long xe = xs + per_x < steps ? xs + per_x : steps;
  const long long wl = (long long)(blockIdx.x >> 3) * (kThreads / 64) + wave;
  const long long nwl = (long long)(gridDim.x >> 3) * (kThreads / 64);
  for (long long s = xs + wl; s < xe; s += nwl) {
    const long long bb = s / steps_per_b;
    const long long p0 = (s - bb * steps_per_b) * 64 + 4 * blk;
    float4 gzv[CT], xv[CT];
#pragma unroll
    for (int T = 0; T < CT; ++T) {
      const long long e = (bb * C + 4 * T + j4) * N + p0;
      const v4f zq = ld_once<STREAM>(reinterpret_cast<const v4f*>(z + e));
      const v4f gq = ld_once<STREAM>(reinterpret_cast<const v4f*>(gout + e));
      const v4f xq = ld_once<STREAM>(reinterpret_cast<const v4f*>(x + e));
      const float4 zv = make_float4(zq[0], zq[1], zq[2], zq[3]);
      float4 g = make_float4(gq[0], gq[1], gq[2], gq[3]);
      xv[T] = make_float4(xq[0], xq[1], xq[2], xq[3]);
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
      st_once<STREAM>(reinterpret_cast<v4f*>(gz_out + e), v4f{g.x, g.y, g.z, g.w});
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
    float* __restrict__ gb, int accumulate) {
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
    // accumulate: the sums are added to what gW and gb hold (a step over several calls)
    if (q < Co * Ci) { if (gW != nullptr) gW[q] = float(accumulate ? t + double(gW[q]) : t); }
    else if (gb != nullptr) gb[q - Co * Ci] = float(accumulate ? t + double(gb[q - Co * Ci]) : t);
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

// Four consecutive points per thread (16-byte loads and stores); the arithmetic of a point is
// the scalar kernel's, term by term.  For point counts that are multiples of 4 and 16-byte
// aligned tensors.
template <int CO>
__global__ __launch_bounds__(kThreads) void pointwise_linear_v4_kernel(
    int Ci, int Co, long long np4, const v4f* __restrict__ x, const float* __restrict__ W,
    const float* __restrict__ bias, v4f* __restrict__ y) {
  const long long p = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long b = blockIdx.y;
  if (p >= np4) return;
  v4f acc[CO];
#pragma unroll
  for (int o = 0; o < CO; ++o) {
    const float bo = (bias != nullptr && o < Co) ? bias[o] : 0.f;
    acc[o] = v4f{bo, bo, bo, bo};
  }
  for (int i = 0; i < Ci; ++i) {
    const v4f xv = __builtin_nontemporal_load(&x[(b * Ci + i) * np4 + p]);
#pragma unroll
    for (int o = 0; o < CO; ++o)
      if (o < Co) {
        const float w = W[o * Ci + i];
        acc[o].x = fmaf(w, xv.x, acc[o].x);
        acc[o].y = fmaf(w, xv.y, acc[o].y);
        acc[o].z = fmaf(w, xv.z, acc[o].z);
        acc[o].w = fmaf(w, xv.w, acc[o].w);
      }
  }
#pragma unroll
  for (int o = 0; o < CO; ++o)
    if (o < Co) y[(b * Co + o) * np4 + p] = acc[o];
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
  // every element is read and written once per step: nontemporal accesses
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kThreads) {
    const float gi = __builtin_nontemporal_load(g + i);
    const float mi = fmaf(beta1, __builtin_nontemporal_load(m + i), omb1 * gi);
    const float vi = fmaf(beta2, __builtin_nontemporal_load(v + i), omb2 * gi * gi);
    __builtin_nontemporal_store(mi, m + i);
    __builtin_nontemporal_store(vi, v + i);
    __builtin_nontemporal_store(__builtin_nontemporal_load(p + i) - lr * (mi * c1) / (sqrtf(vi * c2) + eps), p + i);
  }
}

// Input lifts of Sec. 2.4 (eqs. (8)-(9)) in one sweep: a_1 = W_t a + b_t along a time axis of
// length one, then nu = W_c a_1 + b_c along the channels, i.e.
//   nu[b][c][p][t] = W_t[t] s_c(p) + b_t[t] r_c + b_c[c],  s_c(p) = sum_j W_c[c][j] a[b][j][p],
//   r_c = sum_j W_c[c][j].
// One thread: one spatial point and four consecutive t; the output (the only large tensor) is
// written once, a is read through the cache by the threads that share a point.
template <int CO, bool STREAM>
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
        st_once<STREAM>(reinterpret_cast<v4f*>(dst), v4f{v[0], v[1], v[2], v[3]});
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
template <int CI, bool STREAM>
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
      for (int u = 0; u < 8; ++u) gv[u] = live ? ld_once<STREAM>(&gp[(sp + u) * Nt]) : 0.f;
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

}  // namespace

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
    int64_t nb = ((steps + 3) / 4 + 7) / 8 * 8;      // a multiple of 8: see the kernel's step ranges
    if (nb > 1024) nb = 1024;
    *nslots = (int)nb * 4;
    const dim3 grid((unsigned)nb);
    const bool stream = (int64_t)B * Co * N * 4 >= kStreamBytes;      // each tensor is touched once
    switch (Co / 4) {
#define FNO_BPW(CTV)                                                                               \
  case CTV:                                                                                        \
    if (stream)                                                                                    \
      hipLaunchKernelGGL((bwd_pointwise_mfma_kernel<CTV, true>), grid, dim3(kThreads), 0, s, z, gout, x,  \
                         gz_out, part, B, (long long)N, act, mse_target, (float)mse_scale);        \
    else                                                                                           \
      hipLaunchKernelGGL((bwd_pointwise_mfma_kernel<CTV, false>), grid, dim3(kThreads), 0, s, z, gout, x, \
                         gz_out, part, B, (long long)N, act, mse_target, (float)mse_scale);        \
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
                                  float* gb, int accumulate, hipStream_t s) {
  const int npairs = Co * Ci + Co;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((npairs + 63) / 64), dim3(64 * kRedGroups), 0, s, part,
                     nblk, Co, Ci, gW, gb, accumulate);
  return hipGetLastError();
}

hipError_t launch_pointwise_linear(int B, int Ci, int Co, int64_t np, const float* x, const float* W,
                                   const float* bias, float* y, hipStream_t s) {
  const int64_t nb = (np + kThreads - 1) / kThreads;
  if (nb > 0x7fffffffLL || B > 65535 || Co > 32) return hipErrorInvalidValue;
  if (nb == 0 || B == 0) return hipSuccess;
  if (np % 4 == 0 && Co <= 20 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & 15) == 0) {
    const int64_t np4 = np / 4;
    dim3 grid4((unsigned)((np4 + kThreads - 1) / kThreads), (unsigned)B);
    if (Co <= 8)
      hipLaunchKernelGGL((pointwise_linear_v4_kernel<8>), grid4, dim3(kThreads), 0, s, Ci, Co,
                         (long long)np4, reinterpret_cast<const v4f*>(x), W, bias,
                         reinterpret_cast<v4f*>(y));
    else
      hipLaunchKernelGGL((pointwise_linear_v4_kernel<20>), grid4, dim3(kThreads), 0, s, Ci, Co,
                         (long long)np4, reinterpret_cast<const v4f*>(x), W, bias,
                         reinterpret_cast<v4f*>(y));
    return hipGetLastError();
  }
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
  // the lifted tensor is written once: as a stream when it is larger than the caches
  const bool stream = (int64_t)B * Co * np * Nt * 4 >= kStreamBytes;
#define FNO_TL(COV)                                                                                          \
  do {                                                                                                       \
    if (stream)                                                                                              \
      hipLaunchKernelGGL((time_lift_kernel<COV, true>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)np, Nt, a, \
                         wt, bt, wc, bc, out);                                                               \
    else                                                                                                     \
      hipLaunchKernelGGL((time_lift_kernel<COV, false>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)np, Nt, a, \
                         wt, bt, wc, bc, out);                                                               \
  } while (0)
  if (Co <= 8) FNO_TL(8); else if (Co <= 20) FNO_TL(20); else FNO_TL(32);
#undef FNO_TL
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
  // the cotangent of the lifted tensor is read once: as a stream when it is larger than the caches
  const bool stream = (int64_t)B * Co * S * Nt * 4 >= kStreamBytes;
#define FNO_TLB(CIV)                                                                                         \
  do {                                                                                                       \
    if (stream)                                                                                              \
      hipLaunchKernelGGL((time_lift_bwd_kernel<CIV, true>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)S, Nt, \
                         cpb, a, g, part);                                                                   \
    else                                                                                                     \
      hipLaunchKernelGGL((time_lift_bwd_kernel<CIV, false>), grid, dim3(kThreads), 0, s, Ci, Co, (long long)S, Nt, \
                         cpb, a, g, part);                                                                   \
  } while (0)
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
                       part, nblk, Co, Ci, gW, gb, 0);
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
