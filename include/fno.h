/*
 * fno.h -- C ABI of libfno: the 4D (x,y,z,t) Fourier-neural-operator spectral convolution
 * and FNO block, forward and adjoint, as hand-written HIP kernels for gfx950 (MI355X).
 *
 * What the calls compute follows the paper's statement of the layer
 * (Grady et al., "Model-Parallel Fourier Neural Operators ...", arXiv 2204.01205):
 *   - eq. (2), Sec. 1.4 and the block update of Sec. 2.4:  nu_{k+1} = sigma(W nu_k + K(phi) nu_k)
 *   - eq. (3), Sec. 1.4:  K(phi) nu = F^{-1}( R_phi . F nu ), R_phi = low-pass restriction to a
 *     user-chosen number of modes per dimension plus a learned complex weight per kept mode
 *   - eq. (4), Sec. 2.2:  y = W x + b contracted along the channel dimension
 *   - eq. (7), Sec. 2.3 and the Fig. 5 caption: F^T is the adjoint (inverse) transform, used
 *     for the backward pass
 *
 * Conventions (all calls):
 *   - Tensors are dense, row-major, layout NCXYZT (Sec. 3.1): x[b][c][nx][ny][nz][nt], t contiguous.
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *     frees or synchronises; scratch comes from the caller's workspace `ws` (device memory,
 *     256-byte aligned, at least fno_workspace_bytes() bytes).  Descriptors are host structs
 *     read during the call only.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     the call returns without waiting.
 *   - Complex tensors are interleaved (re, im) float pairs.  Grid-sized and mode-sized tensors
 *     must be 16-byte aligned (FNO_EINVAL otherwise).
 *   - Return value: FNO_OK (0) or a negative FNO_E* code.  On an argument error nothing is
 *     launched and no output byte is written.
 *   - Two calls that share a workspace or an output must be ordered by the caller.
 *
 * Kept modes.  With modes = (mx, my, mz, mt) the spatial axes keep the signed frequencies
 *   rule 0:  0..m-1, -m..-1      (L = 2m)        rule 1:  0..m, -m..-1     (L = 2m+1)
 * in exactly this order along the weight tensor's mode axes, and the real-transform axis t
 * keeps 0..mt-1.  Requirements: 1 <= L <= N on x,y,z and 1 <= mt <= Nt/2 + 1.
 *
 * Forward transform is unnormalised; the inverse carries 1/(Nx Ny Nz Nt) and is a complex
 * inverse over x,y,z followed by a complex-to-real step over t, i.e.
 *   y[n] = (1/N) Re sum_k c_kt Yhat[k] exp(+i theta(k,n)),   c_kt = 1 for kt = 0 and kt = Nt/2, else 2.
 */
#ifndef FNO_H_
#define FNO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  FNO_OK = 0,
  FNO_EINVAL = -1,        /* null required pointer, non-positive size, too many modes, bad flag  */
  FNO_EUNSUPPORTED = -2,  /* valid request outside what the kernels cover (see fno_status_string) */
  FNO_ENOSPC = -3,        /* workspace too small or misaligned                                    */
  FNO_EHIP = -4           /* the HIP runtime refused a launch or copy                             */
};

/* GELU is z Phi(z) with Phi the normal distribution function (the erf form, not the tanh one).  The
 * kernels evaluate erf by the rational form of Abramowitz & Stegun 7.1.28 (|error| <= 3e-7) in the
 * forward epilogues, by their 7.1.26 (|error| <= 1.5e-7, sharing its exponential with the density) in
 * the matrix-core backward kernels, and by the float erff / expf routines in the generic backward
 * kernel; in every case the activation and its slope are within 1e-6 (absolute) of
 * the float64 definition, far inside the 1e-5 relative L2 the library is tested to. */
enum { FNO_ACT_IDENTITY = 0, FNO_ACT_GELU = 1 };

enum {
  FNO_OP_SPECTRAL_CONV_FWD = 0,
  FNO_OP_SPECTRAL_CONV_BWD = 1,
  FNO_OP_BLOCK_FWD = 2,
  FNO_OP_BLOCK_BWD = 3
};

enum {
  FNO_FLAG_MSE_TARGET = 1,       /* block_bwd: `gout` holds a target field; the upstream gradient is that of
                                    the mean squared error, 2 (sigma(z) - target) / (B Cout N)            */
  FNO_FLAG_ACCUMULATE_GRADS = 2, /* block_bwd, spectral_conv_bwd: the parameter gradients (gR, gW, gb) are
                                    added to what the output buffers hold instead of overwriting them: the
                                    gradient of a broadcast weight is a sum (Sec. 2.1), and a step made of
                                    several calls (one per sample or per shard) continues that sum.  gx is
                                    always overwritten.                                                    */
  FNO_FLAG_TABLES_READY = 4      /* every call with a workspace: the twiddle tables for this descriptor are in
                                    `ws` already (written by fno_plan_tables on the same workspace, nothing
                                    else having written there since except the library's own calls with the
                                    same grid, modes and mode rule); the call then skips the four small
                                    kernels that rebuild them                                              */
};

typedef struct {
  int32_t batch;       /* B >= 1                                                      */
  int32_t c_in;        /* input channel width                                         */
  int32_t c_out;       /* output channel width (<= 32 for the block calls)            */
  int32_t grid[4];     /* Nx, Ny, Nz, Nt                                              */
  int32_t modes[4];    /* mx, my, mz: per-side count on x,y,z ; mt: count on t        */
  int32_t mode_rule;   /* 0 or 1, see above                                           */
  int32_t activation;  /* FNO_ACT_*; used by the block calls only                     */
  int32_t flags;       /* FNO_FLAG_* bits                                             */
} fno_desc;

/* Size in bytes of the workspace the given FNO_OP_* needs for this descriptor (host-only). */
int fno_workspace_bytes(const fno_desc* desc, int op, size_t* bytes);

/* Writes the twiddle tables of the transforms (Sec. 2.3: one truncated DFT per axis; they depend on
 * the grid, the kept modes and the mode rule only) into the workspace, on `stream`.  Optional: every
 * call rebuilds them itself unless its descriptor carries FNO_FLAG_TABLES_READY.  The table region
 * sits at the same place in the workspace of every FNO_OP_*, so one plan serves all four calls on
 * that workspace.  ws, ws_bytes as for the op given. */
int fno_plan_tables(const fno_desc* desc, int op, void* ws, size_t ws_bytes, void* stream);

/* Kept signed frequencies of axis 0..3 (x,y,z,t) in weight-tensor order (host-only).
 * out_k (host, nullable) receives *out_n values; out_n (host) receives the count. */
int fno_mode_indices(const fno_desc* desc, int axis, int32_t* out_k, int32_t* out_n);

/* Spectral convolution, eq. (3):  y = K(phi) x.
 *   x         in   float  [B][Cin][Nx][Ny][Nz][Nt]
 *   R         in   cfloat [Cin][Cout][Lx][Ly][Lz][mt]
 *   y         out  float  [B][Cout][Nx][Ny][Nz][Nt]
 *   xhat_save out  cfloat [B][Cin][Lx][Ly][Lz][mt], nullable: the kept forward spectrum F x */
int fno_spectral_conv_fwd(const fno_desc* desc, const float* x, const float* R, float* y,
                          float* xhat_save, void* ws, size_t ws_bytes, void* stream);

/* Adjoint of the spectral convolution (eq. (7): the transposed transform chain).
 *   x          in  float, used only when xhat_saved is NULL (then F x is recomputed)
 *   xhat_saved in  cfloat [B][Cin][Lx][Ly][Lz][mt], nullable
 *   gy         in  float  [B][Cout][grid]     dL/dy
 *   gx         out float  [B][Cin][grid]      dL/dx, nullable
 *   gR         out cfloat [Cin][Cout][modes]  dL/dRe R + i dL/dIm R, nullable (overwritten, or added
 *                                             to with FNO_FLAG_ACCUMULATE_GRADS) */
int fno_spectral_conv_bwd(const fno_desc* desc, const float* x, const float* xhat_saved,
                          const float* R, const float* gy, float* gx, float* gR,
                          void* ws, size_t ws_bytes, void* stream);

/* One FNO block, eq. (2):  out = sigma(W x + b + K(phi) x), Cin == Cout.
 *   W  in float [Cout][Cin]     b  in float [Cout], nullable (= 0)
 *   out        out float [B][Cout][grid]
 *   z_save     out float [B][Cout][grid], nullable: the pre-activation, needed by fno_block_bwd
 *   xhat_save  out cfloat, nullable, as above */
int fno_block_fwd(const fno_desc* desc, const float* x, const float* R, const float* W,
                  const float* b, float* out, float* z_save, float* xhat_save,
                  void* ws, size_t ws_bytes, void* stream);

/* Adjoint of the block.  z_saved is the pre-activation from fno_block_fwd; gout is dL/dout, or
 * with FNO_FLAG_MSE_TARGET the target field of a mean-squared-error loss.
 *   gx out float [B][Cin][grid], gR out cfloat [Cin][Cout][modes], gW out float [Cout][Cin],
 *   gb out float [Cout]; each nullable, each overwritten (gR, gW, gb added to instead with
 *   FNO_FLAG_ACCUMULATE_GRADS).  gW and gb are sums over all batch
 *   entries and grid points (the adjoint of broadcasting W and b, Sec. 2.1), reduced in a fixed
 *   order so repeated calls give identical bits. */
int fno_block_bwd(const fno_desc* desc, const float* x, const float* R, const float* W,
                  const float* z_saved, const float* xhat_saved, const float* gout,
                  float* gx, float* gR, float* gW, float* gb,
                  void* ws, size_t ws_bytes, void* stream);

/* Channel lift of Sec. 2.4 (eq. (11)):  y[b][o][p] = sum_i W[o][i] x[b][i][p] + bias[o] over
 * npoints contiguous points per channel.  bias nullable.  c_out <= 32. */
int fno_pointwise_linear(int32_t batch, int32_t c_in, int32_t c_out, int64_t npoints,
                         const float* x, const float* W, const float* bias, float* y, void* stream);

/* Input lifts of Sec. 2.4 (eqs. (8)-(9)), fused: the input a [B][c_in][nspace] has a time axis of
 * length one; a_1 = Wt a + bt along time (Wt, bt: nt values each), then the channel lift
 * nu = Wc a_1 + bc (Wc [c_out][c_in], bc [c_out]) gives out [B][c_out][nspace][nt], t contiguous.
 * All pointers are device pointers owned by the caller; bt and bc nullable; out 16-byte aligned
 * when nt is a multiple of 4; c_out <= 32.  Asynchronous on `stream`; nothing is launched on an
 * argument error. */
int fno_time_lift(int32_t batch, int32_t c_in, int32_t c_out, int64_t nspace, int32_t nt, const float* a,
                  const float* Wt, const float* bt, const float* Wc, const float* bc, float* out,
                  void* stream);

/* Adjoint of fno_time_lift (Sec. 2.4, eqs. (8)-(9); sums over broadcast axes, Sec. 2.1) with
 * respect to its parameters, for a cotangent g [B][c_out][nspace][nt] of its output:
 *   gbc[o] = sum g,  gWc[o][i] = sum g (Wt[t] a[b][i][s] + bt[t]),
 *   gWt[t] = sum g Wc[o][i] a[b][i][s],  gbt[t] = sum g Wc[o][i]
 * (each over every index not on the left).  The input a is data: its gradient is not formed.
 * Every output is nullable and overwritten; fixed summation order, the same bits on every run.
 * ws: device scratch of fno_time_lift_bwd_workspace_bytes(c_in, c_out, nt) bytes, 8-byte aligned,
 * owned by the caller.  c_in <= 8, batch <= 1024.  Asynchronous on `stream`; nothing is
 * launched on an argument error. */
int fno_time_lift_bwd_workspace_bytes(int32_t c_in, int32_t c_out, int32_t nt, size_t* bytes);
int fno_time_lift_bwd(int32_t batch, int32_t c_in, int32_t c_out, int64_t nspace, int32_t nt, const float* a,
                      const float* Wt, const float* bt, const float* Wc, const float* g, float* gWt,
                      float* gbt, float* gWc, float* gbc, void* ws, size_t ws_bytes, void* stream);

/* Adjoints of fno_pointwise_linear and fno_pointwise_mlp2 (what the backward of a whole network
 * needs around its blocks).  For a cotangent g of the output:
 *   linear:  gx = W^T g  [B][c_in][npoints];  gW[o][i] = sum g[b][o][p] x[b][i][p];  gb[o] = sum g
 *   mlp2:    with h = W1 x + b1:  gW2[o][k] = sum g_o gelu(h_k), gb2 = sum g,
 *            gh = (W2^T g) gelu'(h), gW1[k][i] = sum gh_k x_i, gb1 = sum gh, gx = W1^T gh.
 * The sums run over all batch entries and points (the adjoint of broadcasting the weights,
 * Sec. 2.1) in a fixed order: the same bits on every run.  Every output is nullable and
 * overwritten.  ws: device scratch of fno_pointwise_bwd_workspace_bytes(c_in, hidden, c_out)
 * bytes (hidden = 0 for the linear map), 8-byte aligned, owned by the caller.  Widths: c_in,
 * c_out <= 32 (linear); c_in <= 32, c_out <= 4, hidden <= 1024 (mlp2). */
int fno_pointwise_bwd_workspace_bytes(int32_t c_in, int32_t hidden, int32_t c_out, size_t* bytes);
int fno_pointwise_linear_bwd(int32_t batch, int32_t c_in, int32_t c_out, int64_t npoints, const float* x,
                             const float* W, const float* g, float* gx, float* gW, float* gb, void* ws,
                             size_t ws_bytes, void* stream);
int fno_pointwise_mlp2_bwd(int32_t batch, int32_t c_in, int32_t hidden, int32_t c_out, int64_t npoints,
                           const float* x, const float* W1, const float* b1, const float* W2, const float* g,
                           float* gx, float* gW1, float* gb1, float* gW2, float* gb2, void* ws,
                           size_t ws_bytes, void* stream);

/* Relative L2 misfit of Sec. 4 over n floats:  loss = ||pred - target||_2 / ||target||_2, written to
 * the device scalar `loss` (nullable), and its gradient with respect to pred,
 * (pred - target) / (||pred - target||_2 ||target||_2), written to grad (nullable, n floats; all
 * zero when pred equals target).  The sums are accumulated in double in a fixed order: the same
 * bits on every run.  ws: device scratch of fno_rel_l2_workspace_bytes() bytes, 8-byte aligned,
 * owned by the caller.  A zero target gives the IEEE result of the division.  Asynchronous on
 * `stream`; nothing is launched on an argument error. */
int fno_rel_l2_workspace_bytes(size_t* bytes);
int fno_rel_l2_loss(int64_t n, const float* pred, const float* target, float* loss, float* grad,
                    void* ws, size_t ws_bytes, void* stream);

/* One step of Adam (the optimiser of Sec. 4; Kingma & Ba, Algorithm 1) in place on n floats:
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 *   param -= lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps).
 * step counts from 1.  Complex parameters (the spectral weights) are passed as 2n floats: real
 * and imaginary parts are updated as separate reals.  All pointers are device pointers owned by
 * the caller. */
int fno_adam_step(int64_t n, float* param, const float* grad, float* m, float* v, double lr, double beta1,
                  double beta2, double eps, int32_t step, void* stream);

/* Projection to the output channels (end of Sec. 2.4) through one hidden layer, fused per point:
 *   y = W2 gelu(W1 x + b1) + b2,  W1 [hidden][c_in], W2 [c_out][hidden].  The hidden tensor is
 * never stored.  c_in <= 32, c_out <= 4. */
int fno_pointwise_mlp2(int32_t batch, int32_t c_in, int32_t hidden, int32_t c_out, int64_t npoints,
                       const float* x, const float* W1, const float* b1, const float* W2,
                       const float* b2, float* y, void* stream);

/* For callers that cannot allocate device memory or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): fno_spectral_conv_fwd with the
 * workspace taken from a fixed array of FNO_STATIC_SCRATCH_BYTES bytes of device memory that the
 * library owns (one copy per GPU it runs on, held until the process ends).  Arguments, layout,
 * results and error codes are those of fno_spectral_conv_fwd; the call allocates and frees
 * nothing.  Shapes whose fno_workspace_bytes(FNO_OP_SPECTRAL_CONV_FWD) exceeds the array are
 * refused with FNO_ENOSPC and nothing is launched.  The first call on a device looks up the
 * array's address there (make that call outside any capture).  All calls on one GPU share the
 * array: every byte a call reads from it is written earlier by the same call, so leftovers of the
 * previous call do no harm, but two calls that overlap in time on one GPU (different streams or
 * threads) race; order them. */
#define FNO_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int fno_spectral_conv_fwd_static(const fno_desc* desc, const float* x, const float* R, float* y,
                                 float* xhat_save, void* stream);

/* Benchmark hooks, outside the paper's layer: per-stage timing.  While enabled, every library call brackets each kernel it
 * launches with a pair of HIP events on the call's stream (events are created on first use and
 * kept).  fno_timing_enable takes a mask of stages, bit (1 << FNO_STAGE_*) per stage, FNO_TIMING_ALL
 * for every stage, 0 to switch timing off: an event pair costs a few microseconds of idle time
 * between kernels, so a caller that times a whole step and wants one kernel's duration from the
 * same run enables that stage alone.  fno_timing_read waits for the recorded events, returns up to `capacity` records in
 * launch order (stage id FNO_STAGE_*, elapsed milliseconds; host arrays) and clears the log.
 * This log is the library's only process-wide state and is not thread-safe; leave it disabled
 * under graph capture.  At most 8192 records are kept between reads. */
enum {
  FNO_STAGE_TZ_FWD = 0, FNO_STAGE_Y_FWD = 1, FNO_STAGE_X_FWD = 2, FNO_STAGE_MIX = 3,
  FNO_STAGE_X_INV = 4, FNO_STAGE_Y_INV = 5, FNO_STAGE_ZT_INV = 6, FNO_STAGE_MIX_BWD = 7,
  FNO_STAGE_BWD_POINTWISE = 8
};
#define FNO_TIMING_ALL (-1)
int fno_timing_enable(int stage_mask);
int fno_timing_read(int32_t* stages, float* ms, int32_t capacity, int32_t* count);

/* Text for a status code; for FNO_EHIP / FNO_EUNSUPPORTED the calling thread's last detail. */
const char* fno_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FNO_H_ */
