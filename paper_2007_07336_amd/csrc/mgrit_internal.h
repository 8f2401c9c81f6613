// Internal declarations shared by the host schedule and the HIP kernels of the MGRIT-FAS
// library.  Not part of the public C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mgrit {

// Affine map from the group index of a launch to a point (or layer) index of an array that
// is laid out [points][E]:  idx = base + gi * stride.  A negative stride walks the layer
// axis backwards (adjoint sweeps).
struct PtMap {
  long long base;
  long long stride;
};

// One layer-batched step launch: every group gi evaluates, for its own input point and its
// own layer parameters,
//     z   = A_layer * (Dm ? Dm .* X : X) + bias
//     phi = X + hs * act(z)                                   (Sec. II, Eq. (1))
//     out = sp * phi + c1 * E1 + c2 * E2                      (mode PHI)
//     out = act'(z)                                           (mode DACT)
// which covers F-/C-relaxation, the C-point residual, the FAS right-hand side and the adjoint
// steps (Sec. III-B, III-C).  If norm_partial is set, every workgroup also writes the sum of
// out^2 over its tile to norm_partial[linear block index].
struct StepArgs {
  const float* X;   PtMap xm;
  const float* Dm;  PtMap dm;      // optional elementwise multiplier of the matrix operand (the act' cache);
                                   // its storage type is the weights' type: float, or bf16 when dbf16 is set
  const void*  W;   PtMap wm;      // weights of layer wm(gi); element type = template parameter
  int wn;                          // dense only, 1: W holds W[k][n] (contraction index slowest), as the adjoint reads the
                                   // caller's weights without a transposed copy; 0: W[n][k].  Needs K == Nf and Dm.
  const float* bias;               // [layers][Nf] or null (same layer index as W)
  float* Out;       PtMap om;      // may be null when only the norm is wanted
  const float* E1;  PtMap e1m;  float c1;
  const float* E2;  PtMap e2m;  float c2;
  float sp, hs;
  float* norm_partial;
  int mode;                        // MODE_PHI / MODE_DACT
  int act;                         // 0 tanh, 1 relu, 2 identity
  int M;                           // rows per state: B (dense) or B*Himg*Wimg (conv)
  int Nf;                          // features per row: q (dense) or C (conv)
  int K;                           // contraction length per output: q or 9*C
  int Himg, Wimg, TH;              // conv only: image size and rows of an output tile
  unsigned wmagic;                 // conv only: ceil(2^20 / Wimg), filled in by the launch wrapper
  int tiles;                       // workgroups per group (filled in by the launch wrapper)
  int dbf16;                       // 1: Dm (input) and the output of MODE_DACT are bf16 arrays
  int wstream;                     // 1: all layers' weights together exceed the last-level cache, load them
                                   // non-temporally; 0: they fit and later launches of the solve find them there
  int skip0, skipper;              // conv only, skipper > 0: groups skip0, skip0 + skipper, ... do nothing (their
                                   // layer is a fully connected one, served by a dense launch) and write 0 to
                                   // their norm partials
  long long E;                     // M * Nf
  long long wsize;                 // Nf * K elements per layer
};

enum { MODE_PHI = 0, MODE_DACT = 1 };
enum { ACT_TANH = 0, ACT_RELU = 1, ACT_IDENT = 2 };

// Parameter gradient launch (one group per layer n):
//   G = Dm[n] .* Lam[n+1];  dW[n] = hs * G^T (*) U[n];  db[n] = hs * sum G
struct GradArgs {
  const float* U;   PtMap um;
  const float* Lam; PtMap lm;
  const float* Dm;  PtMap dm;        // act' cache in the weights' type (float, or bf16 for a bf16 problem)
  float* dW;                        // [layers][Nf][K] float
  float* db;                        // [layers][Nf] or null
  float hs;
  int M, Nf, K, Himg, Wimg, B;
  int tiles;                        // workgroups per layer (filled in by the launch wrapper)
  long long E, wsize;
  // conv, all taps in one workgroup (filled in by the launch wrapper from conv_grad_geom)
  float* partial;                   // [chunks][layers][wsize] partial sums when a layer is split into chunks
  int layers;
  int gWp, gR, gKL, gPU, gPG, gspi, gslabs, gchunks, gspc;
};
// Geometry of the conv gradient kernel that forms all nine taps in one workgroup: a slab is gR image rows
// of one image (row pitch gWp, a multiple of 8), the contraction over a slab runs over gKL pixel slots,
// the layer's slabs are split into `chunks` workgroups whose partial sums a second kernel adds in a fixed order.
struct ConvGradGeom {
  int Wp, R, KL, PU, PG, spi, slabs, chunks, spc;
  size_t smem;
  bool ok;                          // false: image row too wide for this kernel (one workgroup per tap is used)
};
ConvGradGeom conv_grad_geom(int B, int Himg, int Wimg, int C, int dtype, int layers);
size_t     conv_grad_partial_bytes(int B, int Himg, int Wimg, int C, int dtype, int layers);

// ---- launch wrappers (defined in mgrit_kernels.hip); all enqueue on `s` and return the HIP status
hipError_t launch_step(const StepArgs& a, int layer_kind, int dtype, int groups, hipStream_t s);
int        step_grid_blocks(const StepArgs& a, int layer_kind, int dtype, int groups);  // workgroups per group
int        conv_tile_rows(int Himg, int Wimg, int C, int dtype);            // TH, or 0 if unsupported
hipError_t launch_grad(const GradArgs& a, int layer_kind, int dtype, int groups, hipStream_t s);

// out[om(gi)] = in[im(gi)]                      (injection restriction, initial guesses)
hipError_t launch_copy_points(float* out, PtMap om, const float* in, PtMap im, long long E, int groups,
                              hipStream_t s);
hipError_t launch_copy_points_norm(float* out, PtMap om, const float* in, PtMap im, long long E, int groups,
                                   const float* partial, int n, double scale, double* nout, hipStream_t s);
// out[om(gi)] = 0
hipError_t launch_zero_points(float* out, PtMap om, long long E, int groups, hipStream_t s);
// U[um(gi)] += V[vm(gi)] - U[um(gi)]  evaluated as  U + (V - U)      (C-point correction)
hipError_t launch_correct(float* U, PtMap um, const float* V, PtMap vm, long long E, int groups,
                          hipStream_t s);
// partial[slot0 + block] = sum over this block's chunk of (a - b)^2 ; returns blocks used
hipError_t launch_diff_sq(const float* a, const float* b, long long n, float* partial, int* blocks_used,
                          hipStream_t s);
int        diff_sq_blocks(long long n);
// out[0] = sqrt(sum_{i<n} partial[i]) * scale, summed in a fixed order in double
hipError_t launch_norm_final(const float* partial, int n, double scale, double* out, hipStream_t s);
// transposed parameter copies for the adjoint: dense Wt[n][i][o] = W[n][o][i];
// conv Kt[n][i][2-dy][2-dx][o] = K[n][o][dy][dx][i]
hipError_t launch_transpose_weights(const void* W, void* Wt, int layer_kind, int dtype, int layers, int Nf,
                                    hipStream_t s);

// Fused F-relaxation sweep (dense layers): workgroup (interval ci, slice of 32 batch rows) starts from
// S[sm(ci)] and performs nsteps layer steps in sequence with the state slice resident in LDS -- a dense
// layer acts on every batch row by itself, so the slices of an interval never exchange anything:
//   step k = 1..nsteps:  u <- u + hs * act(A_layer (Dm_layer .* u) + bias_layer) + G[gb + ci*gs + k]
//   layer(k) = lb + ci*ls + (k-1)*lk;   the state after step k is stored to X[xb + ci*xs + k*xk]
// One launch replaces the nsteps lockstep launches of a sweep (Sec. III-C, Fig. 3).
struct SweepArgs {
  const float* S;  PtMap sm;
  float* X;  long long xb, xs, xk;
  const float* G;  long long gb, gs;     // optional right-hand side (null: none)
  const void* W;  const float* bias;     // weights in the problem's type; bias may be null
  int wn;                                // dense sweep, 1: W holds W[k][n] (the adjoint on the caller's weights)
  const void* Dm;                        // optional act' factors in the weights' type, [layers][E]
  long long lb, ls, lk;
  float hs;
  int act, nsteps, nchains, M, q;
  long long E, wsize;
  int Himg, Wimg, C;                     // convolution sweep only (then M = images per state)
};
bool       sweep_supported(int q, int dtype);
int        sweep_blocks(int M, int nchains);
hipError_t launch_sweep(const SweepArgs& a, int dtype, hipStream_t s);
// The same for 3x3 convolution layers of at most 16 float channels on images small enough for one workgroup
// (a convolution needs its neighbours' rows, so the unit is a whole image): workgroup (interval ci, image).
bool       conv_sweep_supported(int Himg, int Wimg, int C, int dtype);
hipError_t launch_conv_sweep(const SweepArgs& a, hipStream_t s);

// launch tracing (diagnostic): kernel classes, and begin / collect
enum { TRACE_DENSE_F32_64 = 0, TRACE_DENSE_F32_128, TRACE_DENSE_BF16_64, TRACE_DENSE_BF16_128,
       TRACE_CONV_F32, TRACE_CONV_BF16, TRACE_GRAD, TRACE_SWEEP_F32, TRACE_SWEEP_BF16, TRACE_DENSE_F32_KS8,
       TRACE_DENSE_F32_KS, TRACE_DENSE_BF16_KS, TRACE_DENSE_BF16_KS8, TRACE_CONV_SWEEP_F32, TRACE_NCLASS };
void trace_begin();
int  trace_end(double* ms, long long* launches, long long* units, double* bytes, int ncls);
void trace_before(hipStream_t s);
void trace_after(hipStream_t s, int cls, long long units, double bytes);

}  // namespace mgrit
