/*
 * mgrit.h -- C ABI of the layer-parallel multigrid (MGRIT-FAS) solver for residual networks
 *            u^{n+1} = u^n + h F(u^n; theta^n),  n = 0..N-1          (paper Sec. II, Eq. (1))
 * on one AMD MI355X (gfx950).  Plain C: only pointers and sizes cross this boundary.
 *
 * Index convention.  N layer steps, N+1 states u^0..u^N ("points" 0..N), parameters
 * theta^0..theta^{N-1}.  The coarsening factor (the paper's c, Sec. III-C) is called m here.
 * Level l has N_l = N / m^l steps and step size h_l = m^l h; point j of level l is fine
 * point j m^l and uses theta^{j m^l} (injection of states, residuals and parameters,
 * Sec. III-C, Eq. (23)).
 *
 * Memory.  The caller owns every buffer.  Pointers marked "device" are HIP device pointers
 * aligned to 256 bytes; pointers marked "host" are ordinary host pointers.  The library
 * allocates no device memory and keeps no state of a solve between calls.  What it does keep, per
 * process, is bookkeeping: for every kernel that needs more than 64 KB of LDS, the largest size it
 * has been raised to on each device (the opt-in is a per-device attribute of the kernel, set at
 * the first launch that needs it), and the optional launch trace at the end of this file.  None
 * of this is guarded: call the library from one host thread at a time.  All device work is enqueued
 * on `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).  A call that
 * writes a host output (resnorm_hist, iters_done, norm_out) synchronises that stream before
 * it returns; otherwise it returns with its work in flight on the stream.  Such a call (tol <= 0,
 * no host outputs) consists of kernel launches only, so it may be recorded into a HIP graph by
 * stream capture and replayed.  Run the same call once outside the capture first: the first launch of
 * a kernel that uses more than 64 KB of LDS sets an attribute of that kernel on the current device.
 *
 * Environment (diagnostic switches, read at every call; results agree with the default path to rounding).
 * MGRIT_NO_SWEEP=1 makes the library use one launch per layer step also where it would fuse the steps of an
 * F-relaxation sweep into one launch (dense layers of width 128 or 256, or float convolution layers of at
 * most 16 channels on images of at most 832 pixels, with many coarse intervals).  MGRIT_SWEEP_WAVES=4 runs
 * the fused sweep of width 256 with four instead of eight wavefronts.  MGRIT_GRAD_NARROW=1 keeps the
 * parameter gradient of dense layers of width 512 and more on the 128x128 tiles of narrower layers.
 * MGRIT_MASKED_STEP=1 sends dense layer steps whose batch, width and contraction length are whole multiples of
 * the tile through the bounds-masked loop that ragged shapes use.
 * MGRIT_STEP_REREAD=1 makes the epilogue of the bf16 128x128 dense tile read the state for the skip connection
 * from memory again instead of keeping it in registers from the contraction loop.
 * MGRIT_CGRAD_WAVES=4 runs the parameter gradient of convolution layers with more than 32 channels with four
 * wavefronts per workgroup, as for narrower layers, instead of eight.
 * MGRIT_CONV_GENERIC=1 keeps bf16 convolution layers of 64 channels on the kernel that takes the channel count at
 * run time instead of the one compiled for 64.
 * MGRIT_ADJ_TRANSPOSED=1 runs the adjoint of dense and fully connected layers on transposed copies of their
 * weights, made in the workspace at every call, instead of reading the caller's arrays along their slow index;
 * the workspace queries then include those copies, so set it before the query as well as before the call.
 *
 * Layouts (all row-major, last index fastest):
 *   dense: state [B][q] float;  W [N][q_out][q_in];  b [N][q] float
 *   conv : state [B][Himg][Wimg][C] float (NHWC);  W [N][C_out][3][3][C_in];  b [N][C] float
 *          3x3, stride 1, one pixel of zero padding, cross-correlation:
 *          z[b,y,x,o] = sum_{dy,dx,i} W[o][dy][dx][i] u[b,y+dy-1,x+dx-1,i] + b[o]
 *   W is float when dtype = MGRIT_FP32 and bf16 (upper 16 bits of a float, 2 bytes) when
 *   dtype = MGRIT_BF16.  With MGRIT_BF16 the matrix-core operands (weights and the state
 *   operand of the affine map; in the parameter gradient G = act' * Lam and U, and for conv
 *   layers also the G that is summed into db) are rounded to bf16 and everything else --
 *   accumulation, bias, activation, the skip add, states, residuals, corrections -- is float.
 *   State arrays over points are [N+1][state].
 *
 * Return value of every int32_t function: MGRIT_OK or one of the negative codes below.
 * Nothing is printed and nothing is thrown.
 */
#ifndef MGRIT_H
#define MGRIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MGRIT_OK = 0,
  MGRIT_ERR_POINTER = -1,     /* required pointer NULL or not 256-byte aligned              */
  MGRIT_ERR_PROBLEM = -2,     /* invalid problem: N < 1, m < 2, bad enum, sizes <= 0, ...    */
  MGRIT_ERR_WORKSPACE = -3,   /* workspace smaller than mgrit_*_workspace_bytes()            */
  MGRIT_ERR_UNSUPPORTED = -4, /* valid request that this build does not implement            */
  MGRIT_ERR_NONFINITE = -5,   /* a residual norm came out NaN or Inf                         */
  MGRIT_ERR_HIP = -6          /* a HIP runtime call failed                                   */
};

enum { MGRIT_RELAX_F = 0, MGRIT_RELAX_FCF = 1 };           /* Sec. III-C, Fig. 3, Alg. 1 step 1 */
enum { MGRIT_NORM_L2 = 0, MGRIT_NORM_RMS = 1 };            /* RMS = L2 / sqrt(#entries)         */
enum { MGRIT_LAYER_DENSE = 0, MGRIT_LAYER_CONV3X3 = 1 };
enum { MGRIT_ACT_TANH = 0, MGRIT_ACT_RELU = 1 };
enum { MGRIT_FP32 = 0, MGRIT_BF16 = 1 };
enum { MGRIT_INIT_ZERO = 0, MGRIT_INIT_COPY = 1, MGRIT_INIT_USER = 2, MGRIT_INIT_NESTED = 3 };
enum { MGRIT_MAX_LEVELS = 16 };

typedef struct mgrit_problem {
  int32_t N;           /* layer steps, >= 1 (at most 65535 in this build)     (Sec. II, Eq. (1)) */
  float   h;           /* fine step size                                      (Sec. II, Eq. (1)) */
  int32_t m;           /* coarsening factor, >= 2                             (Sec. III-C)       */
  int32_t max_levels;  /* 1 = serial propagation, 2 = two-level scheme of Alg. 1,
                          > 2 = the scheme applied recursively (V-cycle)      (Sec. III-A)       */
  int32_t min_coarse;  /* a level with N_l <= min_coarse is not coarsened further; values < 1
                          act as 1                                                               */
  int32_t relax;       /* MGRIT_RELAX_F or MGRIT_RELAX_FCF                    (Alg. 1 step 1)    */
  int32_t cycle;       /* 0 = V-cycle (the only one defined)                                     */
  int32_t max_iter;    /* number of cycles; with tol > 0 an upper bound       (Sec. IV-A)        */
  float   tol;         /* > 0: stop after the first cycle whose residual norm is <= tol
                          (Alg. 1 step 6); <= 0: run exactly max_iter cycles                     */
  int32_t norm_kind;   /* MGRIT_NORM_L2 or MGRIT_NORM_RMS                                        */
  int32_t layer;       /* MGRIT_LAYER_DENSE or MGRIT_LAYER_CONV3X3                                */
  int32_t act;         /* MGRIT_ACT_TANH or MGRIT_ACT_RELU                                       */
  int32_t dtype;       /* MGRIT_FP32 or MGRIT_BF16                                               */
  int32_t B, q;        /* dense: batch and width                                                 */
  int32_t C, Himg, Wimg; /* conv: channels, image height and width                               */
  int32_t init;        /* initial guess of the fine C-points: MGRIT_INIT_ZERO, MGRIT_INIT_COPY
                          (every C-point := the known end value u^0, resp. lambda^N),
                          MGRIT_INIT_USER (take them from the in/out array) or MGRIT_INIT_NESTED
                          (nested iteration: the coarsest level's equation L(V) = (u^0, 0, .., 0)
                          with its own step size is solved in sequence; going up, the C-points of
                          each level take the coarser level's values and its F-points follow by
                          F-relaxation, Sec. III-A / III-C; the paper prints no start-up procedure.
                          Costs N_coarsest + sum over the middle levels of N_l (m-1)/m layer steps) */
} mgrit_problem_t;

/* Level hierarchy (Sec. III-C: every m-th layer of a level is also a member of the next
 * coarser level).  Coarsening goes on while fewer than max_levels levels exist and the level
 * has more than min_coarse steps and at least m of them; N_{l+1} = floor(N_l / m), and a level
 * whose size is not a multiple of m ends in N_l mod m trailing F-points, which F-relaxation
 * updates behind the last C-point (a case the paper does not treat).  This is the hierarchy of
 * the forward solve; the adjoint solve uses the mirror image, counted from layer N (its
 * level-l points are the fine points N - j m^l).
 * Host only, integer only.  n_levels <- number of levels L; N_l[l] <- steps
 * on level l (array of MGRIT_MAX_LEVELS entries); fine_index <- concatenation over levels of
 * the fine point index of every point, sum_l (N_l + 1) entries.  N_l and fine_index may be
 * NULL (then only the count is returned).  Errors: MGRIT_ERR_PROBLEM. */
int32_t mgrit_level_map(const mgrit_problem_t* p, int32_t* n_levels, int32_t* N_l, int32_t* fine_index);

/* Bytes of device workspace the forward solve / residual norm, and the adjoint solve, need
 * for this problem; 0 if the problem is invalid.  Host only. */
size_t mgrit_workspace_bytes(const mgrit_problem_t* p);
size_t mgrit_adjoint_workspace_bytes(const mgrit_problem_t* p);

/* Forward solve of L_h(U) = f_h = (u0, 0, .., 0) (Sec. III-C, Eq. (18)) by max_iter FAS cycles
 * of Alg. 1: relaxation, residual at the C-points, injection, coarse FAS equation
 * L_H(V) = L_H(U_H) + R_H (Eq. (24)) solved recursively / serially on the coarsest level,
 * C-point correction, F-relaxation.  With max_levels = 1 this is serial propagation.
 *   W, b      device, read only
 *   u0        device [state], read only
 *   U         device [(N+1)][state]; out; with init = MGRIT_INIT_USER also in (its C-points)
 *   resnorm_hist  host [max_iter] or NULL; entry k <- norm of the C-point residual of the fine
 *             level evaluated in cycle k after relaxation and before the correction
 *   iters_done    host or NULL; <- cycles run
 *   workspace device, workspace_bytes >= mgrit_workspace_bytes(p)
 * Errors: all codes above; on MGRIT_ERR_NONFINITE U holds the diverged iterate. */
int32_t mgrit_fas_forward(const mgrit_problem_t* p, const void* W, const float* b, const float* u0,
                          float* U, double* resnorm_hist, int32_t* iters_done,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* The forward solve for callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: mgrit_fas_forward without the workspace argument.  Its
 * workspace is a fixed array of MGRIT_STATIC_SCRATCH_BYTES in device memory that belongs to the library; every
 * GPU the library runs on holds one copy until the process ends.  The call itself allocates and frees nothing,
 * on the device or through any allocating runtime call; inputs and outputs are the caller's as above, results are
 * those of mgrit_fas_forward (same kernels, same schedule).
 *   - MGRIT_ERR_WORKSPACE if mgrit_workspace_bytes(p) exceeds MGRIT_STATIC_SCRATCH_BYTES (the plain dense
 *     q = 256, N = 256, B = 128 workload needs 32 MB; the two large benchmark workloads do not fit).
 *   - The first call on a device looks up the address of that device's copy of the array; make it outside
 *     a stream capture (the same rule as for the LDS attribute above).  With tol <= 0 and both host outputs
 *     NULL the call is kernel launches only.
 *   - All calls on one GPU share that GPU's array, whatever their streams: calls that overlap in time on one
 *     GPU race on it.  Nothing in it has to be cleared between calls -- every part is written before it is
 *     read -- so a call may follow one with a different problem.
 * Errors otherwise as mgrit_fas_forward; MGRIT_ERR_UNSUPPORTED for a device index above 63. */
enum { MGRIT_STATIC_SCRATCH_BYTES = 64 * 1024 * 1024 };
int32_t mgrit_fas_forward_static(const mgrit_problem_t* p, const void* W, const float* b, const float* u0,
                                 float* U, double* resnorm_hist, int32_t* iters_done, void* hip_stream);

/* Adjoint (backward) solve by the same cycle on the reversed layer axis.  The paper states
 * that the multigrid removes the serial backward propagation as well (Sec. III-C) and prints
 * no equations; the system solved is the exact reverse-mode derivative of Eq. (1):
 *   z^n = A_n U^n + b_n,  G^n = act'(z^n) * Lam^{n+1},  Lam^n = Lam^{n+1} + h A_n^T G^n,
 * with terminal value Lam^N = lamN, linearised about the given states U (converged or not);
 * the level-l step from point j+1 to point j uses U and theta of fine point j m^l and step h_l.
 * Afterwards dW[n] = h G^n (U^n)^T (summed over the batch / batch and pixels) and
 * db[n] = h sum G^n from the final Lam.
 *   U     device [(N+1)][state], read only      lamN  device [state], read only
 *   Lam   device [(N+1)][state]; out (in for init = MGRIT_INIT_USER)
 *   dW    device float, same shape as W (dense [N][q][q], conv [N][C][3][3][C]), overwritten, or NULL;
 *         db like b, or NULL
 *   workspace_bytes >= mgrit_adjoint_workspace_bytes(p)
 * resnorm_hist / iters_done as above (residual of the adjoint system). */
int32_t mgrit_fas_adjoint(const mgrit_problem_t* p, const void* W, const float* b, const float* U,
                          const float* lamN, float* Lam, float* dW, float* db,
                          double* resnorm_hist, int32_t* iters_done,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* || f_h - L_h(U) || over all N+1 points of the fine level (Sec. III-C, Eq. (19); Sec. IV-A).
 *   norm_out  host, required.  Always synchronises the stream. */
int32_t mgrit_residual_norm(const mgrit_problem_t* p, const void* W, const float* b, const float* u0,
                            const float* U, double* norm_out,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- Stacks that mix convolution layers with periodic fully connected layers (Sec. IV-E: blocks of one
 * fully connected layer with equal input and output size followed by a run of residual convolution layers).
 * The problem is a MGRIT_LAYER_CONV3X3 problem; in addition every fc_period-th layer, n = 0, fc_period,
 * 2 fc_period, ... < N, is a fully connected layer acting on the flattened sample,
 *   u^{n+1}[b] = u^n[b] + h act(Wfc_k vec(u^n[b]) + bfc_k),   k = n / fc_period,
 * vec = the sample's [Himg][Wimg][C] values in storage order, d = Himg*Wimg*C of them.  The paper does not say
 * whether its fully connected layers carry the skip connection; here they do, so that every layer has the form of
 * Eq. (1).  Coarse levels inject layers as before (a coarse step uses the kind and parameters of its first fine
 * layer).  The slots of W, b (and dW, db) at the fully connected layers' indices keep the [N] layout: their
 * input values are ignored, and dW, db are written as zero there.
 *   fc_period  >= 2;  n_fc = ceil(N / fc_period)
 *   Wfc   device [n_fc][d][d] ([out][in], element type as W)   bfc   device [n_fc][d] float
 *   dWfc  device float [n_fc][d][d], dbfc device [n_fc][d]: adjoint only, overwritten; computed when dW / db are
 *         (dWfc with dW, dbfc with db) and then required
 * MGRIT_ERR_UNSUPPORTED if d*d exceeds 2^31 - 1.  Everything else is as in the plain entry points. */
typedef struct mgrit_fc_layers {
  int32_t     fc_period;
  const void* Wfc;
  const float* bfc;
  float*      dWfc;
  float*      dbfc;
} mgrit_fc_layers_t;

size_t  mgrit_workspace_bytes_mixed(const mgrit_problem_t* p, int32_t fc_period);
size_t  mgrit_adjoint_workspace_bytes_mixed(const mgrit_problem_t* p, int32_t fc_period);
int32_t mgrit_fas_forward_mixed(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                                const float* u0, float* U, double* resnorm_hist, int32_t* iters_done,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
int32_t mgrit_fas_adjoint_mixed(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                                const float* U, const float* lamN, float* Lam, float* dW, float* db,
                                double* resnorm_hist, int32_t* iters_done,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
int32_t mgrit_residual_norm_mixed(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W,
                                  const float* b, const float* u0, const float* U, double* norm_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Diagnostic launch tracing, off by default and the one piece of state the library keeps: between
 * mgrit_trace_begin() and mgrit_trace_end() every layer-step and gradient launch is bracketed by a
 * pair of HIP events on its stream.  mgrit_trace_end synchronises on the last event and returns,
 * per kernel class (MGRIT_TRACE_*), the summed elapsed milliseconds, the number of launches, the
 * number of layer steps (groups) they processed and (bytes, may be NULL) their algorithmic bytes --
 * per layer step the layer's weights and bias, the input state, every fused epilogue operand, the
 * act' factor and the output, each moved once; arrays of n_classes entries, host.  Not thread
 * safe; meant for the benchmark's roofline figures (Sec. IV-B reports such a timeline). */
enum {
  MGRIT_TRACE_DENSE_F32_T64 = 0, MGRIT_TRACE_DENSE_F32_T128, MGRIT_TRACE_DENSE_BF16_T64,
  MGRIT_TRACE_DENSE_BF16_T128, MGRIT_TRACE_CONV_F32, MGRIT_TRACE_CONV_BF16, MGRIT_TRACE_GRAD,
  MGRIT_TRACE_SWEEP_F32, MGRIT_TRACE_SWEEP_BF16, MGRIT_TRACE_DENSE_F32_KSPLIT8,
  MGRIT_TRACE_DENSE_F32_KSPLIT, MGRIT_TRACE_DENSE_BF16_KSPLIT, MGRIT_TRACE_DENSE_BF16_KSPLIT8,
  MGRIT_TRACE_CONV_SWEEP_F32, MGRIT_TRACE_NCLASS
};
void    mgrit_trace_begin(void);
int32_t mgrit_trace_end(double* ms, int64_t* launches, int64_t* units, double* bytes, int32_t n_classes);

#ifdef __cplusplus
}
#endif
#endif /* MGRIT_H */
