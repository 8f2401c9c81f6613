// Host side of the MGRIT-FAS library: argument checks, the level hierarchy, the workspace
// layout and the launch schedule of the FAS V-cycle (forward and adjoint).  Every arithmetic
// step of the method runs in the HIP kernels of mgrit_kernels.hip; this file only decides
// which launch comes next.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/mgrit.h"
#include "mgrit_internal.h"

using namespace mgrit;

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
// MGRIT_ADJ_TRANSPOSED=1 in the environment: the adjoint of dense and fully connected layers runs on a transposed
// copy of the weights in the workspace (diagnostic; by default the kernels read the caller's array k-major)
inline bool adjoint_transposed_copy() {
  const char* e = getenv("MGRIT_ADJ_TRANSPOSED");
  return e && e[0] == '1';
}
inline bool aligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) % ALIGN) == 0; }

// The fused F-relaxation sweep (one launch per sweep instead of one per step) can be switched off with
// MGRIT_NO_SWEEP=1 in the environment; the tests run both ways.
inline bool sweep_enabled() {
  const char* e = getenv("MGRIT_NO_SWEEP");
  return !(e && e[0] == '1');
}

struct Plan {
  int L;
  int Nl[MGRIT_MAX_LEVELS];
  long long mpow[MGRIT_MAX_LEVELS];
  float hl[MGRIT_MAX_LEVELS];
  long long E, wsize;
  int M, Nf, K, TH;
  size_t esize;                        // bytes per weight element
  size_t off_X[MGRIT_MAX_LEVELS], off_g[MGRIT_MAX_LEVELS], off_R[MGRIT_MAX_LEVELS];
  size_t off_partial, n_partial, off_hist, off_Wt, off_D, off_gpart;
  size_t bytes_fwd, bytes_adj;
  // mixed stacks (Sec. IV-E): every fcP-th layer is fully connected on the flattened sample; 0 = none
  int fcP, nfc, B;
  long long dfc, wsize_fc;             // flattened sample size d and d*d
  size_t off_Wfct;                     // transposed fully connected weights (adjoint)
};

// Level hierarchy (Sec. III-C): coarsen by m while fewer than max_levels levels exist and the
// current level has more than min_coarse steps and at least one whole coarse interval.  Points
// 0, m, 2m, .. of a level are its C-points; a level whose size is not a multiple of m ends in
// fewer than m trailing F-points, and the next level has floor(N_l / m) steps.
int build_levels(const mgrit_problem_t* p, int* L, int* Nl) {
  if (!p) return MGRIT_ERR_POINTER;
  if (p->N < 1 || p->m < 2 || p->max_levels < 1 || p->max_levels > MGRIT_MAX_LEVELS) return MGRIT_ERR_PROBLEM;
  const int minc = p->min_coarse < 1 ? 1 : p->min_coarse;
  int n = 1;
  Nl[0] = p->N;
  while (n < p->max_levels && Nl[n - 1] > minc && Nl[n - 1] >= p->m) {
    Nl[n] = Nl[n - 1] / p->m;
    ++n;
  }
  *L = n;
  return MGRIT_OK;
}

int make_plan(const mgrit_problem_t* p, Plan* pl, int fcP = 0) {
  memset(pl, 0, sizeof(*pl));
  int rc = build_levels(p, &pl->L, pl->Nl);
  if (rc != MGRIT_OK) return rc;
  if (fcP != 0 && (fcP < 2 || p->layer != MGRIT_LAYER_CONV3X3)) return MGRIT_ERR_PROBLEM;
  if (!(p->h > 0.0f) || !isfinite(p->h)) return MGRIT_ERR_PROBLEM;
  if (p->N > 65535) return MGRIT_ERR_UNSUPPORTED;            // layers / points index one grid dimension of the transfer kernels
  if (p->relax != MGRIT_RELAX_F && p->relax != MGRIT_RELAX_FCF) return MGRIT_ERR_PROBLEM;
  if (p->cycle != 0 || p->max_iter < 1) return MGRIT_ERR_PROBLEM;
  if (p->norm_kind != MGRIT_NORM_L2 && p->norm_kind != MGRIT_NORM_RMS) return MGRIT_ERR_PROBLEM;
  if (p->layer != MGRIT_LAYER_DENSE && p->layer != MGRIT_LAYER_CONV3X3) return MGRIT_ERR_PROBLEM;
  if (p->act != MGRIT_ACT_TANH && p->act != MGRIT_ACT_RELU) return MGRIT_ERR_PROBLEM;
  if (p->dtype != MGRIT_FP32 && p->dtype != MGRIT_BF16) return MGRIT_ERR_PROBLEM;
  if (p->init < MGRIT_INIT_ZERO || p->init > MGRIT_INIT_NESTED) return MGRIT_ERR_PROBLEM;
  if (p->layer == MGRIT_LAYER_DENSE) {
    if (p->B < 1 || p->q < 1) return MGRIT_ERR_PROBLEM;
    if (p->q % 8 != 0) return MGRIT_ERR_UNSUPPORTED;       // 16-byte operand pieces
    if ((long long)p->B * p->q > 0x7fffffffLL) return MGRIT_ERR_UNSUPPORTED;   // 32-bit offsets inside a state
    pl->M = p->B; pl->Nf = p->q; pl->K = p->q; pl->TH = 0;
  } else {
    if (p->B < 1 || p->C < 1 || p->Himg < 1 || p->Wimg < 1) return MGRIT_ERR_PROBLEM;
    if (p->C % 8 != 0 || p->C > 64 || p->Wimg > 256) return MGRIT_ERR_UNSUPPORTED;
    if ((long long)p->B * p->Himg * p->Wimg * p->C > 0x7fffffffLL) return MGRIT_ERR_UNSUPPORTED;
    pl->M = p->B * p->Himg * p->Wimg; pl->Nf = p->C; pl->K = 9 * p->C;
    pl->TH = conv_tile_rows(p->Himg, p->Wimg, p->C, p->dtype);
    if (pl->TH < 1) return MGRIT_ERR_UNSUPPORTED;
  }
  pl->E = (long long)pl->M * pl->Nf;
  pl->wsize = (long long)pl->Nf * pl->K;
  pl->esize = p->dtype == MGRIT_FP32 ? 4 : 2;
  pl->B = p->B;
  if (fcP) {
    pl->fcP = fcP;
    pl->nfc = (p->N + fcP - 1) / fcP;
    pl->dfc = (long long)p->Himg * p->Wimg * p->C;
    if (pl->dfc * pl->dfc > 0x7fffffffLL) return MGRIT_ERR_UNSUPPORTED;      // 32-bit offsets inside a weight matrix
    pl->wsize_fc = pl->dfc * pl->dfc;
  }
  long long mp = 1;
  for (int l = 0; l < pl->L; ++l) {
    pl->mpow[l] = mp;
    pl->hl[l] = p->h * (float)mp;
    mp *= p->m;
  }
  // workspace: coarse-level states and right-hand sides, C-point residuals, norm partials,
  // residual history; for the adjoint also the transposed weights and the act' cache
  size_t off = 0;
  for (int l = 1; l < pl->L; ++l) {
    pl->off_X[l] = off; off = align_up(off + (size_t)(pl->Nl[l] + 1) * pl->E * 4);
    pl->off_g[l] = off; off = align_up(off + (size_t)(pl->Nl[l] + 1) * pl->E * 4);
  }
  for (int l = 0; l + 1 < pl->L; ++l) {
    pl->off_R[l] = off; off = align_up(off + (size_t)(pl->Nl[l + 1] + 1) * pl->E * 4);
  }
  StepArgs a;
  memset(&a, 0, sizeof(a));
  a.M = pl->M; a.Nf = pl->Nf; a.K = pl->K; a.Himg = p->Himg; a.Wimg = p->Wimg; a.TH = pl->TH;
  size_t np = (size_t)step_grid_blocks(a, p->layer, p->dtype, p->N) * p->N + diff_sq_blocks(pl->E);
  if (np > 0x7fffffffu) return MGRIT_ERR_UNSUPPORTED;       // the largest launch (all N layers) must fit a 1-D grid
  if (pl->L > 1) {
    size_t np1 = (size_t)step_grid_blocks(a, p->layer, p->dtype, pl->Nl[1]) * pl->Nl[1];
    if (np1 > np) np = np1;
  }
  if (fcP)     // the dense launch of the fully connected groups adds its workgroups (at most 32x32 tiles of each)
    np += (size_t)((p->B + 31) / 32) * (size_t)((pl->dfc + 31) / 32) * (size_t)pl->nfc;
  if (np > 0x7fffffffu) return MGRIT_ERR_UNSUPPORTED;
  pl->n_partial = np;
  pl->off_partial = off; off = align_up(off + np * 4);
  pl->off_hist = off; off = align_up(off + (size_t)(p->max_iter + 1) * 8);
  pl->bytes_fwd = off;
  // transposed weights of the adjoint: convolution layers always; dense layers only on request (their kernels
  // read the caller's array k-major)
  const bool wcopy = p->layer != MGRIT_LAYER_DENSE || adjoint_transposed_copy();
  pl->off_Wt = off;
  if (wcopy) off = align_up(off + (size_t)p->N * pl->wsize * pl->esize);
  pl->off_D = off; off = align_up(off + (size_t)p->N * pl->E * pl->esize);   // act' cache, in the weights' type
  pl->off_gpart = off;                 // partial sums of the conv parameter gradient when layers are split
  if (p->layer == MGRIT_LAYER_CONV3X3)
    off = align_up(off + conv_grad_partial_bytes(p->B, p->Himg, p->Wimg, p->C, p->dtype, p->N));
  pl->off_Wfct = off;
  if (fcP && adjoint_transposed_copy()) off = align_up(off + (size_t)pl->nfc * pl->wsize_fc * pl->esize);
  pl->bytes_adj = off;
  return MGRIT_OK;
}

// The cycle is written once, in "sweep order": sweep point 0 carries the known value and the
// sweep advances to sweep point N_l.  The forward solve sweeps up the layer axis; the adjoint
// solve sweeps down it, so sweep point js of its level l is natural fine point N - js m^l (its
// hierarchy counts from layer N, whatever N mod m is).  Only the caller's fine-level array is
// stored in natural order; all workspace arrays are in sweep order.
struct Solver {
  const mgrit_problem_t* p;
  Plan pl;
  hipStream_t s;
  bool adjoint;
  float* X[MGRIT_MAX_LEVELS];
  float* g[MGRIT_MAX_LEVELS];
  float* R[MGRIT_MAX_LEVELS];
  bool plain_rhs = false;              // nested start: every level carries the right-hand side (first, 0, .., 0)
  const void* W;
  int wn = 0, wn_fc = 0;               // adjoint on the caller's dense / fully connected weights as stored: W[k][n]
  const float* bias;
  const float* Dm;
  const void* Wfc = nullptr;           // fully connected layers of a mixed stack (their transposes in the adjoint)
  const float* bfc = nullptr;
  int act;
  float* partial;
  double* hist_dev;
  hipError_t err = hipSuccess;

  void chk(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
  // map of a sweep-order index range of level l's state array to its storage order
  PtMap pm(int l, long long base, long long stride) const {
    if (l == 0 && adjoint) return PtMap{pl.Nl[0] - base, -stride};
    return PtMap{base, stride};
  }
  // layer index used by the sweep step that lands on sweep point js of level l
  PtMap layer_map(int l, long long js0, long long jstride) const {
    if (adjoint) return PtMap{p->N - js0 * pl.mpow[l], -jstride * pl.mpow[l]};
    return PtMap{(js0 - 1) * pl.mpow[l], jstride * pl.mpow[l]};
  }
  StepArgs base_args(int l, long long js0, long long jstride) const {
    StepArgs a;
    memset(&a, 0, sizeof(a));
    a.W = W; a.wn = wn; a.bias = bias; a.wm = layer_map(l, js0, jstride);
    a.Dm = Dm; a.dm = a.wm;
    a.sp = 1.0f; a.hs = pl.hl[l]; a.mode = MODE_PHI; a.act = act;
    a.M = pl.M; a.Nf = pl.Nf; a.K = pl.K; a.Himg = p->Himg; a.Wimg = p->Wimg; a.TH = pl.TH;
    a.E = pl.E; a.wsize = pl.wsize;
    a.dbf16 = p->dtype == MGRIT_BF16 ? 1 : 0;
    // weights that a level touches: above 128 MB they are streamed past the caches, else later sweeps of the
    // same cycle find them in the last-level cache (a coarse level re-reads its few layers several times per cycle)
    a.wstream = (double)pl.Nl[l] * (double)pl.wsize * (double)pl.esize > 128.0 * 1024.0 * 1024.0 ? 1 : 0;
    return a;
  }
  // Groups of a launch whose layer a.wm(gi) is fully connected: gi = g0 + per * j, j < cnt.  The layer index is
  // affine in gi, so the solutions of  layer = 0 (mod fcP)  form an arithmetic progression.
  void fc_subset(const PtMap& wm, int groups, long long* g0, long long* per, int* cnt) const {
    *g0 = 0; *per = 1; *cnt = 0;
    const long long P = pl.fcP;
    if (!P) return;
    const long long st = ((wm.stride % P) + P) % P;
    long long a = st, b = P;                                // gcd(stride mod P, P); gcd(0, P) = P
    while (a) { const long long t = b % a; b = a; a = t; }
    *per = P / b;
    const long long lim = groups < *per ? groups : *per;
    for (long long gi = 0; gi < lim; ++gi)
      if ((((wm.base + gi * wm.stride) % P) + P) % P == 0) {
        *g0 = gi;
        *cnt = (int)((groups - 1 - gi) / *per + 1);
        return;
      }
  }
  StepArgs fc_args(const StepArgs& a, long long g0, long long per) const {
    auto sub = [&](const PtMap& mp) { return PtMap{mp.base + g0 * mp.stride, mp.stride * per}; };
    StepArgs d = a;
    d.xm = sub(a.xm); d.dm = sub(a.dm); d.om = sub(a.om); d.e1m = sub(a.e1m); d.e2m = sub(a.e2m);
    d.wm = PtMap{(a.wm.base + g0 * a.wm.stride) / pl.fcP, a.wm.stride * per / pl.fcP};
    d.W = Wfc; d.wn = wn_fc; d.bias = a.bias ? bfc : nullptr;
    d.M = pl.B; d.Nf = (int)pl.dfc; d.K = (int)pl.dfc; d.Himg = 0; d.Wimg = 0; d.TH = 0;
    d.wsize = pl.wsize_fc;
    d.wstream = (double)pl.nfc * (double)pl.wsize_fc * (double)pl.esize > 128.0 * 1024.0 * 1024.0 ? 1 : 0;
    d.skip0 = 0; d.skipper = 0;
    return d;
  }
  // workgroups (= norm partials) of a step launch over `groups` groups
  int launch_blocks(const StepArgs& a, int groups) const {
    int nb = step_grid_blocks(a, p->layer, p->dtype, groups) * groups;
    if (pl.fcP) {
      long long g0, per; int cnt;
      fc_subset(a.wm, groups, &g0, &per, &cnt);
      if (cnt) nb += step_grid_blocks(fc_args(a, g0, per), MGRIT_LAYER_DENSE, p->dtype, cnt) * cnt;
    }
    return nb;
  }
  void launch(const StepArgs& a, int groups) {
    if (err != hipSuccess) return;
    if (!pl.fcP) { chk(launch_step(a, p->layer, p->dtype, groups, s)); return; }
    // mixed stack: the convolution kernel passes over the fully connected groups, a dense launch serves them
    long long g0, per; int cnt;
    fc_subset(a.wm, groups, &g0, &per, &cnt);
    StepArgs c = a;
    if (cnt) { c.skip0 = (int)g0; c.skipper = (int)per; }
    if (cnt < groups || a.norm_partial) chk(launch_step(c, p->layer, p->dtype, groups, s));
    if (cnt && err == hipSuccess) {
      StepArgs d = fc_args(a, g0, per);
      if (a.norm_partial) d.norm_partial = a.norm_partial + (size_t)step_grid_blocks(a, p->layer, p->dtype, groups) * groups;
      chk(launch_step(d, MGRIT_LAYER_DENSE, p->dtype, cnt, s));
    }
  }
  // X[js] = Phi(X[js-1]) + g[js] for js = js0 + gi*jstride        (relaxation, coarsest solve)
  void propagate(int l, long long js0, long long jstride, int groups) {
    StepArgs a = base_args(l, js0, jstride);
    a.X = X[l]; a.xm = pm(l, js0 - 1, jstride);
    a.Out = X[l]; a.om = pm(l, js0, jstride);
    if (g[l] && !plain_rhs) { a.E1 = g[l]; a.e1m = PtMap{js0, jstride}; a.c1 = 1.0f; }
    launch(a, groups);
  }
  // One fused launch per F-relaxation sweep where it pays: dense layers of a supported width or convolution
  // layers of at most 16 float channels on images that fit one workgroup, at least two steps per interval, and
  // enough workgroups -- (interval, 32-row slice) or (interval, image) -- to occupy the chip; with fewer, the
  // lockstep launches (which spread one step over many workgroups) are as fast.
  bool use_sweep(int l) const {
    if (pl.fcP || p->m < 3 || !sweep_enabled()) return false;
    if (p->layer == MGRIT_LAYER_CONV3X3)         // workgroup = (interval, image)
      return conv_sweep_supported(p->Himg, p->Wimg, p->C, p->dtype) && (long long)pl.B * pl.Nl[l + 1] >= 128;
    if (!sweep_supported(p->q, p->dtype)) return false;
    return sweep_blocks(pl.M, pl.Nl[l + 1]) >= 128;
  }
  void f_relax(int l) {                                        // Sec. III-C, Fig. 3
    const int Nc = pl.Nl[l + 1];
    const int tail = pl.Nl[l] - Nc * p->m;                     // F-points behind the last C-point (< m)
    if (use_sweep(l)) {
      SweepArgs a;
      memset(&a, 0, sizeof(a));
      const long long mp = pl.mpow[l];
      const PtMap unit = pm(l, 0, 1);                          // storage index of sweep point js = base + js * stride
      a.S = X[l]; a.sm = pm(l, 0, p->m);
      a.X = X[l]; a.xb = unit.base; a.xs = unit.stride * p->m; a.xk = unit.stride;
      if (g[l] && !plain_rhs) { a.G = g[l]; a.gb = 0; a.gs = p->m; }
      a.W = W; a.wn = wn; a.bias = bias; a.Dm = Dm;
      if (adjoint) { a.lb = p->N - mp;           a.ls = -(long long)p->m * mp; a.lk = -mp; }
      else         { a.lb = 0;                   a.ls = (long long)p->m * mp;  a.lk = mp; }
      a.hs = pl.hl[l]; a.act = act; a.nsteps = p->m - 1; a.nchains = Nc;
      a.M = pl.M; a.q = pl.Nf; a.E = pl.E; a.wsize = pl.wsize;
      if (p->layer == MGRIT_LAYER_CONV3X3) {
        a.M = pl.B; a.Himg = p->Himg; a.Wimg = p->Wimg; a.C = p->C;
        if (err == hipSuccess) chk(launch_conv_sweep(a, s));
      } else if (err == hipSuccess) {
        chk(launch_sweep(a, p->dtype, s));
      }
      for (int k = 1; k <= tail; ++k) propagate(l, (long long)Nc * p->m + k, p->m, 1);
      return;
    }
    for (int k = 1; k < p->m; ++k) propagate(l, k, p->m, Nc + (k <= tail ? 1 : 0));
  }
  void c_relax(int l) { propagate(l, p->m, p->m, pl.Nl[l + 1]); }

  // Nested-iteration start: the coarsest level's own equation is solved in sequence from the known
  // value; going up, the C-points of a level take the coarser level's values and (on the middle
  // levels) the F-points follow by F-relaxation.  The fine level's F-points are left to the opening
  // relaxation of the first cycle.
  void nested_start(const float* first) {
    const int m = p->m;
    plain_rhs = true;
    const int lc = pl.L - 1;
    chk(launch_copy_points(X[lc], pm(lc, 0, 0), first, PtMap{0, 0}, pl.E, 1, s));
    for (int j = 1; j <= pl.Nl[lc]; ++j) propagate(lc, j, 1, 1);
    for (int l = lc - 1; l >= 0; --l) {
      chk(launch_copy_points(X[l], pm(l, 0, m), X[l + 1], PtMap{0, 1}, pl.E, pl.Nl[l + 1] + 1, s));
      if (l > 0) f_relax(l);
    }
    plain_rhs = false;
  }

  void cycle(int l, int iter, bool skip_opening_relax) {
    const int m = p->m;
    if (l == pl.L - 1) {                                        // coarsest level: serial solve
      // X[l][0] already holds the known value: the injection copied it together with the other points
      for (int j = 1; j <= pl.Nl[l]; ++j) propagate(l, j, 1, 1);
      return;
    }
    const int Nc = pl.Nl[l + 1];
    if (!skip_opening_relax) f_relax(l);                        // Alg. 1 step 1
    if (p->relax == MGRIT_RELAX_FCF) { c_relax(l); f_relax(l); }
    {                                                           // residual at the C-points, Eq. (19)
      StepArgs a = base_args(l, m, m);
      a.X = X[l]; a.xm = pm(l, m - 1, m);
      a.Out = R[l]; a.om = PtMap{1, 1};
      a.E1 = X[l]; a.e1m = pm(l, m, m); a.c1 = -1.0f;
      if (g[l]) { a.E2 = g[l]; a.e2m = PtMap{m, m}; a.c2 = 1.0f; }
      if (l == 0) a.norm_partial = partial;
      launch(a, Nc);
      // Alg. 1 step 2: injection of the C-points (the residual of point 0 is identically zero); on the fine
      // level the same launch also sums the norm partials of the residual launch (Alg. 1 step 6)
      if (l == 0) {
        const int nb = launch_blocks(a, Nc);
        const double scale = p->norm_kind == MGRIT_NORM_RMS ? 1.0 / sqrt((double)(Nc + 1) * (double)pl.E) : 1.0;
        chk(launch_copy_points_norm(X[l + 1], PtMap{0, 1}, X[l], pm(l, 0, m), pl.E, Nc + 1, partial, nb, scale,
                                    hist_dev + iter, s));
      } else {
        chk(launch_copy_points(X[l + 1], PtMap{0, 1}, X[l], pm(l, 0, m), pl.E, Nc + 1, s));
      }
    }
    // g[l+1][0] = U[0] + R[0] is the known value at point 0 in every cycle (R[0] = 0): set once per solve
    {                                                           // Alg. 1 step 3: S_H = L_H(U_H) + R_H
      StepArgs a = base_args(l + 1, 1, 1);
      a.X = X[l + 1]; a.xm = PtMap{0, 1};
      a.Out = g[l + 1]; a.om = PtMap{1, 1};
      a.sp = -1.0f;
      a.E1 = X[l + 1]; a.e1m = PtMap{1, 1}; a.c1 = 1.0f;
      a.E2 = R[l]; a.e2m = PtMap{1, 1}; a.c2 = 1.0f;
      launch(a, Nc);
    }
    cycle(l + 1, iter, false);                                  // solve for V_H (in place of U_H)
    // Alg. 1 steps 4, 5: C-points += V_H - U_H, where U_H is still held by the C-points themselves
    chk(launch_correct(X[l], pm(l, m, m), X[l + 1], PtMap{1, 1}, pl.E, Nc, s));
    f_relax(l);
  }
};

int check_finite(const double* h, int n) {
  for (int i = 0; i < n; ++i)
    if (!isfinite(h[i])) return MGRIT_ERR_NONFINITE;
  return MGRIT_OK;
}

// Runs the solve loop shared by the forward and the adjoint entry point.
int run_solver(Solver& sv, const float* first, double* resnorm_hist, int32_t* iters_done) {
  const mgrit_problem_t* p = sv.p;
  const Plan& pl = sv.pl;
  const int m = p->m;
  // known value at sweep point 0 and initial guess of the C-points
  if (pl.L > 1 && p->init == MGRIT_INIT_ZERO)
    sv.chk(launch_zero_points(sv.X[0], sv.pm(0, m, m), pl.E, pl.Nl[1], sv.s));
  if (pl.L > 1 && p->init == MGRIT_INIT_COPY)
    sv.chk(launch_copy_points(sv.X[0], sv.pm(0, m, m), first, PtMap{0, 0}, pl.E, pl.Nl[1], sv.s));
  sv.chk(launch_copy_points(sv.X[0], sv.pm(0, 0, 0), first, PtMap{0, 0}, pl.E, 1, sv.s));
  for (int l = 1; l < pl.L; ++l)       // right-hand side of point 0 on the coarse levels: the known value
    sv.chk(launch_copy_points(sv.g[l], PtMap{0, 0}, first, PtMap{0, 0}, pl.E, 1, sv.s));
  if (pl.L > 1 && p->init == MGRIT_INIT_NESTED) sv.nested_start(first);

  int iters = 0;
  int rc = MGRIT_OK;
  if (pl.L == 1) {
    sv.cycle(0, 0, false);
    iters = 1;
    if (resnorm_hist) resnorm_hist[0] = 0.0;
    if (sv.err == hipSuccess && (resnorm_hist || iters_done)) sv.chk(hipStreamSynchronize(sv.s));
  } else {
    for (int k = 0; k < p->max_iter && sv.err == hipSuccess; ++k) {
      sv.cycle(0, k, k > 0);
      ++iters;
      if (p->tol > 0.0f) {
        double v = 0.0;
        sv.chk(hipMemcpyAsync(&v, sv.hist_dev + k, sizeof(double), hipMemcpyDeviceToHost, sv.s));
        sv.chk(hipStreamSynchronize(sv.s));
        if (sv.err != hipSuccess) break;
        if (resnorm_hist) resnorm_hist[k] = v;
        if (!isfinite(v)) { rc = MGRIT_ERR_NONFINITE; break; }
        if (v <= (double)p->tol) break;
      }
    }
    if (!(p->tol > 0.0f) && resnorm_hist && sv.err == hipSuccess) {
      sv.chk(hipMemcpyAsync(resnorm_hist, sv.hist_dev, sizeof(double) * iters, hipMemcpyDeviceToHost, sv.s));
      sv.chk(hipStreamSynchronize(sv.s));
      if (sv.err == hipSuccess) rc = check_finite(resnorm_hist, iters);
    } else if (iters_done && sv.err == hipSuccess) {
      sv.chk(hipStreamSynchronize(sv.s));
    }
  }
  if (iters_done) *iters_done = iters;
  if (sv.err != hipSuccess) return MGRIT_ERR_HIP;
  return rc;
}

void bind_workspace(Solver& sv, void* workspace) {
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const Plan& pl = sv.pl;
  for (int l = 1; l < pl.L; ++l) {
    sv.X[l] = reinterpret_cast<float*>(ws + pl.off_X[l]);
    sv.g[l] = reinterpret_cast<float*>(ws + pl.off_g[l]);
  }
  for (int l = 0; l + 1 < pl.L; ++l) {
    sv.R[l] = reinterpret_cast<float*>(ws + pl.off_R[l]);
  }
  sv.partial = reinterpret_cast<float*>(ws + pl.off_partial);
  sv.hist_dev = reinterpret_cast<double*>(ws + pl.off_hist);
}

// checks of the fully connected part of a mixed stack (fc == nullptr: plain stack)
int check_fc(const mgrit_fc_layers_t* fc, bool adjoint, const float* dW, const float* db) {
  if (!fc) return MGRIT_OK;
  if (!fc->Wfc || !fc->bfc || !aligned(fc->Wfc) || !aligned(fc->bfc)) return MGRIT_ERR_POINTER;
  if (adjoint) {
    if ((dW && !fc->dWfc) || (db && !fc->dbfc)) return MGRIT_ERR_POINTER;
    if (!aligned(fc->dWfc) || !aligned(fc->dbfc)) return MGRIT_ERR_POINTER;
  }
  return MGRIT_OK;
}

int forward_impl(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                 const float* u0, float* U, double* resnorm_hist, int32_t* iters_done, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  if (!p || !W || !b || !u0 || !U || !workspace) return MGRIT_ERR_POINTER;
  if (!aligned(W) || !aligned(b) || !aligned(u0) || !aligned(U) || !aligned(workspace)) return MGRIT_ERR_POINTER;
  int rc = check_fc(fc, false, nullptr, nullptr);
  if (rc != MGRIT_OK) return rc;
  Solver sv;
  rc = make_plan(p, &sv.pl, fc ? fc->fc_period : 0);
  if (rc != MGRIT_OK) return rc;
  if (fc && !sv.pl.fcP) return MGRIT_ERR_PROBLEM;
  if (workspace_bytes < sv.pl.bytes_fwd) return MGRIT_ERR_WORKSPACE;
  sv.p = p; sv.s = static_cast<hipStream_t>(hip_stream); sv.adjoint = false;
  memset(sv.X, 0, sizeof(sv.X)); memset(sv.g, 0, sizeof(sv.g)); memset(sv.R, 0, sizeof(sv.R));
  sv.X[0] = U;
  sv.W = W; sv.bias = b; sv.Dm = nullptr; sv.act = p->act;
  if (fc) { sv.Wfc = fc->Wfc; sv.bfc = fc->bfc; }
  bind_workspace(sv, workspace);
  return run_solver(sv, u0, resnorm_hist, iters_done);
}

int adjoint_impl(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                 const float* U, const float* lamN, float* Lam, float* dW, float* db, double* resnorm_hist,
                 int32_t* iters_done, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p || !W || !b || !U || !lamN || !Lam || !workspace) return MGRIT_ERR_POINTER;
  if (!aligned(W) || !aligned(b) || !aligned(U) || !aligned(lamN) || !aligned(Lam) || !aligned(workspace) ||
      !aligned(dW) || !aligned(db))
    return MGRIT_ERR_POINTER;
  int rc = check_fc(fc, true, dW, db);
  if (rc != MGRIT_OK) return rc;
  Solver sv;
  rc = make_plan(p, &sv.pl, fc ? fc->fc_period : 0);
  if (rc != MGRIT_OK) return rc;
  if (fc && !sv.pl.fcP) return MGRIT_ERR_PROBLEM;
  if (workspace_bytes < sv.pl.bytes_adj) return MGRIT_ERR_WORKSPACE;
  const Plan& pl = sv.pl;
  sv.p = p; sv.s = static_cast<hipStream_t>(hip_stream); sv.adjoint = true;
  memset(sv.X, 0, sizeof(sv.X)); memset(sv.g, 0, sizeof(sv.g)); memset(sv.R, 0, sizeof(sv.R));
  sv.X[0] = Lam;
  bind_workspace(sv, workspace);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  void* Wt = ws + pl.off_Wt;
  void* Wfct = ws + pl.off_Wfct;
  float* D = reinterpret_cast<float*>(ws + pl.off_D);
  // transposed parameters (convolution layers, whose taps are mirrored as well; dense and fully connected
  // matrices only on request), and act'(A_n U^n + b_n) for every layer in one grouped launch
  const bool copy_dense = adjoint_transposed_copy();
  const bool copy_main = p->layer != MGRIT_LAYER_DENSE || copy_dense;
  if (copy_main) sv.chk(launch_transpose_weights(W, Wt, p->layer, p->dtype, p->N, pl.Nf, sv.s));
  if (fc && copy_dense) sv.chk(launch_transpose_weights(fc->Wfc, Wfct, MGRIT_LAYER_DENSE, p->dtype, pl.nfc, (int)pl.dfc, sv.s));
  {
    sv.W = W; sv.bias = b; sv.Dm = nullptr; sv.act = p->act;
    if (fc) { sv.Wfc = fc->Wfc; sv.bfc = fc->bfc; }
    StepArgs a = sv.base_args(0, 1, 1);
    a.wm = PtMap{0, 1};
    a.mode = MODE_DACT;
    a.X = U; a.xm = PtMap{0, 1};
    a.Out = D; a.om = PtMap{0, 1};
    sv.launch(a, p->N);
  }
  sv.bias = nullptr; sv.Dm = D; sv.act = ACT_IDENT;
  if (copy_main) sv.W = Wt; else { sv.W = W; sv.wn = 1; }
  if (fc) {
    sv.bfc = nullptr;
    if (copy_dense) sv.Wfc = Wfct; else { sv.Wfc = fc->Wfc; sv.wn_fc = 1; }
  }
  rc = run_solver(sv, lamN, resnorm_hist, iters_done);
  if (rc != MGRIT_OK && rc != MGRIT_ERR_NONFINITE) return rc;
  if (dW || db) {
    GradArgs ga;
    memset(&ga, 0, sizeof(ga));
    ga.U = U; ga.um = PtMap{0, 1};
    ga.Lam = Lam; ga.lm = PtMap{1, 1};
    ga.Dm = D; ga.dm = PtMap{0, 1};
    ga.dW = dW; ga.db = db; ga.hs = p->h;
    ga.M = pl.M; ga.Nf = pl.Nf; ga.K = pl.K; ga.Himg = p->Himg; ga.Wimg = p->Wimg; ga.B = p->B;
    ga.E = pl.E; ga.wsize = pl.wsize;
    ga.partial = reinterpret_cast<float*>(ws + pl.off_gpart);
    if (launch_grad(ga, p->layer, p->dtype, p->N, sv.s) != hipSuccess) return MGRIT_ERR_HIP;
    if (fc) {
      // the convolution gradient ran over every layer: its slots at the fully connected layers are defined as
      // zero; their own gradient is the dense contraction over the batch
      const long long P = pl.fcP;
      if (dW) sv.chk(launch_zero_points(dW, PtMap{0, P}, pl.wsize, pl.nfc, sv.s));
      if (db) sv.chk(launch_zero_points(db, PtMap{0, P}, pl.Nf, pl.nfc, sv.s));
      GradArgs gd;
      memset(&gd, 0, sizeof(gd));
      gd.U = U; gd.um = PtMap{0, P};
      gd.Lam = Lam; gd.lm = PtMap{1, P};
      gd.Dm = D; gd.dm = PtMap{0, P};
      gd.dW = dW ? fc->dWfc : nullptr; gd.db = db ? fc->dbfc : nullptr; gd.hs = p->h;
      gd.M = p->B; gd.Nf = (int)pl.dfc; gd.K = (int)pl.dfc; gd.B = p->B;
      gd.E = pl.E; gd.wsize = pl.wsize_fc;
      if (sv.err != hipSuccess || launch_grad(gd, MGRIT_LAYER_DENSE, p->dtype, pl.nfc, sv.s) != hipSuccess)
        return MGRIT_ERR_HIP;
    }
    if (resnorm_hist || iters_done)
      if (hipStreamSynchronize(sv.s) != hipSuccess) return MGRIT_ERR_HIP;
  }
  return rc;
}

int residual_norm_impl(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                       const float* u0, const float* U, double* norm_out, void* workspace, size_t workspace_bytes,
                       void* hip_stream) {
  if (!p || !W || !b || !u0 || !U || !norm_out || !workspace) return MGRIT_ERR_POINTER;
  if (!aligned(W) || !aligned(b) || !aligned(u0) || !aligned(U) || !aligned(workspace)) return MGRIT_ERR_POINTER;
  int rc = check_fc(fc, false, nullptr, nullptr);
  if (rc != MGRIT_OK) return rc;
  Solver sv;
  rc = make_plan(p, &sv.pl, fc ? fc->fc_period : 0);
  if (rc != MGRIT_OK) return rc;
  if (fc && !sv.pl.fcP) return MGRIT_ERR_PROBLEM;
  if (workspace_bytes < sv.pl.bytes_fwd) return MGRIT_ERR_WORKSPACE;
  const Plan& pl = sv.pl;
  sv.p = p; sv.s = static_cast<hipStream_t>(hip_stream); sv.adjoint = false;
  memset(sv.X, 0, sizeof(sv.X)); memset(sv.g, 0, sizeof(sv.g)); memset(sv.R, 0, sizeof(sv.R));
  sv.W = W; sv.bias = b; sv.Dm = nullptr; sv.act = p->act;
  if (fc) { sv.Wfc = fc->Wfc; sv.bfc = fc->bfc; }
  bind_workspace(sv, workspace);
  // rows n = 1..N of f_h - L_h(U): Phi(U[n-1]) - U[n]; row 0: u0 - U[0]
  StepArgs a = sv.base_args(0, 1, 1);
  a.X = U; a.xm = PtMap{0, 1};
  a.E1 = U; a.e1m = PtMap{1, 1}; a.c1 = -1.0f;
  a.norm_partial = sv.partial;
  sv.launch(a, p->N);
  const int nb = sv.launch_blocks(a, p->N);
  int nb0 = 0;
  sv.chk(launch_diff_sq(u0, U, pl.E, sv.partial + nb, &nb0, sv.s));
  const double scale = p->norm_kind == MGRIT_NORM_RMS ? 1.0 / sqrt((double)(p->N + 1) * (double)pl.E) : 1.0;
  sv.chk(launch_norm_final(sv.partial, nb + nb0, scale, sv.hist_dev, sv.s));
  double v = 0.0;
  sv.chk(hipMemcpyAsync(&v, sv.hist_dev, sizeof(double), hipMemcpyDeviceToHost, sv.s));
  sv.chk(hipStreamSynchronize(sv.s));
  if (sv.err != hipSuccess) return MGRIT_ERR_HIP;
  *norm_out = v;
  return isfinite(v) ? MGRIT_OK : MGRIT_ERR_NONFINITE;
}

// Workspace of the entry point that allocates nothing: a fixed array in device memory that every GPU the
// library runs on holds until the process ends.  In host code its name is only a handle; the address of a
// device's copy comes from hipGetSymbolAddress, once per device, and only that address is handed to kernels.
__device__ __align__(256) unsigned char scratch[MGRIT_STATIC_SCRATCH_BYTES];
void* g_scratch_ptr[64] = {};

}  // namespace

extern "C" {

int32_t mgrit_level_map(const mgrit_problem_t* p, int32_t* n_levels, int32_t* N_l, int32_t* fine_index) {
  if (!p || !n_levels) return MGRIT_ERR_POINTER;
  int L, Nl[MGRIT_MAX_LEVELS];
  const int rc = build_levels(p, &L, Nl);
  if (rc != MGRIT_OK) return rc;
  *n_levels = L;
  long long mp = 1;
  size_t pos = 0;
  for (int l = 0; l < L; ++l) {
    if (N_l) N_l[l] = Nl[l];
    if (fine_index)
      for (int j = 0; j <= Nl[l]; ++j) fine_index[pos++] = (int32_t)(j * mp);
    mp *= p->m;
  }
  return MGRIT_OK;
}

size_t mgrit_workspace_bytes(const mgrit_problem_t* p) {
  Plan pl;
  if (!p || make_plan(p, &pl) != MGRIT_OK) return 0;
  return pl.bytes_fwd;
}

size_t mgrit_adjoint_workspace_bytes(const mgrit_problem_t* p) {
  Plan pl;
  if (!p || make_plan(p, &pl) != MGRIT_OK) return 0;
  return pl.bytes_adj;
}

int32_t mgrit_fas_forward(const mgrit_problem_t* p, const void* W, const float* b, const float* u0, float* U,
                          double* resnorm_hist, int32_t* iters_done, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  return forward_impl(p, nullptr, W, b, u0, U, resnorm_hist, iters_done, workspace, workspace_bytes, hip_stream);
}

int32_t mgrit_fas_adjoint(const mgrit_problem_t* p, const void* W, const float* b, const float* U, const float* lamN,
                          float* Lam, float* dW, float* db, double* resnorm_hist, int32_t* iters_done,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  return adjoint_impl(p, nullptr, W, b, U, lamN, Lam, dW, db, resnorm_hist, iters_done, workspace, workspace_bytes,
                      hip_stream);
}

int32_t mgrit_residual_norm(const mgrit_problem_t* p, const void* W, const float* b, const float* u0, const float* U,
                            double* norm_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return residual_norm_impl(p, nullptr, W, b, u0, U, norm_out, workspace, workspace_bytes, hip_stream);
}

int32_t mgrit_fas_forward_static(const mgrit_problem_t* p, const void* W, const float* b, const float* u0, float* U,
                                 double* resnorm_hist, int32_t* iters_done, void* hip_stream) {
  Plan pl;
  if (!p) return MGRIT_ERR_POINTER;
  const int rc = make_plan(p, &pl);
  if (rc != MGRIT_OK) return rc;
  if (pl.bytes_fwd > (size_t)MGRIT_STATIC_SCRATCH_BYTES) return MGRIT_ERR_WORKSPACE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return MGRIT_ERR_HIP;
  if (dev < 0 || dev >= 64) return MGRIT_ERR_UNSUPPORTED;
  if (!g_scratch_ptr[dev]) {                     // first call on this device: look up its copy of the array
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MGRIT_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  // nothing in the workspace has to start at zero: every array in it is written before it is read
  return forward_impl(p, nullptr, W, b, u0, U, resnorm_hist, iters_done, g_scratch_ptr[dev],
                      (size_t)MGRIT_STATIC_SCRATCH_BYTES, hip_stream);
}

size_t mgrit_workspace_bytes_mixed(const mgrit_problem_t* p, int32_t fc_period) {
  Plan pl;
  if (!p || fc_period < 2 || make_plan(p, &pl, fc_period) != MGRIT_OK) return 0;
  return pl.bytes_fwd;
}

size_t mgrit_adjoint_workspace_bytes_mixed(const mgrit_problem_t* p, int32_t fc_period) {
  Plan pl;
  if (!p || fc_period < 2 || make_plan(p, &pl, fc_period) != MGRIT_OK) return 0;
  return pl.bytes_adj;
}

int32_t mgrit_fas_forward_mixed(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                                const float* u0, float* U, double* resnorm_hist, int32_t* iters_done,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!fc) return MGRIT_ERR_POINTER;
  return forward_impl(p, fc, W, b, u0, U, resnorm_hist, iters_done, workspace, workspace_bytes, hip_stream);
}

int32_t mgrit_fas_adjoint_mixed(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W, const float* b,
                                const float* U, const float* lamN, float* Lam, float* dW, float* db,
                                double* resnorm_hist, int32_t* iters_done, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
  if (!fc) return MGRIT_ERR_POINTER;
  return adjoint_impl(p, fc, W, b, U, lamN, Lam, dW, db, resnorm_hist, iters_done, workspace, workspace_bytes,
                      hip_stream);
}

int32_t mgrit_residual_norm_mixed(const mgrit_problem_t* p, const mgrit_fc_layers_t* fc, const void* W,
                                  const float* b, const float* u0, const float* U, double* norm_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!fc) return MGRIT_ERR_POINTER;
  return residual_norm_impl(p, fc, W, b, u0, U, norm_out, workspace, workspace_bytes, hip_stream);
}

void mgrit_trace_begin(void) { trace_begin(); }

int32_t mgrit_trace_end(double* ms, int64_t* launches, int64_t* units, double* bytes, int32_t n_classes) {
  if (!ms || !launches || !units || n_classes < 1) return MGRIT_ERR_POINTER;
  long long l[TRACE_NCLASS], u[TRACE_NCLASS];
  double m[TRACE_NCLASS], b[TRACE_NCLASS];
  if (trace_end(m, l, u, b, TRACE_NCLASS) != 0) return MGRIT_ERR_HIP;
  for (int i = 0; i < n_classes; ++i) {
    ms[i] = i < TRACE_NCLASS ? m[i] : 0.0;
    launches[i] = i < TRACE_NCLASS ? l[i] : 0;
    units[i] = i < TRACE_NCLASS ? u[i] : 0;
    if (bytes) bytes[i] = i < TRACE_NCLASS ? b[i] : 0.0;
  }
  return MGRIT_OK;
}

}  // extern "C"
