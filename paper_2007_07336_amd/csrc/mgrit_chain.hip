// Temporally fused relaxation for dense layers (gfx950 / CDNA4).
//
// A dense residual-block step acts on every batch row independently, so one workgroup can own
// a slice of 32 batch rows of one coarse interval and march through ALL the steps of that
// interval -- F-relaxation, the C-relaxation step, the residual / FAS right-hand side -- with the
// state slice resident in LDS.  One launch then performs a whole relaxation sweep of a level
// (Sec. III-C, Fig. 3; Alg. 1 steps 1-3) instead of one launch per layer step, and the serial
// solve of the coarsest level is a single launch.  The weights of each layer are streamed from
// L2/HBM straight into the B-operand registers of the MFMA through a 4-deep register ring (no
// LDS staging: a weight element is used by exactly one wavefront of the workgroup).
#include "mgrit_internal.h"

namespace mgrit {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int NT = 256;
constexpr int R = 32;        // batch rows per workgroup
constexpr int NST = 4;       // weight ring stages; a stage is 8 x 16 bytes per lane

template <typename T> struct COp;
template <> struct COp<float>  { static constexpr int KU = 64;  static constexpr int PAD = 4; };
template <> struct COp<__bf16> { static constexpr int KU = 128; static constexpr int PAD = 8; };

__device__ __forceinline__ void st_op4(float* d, float4 v) { *reinterpret_cast<float4*>(d) = v; }
__device__ __forceinline__ void st_op4(__bf16* d, float4 v) {
  bf16x4 o;
  o[0] = static_cast<__bf16>(v.x); o[1] = static_cast<__bf16>(v.y);
  o[2] = static_cast<__bf16>(v.z); o[3] = static_cast<__bf16>(v.w);
  *reinterpret_cast<bf16x4*>(d) = o;
}

// one ring stage of weights against the operand tile(s): KU values of k
__device__ __forceinline__ void mma_unit(const float* arow, const uint4 (&w)[8], floatx16& acc) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float4 a = *reinterpret_cast<const float4*>(arow + 16 * (j >> 1) + 4 * (j & 1));
    const float4 b = *reinterpret_cast<const float4*>(&w[j]);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
  }
}
__device__ __forceinline__ void mma_unit(const __bf16* arow, const uint4 (&w)[8], floatx16& acc) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + 16 * j);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(&w[j]);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
  }
}
// element offset (in k) of piece j of a stage for lane group g -- must match mma_unit
__device__ __forceinline__ int piece_k(float, int j, int g) { return 16 * (j >> 1) + 8 * g + 4 * (j & 1); }
__device__ __forceinline__ int piece_k(__bf16, int j, int g) { return 16 * j + 8 * g; }
// offset of the lane's operand row start for group g (the A side of the same mapping)
__device__ __forceinline__ int arow_k(float, int g) { return 8 * g; }
__device__ __forceinline__ int arow_k(__bf16, int g) { return 8 * g; }

__device__ __forceinline__ float c_act(float z, int act) {
  if (act == ACT_TANH) return tanhf(z);
  if (act == ACT_RELU) return fmaxf(z, 0.0f);
  return z;
}

template <typename WT>
__global__ __launch_bounds__(NT) void dense_chain_kernel(ChainArgs a) {
  constexpr int KU = COp<WT>::KU, PAD = COp<WT>::PAD;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float red[4];
  const int q = a.q;
  const int AST = q + PAD;                               // operand row stride (elements)
  float* S = reinterpret_cast<float*>(smem);             // [R][q] fp32 master state
  WT* A = reinterpret_cast<WT*>(S + R * q);              // [R][AST] operand of the current step
  WT* A0 = A + R * AST;                                  // [R][AST] operand of the coarse step (adjoint only)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, c = lane & 31;
  int L = blockIdx.x;
  {
    const int total = gridDim.x;
    if ((total & 7) == 0) L = (L & 7) * (total >> 3) + (L >> 3);   // slices of a chain share an XCD
  }
  const int nsl = (a.M + R - 1) / R;
  const long long ci = L / nsl;                          // chain (coarse interval)
  const int r0 = (L % nsl) * R;                          // first batch row of the slice
  const int rows = min(R, a.M - r0);
  const int q4 = q >> 2;
  const long long slice_off = (long long)r0 * q;

  // ---- chain start -> S (and to the state array if asked)
  {
    const float* sp = a.S + (a.sm.base + ci * a.sm.stride) * a.E + slice_off;
    float* xs = a.write_start ? a.X + (a.xb + ci * a.xs) * a.E + slice_off : nullptr;
    float* cb0 = (a.last == LAST_CRELAX && ci == 0) ? a.Cb + slice_off : nullptr;
    float* xh0 = (a.last == LAST_RESID && ci == 0) ? a.XH + slice_off : nullptr;
    float* gh0 = (a.last == LAST_RESID && ci == 0) ? a.GH + slice_off : nullptr;
    for (int p = tid; p < R * q4; p += NT) {
      const int row = p / q4, c4 = (p % q4) * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row < rows) {
        v = *reinterpret_cast<const float4*>(sp + (long long)row * q + c4);
        if (xs) *reinterpret_cast<float4*>(xs + (long long)row * q + c4) = v;
        if (cb0) *reinterpret_cast<float4*>(cb0 + (long long)row * q + c4) = v;
        if (xh0) *reinterpret_cast<float4*>(xh0 + (long long)row * q + c4) = v;
        if (gh0) *reinterpret_cast<float4*>(gh0 + (long long)row * q + c4) = v;
      }
      *reinterpret_cast<float4*>(S + row * q + c4) = v;
    }
  }
  __syncthreads();

  // operand of a step: (Dm[layer] .* S) converted to the matrix-core type
  auto build_operand = [&](WT* dst, long long layer) {
    const float* dp = a.Dm ? a.Dm + layer * a.E + slice_off : nullptr;
    for (int p = tid; p < R * q4; p += NT) {
      const int row = p / q4, c4 = (p % q4) * 4;
      float4 v = *reinterpret_cast<const float4*>(S + row * q + c4);
      if (dp && row < rows) {
        const float4 d = *reinterpret_cast<const float4*>(dp + (long long)row * q + c4);
        v.x *= d.x; v.y *= d.y; v.z *= d.z; v.w *= d.w;
      }
      st_op4(dst + row * AST + c4, v);
    }
  };

  const int nsteps = a.nsteps;
  const bool want_tau = (a.last == LAST_RESID);
  const bool tau_last = want_tau && a.tau_on_last_step;   // adjoint: coarse step shares the LAST step's weights
  const long long layer_of_last = a.lb + ci * a.ls + (long long)(nsteps - 1) * a.lk;
  if (tau_last) build_operand(A0, layer_of_last);
  build_operand(A, a.lb + ci * a.ls);
  __syncthreads();

  const int NBW = q >> 7;                                // 32-column blocks per wavefront (q = 128 * NBW)
  const int UPB = q / KU;                                // ring stages per column block
  const long long total = (long long)nsteps * NBW * UPB;
  const WT* Wbase = reinterpret_cast<const WT*>(a.W);

  // ---- weight ring: prefetch stream counters (pk: step 1-based, pt: block, pu: stage in block)
  uint4 wr[NST][8];
  int pk = 1, pt = 0, pu = 0;
  auto issue = [&](uint4 (&dst)[8]) {
    const long long layer = a.lb + ci * a.ls + (long long)(pk - 1) * a.lk;
    const int n = (wave * NBW + pt) * 32 + c;
    const WT* wp = Wbase + layer * a.wsize + (long long)n * q + pu * KU;
#pragma unroll
    for (int j = 0; j < 8; ++j) dst[j] = *reinterpret_cast<const uint4*>(wp + piece_k(WT(), j, g));
    if (++pu == UPB) { pu = 0; if (++pt == NBW) { pt = 0; ++pk; } }
  };
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < total) issue(wr[s]);

  // ---- consume stream counters
  int k = 1, t = 0, u = 0;
  floatx16 acc, accH;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[r] = 0.0f; accH[r] = 0.0f; }
  float sq = 0.0f;

  auto block_epilogue = [&]() {
    // finished column block t of step k: rows 8*(r/4)+4*g+r%4, column n
    const bool is_last = (k == nsteps);
    const long long layer = a.lb + ci * a.ls + (long long)(k - 1) * a.lk;
    const int n = (wave * NBW + t) * 32 + c;
    const float bv = a.bias ? a.bias[layer * q + n] : 0.0f;
    const float* gp = a.G ? a.G + (a.gb + ci * a.gs + k) * a.E + slice_off : nullptr;
    float* xo = nullptr;
    if (!is_last || a.last == LAST_F) xo = a.X + (a.xb + ci * a.xs + (long long)k * a.xk) * a.E + slice_off;
    else if (a.last == LAST_CRELAX) xo = a.Cb + (a.cbb + ci * a.cbs) * a.E + slice_off;
    float* ghp = want_tau ? a.GH + (ci + 1) * a.E + slice_off : nullptr;
    const float* uep = (is_last && want_tau) ? a.Ue + (a.uem.base + ci * a.uem.stride) * a.E + slice_off : nullptr;
    float* xhp = (is_last && want_tau) ? a.XH + (ci + 1) * a.E + slice_off : nullptr;
    float* xlp = (is_last && want_tau && a.Xlast && ci == a.nchains - 1) ? a.Xlast + a.xlast_pt * a.E + slice_off : nullptr;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + 4 * g + (r & 3);
      if (row >= rows) continue;
      const long long off = (long long)row * q + n;
      const float sold = S[row * q + n];
      const float f = c_act(acc[r] + bv, a.act);
      float unew = sold + a.hs * f;
      if (gp) unew += gp[off];
      if (want_tau && !tau_last && k == 1) ghp[off] = -(sold + a.hsH * f);   // -Phi_H(start), finished below
      if (xo) xo[off] = unew;
      if (is_last && want_tau) {
        const float ue = uep[off];
        const float res = unew - ue;                     // g - U + Phi(U_prev)          Eq. (19)
        sq += res * res;
        float phiH_neg;
        if (tau_last) {
          const float s0 = a.S[(a.sm.base + ci * a.sm.stride) * a.E + slice_off + off];
          phiH_neg = -(s0 + a.hsH * c_act(accH[r] + bv, a.act));
        } else {
          phiH_neg = ghp[off];
        }
        ghp[off] = phiH_neg + ue + res;                  // S_H = U_H - Phi_H(U_H prev) + R   Eq. (15), (24)
        xhp[off] = ue;                                   // injection, Eq. (23)
        if (xlp) xlp[off] = ue;
      }
      if (!is_last) S[row * q + n] = unew;
    }
  };

  for (long long u0 = 0; u0 < total; u0 += NST) {
#pragma unroll
    for (int sl = 0; sl < NST; ++sl) {
      if (u0 + sl < total) {
        if (u0 + sl + NST - 1 < total) issue(wr[(sl + NST - 1) % NST]);
        {
          const WT* arow = A + c * AST + u * KU + arow_k(WT(), g);
          mma_unit(arow, wr[sl], acc);
          if (tau_last && k == nsteps) mma_unit(A0 + c * AST + u * KU + arow_k(WT(), g), wr[sl], accH);
        }
        if (++u == UPB) {
          u = 0;
          block_epilogue();
#pragma unroll
          for (int r = 0; r < 16; ++r) { acc[r] = 0.0f; accH[r] = 0.0f; }
          if (++t == NBW) {
            t = 0;
            ++k;
            if (k <= nsteps) {                            // next step: new operand from the updated state
              __syncthreads();
              build_operand(A, a.lb + ci * a.ls + (long long)(k - 1) * a.lk);
              __syncthreads();
            }
          }
        }
      }
    }
  }

  if (a.norm_partial) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
    __syncthreads();
    if (lane == 0) red[wave] = sq;
    __syncthreads();
    if (tid == 0) a.norm_partial[L] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

}  // namespace

bool chain_supported(int q, int dtype, bool needs_a0) {
  if (q % 128 != 0 || q > 512) return false;
  return chain_smem_bytes(q, dtype, needs_a0) <= 150 * 1024;
}

size_t chain_smem_bytes(int q, int dtype, bool needs_a0) {
  const size_t es = dtype == 0 ? 4 : 2, pad = dtype == 0 ? 4 : 8;
  return (size_t)R * q * 4 + (size_t)(needs_a0 ? 2 : 1) * R * (q + pad) * es;
}

int chain_blocks(int M, int nchains) { return ((M + R - 1) / R) * nchains; }

hipError_t launch_chain(const ChainArgs& a, int dtype, hipStream_t s) {
  if (a.nchains <= 0 || a.nsteps <= 0) return hipSuccess;
  const bool a0 = a.last == LAST_RESID && a.tau_on_last_step;
  const size_t smem = chain_smem_bytes(a.q, dtype, a0);
  const int blocks = chain_blocks(a.M, a.nchains);
  hipError_t e;
  if (dtype == 0) {
    if (smem > 48 * 1024) {
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(dense_chain_kernel<float>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
    }
    trace_before(s);
    hipLaunchKernelGGL((dense_chain_kernel<float>), dim3(blocks), dim3(NT), smem, s, a);
    e = hipGetLastError();
    trace_after(s, TRACE_CHAIN_F32, (long long)a.nchains * a.nsteps, 0.0);
  } else {
    if (smem > 48 * 1024) {
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(dense_chain_kernel<__bf16>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (e != hipSuccess) return e;
    }
    trace_before(s);
    hipLaunchKernelGGL((dense_chain_kernel<__bf16>), dim3(blocks), dim3(NT), smem, s, a);
    e = hipGetLastError();
    trace_after(s, TRACE_CHAIN_BF16, (long long)a.nchains * a.nsteps, 0.0);
  }
  return e;
}

}  // namespace mgrit
