// HIP kernels (gfx950 / CDNA4) of the MGRIT-FAS library: layer-batched residual-block steps
// as grouped MFMA GEMMs / implicit-GEMM 3x3 convolutions with a fused epilogue, the
// bandwidth-bound transfer kernels, the norm reduction and the parameter-gradient kernel.
#include "mgrit_internal.h"

#include <stdlib.h>

#include <type_traits>
#include <vector>

namespace mgrit {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int NT = 256;  // threads per workgroup (4 wavefronts of 64)

// ------------------------------------------------------------------------------------------
// Optional launch tracing (diagnostic, off by default): brackets every step / gradient launch
// with a pair of HIP events on the launch stream and sums elapsed time per kernel class.
// ------------------------------------------------------------------------------------------
namespace {
struct Trace {
  bool on = false;
  std::vector<hipEvent_t> ev;       // pairs
  std::vector<int> cls;
  std::vector<long long> units;
  std::vector<double> bytes;        // algorithmic bytes of the launch (every operand moved once)
  size_t used = 0;                  // pairs in use
} g_trace;

}  // namespace

void trace_before(hipStream_t s) {
  if (!g_trace.on) return;
  if (g_trace.used * 2 + 2 > g_trace.ev.size()) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { g_trace.on = false; return; }
    g_trace.ev.push_back(a);
    g_trace.ev.push_back(b);
  }
  (void)hipEventRecord(g_trace.ev[g_trace.used * 2], s);
}
void trace_after(hipStream_t s, int cls, long long units, double bytes) {
  if (!g_trace.on) return;
  (void)hipEventRecord(g_trace.ev[g_trace.used * 2 + 1], s);
  if (g_trace.cls.size() <= g_trace.used) {
    g_trace.cls.resize(g_trace.used + 1); g_trace.units.resize(g_trace.used + 1); g_trace.bytes.resize(g_trace.used + 1);
  }
  g_trace.cls[g_trace.used] = cls;
  g_trace.units[g_trace.used] = units;
  g_trace.bytes[g_trace.used] = bytes;
  ++g_trace.used;
}

void trace_begin() { g_trace.on = true; g_trace.used = 0; }
int trace_end(double* ms, long long* launches, long long* units, double* bytes, int ncls) {
  g_trace.on = false;
  for (int i = 0; i < ncls; ++i) { ms[i] = 0.0; launches[i] = 0; units[i] = 0; bytes[i] = 0.0; }
  if (g_trace.used == 0) return 0;
  if (hipEventSynchronize(g_trace.ev[g_trace.used * 2 - 1]) != hipSuccess) return -1;
  for (size_t i = 0; i < g_trace.used; ++i) {
    float t = 0.0f;
    if (hipEventElapsedTime(&t, g_trace.ev[2 * i], g_trace.ev[2 * i + 1]) != hipSuccess) return -1;
    const int c = g_trace.cls[i];
    if (c >= 0 && c < ncls) { ms[c] += t; launches[c] += 1; units[c] += g_trace.units[i]; bytes[c] += g_trace.bytes[i]; }
  }
  g_trace.used = 0;
  return 0;
}

// ------------------------------------------------------------------------------------------
// Operand traits.  Matrix-core operands live in LDS as rows of KSTEP-multiples, k fastest.
//   float : v_mfma_f32_32x32x2_f32, a lane feeds 4 consecutive k over 4 instructions
//   bf16  : v_mfma_f32_32x32x16_bf16, a lane feeds 8 consecutive k per instruction
// ------------------------------------------------------------------------------------------
template <typename T> struct Op;
template <> struct Op<float> {
  static constexpr int KSTEP = 8;   // k consumed by one mma_step
  static constexpr int VEC = 4;     // elements per 16-byte piece
  static constexpr int PAD = 4;     // row padding in LDS (elements)
};
template <> struct Op<__bf16> {
  static constexpr int KSTEP = 16;
  static constexpr int VEC = 8;
  static constexpr int PAD = 8;
};

// 16-byte load of layer weights.  STREAM: non-temporal, for parameter sets larger than the 256 MB last-level
// cache -- a weight is used once per launch and must not push out the states, which the next launch reads
// again.  Otherwise a plain load: the whole parameter set stays cached across the launches of a solve
// (measured: 6 % on the q=256 workload with 64 MB of weights, the other way round -0.5 % with 2 GB).
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
template <bool STREAM, typename T>
__device__ __forceinline__ uint4 ld_weights(const T* p) {
  if (STREAM) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
  }
  return *reinterpret_cast<const uint4*>(p);
}
// The act' cache of the adjoint sweep (and of the parameter gradient) is stored in the weights' type: float, or
// bf16 when the matrix-core operands are bf16 anyway (half the bytes of its many reads).  Four consecutive
// values are loaded raw -- no conversion next to the load, which would make the compiler wait for it -- and
// widened when they are used.
__device__ __forceinline__ float4 ld_d4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ uint2 ld_d4(const __bf16* p) { return *reinterpret_cast<const uint2*>(p); }
__device__ __forceinline__ float4 d4_to_f4(float4 r) { return r; }
__device__ __forceinline__ float4 d4_to_f4(uint2 r) {
  return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                     __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
}
template <typename T> struct DRaw;
template <> struct DRaw<float>  { typedef float4 type; };
template <> struct DRaw<__bf16> { typedef uint2 type; };
__device__ __forceinline__ void cvt_store4(float* dst, float4 v) { *reinterpret_cast<float4*>(dst) = v; }
__device__ __forceinline__ void cvt_store4(__bf16* dst, float4 v) {
  bf16x4 o;
  o[0] = static_cast<__bf16>(v.x);   // round to nearest even
  o[1] = static_cast<__bf16>(v.y);
  o[2] = static_cast<__bf16>(v.z);
  o[3] = static_cast<__bf16>(v.w);
  *reinterpret_cast<bf16x4*>(dst) = o;
}

// One KSTEP of the contraction for a TM x TN arrangement of 32x32 blocks.  ap[tm] / bp[tn]
// point at this lane's row (lane % 32 already applied) at the current k offset.
template <int TM, int TN>
__device__ __forceinline__ void mma_step(const float* const (&ap)[TM], const float* const (&bp)[TN],
                                         floatx16 (&acc)[TM][TN], int g) {
  float4 a[TM], b[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const float4*>(ap[i] + 4 * g);
#pragma unroll
  for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const float4*>(bp[j] + 4 * g);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].x, b[j].x, acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].y, b[j].y, acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].z, b[j].z, acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].w, b[j].w, acc[i][j], 0, 0, 0);
    }
}
template <int TM, int TN>
__device__ __forceinline__ void mma_step(const __bf16* const (&ap)[TM], const __bf16* const (&bp)[TN],
                                         floatx16 (&acc)[TM][TN], int g) {
  bf16x8 a[TM], b[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(ap[i] + 8 * g);
#pragma unroll
  for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(bp[j] + 8 * g);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
}

// The same with the weight slab k-major in LDS (row = k, pitch BNP, column = output feature), as the adjoint reads
// W[k][n] untransposed: bk points at row ks of the slab, bcol[j] is this lane's column of block j.
//   float : one value per lane and matrix instruction, k = ks + 4 g + t for instruction t (the A fragment's pairing)
//   bf16  : two LDS transpose reads per fragment.  Within each group of 16 lanes, ds_read_b64_tr_b16 hands lane i
//           element i % 4 of the 8-byte pieces addressed by lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4; with lane
//           l of a group pointing at row l / 4, columns 4 (l % 4) .. + 3, lane i receives rows 0..3 of column i.
typedef short short4v __attribute__((ext_vector_type(4)));
template <int TM, int TN>
__device__ __forceinline__ void mma_step_wn(const float* const (&ap)[TM], const float* bk, int BNP, const int (&bcol)[TN],
                                            floatx16 (&acc)[TM][TN], int g) {
  float4 a[TM];
  float b[TN][4];
#pragma unroll
  for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const float4*>(ap[i] + 4 * g);
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int t = 0; t < 4; ++t) b[j][t] = bk[(4 * g + t) * BNP + bcol[j]];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].x, b[j][0], acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].y, b[j][1], acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].z, b[j][2], acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i].w, b[j][3], acc[i][j], 0, 0, 0);
    }
}
template <int TM, int TN>
__device__ __forceinline__ void mma_step_wn(const __bf16* const (&ap)[TM], const __bf16* bk, int BNP, const int (&bcol)[TN],
                                            floatx16 (&acc)[TM][TN], int g) {
  bf16x8 a[TM], b[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(ap[i] + 8 * g);
  const int l16 = threadIdx.x & 15;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    // bcol[j] = first column of the block + lane % 32; this lane's piece: row 8 g + l16 / 4 (+ 4), columns
    // (bcol - l16) + 4 (l16 % 4) .. + 3, i.e. the 16-column half its group covers
    const __bf16* q = bk + (8 * g + (l16 >> 2)) * BNP + (bcol[j] - l16) + 4 * (l16 & 3);
    typedef __attribute__((address_space(3))) short4v* lds_s4;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(q));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4)(q + 4 * BNP));
    const bf16x4 l4 = __builtin_bit_cast(bf16x4, lo), h4 = __builtin_bit_cast(bf16x4, hi);
    b[j] = __builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7);
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
}

__device__ __forceinline__ floatx16 zero16() {
  floatx16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.0f;
  return z;
}
// tanh(z) = 1 - 2 / (e^{2z} + 1) on the hardware exp2 / rcp units: absolute error about 2e-7
// (the library tanhf costs ~100 instructions per element, which dominated the epilogue).  The
// result enters the state scaled by h, so the absolute error is what matters.
__device__ __forceinline__ float fast_tanh(float z) {
  const float e = __builtin_amdgcn_exp2f(z * 2.885390081777927f);      // e^{2z}; inf / 0 saturate correctly
  return 1.0f - 2.0f * __builtin_amdgcn_rcpf(e + 1.0f);
}
__device__ __forceinline__ float act_fn(float z, int act) {
  if (act == ACT_TANH) return fast_tanh(z);
  if (act == ACT_RELU) return fmaxf(z, 0.0f);
  return z;
}
__device__ __forceinline__ float act_prime(float z, int act) {
  if (act == ACT_TANH) { float t = fast_tanh(z); return 1.0f - t * t; }
  if (act == ACT_RELU) return z > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}
// The same with the activation as a compile-time value: the epilogues of the tiled kernels branch on it once
// per workgroup instead of once per element (a chain of scalar compares and branches around every one of a
// lane's 64 output values took longer than their arithmetic).
template <int ACT> __device__ __forceinline__ float act_fn_c(float z) {
  if (ACT == ACT_TANH) return fast_tanh(z);
  if (ACT == ACT_RELU) return fmaxf(z, 0.0f);
  return z;
}
template <int ACT> __device__ __forceinline__ float act_prime_c(float z) {
  if (ACT == ACT_TANH) { float t = fast_tanh(z); return 1.0f - t * t; }
  if (ACT == ACT_RELU) return z > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}

__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  // fixed order over the wavefronts of the workgroup (4, or 8 in the k-split kernel), two at a time
  float s = (red[0] + red[1]) + (red[2] + red[3]);
  for (int i = 4; i < (int)(blockDim.x >> 6); i += 2) s += red[i] + red[i + 1];
  return s;
}

// (In the kernels below the wavefront index is read with readfirstlane: the compiler cannot see that tid >> 6 is
// the same in all lanes, and with a scalar index the address arithmetic and conditions that depend on it stay on
// the scalar unit.)
// XCD-aware workgroup order: hardware deals consecutive workgroup ids round-robin to the 8
// XCDs; remap so that consecutive logical tiles (which share a group's state and weights)
// land on the same XCD and meet in its L2.
__device__ __forceinline__ int logical_block() {
  int total = gridDim.x, L = blockIdx.x;
  if ((total & 7) == 0) L = (L & 7) * (total >> 3) + (L >> 3);
  return L;
}

// Fused epilogue shared by the dense and the conv kernel, one 32x32 accumulator block at a time:
// register r of lane (g, c) holds row = row0 + 8*(r/4) + 4*g + r%4, column = col0 + c.
struct EpiPtrs {
  const float* Xp;
  float* Op_;
  const float* E1p;
  const float* E2p;
  const float* bp;
};
__device__ __forceinline__ EpiPtrs epi_ptrs(const StepArgs& a, int gi, long long layer) {
  EpiPtrs e;
  e.Xp = a.X + (a.xm.base + gi * a.xm.stride) * a.E;
  e.Op_ = a.Out ? a.Out + (a.om.base + gi * a.om.stride) * a.E : nullptr;
  e.E1p = a.E1 ? a.E1 + (a.e1m.base + gi * a.e1m.stride) * a.E : nullptr;
  e.E2p = a.E2 ? a.E2 + (a.e2m.base + gi * a.e2m.stride) * a.E : nullptr;
  e.bp = a.bias ? a.bias + layer * a.Nf : nullptr;
  return e;
}
// The accumulators of a wavefront's sub-tile go through an LDS staging buffer so that global
// memory is touched in whole rows: a lane handles 4 consecutive columns (one float4) and a wave
// instruction covers 64 / (8 TN) full rows of the sub-tile.  Per 32-row block row: registers ->
// stage (column-consecutive lanes), then batches of row reads with all global loads of a batch
// issued before its arithmetic and stores.  `stage_all` is workgroup LDS of at least
// 4 * 32 * (32 TN + 4) floats that the main loop no longer needs.
// With XREG the skip-connection operand x is not read from memory: the caller hands it over in registers,
// xreg[tm * NIT + h] = the float4 this lane handles in instruction h of block row tm (the conv kernel
// loads its input tile in exactly this arrangement).
// `stage_block(tm, stage)` writes the wavefront's accumulators of block row tm (32 rows x CW columns) to
// `stage` with row stride CW + 4; it is the only part that depends on the MFMA shape.
template <int ACT, int TM, int CW, bool XREG, int NX, typename StageFn>
__device__ __forceinline__ void epilogue_rows_act(const StepArgs& a, int gi, long long layer, StageFn stage_block,
                                              const long long (&row0)[TM], long long row_end, int colbase, int L,
                                              float* red, float* stage_all, const float4 (&xreg)[NX]) {
  constexpr int SW = CW + 4;                 // staging row stride in floats
  constexpr int LPR = CW / 4;                // lanes per sub-tile row
  constexpr int RPI = 64 / LPR;              // rows per wave instruction
  constexpr int NIT = 32 / RPI;              // instructions per block row
  static_assert(!XREG || NX == TM * NIT, "one register operand per lane and row instruction");
  constexpr int HB = NIT < 4 ? NIT : (CW >= 128 ? 8 : 4);   // instructions batched together (register budget)
  const EpiPtrs e = epi_ptrs(a, gi, layer);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* stage = stage_all + wave * 32 * SW;
  const int lrow = lane / LPR, colq = (lane % LPR) * 4;
  const int col = colbase + colq;
  const bool colok = col < a.Nf;
  float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
  if (colok && e.bp) bv = *reinterpret_cast<const float4*>(e.bp + col);
  const bool dact = a.mode == MODE_DACT;
  float sq = 0.0f;
  __syncthreads();                           // every wave is done reading the main loop's LDS tiles
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    stage_block(tm, stage);
#pragma unroll
    for (int h0 = 0; h0 < NIT; h0 += HB) {
      float4 z[HB], xv[HB], e1[HB], e2[HB];
      unsigned off[HB];
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        const int rl = (h0 + i) * RPI + lrow;
        const long long row = row0[tm] + rl;
        const bool ok = colok && row < row_end;
        off[i] = ok ? (unsigned)(row * a.Nf + col) : 0u;          // a state has fewer than 2^31 elements
        z[i] = *reinterpret_cast<const float4*>(&stage[rl * SW + colq]);
      }
      const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
      // unconditional loads (rows / columns outside the tile read element 0 and are never stored)
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        if (XREG) xv[i] = xreg[XREG ? tm * NIT + h0 + i : 0];
        else xv[i] = dact ? zero : *reinterpret_cast<const float4*>(e.Xp + off[i]);
      }
      if (e.E1p) {
#pragma unroll
        for (int i = 0; i < HB; ++i) e1[i] = *reinterpret_cast<const float4*>(e.E1p + off[i]);
      } else {
#pragma unroll
        for (int i = 0; i < HB; ++i) e1[i] = zero;
      }
      if (e.E2p) {
#pragma unroll
        for (int i = 0; i < HB; ++i) e2[i] = *reinterpret_cast<const float4*>(e.E2p + off[i]);
      } else {
#pragma unroll
        for (int i = 0; i < HB; ++i) e2[i] = zero;
      }
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        float4 o;
        if (dact) {
          o.x = act_prime_c<ACT>(z[i].x + bv.x); o.y = act_prime_c<ACT>(z[i].y + bv.y);
          o.z = act_prime_c<ACT>(z[i].z + bv.z); o.w = act_prime_c<ACT>(z[i].w + bv.w);
        } else {
          o.x = a.sp * (xv[i].x + a.hs * act_fn_c<ACT>(z[i].x + bv.x)) + a.c1 * e1[i].x + a.c2 * e2[i].x;
          o.y = a.sp * (xv[i].y + a.hs * act_fn_c<ACT>(z[i].y + bv.y)) + a.c1 * e1[i].y + a.c2 * e2[i].y;
          o.z = a.sp * (xv[i].z + a.hs * act_fn_c<ACT>(z[i].z + bv.z)) + a.c1 * e1[i].z + a.c2 * e2[i].z;
          o.w = a.sp * (xv[i].w + a.hs * act_fn_c<ACT>(z[i].w + bv.w)) + a.c1 * e1[i].w + a.c2 * e2[i].w;
        }
        xv[i] = o;
      }
#pragma unroll
      for (int i = 0; i < HB; ++i) {
        const int rl = (h0 + i) * RPI + lrow;
        const long long row = row0[tm] + rl;
        if (colok && row < row_end) {
          if (dact && a.dbf16) {                     // act' cache of a bf16 problem: 4 x bf16
            __bf16* ob = reinterpret_cast<__bf16*>(a.Out) + (a.om.base + gi * a.om.stride) * a.E;
            cvt_store4(ob + (unsigned)(row * a.Nf + col), xv[i]);
          } else if (e.Op_) {
            *reinterpret_cast<float4*>(e.Op_ + (unsigned)(row * a.Nf + col)) = xv[i];
          }
          sq += (xv[i].x * xv[i].x + xv[i].y * xv[i].y) + (xv[i].z * xv[i].z + xv[i].w * xv[i].w);
        }
      }
    }
  }
  if (a.norm_partial) {
    const float s = block_sum(sq, red);
    if (threadIdx.x == 0) a.norm_partial[L] = s;
  }
}

template <int TM, int CW, bool XREG, int NX, typename StageFn>
__device__ __forceinline__ void epilogue_rows(const StepArgs& a, int gi, long long layer, StageFn stage_block,
                                              const long long (&row0)[TM], long long row_end, int colbase, int L,
                                              float* red, float* stage_all, const float4 (&xreg)[NX]) {
  if (a.act == ACT_TANH)      epilogue_rows_act<ACT_TANH, TM, CW, XREG, NX>(a, gi, layer, stage_block, row0, row_end, colbase, L, red, stage_all, xreg);
  else if (a.act == ACT_RELU) epilogue_rows_act<ACT_RELU, TM, CW, XREG, NX>(a, gi, layer, stage_block, row0, row_end, colbase, L, red, stage_all, xreg);
  else                        epilogue_rows_act<ACT_IDENT, TM, CW, XREG, NX>(a, gi, layer, stage_block, row0, row_end, colbase, L, red, stage_all, xreg);
}

// 32x32 MFMA blocks: register r of a lane holds row 8 (r / 4) + 4 g + r % 4, column c of the block
template <int TM, int TN, bool XREG = false, int NX = 1>
__device__ __forceinline__ void epilogue(const StepArgs& a, int gi, long long layer, floatx16 (&acc)[TM][TN],
                                         const long long (&row0)[TM], long long row_end, int colbase, int L,
                                         float* red, float* stage_all, const float4 (&xreg)[NX]) {
  const int lane = threadIdx.x & 63, g = lane >> 5, c = lane & 31;
  auto stage_block = [&](int tm, float* stage) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * g + (r & 3)) * (TN * 32 + 4) + tn * 32 + c] = acc[tm][tn][r];
  };
  epilogue_rows<TM, TN * 32, XREG, NX>(a, gi, layer, stage_block, row0, row_end, colbase, L, red, stage_all, xreg);
}
template <int TM, int TN>
__device__ __forceinline__ void epilogue(const StepArgs& a, int gi, long long layer, floatx16 (&acc)[TM][TN],
                                         const long long (&row0)[TM], long long row_end, int colbase, int L,
                                         float* red, float* stage_all) {
  const float4 none[1] = {make_float4(0.f, 0.f, 0.f, 0.f)};
  epilogue<TM, TN, false, 1>(a, gi, layer, acc, row0, row_end, colbase, L, red, stage_all, none);
}

// ------------------------------------------------------------------------------------------
// Dense layer-batched step: per group  [M x K] * [Nf x K]^T,  M = batch, Nf = K = q.
// 4 wavefronts arranged WR x WC, each owning TM x TN blocks of 32x32.  Both operands are
// staged through LDS in BK-wide slabs with a register prefetch of the next slab.
// ------------------------------------------------------------------------------------------
// XR (with FULL, square layers, BN = 2 BK, PF = 1): the two k slabs of the state operand that cover the tile's own
// output columns are kept in registers when they pass through, as the skip-connection operand of the epilogue, and
// the epilogue works on the whole 128 x 128 tile in the arrangement of those loads (thread -> 8 rows x 4 columns of
// each 64-column half), so the state is read from memory once per step instead of twice.
// WN: the weights are read as stored, W[k][n] (the adjoint's product, Out = G W): the slab sits k-major in LDS
// and the fragments come from mma_step_wn; otherwise W[n][k] with k fastest (the forward product, Out = X W^T).
template <typename WT, int BM, int BN, int WR, int WC, int BK, int PF, bool WS, bool HD = true, bool FULL = false, bool XR = false, bool WN = false>
__global__ __launch_bounds__(64 * WR * WC, WR * WC == 8 ? 4 : (XR && WN) ? 2 : 1) void dense_step_kernel(StepArgs a) {
  constexpr int NTH = 64 * WR * WC;
  constexpr int ST = BK + Op<WT>::PAD, VEC = Op<WT>::VEC, KSTEP = Op<WT>::KSTEP;
  constexpr int TM = BM / WR / 32, TN = BN / WC / 32;
  constexpr int AP = BM * BK / 4 / NTH;      // float4 pieces of the state slab per thread
  constexpr int BP = BN * BK / VEC / NTH;    // 16-byte pieces of the weight slab per thread
  static_assert(AP >= 1 && BP >= 1 && (WR * WC == 4 || WR * WC == 8) && BK % KSTEP == 0, "tile does not fit the workgroup");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  WT* As = reinterpret_cast<WT*>(smem_raw);          // [BM][ST]
  constexpr int BNP = BN + (sizeof(WT) == 2 ? 16 : 4);   // WN: pitch of a k row (bf16: 32 bytes modulo 128, conflict-free transpose reads)
  constexpr int BPR = WN ? BN / VEC : BK / VEC;      // 16-byte pieces per slab row of the weights
  WT* Bs = As + BM * ST;                             // [BN][ST], or [BK][BNP] with WN
  __shared__ float red[WR * WC];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int tiles_n = (a.Nf + BN - 1) / BN;
  const int L = logical_block();
  const int gi = L / a.tiles, tile = L % a.tiles;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const long long layer = a.wm.base + gi * a.wm.stride;
  const float* Xp = a.X + (a.xm.base + gi * a.xm.stride) * a.E;
  const WT* Dp = HD && a.Dm ? reinterpret_cast<const WT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E : nullptr;
  const WT* Wp = reinterpret_cast<const WT*>(a.W) + layer * a.wsize;
  const int K = a.K;
  typedef typename DRaw<WT>::type DR;

  // PF register sets hold the slabs in flight from global memory.  Loads are unconditional (a
  // predicated load makes the compiler wait for it right away, which serialises the whole slab):
  // out-of-range pieces read element 0 instead and are zeroed when the slab goes to LDS.
  float4 areg[PF][AP];
  constexpr int DP = HD ? AP : 1;          // without the act' factor (HD false) its registers are not reserved
  DR dreg[PF][DP];
  uint4 breg[PF][BP];
  unsigned amask[PF], bmask[PF];
  // FULL (the launch wrapper has checked it): M, Nf and K are whole multiples of the tile, an operand of one group
  // spans less than 4 GB, and HD says whether the act' factor is there.  Then nothing is masked, and a piece's
  // address is a workgroup-uniform base plus a 32-bit byte offset that costs one vector addition per load -- with
  // bf16 matrix instructions the masks, selects and 64-bit address arithmetic of the general path take several
  // times as many issue cycles as the multiplications of a slab.
  const unsigned aoff0 = FULL ? (unsigned)((m0 + tid / (BK / 4)) * K + (tid % (BK / 4)) * 4) : 0u;
  const unsigned boff0 = !FULL ? 0u : WN ? (unsigned)((tid / BPR) * a.Nf + n0 + (tid % BPR) * VEC)
                                         : (unsigned)((n0 + tid / BPR) * K + (tid % BPR) * VEC);
  const unsigned astep = (unsigned)(NTH / (BK / 4)) * (unsigned)K;
  const unsigned bstep = (unsigned)(NTH / BPR) * (unsigned)(WN ? a.Nf : K);
  const char* Xc = reinterpret_cast<const char*>(Xp);
  const char* Dc = reinterpret_cast<const char*>(Dp);
  const char* Wc = reinterpret_cast<const char*>(Wp);
  auto load_slab = [&](float4 (&ar)[AP], DR (&dr)[DP], uint4 (&br)[BP], unsigned& am, unsigned& bm, int k0) {
    if constexpr (FULL) {
#pragma unroll
      for (int i = 0; i < AP; ++i) {
        const unsigned off = aoff0 + (unsigned)i * astep + (unsigned)k0;
        ar[i] = *reinterpret_cast<const float4*>(Xc + 4u * off);
        if (HD) dr[HD ? i : 0] = ld_d4(reinterpret_cast<const WT*>(Dc + (unsigned)sizeof(WT) * off));
      }
#pragma unroll
      for (int i = 0; i < BP; ++i) {
        const unsigned off = boff0 + (unsigned)i * bstep + (WN ? (unsigned)k0 * (unsigned)a.Nf : (unsigned)k0);
        br[i] = ld_weights<WS>(reinterpret_cast<const WT*>(Wc + (unsigned)sizeof(WT) * off));
      }
      return;
    }
    am = 0; bm = 0;
#pragma unroll
    for (int i = 0; i < AP; ++i) {
      const int p = tid + NTH * i, row = p / (BK / 4), kc = (p % (BK / 4)) * 4;
      const bool ok = m0 + row < a.M && k0 + kc < K;
      const unsigned off = ok ? (unsigned)((m0 + row) * K + k0 + kc) : 0u;
      am |= ok ? (1u << i) : 0u;
      ar[i] = *reinterpret_cast<const float4*>(Xp + off);
      if (HD && Dp) dr[HD ? i : 0] = ld_d4(Dp + off);
    }
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      const int p = tid + NTH * i, row = p / BPR, kc = (p % BPR) * VEC;     // WN: row = k, kc = column
      const bool ok = WN ? (k0 + row < K && n0 + kc < a.Nf) : (n0 + row < a.Nf && k0 + kc < K);
      const unsigned off = !ok ? 0u : WN ? (unsigned)((k0 + row) * a.Nf + n0 + kc) : (unsigned)((n0 + row) * K + k0 + kc);
      bm |= ok ? (1u << i) : 0u;
      br[i] = ld_weights<WS>(Wp + off);
    }
  };
  auto store_slab = [&](const float4 (&ar)[AP], const DR (&dr)[DP], const uint4 (&br)[BP], unsigned am,
                        unsigned bm) {
#pragma unroll
    for (int i = 0; i < AP; ++i) {
      const int p = tid + NTH * i, row = p / (BK / 4), kc = (p % (BK / 4)) * 4;
      float4 v = ar[i];
      if (HD && (FULL || Dp)) { const float4 d = d4_to_f4(dr[HD ? i : 0]); v.x *= d.x; v.y *= d.y; v.z *= d.z; v.w *= d.w; }
      if (!FULL && !((am >> i) & 1u)) v = make_float4(0.f, 0.f, 0.f, 0.f);
      cvt_store4(&As[row * ST + kc], v);
    }
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      const int p = tid + NTH * i, row = p / BPR, kc = (p % BPR) * VEC;
      uint4 v = br[i];
      if (!FULL && !((bm >> i) & 1u)) v = make_uint4(0, 0, 0, 0);
      *reinterpret_cast<uint4*>(&Bs[row * (WN ? BNP : ST) + kc]) = v;
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = zero16();
  static_assert(!XR || (FULL && PF == 1 && BN == 2 * BK && BM == 128 && NTH == 256), "XR: whole 128 x 128 tiles, two slabs per tile width");
  constexpr int NXO = XR ? AP : 1;
  float4 xown[2][NXO];

  const int wm0 = (wave / WC) * (BM / WR), wn0 = (wave % WC) * (BN / WC);
  // The k slabs are visited in a rotated order that depends on the group: with a power-of-two
  // row pitch every workgroup would otherwise ask the same HBM channels for the same k at the
  // same time.  Workgroups of one group keep a common order, so they still meet in L2.
  const int nk = (K + BK - 1) / BK;
  const int rot = (int)(((long long)gi * 5) % nk);
  auto slab_k0 = [&](int j) { int sl = rot + j; if (sl >= nk) sl -= nk; return sl * BK; };
#pragma unroll
  for (int sidx = 0; sidx < PF; ++sidx)
    if (sidx < nk) load_slab(areg[sidx], dreg[sidx], breg[sidx], amask[sidx], bmask[sidx], slab_k0(sidx));
  for (int it0 = 0; it0 < nk; it0 += PF) {
#pragma unroll
    for (int sidx = 0; sidx < PF; ++sidx) {
      const int it = it0 + sidx;
      if (it < nk) {
        __syncthreads();
        store_slab(areg[sidx], dreg[sidx], breg[sidx], amask[sidx], bmask[sidx]);
        if constexpr (XR) {
          const int kcur = slab_k0(it);
          // (component by component: a struct copy under a condition becomes a memcpy into private memory,
          // which would put the kept slabs into scratch)
          if (kcur == n0) {
#pragma unroll
            for (int q = 0; q < AP; ++q) {
              xown[0][q].x = areg[sidx][q].x; xown[0][q].y = areg[sidx][q].y;
              xown[0][q].z = areg[sidx][q].z; xown[0][q].w = areg[sidx][q].w;
            }
          } else if (kcur == n0 + BK) {
#pragma unroll
            for (int q = 0; q < AP; ++q) {
              xown[1][q].x = areg[sidx][q].x; xown[1][q].y = areg[sidx][q].y;
              xown[1][q].z = areg[sidx][q].z; xown[1][q].w = areg[sidx][q].w;
            }
          }
        }
        __syncthreads();
        if (it + PF < nk) load_slab(areg[sidx], dreg[sidx], breg[sidx], amask[sidx], bmask[sidx], slab_k0(it + PF));
#pragma unroll
        for (int ks = 0; ks < BK; ks += KSTEP) {
          const WT* ap[TM];
#pragma unroll
          for (int i = 0; i < TM; ++i) ap[i] = &As[(wm0 + i * 32 + c) * ST + ks];
          if constexpr (WN) {
            int bcol[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) bcol[j] = wn0 + j * 32 + c;
            mma_step_wn<TM, TN>(ap, Bs + ks * BNP, BNP, bcol, acc, g);
          } else {
            const WT* bp[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) bp[j] = &Bs[(wn0 + j * 32 + c) * ST + ks];
            mma_step<TM, TN>(ap, bp, acc, g);
          }
        }
      }
    }
  }

  if constexpr (XR) {
    // whole-tile epilogue: accumulators -> LDS [BM][BN + 4], then thread (rq, cq) handles rows rq + 16 i, columns
    // 64 half + 4 cq .. + 3 -- the float4 it loaded for the state slabs k0 = n0 and n0 + BK
    constexpr int SWF = BN + 4;
    float* stage = reinterpret_cast<float*>(smem_raw);
    __syncthreads();                           // every wavefront is done reading the operand tiles
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int jn = 0; jn < TN; ++jn)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          stage[(wm0 + i * 32 + 8 * (r >> 2) + 4 * g + (r & 3)) * SWF + wn0 + jn * 32 + c] = acc[i][jn][r];
    __syncthreads();
    const EpiPtrs e = epi_ptrs(a, gi, layer);
    const int rq = tid / (BK / 4), cq = (tid % (BK / 4)) * 4;
    const bool dact = a.mode == MODE_DACT;
    float sq = 0.0f;
    auto tile_rows = [&](auto actc) {
    constexpr int ACT = decltype(actc)::value;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int col = n0 + half * BK + cq;
      float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e.bp) bv = *reinterpret_cast<const float4*>(e.bp + col);
#pragma unroll
      for (int h0 = 0; h0 < AP; h0 += 4) {
        float4 z[4], e1[4], e2[4];
        unsigned off[4];
        const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int row = rq + (NTH / (BK / 4)) * (h0 + u);
          off[u] = (unsigned)((m0 + row) * a.Nf + col);
          z[u] = *reinterpret_cast<const float4*>(&stage[row * SWF + half * BK + cq]);
        }
        // (branches, not selects: a select between a load and a constant becomes a select of two addresses,
        // one of them in private memory, and a generic load)
        if (e.E1p) {
#pragma unroll
          for (int u = 0; u < 4; ++u) e1[u] = *reinterpret_cast<const float4*>(e.E1p + off[u]);
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) e1[u] = zero;
        }
        if (e.E2p) {
#pragma unroll
          for (int u = 0; u < 4; ++u) e2[u] = *reinterpret_cast<const float4*>(e.E2p + off[u]);
        } else {
#pragma unroll
          for (int u = 0; u < 4; ++u) e2[u] = zero;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const float4 xv = xown[half][XR ? h0 + u : 0];
          float4 o;
          if (dact) {
            o.x = act_prime_c<ACT>(z[u].x + bv.x); o.y = act_prime_c<ACT>(z[u].y + bv.y);
            o.z = act_prime_c<ACT>(z[u].z + bv.z); o.w = act_prime_c<ACT>(z[u].w + bv.w);
          } else {
            o.x = a.sp * (xv.x + a.hs * act_fn_c<ACT>(z[u].x + bv.x)) + a.c1 * e1[u].x + a.c2 * e2[u].x;
            o.y = a.sp * (xv.y + a.hs * act_fn_c<ACT>(z[u].y + bv.y)) + a.c1 * e1[u].y + a.c2 * e2[u].y;
            o.z = a.sp * (xv.z + a.hs * act_fn_c<ACT>(z[u].z + bv.z)) + a.c1 * e1[u].z + a.c2 * e2[u].z;
            o.w = a.sp * (xv.w + a.hs * act_fn_c<ACT>(z[u].w + bv.w)) + a.c1 * e1[u].w + a.c2 * e2[u].w;
          }
          if (dact && a.dbf16) {
            __bf16* ob = reinterpret_cast<__bf16*>(a.Out) + (a.om.base + gi * a.om.stride) * a.E;
            cvt_store4(ob + off[u], o);
          } else if (e.Op_) {
            *reinterpret_cast<float4*>(e.Op_ + off[u]) = o;
          }
          sq += (o.x * o.x + o.y * o.y) + (o.z * o.z + o.w * o.w);
        }
      }
    }
    };
    if (a.act == ACT_TANH)      tile_rows(std::integral_constant<int, ACT_TANH>{});
    else if (a.act == ACT_RELU) tile_rows(std::integral_constant<int, ACT_RELU>{});
    else                        tile_rows(std::integral_constant<int, ACT_IDENT>{});
    if (a.norm_partial) {
      const float sum = block_sum(sq, red);
      if (threadIdx.x == 0) a.norm_partial[L] = sum;
    }
    return;
  }
  long long row0[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) row0[i] = m0 + wm0 + i * 32;
  epilogue<TM, TN>(a, gi, layer, acc, row0, (long long)a.M, n0 + wn0, L, red, reinterpret_cast<float*>(smem_raw));
}

// ------------------------------------------------------------------------------------------
// Dense step for SMALL launches (coarse levels, narrow layers) and for skinny ones (at most 32 rows and a
// long contraction, e.g. a fully connected layer on 32 flattened images, which only streams its weights),
// built for latency instead of reuse: a workgroup owns a 32-row x 32-column output tile and its NW wavefronts
// split the contraction in pieces of KC / 2 values of k (128 bytes of a weight row), round robin.  A wavefront
// loads its piece of both operands with whole-line accesses (8 lanes per 128-byte row piece), passes it through
// an LDS area of its own and reads the MFMA fragments from there -- no workgroup barrier in the k loop -- with
// the loads of its next two pieces in flight in two register sets.  (Fragment loads straight from global
// memory touch 32 cache lines per instruction and use 32 bytes of each: the address path of the CU, not the
// memory, then sets the time -- 1.79 against 1.63 ms per step of the q = 256 workload, 7.5 against 5.7 ms for
// the stack with 4096-wide fully connected layers.)  The operands of the fused epilogue are requested before
// the k loop starts; the NW partial tiles are summed through LDS in a fixed order.  NW = 4, or 8 when the
// launch has fewer workgroups than the chip has CUs: the time of such a launch is the number of pieces a
// wavefront walks through times the memory latency.
// WN: the weights are W[k][n] (the adjoint on the caller's array).  A piece is then KC / 2 rows of 32 columns
// (128 or 64 bytes each), staged k-major with a row pitch of 36 elements and read with mma_step_wn's accesses.
// ------------------------------------------------------------------------------------------
template <typename WT> struct KsOp;
template <> struct KsOp<float>  { static constexpr int KC = 64;  };   // a piece is KC / 2 values of k: 4 fragments x (4 k per lane group) x 2 groups
template <> struct KsOp<__bf16> { static constexpr int KC = 128; };   // 4 fragments x (8 k per lane group) x 2 groups

__device__ __forceinline__ void ks_piece(const float* ap, const float* bp, floatx16& acc) {
  const float4 av = *reinterpret_cast<const float4*>(ap), bv = *reinterpret_cast<const float4*>(bp);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, bv.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, bv.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, bv.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, bv.w, acc, 0, 0, 0);
}
__device__ __forceinline__ void ks_piece(const __bf16* ap, const __bf16* bp, floatx16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8*>(ap), *reinterpret_cast<const bf16x8*>(bp),
                                                acc, 0, 0, 0);
}
// its LDS: per wavefront one [32][KC / 2 + PAD] area for each operand (144-byte rows)
template <typename WT> constexpr size_t ksplit_smem(int nw) {
  return (size_t)nw * 2 * 32 * (KsOp<WT>::KC / 2 + Op<WT>::PAD) * sizeof(WT);
}

template <typename WT, bool WS, int NW, bool WN = false>
__global__ __launch_bounds__(NW * 64) void dense_ksplit_kernel(StepArgs a) {
  static_assert(NW == 4 || NW == 8, "four or eight wavefronts");
  constexpr int KC = KsOp<WT>::KC;
  constexpr bool BF = sizeof(WT) == 2;
  constexpr int KL = BF ? 8 : 4;                    // consecutive k a lane feeds per piece
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];   // the wavefronts' staging areas
  static_assert(ksplit_smem<WT>(NW) >= sizeof(float) * NW * 32 * 36, "the partial tiles reuse the staging areas");
  float (*part)[32][36] = reinterpret_cast<float (*)[32][36]>(smem_raw);     // [NW][32][36], after the k loop
  __shared__ float red[NW];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int tiles_n = (a.Nf + 31) / 32;
  const int L = logical_block();
  const int gi = L / a.tiles, tile = L % a.tiles;
  const int m0 = (tile / tiles_n) * 32, n0 = (tile % tiles_n) * 32;
  const long long layer = a.wm.base + gi * a.wm.stride;
  const float* Xp = a.X + (a.xm.base + gi * a.xm.stride) * a.E;
  const WT* Dp = a.Dm ? reinterpret_cast<const WT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E : nullptr;
  const WT* Wp = reinterpret_cast<const WT*>(a.W) + layer * a.wsize;
  const int K = a.K;
  typedef typename DRaw<WT>::type DR;
  const EpiPtrs e = epi_ptrs(a, gi, layer);

  // ---- epilogue operands first (one float4 per thread of the first four wavefronts: row tid/8, columns
  // 4*(tid%8)..+3)
  const int erow = m0 + ((tid & 255) >> 3), ecol = n0 + 4 * (tid & 7);
  const bool eok = (NW == 4 || tid < 256) && erow < a.M && ecol < a.Nf;
  const unsigned eoff = eok ? (unsigned)(erow * a.Nf + ecol) : 0u;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool dact = a.mode == MODE_DACT;
  float4 xv = zero, e1 = zero, e2 = zero, bv = zero;
  if (!dact) xv = *reinterpret_cast<const float4*>(e.Xp + eoff);
  if (e.E1p) e1 = *reinterpret_cast<const float4*>(e.E1p + eoff);
  if (e.E2p) e2 = *reinterpret_cast<const float4*>(e.E2p + eoff);
  if (e.bp && ecol < a.Nf) bv = *reinterpret_cast<const float4*>(e.bp + ecol);

  // ---- k loop.  MFMA lane (c, g) feeds row m0+c of the state and row n0+c of the weights, KL consecutive k
  // at offset 2*KL*j + KL*g of the piece in fragment j
  floatx16 acc1[1][1];
  floatx16& acc = acc1[0][0];
  acc = zero16();
  {
    // pieces of KH = KC / 2 values of k (128 bytes of a weight row): two of them are in flight in two register
    // sets, so the loads of the next piece never wait for the current one to be consumed
    constexpr int VEC = Op<WT>::VEC;
    constexpr int KH = KC / 2;
    constexpr int LST = KH + Op<WT>::PAD;           // LDS row stride in elements (144 bytes)
    constexpr int WI = 4;                           // weight loads per piece: 8 rows x 8 lanes (128 bytes) each
    constexpr int APR = KH / 4;                     // float4 parts of a state row per piece: 8 or 16
    constexpr int ARI = 64 / APR;                   // state rows per load instruction: 8 or 4
    constexpr int AI = 32 / ARI;                    // state loads per piece: 4 or 8
    WT* Wl = reinterpret_cast<WT*>(smem_raw) + wave * (2 * 32 * LST);
    WT* Al = Wl + 32 * LST;
    const int wrl = lane >> 3, wkc = (lane & 7) * VEC;          // weights: row 8 i + wrl
    // WN: 32 / VEC lanes cover the 32 columns of a k row, 64 / (32 / VEC) rows per load instruction
    constexpr int NLR = 32 / VEC, NRI = 64 / NLR, NPITCH = 36;
    static_assert(!WN || (NRI * WI == KH && KH * NPITCH <= 32 * LST), "a k-major piece fills the same staging area");
    const int nrl = lane / NLR, nnc = (lane % NLR) * VEC;       // k row NRI i + nrl, columns nnc .. + VEC - 1
    const int arl = lane / APR, akc = (lane % APR) * 4;         // state: row ARI i + arl
    uint4 wr[2][WI];
    float4 ar[2][AI];
    DR dr[2][AI];
    unsigned wmask[2] = {0u, 0u}, amask[2] = {0u, 0u};
    auto load_piece = [&](uint4 (&w)[WI], float4 (&x)[AI], DR (&d)[AI], unsigned& wm, unsigned& am, int k0) {
      wm = 0; am = 0;
#pragma unroll
      for (int i = 0; i < WI; ++i) {
        bool ok;
        unsigned off;
        if constexpr (WN) {
          const int k = k0 + NRI * i + nrl, col = n0 + nnc;
          ok = k < K && col < a.Nf;                  // Nf % 8 == 0: a 16-byte part is in or out as a whole
          off = (unsigned)(k * a.Nf + col);
        } else {
          const int row = n0 + 8 * i + wrl, k = k0 + wkc;
          ok = row < a.Nf && k < K;                  // K % 8 == 0: a 16-byte part is in or out as a whole
          off = (unsigned)(row * K + k);
        }
        wm |= ok ? (1u << i) : 0u;
        w[i] = ld_weights<WS>(Wp + (ok ? off : 0u));
      }
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        const int row = m0 + ARI * i + arl, k = k0 + akc;
        const bool ok = row < a.M && k < K;
        const unsigned off = ok ? (unsigned)(row * K + k) : 0u;
        am |= ok ? (1u << i) : 0u;
        x[i] = *reinterpret_cast<const float4*>(Xp + off);
        if (Dp) d[i] = ld_d4(Dp + off);
      }
    };
    // one piece: registers -> this wavefront's LDS area -> MFMA fragments.  The area belongs to this wavefront
    // alone, whose LDS operations execute in order; the fences only keep the compiler from moving the fragment
    // reads across the stores.
    auto consume_piece = [&](const uint4 (&w)[WI], const float4 (&x)[AI], const DR (&d)[AI], unsigned wm, unsigned am) {
#pragma unroll
      for (int i = 0; i < WI; ++i) {
        uint4 v = w[i];
        if (!((wm >> i) & 1u)) v = make_uint4(0, 0, 0, 0);
        if constexpr (!WN) {
          *reinterpret_cast<uint4*>(&Wl[(8 * i + wrl) * LST + wkc]) = v;
        } else if constexpr (BF) {                   // 72-byte rows: two 8-byte stores
          uint2* q = reinterpret_cast<uint2*>(&Wl[(NRI * i + nrl) * NPITCH + nnc]);
          q[0] = make_uint2(v.x, v.y); q[1] = make_uint2(v.z, v.w);
        } else {
          *reinterpret_cast<uint4*>(&Wl[(NRI * i + nrl) * NPITCH + nnc]) = v;
        }
      }
#pragma unroll
      for (int i = 0; i < AI; ++i) {
        float4 v = x[i];
        if (Dp) { const float4 dd = d4_to_f4(d[i]); v.x *= dd.x; v.y *= dd.y; v.z *= dd.z; v.w *= dd.w; }
        if (!((am >> i) & 1u)) v = zero;
        cvt_store4(&Al[(ARI * i + arl) * LST + akc], v);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if constexpr (WN) {
          const WT* ap[1] = {&Al[c * LST + 2 * KL * j]};
          const int bcol[1] = {c};
          mma_step_wn<1, 1>(ap, Wl + 2 * KL * j * NPITCH, NPITCH, bcol, acc1, g);
        } else {
          ks_piece(&Al[c * LST + 2 * KL * j + KL * g], &Wl[c * LST + 2 * KL * j + KL * g], acc);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // piece h of the contraction starts at k = h * KH; this wavefront takes h = wave, wave + NW, ...
    const int nh = (K + KH - 1) / KH;
    int h = wave;
    if (h < nh) load_piece(wr[0], ar[0], dr[0], wmask[0], amask[0], h * KH);
    if (h + NW < nh) load_piece(wr[1], ar[1], dr[1], wmask[1], amask[1], (h + NW) * KH);
    for (; h < nh; h += 2 * NW) {
      consume_piece(wr[0], ar[0], dr[0], wmask[0], amask[0]);
      if (h + 2 * NW < nh) load_piece(wr[0], ar[0], dr[0], wmask[0], amask[0], (h + 2 * NW) * KH);
      if (h + NW < nh) {
        consume_piece(wr[1], ar[1], dr[1], wmask[1], amask[1]);
        if (h + 3 * NW < nh) load_piece(wr[1], ar[1], dr[1], wmask[1], amask[1], (h + 3 * NW) * KH);
      }
    }
    __syncthreads();                                 // every wavefront has left its staging area: the partial tiles go there
  }

  // ---- sum the NW partial tiles (fixed order) and apply the fused epilogue
#pragma unroll
  for (int r = 0; r < 16; ++r) part[wave][8 * (r >> 2) + 4 * g + (r & 3)][c] = acc[r];
  __syncthreads();
  const int pr = (tid & 255) >> 3, pc = 4 * (tid & 7);
  float4 z = *reinterpret_cast<const float4*>(&part[0][pr][pc]);
#pragma unroll
  for (int w = 1; w < NW; ++w) {
    const float4 t = *reinterpret_cast<const float4*>(&part[w][pr][pc]);
    z.x += t.x; z.y += t.y; z.z += t.z; z.w += t.w;
  }
  float4 o;
  if (dact) {
    o.x = act_prime(z.x + bv.x, a.act); o.y = act_prime(z.y + bv.y, a.act);
    o.z = act_prime(z.z + bv.z, a.act); o.w = act_prime(z.w + bv.w, a.act);
  } else {
    o.x = a.sp * (xv.x + a.hs * act_fn(z.x + bv.x, a.act)) + a.c1 * e1.x + a.c2 * e2.x;
    o.y = a.sp * (xv.y + a.hs * act_fn(z.y + bv.y, a.act)) + a.c1 * e1.y + a.c2 * e2.y;
    o.z = a.sp * (xv.z + a.hs * act_fn(z.z + bv.z, a.act)) + a.c1 * e1.z + a.c2 * e2.z;
    o.w = a.sp * (xv.w + a.hs * act_fn(z.w + bv.w, a.act)) + a.c1 * e1.w + a.c2 * e2.w;
  }
  float sq = 0.0f;
  if (eok) {
    if (dact && a.dbf16) cvt_store4(reinterpret_cast<__bf16*>(a.Out) + (a.om.base + gi * a.om.stride) * a.E + eoff, o);
    else if (e.Op_) *reinterpret_cast<float4*>(e.Op_ + eoff) = o;
    sq = (o.x * o.x + o.y * o.y) + (o.z * o.z + o.w * o.w);
  }
  if (a.norm_partial) {
    const float s = block_sum(sq, red);
    if (threadIdx.x == 0) a.norm_partial[L] = s;
  }
}

// ------------------------------------------------------------------------------------------
// 3x3 convolution layer-batched step as an implicit GEMM: per group M = B*H*W pixels,
// N = C output channels, K = 9*C.  A workgroup owns TH full image rows of one image (at most
// 256 pixels = 8 blocks of 32, two per wavefront); the input patch with its one-pixel halo is
// loaded to LDS once (zero padding materialised there) and the nine taps read it at shifted
// offsets, while the [C_out][C_in] weight slice of each tap streams through LDS.
// ------------------------------------------------------------------------------------------
// N16 (float only, at most 16 channels): the output-channel side uses 16x16x4 MFMA blocks, so none of the
// matrix-core work is spent on padding columns; a wavefront then owns 4 blocks of 16 pixels.
typedef float floatx4 __attribute__((ext_vector_type(4)));
// p / w for 0 <= p < 4096 and 1 <= w <= 256 with magic = ceil(2^20 / w): exact because p * (magic * w - 2^20) < 2^20
__device__ __forceinline__ int div_small(int p, unsigned magic) { return (int)(((unsigned)p * magic) >> 20); }
// CFIX > 0: the channel count is this compile-time value (a multiple of the MFMA's k step that fills the
// workgroup's output columns), so the tap loop unrolls with its LDS reads ahead of the matrix instructions and
// the weight pieces need neither masks nor divisions -- with bf16 matrix instructions a tap is 16 of them per
// wavefront, and a rolled k loop that waits for every fragment read takes several times as long.
template <typename WT, int TN, bool N16 = false, int CFIX = 0>
__global__ __launch_bounds__(NT, 2) void conv_step_kernel(StepArgs a) {   // two workgroups per CU: at most 256 registers
  static_assert(!N16 || (sizeof(WT) == 4 && TN == 1), "the 16-wide variant is float only");
  static_assert(CFIX == 0 || (!N16 && CFIX == 32 * TN && CFIX % Op<WT>::KSTEP == 0), "fixed channel count = output columns");
  constexpr int VEC = Op<WT>::VEC, KSTEP = N16 ? 16 : Op<WT>::KSTEP, PAD = Op<WT>::PAD;
  constexpr int TM = 2;
  constexpr int CW = N16 ? 16 : 32 * TN;    // output channels a workgroup covers
  constexpr int CPMAX = CW;
  constexpr int WP = (CW * CPMAX / VEC + NT - 1) / NT;        // weight pieces per thread per tap
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  __shared__ float red[4];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int C = CFIX ? CFIX : a.Nf, H = a.Himg, Wd = a.Wimg, TH = a.TH;
  const int Cp = N16 ? 16 : CFIX ? CFIX : (C + KSTEP - 1) / KSTEP * KSTEP;   // a compile-time value in the 16-wide and the fixed variant
  const int CS = Cp + PAD;
  const int PW = Wd + 2;
  WT* patch = reinterpret_cast<WT*>(smem_raw);
  WT* wts = patch + (TH + 2) * PW * CS;

  const int L = logical_block();
  const int gi = L / a.tiles, tile = L % a.tiles;
  if (a.skipper > 0 && gi >= a.skip0 && (gi - a.skip0) % a.skipper == 0) {   // not a convolution layer (whole workgroup)
    if (a.norm_partial && threadIdx.x == 0) a.norm_partial[L] = 0.0f;
    return;
  }
  const int tiles_per_img = (H + TH - 1) / TH;
  const int bimg = tile / tiles_per_img, y0 = (tile % tiles_per_img) * TH;
  const long long layer = a.wm.base + gi * a.wm.stride;
  const float* Xp = a.X + (a.xm.base + gi * a.xm.stride) * a.E;
  const WT* Dp = a.Dm ? reinterpret_cast<const WT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E : nullptr;
  const WT* Wp = reinterpret_cast<const WT*>(a.W) + layer * a.wsize;
  typedef typename DRaw<WT>::type DR;

  // 16-wide variant: the nine [C_out][C_in] slices are 9 x 16 x 16 floats in all.  They are requested first (their
  // latency hides behind the patch loads), written to LDS once, and the taps run without a weight ring and
  // without barriers between them.
  constexpr int WALL = N16 ? 3 : 1;           // 16-byte pieces per thread: 9 taps x 16 rows x 4 pieces = 576 <= 3 x 256
  uint4 wall[WALL];
  unsigned wallmask = 0;
  if constexpr (N16) {
#pragma unroll
    for (int i = 0; i < WALL; ++i) {
      const int p = tid + NT * i;
      const int tap = p >> 6, row = (p >> 2) & 15, kc = (p & 3) * 4;
      const bool ok = p < 576 && row < C && kc < C;
      const unsigned off = ok ? (unsigned)((row * 9 + tap) * C + kc) : 0u;
      wallmask |= ok ? (1u << i) : 0u;
      wall[i] = *reinterpret_cast<const uint4*>(Wp + off);
    }
  }

  // ---- input patch -> LDS (converted to the operand type).  The tile's own pixels are loaded in the
  // arrangement of the epilogue (lane -> 4 channels of a pixel row, NIT rows per 32-pixel block), so the
  // float values stay in registers as the skip-connection operand and the state is read from memory once;
  // the halo rows above and below come in the same batch.  Loads are unconditional (pieces outside the
  // image or the tile read element 0 and are zeroed afterwards); the side columns of the patch are the
  // zero padding of the image.
  constexpr int LPR = CW / 4, RPI = 64 / LPR, NIT = 32 / RPI, NX = TM * NIT;
  const int npx = min(TH, H - y0) * Wd;      // valid pixels of this tile
  const int lrow = lane / LPR, colq = (lane % LPR) * 4;
  float4 xreg[NX];
  {
    unsigned okm = 0;
#pragma unroll
    for (int i = 0; i < NX; ++i) {
      const int p = (wave * TM + i / NIT) * 32 + (i % NIT) * RPI + lrow;      // tile pixel
      const bool ok = p < npx && colq < C;
      const unsigned off = ok ? (unsigned)((((long long)bimg * H + y0) * Wd + p) * C + colq) : 0u;
      okm |= ok ? (1u << i) : 0u;
      xreg[i] = *reinterpret_cast<const float4*>(Xp + off);
    }
    // halo: patch rows 0 and TH+1 (image rows y0-1 and y0+TH), interior columns only
    const int cq = Cp / 4;
    const int htotal = 2 * Wd * cq;
    constexpr int HU = N16 ? 1 : 4;          // the 16-wide variant has small halos: one piece per thread and pass
    for (int p0 = tid; p0 < htotal; p0 += NT * HU) {
      float4 v[HU];
      DR d[HU];
      unsigned hm = 0;
#pragma unroll
      for (int u = 0; u < HU; ++u) {
        const int p = p0 + u * NT;
        const int pp = p / cq, c4 = (p % cq) * 4;
        const int prow = pp < Wd ? 0 : TH + 1, gx = pp < Wd ? pp : pp - Wd;
        const int gy = y0 - 1 + prow;
        const bool ok = p < htotal && gy >= 0 && gy < H && c4 < C;
        const unsigned off = ok ? (unsigned)((((long long)bimg * H + gy) * Wd + gx) * C + c4) : 0u;
        hm |= ok ? (1u << u) : 0u;
        v[u] = *reinterpret_cast<const float4*>(Xp + off);
        if (Dp) d[u] = ld_d4(Dp + off);
      }
#pragma unroll
      for (int u = 0; u < HU; ++u) {
        const int p = p0 + u * NT;
        if (p < htotal) {
          const int pp = p / cq, c4 = (p % cq) * 4;
          const int prow = pp < Wd ? 0 : TH + 1, gx = pp < Wd ? pp : pp - Wd;
          float4 w = v[u];
          if (Dp) { const float4 dd = d4_to_f4(d[u]); w.x *= dd.x; w.y *= dd.y; w.z *= dd.z; w.w *= dd.w; }
          if (!((hm >> u) & 1u)) w = make_float4(0.f, 0.f, 0.f, 0.f);
          cvt_store4(&patch[(prow * PW + gx + 1) * CS + c4], w);
        }
      }
    }
    // side columns (x = -1 and x = Wd) of every patch row: zero
    for (int p = tid; p < 2 * (TH + 2) * cq; p += NT) {
      const int pp = p / cq, c4 = (p % cq) * 4;
      const int prow = pp >> 1, pcol = (pp & 1) ? PW - 1 : 0;
      cvt_store4(&patch[(prow * PW + pcol) * CS + c4], make_float4(0.f, 0.f, 0.f, 0.f));
    }
    // the tile's own pixels: operand copy to LDS (zero below the last valid row and for padded channels);
    // the act' factors of the adjoint sweep are fetched one block row at a time to bound the registers
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
      DR dreg[NIT];
      if (Dp) {
#pragma unroll
        for (int h = 0; h < NIT; ++h) {
          const int p = (wave * TM + tm) * 32 + h * RPI + lrow;
          const bool ok = (okm >> (tm * NIT + h)) & 1u;
          const unsigned off = ok ? (unsigned)((((long long)bimg * H + y0) * Wd + p) * C + colq) : 0u;
          dreg[h] = ld_d4(Dp + off);
        }
      }
#pragma unroll
      for (int h = 0; h < NIT; ++h) {
        const int i = tm * NIT + h;
        const int p = (wave * TM + tm) * 32 + h * RPI + lrow;
        if (p < TH * Wd && colq < Cp) {
          float4 w = xreg[i];
          if (Dp) { const float4 dd = d4_to_f4(dreg[h]); w.x *= dd.x; w.y *= dd.y; w.z *= dd.z; w.w *= dd.w; }
          if (!((okm >> i) & 1u)) w = make_float4(0.f, 0.f, 0.f, 0.f);
          const int py = div_small(p, a.wmagic);           // p / Wd without the division sequence
          cvt_store4(&patch[((py + 1) * PW + (p - py * Wd) + 1) * CS + colq], w);
        }
      }
    }
  }

  // ---- weight slice of one tap: rows = output channel, k = input channel
  const int wq = Cp / VEC;
  const int wtotal = CW * wq;
  // two register sets and two LDS buffers: while tap t is multiplied out of one buffer, tap t+1
  // goes from registers into the other and taps t+2, t+3 are in flight from global memory
  uint4 wreg[2][WP];
  unsigned wmask[2] = {0u, 0u};
  auto load_w = [&](uint4 (&wr)[WP], unsigned& wm, int tap) {
    wm = 0;
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int p = tid + NT * i;
      const int row = p / wq, kc = (p % wq) * VEC;
      const bool ok = p < wtotal && row < C && kc < C;
      const unsigned off = ok ? (unsigned)((row * 9 + tap) * C + kc) : 0u;
      wm |= ok ? (1u << i) : 0u;
      wr[i] = *reinterpret_cast<const uint4*>(Wp + off);
    }
  };
  auto store_w = [&](const uint4 (&wr)[WP], unsigned wm, WT* dst) {
#pragma unroll
    for (int i = 0; i < WP; ++i) {
      const int p = tid + NT * i;
      if (p < wtotal) {
        const int row = p / wq, kc = (p % wq) * VEC;
        uint4 v = wr[i];
        if (!((wm >> i) & 1u)) v = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(&dst[row * CS + kc]) = v;
      }
    }
  };
  if constexpr (!N16) {
    load_w(wreg[0], wmask[0], 0);
    load_w(wreg[1], wmask[1], 1);
  }

  // A-operand rows of this lane: 32x32 blocks -> pixel (wave*TM + i)*32 + lane%32;
  // 16x16 blocks -> pixel wave*64 + 16*b + lane%16 (k group lane/16)
  constexpr int NA = N16 ? 4 : TM;
  const int r16 = lane & 15, kq = lane >> 4;
  int aoff[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int p = N16 ? wave * 64 + 16 * i + r16 : (wave * TM + i) * 32 + c;
    if (p >= npx) p = 0;                      // masked rows compute on pixel 0 and are dropped
    const int py = div_small(p, a.wmagic);
    aoff[i] = (py * PW + (p - py * Wd)) * CS;
  }

  floatx16 acc[TM][TN];
  floatx4 acc16[4];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = zero16();
#pragma unroll
  for (int i = 0; i < 4; ++i) acc16[i] = floatx4{0.f, 0.f, 0.f, 0.f};

  const bool wave_active = (wave * TM) * 32 < npx;
  if constexpr (N16) {
    // all nine slices to LDS: [tap][C_out][CS]
#pragma unroll
    for (int i = 0; i < WALL; ++i) {
      const int p = tid + NT * i;
      if (p < 576) {
        const int tap = p >> 6, row = (p >> 2) & 15, kc = (p & 3) * 4;
        uint4 v = wall[i];
        if (!((wallmask >> i) & 1u)) v = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(&wts[(tap * 16 + row) * CS + kc]) = v;
      }
    }
    __syncthreads();                          // patch and weights are in LDS
    if (wave_active) {
      const float* pf = reinterpret_cast<const float*>(patch);
      const float* wf = reinterpret_cast<const float*>(wts);
      // NB of this wavefront's four 16-pixel blocks hold pixels of the tile (a compile-time value inside the tap
      // loop: a tile of 7 x 28 pixels leaves the last wavefront one block of four, and its three empty ones would
      // take matrix-core time from the other workgroups on the SIMD)
      auto taps = [&](auto nbc) {
        constexpr int NB = decltype(nbc)::value;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          const int toff = ((tap / 3) * PW + (tap % 3)) * CS;
          // lane (r16, kq) feeds k = 4 kq .. + 3, one value per instruction (any fixed pairing of the lanes'
          // k values is a valid order of the sum)
          const float4 bf = *reinterpret_cast<const float4*>(wf + (tap * 16 + r16) * CS + 4 * kq);
#pragma unroll
          for (int i = 0; i < NB; ++i) {
            const float4 af = *reinterpret_cast<const float4*>(pf + aoff[i] + toff + 4 * kq);
            acc16[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, bf.x, acc16[i], 0, 0, 0);
            acc16[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, bf.y, acc16[i], 0, 0, 0);
            acc16[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, bf.z, acc16[i], 0, 0, 0);
            acc16[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, bf.w, acc16[i], 0, 0, 0);
          }
        }
      };
      const int nb = (npx - wave * 64 + 15) >> 4;            // >= 1 here; uniform
      if (nb >= 4)      taps(std::integral_constant<int, 4>{});
      else if (nb == 3) taps(std::integral_constant<int, 3>{});
      else if (nb == 2) taps(std::integral_constant<int, 2>{});
      else              taps(std::integral_constant<int, 1>{});
    }
  } else {
    WT* wbuf[2] = {wts, wts + CW * CS};
    store_w(wreg[0], wmask[0], wbuf[0]);
    load_w(wreg[0], wmask[0], 2);
    __syncthreads();                            // patch and tap 0 are in LDS
    for (int tap0 = 0; tap0 < 9; tap0 += 2) {
#pragma unroll
      for (int sidx = 0; sidx < 2; ++sidx) {
        const int tap = tap0 + sidx;
        if (tap < 9) {
          // buffer sidx holds tap; register set 1-sidx holds tap+1, set sidx has tap+2 in flight
          if (tap + 1 < 9) store_w(wreg[1 - sidx], wmask[1 - sidx], wbuf[1 - sidx]);
          if (tap + 3 < 9) load_w(wreg[1 - sidx], wmask[1 - sidx], tap + 3);
          if (wave_active) {
            const int toff = ((tap / 3) * PW + (tap % 3)) * CS;
            const WT* wt = wbuf[sidx];
            auto kstep = [&](int ks) {
              const WT* ap[TM];
              const WT* bp[TN];
#pragma unroll
              for (int i = 0; i < TM; ++i) ap[i] = patch + aoff[i] + toff + ks;
#pragma unroll
              for (int j = 0; j < TN; ++j) bp[j] = wt + (j * 32 + c) * CS + ks;
              mma_step<TM, TN>(ap, bp, acc, g);
            };
            if constexpr (CFIX > 0) {
#pragma unroll
              for (int ks = 0; ks < CFIX; ks += KSTEP) kstep(ks);
            } else {
              for (int ks = 0; ks < Cp; ks += KSTEP) kstep(ks);
            }
          }
          __syncthreads();                      // tap+1 visible; everyone is done with this buffer
        }
      }
    }
  }

  const long long img_row0 = ((long long)bimg * H + y0) * Wd;   // global pixel row of tile pixel 0
  long long row0[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) row0[i] = img_row0 + (wave * TM + i) * 32;
  if constexpr (N16) {
    // 16x16 blocks: register v of a lane holds row 4 (lane / 16) + v, column lane % 16 of the block;
    // block row tm of the epilogue is the pair of blocks 2 tm, 2 tm + 1
    auto stage_block = [&](int tm, float* stage) {
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) stage[(16 * b + 4 * kq + v) * (CW + 4) + r16] = acc16[2 * tm + b][v];
    };
    epilogue_rows<TM, CW, true, NX>(a, gi, layer, stage_block, row0, img_row0 + npx, 0, L, red,
                                    reinterpret_cast<float*>(smem_raw), xreg);
  } else {
    epilogue<TM, TN, true, NX>(a, gi, layer, acc, row0, img_row0 + npx, 0, L, red, reinterpret_cast<float*>(smem_raw), xreg);
  }
}

// A kernel that uses more than 64 KB of dynamic LDS has to opt in, once per device (the attribute belongs to
// the device's copy of the kernel).  One of these per kernel instance remembers the largest size each device
// has been raised to.
struct LdsOptIn {
  size_t seen[64] = {};
  bool need(size_t smem) {
    if (smem <= 64 * 1024) return false;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return true;
    if (smem <= seen[dev]) return false;
    seen[dev] = smem;
    return true;
  }
};

// ------------------------------------------------------------------------------------------
// launch configuration
// ------------------------------------------------------------------------------------------
int conv_tile_rows(int Himg, int Wimg, int C, int dtype) {
  if (Wimg > 256 || Wimg < 1 || Himg < 1 || C < 1 || C > 64) return 0;
  int thmax = 256 / Wimg;
  if (thmax > Himg) thmax = Himg;
  const bool n16 = dtype == 0 && C <= 16;       // as conv_uses_n16
  const int kstep = n16 ? 16 : dtype == 0 ? 8 : 16, pad = dtype == 0 ? 4 : 8, es = dtype == 0 ? 4 : 2;
  const int Cp = (C + kstep - 1) / kstep * kstep, CS = Cp + pad;
  const int cw = n16 ? 16 : C <= 32 ? 32 : 64;
  const int wslices = n16 ? 9 : 2;              // weight slices resident in LDS
  while (thmax > 1 && ((size_t)(thmax + 2) * (Wimg + 2) + wslices * cw) * CS * es > 72 * 1024) --thmax;
  const int ntiles = (Himg + thmax - 1) / thmax;
  return (Himg + ntiles - 1) / ntiles;        // balanced tile height
}

static bool conv_uses_n16(const StepArgs& a, int dtype) { return dtype == 0 && a.Nf <= 16; }
static size_t conv_smem_bytes(const StepArgs& a, int dtype) {
  const bool n16 = conv_uses_n16(a, dtype);
  const int kstep = n16 ? 16 : dtype == 0 ? 8 : 16, pad = dtype == 0 ? 4 : 8, es = dtype == 0 ? 4 : 2;
  const int Cp = (a.Nf + kstep - 1) / kstep * kstep, CS = Cp + pad;
  const int cw = n16 ? 16 : a.Nf <= 32 ? 32 : 64;
  const size_t main_loop = ((size_t)(a.TH + 2) * (a.Wimg + 2) + (n16 ? 9 : 2) * cw) * CS * es;   // patch + weight slices
  const size_t staging = (size_t)4 * 32 * (cw + 4) * 4;             // epilogue staging buffer
  return main_loop > staging ? main_loop : staging;
}

// Dense tile choice: the largest tile that still gives every CU a workgroup, else the smallest.
//   0: 64x64   1: 128x128 (two workgroups per CU; a 256x256 bf16 tile with one workgroup per CU halves the
//   L2 traffic but measured 8-19 % slower at every group count, its single wavefront per SIMD cannot keep
//   enough loads in flight)
//  -1: 32x32 with the contraction split over the wavefronts (latency-bound small launches; also every long
//      contraction with at most 32 rows, which only streams its weights: a 64-row tile would be half empty)
static bool dense_skinny(const StepArgs& a) { return a.M <= 32 && a.K >= 2048; }
static int dense_tile_class(const StepArgs& a, int dtype, int groups) {
  auto wgs = [&](int t) { return (long long)((a.M + t - 1) / t) * ((a.Nf + t - 1) / t) * groups; };
  if (dense_skinny(a)) return -1;
  if (wgs(128) >= 256) return 1;
  if (wgs(64) < 256) return -1;      // fewer 64x64 tiles than CUs (measured: at 256 the tiled kernel already wins)
  return 0;
}
static int dense_tile_edge(int cls) { return cls == 1 ? 128 : cls == 0 ? 64 : 32; }

int step_grid_blocks(const StepArgs& a, int layer_kind, int dtype, int groups) {
  if (layer_kind == 1) {
    const int B = a.M / (a.Himg * a.Wimg);
    return B * ((a.Himg + a.TH - 1) / a.TH);
  }
  const int t = dense_tile_edge(dense_tile_class(a, dtype, groups));
  return ((a.M + t - 1) / t) * ((a.Nf + t - 1) / t);
}

// A failed LDS opt-in of a step kernel: the launch is skipped and launch_step returns this status.
static hipError_t g_step_attr_err = hipSuccess;
static bool step_opt_in(LdsOptIn& opt, const void* kernel, size_t smem) {
  if (!opt.need(smem)) return true;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) { g_step_attr_err = e; opt = LdsOptIn(); return false; }
  return true;
}
template <typename WT, int BM, int BN, int BK, int PF, bool WS, int WR, int WC, bool HD, bool FULL, bool XR = false, bool WN = false>
static void launch_dense_k(dim3 grid, hipStream_t s, const StepArgs& a) {
  constexpr size_t bn_rows = (size_t)BN * (BK + Op<WT>::PAD), bk_rows = (size_t)BK * (BN + (sizeof(WT) == 2 ? 16 : 4));
  constexpr size_t tiles_b = ((size_t)BM * (BK + Op<WT>::PAD) + (WN ? bk_rows : bn_rows)) * sizeof(WT);
  constexpr size_t stage_b = XR ? (size_t)BM * (BN + 4) * sizeof(float)                   // whole-tile epilogue staging
                                : (size_t)(WR * WC) * 32 * (BN / WC + 4) * sizeof(float);  // per-wavefront staging
  constexpr size_t smem = tiles_b > stage_b ? tiles_b : stage_b;
  static LdsOptIn opt;
  if (!step_opt_in(opt, reinterpret_cast<const void*>(dense_step_kernel<WT, BM, BN, WR, WC, BK, PF, WS, HD, FULL, XR, WN>), smem)) return;
  hipLaunchKernelGGL((dense_step_kernel<WT, BM, BN, WR, WC, BK, PF, WS, HD, FULL, XR, WN>), grid, dim3(64 * WR * WC), smem, s, a);
}
// Whole tiles and 32-bit byte offsets within one group's operands: the kernel's unmasked path.
template <typename WT, int BM, int BN, int BK>
static bool dense_full(const StepArgs& a) {
  const char* e = getenv("MGRIT_MASKED_STEP");
  if (e && e[0] == '1') return false;
  return a.M % BM == 0 && a.Nf % BN == 0 && a.K % BK == 0 && (long long)a.M * a.K < (1ll << 30) &&
         (long long)a.Nf * a.K * (long long)sizeof(WT) < (1ll << 32);
}
// The skip-connection operand from the registers of the k loop: square layers on the bf16 128 x 128 tile
// (MGRIT_STEP_REREAD=1 keeps the epilogue's own read of the state)
template <typename WT, int BM, int BN, int BK, int PF>
static bool dense_xr(const StepArgs& a) {
  if (!(sizeof(WT) == 2 && BM == 128 && BN == 128 && BK == 64 && PF == 1)) return false;
  const char* e = getenv("MGRIT_STEP_REREAD");
  if (e && e[0] == '1') return false;
  return a.K == a.Nf && a.mode != MODE_DACT;
}
template <typename WT, int BM, int BN, int BK, int PF, bool WS, int WR = 2, int WC = 2>
static void launch_dense_ws(dim3 grid, hipStream_t s, const StepArgs& a) {
  const bool wn = a.wn != 0;                        // adjoint steps: they all carry the act' operand (HD)
  if (dense_full<WT, BM, BN, BK>(a)) {
    if constexpr (sizeof(WT) == 2 && BM == 128 && BN == 128 && BK == 64 && PF == 1 && WR == 2 && WC == 2) {
      if (dense_xr<WT, BM, BN, BK, PF>(a)) {
        if (a.Dm && wn) launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, true, true, true, true>(grid, s, a);
        else if (a.Dm)  launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, true, true, true>(grid, s, a);
        else            launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, false, true, true>(grid, s, a);
        return;
      }
    }
    if (a.Dm && wn) launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, true, true, false, true>(grid, s, a);
    else if (a.Dm)  launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, true, true>(grid, s, a);
    else            launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, false, true>(grid, s, a);
  } else {
    if (wn) launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, true, false, false, true>(grid, s, a);
    else    launch_dense_k<WT, BM, BN, BK, PF, WS, WR, WC, true, false>(grid, s, a);
  }
}
template <typename WT, int BM, int BN, int BK, int PF, int WR = 2, int WC = 2>
static void launch_dense(dim3 grid, hipStream_t s, const StepArgs& a) {
  if (a.wstream) launch_dense_ws<WT, BM, BN, BK, PF, true, WR, WC>(grid, s, a);
  else           launch_dense_ws<WT, BM, BN, BK, PF, false, WR, WC>(grid, s, a);
}
template <typename WT, bool WS, int NW>
static void launch_ksplit_nw(dim3 grid, hipStream_t s, const StepArgs& a) {
  constexpr size_t smem = ksplit_smem<WT>(NW);
  static LdsOptIn opt, optn;
  if (a.wn) {
    if (!step_opt_in(optn, reinterpret_cast<const void*>(dense_ksplit_kernel<WT, WS, NW, true>), smem)) return;
    hipLaunchKernelGGL((dense_ksplit_kernel<WT, WS, NW, true>), grid, dim3(NW * 64), smem, s, a);
    return;
  }
  if (!step_opt_in(opt, reinterpret_cast<const void*>(dense_ksplit_kernel<WT, WS, NW>), smem)) return;
  hipLaunchKernelGGL((dense_ksplit_kernel<WT, WS, NW>), grid, dim3(NW * 64), smem, s, a);
}
template <typename WT>
static void launch_ksplit(dim3 grid, hipStream_t s, const StepArgs& a) {
  const bool wide = grid.x < 256;            // fewer workgroups than CUs: eight wavefronts split the contraction
  if (a.wstream) { if (wide) launch_ksplit_nw<WT, true, 8>(grid, s, a);  else launch_ksplit_nw<WT, true, 4>(grid, s, a); }
  else           { if (wide) launch_ksplit_nw<WT, false, 8>(grid, s, a); else launch_ksplit_nw<WT, false, 4>(grid, s, a); }
}

template <typename WT, int TN, bool N16 = false, int CFIX = 0>
static void launch_conv(dim3 grid, size_t smem, hipStream_t s, const StepArgs& a) {
  static LdsOptIn opt;
  if (!step_opt_in(opt, reinterpret_cast<const void*>(conv_step_kernel<WT, TN, N16, CFIX>), smem)) return;
  hipLaunchKernelGGL((conv_step_kernel<WT, TN, N16, CFIX>), grid, dim3(NT), smem, s, a);
}
// MGRIT_CONV_GENERIC=1 in the environment keeps 64-channel bf16 layers on the kernel with a run-time channel count
static bool conv_fixed_channels(const StepArgs& a, int dtype) {
  const char* e = getenv("MGRIT_CONV_GENERIC");
  return dtype == 1 && a.Nf == 64 && !(e && e[0] == '1');
}

hipError_t launch_step(const StepArgs& a_in, int layer_kind, int dtype, int groups, hipStream_t s) {
  if (groups <= 0) return hipSuccess;
  // k-major weights: dense adjoint steps only (square matrix, act' operand present)
  if (a_in.wn && (layer_kind != 0 || !a_in.Dm || a_in.K != a_in.Nf || a_in.mode != MODE_PHI)) return hipErrorInvalidValue;
  StepArgs a = a_in;
  a.tiles = step_grid_blocks(a, layer_kind, dtype, groups);
  const dim3 grid((unsigned)a.tiles * (unsigned)groups);
  g_step_attr_err = hipSuccess;
  trace_before(s);
  int cls;
  if (layer_kind == 1) {
    a.wmagic = ((1u << 20) + (unsigned)a.Wimg - 1u) / (unsigned)a.Wimg;
    const size_t smem = conv_smem_bytes(a, dtype);
    cls = dtype == 0 ? TRACE_CONV_F32 : TRACE_CONV_BF16;
    if (conv_uses_n16(a, dtype)) {
      launch_conv<float, 1, true>(grid, smem, s, a);
    } else if (a.Nf <= 32) {
      if (dtype == 0) launch_conv<float, 1>(grid, smem, s, a);
      else            launch_conv<__bf16, 1>(grid, smem, s, a);
    } else {
      if (dtype == 0) launch_conv<float, 2>(grid, smem, s, a);
      else if (conv_fixed_channels(a, dtype)) launch_conv<__bf16, 2, false, 64>(grid, smem, s, a);
      else            launch_conv<__bf16, 2>(grid, smem, s, a);
    }
  } else {
    const int tc = dense_tile_class(a, dtype, groups);
    if (tc == -1) {
      // the 4- and the 8-wavefront form are different kernels to a profiler: separate classes
      if (grid.x < 256) cls = dtype == 0 ? TRACE_DENSE_F32_KS8 : TRACE_DENSE_BF16_KS8;
      else              cls = dtype == 0 ? TRACE_DENSE_F32_KS : TRACE_DENSE_BF16_KS;
      if (dtype == 0) launch_ksplit<float>(grid, s, a);
      else            launch_ksplit<__bf16>(grid, s, a);
    } else if (tc == 1) {
      cls = dtype == 0 ? TRACE_DENSE_F32_128 : TRACE_DENSE_BF16_128;
      if (dtype == 0) launch_dense<float, 128, 128, 32, 2>(grid, s, a);
      else            launch_dense<__bf16, 128, 128, 64, 1>(grid, s, a);
    } else {
      cls = dtype == 0 ? TRACE_DENSE_F32_64 : TRACE_DENSE_BF16_64;
      if (dtype == 0) launch_dense<float, 64, 64, 64, 2>(grid, s, a);
      else            launch_dense<__bf16, 64, 64, 128, 2>(grid, s, a);
    }
  }
  hipError_t e = hipGetLastError();
  if (g_step_attr_err != hipSuccess) e = g_step_attr_err;
  int worked = groups;                 // groups that did a layer step (a mixed stack's convolution launch skips some)
  if (layer_kind == 1 && a.skipper > 0 && a.skip0 < groups) worked -= (groups - 1 - a.skip0) / a.skipper + 1;
  // algorithmic bytes: per layer step the layer's weights and bias once, the input state, every fused epilogue
  // operand and the act' factor once, the output once
  const double es = dtype == 0 ? 4.0 : 2.0;
  double per = (double)a.wsize * es + (a.bias ? 4.0 * a.Nf : 0.0) + 4.0 * (double)a.E;
  if (a.E1 && a.c1 != 0.0f) per += 4.0 * (double)a.E;
  if (a.E2 && a.c2 != 0.0f) per += 4.0 * (double)a.E;
  if (a.Dm) per += es * (double)a.E;
  if (a.Out) per += (a.mode == MODE_DACT ? es : 4.0) * (double)a.E;
  trace_after(s, cls, worked, per * worked);
  return e;
}

// ------------------------------------------------------------------------------------------
// Transfer kernels: one float4 per thread, grid = (chunks of a state, points)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void copy_points_kernel(float* out, PtMap om, const float* in, PtMap im,
                                                         long long E4) {
  const long long gi = blockIdx.y;
  const float4* src = reinterpret_cast<const float4*>(in) + (im.base + gi * im.stride) * E4;
  float4* dst = reinterpret_cast<float4*>(out) + (om.base + gi * om.stride) * E4;
  for (long long i = (long long)blockIdx.x * NT + threadIdx.x; i < E4; i += (long long)gridDim.x * NT) dst[i] = src[i];
}
__global__ __launch_bounds__(NT) void zero_points_kernel(float* out, PtMap om, long long E4) {
  const long long gi = blockIdx.y;
  float4* dst = reinterpret_cast<float4*>(out) + (om.base + gi * om.stride) * E4;
  for (long long i = (long long)blockIdx.x * NT + threadIdx.x; i < E4; i += (long long)gridDim.x * NT)
    dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}
__global__ __launch_bounds__(NT) void correct_kernel(float* U, PtMap um, const float* V, PtMap vm, long long E4) {
  const long long gi = blockIdx.y;
  float4* u = reinterpret_cast<float4*>(U) + (um.base + gi * um.stride) * E4;
  const float4* v = reinterpret_cast<const float4*>(V) + (vm.base + gi * vm.stride) * E4;
  for (long long i = (long long)blockIdx.x * NT + threadIdx.x; i < E4; i += (long long)gridDim.x * NT) {
    float4 x = u[i];
    const float4 y = v[i];
    x.x += y.x - x.x; x.y += y.y - x.y; x.z += y.z - x.z; x.w += y.w - x.w;
    u[i] = x;
  }
}
static dim3 xfer_grid(long long E4, int groups) {
  long long bx = (E4 + NT - 1) / NT;
  if (bx > 4096) bx = 4096;
  if (bx < 1) bx = 1;
  return dim3((unsigned)bx, (unsigned)groups);
}
hipError_t launch_copy_points(float* out, PtMap om, const float* in, PtMap im, long long E, int groups,
                              hipStream_t s) {
  if (groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(copy_points_kernel, xfer_grid(E / 4, groups), dim3(NT), 0, s, out, om, in, im, E / 4);
  return hipGetLastError();
}
hipError_t launch_zero_points(float* out, PtMap om, long long E, int groups, hipStream_t s) {
  if (groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(zero_points_kernel, xfer_grid(E / 4, groups), dim3(NT), 0, s, out, om, E / 4);
  return hipGetLastError();
}
hipError_t launch_correct(float* U, PtMap um, const float* V, PtMap vm, long long E, int groups, hipStream_t s) {
  if (groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(correct_kernel, xfer_grid(E / 4, groups), dim3(NT), 0, s, U, um, V, vm, E / 4);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Norm reduction: float partial sums per workgroup, summed in a fixed order in double.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void diff_sq_kernel(const float* a, const float* b, long long n4, float* partial) {
  __shared__ float red[4];
  const float4* x = reinterpret_cast<const float4*>(a);
  const float4* y = reinterpret_cast<const float4*>(b);
  float s = 0.0f;
  for (long long i = (long long)blockIdx.x * NT + threadIdx.x; i < n4; i += (long long)gridDim.x * NT) {
    const float4 p = x[i], q = y[i];
    const float d0 = p.x - q.x, d1 = p.y - q.y, d2 = p.z - q.z, d3 = p.w - q.w;
    s += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
  }
  s = block_sum(s, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}
int diff_sq_blocks(long long n) {
  long long b = (n / 4 + NT * 4 - 1) / (NT * 4);
  if (b > 1024) b = 1024;
  if (b < 1) b = 1;
  return (int)b;
}
hipError_t launch_diff_sq(const float* a, const float* b, long long n, float* partial, int* blocks_used,
                          hipStream_t s) {
  const int nb = diff_sq_blocks(n);
  hipLaunchKernelGGL(diff_sq_kernel, dim3(nb), dim3(NT), 0, s, a, b, n / 4, partial);
  if (blocks_used) *blocks_used = nb;
  return hipGetLastError();
}
__global__ __launch_bounds__(NT) void norm_final_kernel(const float* partial, int n, double scale, double* out) {
  __shared__ double red[NT];
  double s = 0.0;
  for (int i = threadIdx.x; i < n; i += NT) s += (double)partial[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = NT / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = sqrt(red[0]) * scale;
}
// The injection copy of the fine level and the final norm reduction of the same cycle in one launch: block
// row `groups` (one past the copies) holds the reduction, done by its first workgroup exactly as above.
__global__ __launch_bounds__(NT) void copy_points_norm_kernel(float* out, PtMap om, const float* in, PtMap im,
                                                              long long E4, int groups, const float* partial, int n,
                                                              double scale, double* nout) {
  __shared__ double red[NT];
  if ((int)blockIdx.y == groups) {
    if (blockIdx.x != 0) return;
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += NT) s += (double)partial[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = NT / 2; o > 0; o >>= 1) {
      if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
      __syncthreads();
    }
    if (threadIdx.x == 0) nout[0] = sqrt(red[0]) * scale;
    return;
  }
  const long long gi = blockIdx.y;
  const float4* src = reinterpret_cast<const float4*>(in) + (im.base + gi * im.stride) * E4;
  float4* dst = reinterpret_cast<float4*>(out) + (om.base + gi * om.stride) * E4;
  for (long long i = (long long)blockIdx.x * NT + threadIdx.x; i < E4; i += (long long)gridDim.x * NT) dst[i] = src[i];
}
hipError_t launch_copy_points_norm(float* out, PtMap om, const float* in, PtMap im, long long E, int groups,
                                   const float* partial, int n, double scale, double* nout, hipStream_t s) {
  if (groups <= 0) return launch_norm_final(partial, n, scale, nout, s);
  hipLaunchKernelGGL(copy_points_norm_kernel, xfer_grid(E / 4, groups + 1), dim3(NT), 0, s, out, om, in, im, E / 4,
                     groups, partial, n, scale, nout);
  return hipGetLastError();
}
hipError_t launch_norm_final(const float* partial, int n, double scale, double* out, hipStream_t s) {
  hipLaunchKernelGGL(norm_final_kernel, dim3(1), dim3(NT), 0, s, partial, n, scale, out);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Transposed parameter copies for the adjoint sweep
// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ __launch_bounds__(NT) void transpose_dense_kernel(const WT* W, WT* Wt, int q) {
  // 64x64 tile per workgroup; a thread moves 4 consecutive elements, so a row segment of the tile is
  // 128 (2-byte elements) or 256 contiguous bytes on both the reading and the writing side.  q % 8 == 0,
  // hence a group of 4 is inside the matrix or outside it as a whole.
  __shared__ WT tile[64][64 + 4];
  const long long layer = blockIdx.z;
  const WT* src = W + layer * (long long)q * q;
  WT* dst = Wt + layer * (long long)q * q;
  const int tx = (threadIdx.x & 15) * 4, ty = threadIdx.x >> 4;   // 16 groups of 4 across, 16 rows down
  const int x0 = blockIdx.x * 64, y0 = blockIdx.y * 64;
#pragma unroll
  for (int j = 0; j < 64; j += 16) {
    const int y = y0 + ty + j;
    if (y < q && x0 + tx < q) {
      const WT* p = src + (long long)y * q + x0 + tx;
      tile[ty + j][tx] = p[0]; tile[ty + j][tx + 1] = p[1]; tile[ty + j][tx + 2] = p[2]; tile[ty + j][tx + 3] = p[3];
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 64; j += 16) {
    const int x = x0 + ty + j;                     // row of the transposed matrix
    if (x < q && y0 + tx < q) {
      WT* p = dst + (long long)x * q + y0 + tx;
      p[0] = tile[tx][ty + j]; p[1] = tile[tx + 1][ty + j]; p[2] = tile[tx + 2][ty + j]; p[3] = tile[tx + 3][ty + j];
    }
  }
}
template <typename WT>
__global__ __launch_bounds__(NT) void transpose_conv_kernel(const WT* K, WT* Kt, int C, long long total) {
  // Kt[n][i][2-dy][2-dx][o] = K[n][o][dy][dx][i]
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int o = idx % C;
    long long t = idx / C;
    const int tapf = t % 9;
    t /= 9;
    const int i = t % C;
    const long long n = t / C;
    Kt[idx] = K[((n * C + o) * 9 + (8 - tapf)) * C + i];
  }
}
hipError_t launch_transpose_weights(const void* W, void* Wt, int layer_kind, int dtype, int layers, int Nf,
                                    hipStream_t s) {
  if (layer_kind == 0) {
    dim3 grid((Nf + 63) / 64, (Nf + 63) / 64, layers);
    if (dtype == 0) hipLaunchKernelGGL((transpose_dense_kernel<float>), grid, dim3(NT), 0, s, (const float*)W, (float*)Wt, Nf);
    else hipLaunchKernelGGL((transpose_dense_kernel<uint16_t>), grid, dim3(NT), 0, s, (const uint16_t*)W, (uint16_t*)Wt, Nf);
  } else {
    const long long total = (long long)layers * Nf * 9 * Nf;
    long long nb = (total + NT - 1) / NT;
    if (nb > 65535) nb = 65535;
    if (dtype == 0) hipLaunchKernelGGL((transpose_conv_kernel<float>), dim3((unsigned)nb), dim3(NT), 0, s, (const float*)W, (float*)Wt, Nf, total);
    else hipLaunchKernelGGL((transpose_conv_kernel<uint16_t>), dim3((unsigned)nb), dim3(NT), 0, s, (const uint16_t*)W, (uint16_t*)Wt, Nf, total);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Parameter gradient (dense): dW[n] = hs * G^T U[n], G = Dm[n] .* Lam[n+1]; contraction over
// the batch.  128x128 output tile per workgroup (2x2 wavefronts of 64x64).  Both operands are
// stored batch-row-major in memory, i.e. with the contraction index slowest, so each thread
// loads a 4 (rows) x 4 (columns) block with row-contiguous float4 loads, transposes it in
// registers and writes 4 consecutive k per column to LDS, where the usual k-fastest fragments
// are read.  The bias gradient db[n] = hs * (column sums of G) rides along: the tiles of the first tile
// column add up the unrounded G values that pass through their threads (fixed order: a thread's rows in
// sequence, then the eight threads of a column group by a butterfly).
// ------------------------------------------------------------------------------------------
template <typename OT>
__global__ __launch_bounds__(NT) void dense_grad_kernel(GradArgs a) {
  constexpr int BKR = 32, ST = BKR + Op<OT>::PAD, KSTEP = Op<OT>::KSTEP;
  constexpr int BM = 128, BN = 128, TM = 2, TN = 2;
  // operand tiles during the contraction, afterwards the staging buffer of the row-wise output stores
  constexpr int SW = 64 + 4;                          // staging row stride (floats) of a wavefront's 32 x 64 block row
  constexpr size_t TILE_B = (size_t)(BM + BN) * ST * sizeof(OT), STAGE_B = (size_t)4 * 32 * SW * sizeof(float);
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[TILE_B > STAGE_B ? TILE_B : STAGE_B];
  OT* As = reinterpret_cast<OT*>(lds_raw);
  OT* Bs = As + BM * ST;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int q = a.Nf;
  const int tiles_n = (q + BN - 1) / BN;
  const int L = logical_block();
  const int gi = L / a.tiles, tile = L % a.tiles;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const float* Up = a.U + (a.um.base + gi * a.um.stride) * a.E;
  const float* Lp = a.Lam + (a.lm.base + gi * a.lm.stride) * a.E;
  const OT* Dp = reinterpret_cast<const OT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E;
  float* dWp = a.dW ? a.dW + (long long)gi * a.wsize : nullptr;
  typedef typename DRaw<OT>::type DR;

  const int rb = tid & 7, cb = tid >> 3;             // 4 batch rows x 4 columns per thread
  const bool aok = m0 + 4 * cb < q, bok = n0 + 4 * cb < q;      // q % 4 == 0: a float4 is in or out as a whole
  float4 lv[4], uv[4];
  DR dv[4];
  unsigned rmask = 0;
  const bool bias = a.db != nullptr && n0 == 0;       // workgroup-uniform
  if (!a.dW && !bias) return;                         // bias gradient alone: the first tile column does it, the same way
  float gs[4] = {0.f, 0.f, 0.f, 0.f};                 // running column sums of G (columns m0 + 4 cb .. + 3)
  auto load_slab = [&](int r0) {
    rmask = 0;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int row = r0 + 4 * rb + rr;
      const bool rok = row < a.M;
      rmask |= rok ? (1u << rr) : 0u;
      const unsigned offa = (rok && aok) ? (unsigned)(row * q + m0 + 4 * cb) : 0u;
      const unsigned offb = (rok && bok) ? (unsigned)(row * q + n0 + 4 * cb) : 0u;
      dv[rr] = ld_d4(Dp + offa);
      lv[rr] = *reinterpret_cast<const float4*>(Lp + offa);
      uv[rr] = *reinterpret_cast<const float4*>(Up + offb);
    }
  };
  auto store_slab = [&]() {
    float gk[4][4], uk[4][4];                         // [column][k]
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const bool rok = (rmask >> rr) & 1u;
      const float ga = (rok && aok) ? 1.0f : 0.0f, ub = (rok && bok) ? 1.0f : 0.0f;
      const float4 dd = d4_to_f4(dv[rr]);
      gk[0][rr] = ga * dd.x * lv[rr].x; gk[1][rr] = ga * dd.y * lv[rr].y;
      gk[2][rr] = ga * dd.z * lv[rr].z; gk[3][rr] = ga * dd.w * lv[rr].w;
      uk[0][rr] = ub * uv[rr].x; uk[1][rr] = ub * uv[rr].y; uk[2][rr] = ub * uv[rr].z; uk[3][rr] = ub * uv[rr].w;
    }
    if (bias) {
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) gs[cc] += (gk[cc][0] + gk[cc][1]) + (gk[cc][2] + gk[cc][3]);
    }
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      cvt_store4(&As[(4 * cb + cc) * ST + 4 * rb], make_float4(gk[cc][0], gk[cc][1], gk[cc][2], gk[cc][3]));
      cvt_store4(&Bs[(4 * cb + cc) * ST + 4 * rb], make_float4(uk[cc][0], uk[cc][1], uk[cc][2], uk[cc][3]));
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = zero16();
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;
  load_slab(0);
  for (int r0 = 0; r0 < a.M; r0 += BKR) {
    __syncthreads();
    store_slab();
    __syncthreads();
    if (r0 + BKR < a.M) load_slab(r0 + BKR);
#pragma unroll
    for (int ks = 0; ks < BKR; ks += KSTEP) {
      const OT* ap[TM];
      const OT* bp[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) ap[i] = &As[(wm0 + i * 32 + c) * ST + ks];
#pragma unroll
      for (int j = 0; j < TN; ++j) bp[j] = &Bs[(wn0 + j * 32 + c) * ST + ks];
      mma_step<TM, TN>(ap, bp, acc, g);
    }
  }
  if (bias) {                                         // the eight threads rb = 0..7 of a column group are neighbouring lanes
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      gs[cc] += __shfl_xor(gs[cc], 1);
      gs[cc] += __shfl_xor(gs[cc], 2);
      gs[cc] += __shfl_xor(gs[cc], 4);
    }
    if (rb == 0 && aok)
      *reinterpret_cast<float4*>(a.db + (long long)gi * q + m0 + 4 * cb) =
          make_float4(a.hs * gs[0], a.hs * gs[1], a.hs * gs[2], a.hs * gs[3]);
  }
  // output through LDS so that a lane stores a float4 and 16 lanes a whole 256-byte row segment
  __syncthreads();
  float* stage = reinterpret_cast<float*>(lds_raw) + wave * 32 * SW;
  const int lrow = lane >> 4, colq = (lane & 15) * 4;
  const int col = n0 + wn0 + colq;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * g + (r & 3)) * SW + j * 32 + c] = acc[i][j][r];
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      const int rl = 4 * h + lrow;
      const int row = m0 + wm0 + i * 32 + rl;
      float4 z = *reinterpret_cast<const float4*>(&stage[rl * SW + colq]);
      z.x *= a.hs; z.y *= a.hs; z.z *= a.hs; z.w *= a.hs;
      if (a.dW && row < q && col < q) *reinterpret_cast<float4*>(dWp + (long long)row * q + col) = z;
    }
  }
}
// The same contraction on a 256x256 output tile for wide layers (q >= 512): eight wavefronts, 2 (rows of dW) x 4
// (columns), each owning 128 x 64.  A 128x128 tile re-reads every operand panel q / 128 times from L2 -- 20 MB per
// layer at q = 1024, five times the 4 MB of dW that go out -- and that traffic, not HBM, set its time; the wide tile
// halves it.  The bias gradient db[o] = hs * sum over the batch of G[.][o] rides along: the column tiles with
// n0 == 0 sum the float G values they stage anyway (per thread over its rows, then over the eight row lanes in a
// fixed order), which spares the separate pass over Dm and Lam.
template <typename OT>
__global__ __launch_bounds__(512) void dense_grad_wide_kernel(GradArgs a) {
  constexpr int BKR = 32, ST = BKR + Op<OT>::PAD, KSTEP = Op<OT>::KSTEP;
  constexpr int BM = 256, BN = 256, TM = 4, TN = 2, NTH = 512;
  constexpr int SW = 64 + 4;                          // staging row stride (floats) of a wavefront's 32 x 64 block row
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];   // operand tiles, later the output staging
  OT* As = reinterpret_cast<OT*>(lds_raw);            // [BM][ST]  G^T: row = output feature o, k = batch row
  OT* Bs = As + BM * ST;                              // [BN][ST]  U^T: row = input feature i
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int q = a.Nf;
  const int tiles_n = (q + BN - 1) / BN;
  const int L = logical_block();
  const int gi = L / a.tiles, tile = L % a.tiles;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
  const float* Up = a.U + (a.um.base + gi * a.um.stride) * a.E;
  const float* Lp = a.Lam + (a.lm.base + gi * a.lm.stride) * a.E;
  const OT* Dp = reinterpret_cast<const OT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E;
  float* dWp = a.dW ? a.dW + (long long)gi * a.wsize : nullptr;
  typedef typename DRaw<OT>::type DR;
  const bool want_db = a.db != nullptr && n0 == 0;

  const int rb = tid & 7, cb = tid >> 3;             // 4 batch rows x 4 columns per thread, of G and of U
  const bool aok = m0 + 4 * cb < q, bok = n0 + 4 * cb < q;      // q % 4 == 0: a float4 is in or out as a whole
  float4 lv[4], uv[4];
  DR dv[4];
  unsigned rmask = 0;
  float bsum[4] = {0.f, 0.f, 0.f, 0.f};
  auto load_slab = [&](int r0) {
    rmask = 0;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int row = r0 + 4 * rb + rr;
      const bool rok = row < a.M;
      rmask |= rok ? (1u << rr) : 0u;
      const unsigned offa = (rok && aok) ? (unsigned)(row * q + m0 + 4 * cb) : 0u;
      const unsigned offb = (rok && bok) ? (unsigned)(row * q + n0 + 4 * cb) : 0u;
      dv[rr] = ld_d4(Dp + offa);
      lv[rr] = *reinterpret_cast<const float4*>(Lp + offa);
      uv[rr] = *reinterpret_cast<const float4*>(Up + offb);
    }
  };
  auto store_slab = [&]() {
    float gk[4][4], uk[4][4];                         // [column][k]
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const bool rok = (rmask >> rr) & 1u;
      const float ga = (rok && aok) ? 1.0f : 0.0f, ub = (rok && bok) ? 1.0f : 0.0f;
      const float4 dd = d4_to_f4(dv[rr]);
      gk[0][rr] = ga * dd.x * lv[rr].x; gk[1][rr] = ga * dd.y * lv[rr].y;
      gk[2][rr] = ga * dd.z * lv[rr].z; gk[3][rr] = ga * dd.w * lv[rr].w;
      uk[0][rr] = ub * uv[rr].x; uk[1][rr] = ub * uv[rr].y; uk[2][rr] = ub * uv[rr].z; uk[3][rr] = ub * uv[rr].w;
    }
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      bsum[cc] += (gk[cc][0] + gk[cc][1]) + (gk[cc][2] + gk[cc][3]);
      cvt_store4(&As[(4 * cb + cc) * ST + 4 * rb], make_float4(gk[cc][0], gk[cc][1], gk[cc][2], gk[cc][3]));
      cvt_store4(&Bs[(4 * cb + cc) * ST + 4 * rb], make_float4(uk[cc][0], uk[cc][1], uk[cc][2], uk[cc][3]));
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = zero16();
  const int wm0 = (wave >> 2) * 128, wn0 = (wave & 3) * 64;
  load_slab(0);
  for (int r0 = 0; r0 < a.M; r0 += BKR) {
    __syncthreads();
    store_slab();
    __syncthreads();
    if (r0 + BKR < a.M) load_slab(r0 + BKR);
#pragma unroll
    for (int ks = 0; ks < BKR; ks += KSTEP) {
      const OT* ap[TM];
      const OT* bp[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) ap[i] = &As[(wm0 + i * 32 + c) * ST + ks];
#pragma unroll
      for (int j = 0; j < TN; ++j) bp[j] = &Bs[(wn0 + j * 32 + c) * ST + ks];
      mma_step<TM, TN>(ap, bp, acc, g);
    }
  }
  __syncthreads();                                    // every wavefront is done with the operand tiles
  if (want_db) {
    // the eight row lanes rb of a column block hold partial sums over disjoint batch rows: add them in lane order
    float4* part = reinterpret_cast<float4*>(lds_raw);          // [64 column blocks][8 row lanes]
    part[cb * 8 + rb] = make_float4(bsum[0], bsum[1], bsum[2], bsum[3]);
    __syncthreads();
    if (rb == 0 && aok) {
      float4 t = part[cb * 8];
#pragma unroll
      for (int j = 1; j < 8; ++j) { const float4 v = part[cb * 8 + j]; t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w; }
      t.x *= a.hs; t.y *= a.hs; t.z *= a.hs; t.w *= a.hs;
      *reinterpret_cast<float4*>(a.db + (long long)gi * q + m0 + 4 * cb) = t;
    }
    __syncthreads();
  }
  if (!dWp) return;
  // output through LDS so that a lane stores a float4 and 16 lanes a whole 256-byte row segment
  float* stage = reinterpret_cast<float*>(lds_raw) + wave * 32 * SW;
  const int lrow = lane >> 4, colq = (lane & 15) * 4;
  const int col = n0 + wn0 + colq;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * g + (r & 3)) * SW + j * 32 + c] = acc[i][j][r];
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      const int rl = 4 * h + lrow;
      const int row = m0 + wm0 + i * 32 + rl;
      float4 z = *reinterpret_cast<const float4*>(&stage[rl * SW + colq]);
      z.x *= a.hs; z.y *= a.hs; z.z *= a.hs; z.w *= a.hs;
      if (row < q && col < q) *reinterpret_cast<float4*>(dWp + (long long)row * q + col) = z;
    }
  }
}
template <typename OT> constexpr size_t dense_grad_wide_smem() {
  constexpr size_t tiles = (size_t)512 * (32 + Op<OT>::PAD) * sizeof(OT), stage = (size_t)8 * 32 * 68 * sizeof(float);
  return tiles > stage ? tiles : stage;
}
template <typename OT>
static hipError_t launch_dense_grad_wide(const GradArgs& a, unsigned blocks, hipStream_t s) {
  constexpr size_t smem = dense_grad_wide_smem<OT>();
  static LdsOptIn opt;
  if (opt.need(smem)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(dense_grad_wide_kernel<OT>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((dense_grad_wide_kernel<OT>), dim3(blocks), dim3(512), smem, s, a);
  return hipGetLastError();
}

// Parameter gradient (3x3 conv): dK[n][o][dy][dx][i] = hs * sum over pixels of G[b,y,x,o] *
// U[b,y+dy-1,x+dx-1,i] (zero outside the image), G = Dm .* Lam.  One workgroup per (layer, tap):
// a C x C output tile (C <= 64), contraction over all B*H*W pixels in slabs of 32, operands
// transposed in registers as in the dense kernel.  Every tap re-reads the whole layer, so this form is
// kept only for image rows too wide for the all-taps kernel below.
template <typename OT>
__global__ __launch_bounds__(NT) void conv_grad_tap_kernel(GradArgs a) {
  constexpr int BKR = 32, ST = BKR + Op<OT>::PAD, KSTEP = Op<OT>::KSTEP;
  __shared__ __attribute__((aligned(16))) OT As[64 * ST];
  __shared__ __attribute__((aligned(16))) OT Bs[64 * ST];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int C = a.Nf, H = a.Himg, Wd = a.Wimg;
  const int L = logical_block();
  const int gi = L / 9, tap = L % 9;
  const int dy = tap / 3 - 1, dx = tap % 3 - 1;
  const float* Up = a.U + (a.um.base + gi * a.um.stride) * a.E;
  const float* Lp = a.Lam + (a.lm.base + gi * a.lm.stride) * a.E;
  const OT* Dp = reinterpret_cast<const OT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E;
  float* dKp = a.dW + (long long)gi * a.wsize;
  typedef typename DRaw<OT>::type DR;

  const int rb = tid & 7, cb = (tid >> 3) & 15;      // 4 pixels x 4 channels per thread; threads 128.. idle
  const bool cok = tid < 128 && 4 * cb < C;
  float4 lv[4], uv[4];
  DR dv[4];
  unsigned gmask = 0, umask = 0;
  auto load_slab = [&](int r0) {
    gmask = 0; umask = 0;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const int px = r0 + 4 * rb + rr;
      const bool pok = cok && px < a.M;
      const int x = px % Wd, y = (px / Wd) % H;
      const bool sok = pok && y + dy >= 0 && y + dy < H && x + dx >= 0 && x + dx < Wd;
      gmask |= pok ? (1u << rr) : 0u;
      umask |= sok ? (1u << rr) : 0u;
      const unsigned og = pok ? (unsigned)(px * C + 4 * cb) : 0u;
      const unsigned ou = sok ? (unsigned)((px + dy * Wd + dx) * C + 4 * cb) : 0u;
      dv[rr] = ld_d4(Dp + og);
      lv[rr] = *reinterpret_cast<const float4*>(Lp + og);
      uv[rr] = *reinterpret_cast<const float4*>(Up + ou);
    }
  };
  auto store_slab = [&]() {
    if (tid >= 128) return;
    float gk[4][4], uk[4][4];
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
      const float ga = ((gmask >> rr) & 1u) ? 1.0f : 0.0f, ub = ((umask >> rr) & 1u) ? 1.0f : 0.0f;
      const float4 dd = d4_to_f4(dv[rr]);
      gk[0][rr] = ga * dd.x * lv[rr].x; gk[1][rr] = ga * dd.y * lv[rr].y;
      gk[2][rr] = ga * dd.z * lv[rr].z; gk[3][rr] = ga * dd.w * lv[rr].w;
      uk[0][rr] = ub * uv[rr].x; uk[1][rr] = ub * uv[rr].y; uk[2][rr] = ub * uv[rr].z; uk[3][rr] = ub * uv[rr].w;
    }
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      cvt_store4(&As[(4 * cb + cc) * ST + 4 * rb], make_float4(gk[cc][0], gk[cc][1], gk[cc][2], gk[cc][3]));
      cvt_store4(&Bs[(4 * cb + cc) * ST + 4 * rb], make_float4(uk[cc][0], uk[cc][1], uk[cc][2], uk[cc][3]));
    }
  };

  floatx16 acc[1][1];
  acc[0][0] = zero16();
  const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
  load_slab(0);
  for (int r0 = 0; r0 < a.M; r0 += BKR) {
    __syncthreads();
    store_slab();
    __syncthreads();
    if (r0 + BKR < a.M) load_slab(r0 + BKR);
#pragma unroll
    for (int ks = 0; ks < BKR; ks += KSTEP) {
      const OT* ap[1] = {&As[(wm0 + c) * ST + ks]};
      const OT* bp[1] = {&Bs[(wn0 + c) * ST + ks]};
      mma_step<1, 1>(ap, bp, acc, g);
    }
  }
  const int ci = wn0 + c;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int co = wm0 + 8 * (r >> 2) + 4 * g + (r & 3);
    if (co < C && ci < C) dKp[((long long)co * 9 + tap) * C + ci] = a.hs * acc[0][0][r];
  }
}

// Parameter gradient (3x3 conv), all nine taps in one workgroup.  Written as one product per layer,
//   dK[o][n] = sum over pixels p of G[p][o] * S[p][n],   n = tap * C + i,   S[p][tap*C+i] = U[p + tap][i],
// which is exactly the row-major [C][9C] layout of dK[o][dy][dx][i].  A workgroup walks over slabs of gR
// image rows of one image.  Per slab the 4 (pixels) x 4 (channels) register transposes of the dense
// gradient kernel put G as [o][pixel] and U as [i][patch pixel] into LDS, the latter three times, shifted
// by dx = -1, 0, +1, so that every 16-byte fragment read of a tap is aligned; dy is a whole-row offset.
// A lane's B-operand row is fixed by its column n (tap and input channel), so the k loop is a plain
// GEMM loop over the slab's pixel slots.  The wavefront w owns the 32-column blocks w, w+4, w+8, ...
// LDS is cleared once; slots that are never written (row padding, the column left of x = 0 in the
// dx = -1 copy, ...) stay zero, rows outside the image are written as zeros every slab.
// With few layers the slabs of a layer are split over `gchunks` workgroups that write partial sums.
// N16 (float, at most 16 channels): 16x16x4 blocks, so the output-channel side carries no padding rows (a 32-row
// block would be half empty at 16 channels, and this kernel is bound by the matrix cores); wavefront w then owns the
// 16-column blocks w, w+4, ..
// NWV wavefronts: 4, or 8 for more than 32 channels -- there the accumulators of four wavefronts (2 x 5 blocks
// each) leave room for one workgroup per CU anyway, and with eight the transposing stores of a slab, which
// take longer than its matrix instructions, are spread over twice the threads.
template <typename OT, int TM, int TN, bool N16 = false, int NWV = 4>
__global__ __launch_bounds__(64 * NWV) void conv_grad_kernel(GradArgs a) {
  constexpr int NTH = 64 * NWV;
  constexpr int UB = NWV == 8 ? 2 : 3;                  // 4x4 blocks of the U patch per thread, at most
  static_assert(!N16 || (sizeof(OT) == 4 && TM == 1), "the 16-wide variant is float only");
  constexpr int KSTEP = N16 ? 16 : Op<OT>::KSTEP;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int C = a.Nf, H = a.Himg, Wd = a.Wimg;
  const int Wp = a.gWp, R = a.gR, PU = a.gPU, PG = a.gPG, KL = a.gKL;
  OT* Ut = reinterpret_cast<OT*>(smem_raw);             // [3][C][PU]
  OT* Gt = Ut + 3 * C * PU;                             // [C][PG]
  OT* ones = Gt + C * PG;                               // [PU] of 1: the operand row of column 9C, the bias gradient
  const int L = logical_block();
  const int gi = L / a.gchunks, ch = L % a.gchunks;
  const float* Up = a.U + (a.um.base + gi * a.um.stride) * a.E;
  const float* Lp = a.Lam + (a.lm.base + gi * a.lm.stride) * a.E;
  const OT* Dp = reinterpret_cast<const OT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E;
  typedef typename DRaw<OT>::type DR;

  {
    const int n16 = (int)(((size_t)3 * C * PU + (size_t)C * PG) * sizeof(OT) / 16);
    for (int p = tid; p < n16; p += NTH) reinterpret_cast<uint4*>(smem_raw)[p] = make_uint4(0u, 0u, 0u, 0u);
    for (int p = tid; p < PU; p += NTH) ones[p] = static_cast<OT>(1.0f);
  }

  // this thread's 4x4 blocks: one of G, up to UB of the U patch (x group fastest, then channel group, then row)
  const int CG = C >> 2, XG = (Wd + 3) >> 2;
  const int nGb = R * XG * CG, nUb = (R + 2) * XG * CG;
  const bool gact = tid < nGb;
  const int gb = gact ? tid : 0;
  // (x group fastest: the lanes of a store instruction then spread over the pixel slots of a channel row, 8 bytes
  // apart, instead of over channel rows, whose pitch maps every second one to the same LDS banks)
  const int g_xg = gb % XG, g_cg = (gb / XG) % CG, g_r = gb / (CG * XG);
  bool uact[UB];
  int u_cg[UB], u_xg[UB], u_r[UB];
#pragma unroll
  for (int t = 0; t < UB; ++t) {
    const int blk = tid + NTH * t;
    uact[t] = blk < nUb;
    const int ub = uact[t] ? blk : 0;
    u_xg[t] = ub % XG; u_cg[t] = (ub / XG) % CG; u_r[t] = ub / (CG * XG);
  }
  const bool lane_shift = (64 % XG) == 0;              // uniform; else the shifted copies are stored element by element
  float4 lv[4], uv[UB][4];
  DR dv[4];
  unsigned gmask = 0, umask[UB] = {};
  auto load_slab = [&](int sl) {
    const int b = sl / a.gspi, y0 = (sl % a.gspi) * R;
    {
      const int y = y0 + g_r;
      const bool rok = gact && y < H;
      gmask = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int x = 4 * g_xg + j;
        const bool ok = rok && x < Wd;
        gmask |= ok ? (1u << j) : 0u;
        const unsigned off = ok ? (unsigned)((((long long)b * H + y) * Wd + x) * C + 4 * g_cg) : 0u;
        dv[j] = ld_d4(Dp + off);
        lv[j] = *reinterpret_cast<const float4*>(Lp + off);
      }
    }
#pragma unroll
    for (int t = 0; t < UB; ++t) {
      if (NTH * t >= nUb) break;                        // uniform
      const int y = y0 - 1 + u_r[t];
      const bool rok = uact[t] && y >= 0 && y < H;
      umask[t] = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int x = 4 * u_xg[t] + j;
        const bool ok = rok && x < Wd;
        umask[t] |= ok ? (1u << j) : 0u;
        const unsigned off = ok ? (unsigned)((((long long)b * H + y) * Wd + x) * C + 4 * u_cg[t]) : 0u;
        uv[t][j] = *reinterpret_cast<const float4*>(Up + off);
      }
    }
  };
  auto store_slab = [&]() {
    if (gact) {
      float gk[4][4];                                   // [channel][pixel]
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = (gmask >> j) & 1u;
        const float4 dd = d4_to_f4(dv[j]);
        gk[0][j] = ok ? dd.x * lv[j].x : 0.0f; gk[1][j] = ok ? dd.y * lv[j].y : 0.0f;
        gk[2][j] = ok ? dd.z * lv[j].z : 0.0f; gk[3][j] = ok ? dd.w * lv[j].w : 0.0f;
      }
#pragma unroll
      for (int cc = 0; cc < 4; ++cc)
        cvt_store4(&Gt[(4 * g_cg + cc) * PG + g_r * Wp + 4 * g_xg], make_float4(gk[cc][0], gk[cc][1], gk[cc][2], gk[cc][3]));
    }
#pragma unroll
    for (int t = 0; t < UB; ++t) {
      if (NTH * t >= nUb) break;                        // uniform
      float uk[4][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = uact[t] && ((umask[t] >> j) & 1u);
        uk[0][j] = ok ? uv[t][j].x : 0.0f; uk[1][j] = ok ? uv[t][j].y : 0.0f;
        uk[2][j] = ok ? uv[t][j].z : 0.0f; uk[3][j] = ok ? uv[t][j].w : 0.0f;
      }
      const int col = 4 * u_xg[t];
      if (lane_shift) {
        // The x groups of an image row sit in consecutive lanes of one wavefront (XG divides 64): the pixel left of
        // this thread's four comes from lane - 1 and the one right of them from lane + 1 (zero at the row's ends),
        // so each of the three copies is one aligned 8- or 16-byte store per channel instead of four 2- or 4-byte ones.
        // Every lane takes part in the exchange; only threads that own a block store.
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
          float left = __shfl_up(uk[cc][3], 1), right = __shfl_down(uk[cc][0], 1);
          if (u_xg[t] == 0) left = 0.0f;
          if (u_xg[t] == XG - 1) right = 0.0f;
          if (uact[t]) {
            const int i = 4 * u_cg[t] + cc;
            cvt_store4(Ut + (0 * C + i) * PU + u_r[t] * Wp + col, make_float4(left, uk[cc][0], uk[cc][1], uk[cc][2]));
            cvt_store4(Ut + (1 * C + i) * PU + u_r[t] * Wp + col, make_float4(uk[cc][0], uk[cc][1], uk[cc][2], uk[cc][3]));
            cvt_store4(Ut + (2 * C + i) * PU + u_r[t] * Wp + col, make_float4(uk[cc][1], uk[cc][2], uk[cc][3], right));
          }
        }
        continue;
      }
      if (!uact[t]) continue;
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int i = 4 * u_cg[t] + cc;
        OT* rowm = Ut + (0 * C + i) * PU + u_r[t] * Wp;   // dx = -1: slot xx holds U[x = xx - 1]
        OT* row0 = Ut + (1 * C + i) * PU + u_r[t] * Wp;   // dx =  0
        OT* rowp = Ut + (2 * C + i) * PU + u_r[t] * Wp;   // dx = +1: slot xx holds U[x = xx + 1]
        cvt_store4(row0 + col, make_float4(uk[cc][0], uk[cc][1], uk[cc][2], uk[cc][3]));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (col + j + 1 < Wp) rowm[col + j + 1] = static_cast<OT>(uk[cc][j]);
          if (col + j - 1 >= 0) rowp[col + j - 1] = static_cast<OT>(uk[cc][j]);
        }
      }
    }
  };

  // this lane's operand rows: output channel o for A, column n = tap * C + i for B; column 9C multiplies G by
  // ones, which sums it over the pixels (the bias gradient).  Clamped: blocks past the end compute values
  // that are never stored.
  constexpr int BW = N16 ? 16 : 32;                     // block width: rows of A and columns of B per block
  const int bl = N16 ? (lane & 15) : c;                 // this lane's row / column inside a block
  const int kq = lane >> 4;                             // 16-wide blocks: the lane's quarter of a k step
  const OT* arow[TM];
  const OT* brow[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) arow[i] = Gt + min(BW * i + bl, C - 1) * PG;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = min(BW * (wave + NWV * j) + bl, 9 * C);
    const int tap = n / C, ii = n % C;
    brow[j] = n == 9 * C ? ones : Ut + ((tap % 3) * C + ii) * PU + (tap / 3) * Wp;
  }
  floatx16 acc[TM][TN];
  floatx4 acc16[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = zero16();
#pragma unroll
  for (int j = 0; j < TN; ++j) acc16[j] = floatx4{0.f, 0.f, 0.f, 0.f};

  const int s_begin = ch * a.gspc, s_end = min(s_begin + a.gspc, a.gslabs);
  if (s_begin < s_end) load_slab(s_begin);
  for (int sl = s_begin; sl < s_end; ++sl) {
    __syncthreads();
    store_slab();
    __syncthreads();
    if (sl + 1 < s_end) load_slab(sl + 1);
    for (int ks = 0; ks < KL; ks += KSTEP) {
      if constexpr (N16) {
        // lane (bl, kq) feeds k = ks + 4 kq .. + 3, one value per instruction
        const float4 af = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(arow[0]) + ks + 4 * kq);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const float4 bf = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(brow[j]) + ks + 4 * kq);
          acc16[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, bf.x, acc16[j], 0, 0, 0);
          acc16[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, bf.y, acc16[j], 0, 0, 0);
          acc16[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, bf.z, acc16[j], 0, 0, 0);
          acc16[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, bf.w, acc16[j], 0, 0, 0);
        }
      } else {
        const OT* ap[TM];
        const OT* bp[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) ap[i] = arow[i] + ks;
#pragma unroll
        for (int j = 0; j < TN; ++j) bp[j] = brow[j] + ks;
        mma_step<TM, TN>(ap, bp, acc, g);
      }
    }
  }
  const bool direct = a.gchunks == 1;
  const int NC = 9 * C;
  const long long pstride = a.wsize + C;                // a partial-sum record: dK of the layer, then db
  float* dKd = direct ? (a.dW ? a.dW + (long long)gi * a.wsize : nullptr)
                      : a.partial + ((long long)ch * a.layers + gi) * pstride;
  float* dbd = direct ? (a.db ? a.db + (long long)gi * C : nullptr)
                      : a.partial + ((long long)ch * a.layers + gi) * pstride + a.wsize;
  const float scale = direct ? a.hs : 1.0f;
  if constexpr (N16) {
    // register v of lane (bl, kq) holds row o = 4 kq + v, column n = 16 (wave + 4 j) + bl of the block
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = 16 * (wave + NWV * j) + bl;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int o = 4 * kq + v;
        if (o < C) {
          if (n < NC) { if (dKd) dKd[(long long)o * NC + n] = scale * acc16[j][v]; }
          else if (n == NC) { if (dbd) dbd[o] = scale * acc16[j][v]; }
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = 32 * (wave + NWV * j) + c;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int o = 32 * i + 8 * (r >> 2) + 4 * g + (r & 3);
          if (o < C) {
            if (n < NC) { if (dKd) dKd[(long long)o * NC + n] = scale * acc[i][j][r]; }
            else if (n == NC) { if (dbd) dbd[o] = scale * acc[i][j][r]; }
          }
        }
      }
  }
}
// dK and db = hs * (sum of the chunk partial sums, in chunk order).  A record holds wsize values of dK and C of db.
__global__ __launch_bounds__(NT) void conv_grad_reduce_kernel(const float* partial, float* dW, float* db, int layers,
                                                              long long wsize, int C, int chunks, float hs) {
  const long long rec4 = (wsize + C) / 4, total4 = rec4 * layers;
  const float4* src = reinterpret_cast<const float4*>(partial);
  for (long long i = (long long)blockIdx.x * NT + threadIdx.x; i < total4; i += (long long)gridDim.x * NT) {
    float4 s = src[i];
    for (int k = 1; k < chunks; ++k) {
      const float4 v = src[(long long)k * total4 + i];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    const float4 o = make_float4(hs * s.x, hs * s.y, hs * s.z, hs * s.w);
    const long long layer = i / rec4, e = (i % rec4) * 4;
    if (e < wsize) { if (dW) *reinterpret_cast<float4*>(dW + layer * wsize + e) = o; }
    else if (db) *reinterpret_cast<float4*>(db + layer * C + (e - wsize)) = o;
  }
}

// db[n][o] = hs * sum over rows of Dm .* Lam (fixed order).  64 columns per workgroup: 16 lanes of
// float4 across, 16 row lanes down, then a fixed-order LDS reduction over the row lanes.
template <typename OT>
__global__ __launch_bounds__(NT) void bias_grad_kernel(GradArgs a) {
  __shared__ float4 part[16][17];
  const int gi = blockIdx.y;
  const float* Lp = a.Lam + (a.lm.base + gi * a.lm.stride) * a.E;
  const OT* Dp = reinterpret_cast<const OT*>(a.Dm) + (a.dm.base + gi * a.dm.stride) * a.E;
  const int cx = threadIdx.x & 15, ry = threadIdx.x >> 4;
  const int col = blockIdx.x * 64 + 4 * cx;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (col < a.Nf) {
    for (int r = ry; r < a.M; r += 16) {
      const unsigned off = (unsigned)(r * a.Nf + col);
      const float4 d = d4_to_f4(ld_d4(Dp + off)), l = *reinterpret_cast<const float4*>(Lp + off);
      s.x += d.x * l.x; s.y += d.y * l.y; s.z += d.z * l.z; s.w += d.w * l.w;
    }
  }
  part[ry][cx] = s;
  __syncthreads();
  if (ry == 0 && col < a.Nf) {
    float4 t = part[0][cx];
    for (int j = 1; j < 16; ++j) { t.x += part[j][cx].x; t.y += part[j][cx].y; t.z += part[j][cx].z; t.w += part[j][cx].w; }
    t.x *= a.hs; t.y *= a.hs; t.z *= a.hs; t.w *= a.hs;
    *reinterpret_cast<float4*>(a.db + (long long)gi * a.Nf + col) = t;
  }
}

// wavefronts of the all-taps gradient kernel: eight for more than 32 channels (MGRIT_CGRAD_WAVES=4: always four)
int conv_grad_waves(int C) {
  const char* e = getenv("MGRIT_CGRAD_WAVES");
  if (e && e[0] == '4') return 4;
  return C > 32 ? 8 : 4;
}
ConvGradGeom conv_grad_geom(int B, int Himg, int Wimg, int C, int dtype, int layers) {
  ConvGradGeom gm = {};
  const int nth = 64 * conv_grad_waves(C);
  const int es = dtype == 0 ? 4 : 2, pad = dtype == 0 ? Op<float>::PAD : Op<__bf16>::PAD;
  const int kstep = (dtype == 0 && C <= 16) ? 16 : dtype == 0 ? Op<float>::KSTEP : Op<__bf16>::KSTEP;   // as conv_grad_n16
  gm.Wp = (Wimg + 7) & ~7;
  // Image rows per slab.  A thread transposes at most one 4x4 block of G and three of the U patch per slab, so
  // R * blocks_per_row <= 256 and (R + 2) * blocks_per_row <= 768; 64 / Wp rows always satisfy that (64 channels,
  // 32 columns: 2 rows).  With fewer channels more rows fit, and a slab is worth a fixed two barriers and one
  // memory latency whatever its size: take as many as keep the workgroup under 72 KB of LDS (two per CU).
  const int bpr = ((Wimg + 3) / 4) * ((C + 3) / 4);    // 4x4 blocks per image row
  auto smem_of = [&](int R) {
    const int KL = (R * gm.Wp + kstep - 1) / kstep * kstep, PU = (R + 2) * gm.Wp + pad, PG = KL + pad;
    return ((size_t)3 * C * PU + (size_t)C * PG + PU) * es;             // U copies, G, the row of ones
  };
  int Rmin = 64 / gm.Wp;
  if (Rmin < 1) Rmin = 1;
  int R = nth / (bpr > 0 ? bpr : 1);
  if (R < Rmin) R = Rmin;
  const size_t lds_cap = (size_t)(nth == 256 ? 72 : 150) * 1024;   // two workgroups per CU, or one of eight wavefronts
  while (R > Rmin && ((R + 2) * bpr > (nth == 256 ? 3 : 2) * nth || smem_of(R) > lds_cap)) --R;
  if (R > Himg) R = Himg;
  R = (Himg + (Himg + R - 1) / R - 1) / ((Himg + R - 1) / R);         // the same number of slabs, of balanced height
  gm.R = R;
  const int KP = gm.R * gm.Wp;
  gm.KL = (KP + kstep - 1) / kstep * kstep;
  gm.PU = (gm.R + 2) * gm.Wp + pad;                     // reads reach slot 2*Wp + KL - 1 <= (R+2)*Wp + pad - 1
  gm.PG = gm.KL + pad;
  gm.spi = (Himg + gm.R - 1) / gm.R;
  gm.slabs = B * gm.spi;
  gm.smem = smem_of(gm.R);
  gm.ok = Wimg <= 64 && gm.smem <= (size_t)150 * 1024;
  int ch = (512 + layers - 1) / (layers > 0 ? layers : 1);  // aim at two workgroups per compute unit
  if (ch > 64) ch = 64;
  if (ch > gm.slabs) ch = gm.slabs;
  if (ch < 1) ch = 1;
  gm.spc = (gm.slabs + ch - 1) / ch;
  gm.chunks = (gm.slabs + gm.spc - 1) / gm.spc;
  return gm;
}
size_t conv_grad_partial_bytes(int B, int Himg, int Wimg, int C, int dtype, int layers) {
  const ConvGradGeom gm = conv_grad_geom(B, Himg, Wimg, C, dtype, layers);
  if (!gm.ok || gm.chunks <= 1) return 0;
  return (size_t)gm.chunks * layers * (9 * C * C + C) * sizeof(float);
}
static void launch_bias_grad(const GradArgs& a, int dtype, int groups, hipStream_t s) {
  const dim3 grid((a.Nf + 63) / 64, groups);
  if (dtype == 0) hipLaunchKernelGGL((bias_grad_kernel<float>), grid, dim3(NT), 0, s, a);
  else            hipLaunchKernelGGL((bias_grad_kernel<__bf16>), grid, dim3(NT), 0, s, a);
}
template <typename OT, int TM, int TN, bool N16 = false, int NWV = 4>
static hipError_t launch_conv_grad(const GradArgs& a, unsigned blocks, size_t smem, hipStream_t s) {
  if (smem > 64 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(conv_grad_kernel<OT, TM, TN, N16, NWV>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((conv_grad_kernel<OT, TM, TN, N16, NWV>), dim3(blocks), dim3(64 * NWV), smem, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Fused F-relaxation sweep for dense layers.  A workgroup owns 32 batch rows of one coarse interval
// and marches through all steps of the sweep: the fp32 state slice S and its matrix-core operand
// copy A (Dm .* S in the operand type) stay in LDS, the weights of each layer stream through two LDS
// slabs of BK values of k (whole-line loads into a register ring of PF slabs, running ahead
// across layer boundaries; while one slab is multiplied the next is written to the other buffer).  Every
// wavefront loads, stages and multiplies its own weight rows only, so the slab loop has no workgroup barrier.  The raw sums of a step go through the slab buffer that has just become free, so that
// the update -- new state to LDS and to global memory, next operand -- is one float4 pass over whole rows.  Wavefront w of NWV owns the column blocks w*NBW .. w*NBW + NBW - 1 of 32 columns;
// q = 32 * NBW * NWV.  Width 256 runs with eight wavefronts of one column block each: two per SIMD, so that one
// wavefront's fragment reads and float4 passes hide behind the other's matrix instructions (four wavefronts of two
// blocks left the matrix cores idle half of the time).
// WN: the weights are W[k][n] (the adjoint sweep on the caller's array): a slab is BK rows of k, of which a wavefront
// loads and stages its own columns, k-major with pitch Q + 4 (float) or Q + 16 (bf16) -- no larger than the n-major
// slab -- and the fragments come from mma_step_wn.
// ------------------------------------------------------------------------------------------
constexpr int SWEEP_R = 32;
template <typename WT> struct SweepOp;
template <> struct SweepOp<float>  { static constexpr int BK = 32; };
template <> struct SweepOp<__bf16> { static constexpr int BK = 64; };

template <typename WT, int NBW, int PF, int NWV, bool WN = false>
__global__ __launch_bounds__(64 * NWV) void dense_sweep_kernel(SweepArgs a) {
  constexpr int NT = 64 * NWV;                  // shadows the file-wide 256: NWV wavefronts
  constexpr int R = SWEEP_R, BK = SweepOp<WT>::BK, VEC = Op<WT>::VEC, KSTEP = Op<WT>::KSTEP, PAD = Op<WT>::PAD;
  constexpr int Q = 32 * NBW * NWV, Q4 = Q / 4;
  constexpr int AST = Q + PAD, ST = BK + PAD;
  constexpr int PPR = BK / VEC;                 // 16-byte pieces per weight row and slab (one 128-byte line)
  constexpr int WROWS = 32 * NBW;               // weight rows (output columns) of a wavefront
  constexpr int BP = WROWS * PPR / 64;          // pieces per lane and slab
  constexpr int NSL = Q / BK;                   // slabs per layer
  static_assert(WROWS * PPR % 64 == 0 && R * Q4 % NT == 0, "slab and slice must divide over the lanes");
  constexpr int QP = Q + (sizeof(WT) == 2 ? 16 : 4);    // k-major slab: row pitch
  constexpr int PPN = WROWS / VEC;                      // ... and 16-byte pieces of a wavefront's columns per k row
  constexpr int BUF = WN ? BK * QP : Q * ST;            // elements of one slab buffer
  static_assert(BK * QP <= Q * ST, "the k-major slab fits the n-major one's buffer");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* S = reinterpret_cast<float*>(smem_raw);           // [R][Q] state slice
  WT* A = reinterpret_cast<WT*>(S + R * Q);                // [R][AST] operand of the current step
  WT* Bs = A + R * AST;                                    // [2][Q][ST] weight slabs: row = output column, k fastest

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = lane >> 5, c = lane & 31;
  const int L = logical_block();
  const int nsl = (a.M + R - 1) / R;
  const long long ci = L / nsl;
  const int r0 = (L % nsl) * R;
  const int rows = min(R, a.M - r0);
  const long long slice_off = (long long)r0 * Q;
  const WT* Wall = reinterpret_cast<const WT*>(a.W);
  const WT* Dall = reinterpret_cast<const WT*>(a.Dm);
  auto layer_of = [&](int k) { return a.lb + ci * a.ls + (long long)(k - 1) * a.lk; };

  // ---- weight slabs: the sweep's slabs are numbered through, it = (k - 1) * NSL + sl; PF of them are in
  // flight in registers (a workgroup has a CU to itself, so the loaded memory latency is hidden by depth)
  const int total = a.nsteps * NSL;
  uint4 breg[PF][BP];
  auto load_slab = [&](uint4 (&br)[BP], int it) {
    const WT* Wp = Wall + layer_of(it / NSL + 1) * a.wsize + (it % NSL) * (WN ? BK * Q : BK);   // slab = k range
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      if constexpr (WN) {
        const int p = lane + 64 * i, kr = p / PPN, col = wave * WROWS + (p % PPN) * VEC;
        br[i] = ld_weights<false>(Wp + kr * Q + col);
      } else {
        const int p = lane + 64 * i, row = wave * WROWS + p / PPR, kc = (p % PPR) * VEC;
        br[i] = ld_weights<false>(Wp + row * Q + kc);
      }
    }
  };
  auto store_slab = [&](const uint4 (&br)[BP], WT* dst) {
#pragma unroll
    for (int i = 0; i < BP; ++i) {
      if constexpr (WN) {
        const int p = lane + 64 * i, kr = p / PPN, col = wave * WROWS + (p % PPN) * VEC;
        *reinterpret_cast<uint4*>(&dst[kr * QP + col]) = br[i];
      } else {
        const int p = lane + 64 * i, row = wave * WROWS + p / PPR, kc = (p % PPR) * VEC;
        *reinterpret_cast<uint4*>(&dst[row * ST + kc]) = br[i];
      }
    }
  };
  // A wavefront loads, stages and multiplies only its own weight rows, so the slab pipeline needs no workgroup
  // barrier: its LDS operations execute in order, and the fences only keep the compiler from moving the
  // fragment reads across the stores.
  auto wave_sync = [&]() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
#pragma unroll
  for (int sidx = 0; sidx < PF; ++sidx)
    if (sidx < total) load_slab(breg[sidx], sidx);

  // ---- start state -> S (rows past the batch end are zero; loads are unconditional)
  {
    const float* sp = a.S + (a.sm.base + ci * a.sm.stride) * a.E + slice_off;
#pragma unroll
    for (int i = 0; i < R * Q4 / NT; ++i) {
      const int p = tid + NT * i, row = p / Q4, c4 = (p % Q4) * 4;
      const bool ok = row < rows;
      float4 v = *reinterpret_cast<const float4*>(sp + (ok ? row * Q + c4 : 0));
      if (!ok) v = make_float4(0.f, 0.f, 0.f, 0.f);
      *reinterpret_cast<float4*>(S + row * Q + c4) = v;
    }
  }
  // The column group of a thread in the float4 passes over the slice is the same for all its pieces
  // (256 threads are a multiple of the Q/4 pieces of a row)
  const int c4t = (tid % Q4) * 4;
  // operand of a step from the state slice: (Dm[layer] .* S) in the matrix-core type
  auto build_operand = [&](long long layer) {
    const WT* dp = Dall ? Dall + layer * a.E + slice_off : nullptr;
#pragma unroll
    for (int i = 0; i < R * Q4 / NT; ++i) {
      const int row = (tid + NT * i) / Q4;
      float4 v = *reinterpret_cast<const float4*>(S + row * Q + c4t);
      if (dp) {
        const float4 d = d4_to_f4(ld_d4(dp + (row < rows ? row * Q + c4t : 0)));
        v.x *= d.x; v.y *= d.y; v.z *= d.z; v.w *= d.w;       // rows past the end hold 0 in S
      }
      cvt_store4(&A[row * AST + c4t], v);
    }
  };
  __syncthreads();                                         // S complete
  build_operand(layer_of(1));
  // slab j lives in ring slot j % PF and goes to LDS buffer j % 2; a slot is reloaded with slab j + PF as
  // soon as slab j has been written to LDS
  static_assert(NSL % PF == 0 && PF % 2 == 0, "ring slot and LDS buffer of a slab must be compile-time values");
  store_slab(breg[0], Bs);
  if (PF < total) load_slab(breg[0], PF);
  __syncthreads();                                         // the first operand is complete

  for (int k = 1; k <= a.nsteps; ++k) {
    floatx16 acc[1][NBW];
    // bias of this thread's column group in the float4 pass: requested before the contraction, its latency
    // would otherwise open the epilogue
    const long long layer = layer_of(k);
    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (a.bias) bv = *reinterpret_cast<const float4*>(a.bias + layer * Q + c4t);
#pragma unroll
    for (int t = 0; t < NBW; ++t) acc[0][t] = zero16();
    for (int sl0 = 0; sl0 < NSL; sl0 += PF) {
#pragma unroll
      for (int sidx = 0; sidx < PF; ++sidx) {
        const int sl = sl0 + sidx, it = (k - 1) * NSL + sl;
        wave_sync();                                       // slab it of this wavefront is in LDS; slab it-1 consumed
        if (it + 1 < total) {                              // next slab (maybe the next layer's first) -> other buffer
          store_slab(breg[(sidx + 1) % PF], Bs + ((sidx + 1) & 1) * BUF);
          if (it + 1 + PF < total) load_slab(breg[(sidx + 1) % PF], it + 1 + PF);
        }
        const WT* Bcur = Bs + (sidx & 1) * BUF;
#pragma unroll
        for (int ks = 0; ks < BK; ks += KSTEP) {
          const WT* ap[1] = {&A[c * AST + sl * BK + ks]};
          if constexpr (WN) {
            int bcol[NBW];
#pragma unroll
            for (int t = 0; t < NBW; ++t) bcol[t] = (wave * NBW + t) * 32 + c;
            mma_step_wn<1, NBW>(ap, Bcur + ks * QP, QP, bcol, acc, g);
          } else {
            const WT* bp[NBW];
#pragma unroll
            for (int t = 0; t < NBW; ++t) bp[t] = &Bcur[((wave * NBW + t) * 32 + c) * ST + ks];
            mma_step<1, NBW>(ap, bp, acc, g);
          }
        }
      }
    }
    // ---- epilogue of step k.  The raw sums go through the weight buffer that the last slab has just left
    // (the other one already holds the next layer's first slab), so that the update is one float4 pass over
    // whole rows: new state to S and to global memory, and the next step's operand to A.
    __syncthreads();                                       // every wavefront is done with that buffer and with A
    constexpr int ZST = Q + 4;
    float* Z = reinterpret_cast<float*>(Bs + ((NSL - 1) & 1) * BUF);          // [R][ZST], fits: 128 Q + 512 bytes in either layout
    static_assert((size_t)BUF * sizeof(WT) >= sizeof(float) * R * ZST, "the raw sums fit a slab buffer");
#pragma unroll
    for (int t = 0; t < NBW; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r)                          // lane holds rows 8*(r/4) + 4*g + r%4 of column n
        Z[(8 * (r >> 2) + 4 * g + (r & 3)) * ZST + (wave * NBW + t) * 32 + c] = acc[0][t][r];
    __syncthreads();
    {
      const float* gp = a.G ? a.G + (a.gb + ci * a.gs + k) * a.E + slice_off : nullptr;
      float* xo = a.X + (a.xb + ci * a.xs + (long long)k * a.xk) * a.E + slice_off;
      const bool build = k < a.nsteps;
      const WT* dp = (Dall && build) ? Dall + layer_of(k + 1) * a.E + slice_off : nullptr;
      // (the activation as a compile-time value inside the pass: one branch per step, not four per float4)
      auto update_pass = [&](auto actc) {
      constexpr int ACT = decltype(actc)::value;
#pragma unroll
      for (int i = 0; i < R * Q4 / NT; ++i) {
        const int row = (tid + NT * i) / Q4;
        const bool ok = row < rows;
        const int off = ok ? row * Q + c4t : 0;
        const float4 z = *reinterpret_cast<const float4*>(Z + row * ZST + c4t);
        float4 u = *reinterpret_cast<const float4*>(S + row * Q + c4t);
        u.x += a.hs * act_fn_c<ACT>(z.x + bv.x); u.y += a.hs * act_fn_c<ACT>(z.y + bv.y);
        u.z += a.hs * act_fn_c<ACT>(z.z + bv.z); u.w += a.hs * act_fn_c<ACT>(z.w + bv.w);
        if (gp) {
          const float4 gv = *reinterpret_cast<const float4*>(gp + off);
          u.x += gv.x; u.y += gv.y; u.z += gv.z; u.w += gv.w;
        }
        if (!ok) u = make_float4(0.f, 0.f, 0.f, 0.f);       // rows past the batch end stay zero
        *reinterpret_cast<float4*>(S + row * Q + c4t) = u;
        if (ok) *reinterpret_cast<float4*>(xo + off) = u;
        if (build) {
          if (dp) {
            const float4 d = d4_to_f4(ld_d4(dp + off));
            u.x *= d.x; u.y *= d.y; u.z *= d.z; u.w *= d.w;
          }
          cvt_store4(&A[row * AST + c4t], u);
        }
      }
      };
      if (a.act == ACT_TANH)      update_pass(std::integral_constant<int, ACT_TANH>{});
      else if (a.act == ACT_RELU) update_pass(std::integral_constant<int, ACT_RELU>{});
      else                        update_pass(std::integral_constant<int, ACT_IDENT>{});
    }
    __syncthreads();                                       // next operand complete; the sums' buffer is free again
  }
}

static size_t sweep_smem_bytes(int q, int dtype) {
  const size_t es = dtype == 0 ? 4 : 2, pad = dtype == 0 ? Op<float>::PAD : Op<__bf16>::PAD;
  const size_t bk = dtype == 0 ? SweepOp<float>::BK : SweepOp<__bf16>::BK;
  return (size_t)SWEEP_R * q * 4 + (size_t)SWEEP_R * (q + pad) * es + (size_t)2 * q * (bk + pad) * es;
}
bool sweep_supported(int q, int dtype) {
  return (q == 128 || q == 256) && sweep_smem_bytes(q, dtype) <= (size_t)150 * 1024;
}
int sweep_blocks(int M, int nchains) { return ((M + SWEEP_R - 1) / SWEEP_R) * nchains; }

template <typename WT, int NBW, int NWV, bool WN = false>
static hipError_t launch_sweep_t(const SweepArgs& a, unsigned blocks, size_t smem, hipStream_t s) {
  if constexpr (!WN) {
    if (a.wn) return launch_sweep_t<WT, NBW, NWV, true>(a, blocks, smem, s);
  }
  // weight slabs in flight in registers: as many as a layer has, at most 4 (eight measured no faster and
  // take 256 registers of a lane)
  constexpr int NSLABS = 32 * NBW * NWV / SweepOp<WT>::BK;
  constexpr int PF = NSLABS < 4 ? NSLABS : 4;
  static LdsOptIn opt;
  if (opt.need(smem)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(dense_sweep_kernel<WT, NBW, PF, NWV, WN>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((dense_sweep_kernel<WT, NBW, PF, NWV, WN>), dim3(blocks), dim3(64 * NWV), smem, s, a);
  return hipGetLastError();
}
// MGRIT_SWEEP_WAVES=4 in the environment runs width 256 with four wavefronts of two column blocks (diagnostic)
static bool sweep_four_waves() {
  const char* e = getenv("MGRIT_SWEEP_WAVES");
  return e && e[0] == '4';
}
hipError_t launch_sweep(const SweepArgs& a, int dtype, hipStream_t s) {
  if (a.nchains <= 0 || a.nsteps <= 0) return hipSuccess;
  if (!sweep_supported(a.q, dtype) || a.M < 1) return hipErrorInvalidValue;
  const size_t smem = sweep_smem_bytes(a.q, dtype);
  const unsigned blocks = (unsigned)sweep_blocks(a.M, a.nchains);
  const bool wide = a.q == 256, w4 = sweep_four_waves();
  trace_before(s);
  hipError_t e = hipErrorInvalidValue;
  if (dtype == 0) {
    if (!wide) e = launch_sweep_t<float, 1, 4>(a, blocks, smem, s);
    else if (w4) e = launch_sweep_t<float, 2, 4>(a, blocks, smem, s);
    else e = launch_sweep_t<float, 1, 8>(a, blocks, smem, s);
  } else {
    if (!wide) e = launch_sweep_t<__bf16, 1, 4>(a, blocks, smem, s);
    else if (w4) e = launch_sweep_t<__bf16, 2, 4>(a, blocks, smem, s);
    else e = launch_sweep_t<__bf16, 1, 8>(a, blocks, smem, s);
  }
  // algorithmic bytes per layer step: weights and bias, the act' factor, the right-hand side, the state out
  // (the state in is read once per chain)
  const double es = dtype == 0 ? 4.0 : 2.0;
  const double per = (double)a.wsize * es + (a.bias ? 4.0 * a.q : 0.0) + (a.Dm ? es : 0.0) * (double)a.E +
                     (a.G ? 4.0 : 0.0) * (double)a.E + 4.0 * (double)a.E;
  trace_after(s, dtype == 0 ? TRACE_SWEEP_F32 : TRACE_SWEEP_BF16, (long long)a.nchains * a.nsteps,
              (double)a.nchains * (a.nsteps * per + 4.0 * (double)a.E));
  return e;
}

// ------------------------------------------------------------------------------------------
// Fused F-relaxation sweep for 3x3 convolution layers with at most 16 float channels.  A workgroup owns one
// image of one coarse interval and marches through all steps of the sweep.  In LDS: the fp32 state of the image
// St [pixel][20], its matrix-core operand P (Dm .* state) as a patch with a one-pixel frame of zeros
// [(H+2)(W+2)][20], and the nine 16x16 weight slices of the current layer.  A step multiplies 16-pixel blocks
// (wavefront w of eight takes blocks w, w+8, ..) with v_mfma_f32_16x16x4_f32 over the nine taps and adds h*act(.) into St
// right away (St is not an operand, so no barrier is needed for that); after a barrier one float4 pass over
// whole pixels adds the right-hand side, stores the new state to global memory and writes the next operand.
// ------------------------------------------------------------------------------------------
constexpr int CSW_CS = 20;                       // floats per pixel in LDS (16 channels + 4 padding)
constexpr int CSW_MAXBLK = 52;                   // 16-pixel blocks per image at most
constexpr int CSW_PASS = (CSW_MAXBLK * 16 * 4 + 511) / 512;   // float4 pieces per thread in a pass over the image at most
constexpr int CSW_NT = 512;                      // eight wavefronts: two per SIMD hide each other's LDS and barrier waits
static size_t conv_sweep_smem(int Himg, int Wimg) {
  return ((size_t)Himg * Wimg + (size_t)(Himg + 2) * (Wimg + 2) + 9 * 16) * CSW_CS * sizeof(float);
}
bool conv_sweep_supported(int Himg, int Wimg, int C, int dtype) {
  if (dtype != 0 || (C != 8 && C != 16) || Himg < 1 || Wimg < 1 || Wimg > 256) return false;
  if ((Himg * Wimg + 15) / 16 > CSW_MAXBLK) return false;
  return conv_sweep_smem(Himg, Wimg) <= (size_t)150 * 1024;
}

template <int ACT>          // the activation as a compile-time value (one branch per launch, not per state value)
__global__ __launch_bounds__(CSW_NT) void conv_sweep_kernel(SweepArgs a, unsigned wmagic) {
  constexpr int NT = CSW_NT;                                 // shadows the file-wide 256
  constexpr int CS = CSW_CS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int H = a.Himg, Wd = a.Wimg, C = a.C, HW = H * Wd, PW = Wd + 2;
  float* St = reinterpret_cast<float*>(smem_raw);            // [HW][CS]
  float* P = St + HW * CS;                                   // [(H+2)*(W+2)][CS]
  float* Wt = P + (H + 2) * PW * CS;                         // [9][16][CS]
  const int tid = threadIdx.x, lane = tid & 63, r16 = lane & 15, kq = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // the same in every lane: block conditions stay scalar
  const int L = logical_block();
  const long long ci = L / a.M;
  const int img = L % a.M;
  const long long img_off = (long long)img * HW * C;
  const float* Wall = reinterpret_cast<const float*>(a.W);
  const float* Dall = reinterpret_cast<const float*>(a.Dm);
  auto layer_of = [&](int k) { return a.lb + ci * a.ls + (long long)(k - 1) * a.lk; };
  const int cq = C / 4, n4 = HW * cq;                        // float4 pieces of a pixel (2 or 4) / of the image
  const int cqs = C == 16 ? 2 : 1;                           // log2(cq)
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);

  // weight slices of a layer: 9 taps x 16 rows x 4 pieces = 576 pieces of 16 bytes, rows / channels past C are zero
  uint4 wall[2];
  unsigned wallmask = 0;
  auto load_w = [&](long long layer) {
    const float* Wp = Wall + layer * a.wsize;
    wallmask = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = tid + NT * i;
      const int tap = p >> 6, row = (p >> 2) & 15, kc = (p & 3) * 4;
      const bool ok = p < 576 && row < C && kc < C;
      wallmask |= ok ? (1u << i) : 0u;
      wall[i] = *reinterpret_cast<const uint4*>(Wp + (ok ? (unsigned)((row * 9 + tap) * C + kc) : 0u));
    }
  };
  auto store_w = [&]() {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = tid + NT * i;
      if (p < 576) {
        const int tap = p >> 6, row = (p >> 2) & 15, kc = (p & 3) * 4;
        uint4 v = wall[i];
        if (!((wallmask >> i) & 1u)) v = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(&Wt[(tap * 16 + row) * CS + kc]) = v;
      }
    }
  };
  load_w(layer_of(1));

  // ---- the frame of the operand patch, and with fewer than 16 channels the channels past C, are zero for the
  // whole sweep: cleared once (the frame alone when every channel is written)
  if (C < 16) {
    for (int p = tid; p < (H + 2) * PW * (CS / 4); p += NT) *reinterpret_cast<float4*>(P + 4 * p) = zero;
  } else {
    const int nfr = 2 * PW + 2 * H;                          // top and bottom rows, left and right columns
    for (int p = tid; p < nfr * 4; p += NT) {
      const int f = p >> 2, c4 = (p & 3) * 4;
      int fy, fx;
      if (f < PW) { fy = 0; fx = f; }
      else if (f < 2 * PW) { fy = H + 1; fx = f - PW; }
      else { const int t = f - 2 * PW; fy = 1 + (t >> 1); fx = (t & 1) ? PW - 1 : 0; }
      *reinterpret_cast<float4*>(P + (fy * PW + fx) * CS + c4) = zero;
    }
  }
  __syncthreads();
  {
    const float* sp = a.S + (a.sm.base + ci * a.sm.stride) * a.E + img_off;
    const float* dp = Dall ? Dall + layer_of(1) * a.E + img_off : nullptr;
    for (int p = tid; p < n4; p += NT) {
      const int px = p >> cqs, c4 = (p - (px << cqs)) * 4;
      const float4 v = *reinterpret_cast<const float4*>(sp + 4 * p);
      *reinterpret_cast<float4*>(St + px * CS + c4) = v;
      float4 o = v;
      if (dp) { const float4 d = *reinterpret_cast<const float4*>(dp + 4 * p); o.x *= d.x; o.y *= d.y; o.z *= d.z; o.w *= d.w; }
      const int py = div_small(px, wmagic);
      *reinterpret_cast<float4*>(P + ((py + 1) * PW + (px - py * Wd) + 1) * CS + c4) = o;
    }
  }
  store_w();
  __syncthreads();

  const int nblk = (HW + 15) / 16;
  for (int k = 1; k <= a.nsteps; ++k) {
    const long long layer = layer_of(k);
    if (k < a.nsteps) load_w(layer_of(k + 1));               // next layer's slices: in flight during this step
    float bo = 0.0f;
    if (a.bias && r16 < C) bo = a.bias[layer * C + r16];
    // the pass at the end of the step needs the right-hand side and the next step's act' factors: requested now,
    // their latency passes behind the matrix instructions
    const bool build = k < a.nsteps;
    const float* gp = a.G ? a.G + (a.gb + ci * a.gs + k) * a.E + img_off : nullptr;
    const float* dp = (Dall && build) ? Dall + layer_of(k + 1) * a.E + img_off : nullptr;
    float4 gpre[CSW_PASS], dpre[CSW_PASS];
#pragma unroll
    for (int i = 0; i < CSW_PASS; ++i) {
      const int p = tid + NT * i;
      const unsigned off = p < n4 ? 4u * (unsigned)p : 0u;
      if (gp) gpre[i] = *reinterpret_cast<const float4*>(gp + off);
      if (dp) dpre[i] = *reinterpret_cast<const float4*>(dp + off);
    }
    // the nine B fragments of this lane (output channel r16, input channels 4 kq .. + 3) serve every block
    float4 bf[9];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) bf[tap] = *reinterpret_cast<const float4*>(Wt + (tap * 16 + r16) * CS + 4 * kq);
    // four blocks at a time: their accumulators are independent, so consecutive matrix instructions never
    // wait for each other.
    // (NV, the number of blocks of the group inside the image, is a compile-time value: a run-time count put a
    // compare and a branch around every matrix instruction of the image's last group)
    auto group = [&](int blk0, auto nvc) {
      constexpr int NV = decltype(nvc)::value;
      const float* ap[4];
      floatx4 acc[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int p = (blk0 + 8 * i) * 16 + r16;                   // this lane's A row: pixel p (rows past the image use pixel 0)
        if (p >= HW) p = 0;
        const int py = div_small(p, wmagic);
        ap[i] = P + (py * PW + (p - py * Wd)) * CS + 4 * kq;
        acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        const int toff = ((tap / 3) * PW + (tap % 3)) * CS;
        float4 af[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) if (i < NV) af[i] = *reinterpret_cast<const float4*>(ap[i] + toff);
#pragma unroll
        for (int i = 0; i < 4; ++i) if (i < NV) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i].x, bf[tap].x, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) if (i < NV) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i].y, bf[tap].y, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) if (i < NV) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i].z, bf[tap].z, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) if (i < NV) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[i].w, bf[tap].w, acc[i], 0, 0, 0);
      }
      // register v of a lane holds pixel 4 kq + v of the block, output channel r16.  All sixteen state values
      // are read before the first is written back (written as one read-modify-write each, every read would wait
      // for the write before it: the compiler cannot tell that the addresses differ).
      float sv[4][4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int pv = (blk0 + 8 * i) * 16 + 4 * kq + v;   // >= HW past the image
          if (i < NV) sv[i][v] = St[(pv < HW ? pv : 0) * CS + r16];
        }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int pv = (blk0 + 8 * i) * 16 + 4 * kq + v;
          if (i < NV && pv < HW && r16 < C) St[pv * CS + r16] = sv[i][v] + a.hs * act_fn_c<ACT>(acc[i][v] + bo);
        }
    };
    for (int blk0 = wave; blk0 < nblk; blk0 += 32) {
      const int nv = (nblk - blk0 + 7) / 8;                  // the same for all lanes of the wavefront
      if (nv >= 4)      group(blk0, std::integral_constant<int, 4>{});
      else if (nv == 3) group(blk0, std::integral_constant<int, 3>{});
      else if (nv == 2) group(blk0, std::integral_constant<int, 2>{});
      else              group(blk0, std::integral_constant<int, 1>{});
    }
    __syncthreads();                                         // every block is done with P and has updated St
    {
      float* xo = a.X + (a.xb + ci * a.xs + (long long)k * a.xk) * a.E + img_off;
#pragma unroll
      for (int i = 0; i < CSW_PASS; ++i) {
        const int p = tid + NT * i;
        if (p < n4) {
          const int px = p >> cqs, c4 = (p - (px << cqs)) * 4;
          float4 u = *reinterpret_cast<const float4*>(St + px * CS + c4);
          if (gp) {
            u.x += gpre[i].x; u.y += gpre[i].y; u.z += gpre[i].z; u.w += gpre[i].w;
            *reinterpret_cast<float4*>(St + px * CS + c4) = u;
          }
          *reinterpret_cast<float4*>(xo + 4 * p) = u;
          if (build) {
            if (dp) { u.x *= dpre[i].x; u.y *= dpre[i].y; u.z *= dpre[i].z; u.w *= dpre[i].w; }
            const int py = div_small(px, wmagic);
            *reinterpret_cast<float4*>(P + ((py + 1) * PW + (px - py * Wd) + 1) * CS + c4) = u;
          }
        }
      }
      if (build) store_w();
    }
    __syncthreads();                                         // next operand and weight slices complete
  }
}

hipError_t launch_conv_sweep(const SweepArgs& a, hipStream_t s) {
  if (a.nchains <= 0 || a.nsteps <= 0) return hipSuccess;
  if (!conv_sweep_supported(a.Himg, a.Wimg, a.C, 0) || a.M < 1) return hipErrorInvalidValue;
  const size_t smem = conv_sweep_smem(a.Himg, a.Wimg);
  const int actc = a.act == ACT_TANH ? 0 : a.act == ACT_RELU ? 1 : 2;
  const void* kfn = actc == 0 ? reinterpret_cast<const void*>(conv_sweep_kernel<ACT_TANH>)
                  : actc == 1 ? reinterpret_cast<const void*>(conv_sweep_kernel<ACT_RELU>)
                              : reinterpret_cast<const void*>(conv_sweep_kernel<ACT_IDENT>);
  static LdsOptIn opt[3];
  if (opt[actc].need(smem)) {
    const hipError_t e = hipFuncSetAttribute(kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
  }
  const unsigned blocks = (unsigned)a.M * (unsigned)a.nchains;
  const unsigned wmagic = ((1u << 20) + (unsigned)a.Wimg - 1u) / (unsigned)a.Wimg;
  trace_before(s);
  if (actc == 0)      hipLaunchKernelGGL(conv_sweep_kernel<ACT_TANH>, dim3(blocks), dim3(CSW_NT), smem, s, a, wmagic);
  else if (actc == 1) hipLaunchKernelGGL(conv_sweep_kernel<ACT_RELU>, dim3(blocks), dim3(CSW_NT), smem, s, a, wmagic);
  else                hipLaunchKernelGGL(conv_sweep_kernel<ACT_IDENT>, dim3(blocks), dim3(CSW_NT), smem, s, a, wmagic);
  const hipError_t e = hipGetLastError();
  // algorithmic bytes per layer step: weights and bias, the act' factor, the right-hand side, the state out
  // (the state in is read once per chain)
  const double per = 4.0 * (double)a.wsize + (a.bias ? 4.0 * a.C : 0.0) + (a.Dm ? 4.0 : 0.0) * (double)a.E +
                     (a.G ? 4.0 : 0.0) * (double)a.E + 4.0 * (double)a.E;
  trace_after(s, TRACE_CONV_SWEEP_F32, (long long)a.nchains * a.nsteps, (double)a.nchains * (a.nsteps * per + 4.0 * (double)a.E));
  return e;
}

// MGRIT_GRAD_NARROW=1 in the environment keeps wide dense layers on the 128x128 gradient kernel with its separate
// bias pass (diagnostic; the tests compare both)
static bool dense_grad_narrow_forced() {
  const char* e = getenv("MGRIT_GRAD_NARROW");
  return e && e[0] == '1';
}
hipError_t launch_grad(const GradArgs& a_in, int layer_kind, int dtype, int groups, hipStream_t s) {
  if (groups <= 0) return hipSuccess;
  GradArgs a = a_in;
  trace_before(s);
  bool db_done = false;
  if (layer_kind == 0 && a.Nf >= 512 && !dense_grad_narrow_forced()) {
    // wide layers: 256x256 tiles, the bias gradient in the same launch
    a.tiles = ((a.Nf + 255) / 256) * ((a.Nf + 255) / 256);
    if (a.dW || a.db) {
      const unsigned blocks = (unsigned)a.tiles * (unsigned)groups;
      const hipError_t e = dtype == 0 ? launch_dense_grad_wide<float>(a, blocks, s) : launch_dense_grad_wide<__bf16>(a, blocks, s);
      if (e != hipSuccess) { trace_after(s, TRACE_GRAD, groups, 0.0); return e; }
    }
    db_done = true;
  } else if (layer_kind == 0) {
    a.tiles = ((a.Nf + 127) / 128) * ((a.Nf + 127) / 128);
    if (a.dW || a.db) {                                    // the bias gradient, if wanted, in the same launch
      dim3 grid((unsigned)a.tiles * (unsigned)groups);
      if (dtype == 0) hipLaunchKernelGGL((dense_grad_kernel<float>), grid, dim3(NT), 0, s, a);
      else            hipLaunchKernelGGL((dense_grad_kernel<__bf16>), grid, dim3(NT), 0, s, a);
      db_done = true;
    }
  } else if (a.dW || a.db) {
    const ConvGradGeom gm = conv_grad_geom(a.B, a.Himg, a.Wimg, a.Nf, dtype, groups);
    if (!gm.ok) {                                          // wide image rows: one workgroup per (layer, tap)
      a.tiles = 9;
      if (a.dW) {
        dim3 grid(9u * (unsigned)groups);
        if (dtype == 0) hipLaunchKernelGGL((conv_grad_tap_kernel<float>), grid, dim3(NT), 0, s, a);
        else            hipLaunchKernelGGL((conv_grad_tap_kernel<__bf16>), grid, dim3(NT), 0, s, a);
      }
      if (a.db) launch_bias_grad(a, dtype, groups, s);
    } else {                                               // all taps and the bias gradient in one kernel
      a.layers = groups;
      a.gWp = gm.Wp; a.gR = gm.R; a.gKL = gm.KL; a.gPU = gm.PU; a.gPG = gm.PG;
      a.gspi = gm.spi; a.gslabs = gm.slabs; a.gchunks = gm.chunks; a.gspc = gm.spc;
      a.tiles = gm.chunks;
      const bool n16 = dtype == 0 && a.Nf <= 16;            // 16x16x4 blocks (8 or 16 float channels)
      const int nwv = conv_grad_waves(a.Nf);
      const int tm = a.Nf > 32 ? 2 : 1, tn = n16 ? ((9 * a.Nf + 1 + 15) / 16 + 3) / 4 : ((9 * a.Nf + 1 + 31) / 32 + nwv - 1) / nwv;
      hipError_t e = hipErrorInvalidValue;                 // also the result if the partial-sum buffer is missing
      const unsigned blocks = (unsigned)gm.chunks * (unsigned)groups;
      const bool have_buf = gm.chunks == 1 || a.partial != nullptr;
      if (have_buf && n16 && tn == 2) e = launch_conv_grad<float, 1, 2, true>(a, blocks, gm.smem, s);      // 8 channels: 73 columns
      else if (have_buf && n16 && tn == 3) e = launch_conv_grad<float, 1, 3, true>(a, blocks, gm.smem, s); // 16 channels: 145 columns
      else {
#define MGRIT_CG(TM_, TN_)                                                                                     \
      if (have_buf && tm == TM_ && tn == TN_)                                                                   \
        e = dtype == 0 ? launch_conv_grad<float, TM_, TN_>(a, blocks, gm.smem, s)                               \
                       : launch_conv_grad<__bf16, TM_, TN_>(a, blocks, gm.smem, s);
      if (nwv == 4) { MGRIT_CG(1, 1) MGRIT_CG(1, 2) MGRIT_CG(1, 3) MGRIT_CG(2, 3) MGRIT_CG(2, 4) MGRIT_CG(2, 5) }
#undef MGRIT_CG
      // eight wavefronts (33 .. 64 channels: 10 .. 19 column blocks of 32, two or three per wavefront)
      if (have_buf && nwv == 8 && tn == 2)
        e = dtype == 0 ? launch_conv_grad<float, 2, 2, false, 8>(a, blocks, gm.smem, s) : launch_conv_grad<__bf16, 2, 2, false, 8>(a, blocks, gm.smem, s);
      if (have_buf && nwv == 8 && tn == 3)
        e = dtype == 0 ? launch_conv_grad<float, 2, 3, false, 8>(a, blocks, gm.smem, s) : launch_conv_grad<__bf16, 2, 3, false, 8>(a, blocks, gm.smem, s);
      }
      if (e != hipSuccess) { trace_after(s, TRACE_GRAD, groups, 0.0); return e; }
      if (gm.chunks > 1) {
        const long long total4 = (long long)groups * (a.wsize + a.Nf) / 4;
        long long nb = (total4 + NT - 1) / NT;
        if (nb > 4096) nb = 4096;
        hipLaunchKernelGGL(conv_grad_reduce_kernel, dim3((unsigned)nb), dim3(NT), 0, s, a.partial, a.dW, a.db, groups,
                           a.wsize, a.Nf, gm.chunks, a.hs);
      }
    }
  }
  if (a.db && layer_kind == 0 && !db_done) launch_bias_grad(a, dtype, groups, s);
  const hipError_t e = hipGetLastError();
  // algorithmic bytes of a layer's gradient: U, Lam and the act' factors in, dW and db out
  const double ges = dtype == 0 ? 4.0 : 2.0;
  trace_after(s, TRACE_GRAD, groups,
              (double)groups * ((8.0 + ges) * (double)a.E + (a.dW ? 4.0 * (double)a.wsize : 0.0) + (a.db ? 4.0 * a.Nf : 0.0)));
  return e;
}

}  // namespace mgrit
