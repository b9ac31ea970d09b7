// Device code of the specialised FusedMM kernels (gfx950, wave64).
//
// Work decomposition (one launch covers all three kinds of workgroup):
//   * packed rows : short rows; a wavefront is cut into S = 64/G lane groups, each
//                   lane group owns one row (UpdateU of Algorithm 1 per lane group);
//   * wave rows   : one wavefront per row; its S lane groups take different stored
//                   entries of the same row and are summed across groups at the end;
//   * chunks      : long rows; a workgroup of 4 wavefronts takes a contiguous chunk of
//                   the row's entries, sums the 4 wavefront partials through LDS in a
//                   fixed order and stores either z_u (single chunk) or a partial row.
// In every kind a lane group of G lanes holds x_u and the z_u accumulator in VGPRs
// (the register blocking of Section IV-A), gathers y_v with 16-byte loads that are
// contiguous across the group, reduces ROP across the group with DPP/swizzle, applies
// SOP and folds MOP+AOP into FMAs.  z_u is written once with non-temporal stores.
#pragma once
#include "fusedmm_internal.h"
#include "../../include/fusedmm.h"

namespace fmm {

// The element type of X, Y, Z, the edge values and all arithmetic: float, or double when a translation unit
// defines FMM_F64 before including this header (the instances behind fusedmm_execute_f64).  A row register
// then holds four doubles (32 bytes, two 16-byte loads); everything else is the same code.
#ifdef FMM_F64
typedef double real;
#else
typedef float real;
#endif
typedef real vec4 __attribute__((ext_vector_type(4)));
// The same four elements where they lie in global memory: rows of X, Y and Z only have to be aligned to one
// element (any leading dimension, any column offset).  The hardware takes a 16-byte access at any 4-byte address,
// so this costs nothing where the rows are aligned; in LDS and registers the natural alignment stays.
typedef real vec4g __attribute__((ext_vector_type(4), aligned(sizeof(real))));

// the typed views of the untyped-by-precision pointers of KernelArgs
__device__ __forceinline__ const real* values_of(const KernelArgs& a) { return reinterpret_cast<const real*>(a.values); }
__device__ __forceinline__ const real* X_of(const KernelArgs& a) { return reinterpret_cast<const real*>(a.X); }
__device__ __forceinline__ real* Z_of(const KernelArgs& a) { return reinterpret_cast<real*>(a.Z); }
__device__ __forceinline__ real* partials_of(const KernelArgs& a) { return reinterpret_cast<real*>(a.partials); }

// hardware approximations in fp32 (1 ulp), library routines in fp64
__device__ __forceinline__ float rcp_(float v) { return __builtin_amdgcn_rcpf(v); }
__device__ __forceinline__ double rcp_(double v) { return 1.0 / v; }
__device__ __forceinline__ float exp2_(float v) { return __builtin_amdgcn_exp2f(v); }
__device__ __forceinline__ double exp2_(double v) { return exp2(v); }
__device__ __forceinline__ float sqrt_(float v) { return __builtin_amdgcn_sqrtf(v); }
__device__ __forceinline__ double sqrt_(double v) { return sqrt(v); }
__device__ __forceinline__ float fma_(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float max_(float a, float b) { return fmaxf(a, b); }
__device__ __forceinline__ double max_(double a, double b) { return fmax(a, b); }
__device__ __forceinline__ float min_(float a, float b) { return fminf(a, b); }
__device__ __forceinline__ double min_(double a, double b) { return fmin(a, b); }
constexpr real kLog2e = (real)1.4426950408889634;

// ---------------------------------------------------------------------------------------
// cross-lane helpers
// ---------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v) {  // the two halves move separately
  const uint64_t u = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xF, 0xF, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xF, 0xF, true);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// value of lane (lane ^ MASK); MASK a power of two
template <int MASK>
__device__ __forceinline__ double lane_xor(double v) {
  if constexpr (MASK == 1) return dpp_mov<0xB1>(v);
  else if constexpr (MASK == 2) return dpp_mov<0x4E>(v);
  else if constexpr (MASK == 8) return dpp_mov<0x128>(v);
  else if constexpr (MASK == 16) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)u, 0x401F);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)(u >> 32), 0x401F);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
  } else return __shfl_xor(v, MASK);
}
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
  if constexpr (MASK == 1) return dpp_mov<0xB1>(v);        // quad_perm [1,0,3,2]
  else if constexpr (MASK == 2) return dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
  else if constexpr (MASK == 8) return dpp_mov<0x128>(v);  // row_ror:8
  else if constexpr (MASK == 16)
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));  // swap 16
  else return __shfl_xor(v, MASK);
}

// Sum over each aligned group of G lanes, result in every lane of the group.
template <int G>
__device__ __forceinline__ real group_allreduce(real v) {
  static_assert(G == 8 || G == 16 || G == 32 || G == 64, "lane group size");
  v += dpp_mov<0xB1>(v);                      // lanes ^1
  v += dpp_mov<0x4E>(v);                      // lanes ^2   -> quad sums
  v += dpp_mov<0x141>(v);                     // row_half_mirror -> sums of 8
  if constexpr (G >= 16) v += dpp_mov<0x140>(v);  // row_mirror -> sums of 16
  if constexpr (G >= 32) v += lane_xor<16>(v);
  if constexpr (G >= 64) v += lane_xor<32>(v);
  return v;
}

// Product over each aligned group of G lanes (ROP = RMUL), result in every lane of the group.
template <int G>
__device__ __forceinline__ real group_allreduce_mul(real v) {
  v *= dpp_mov<0xB1>(v);
  v *= dpp_mov<0x4E>(v);
  v *= dpp_mov<0x141>(v);
  if constexpr (G >= 16) v *= dpp_mov<0x140>(v);
  if constexpr (G >= 32) v *= lane_xor<16>(v);
  if constexpr (G >= 64) v *= lane_xor<32>(v);
  return v;
}

// AOP on two values: SUM, MAX or MIN (aop is wave-uniform).
__device__ __forceinline__ real aop_apply(int aop, real z, real w) {
  return aop == FUSEDMM_AOP_SUM ? z + w : (aop == FUSEDMM_AOP_MAX ? max_(z, w) : min_(z, w));
}

// What a compile-time pattern fixes (PAT_RUNTIME decides the same things from the launch arguments).
template <int P>
struct PatTraits {
  static constexpr bool gcn = (P == PAT_GCN || P == PAT_GCN_MAX || P == PAT_GCN_MIN);
  static constexpr bool dot = (P == PAT_DOT || P == PAT_DOT_MM);
  static constexpr bool dist = (P == PAT_DIST || P == PAT_DIST_MM);
  static constexpr bool family = dot || dist;                       // scalar steps read at run time
  static constexpr bool flips = (P == PAT_DOT_MM || P == PAT_DIST_MM);  // accumulates sign * w by MAX, stores sign * z
  static constexpr bool uses_x = (!gcn && P != PAT_VISIT);
  static constexpr bool uses_val = (gcn || P == PAT_SIGNED_SIGMOID);
  static constexpr bool loads_y = (P != PAT_VISIT);
  // rows may be narrower than the instance whatever the launch says (the other patterns have a masked and an
  // unmasked instance, chosen by kPatMasked)
  static constexpr bool masked = (P == PAT_RUNTIME || family);
  // how messages are accumulated when it is fixed at compile time, and whether a row stored whole
  // may have to be divided by its length (mean pooling: a.mean)
  static constexpr int aop = (P == PAT_GCN_MAX || flips) ? FUSEDMM_AOP_MAX : (P == PAT_GCN_MIN ? FUSEDMM_AOP_MIN : FUSEDMM_AOP_SUM);
  static constexpr bool means = (P == PAT_RUNTIME || P == PAT_GCN || P == PAT_DOT || P == PAT_DIST);
};
// How an instance treats rows narrower than its size: not at all, by whole 4-element pieces, or down to the
// element.
enum : int { kMaskNone = 0, kMaskPieces = 1, kMaskRagged = 2 };
template <int PM>
constexpr int mask_mode() {
  if ((PM & kPatRagged) != 0) return kMaskRagged;
  return (PatTraits<(PM & ~(kPatMasked | kPatRagged))>::masked || (PM & kPatMasked) != 0) ? kMaskPieces : kMaskNone;
}
// Sum of the same lane-in-group position over all S = 64/G groups of the wavefront.
template <int G>
__device__ __forceinline__ real cross_group_allreduce(real v) {
  if constexpr (G <= 8) v += lane_xor<8>(v);
  if constexpr (G <= 16) v += lane_xor<16>(v);
  if constexpr (G <= 32) v += lane_xor<32>(v);
  return v;
}

// The same across-group combination with a run-time AOP.
template <int G>
__device__ __forceinline__ real cross_group_allreduce_aop(int aop, real v) {
  if constexpr (G <= 8) v = aop_apply(aop, v, lane_xor<8>(v));
  if constexpr (G <= 16) v = aop_apply(aop, v, lane_xor<16>(v));
  if constexpr (G <= 32) v = aop_apply(aop, v, lane_xor<32>(v));
  return v;
}

template <int P, int G, int V>
__device__ __forceinline__ void combine_groups(const KernelArgs& a, vec4 (&z)[V]) {
#pragma unroll
  for (int i = 0; i < V; ++i) {
    if constexpr (P == PAT_RUNTIME) {
      z[i].x = cross_group_allreduce_aop<G>(a.aop, z[i].x);
      z[i].y = cross_group_allreduce_aop<G>(a.aop, z[i].y);
      z[i].z = cross_group_allreduce_aop<G>(a.aop, z[i].z);
      z[i].w = cross_group_allreduce_aop<G>(a.aop, z[i].w);
    } else if constexpr (PatTraits<P>::aop != FUSEDMM_AOP_SUM) {
      z[i].x = cross_group_allreduce_aop<G>(PatTraits<P>::aop, z[i].x);
      z[i].y = cross_group_allreduce_aop<G>(PatTraits<P>::aop, z[i].y);
      z[i].z = cross_group_allreduce_aop<G>(PatTraits<P>::aop, z[i].z);
      z[i].w = cross_group_allreduce_aop<G>(PatTraits<P>::aop, z[i].w);
    } else {
      z[i].x = cross_group_allreduce<G>(z[i].x);
      z[i].y = cross_group_allreduce<G>(z[i].y);
      z[i].z = cross_group_allreduce<G>(z[i].z);
      z[i].w = cross_group_allreduce<G>(z[i].w);
    }
  }
}

__device__ __forceinline__ vec4 ld4(const real* p) { return *reinterpret_cast<const vec4g*>(p); }

// The last piece of a row whose length is not a multiple of 4: its first `tail` (1..3) elements, the rest zero /
// untouched.  Element by element, so that nothing beyond the end of the row (and of the matrix) is touched.
__device__ __forceinline__ vec4 ld_tail(const real* p, int tail) {
  vec4 v = {0.f, 0.f, 0.f, 0.f};
  v.x = p[0];
  if (tail > 1) v.y = p[1];
  if (tail > 2) v.z = p[2];
  return v;
}
__device__ __forceinline__ void st_tail(real* p, const vec4& v, int tail) {
  __builtin_nontemporal_store(v.x, p);
  if (tail > 1) __builtin_nontemporal_store(v.y, p + 1);
  if (tail > 2) __builtin_nontemporal_store(v.z, p + 2);
}
__device__ __forceinline__ void st4(real* p, const vec4& v) {
  __builtin_nontemporal_store(static_cast<vec4g>(v), reinterpret_cast<vec4g*>(p));
}

// Four elements of a row of Y stored in 2-byte elements (8 bytes as two 32-bit words) as four floats: bfloat16
// is the upper 16 bits of the float and is widened by shifts, IEEE half by the hardware conversion.  The
// arithmetic stays fp32 in every case.
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
template <int YF>
__device__ __forceinline__ vec4 widen4(v2u raw) {
  if constexpr (YF == kYBf16) {
    return vec4{__builtin_bit_cast(float, raw.x << 16), __builtin_bit_cast(float, raw.x & 0xffff0000u),
               __builtin_bit_cast(float, raw.y << 16), __builtin_bit_cast(float, raw.y & 0xffff0000u)};
  } else {
    typedef _Float16 v4h __attribute__((ext_vector_type(4)));
    const v4h h = __builtin_bit_cast(v4h, raw);
    return vec4{(float)h.x, (float)h.y, (float)h.z, (float)h.w};
  }
}

// Which 4-float piece of a row register i of lane g holds.  C = 1: piece g + G*i (a lane group reads
// G consecutive 16-byte pieces per step).  C = 2 (rows of 2-byte elements read 16 bytes = 8 elements
// at a time): registers 2j and 2j+1 hold the two pieces of chunk g + G*j.
template <int G, int C>
__device__ __forceinline__ int piece_index(int g, int i) {
  if constexpr (C == 1) return g + G * i; else return 2 * (g + G * (i / 2)) + (i & 1);
}

// What a lane holds of a gathered row of Y between the loads and the arithmetic: the registers as loaded -- V 16-byte
// pieces of fp32 (fp64) elements, or, for rows of 2-byte elements, V 8-byte loads (C = 1) or V / 2 16-byte loads (C = 2).
// Nothing may use a loaded value while the loads of the other rows in flight are still to be issued (the use would
// make them wait), so placing, trimming and widening are left to finish_row.
template <bool Native, int V, int C>
struct RowBuf;
template <int V, int C>
struct RowBuf<true, V, C> { vec4 r[V]; };
template <int V>
struct RowBuf<false, V, 1> { v2u r[V]; };
template <int V>
struct RowBuf<false, V, 2> { v4u r[V / 2]; };

template <bool Native, int V, int C>
__device__ __forceinline__ void clear(RowBuf<Native, V, C>& b) {
  constexpr int N = sizeof(b.r) / sizeof(b.r[0]);
#pragma unroll
  for (int i = 0; i < N; ++i) b.r[i] = {};
}

// One lane's share of row `col` of Y as loaded, in the layout of piece_index<G, C>: fp32 (fp64 in the
// double-precision build) rows by one 16-byte load per piece; rows of 2-byte elements by one 8-byte load per
// piece (C = 1) or one 16-byte load per two pieces (C = 2: half as many load instructions per row, and it is
// the number of load instructions that occupies the return path).
// The address is one 32 x 32 -> 64-bit multiply-add: column index (validated, non-negative) times the row
// pitch in bytes (below 2^32, checked by the host) plus the lane's own offset.
// M = kMaskPieces: pieces at or beyond a.d_pieces read as zero (a dimension below the instance's own);
// M = kMaskRagged: and the row may end inside its last piece (a dimension that is not a multiple of 4).
template <int YF, int G, int V, int C, int M>
__device__ __forceinline__ void gather_row(const KernelArgs& a, int col, int g, RowBuf<YF == kYF32, V, C>& b) {
  const uint32_t pitch = (uint32_t)a.ldy * (YF == kYF32 ? (uint32_t)sizeof(real) : 2u);
  const char* row = static_cast<const char*>(a.Y) + (uint64_t)(uint32_t)col * (uint64_t)pitch;
  if constexpr (YF == kYF32) {
    static_assert(C == 1, "one 16-byte load per piece");
    // Ragged rows: the piece the row ends in is fetched by the same 16-byte load instruction as the whole pieces.
    // It then holds, beyond the row, the first elements of the next row of Y or padding -- inside the matrix either
    // way -- except in the last row of Y (the last few when ldy < 3), after which the allocation may end: there the
    // load is moved back so that it ends with the row.  finish_row puts the elements in place and zeros the rest.
    const int back = (M == kMaskRagged && col >= a.y_first_back_row) ? 4 - a.d_tail : 0;
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const int piece = g + G * i;
      if (M == kMaskNone || piece < a.d_pieces) {
        const real* p = reinterpret_cast<const real*>(row) + 4 * piece;
        if constexpr (M == kMaskRagged) p -= piece == a.d_full ? back : 0;
        b.r[i] = *reinterpret_cast<const vec4g*>(p);
      } else {
        b.r[i] = vec4{0.f, 0.f, 0.f, 0.f};
      }
    }
  } else if constexpr (C == 1) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const int piece = g + G * i;
      if (M == kMaskNone || piece < a.d_pieces) b.r[i] = *reinterpret_cast<const v2u*>(row + (size_t)piece * 8u);
      else b.r[i] = v2u{0u, 0u};
    }
  } else {
    static_assert(V % 2 == 0, "16-byte chunks of 2-byte elements");
#pragma unroll
    for (int j = 0; j < V / 2; ++j) {
      const int chunk = g + G * j;
      if (M == kMaskNone || 2 * chunk + 1 < a.d_pieces) b.r[j] = *reinterpret_cast<const v4u*>(row + (size_t)chunk * 16u);
      else b.r[j] = v4u{0u, 0u, 0u, 0u};
    }
  }
}

// The row as the arithmetic wants it, V registers of four elements, from what gather_row loaded: rows of 2-byte
// elements are widened; in the ragged instances the gathered piece the row ends in (piece d_full: register
// d_full / G of lane d_full % G) holds d_tail elements of the row -- at its front, followed by whatever comes after
// the row, or, from row y_first_back_row of Y on, at its back -- which are moved to the front and the rest zeroed
// (selects, not products: what lies beyond the row may be anything).
template <int YF, int G, int V, int C, int M>
__device__ __forceinline__ void finish_row(const KernelArgs& a, int g, int col, const RowBuf<YF == kYF32, V, C>& b, vec4 (&y)[V]) {
  if constexpr (YF == kYF32) {
#pragma unroll
    for (int i = 0; i < V; ++i) y[i] = b.r[i];
    if constexpr (M == kMaskRagged) {
      const int it = a.d_full / G;  // wave-uniform
      const bool mine = g == a.d_full % G;
      const bool moved = col >= a.y_first_back_row;
      const int t = a.d_tail;
#pragma unroll
      for (int i = 0; i < V; ++i) {
        if (i == it) {
          const vec4 v = y[i];
          const real fx = moved ? (t == 1 ? v.w : (t == 2 ? v.z : v.y)) : v.x;
          const real fy = t > 1 ? (moved ? (t == 2 ? v.w : v.z) : v.y) : (real)0;
          const real fz = t > 2 ? (moved ? v.w : v.z) : (real)0;
          y[i].x = mine ? fx : v.x;
          y[i].y = mine ? fy : v.y;
          y[i].z = mine ? fz : v.z;
          y[i].w = mine ? (real)0 : v.w;
        }
      }
    }
  } else if constexpr (C == 1) {
#pragma unroll
    for (int i = 0; i < V; ++i) y[i] = widen4<YF>(b.r[i]);
  } else {
#pragma unroll
    for (int j = 0; j < V / 2; ++j) {
      y[2 * j] = widen4<YF>(v2u{b.r[j].x, b.r[j].y});
      y[2 * j + 1] = widen4<YF>(v2u{b.r[j].z, b.r[j].w});
    }
  }
}

// Loads of data that is read once (column indices, edge values, x_u) carry no cache hint: a non-temporal
// hint on them was measured at -1 % kernel time on the two largest workloads and +3..10 % on the two where
// X aliases Y (x_u is then also somebody's y_v).  Hinting the gathers of rarely used rows of Y (chosen by
// the plan from the entry counts of the columns) raised the L2 hit rate by 3.5 points and cost 15-100 %.
template <class T>
__device__ __forceinline__ T ld_stream(const T* p) { return *p; }
__device__ __forceinline__ vec4 ld4_stream(const real* p) { return *reinterpret_cast<const vec4g*>(p); }


// ---------------------------------------------------------------------------------------
// per-entry arithmetic: VOP, ROP, SOP, MOP, AOP for one stored entry, on one lane group
// ---------------------------------------------------------------------------------------
// whether x_u / the edge values are read: fixed per pattern, a (uniform) run-time fact for PAT_RUNTIME
template <int P>
__device__ __forceinline__ bool reads_x(const KernelArgs& a) {
  if constexpr (P == PAT_RUNTIME) return a.vop != FUSEDMM_VOP_SEL2ND; else return PatTraits<P>::uses_x;
}
template <int P>
__device__ __forceinline__ bool reads_values(const KernelArgs& a) {
  if constexpr (P == PAT_RUNTIME) return a.sop == FUSEDMM_SOP_EDGE_VALUE || a.sop == kSopValueMinusSigmoid;
  else if constexpr (PatTraits<P>::family) return a.sop == kSopValueMinusSigmoid;
  else return PatTraits<P>::uses_val;
}

__device__ __forceinline__ real rt_vop(int vop, real x, real y) {
  switch (vop) {
    case FUSEDMM_VOP_MUL: return x * y;
    case FUSEDMM_VOP_SEL2ND: return y;
    case FUSEDMM_VOP_SUB: return x - y;
    default: return x + y;
  }
}
__device__ __forceinline__ real rt_sop(int sop, real s, real alpha) {
  switch (sop) {
    case FUSEDMM_SOP_SIGMOID: return rcp_(1.0f + exp2_(-s * kLog2e));
    case FUSEDMM_SOP_ONE_MINUS_SIGMOID: return rcp_(1.0f + exp2_(s * kLog2e));
    case FUSEDMM_SOP_INV_1P: return rcp_(1.0f + s);
    case FUSEDMM_SOP_SCAL: return alpha * s;
    default: return s;
  }
}

// the scale of the families' exponent, +-log2 e, in the element type's own precision
__device__ __forceinline__ real sop_scale(const KernelArgs& a) {
#ifdef FMM_F64
  return a.sop_c1 < 0.f ? -kLog2e : kLog2e;
#else
  return a.sop_c1;
#endif
}

template <int P, int G, int V, bool CHECK>
__device__ __forceinline__ void edge_update(const vec4 (&x)[V], const vec4 (&y)[V], real aval, const KernelArgs& a,
                                            bool valid, vec4 (&z)[V], int nv = V, int lane_tail = 0) {
  const real alpha = a.alpha;
  if constexpr (P == PAT_RUNTIME) {
    // Every op of the selector, the five steps in order.  The selectors are wave-uniform, so each
    // step is one scalar branch around a loop over this lane's elements, not a choice per element.
    vec4 t[V];
    switch (a.vop) {  // VOP
      case FUSEDMM_VOP_MUL:
#pragma unroll
        for (int i = 0; i < V; ++i) t[i] = x[i] * y[i];
        break;
      case FUSEDMM_VOP_SEL2ND:
#pragma unroll
        for (int i = 0; i < V; ++i) t[i] = y[i];
        break;
      case FUSEDMM_VOP_SUB:
#pragma unroll
        for (int i = 0; i < V; ++i) t[i] = x[i] - y[i];
        break;
      default:
#pragma unroll
        for (int i = 0; i < V; ++i) t[i] = x[i] + y[i];
    }
    const bool scalar_h = a.sop == FUSEDMM_SOP_EDGE_VALUE || a.rop != FUSEDMM_ROP_NOOP;
    real h = aval;
    if (a.sop != FUSEDMM_SOP_EDGE_VALUE && a.rop != FUSEDMM_ROP_NOOP) {  // ROP, then SOP on the scalar
      real s;
      if (a.rop == FUSEDMM_ROP_RMUL) {
        real p = 1.f;  // registers beyond the row's width hold padding, not factors
#pragma unroll
        for (int i = 0; i < V; ++i) {
          if (i >= nv) continue;
          if (i == nv - 1 && lane_tail > 0)  // the row ends inside this lane's last piece
            p *= t[i].x * (lane_tail > 1 ? t[i].y : (real)1) * (lane_tail > 2 ? t[i].z : (real)1);
          else p *= t[i].x * t[i].y * t[i].z * t[i].w;
        }
        s = group_allreduce_mul<G>(p);
      } else if (a.rop == FUSEDMM_ROP_RSUM) {
        real p = 0.f;
#pragma unroll
        for (int i = 0; i < V; ++i) p += (t[i].x + t[i].y) + (t[i].z + t[i].w);
        s = group_allreduce<G>(p);
      } else {
        real p = 0.f;
#pragma unroll
        for (int i = 0; i < V; ++i) p += (t[i].x * t[i].x + t[i].y * t[i].y) + (t[i].z * t[i].z + t[i].w * t[i].w);
        s = group_allreduce<G>(p);
        if (a.rop == FUSEDMM_ROP_NORM2) s = sqrt_(s);
      }
      h = a.sop == kSopValueMinusSigmoid ? aval - rt_sop(FUSEDMM_SOP_SIGMOID, s, alpha) : rt_sop(a.sop, s, alpha);
    }
    vec4 w[V];
    if (scalar_h) {  // MOP with a scalar message
      if (a.mop == FUSEDMM_MOP_SEL2ND) {
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = y[i];
      } else if (a.mop == FUSEDMM_MOP_MUL_Y) {
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = h * y[i];
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = h * t[i];
      }
    } else {  // vector message: SOP on every element of t, then MOP element by element
      vec4 hv[V];
      switch (a.sop) {
        case FUSEDMM_SOP_SIGMOID:
#pragma unroll
          for (int i = 0; i < V; ++i)
            hv[i] = vec4{rt_sop(FUSEDMM_SOP_SIGMOID, t[i].x, alpha), rt_sop(FUSEDMM_SOP_SIGMOID, t[i].y, alpha),
                        rt_sop(FUSEDMM_SOP_SIGMOID, t[i].z, alpha), rt_sop(FUSEDMM_SOP_SIGMOID, t[i].w, alpha)};
          break;
        case FUSEDMM_SOP_ONE_MINUS_SIGMOID:
#pragma unroll
          for (int i = 0; i < V; ++i)
            hv[i] = vec4{rt_sop(FUSEDMM_SOP_ONE_MINUS_SIGMOID, t[i].x, alpha), rt_sop(FUSEDMM_SOP_ONE_MINUS_SIGMOID, t[i].y, alpha),
                        rt_sop(FUSEDMM_SOP_ONE_MINUS_SIGMOID, t[i].z, alpha), rt_sop(FUSEDMM_SOP_ONE_MINUS_SIGMOID, t[i].w, alpha)};
          break;
        case FUSEDMM_SOP_INV_1P:
#pragma unroll
          for (int i = 0; i < V; ++i)
            hv[i] = vec4{rt_sop(FUSEDMM_SOP_INV_1P, t[i].x, alpha), rt_sop(FUSEDMM_SOP_INV_1P, t[i].y, alpha),
                        rt_sop(FUSEDMM_SOP_INV_1P, t[i].z, alpha), rt_sop(FUSEDMM_SOP_INV_1P, t[i].w, alpha)};
          break;
        case FUSEDMM_SOP_SCAL:
#pragma unroll
          for (int i = 0; i < V; ++i) hv[i] = alpha * t[i];
          break;
        default:
#pragma unroll
          for (int i = 0; i < V; ++i) hv[i] = t[i];
      }
      if (a.mop == FUSEDMM_MOP_SEL2ND) {
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = y[i];
      } else if (a.mop == FUSEDMM_MOP_MUL_Y) {
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = hv[i] * y[i];
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) w[i] = hv[i] * t[i];
      }
    }
    if (CHECK && !valid) {  // 0 is neutral for SUM and, from a zero start, for MAX and MIN
#pragma unroll
      for (int i = 0; i < V; ++i) w[i] = vec4{0.f, 0.f, 0.f, 0.f};
    }
    if (a.aop == FUSEDMM_AOP_SUM) {  // AOP
#pragma unroll
      for (int i = 0; i < V; ++i) z[i] += w[i];
    } else if (a.aop == FUSEDMM_AOP_MAX) {
#pragma unroll
      for (int i = 0; i < V; ++i)
        z[i] = vec4{max_(z[i].x, w[i].x), max_(z[i].y, w[i].y), max_(z[i].z, w[i].z), max_(z[i].w, w[i].w)};
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i)
        z[i] = vec4{min_(z[i].x, w[i].x), min_(z[i].y, w[i].y), min_(z[i].z, w[i].z), min_(z[i].w, w[i].w)};
    }
    return;
  }
  if constexpr (PatTraits<P>::family) {
    // The vector loops of the tuple are fixed (dot product or difference / sum of the operands, scalar times
    // vector, SUM or MAX); what acts on the scalar -- NORM2's square root, SOP, SEL2ND's h = 1, the sign of a
    // MIN -- is read from the arguments, wave-uniform.
    vec4 t[V];
    real p = 0.f;
    if constexpr (PatTraits<P>::dot) {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        p = fma_(x[i].x, y[i].x, p);
        p = fma_(x[i].y, y[i].y, p);
        p = fma_(x[i].z, y[i].z, p);
        p = fma_(x[i].w, y[i].w, p);
      }
    } else {
      const real ys = a.ysign;
#pragma unroll
      for (int i = 0; i < V; ++i) t[i] = ys * y[i] + x[i];
      if (a.rop == FUSEDMM_ROP_RSUM) {
#pragma unroll
        for (int i = 0; i < V; ++i) p += (t[i].x + t[i].y) + (t[i].z + t[i].w);
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          p = fma_(t[i].x, t[i].x, p);
          p = fma_(t[i].y, t[i].y, p);
          p = fma_(t[i].z, t[i].z, p);
          p = fma_(t[i].w, t[i].w, p);
        }
      }
    }
    real s = group_allreduce<G>(p);
    if (a.rop == FUSEDMM_ROP_NORM2) s = sqrt_(s);
    const real u = a.sop_exp ? exp2_(sop_scale(a) * s) : s;
    real h = a.sop_rcp ? rcp_(1.0f + u) : a.sop_lin * s;
    if (a.sop == kSopValueMinusSigmoid) h = aval - h;
    if (a.mop == FUSEDMM_MOP_SEL2ND) h = 1.0f;
    if constexpr (PatTraits<P>::flips) h *= a.sign;
    if (CHECK && !valid) h = 0.f;
    if (a.mop == FUSEDMM_MOP_MUL_T) {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        vec4 o;
        if constexpr (PatTraits<P>::dot) o = x[i] * y[i]; else o = t[i];
        if constexpr (PatTraits<P>::flips) {
          const vec4 w = h * o;
          z[i] = vec4{max_(z[i].x, w.x), max_(z[i].y, w.y), max_(z[i].z, w.z), max_(z[i].w, w.w)};
        } else {
          z[i] += h * o;
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < V; ++i) {
        if constexpr (PatTraits<P>::flips) {
          const vec4 w = h * y[i];
          z[i] = vec4{max_(z[i].x, w.x), max_(z[i].y, w.y), max_(z[i].z, w.z), max_(z[i].w, w.w)};
        } else {
          z[i] += h * y[i];
        }
      }
    }
  } else if constexpr (PatTraits<P>::gcn) {
    // VOP = SEL2ND, ROP/SOP no-ops: h = a_uv; MOP: w = h * y; AOP: sum, or maximum / minimum from the
    // zero start (an entry beyond the end contributes w = 0, neutral for all three)
    real h = aval;
    if (CHECK && !valid) h = 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) {
      if constexpr (P == PAT_GCN) {
        z[i] += h * y[i];
      } else {
        const vec4 w = h * y[i];
        z[i].x = aop_apply(PatTraits<P>::aop, z[i].x, w.x); z[i].y = aop_apply(PatTraits<P>::aop, z[i].y, w.y);
        z[i].z = aop_apply(PatTraits<P>::aop, z[i].z, w.z); z[i].w = aop_apply(PatTraits<P>::aop, z[i].w, w.w);
      }
    }
  } else if constexpr (P == PAT_SIGMOID || P == PAT_ONE_MINUS_SIGMOID || P == PAT_SIGNED_SIGMOID) {
    real p = 0.f;  // VOP = MUL and this lane's share of ROP = RSUM
#pragma unroll
    for (int i = 0; i < V; ++i) {
      p = fma_(x[i].x, y[i].x, p);
      p = fma_(x[i].y, y[i].y, p);
      p = fma_(x[i].z, y[i].z, p);
      p = fma_(x[i].w, y[i].w, p);
    }
    const real s = group_allreduce<G>(p);
    // SOP: sigma(s) = 1/(1+2^(-s log2 e)); 1-sigma(s) = sigma(-s).  2^big = inf -> h = 0, no NaN.
    const real e = exp2_(P == PAT_ONE_MINUS_SIGMOID ? s * kLog2e : -s * kLog2e);
    real h = rcp_(1.0f + e);
    if constexpr (P == PAT_SIGNED_SIGMOID) h = aval - h;  // 1 - sigmoid on stored entries, -sigmoid on samples
    if (CHECK && !valid) h = 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) z[i] += h * y[i];  // MOP = MUL with y_v, AOP = SUM
  } else if constexpr (P == PAT_TDIST || P == PAT_FR) {
    vec4 t[V];
    real p = 0.f;  // VOP = SUB, ROP = sum of squares
#pragma unroll
    for (int i = 0; i < V; ++i) {
      t[i] = x[i] - y[i];
      p = fma_(t[i].x, t[i].x, p);
      p = fma_(t[i].y, t[i].y, p);
      p = fma_(t[i].z, t[i].z, p);
      p = fma_(t[i].w, t[i].w, p);
    }
    const real s = group_allreduce<G>(p);
    real h = (P == PAT_TDIST) ? rcp_(1.0f + s) : alpha * sqrt_(s);
    if (CHECK && !valid) h = 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) z[i] += h * t[i];  // MOP = MUL with the VOP output
  }
}

// ---------------------------------------------------------------------------------------
// One wavefront accumulates the stored entries [e0, e1) of a single row.  The S lane groups
// take entries round-robin inside batches of 64; z holds this group's partial sum.
// ---------------------------------------------------------------------------------------
template <int PM, int D, int G, int U, int YF, int C>
__device__ __forceinline__ void wave_accumulate(const KernelArgs& a, int64_t e0, int64_t e1,
                                                const vec4 (&x)[D / (4 * G)], vec4 (&z)[D / (4 * G)], int lane) {
  constexpr int V = D / (4 * G);
  constexpr int S = 64 / G;
  static_assert(S * U <= 64 && 64 % (S * U) == 0, "unroll must tile a batch of 64 entries");
  constexpr int P = PM & ~(kPatMasked | kPatRagged);
  constexpr int kMask = mask_mode<PM>();
  using T = PatTraits<P>;
  const int slot = lane / G;
  const int g = lane % G;
  const bool use_val = reads_values<P>(a);
  int nv = V;  // registers of this lane that hold elements of the row (all of them unless the row is narrower)
  int lane_tail = 0;  // elements in this lane's last such register if the row ends inside it, else 0
  if constexpr (P == PAT_RUNTIME) {
    nv = 0;
#pragma unroll
    for (int i = 0; i < V; ++i) nv += piece_index<G, C>(g, i) < a.d_pieces ? 1 : 0;
    if constexpr (kMask == kMaskRagged) {
      if (a.d_tail > 0 && g == a.d_full % G) lane_tail = a.d_tail;
    }
  }

  for (int64_t base = e0; base < e1; base += 64) {
    const int cnt = (int)((e1 - base) < 64 ? (e1 - base) : 64);  // wave-uniform
    int colb = 0;
    real valb = 0.f;
    if (lane < cnt) {
      colb = ld_stream(a.colidx + base + lane);
      if (use_val) valb = ld_stream(values_of(a) + base + lane);
    }
    for (int k0 = 0; k0 < cnt; k0 += S * U) {
      int c[U];
      real av[U];
      RowBuf<YF == kYF32, V, C> rows[U];
      if (k0 + S * U <= cnt) {
        // every lane group has a stored entry in each of the U steps
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = k0 + u * S + slot;
          c[u] = __shfl(colb, j);
          av[u] = use_val ? __shfl(valb, j) : 0.f;
        }
        if constexpr (T::loads_y) {
#pragma unroll
          for (int u = 0; u < U; ++u) gather_row<YF, G, V, C, kMask>(a, c[u], g, rows[u]);
#pragma unroll
          for (int u = 0; u < U; ++u) {
            vec4 y[V];
            finish_row<YF, G, V, C, kMask>(a, g, c[u], rows[u], y);
            edge_update<P, G, V, false>(x, y, av[u], a, true, z, nv, lane_tail);
          }
        } else {
#pragma unroll
          for (int u = 0; u < U; ++u)
            if (g == 0) atomicAdd(a.visit_counts + (base + k0 + u * S + slot), 1u);
        }
      } else {
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = k0 + u * S + slot;
          ok[u] = j < cnt;
          c[u] = __shfl(colb, j & 63);
          av[u] = use_val ? __shfl(valb, j & 63) : 0.f;
        }
        if constexpr (T::loads_y) {
#pragma unroll
          for (int u = 0; u < U; ++u) {
            clear(rows[u]);
            if (ok[u]) gather_row<YF, G, V, C, kMask>(a, c[u], g, rows[u]);
          }
#pragma unroll
          for (int u = 0; u < U; ++u) {
            vec4 y[V];
            finish_row<YF, G, V, C, kMask>(a, g, c[u], rows[u], y);
            edge_update<P, G, V, true>(x, y, av[u], a, ok[u], z, nv, lane_tail);
          }
        } else {
#pragma unroll
          for (int u = 0; u < U; ++u)
            if (ok[u] && g == 0) atomicAdd(a.visit_counts + (base + k0 + u * S + slot), 1u);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// One lane group accumulates the `deg` stored entries that start at e0 (a short row, a tile, or one
// column-class piece of a row); the S lane groups of the wavefront work on different runs in
// lockstep, maxdeg being the longest of them (wave-uniform).
// ---------------------------------------------------------------------------------------
template <int PM, int D, int G, int U, int YF, int C>
__device__ __forceinline__ void group_accumulate(const KernelArgs& a, int64_t e0, int deg, int maxdeg,
                                                 const vec4 (&x)[D / (4 * G)], vec4 (&z)[D / (4 * G)], int slot, int g, int nv,
                                                 int lane_tail, bool use_val) {
  constexpr int V = D / (4 * G);
  constexpr int P = PM & ~(kPatMasked | kPatRagged);
  constexpr int kMask = mask_mode<PM>();
  using T = PatTraits<P>;
  for (int bb = 0; bb < maxdeg; bb += G) {
    int colb = 0;
    real valb = 0.f;
    if (bb + g < deg) {
      colb = ld_stream(a.colidx + e0 + bb + g);
      if (use_val) valb = ld_stream(values_of(a) + e0 + bb + g);
    }
    const int steps = (maxdeg - bb) < G ? (maxdeg - bb) : G;
    for (int k = 0; k < steps; k += U) {
      bool ok[U];
      int c[U];
      real av[U];
      RowBuf<YF == kYF32, V, C> rows[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        ok[u] = (bb + k + u) < deg;
        c[u] = __shfl(colb, slot * G + k + u);
        av[u] = use_val ? __shfl(valb, slot * G + k + u) : 0.f;
      }
      if constexpr (T::loads_y) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          clear(rows[u]);
          if (ok[u]) gather_row<YF, G, V, C, kMask>(a, c[u], g, rows[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          vec4 y[V];
          finish_row<YF, G, V, C, kMask>(a, g, c[u], rows[u], y);
          edge_update<P, G, V, true>(x, y, av[u], a, ok[u], z, nv, lane_tail);
        }
      } else {
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (ok[u] && g == 0) atomicAdd(a.visit_counts + (e0 + bb + k + u), 1u);
      }
    }
  }
}

template <int D, int G, int C, int M>
__device__ __forceinline__ void load_x(const KernelArgs& a, int64_t row, int g, vec4 (&x)[D / (4 * G)]) {
  const real* xr = X_of(a) + row * a.ldx;
#pragma unroll
  for (int i = 0; i < D / (4 * G); ++i) {
    const int p = piece_index<G, C>(g, i);
    if (M == kMaskNone || p < (M == kMaskRagged ? a.d_full : a.d_pieces)) x[i] = ld4_stream(xr + 4 * p);
    else if (M == kMaskRagged && p < a.d_pieces) x[i] = ld_tail(xr + 4 * p, a.d_tail);
    else x[i] = vec4{0.f, 0.f, 0.f, 0.f};
  }
}

template <int V>
__device__ __forceinline__ void zero(vec4 (&z)[V]) {
#pragma unroll
  for (int i = 0; i < V; ++i) z[i] = vec4{0.f, 0.f, 0.f, 0.f};
}

template <int V>
__device__ __forceinline__ void scale(vec4 (&z)[V], real f) {
#pragma unroll
  for (int i = 0; i < V; ++i) z[i] *= f;
}

template <int D, int G, int C, int M>
__device__ __forceinline__ void store_row(const KernelArgs& a, real* dst, int g, const vec4 (&z)[D / (4 * G)]) {
#pragma unroll
  for (int i = 0; i < D / (4 * G); ++i) {
    const int p = piece_index<G, C>(g, i);
    if (M == kMaskNone || p < (M == kMaskRagged ? a.d_full : a.d_pieces)) st4(dst + 4 * p, z[i]);
    else if (M == kMaskRagged && p < a.d_pieces) st_tail(dst + 4 * p, z[i], a.d_tail);
  }
}

// ---------------------------------------------------------------------------------------
// The fused kernel.  GW/UW: lane-group size and unroll of the wave and chunk paths;
// GP/UP: of the packed path.
//
// A workgroup first decodes what it has been given (uniform across the workgroup):
//   tiled region   blockIdx <  nb_tiled : a BlockItem written by the plan.  Long rows are cut
//                  by column class (a contiguous range of column ids) into tiles; block b runs
//                  on XCD b % 8, and the plan gives XCD k the classes of the k-th eighth of the
//                  column range, class after class, so each XCD's L2 only ever holds its own
//                  slices of Y.
//   chunk region   one ChunkDesc per workgroup (long rows that are not tiled)
//   wave region    4 rows, one per wavefront
//   packed region  4*S short rows, one per lane group
//   zero region    rows without stored entries, kZeroRowsPerBlock per workgroup
// and then runs one of four bodies: chunk, wave segments, packed segments, zero fill.  A segment is
// a run of stored entries of one row with a destination (the row of Z, or a partial row).
// ---------------------------------------------------------------------------------------
// E (always `real`) only makes the single- and double-precision instances of one shape different symbols.
// PM: the pattern, with kPatMasked set when the rows are narrower than D (pieces at or beyond a.d_pieces are
// neither loaded nor stored; the run-time-ops and family instances always work that way) or kPatRagged when
// they also end inside a piece.
template <int PM, int D, int GW0, int UW0, int GP0, int UP0, int YF, class E = real>
__global__ __launch_bounds__(kBlockThreads) void fusedmm_fast_kernel(const KernelArgs a) {
  static_assert(sizeof(E) == sizeof(real), "the element type is fixed per translation unit");
  constexpr int P = PM & ~(kPatMasked | kPatRagged);
  using T = PatTraits<P>;
  constexpr int kMask = mask_mode<PM>();
  constexpr bool kMasked = kMask != kMaskNone;
  // Rows of 2-byte elements are read 16 bytes per lane where the lane group can be halved (it must
  // keep 8 lanes): same bytes in flight per wavefront, half as many load instructions.
  constexpr bool kWideW = YF != kYF32 && GW0 >= 16, kWideP = YF != kYF32 && GP0 >= 16;
  constexpr int GW = kWideW ? GW0 / 2 : GW0, UW = kWideW && UW0 > 1 ? UW0 / 2 : UW0, CW = kWideW ? 2 : 1;
  constexpr int GP = kWideP ? GP0 / 2 : GP0, UP = kWideP && UP0 > 1 ? UP0 / 2 : UP0, CP = kWideP ? 2 : 1;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int b = blockIdx.x;
  __shared__ vec4 stage[kWavesPerBlock][D / 4];

  int kind, first, count;
  bool from_desc;  // segments come from descriptors (tiles) rather than from order[] + rowptr[]
  if (b < a.nb_tiled) {
    const BlockItem it = a.items[b];
    kind = it.kind; first = it.first; count = it.count; from_desc = true;
  } else if (b < a.nb_tiled + a.nb_chunk) {
    kind = kItemChunk; first = b - a.nb_tiled; count = 1; from_desc = false;
  } else if (b < a.nb_tiled + a.nb_chunk + a.nb_wave) {
    kind = kItemWave; first = (b - a.nb_tiled - a.nb_chunk) * kWavesPerBlock;
    count = a.n_wave - first < kWavesPerBlock ? a.n_wave - first : kWavesPerBlock; from_desc = false;
  } else if (b < a.nb_tiled + a.nb_chunk + a.nb_wave + a.nb_packed) {
    constexpr int kRows = kWavesPerBlock * (64 / GP);
    kind = kItemPacked; first = (b - a.nb_tiled - a.nb_chunk - a.nb_wave) * kRows;
    count = a.n_packed - first < kRows ? a.n_packed - first : kRows; from_desc = false;
  } else {
    kind = kItemZero; first = (b - a.nb_tiled - a.nb_chunk - a.nb_wave - a.nb_packed) * kZeroRowsPerBlock;
    count = a.n_empty - first < kZeroRowsPerBlock ? a.n_empty - first : kZeroRowsPerBlock; from_desc = false;
  }

  if (kind == kItemChunk) {
    // ---- a workgroup on one run of entries of a long row -------------------------------
    constexpr int V = D / (4 * GW);
    const ChunkDesc ch = from_desc ? a.tile_descs[first] : a.chunks[first];
    const int per = ((ch.e_count + kWavesPerBlock * 64 - 1) / (kWavesPerBlock * 64)) * 64;
    const int lo = wave * per < ch.e_count ? wave * per : ch.e_count;
    const int hi = (wave + 1) * per < ch.e_count ? (wave + 1) * per : ch.e_count;
    const int g = lane % GW;
    vec4 x[V], z[V];
    zero(z);
    if (reads_x<P>(a)) load_x<D, GW, CW, kMask>(a, ch.row, g, x); else zero(x);
    wave_accumulate<PM, D, GW, UW, YF, CW>(a, ch.e_begin + lo, ch.e_begin + hi, x, z, lane);
    if constexpr (T::loads_y) {
      combine_groups<P, GW, V>(a, z);
      if (lane < GW) {
#pragma unroll
        for (int i = 0; i < V; ++i) stage[wave][piece_index<GW, CW>(g, i)] = z[i];
      }
      __syncthreads();
      // a thread per 16-byte piece of the row (two passes at D = 2048, whose rows have 512 pieces)
#pragma unroll
      for (int pc = threadIdx.x; pc < D / 4; pc += kBlockThreads) {
        if (kMasked && pc >= a.d_pieces) break;
        vec4 s = stage[0][pc];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) {
          const vec4 o = stage[w][pc];
          if constexpr (P == PAT_RUNTIME) {
            s.x = aop_apply(a.aop, s.x, o.x); s.y = aop_apply(a.aop, s.y, o.y);
            s.z = aop_apply(a.aop, s.z, o.z); s.w = aop_apply(a.aop, s.w, o.w);
          } else if constexpr (T::aop != FUSEDMM_AOP_SUM) {
            s.x = aop_apply(T::aop, s.x, o.x); s.y = aop_apply(T::aop, s.y, o.y);
            s.z = aop_apply(T::aop, s.z, o.z); s.w = aop_apply(T::aop, s.w, o.w);
          } else {
            s += o;
          }
        }
        if constexpr (T::flips) s *= a.sign;  // a minimum was run as the maximum of the negated messages
        if constexpr (T::means) {
          if (a.mean && ch.part < 0) s *= (real)1 / (real)ch.e_count;  // the chunk is the whole row
        }
        real* dst = ch.part < 0 ? Z_of(a) + (int64_t)ch.row * a.ldz : partials_of(a) + (int64_t)ch.part * D;
        if (kMask != kMaskRagged || pc < a.d_full) st4(dst + 4 * pc, s);
        else st_tail(dst + 4 * pc, s, a.d_tail);
      }
    }
  } else if (kind == kItemWave) {
    // ---- one segment per wavefront -----------------------------------------------------
    constexpr int V = D / (4 * GW);
    if (wave >= count) return;
    int row;
    int64_t e0, e1;
    real* dst;
    if (from_desc) {
      const ChunkDesc td = a.tile_descs[first + wave];
      row = td.row; e0 = td.e_begin; e1 = td.e_begin + td.e_count;
      dst = partials_of(a) + (int64_t)td.part * D;
    } else {
      row = __builtin_amdgcn_readfirstlane(a.order[first + wave]);
      e0 = a.rowptr[row]; e1 = a.rowptr[row + 1];
      dst = Z_of(a) + (int64_t)row * a.ldz;
    }
    const int g = lane % GW;
    vec4 x[V], z[V];
    zero(z);
    if (reads_x<P>(a)) load_x<D, GW, CW, kMask>(a, row, g, x); else zero(x);
    wave_accumulate<PM, D, GW, UW, YF, CW>(a, e0, e1, x, z, lane);
    if constexpr (T::loads_y) {
      combine_groups<P, GW, V>(a, z);
      if constexpr (T::flips) scale(z, a.sign);
      if constexpr (T::means) {
        if (a.mean && !from_desc) scale(z, (real)1 / (real)(e1 - e0));
      }
      if (lane < GW) store_row<D, GW, CW, kMask>(a, dst, g, z);
    }
  } else if (kind == kItemPacked) {
    // ---- one short segment per lane group ----------------------------------------------
    constexpr int V = D / (4 * GP);
    constexpr int S = 64 / GP;
    static_assert(GP % UP == 0, "packed unroll must divide the lane-group size");
    const int slot = lane / GP;
    const int g = lane % GP;
    const bool use_val = reads_values<P>(a);
    int nv = V, lane_tail = 0;
    if constexpr (P == PAT_RUNTIME) {
      nv = 0;
#pragma unroll
      for (int i = 0; i < V; ++i) nv += piece_index<GP, CP>(g, i) < a.d_pieces ? 1 : 0;
      if constexpr (kMask == kMaskRagged) {
        if (a.d_tail > 0 && g == a.d_full % GP) lane_tail = a.d_tail;
      }
    }
    for (int round = 0; round < count; round += kWavesPerBlock * S) {
      const int idx = round + wave * S + slot;
      const bool has_seg = idx < count;
      int64_t row = 0, e0 = 0;
      int deg = 0;
      real* dst = nullptr;
      if (has_seg) {
        if (from_desc) {
          const ChunkDesc td = a.tile_descs[first + idx];
          row = td.row; e0 = td.e_begin; deg = td.e_count;
          dst = partials_of(a) + (int64_t)td.part * D;
        } else {
          row = a.order[a.n_wave + first + idx];
          e0 = a.rowptr[row];
          deg = (int)(a.rowptr[row + 1] - e0);
          dst = Z_of(a) + row * a.ldz;
        }
      }
      vec4 x[V], z[V];
      zero(z);
      zero(x);
      if (reads_x<P>(a)) {
        if (deg > 0) load_x<D, GP, CP, kMask>(a, row, g, x);
      }
      int maxdeg = deg;  // wave-uniform upper bound of the trip count
      if constexpr (GP <= 8) maxdeg = max(maxdeg, __shfl_xor(maxdeg, 8));
      if constexpr (GP <= 16) maxdeg = max(maxdeg, __shfl_xor(maxdeg, 16));
      if constexpr (GP <= 32) maxdeg = max(maxdeg, __shfl_xor(maxdeg, 32));
      maxdeg = __builtin_amdgcn_readfirstlane(maxdeg);
      group_accumulate<PM, D, GP, UP, YF, CP>(a, e0, deg, maxdeg, x, z, slot, g, nv, lane_tail, use_val);
      if constexpr (T::loads_y) {
        if constexpr (T::flips) scale(z, a.sign);
        if constexpr (T::means) {
          if (a.mean && !from_desc && deg > 0) scale(z, (real)1 / (real)deg);
        }
        if (has_seg) store_row<D, GP, CP, kMask>(a, dst, g, z);
      }
    }
  }
  else if (kind == kItemZero) {
    // ---- rows without stored entries: z_u = 0 (Algorithm 1 initialises z_u and adds nothing) ----
    if constexpr (T::loads_y) {
      const int kPieces = kMasked ? a.d_pieces : D / 4;
      const int32_t* rows = a.order + a.n_wave + a.n_packed + first;
      for (int i = threadIdx.x; i < count * kPieces; i += kBlockThreads) {
        const int64_t row = rows[i / kPieces];
        real* dst = Z_of(a) + row * a.ldz + 4 * (i % kPieces);
        if (kMask != kMaskRagged || i % kPieces < a.d_full) st4(dst, vec4{0.f, 0.f, 0.f, 0.f});
        else st_tail(dst, vec4{0.f, 0.f, 0.f, 0.f}, a.d_tail);
      }
    }
  }
  // kind == kItemNone: padding at the end of an XCD's list, nothing to do
}

}  // namespace fmm
