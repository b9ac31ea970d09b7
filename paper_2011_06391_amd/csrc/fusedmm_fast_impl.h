// Instantiates the specialised kernel for one feature dimension and defines its launcher.
// Included by fusedmm_fast_d*.hip with FMM_D / FMM_GW / FMM_UW / FMM_GP / FMM_UP set, and by
// fusedmm_fast_f64_d*.hip with FMM_F64 as well (double precision: launch_fast_f64_d<D>).
#include "fusedmm_device.h"

namespace fmm {

#define FMM_CAT2(a, b) a##b
#define FMM_CAT(a, b) FMM_CAT2(a, b)
#ifdef FMM_F64
#define FMM_FN(name) FMM_CAT(FMM_CAT(name, _f64_d), FMM_D)
constexpr bool kDouble = true;
#else
#define FMM_FN(name) FMM_CAT(FMM_CAT(name, _d), FMM_D)
constexpr bool kDouble = false;
#endif
// sizes that exist for Y in the build's own element type only (no bfloat16 / half storage): double precision,
// and the largest fp32 size
#if defined(FMM_F64) || defined(FMM_NATIVE_Y_ONLY)
constexpr bool kNativeYOnly = true;
#else
constexpr bool kNativeYOnly = false;
#endif

// Three sets of lane groups and unrolls per size (the last two default to the first):
//   FMM_GW / UW / GP / UP           the application patterns at the size itself: the values a sweep found fastest
//   FMM_GW_R / UW_R / GP_R / UP_R   every other instance -- masked and ragged forms, the tuple families, run-time
//                                   ops.  They need more registers per lane or test a mask per register: at the
//                                   large sizes the narrow lane groups that suit the plain patterns leave the
//                                   ragged forms one wavefront per SIMD (d = 1433 on 32-lane groups: 3.4 ms
//                                   against 1.6 ms on 64) and make the masked ones slower than the full size
//   FMM_GW_2B / ...                 rows of 2-byte elements (the kernel halves the groups where that leaves 8
//                                   lanes, to read 16 bytes per lane)
#ifndef FMM_GW_R
#define FMM_GW_R FMM_GW
#define FMM_UW_R FMM_UW
#define FMM_GP_R FMM_GP
#define FMM_UP_R FMM_UP
#endif
#ifndef FMM_GW_2B
#define FMM_GW_2B FMM_GW_R
#define FMM_UW_2B FMM_UW_R
#define FMM_GP_2B FMM_GP_R
#define FMM_UP_2B FMM_UP_R
#endif

// whether an instance takes the second set
constexpr bool register_heavy(int pm) {
  const int p = pm & ~(kPatMasked | kPatRagged);
  return (pm & (kPatRagged | kPatMasked)) != 0 || p == PAT_RUNTIME || p == PAT_DOT || p == PAT_DOT_MM || p == PAT_DIST || p == PAT_DIST_MM;
}

template <int P, int YF>
static hipError_t launch_one(const KernelArgs& a, hipStream_t stream) {
  const int64_t blocks = (int64_t)a.nb_tiled + a.nb_chunk + a.nb_wave + a.nb_packed + a.nb_zero;
  if (blocks <= 0) return hipSuccess;
  if constexpr (YF != kYF32) {
    hipLaunchKernelGGL((fusedmm_fast_kernel<P, FMM_D, FMM_GW_2B, FMM_UW_2B, FMM_GP_2B, FMM_UP_2B, YF>), dim3((unsigned)blocks),
                       dim3(kBlockThreads), 0, stream, a);
  } else if constexpr (register_heavy(P)) {
    hipLaunchKernelGGL((fusedmm_fast_kernel<P, FMM_D, FMM_GW_R, FMM_UW_R, FMM_GP_R, FMM_UP_R, YF>), dim3((unsigned)blocks),
                       dim3(kBlockThreads), 0, stream, a);
  } else {
    hipLaunchKernelGGL((fusedmm_fast_kernel<P, FMM_D, FMM_GW, FMM_UW, FMM_GP, FMM_UP, YF>), dim3((unsigned)blocks),
                       dim3(kBlockThreads), 0, stream, a);
  }
  return hipGetLastError();
}

// rows per workgroup of the packed region: 4 wavefronts of 64 / GP rows, GP as launch_one chooses it
int FMM_FN(packed_rows_per_block)(int pattern, int y_format) {
  int gp = FMM_GP;
  if (y_format != kYF32) gp = FMM_GP_2B >= 16 ? FMM_GP_2B / 2 : FMM_GP_2B;
  else if (register_heavy(pattern)) gp = FMM_GP_R;
  return kWavesPerBlock * (64 / gp);
}

// the instance for rows narrower than FMM_D (whole 4-element pieces; rows of 2-byte elements: whole 16-byte
// chunks of 8), for the patterns that do not mask by themselves
template <int P, int YF>
static hipError_t launch_masked(const KernelArgs& a, hipStream_t stream) {
  return launch_one<P | kPatMasked, YF>(a, stream);
}

template <int YF>
static hipError_t launch_format(int pattern, const KernelArgs& a, hipStream_t stream) {
  if ((pattern & kPatRagged) != 0) {  // rows that end inside a 16-byte piece: fp32 / fp64 storage only
    if constexpr (YF == kYF32) {
      switch (pattern & ~kPatRagged) {
        case PAT_RUNTIME: return launch_one<PAT_RUNTIME | kPatRagged, kYF32>(a, stream);
        case PAT_DOT: return launch_one<PAT_DOT | kPatRagged, kYF32>(a, stream);
        case PAT_DOT_MM: return launch_one<PAT_DOT_MM | kPatRagged, kYF32>(a, stream);
        case PAT_DIST: return launch_one<PAT_DIST | kPatRagged, kYF32>(a, stream);
        case PAT_DIST_MM: return launch_one<PAT_DIST_MM | kPatRagged, kYF32>(a, stream);
        case PAT_GCN: return launch_one<PAT_GCN | kPatRagged, kYF32>(a, stream);
        case PAT_GCN_MAX: return launch_one<PAT_GCN_MAX | kPatRagged, kYF32>(a, stream);
        case PAT_GCN_MIN: return launch_one<PAT_GCN_MIN | kPatRagged, kYF32>(a, stream);
        case PAT_VISIT: return launch_one<PAT_VISIT | kPatRagged, kYF32>(a, stream);  // the edge-visit hook on these lane groups
        default: return hipErrorInvalidValue;
      }
    }
    return hipErrorInvalidValue;
  }
  const bool m = (pattern & kPatMasked) != 0;
  switch (pattern & ~kPatMasked) {
    case PAT_SIGMOID: return m ? launch_masked<PAT_SIGMOID, YF>(a, stream) : launch_one<PAT_SIGMOID, YF>(a, stream);
    case PAT_ONE_MINUS_SIGMOID:
      return m ? launch_masked<PAT_ONE_MINUS_SIGMOID, YF>(a, stream) : launch_one<PAT_ONE_MINUS_SIGMOID, YF>(a, stream);
    case PAT_GCN: return m ? launch_masked<PAT_GCN, YF>(a, stream) : launch_one<PAT_GCN, YF>(a, stream);
    case PAT_GCN_MAX: return m ? launch_masked<PAT_GCN_MAX, YF>(a, stream) : launch_one<PAT_GCN_MAX, YF>(a, stream);
    case PAT_GCN_MIN: return m ? launch_masked<PAT_GCN_MIN, YF>(a, stream) : launch_one<PAT_GCN_MIN, YF>(a, stream);
    case PAT_TDIST: return m ? launch_masked<PAT_TDIST, YF>(a, stream) : launch_one<PAT_TDIST, YF>(a, stream);
    case PAT_FR: return m ? launch_masked<PAT_FR, YF>(a, stream) : launch_one<PAT_FR, YF>(a, stream);
    case PAT_RUNTIME: return launch_one<PAT_RUNTIME, YF>(a, stream);
    case PAT_DOT: return launch_one<PAT_DOT, YF>(a, stream);
    case PAT_DOT_MM: return launch_one<PAT_DOT_MM, YF>(a, stream);
    case PAT_DIST: return launch_one<PAT_DIST, YF>(a, stream);
    case PAT_DIST_MM: return launch_one<PAT_DIST_MM, YF>(a, stream);
    case PAT_VISIT:  // the edge-visit instance reads no Y: one form is enough
      if constexpr (YF == kYF32) return launch_one<PAT_VISIT, kYF32>(a, stream);
      return hipErrorInvalidValue;
    case PAT_SIGNED_SIGMOID:  // used by the minibatch layer on fp32 embeddings only
      if constexpr (YF == kYF32 && !kDouble)
        return m ? launch_masked<PAT_SIGNED_SIGMOID, kYF32>(a, stream) : launch_one<PAT_SIGNED_SIGMOID, kYF32>(a, stream);
      return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
  }
}

// y_format kYF32 stands for "Y in the element type of the build"; the 2-byte formats exist for fp32 arithmetic only
hipError_t FMM_FN(launch_fast)(int pattern, int y_format, const KernelArgs& a, hipStream_t stream) {
  if constexpr (kNativeYOnly) {
    return y_format == kYF32 ? launch_format<kYF32>(pattern, a, stream) : hipErrorInvalidValue;
  } else {
    switch (y_format) {
      case kYF32: return launch_format<kYF32>(pattern, a, stream);
      case kYBf16: return launch_format<kYBf16>(pattern, a, stream);
      case kYF16: return launch_format<kYF16>(pattern, a, stream);
      default: return hipErrorInvalidValue;
    }
  }
}

}  // namespace fmm
