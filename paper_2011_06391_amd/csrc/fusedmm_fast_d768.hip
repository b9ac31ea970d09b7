// Specialised FusedMM kernels for d = 768 (and, masked, for d = 513 ... 767), one of the sizes halfway between two
// powers of two.  Application patterns: lane groups of 32 lanes (unroll 4) for wave rows and chunks, of 16 lanes
// (unroll 2) for packed short rows.  Every other instance (masked and ragged forms, tuple families, run-time ops):
// 64 lanes (unroll 4) for both.  Rows of 2-byte elements: 64 lanes (unroll 4) and 32 lanes (unroll 2), which the
// kernel halves.  Each set of four tuning values can be overridden on the compiler command line when sweeping.
#define FMM_D 768
#ifndef FMM_GW
#define FMM_GW 32
#define FMM_UW 4
#define FMM_GP 16
#define FMM_UP 2
#endif
#ifndef FMM_GW_R
#define FMM_GW_R 64
#define FMM_UW_R 4
#define FMM_GP_R 64
#define FMM_UP_R 4
#endif
#define FMM_GW_2B 64
#define FMM_UW_2B 4
#define FMM_GP_2B 32
#define FMM_UP_2B 2
#include "fusedmm_fast_impl.h"
