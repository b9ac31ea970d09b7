// Specialised FusedMM kernels for d = 2048 (and, masked, for d = 1537 ... 2047); fp32 storage of Y only.  Application
// patterns: lane groups of 32 lanes (unroll 2) for wave rows, chunks and packed short rows (sixteen 16-byte registers
// per lane and array).  Every other instance (masked and ragged forms, tuple families, run-time ops): 64 lanes
// (unroll 2).  Each set of four tuning values can be overridden on the
// compiler command line when sweeping.
#define FMM_D 2048
#define FMM_NATIVE_Y_ONLY 1
#ifndef FMM_GW
#define FMM_GW 32
#define FMM_UW 2
#define FMM_GP 32
#define FMM_UP 2
#endif
#ifndef FMM_GW_R
#define FMM_GW_R 64
#define FMM_UW_R 2
#define FMM_GP_R 64
#define FMM_UP_R 2
#endif
#include "fusedmm_fast_impl.h"
