// Specialised FusedMM kernels for d = 1024 (and, masked, for d = 769 ... 1023).  Application patterns: lane groups
// of 32 lanes (unroll 4) for wave rows and chunks, of 16 lanes (one row in flight) for packed short rows.
// Every other instance (masked and ragged forms, tuple families, run-time ops) and rows of 2-byte elements: 64 lanes
// (unroll 2) for both.  Each set of four tuning values can be overridden on the
// compiler command line when sweeping.
#define FMM_D 1024
#ifndef FMM_GW
#define FMM_GW 32
#define FMM_UW 4
#define FMM_GP 16
#define FMM_UP 1
#endif
#ifndef FMM_GW_R
#define FMM_GW_R 64
#define FMM_UW_R 2
#define FMM_GP_R 64
#define FMM_UP_R 2
#endif
#include "fusedmm_fast_impl.h"
