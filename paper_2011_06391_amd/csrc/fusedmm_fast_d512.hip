// Specialised FusedMM kernels for d = 512: lane groups of 64 lanes (unroll 4) for wave rows and
// chunks, lane groups of 32 lanes (unroll 2) for packed short rows.  The four tuning
// values can be overridden on the compiler command line when sweeping.
#define FMM_D 512
#ifndef FMM_GW
#define FMM_GW 64
#define FMM_UW 4
#define FMM_GP 32
#define FMM_UP 2
#endif
#include "fusedmm_fast_impl.h"
