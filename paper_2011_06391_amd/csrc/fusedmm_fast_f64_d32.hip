// Specialised FusedMM kernels in double precision for d = 32 (rows of 256 bytes; a row register is 32 bytes):
// lane groups of 8 lanes (unroll 4) for wave rows and chunks, lane groups of 8 lanes (unroll 4) for
// packed short rows.  The four tuning values can be overridden on the compiler command line when sweeping.
#define FMM_F64 1
#define FMM_D 32
#ifndef FMM_GW
#define FMM_GW 8
#define FMM_UW 4
#define FMM_GP 8
#define FMM_UP 4
#endif
#include "fusedmm_fast_impl.h"
