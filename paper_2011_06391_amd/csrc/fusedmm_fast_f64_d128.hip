// Specialised FusedMM kernels in double precision for d = 128 (rows of 1024 bytes; a row register is 32 bytes):
// lane groups of 32 lanes (unroll 4) for wave rows and chunks, lane groups of 16 lanes (unroll 2) for
// packed short rows.  The four tuning values can be overridden on the compiler command line when sweeping.
#define FMM_F64 1
#define FMM_D 128
#ifndef FMM_GW
#define FMM_GW 32
#define FMM_UW 4
#define FMM_GP 16
#define FMM_UP 2
#endif
#include "fusedmm_fast_impl.h"
