// Specialised FusedMM kernels in double precision for d = 2048 (rows of 16384 bytes; a row register is 32 bytes):
// lane groups of 64 lanes (unroll 1) for wave rows and chunks and for packed short rows.  The four tuning values
// can be overridden on the compiler command line when sweeping.
#define FMM_F64 1
#define FMM_D 2048
#ifndef FMM_GW
#define FMM_GW 64
#define FMM_UW 1
#define FMM_GP 64
#define FMM_UP 1
#endif
#include "fusedmm_fast_impl.h"
