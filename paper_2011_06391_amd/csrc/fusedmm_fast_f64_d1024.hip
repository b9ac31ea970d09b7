// Specialised FusedMM kernels in double precision for d = 1024 (rows of 8192 bytes; a row register is 32 bytes):
// lane groups of 64 lanes (unroll 2) for wave rows and chunks and for packed short rows.  The four tuning values
// can be overridden on the compiler command line when sweeping.
#define FMM_F64 1
#define FMM_D 1024
#ifndef FMM_GW
#define FMM_GW 64
#define FMM_UW 2
#define FMM_GP 64
#define FMM_UP 2
#endif
#include "fusedmm_fast_impl.h"
