// Specialised FusedMM kernels for d = 2048 (and, masked, for everything between 1025 and 2047): lane groups of 64
// lanes, eight 16-byte registers per lane for x_u, z_u and the one row of Y in flight.  fp32 storage of Y only.
// The four tuning values can be overridden on the compiler command line when sweeping.
#define FMM_D 2048
#define FMM_NATIVE_Y_ONLY 1
#ifndef FMM_GW
#define FMM_GW 64
#define FMM_UW 1
#define FMM_GP 64
#define FMM_UP 1
#endif
#include "fusedmm_fast_impl.h"
