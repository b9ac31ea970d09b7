// Specialised FusedMM kernels for d = 384 (and, masked, for d = 257 ... 383), one of the sizes halfway between two
// powers of two: lane groups of 32 lanes (unroll 4) for wave rows and chunks, of 16 lanes (unroll 4) for packed
// short rows; three and six 16-byte registers per lane.  The four tuning values can be overridden on the
// compiler command line when sweeping.
#define FMM_D 384
#ifndef FMM_GW
#define FMM_GW 32
#define FMM_UW 4
#define FMM_GP 16
#define FMM_UP 4
#endif
// every other instance (masked and ragged forms, tuple families, run-time ops): 32-lane groups for the packed rows too
#ifndef FMM_GW_R
#define FMM_GW_R 32
#define FMM_UW_R 4
#define FMM_GP_R 32
#define FMM_UP_R 4
#endif
#include "fusedmm_fast_impl.h"
