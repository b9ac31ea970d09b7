// Specialised FusedMM kernels for d = 96 (and, masked, for d = 65 ... 95), one of the sizes halfway between two
// powers of two: lane groups of 8 lanes (unroll 4) for wave rows and chunks, of 8 lanes (unroll 4) for packed
// short rows; three 16-byte registers per lane.  The four tuning values can be overridden on the
// compiler command line when sweeping.
#define FMM_D 96
#ifndef FMM_GW
#define FMM_GW 8
#define FMM_UW 4
#define FMM_GP 8
#define FMM_UP 4
#endif
#include "fusedmm_fast_impl.h"
