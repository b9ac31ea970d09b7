// Specialised FusedMM kernels for d = 192 (and, masked, for d = 129 ... 191), one of the sizes halfway between two
// powers of two: lane groups of 16 lanes (unroll 4) for wave rows and chunks, of 16 lanes (unroll 4) for packed
// short rows; three 16-byte registers per lane.  The four tuning values can be overridden on the
// compiler command line when sweeping.
#define FMM_D 192
#ifndef FMM_GW
#define FMM_GW 16
#define FMM_UW 4
#define FMM_GP 16
#define FMM_UP 4
#endif
#include "fusedmm_fast_impl.h"
