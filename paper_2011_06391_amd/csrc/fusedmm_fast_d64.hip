// Specialised FusedMM kernels for d = 64: lane groups of 16 lanes (unroll 8) for wave rows and
// chunks, lane groups of 8 lanes (unroll 4) for packed short rows.
#define FMM_D 64
#define FMM_GW 16
#define FMM_UW 8
#define FMM_GP 8
#define FMM_UP 4
#include "fusedmm_fast_impl.h"
