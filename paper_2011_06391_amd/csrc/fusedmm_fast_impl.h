// Instantiates the specialised kernel for one feature dimension and defines its launcher.
// Included by fusedmm_fast_d*.hip with FMM_D / FMM_GW / FMM_UW / FMM_GP / FMM_UP set.
#include "fusedmm_device.h"

namespace fmm {

#define FMM_CAT2(a, b) a##b
#define FMM_CAT(a, b) FMM_CAT2(a, b)

template <int P, bool YB>
static hipError_t launch_one(const KernelArgs& a, hipStream_t stream) {
  const int64_t blocks = (int64_t)a.nb_tiled + a.nb_chunk + a.nb_wave + a.nb_packed;
  if (blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL((fusedmm_fast_kernel<P, FMM_D, FMM_GW, FMM_UW, FMM_GP, FMM_UP, YB>), dim3((unsigned)blocks),
                     dim3(kBlockThreads), 0, stream, a);
  return hipGetLastError();
}

int FMM_CAT(packed_rows_per_block_d, FMM_D)() { return kWavesPerBlock * (64 / FMM_GP); }

hipError_t FMM_CAT(launch_fast_d, FMM_D)(int pattern, bool y_bf16, const KernelArgs& a, hipStream_t stream) {
  if (y_bf16) {
    switch (pattern) {
      case PAT_SIGMOID: return launch_one<PAT_SIGMOID, true>(a, stream);
      case PAT_ONE_MINUS_SIGMOID: return launch_one<PAT_ONE_MINUS_SIGMOID, true>(a, stream);
      case PAT_GCN: return launch_one<PAT_GCN, true>(a, stream);
      case PAT_TDIST: return launch_one<PAT_TDIST, true>(a, stream);
      case PAT_FR: return launch_one<PAT_FR, true>(a, stream);
      case PAT_RUNTIME: return launch_one<PAT_RUNTIME, true>(a, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (pattern) {
    case PAT_SIGMOID: return launch_one<PAT_SIGMOID, false>(a, stream);
    case PAT_ONE_MINUS_SIGMOID: return launch_one<PAT_ONE_MINUS_SIGMOID, false>(a, stream);
    case PAT_GCN: return launch_one<PAT_GCN, false>(a, stream);
    case PAT_TDIST: return launch_one<PAT_TDIST, false>(a, stream);
    case PAT_FR: return launch_one<PAT_FR, false>(a, stream);
    case PAT_VISIT: return launch_one<PAT_VISIT, false>(a, stream);
    case PAT_RUNTIME: return launch_one<PAT_RUNTIME, false>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace fmm
