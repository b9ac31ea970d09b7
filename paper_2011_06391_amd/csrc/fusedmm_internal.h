// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmm {

// Pattern ids of the specialised kernels (host dispatch -> template instance).
enum : int { PAT_SIGMOID = 0, PAT_ONE_MINUS_SIGMOID = 1, PAT_GCN = 2, PAT_TDIST = 3, PAT_FR = 4, PAT_VISIT = 5 };

constexpr int kWavesPerBlock = 4;
constexpr int kBlockThreads = 64 * kWavesPerBlock;

// One workgroup's share of a long row.  part < 0: the chunk is the whole row and
// the workgroup stores z_u itself; otherwise it stores partial row `part`.
struct ChunkDesc {
  int64_t e_begin;
  int32_t e_count;
  int32_t row;
  int32_t part;
  int32_t pad;
};

// A row split over several chunks: z_u = partial[first] + ... + partial[first+count-1].
struct MergeDesc {
  int32_t row;
  int32_t first_part;
  int32_t n_parts;
  int32_t pad;
};

struct KernelArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* values;
  const float* X;
  const float* Y;
  float* Z;
  int64_t ldx, ldy, ldz;
  float alpha;
  // schedule: blockIdx in [0, nb_chunk) -> chunks; [nb_chunk, nb_chunk+nb_wave) -> one row
  // per wavefront from order[0 .. n_wave); then packed rows from order[n_wave .. n_wave+n_packed).
  const int32_t* order;
  const ChunkDesc* chunks;
  float* partials;
  uint32_t* visit_counts;
  int32_t n_chunks, n_wave, n_packed;
  int32_t nb_chunk, nb_wave, nb_packed;
};

// Rows per workgroup in the packed range for dimension d (host needs it for the grid).
int packed_rows_per_block(int d);

// Launch the specialised kernel for (pattern, d).  d must be 32/64/128/256/512.
hipError_t launch_fast(int pattern, int d, const KernelArgs& a, hipStream_t stream);

// General kernel: any 1 <= d <= 2048, any op tuple, any alignment; one wavefront per row.
struct GenericArgs {
  const int64_t* rowptr;
  const int32_t* colidx;
  const float* values;
  const float* X;
  const float* Y;
  float* Z;
  int64_t ldx, ldy, ldz;
  int64_t m;
  int32_t d;
  int32_t vop, rop, sop, mop;
  float alpha;
  uint32_t* visit_counts;  // non-null: count visits instead of computing
};
hipError_t launch_generic(const GenericArgs& a, hipStream_t stream);

hipError_t launch_merge(const MergeDesc* merges, int32_t n_merges, const float* partials, int32_t d,
                        float* Z, int64_t ldz, hipStream_t stream);

// flag[0] |= 1 if any colidx entry is outside [0, n).
hipError_t launch_validate_colidx(const int32_t* colidx, int64_t nnz, int64_t n, int32_t* flag, hipStream_t stream);

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);

}  // namespace fmm
