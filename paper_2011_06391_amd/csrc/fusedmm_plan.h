// The plan object behind fusedmm_plan_t, shared by the translation unit that builds it (fusedmm_plan.hip)
// and the one that runs it (fusedmm_api.hip).  Host code only.
#pragma once

#include "../../include/fusedmm.h"
#include "fusedmm_internal.h"

#include <vector>

struct fusedmm_plan {
  int64_t m = 0, n = 0, nnz = 0;
  const int64_t* d_rowptr = nullptr;
  const int32_t* d_colidx = nullptr;
  int32_t small_row_max = 0, split_row_min = 0, chunk_edges = 0, tile_row_min = 0;  // as resolved
  int32_t n_wave = 0, n_packed = 0, n_empty = 0, n_chunks = 0, n_merges = 0, n_parts = 0;  // n_packed: non-empty
  int32_t n_items = 0, n_tile_descs = 0, n_tiled_rows = 0, n_classes = 1;
  bool general_only = false;  // every execute runs the general kernel
  int32_t* d_order = nullptr;
  fmm::ChunkDesc* d_chunks = nullptr;
  fmm::BlockItem* d_items = nullptr;
  fmm::ChunkDesc* d_tile_descs = nullptr;
  fmm::MergeDesc* d_merges = nullptr;
  float* d_partials = nullptr;
  int32_t partials_d = 0;  // scratch holds n_parts rows of this many floats
  // the general kernel's own cut of the rows longer than kGenericSplit (any d, fp32 or fp64)
  fmm::ChunkDesc* d_gen_segs = nullptr;
  fmm::MergeDesc* d_gen_merges = nullptr;
  int32_t n_gen_segs = 0, n_gen_merges = 0;
  void* d_gen_partials = nullptr;
  size_t gen_partials_bytes = 0;
  bool profiling = false;
  struct EventTriple { hipEvent_t before, after, after2; };
  std::vector<EventTriple> events;  // main kernel between before/after; nothing between after/after2
  size_t events_used = 0;
};

namespace fmm {

// Frees everything the plan holds on the device (lists, scratch, profiling events); the object itself stays.
void free_plan_device(fusedmm_plan* p);

// The address, on the current device, of the fixed scratch of fusedmm_execute_static_scratch (every GPU holds
// its own copy at its own address; looked up once per device).
int static_scratch_for_current_device(void** out);

}  // namespace fmm
