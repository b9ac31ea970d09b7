// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fmm {

// Pattern ids of the specialised kernels (host dispatch -> template instance).
// PAT_RUNTIME: the same kernel structure with the five ops read from KernelArgs at run time (any valid tuple).
// PAT_SIGNED_SIGMOID: the sigmoid embedding pattern with the scaling step h = a_uv - sigmoid(s) (kSopValueMinusSigmoid).
// PAT_GCN_MAX / PAT_GCN_MIN: the GCN message (h = a_uv, w = h * y_v) pooled by maximum / minimum instead of
// summed (the pooling variants of Section III-B); mean pooling runs PAT_GCN with the division at the store.
// PAT_DOT / PAT_DIST: two families of tuples with a scalar message, their vector loops fixed at compile time and
// the scalar steps read at run time.  PAT_DOT: VOP = MUL, ROP = RSUM (s = x_u . y_v), any SOP on s, any MOP;
// PAT_DIST: VOP = SUB or ADD, ROP = RSUM, SUMSQ or NORM2, any SOP, any MOP.  The plain ones accumulate by SUM
// (MEAN divides at the store), the _MM ones by MAX or MIN (MIN as the maximum of the negated messages).  They
// also serve the dimensions between two instance sizes for the application patterns they contain.
enum : int { PAT_SIGMOID = 0, PAT_ONE_MINUS_SIGMOID = 1, PAT_GCN = 2, PAT_TDIST = 3, PAT_FR = 4, PAT_VISIT = 5, PAT_RUNTIME = 6,
             PAT_SIGNED_SIGMOID = 7, PAT_GCN_MAX = 8, PAT_GCN_MIN = 9, PAT_DOT = 10, PAT_DOT_MM = 11, PAT_DIST = 12,
             PAT_DIST_MM = 13 };
// pattern | kPatMasked: the instance of that pattern for a dimension between two instance sizes (pieces of a row
// at or beyond KernelArgs::d_pieces are neither loaded nor stored); fp32 / fp64 storage only
constexpr int kPatMasked = 32;
// pattern | kPatRagged: the instance for a dimension that is not a multiple of 4 (the last piece of a row holds
// KernelArgs::d_tail elements, read and written one by one); built for the GCN messages, the tuple families and
// the run-time-ops instance
constexpr int kPatRagged = 64;

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

// What a workgroup of the tiled region does: kind, index of its first descriptor in
// tile_descs[], and how many descriptors (1 for a chunk, <= 4 wave segments, <= 32 packed
// segments).  Items are stored interleaved by XCD: items[j * 8 + k] is the j-th item of XCD k.
enum : int { kItemNone = 0, kItemChunk = 1, kItemWave = 2, kItemPacked = 3, kItemZero = 4 };
// rows without stored entries are only zero-filled: this many per workgroup
constexpr int kZeroRowsPerBlock = 128;
constexpr int kNumXcd = 8;
constexpr int kPackedSegsPerItem = 32;
struct BlockItem {
  int32_t kind;
  int32_t first;
  int32_t count;
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
  // values, X, Z and the partial rows are fp32, or fp64 in the double-precision instances (the kernels read them
  // through typed views); Y likewise, or bfloat16 / half when the launch says so; the leading dimensions count
  // elements of the type in use
  const void* values;
  const void* X;
  const void* Y;
  void* Z;
  int64_t ldx, ldy, ldz;
  float alpha;
  float sign;   // PAT_DOT_MM / PAT_DIST_MM: -1 when the messages are pooled by MIN (run as MAX of the negated messages), else 1
  float ysign;  // PAT_DIST / PAT_DIST_MM: t = x_u + ysign * y_v (-1 for VOP = SUB, 1 for ADD)
  // the families' SOP on the scalar s without a branch: u = sop_exp ? 2^(sop_c1 * s) : s;  h = sop_rcp ? 1 / (1 + u)
  // : sop_lin * s  (sigmoid: c1 = -log2 e; its complement: +log2 e; 1/(1+s): no exponential; SCAL / NOOP: linear)
  float sop_c1, sop_lin;
  int32_t sop_exp, sop_rcp;
  int32_t vop, rop, sop, mop, aop;  // read by the run-time-ops and family instances; aop is SUM, MAX or MIN here
  int32_t mean;                     // PAT_RUNTIME: a row stored whole is divided by its length (mean pooling)
  // Masked instances: the rows have d_pieces 4-element pieces, fewer than D/4 when a dimension below the
  // instance size runs on it (pieces beyond are neither loaded nor stored); the first d_full of them are whole,
  // and when the dimension is not a multiple of 4 the last one holds d_tail (1..3) elements.
  int32_t d_pieces, d_full, d_tail;
  // Ragged instances gather the piece a row of Y ends in with one 16-byte load, which reads up to three elements
  // beyond the row: from this row of Y on that would leave the matrix (the last row, or the last few when ldy < 3),
  // and the load is moved back to end with the row instead.
  int32_t y_first_back_row;
  // schedule: blockIdx ranges, in this order: tiled items, chunks, one row per wavefront from
  // order[0 .. n_wave), packed rows from order[n_wave .. n_wave+n_packed), rows without entries
  // (zero fill only) from order[n_wave+n_packed .. n_wave+n_packed+n_empty).
  const int32_t* order;
  const ChunkDesc* chunks;
  const BlockItem* items;       // tiled region, nb_tiled entries
  const ChunkDesc* tile_descs;  // segments of tiled rows; part is always a partial row
  void* partials;
  uint32_t* visit_counts;
  int32_t n_chunks, n_wave, n_packed, n_empty;
  int32_t nb_tiled, nb_chunk, nb_wave, nb_packed, nb_zero;
};

// Column-class boundaries of the tiled rows.  Row rows[i] is cut into level[i] classes, each
// n_classes / level[i] finest classes wide (finest class k = columns class_start[k] .. class_start[k + 1] - 1,
// class_start holding n_classes + 1 entries on the device); bounds[out_off[i] + c] = offset
// within the row of the first stored entry whose column is in class c or later (c = 0..level[i]).
// unsorted[0] is set if any of those rows has decreasing column indices.
hipError_t launch_tile_bounds(const int64_t* rowptr, const int32_t* colidx, const int32_t* rows, const int32_t* level,
                              const int64_t* out_off, int32_t n_rows, int32_t n_classes, const int32_t* class_start,
                              int32_t* bounds, int32_t* unsorted, hipStream_t stream);

// Rows per workgroup in the packed range for the instance (pattern id, size d, storage format of Y) that
// launch_fast will run (the host needs it for the grid).
int packed_rows_per_block(int pattern, int d, int y_format);

// A scaling step outside the public selector, used by the minibatch layer (the paper's SOP is
// user-definable, Section III-A): h = a_uv - sigmoid(s), which with a_uv = 1 on the stored entries of
// A and a_uv = 0 on negative samples makes attraction and repulsion one FusedMM call.
constexpr int kSopValueMinusSigmoid = 100;


// Storage formats of Y the specialised kernels read (arithmetic is fp32 in the first three).  kYF64 selects
// the double-precision instances: values, X, Y, Z and the partial rows of KernelArgs then all point at doubles
// (the leading dimensions count doubles) and the arithmetic is fp64.
enum : int { kYF32 = 0, kYBf16 = 1, kYF16 = 2, kYF64 = 3 };

// Launch the specialised kernel for (pattern, d).  d must be 32/64/128/256/512/1024.  kYBf16 /
// kYF16: a.Y holds 2-byte elements (every instance except the ragged ones exists in that form).
hipError_t launch_fast(int pattern, int d, int y_format, const KernelArgs& a, hipStream_t stream);

// The kernels for very short feature vectors (one lane per stored entry): d must be 2, 3, 4, 8 or 16, fp32,
// rows of any 4-byte aligned pitch.  Same plan, descriptors and block ranges as launch_fast (the packed range is
// cut into small_packed_rows_per_block(d) rows per workgroup); partial rows are kSmallPartialStride floats apart.
constexpr int kSmallPartialStride = 16;
inline bool is_small_dim(int d) { return d == 2 || d == 3 || d == 4 || d == 8 || d == 16; }
int small_packed_rows_per_block(int d);
hipError_t launch_small(int pattern, int d, const KernelArgs& a, hipStream_t stream);
hipError_t launch_small_merge(const MergeDesc* merges, int32_t n_merges, const float* partials, int32_t d, int32_t aop,
                              const int64_t* rowptr, float* Z, int64_t ldz, hipStream_t stream);

// dst[i] = bfloat16(src[i]), round to nearest even; NaN stays NaN.
hipError_t launch_to_bf16(uint16_t* dst, const float* src, size_t count, hipStream_t stream);
// dst[i] = half(src[i]), round to nearest even.
hipError_t launch_to_f16(uint16_t* dst, const float* src, size_t count, hipStream_t stream);

// General kernel: any 1 <= d <= 2048, any op tuple, any alignment.  One wavefront per row of up to
// kGenericSplit stored entries; longer rows are cut into segments of that length, one wavefront each,
// whose partial rows a second kernel combines in segment order (so a hub row does not serialise it).
// T = float, or double (storage and arithmetic both in T).
constexpr int kGenericSplit = 256;
template <class T>
struct GenericArgsT {
  const int64_t* rowptr;
  const int32_t* colidx;
  const T* values;
  const T* X;
  const T* Y;
  T* Z;
  int64_t ldx, ldy, ldz;
  int64_t m;
  int32_t d;
  int32_t vop, rop, sop, mop, aop;
  T alpha;
  uint32_t* visit_counts;  // non-null: count visits instead of computing
  const ChunkDesc* segs;   // segments of the rows longer than kGenericSplit; part = partial-row slot
  int32_t n_segs;
  const MergeDesc* merges;  // one per such row
  int32_t n_merges;
  T* partials;              // n_segs rows of d elements
};
using GenericArgs = GenericArgsT<float>;
hipError_t launch_generic(const GenericArgsT<float>& a, hipStream_t stream);
hipError_t launch_generic(const GenericArgsT<double>& a, hipStream_t stream);

// aop: FUSEDMM_AOP_SUM / MAX / MIN, how partial rows are combined; FUSEDMM_AOP_MEAN: summed, then
// divided by the row's length taken from rowptr
// d: row width; pstride: distance in floats between partial rows (>= d)
hipError_t launch_merge(const MergeDesc* merges, int32_t n_merges, const float* partials, int32_t d, int32_t pstride,
                        int32_t aop, const int64_t* rowptr, float* Z, int64_t ldz, hipStream_t stream);
hipError_t launch_merge(const MergeDesc* merges, int32_t n_merges, const double* partials, int32_t d, int32_t pstride,
                        int32_t aop, const int64_t* rowptr, double* Z, int64_t ldz, hipStream_t stream);

// Where the stored entries lie along the column range: hist[column * n_buckets / n] += 1 for every stride-th entry.
hipError_t launch_column_histogram(const int32_t* colidx, int64_t nnz, int64_t stride, int64_t n, int32_t n_buckets,
                                   uint32_t* hist, hipStream_t stream);

// flag[0] |= 1 if any colidx entry is outside [0, n).
hipError_t launch_validate_colidx(const int32_t* colidx, int64_t nnz, int64_t n, int32_t* flag, hipStream_t stream);

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);

}  // namespace fmm

// fusedmm_execute for callers inside the library: also accepts fmm::kSopValueMinusSigmoid (needs d_values).
struct fusedmm_plan;
struct fusedmm_ops;
__attribute__((visibility("hidden"))) int fusedmm_execute_private_ops(fusedmm_plan* plan, const fusedmm_ops* ops,
                                                                      int32_t d, const float* d_values, const float* d_X,
                                                                      int64_t ldx, const float* d_Y, int64_t ldy,
                                                                      float* d_Z, int64_t ldz, void* stream);
