/*
 * fusedmm.h -- C ABI of libfusedmm.so: the fused SDDMM-SpMM kernel (FusedMM,
 * arXiv 2011.06391) for AMD MI355X (gfx950), hand-written HIP.
 *
 *     Z = FusedMM(A, X, Y)                                  (paper Section II)
 *     z_u = AOP_{v in N(u)} MOP( SOP( ROP( VOP(x_u, y_v) ) ), . )   (Eq. 1,
 *           Section III-A steps 1-5, Algorithm 1 procedure UpdateU)
 *
 * A is an m x n sparse matrix in CSR, X is m x d, Y is n x d, Z is m x d, all
 * dense matrices row-major fp32 (Table I; Section V-A: single precision).
 * No edge message is ever written to memory (Section II, "the need for a fused
 * kernel"); the library's workspace is O(m + nnz/chunk + splits*d).
 *
 * Conventions
 *   - All array arguments named d_* are DEVICE pointers (HIP global memory of
 *     the current device).  Everything else is a host value or host pointer.
 *   - 0-based indices.  rowptr: int64, m+1 entries, rowptr[0] == 0,
 *     rowptr[m] == nnz, non-decreasing.  colidx: int32, nnz entries, each in
 *     [0, n); order within a row is free; duplicates and self-loops are
 *     processed as stored (every stored entry is visited exactly once).
 *   - Leading dimensions (ldx, ldy, ldz) are in ELEMENTS, >= d.
 *   - d_Y == d_X is allowed.  Z must not overlap X or Y (rows of Y are read by
 *     other rows' gathers while Z is written).
 *   - m == 0 and nnz == 0 are valid.  Rows without stored entries get z_u = 0
 *     (Algorithm 1 initialises z_u to zero); Z is always overwritten.
 *   - Ownership: the caller owns every buffer it passes and must keep
 *     d_rowptr / d_colidx alive and unchanged for the life of the plan (the
 *     plan borrows them).  The plan owns its schedule lists and scratch.
 *   - Errors: every call returns a fusedmm_status.  No exceptions, no abort.
 *     Arguments are validated before anything is launched: on every status except
 *     FUSEDMM_ERR_HIP no output has been written by that call.  FUSEDMM_ERR_HIP reports a
 *     failed launch; kernels of the same call launched before it may already have written Z.
 *   - The execute entry points are asynchronous and neither allocate nor synchronise: the
 *     scratch they need (partial rows of split rows) is reserved by fusedmm_plan_create for
 *     the hinted dimension and by fusedmm_plan_reserve / fusedmm_plan_reserve_f64 beyond it;
 *     a call that would need more returns FUSEDMM_ERR_NOT_RESERVED.
 *   - Threading: calls on one plan must not overlap in time (they share the
 *     plan's scratch).  Different plans are independent.
 *   - stream arguments are hipStream_t handles passed as void* (NULL = the
 *     null stream).
 */
#ifndef FUSEDMM_H_
#define FUSEDMM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FUSEDMM_VERSION 100 /* 0.1.0 */

/* Largest feature dimension accepted.  d in {32, 64, 128, 256, 512} (the
 * paper's sweep, Table VI), 1024, 2048 and the sizes halfway between them
 * (96, 192, ... 1536) run the specialised kernels, every other d the same
 * schedule on the next larger of them, d = 2, 3, 4, 8, 16 kernels of their
 * own (see fusedmm_ops_t below).  Rows of X, Y and Z may start at any
 * element: no alignment beyond that of a float is asked of the fp32 entry
 * points (aligned rows are read fastest: a row that straddles cache lines
 * costs up to a quarter more). */
#define FUSEDMM_MAX_D 2048

typedef enum fusedmm_status {
  FUSEDMM_OK = 0,
  FUSEDMM_ERR_INVALID_ARG = 1,     /* null pointer, negative size, ld < d, bad rowptr/colidx, missing values */
  FUSEDMM_ERR_UNSUPPORTED_OPS = 2, /* op tuple outside the supported set */
  FUSEDMM_ERR_UNSUPPORTED_DIM = 3, /* d < 1 or d > FUSEDMM_MAX_D */
  FUSEDMM_ERR_ALIAS = 4,           /* Z overlaps X or Y */
  FUSEDMM_ERR_ALLOC = 5,           /* host or device allocation failed */
  FUSEDMM_ERR_HIP = 6,             /* a HIP runtime call failed */
  FUSEDMM_ERR_NOT_RESERVED = 7,    /* the plan's scratch was not reserved for this dimension (fusedmm_plan_reserve) */
  FUSEDMM_ERR_SCRATCH_LIMIT = 8    /* fusedmm_execute_static_scratch: the call needs more than FUSEDMM_STATIC_SCRATCH_BYTES */
} fusedmm_status;

/* Step 1, VOP(x_u, y_v) -> t (Section III-A step 1; Table II binary ops). */
typedef enum { FUSEDMM_VOP_MUL = 0, FUSEDMM_VOP_SEL2ND = 1, FUSEDMM_VOP_SUB = 2, FUSEDMM_VOP_ADD = 3 } fusedmm_vop;
/* Step 2, ROP(t) -> s (step 2; Table II reductions; NORM of Table III).  RMUL: product of the elements. */
typedef enum {
  FUSEDMM_ROP_NOOP = 0, FUSEDMM_ROP_RSUM = 1, FUSEDMM_ROP_SUMSQ = 2, FUSEDMM_ROP_NORM2 = 3, FUSEDMM_ROP_RMUL = 4
} fusedmm_rop;
/* Step 3, SOP -> h (step 3).  EDGE_VALUE: h = a_uv (the GCN row of Table III).  After a reduction
 * SOP acts on the scalar s; when ROP is NOOP (and SOP is not EDGE_VALUE) it acts on every element
 * of t and the message h is a vector (Algorithm 1, SOP step: without a reduction the VOP output is
 * what SOP takes). */
typedef enum {
  FUSEDMM_SOP_EDGE_VALUE = 0,
  FUSEDMM_SOP_SIGMOID = 1,           /* 1/(1+exp(-s)) */
  FUSEDMM_SOP_ONE_MINUS_SIGMOID = 2, /* 1 - sigmoid(s), evaluated as sigmoid(-s) = 1/(1+exp(s)): no cancellation for large s */
  FUSEDMM_SOP_INV_1P = 3,            /* 1/(1+s) */
  FUSEDMM_SOP_SCAL = 4,              /* alpha * s */
  FUSEDMM_SOP_NOOP = 5               /* h = s (or h = t) */
} fusedmm_sop;
/* Step 4, MOP(h, .) -> w (step 4): h (.) y_v, h (.) t with t the VOP output, or y_v itself (SEL2ND). */
typedef enum { FUSEDMM_MOP_MUL_Y = 0, FUSEDMM_MOP_MUL_T = 1, FUSEDMM_MOP_SEL2ND = 2 } fusedmm_mop;
/* Step 5, AOP(z_u, w) (step 5; Table II ASUM, AMAX).  z_u starts at 0 (Algorithm 1), so MAX yields
 * max(0, max_v w) and MIN yields min(0, min_v w); rows without entries give 0.  MEAN (the mean
 * pooling of Section III-B's GCN variants) is the SUM divided by the row's number of stored entries. */
typedef enum { FUSEDMM_AOP_SUM = 0, FUSEDMM_AOP_MAX = 1, FUSEDMM_AOP_MIN = 2, FUSEDMM_AOP_MEAN = 3 } fusedmm_aop;

/* The op selector.  Every combination of the values above is valid except that
 * SOP == EDGE_VALUE requires ROP == NOOP (the message is the stored edge value; nothing to reduce).
 * X is read iff VOP != SEL2ND; d_values is read iff SOP == EDGE_VALUE.
 * The five application patterns below, and the GCN pattern with MAX, MIN or MEAN pooling instead of
 * the sum, run kernels of their own when d is 32, 64, 96, 128, 192, ... 1536 or 2048, and masked forms of them
 * (on the next larger size, skipping what lies beyond d) at the other multiples of 4; tuples with a
 * scalar message from a dot product or from the sum / difference of the operands run two families of
 * kernels with their vector loops fixed; every other tuple runs the same schedule with the ops read at
 * run time.  A d that is not a multiple of 4 runs the families, the GCN kernels or the
 * run-time-ops kernel in a form that masks down to the element.  A plan created with general_kernel_only
 * runs the general kernel instead (one wavefront per row or per 256-entry segment of a long row: a
 * correctness path, an order of magnitude slower). */
typedef struct fusedmm_ops {
  int32_t vop, rop, sop, mop, aop;
  float alpha; /* used by FUSEDMM_SOP_SCAL only */
} fusedmm_ops_t;

/* Application patterns (Table III rows 1-3 and the t-distribution pattern). */
typedef enum {
  FUSEDMM_PATTERN_SIGMOID_EMBED = 0,           /* MUL, RSUM, SIGMOID, MUL_Y, SUM */
  FUSEDMM_PATTERN_ONE_MINUS_SIGMOID_EMBED = 1, /* MUL, RSUM, 1-SIGMOID, MUL_Y, SUM */
  FUSEDMM_PATTERN_GCN_SUM = 2,                 /* SEL2ND, NOOP, EDGE_VALUE, MUL_Y, SUM  (= SpMM) */
  FUSEDMM_PATTERN_TDIST = 3,                   /* SUB, SUMSQ, INV_1P, MUL_T, SUM */
  FUSEDMM_PATTERN_FR = 4                       /* SUB, NORM2, SCAL(alpha), MUL_T, SUM */
} fusedmm_pattern;

/* Scheduling knobs of the degree-binned plan (the GPU counterpart of the
 * nnz-balanced 1-D partition, Section III-C).  Zero fields take defaults. */
typedef struct fusedmm_plan_options {
  int32_t small_row_max;   /* rows with <= this many entries are packed several per wavefront (default 64;
                              128 when feature_dim_hint <= 16) */
  int32_t split_row_min;   /* rows with  > this many entries get whole workgroups (default 512; 2048 when
                              feature_dim_hint <= 16) */
  int32_t chunk_edges;     /* entries per workgroup chunk of a split row (default 1024; 8192 when
                              feature_dim_hint <= 16) */
  int32_t column_classes;  /* long rows are cut by contiguous column ranges ("classes") into tiles and
                              all tiles of a class run on one XCD, so that its slice of Y stays in that
                              XCD's L2.  This is the finest number of classes (8, 16, 32, ... up to 512,
                              rounded up); shorter rows use nested coarser levels down to 8 classes.
                              0 = automatic (off while Y is small), 1 = off.  Needs column indices sorted
                              within the long rows, else it is skipped. */
  int32_t tile_row_min;    /* rows with >= this many entries are cut into 8 classes, with twice as many
                              into 16, and so on; 0 = 128 (16 entries per class), 64 on patterns with
                              128 or more stored entries per row on average */
  int32_t feature_dim_hint;/* feature dimension the plan will mostly run with, in 4-byte elements (a plan
                              for fusedmm_execute_f64 passes twice its dimension; for 2-byte storage of Y
                              the fp32 dimension still does well): used by the automatic choice of
                              column_classes, and fusedmm_plan_create reserves the scratch for it (as
                              fusedmm_plan_reserve does); 0 = 128 */
  int32_t general_kernel_only; /* non-zero: every fp32 / fp64 execute of this plan runs the general kernel
                              (one wavefront per row or 256-entry segment, any d), whatever the dimension
                              and alignment: the slow, simple path, kept selectable for cross-checks */
  int32_t host_threads;    /* host threads that build the plan's work lists: 0 = automatic (one per 65 536
                              rows, at most 16 and at most the machine's), k > 0 = exactly min(k, 64); the
                              plan does not depend on it */
} fusedmm_plan_options_t;

typedef struct fusedmm_plan fusedmm_plan_t;

/* Library version (FUSEDMM_VERSION of the build). */
int fusedmm_version(void);

/* Static, NUL-terminated description of a status code. */
const char* fusedmm_status_string(int status);

/* Fill *out (host) with the op tuple of a pattern; alpha is set to 1. */
int fusedmm_ops_preset(int pattern, fusedmm_ops_t* out);

/* Build the schedule for one sparsity pattern (Algorithm 1, Part1D, done the
 * GPU way: rows binned by length, long rows split into chunks).
 *   out        host: receives the plan
 *   m, n, nnz  host: matrix shape (m, n < 2^31)
 *   d_rowptr   device, m+1 int64;  d_colidx  device, nnz int32 (may be NULL if nnz == 0)
 *   options    host, may be NULL
 * Reads rowptr back to the host and validates rowptr and colidx; synchronises
 * the stream; allocates the plan's lists and the scratch for dimensions up to
 * options->feature_dim_hint (128 without options).  Not part of the timed hot path. */
int fusedmm_plan_create(fusedmm_plan_t** out, int64_t m, int64_t n, int64_t nnz,
                        const int64_t* d_rowptr, const int32_t* d_colidx,
                        const fusedmm_plan_options_t* options, void* stream);

/* Build the schedule by measurement (the counterpart of the paper's autotuned kernels,
 * Section IV-B: parameters chosen per machine by timing candidates).  The default plan of
 * fusedmm_plan_create is timed first and stays unless a candidate beats it by 1 %; then one scheduling
 * knob at a time is varied around the best plan so far: finest column classes (off, 8 ... 128), shortest
 * tiled row, chunk length, and the row lengths that separate packed rows, one-wavefront rows and chunked
 * rows (about 16 plans in all).  Every plan is timed by the median of 11 fusedmm_execute calls with the
 * given operands on `stream` (5 or 3 for kernels of more than 5 / 20 ms); the losers are destroyed.
 * Arguments as for fusedmm_plan_create and fusedmm_execute; d_Z is overwritten.  `chosen` (host, may be
 * NULL) receives the winning options, `best_ms` (host, may be NULL) its median time per execute.
 * Synchronises the stream; not for the hot path. */
int fusedmm_plan_create_tuned(fusedmm_plan_t** out, int64_t m, int64_t n, int64_t nnz,
                              const int64_t* d_rowptr, const int32_t* d_colidx,
                              const fusedmm_ops_t* ops, int32_t d, const float* d_values,
                              const float* d_X, int64_t ldx, const float* d_Y, int64_t ldy,
                              float* d_Z, int64_t ldz, void* stream,
                              fusedmm_plan_options_t* chosen, float* best_ms);

/* Grow the plan's scratch (partial rows of split rows, for the specialised and the general kernels)
 * so that every later fusedmm_execute / _bf16y / _f16y call with dimension <= d finds it in place;
 * fusedmm_plan_reserve_f64 does the same for fusedmm_execute_f64.  A dimension that is already covered
 * costs nothing.  May synchronise the device, free and allocate: call it outside the hot path (and
 * outside stream capture).  FUSEDMM_ERR_ALLOC leaves the plan without that scratch. */
int fusedmm_plan_reserve(fusedmm_plan_t* plan, int32_t d);
int fusedmm_plan_reserve_f64(fusedmm_plan_t* plan, int32_t d);

/* Device bytes the plan owns when executing with dimension d. */
int fusedmm_plan_workspace_bytes(const fusedmm_plan_t* plan, int32_t d, size_t* out);

/* Schedule statistics (host ints, any pointer may be NULL): rows packed per
 * wavefront, rows given one wavefront, workgroup chunks of untiled long rows,
 * rows merged from partial rows, partial rows, rows cut by column class, their
 * segments, number of column classes in use (1 = no tiling). */
int fusedmm_plan_stats(const fusedmm_plan_t* plan, int64_t* n_packed_rows, int64_t* n_wave_rows,
                       int64_t* n_chunks, int64_t* n_split_rows, int64_t* n_partials,
                       int64_t* n_tiled_rows, int64_t* n_tile_segments, int64_t* n_column_classes);

/* Z = FusedMM(A, X, Y) with the given ops; asynchronous on `stream`.
 *   d_values  device, nnz fp32 edge values a_uv; NULL unless SOP == EDGE_VALUE
 *   d_X       device, m x d (ldx); may be NULL when VOP == SEL2ND
 *   d_Y       device, n x d (ldy);  d_Z  device, m x d (ldz), overwritten
 * Y is the (n - 1) * ldy + d elements from d_Y on: when d is not a multiple of 4 the kernels may read (never
 * use, never write) up to three elements after the end of a row of Y inside that range -- the start of the
 * next row, or the padding between rows -- and nothing outside it.
 * Does not synchronise and does not allocate.  FUSEDMM_ERR_NOT_RESERVED when the pattern has split
 * rows and d exceeds what fusedmm_plan_create / fusedmm_plan_reserve reserved.  Z must not overlap
 * X, Y or d_values (FUSEDMM_ERR_ALIAS). */
int fusedmm_execute(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d,
                    const float* d_values, const float* d_X, int64_t ldx,
                    const float* d_Y, int64_t ldy, float* d_Z, int64_t ldz, void* stream);

/* fusedmm_execute for callers that cannot allocate and cannot have the plan reserve for them either:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * layout, ownership, errors and result (bit for bit) as fusedmm_execute, same kernels; the only difference
 * is where the partial rows of split rows go: into a fixed array in the library's device image
 * (FUSEDMM_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of the plan's scratch, so the
 * call works at any dimension whatever was reserved.  It calls no allocation routine of any kind.
 *   - Limit: partial rows x kernel size x 4 bytes (fusedmm_plan_stats gives the partial rows; the kernel size
 *     is d rounded up to the next of 32, 64, 96, 128, 192, 256, ... 1536, 2048; for the general kernel: 256-entry segments of long rows x d x 4)
 *     must fit, else FUSEDMM_ERR_SCRATCH_LIMIT and nothing is launched.
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two streams, or
 *     two plans) race on it.  Calls on one stream are ordered and safe.  Nothing in it has to start at
 *     zero (every partial row read was written by the same call), so nothing is cleared.
 *   - The plan must have been created on the device that is current at the call. */
#define FUSEDMM_STATIC_SCRATCH_BYTES (64u << 20)
int fusedmm_execute_static_scratch(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d,
                                   const float* d_values, const float* d_X, int64_t ldx,
                                   const float* d_Y, int64_t ldy, float* d_Z, int64_t ldz, void* stream);

/* The same operation with Y stored as bfloat16 (the upper 16 bits of each fp32 value): the
 * gathered rows are half as long, which is what bounds the kernel; x_u, every step's arithmetic,
 * the accumulation and Z stay fp32.  d_Y_bf16: device, n x d uint16 (ldy in elements, rows
 * 16-byte aligned: base aligned and ldy % 8 == 0; they are read 16 bytes = 8 elements per lane).  d is a
 * multiple of 8 from 8 to 1024 (32, 64, 96, 128, ... 768, 1024 on their own instances, the others on the next larger
 * one; FUSEDMM_ERR_UNSUPPORTED_DIM for any other d, FUSEDMM_ERR_INVALID_ARG for rows that are not
 * aligned).  Any valid op tuple.  The result is that of
 * fusedmm_execute on the fp32 matrix whose entries are the bfloat16 values widened back, up to the
 * order of the fp32 sums (the lane groups are half as wide). */
int fusedmm_execute_bf16y(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d,
                          const float* d_values, const float* d_X, int64_t ldx,
                          const uint16_t* d_Y_bf16, int64_t ldy, float* d_Z, int64_t ldz, void* stream);

/* d_dst[i] = bfloat16(d_src[i]) for i < count, round to nearest even (device pointers,
 * asynchronous on `stream`): the storage format fusedmm_execute_bf16y reads. */
int fusedmm_to_bf16(uint16_t* d_dst, const float* d_src, size_t count, void* stream);

/* The same again with Y stored in IEEE half precision (binary16: 11 significant bits instead of
 * bfloat16's 8, range up to 65504): same layout, alignment and error rules as fusedmm_execute_bf16y;
 * fusedmm_to_f16 converts with round to nearest even (values beyond the half range become infinity).
 * The result is that of fusedmm_execute on the fp32 matrix whose entries are the half values widened
 * back, up to the order of the fp32 sums. */
int fusedmm_execute_f16y(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d,
                         const float* d_values, const float* d_X, int64_t ldx,
                         const uint16_t* d_Y_f16, int64_t ldy, float* d_Z, int64_t ldz, void* stream);
int fusedmm_to_f16(uint16_t* d_dst, const float* d_src, size_t count, void* stream);

/* Double precision (Section V: the method is not tied to single precision): X, Y, Z and the edge
 * values are fp64 and so is every step's arithmetic (the sigmoid's exponential, reciprocals and square
 * roots are the correctly rounded library ones, not the fp32 hardware approximations).  Every d
 * runs the specialised schedule of fusedmm_execute on double-precision instances (32, 64, ... 2048; any
 * other dimension runs on the next larger one; rows may start at any element); a plan created with
 * general_kernel_only runs the general kernel (one wavefront per row or 256-entry segment).  Any valid op
 * tuple either way.  Arguments, layout, ownership and errors as for fusedmm_execute; ops->alpha is widened.  A plan
 * with split rows needs fusedmm_plan_reserve_f64(plan, d) first (FUSEDMM_ERR_NOT_RESERVED otherwise):
 * fusedmm_plan_create reserves for fp32 rows only. */
int fusedmm_execute_f64(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d,
                        const double* d_values, const double* d_X, int64_t ldx,
                        const double* d_Y, int64_t ldy, double* d_Z, int64_t ldz, void* stream);

/* Test hook: run the same schedule and edge indexing as fusedmm_execute would
 * for dimension d (row pointers may be of any alignment class: pass
 * fast_path = 1 to exercise the specialised kernels' indexing, 2 for that of their
 * double-precision instances, 0 for the general kernel's) and add 1 to d_counts[e]
 * for every stored entry e visited.
 * d_counts: device, nnz uint32, zeroed by the caller.  Correct schedules leave
 * every count equal to 1. */
int fusedmm_debug_edge_visits(fusedmm_plan_t* plan, int32_t d, int32_t fast_path,
                              uint32_t* d_counts, void* stream);

/* Per-kernel timing for benchmarks.  When enabled, fusedmm_execute records three HIP events on
 * the launch stream: one before its main kernel, one right after it and one more right after that
 * (at most 4096 calls are retained).  fusedmm_plan_read_profile synchronises those events and
 * returns the summed before->after milliseconds (main kernel + the cost of the bracket itself),
 * the summed after->after2 milliseconds (the cost of an empty bracket: subtract it to get the
 * kernel's own duration, which matters for kernels of a few tens of microseconds) and the number
 * of timed calls, then clears the record.  All pointers are host pointers. */
int fusedmm_plan_set_profiling(fusedmm_plan_t* plan, int32_t enabled);
int fusedmm_plan_read_profile(fusedmm_plan_t* plan, double* main_kernel_ms_sum, double* empty_bracket_ms_sum,
                              int64_t* calls);
/* The same record call by call (for medians): fills at most `capacity` entries of both host arrays,
 * returns how many in *calls, then clears the record. */
int fusedmm_plan_read_profile_samples(fusedmm_plan_t* plan, double* main_kernel_ms, double* empty_bracket_ms,
                                      int64_t capacity, int64_t* calls);

/* Measurement aid: a plain grid-stride copy kernel, dst[i] = src[i] for `bytes` bytes
 * (device pointers, 16-byte aligned, bytes a multiple of 16, non-overlapping),
 * asynchronous on `stream`.  Profilers' memory counters are calibrated against its
 * known traffic (bytes read + bytes written). */
int fusedmm_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);

/* Test hook, host only (no GPU work): which kernel size a feature dimension runs on.  storage: 0 = fp32
 * (fusedmm_execute), 1 = Y in 2-byte elements (fusedmm_execute_bf16y / _f16y), 2 = double precision
 * (fusedmm_execute_f64).  Returns the instance size of the specialised schedule (32, 64, 96, ... 2048: the
 * dimension itself or the next larger size), d itself for the one-lane-per-entry kernels (fp32, d = 2, 3, 4, 8,
 * 16), or 0 when that storage form does not take the dimension.  Also the stride of the partial rows, which
 * fusedmm_execute_static_scratch's limit is counted in. */
int fusedmm_debug_kernel_size(int32_t d, int32_t storage);

/* Free the plan and everything it owns. */
int fusedmm_plan_destroy(fusedmm_plan_t* plan);

/* ---------------------------------------------------------------------------------------------
 * Minibatch embedding epoch: the end-to-end training experiment of Section V (Table VIII: d = 128,
 * batches of 256 vertices, sigmoid embedding pattern of Table III).  A minibatch is a rectangular
 * slice A[B, :] of the adjacency matrix (Section III, Fig. 2); forming the batches is the
 * application's job (Section III-C), which is what this layer does.  The paper does not print the
 * update rule; the one implemented, for batch i = rows [i*batch_rows, min(n, (i+1)*batch_rows)) of
 * a square n x n pattern, batches in order, X being both operand matrices:
 *     Zpos = FusedMM(A[B_i, :], X[B_i], X)  with (MUL, RSUM, 1-SIGMOID, MUL, SUM)
 *     Zneg = FusedMM(N_i,       X[B_i], X)  with (MUL, RSUM,   SIGMOID, MUL, SUM)
 *     X[B_i] <- X[B_i] + lr * (Zpos - Zneg)
 * N_i is the |B_i| x n pattern whose every row holds the n_negative sample columns of batch i.
 * Both calls of a batch read X as the earlier batches left it; the rows of the batch are written
 * after both have finished (stream order), so results do not depend on scheduling.  The library
 * issues the two calls as one FusedMM over the concatenated pattern [A[B_i, :] | N_i] with the scaling
 * step h = a - SIGMOID(s), a = 1 on stored entries and 0 on samples (the same sum, Zpos - Zneg).
 *
 * create : d_rowptr (n+1 int64, device), d_colidx (nnz int32, device) as for fusedmm_plan_create;
 *          d_negatives: device, n_batches * n_negative int32, batch-major, may be NULL when
 *          n_negative == 0.  All three are read once here (the handle keeps its own concatenated
 *          copies and does not refer to them afterwards).  Builds one plan per batch; synchronises
 *          the stream.  Samples outside [0, n) -> FUSEDMM_ERR_INVALID_ARG.
 * reserve: allocates the batch_rows x d result buffer and the plans' scratch for dimension d;
 *          required before the first epoch with a dimension above any reserved so far
 *          (fusedmm_minibatch_epoch never allocates: FUSEDMM_ERR_NOT_RESERVED otherwise).
 * epoch  : one pass over all batches, asynchronous on `stream`, in place on d_X (n rows, leading
 *          dimension ldx >= d).  Any 1 <= d <= FUSEDMM_MAX_D; dispatch as for fusedmm_execute.  Overlapping epochs on one handle must be on one stream.
 * info   : number of batches and of kernel launches one epoch issues (host pointers, may be NULL).
 * Errors as elsewhere: a status is returned and nothing is launched for the failing batch. */
typedef struct fusedmm_minibatch fusedmm_minibatch_t;
int fusedmm_minibatch_create(fusedmm_minibatch_t** out, int64_t n, int64_t nnz, const int64_t* d_rowptr,
                             const int32_t* d_colidx, int32_t batch_rows, int32_t n_negative,
                             const int32_t* d_negatives, void* stream);
int fusedmm_minibatch_reserve(fusedmm_minibatch_t* mb, int32_t d);
int fusedmm_minibatch_epoch(fusedmm_minibatch_t* mb, int32_t d, float lr, float* d_X, int64_t ldx, void* stream);
int fusedmm_minibatch_info(const fusedmm_minibatch_t* mb, int32_t* n_batches, int64_t* launches_per_epoch);
int fusedmm_minibatch_destroy(fusedmm_minibatch_t* mb);

#ifdef __cplusplus
}
#endif
#endif /* FUSEDMM_H_ */
