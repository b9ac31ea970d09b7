// Host side of libfusedmm.so: the C ABI of include/fusedmm.h, argument validation,
// the degree-binned plan (the GPU counterpart of Part1D in Algorithm 1) and dispatch.
#include "../../include/fusedmm.h"
#include "fusedmm_internal.h"

#include <algorithm>
#include <mutex>
#include <new>
#include <thread>
#include <utility>
#include <vector>

using namespace fmm;

struct fusedmm_plan {
  int64_t m = 0, n = 0, nnz = 0;
  const int64_t* d_rowptr = nullptr;
  const int32_t* d_colidx = nullptr;
  int32_t small_row_max = 0, split_row_min = 0, chunk_edges = 0, tile_row_min = 0;  // as resolved
  int32_t n_wave = 0, n_packed = 0, n_empty = 0, n_chunks = 0, n_merges = 0, n_parts = 0;  // n_packed: non-empty
  int32_t n_items = 0, n_tile_descs = 0, n_tiled_rows = 0, n_classes = 1;
  bool general_only = false;  // every execute runs the general kernel
  int32_t* d_order = nullptr;
  ChunkDesc* d_chunks = nullptr;
  BlockItem* d_items = nullptr;
  ChunkDesc* d_tile_descs = nullptr;
  MergeDesc* d_merges = nullptr;
  float* d_partials = nullptr;
  int32_t partials_d = 0;  // scratch holds n_parts rows of this many floats
  // the general kernel's own cut of the rows longer than kGenericSplit (any d, fp32 or fp64)
  ChunkDesc* d_gen_segs = nullptr;
  MergeDesc* d_gen_merges = nullptr;
  int32_t n_gen_segs = 0, n_gen_merges = 0;
  void* d_gen_partials = nullptr;
  size_t gen_partials_bytes = 0;
  bool profiling = false;
  struct EventTriple { hipEvent_t before, after, after2; };
  std::vector<EventTriple> events;  // main kernel between before/after; nothing between after/after2
  size_t events_used = 0;
};

// Fixed scratch of fusedmm_execute_static_scratch: partial rows of split rows, for callers that cannot
// allocate.  One copy per GPU the library runs on, held until the process ends.  In host code the array's
// name only stands for the symbol: its device address is looked up once per device
// (static_scratch_for_current_device) and that pointer is what kernels, copies and fills are given.
static __device__ __align__(256) unsigned char scratch[FUSEDMM_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxScratchDevices = 64;
void* g_scratch_ptr[kMaxScratchDevices] = {};
std::mutex g_scratch_mutex;

// The address of `scratch` on the current device (every GPU holds its own copy at its own address).
int static_scratch_for_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FUSEDMM_ERR_HIP;
  if (dev < 0 || dev >= kMaxScratchDevices) return FUSEDMM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return FUSEDMM_ERR_HIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FUSEDMM_OK;
}

constexpr int32_t kDefaultSmallRowMax = 64;
constexpr int32_t kDefaultSplitRowMin = 512;
constexpr int32_t kDefaultChunkEdges = 1024;
// the same three when the plan is hinted a feature dimension of at most 16
constexpr int32_t kShortDimSmallRowMax = 128;
constexpr int32_t kShortDimSplitRowMin = 2048;
constexpr int32_t kShortDimChunkEdges = 8192;
// Column-class tiling defaults, from sweeps on MI355X: it pays once Y (n rows of the hinted
// dimension) is beyond what the eight 4 MB L2s keep resident anyway (>= 48 MiB; >= 16 MiB on dense patterns,
// where every row of Y is gathered hundreds of times and an eighth of it fits one L2).  The finest level
// keeps a class slice of Y at about 64 MiB on sparse patterns -- there only the often-gathered rows of
// a slice are reused, and they fit an L2 from that size down; finer classes only add partial rows --
// and at about 8 MiB on dense ones (128 stored entries per row on average: every row of the slice is
// reused many times, so the slice itself should come near an L2); it stops at 64 classes.
constexpr int64_t kTilingMinYBytes = 48ll << 20;
constexpr int64_t kTilingMinYBytesDense = 16ll << 20;  // c3's graph at d = 32 (Y = 30 MB): 1.69 -> 1.07 ms with 8 classes
constexpr int64_t kTilingSliceBytesSparse = 64ll << 20;
constexpr int64_t kTilingSliceBytesDense = 8ll << 20;
constexpr int64_t kDenseEntriesPerRow = 128;
constexpr int32_t kAutoMaxColumnClasses = 64;
// class boundaries come from a histogram of the column indices: this many buckets, about this many sampled entries
constexpr int64_t kClassBuckets = 1 << 16;
constexpr int64_t kClassSamples = 1 << 24;
constexpr double kClassWidthWeight = 0.25;
constexpr int32_t kMaxColumnClasses = 512;
constexpr int32_t kDefaultTileEdgesPerClass = 16;
constexpr int32_t kDenseTileEdgesPerClass = 8;
constexpr size_t kMaxProfiledCalls = 4096;
// the plan's passes over the rows run on up to this many host threads, each on at least this many rows
constexpr int kPlanThreads = 16;
constexpr int kPlanThreadsLimit = 64;   // for an explicit fusedmm_plan_options_t::host_threads
constexpr int64_t kPlanRowsPerThread = 1 << 16;

// The instance size a dimension runs on: itself if it has instances of its own, else the next larger one (any
// dimension from kMinWideDim up to kMaxWideDim: the masked instances skip what lies beyond d, element by element in
// the last piece when d is not a multiple of 4), else 0.  The largest size, 1024, exists for fp32 only.
constexpr int32_t kMinWideDim = 9;
constexpr int32_t kMaxWideDim = 1024;
constexpr int32_t kMaxWideDimF64 = 512;
int32_t instance_dim(int32_t d) {
  if (d < kMinWideDim || d > kMaxWideDim) return 0;
  int32_t D = 32;
  while (D < d) D *= 2;
  return D;
}

// The same for double precision: the five sizes up to 512.
int32_t instance_dim_f64(int32_t d) { return d > kMaxWideDimF64 ? 0 : instance_dim(d); }

// The same for Y stored in 2-byte elements: rows are read 16 bytes = 8 elements at a time, so d is a multiple
// of 8, from 8 up to 512.
constexpr int32_t kMaxWideDim2Byte = 512;
int32_t instance_dim_2byte(int32_t d) {
  if (d < 8 || d % 8 != 0 || d > kMaxWideDim2Byte) return 0;
  return std::max<int32_t>(32, instance_dim(d));
}

// How many floats a partial row of the specialised schedule takes when the plan serves dimensions up to d in
// fp32 (the largest instance size among them, and the short-vector kernels' fixed stride) ...
int32_t partial_floats_f32(int32_t d) {
  return std::max<int32_t>(d >= kMaxWideDim ? kMaxWideDim : instance_dim(d), kSmallPartialStride);
}
// ... and in fp64 (two floats per element)
int32_t partial_floats_f64(int32_t d) { return 2 * (d >= kMaxWideDimF64 ? kMaxWideDimF64 : instance_dim_f64(d)); }

bool ops_valid(const fusedmm_ops_t& o, bool allow_private = false) {
  if (allow_private && o.sop == kSopValueMinusSigmoid)  // scalar message from a reduction and the edge value
    return o.vop >= FUSEDMM_VOP_MUL && o.vop <= FUSEDMM_VOP_ADD && o.rop > FUSEDMM_ROP_NOOP && o.rop <= FUSEDMM_ROP_RMUL &&
           o.mop >= FUSEDMM_MOP_MUL_Y && o.mop <= FUSEDMM_MOP_SEL2ND && o.aop >= FUSEDMM_AOP_SUM && o.aop <= FUSEDMM_AOP_MEAN;
  if (o.vop < FUSEDMM_VOP_MUL || o.vop > FUSEDMM_VOP_ADD) return false;
  if (o.rop < FUSEDMM_ROP_NOOP || o.rop > FUSEDMM_ROP_RMUL) return false;
  if (o.sop < FUSEDMM_SOP_EDGE_VALUE || o.sop > FUSEDMM_SOP_NOOP) return false;
  if (o.mop < FUSEDMM_MOP_MUL_Y || o.mop > FUSEDMM_MOP_SEL2ND) return false;
  if (o.aop < FUSEDMM_AOP_SUM || o.aop > FUSEDMM_AOP_MEAN) return false;
  return o.sop != FUSEDMM_SOP_EDGE_VALUE || o.rop == FUSEDMM_ROP_NOOP;
}

// The pattern recogniser: map an op tuple to a specialised kernel, or -1 for the general one.
int recognise(const fusedmm_ops_t& o) {
  if (o.vop == FUSEDMM_VOP_SEL2ND && o.rop == FUSEDMM_ROP_NOOP && o.sop == FUSEDMM_SOP_EDGE_VALUE &&
      o.mop != FUSEDMM_MOP_SEL2ND) {  // the GCN message a_uv * y_v (t = y_v here, so MUL_T is the same) with any
                                      // pooling: sum and mean share an instance
    if (o.aop == FUSEDMM_AOP_MAX) return PAT_GCN_MAX;
    if (o.aop == FUSEDMM_AOP_MIN) return PAT_GCN_MIN;
    return PAT_GCN;
  }
  if (o.aop != FUSEDMM_AOP_SUM) return -1;
  if (o.vop == FUSEDMM_VOP_MUL && o.rop == FUSEDMM_ROP_RSUM && o.mop == FUSEDMM_MOP_MUL_Y) {
    if (o.sop == kSopValueMinusSigmoid) return PAT_SIGNED_SIGMOID;
    if (o.sop == FUSEDMM_SOP_SIGMOID) return PAT_SIGMOID;
    if (o.sop == FUSEDMM_SOP_ONE_MINUS_SIGMOID) return PAT_ONE_MINUS_SIGMOID;
  }
  if (o.vop == FUSEDMM_VOP_SUB && o.mop == FUSEDMM_MOP_MUL_T) {
    if (o.rop == FUSEDMM_ROP_SUMSQ && o.sop == FUSEDMM_SOP_INV_1P) return PAT_TDIST;
    if (o.rop == FUSEDMM_ROP_NORM2 && o.sop == FUSEDMM_SOP_SCAL) return PAT_FR;
  }
  return -1;
}

// The tuple family with compile-time vector loops an op tuple belongs to (scalar message from a dot product,
// or from the sum / difference of the operands), or -1: such a tuple runs faster there than with every step
// read at run time, and the families also take the dimensions between two instance sizes.
int recognise_family(const fusedmm_ops_t& o) {
  if (o.rop == FUSEDMM_ROP_NOOP || o.sop == FUSEDMM_SOP_EDGE_VALUE) return -1;  // vector message, or the edge value
  const bool mm = o.aop == FUSEDMM_AOP_MAX || o.aop == FUSEDMM_AOP_MIN;
  if (o.vop == FUSEDMM_VOP_MUL && o.rop == FUSEDMM_ROP_RSUM) return mm ? PAT_DOT_MM : PAT_DOT;
  if ((o.vop == FUSEDMM_VOP_SUB || o.vop == FUSEDMM_VOP_ADD) &&
      (o.rop == FUSEDMM_ROP_RSUM || o.rop == FUSEDMM_ROP_SUMSQ || o.rop == FUSEDMM_ROP_NORM2))
    return mm ? PAT_DIST_MM : PAT_DIST;
  return -1;
}

// Which instance of the specialised kernel an op tuple runs on: a recognised pattern its own (the masked form of
// it when the dimension lies between two instance sizes), else the tuple family it belongs to, else the one that
// reads its ops at run time.
int choose_pattern(int recognised, int family, int32_t d, int32_t D) {
  if (d % 4 != 0) {
    // rows that end inside a 16-byte piece: the GCN messages, the two tuple families (which hold the other
    // application patterns) and the run-time-ops instance exist in a form that masks down to the element
    if (recognised == PAT_GCN || recognised == PAT_GCN_MAX || recognised == PAT_GCN_MIN) return recognised | kPatRagged;
    return (family >= 0 ? family : PAT_RUNTIME) | kPatRagged;
  }
  if (recognised >= 0) return D == d ? recognised : (recognised | kPatMasked);
  return family >= 0 ? family : PAT_RUNTIME;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlaps(const float* a, int64_t rows_a, int64_t ld_a, const float* b, int64_t rows_b, int64_t ld_b, int32_t d) {
  if (!a || !b || rows_a <= 0 || rows_b <= 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  const uintptr_t a1 = a0 + (uintptr_t)((rows_a - 1) * ld_a + d) * sizeof(float);
  const uintptr_t b1 = b0 + (uintptr_t)((rows_b - 1) * ld_b + d) * sizeof(float);
  return a0 < b1 && b0 < a1;
}

void free_plan_device(fusedmm_plan* p) {
  if (p->d_order) (void)hipFree(p->d_order);
  if (p->d_chunks) (void)hipFree(p->d_chunks);
  if (p->d_merges) (void)hipFree(p->d_merges);
  if (p->d_items) (void)hipFree(p->d_items);
  if (p->d_tile_descs) (void)hipFree(p->d_tile_descs);
  if (p->d_partials) (void)hipFree(p->d_partials);
  if (p->d_gen_segs) (void)hipFree(p->d_gen_segs);
  if (p->d_gen_merges) (void)hipFree(p->d_gen_merges);
  if (p->d_gen_partials) (void)hipFree(p->d_gen_partials);
  for (auto& ev : p->events) {
    (void)hipEventDestroy(ev.before);
    (void)hipEventDestroy(ev.after);
    (void)hipEventDestroy(ev.after2);
  }
  p->events.clear();
}

template <class T>
int upload(T** dst, const std::vector<T>& src, hipStream_t stream) {
  *dst = nullptr;
  if (src.empty()) return FUSEDMM_OK;
  if (hipMalloc(reinterpret_cast<void**>(dst), src.size() * sizeof(T)) != hipSuccess) {
    (void)hipGetLastError();
    return FUSEDMM_ERR_ALLOC;
  }
  if (hipMemcpyAsync(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice, stream) != hipSuccess)
    return FUSEDMM_ERR_HIP;
  return FUSEDMM_OK;
}

// Reserve-time only (fusedmm_plan_create, fusedmm_plan_reserve*): may synchronise the device, free and
// allocate.  The execute entry points never call these; they compare capacities and return
// FUSEDMM_ERR_NOT_RESERVED.
int ensure_partials(fusedmm_plan* p, int32_t d) {
  if (p->n_parts == 0 || d <= p->partials_d) return FUSEDMM_OK;
  if (p->d_partials) {
    if (hipDeviceSynchronize() != hipSuccess) return FUSEDMM_ERR_HIP;  // earlier launches may still use it
    (void)hipFree(p->d_partials);
    p->d_partials = nullptr;
    p->partials_d = 0;
  }
  if (hipMalloc(reinterpret_cast<void**>(&p->d_partials), (size_t)p->n_parts * d * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    return FUSEDMM_ERR_ALLOC;
  }
  p->partials_d = d;
  return FUSEDMM_OK;
}

// Scratch of the general kernel: n_gen_segs partial rows of d elements of elem_bytes each.
int ensure_gen_partials(fusedmm_plan* p, int32_t d, size_t elem_bytes) {
  const size_t need = (size_t)p->n_gen_segs * (size_t)d * elem_bytes;
  if (need <= p->gen_partials_bytes) return FUSEDMM_OK;
  if (p->d_gen_partials) {
    if (hipDeviceSynchronize() != hipSuccess) return FUSEDMM_ERR_HIP;  // earlier launches may still use it
    (void)hipFree(p->d_gen_partials);
    p->d_gen_partials = nullptr;
    p->gen_partials_bytes = 0;
  }
  if (hipMalloc(&p->d_gen_partials, need) != hipSuccess) {
    (void)hipGetLastError();
    return FUSEDMM_ERR_ALLOC;
  }
  p->gen_partials_bytes = need;
  return FUSEDMM_OK;
}

template <class T>
void fill_generic_segments(const fusedmm_plan* p, GenericArgsT<T>* g) {
  g->segs = p->d_gen_segs;
  g->n_segs = p->n_gen_segs;
  g->merges = p->d_gen_merges;
  g->n_merges = p->n_gen_merges;
  g->partials = static_cast<T*>(p->d_gen_partials);
}

// d: the instance size of a wide kernel, or the dimension itself for the kernels for very short feature vectors
void fill_schedule_args(const fusedmm_plan* p, int32_t d, int y_format, KernelArgs* a) {
  a->rowptr = p->d_rowptr;
  a->colidx = p->d_colidx;
  a->order = p->d_order;
  a->chunks = p->d_chunks;
  a->items = p->d_items;
  a->tile_descs = p->d_tile_descs;
  a->nb_tiled = p->n_items;
  a->partials = p->d_partials;
  a->visit_counts = nullptr;
  a->n_chunks = p->n_chunks;
  a->n_wave = p->n_wave;
  a->n_packed = p->n_packed;
  a->n_empty = p->n_empty;
  a->nb_zero = (p->n_empty + kZeroRowsPerBlock - 1) / kZeroRowsPerBlock;
  a->nb_chunk = p->n_chunks;
  a->nb_wave = (p->n_wave + kWavesPerBlock - 1) / kWavesPerBlock;
  const int rpb = (is_small_dim(d) && y_format != kYF64) ? small_packed_rows_per_block(d) : packed_rows_per_block(d, y_format);
  a->nb_packed = rpb > 0 ? (p->n_packed + rpb - 1) / rpb : 0;
}

// what the specialised kernels read of the op tuple
void fill_op_args(const fusedmm_ops_t& ops, KernelArgs* a) {
  a->alpha = ops.alpha;
  a->sign = ops.aop == FUSEDMM_AOP_MIN ? -1.0f : 1.0f;
  a->ysign = ops.vop == FUSEDMM_VOP_SUB ? -1.0f : 1.0f;
  a->sop_exp = ops.sop == FUSEDMM_SOP_SIGMOID || ops.sop == FUSEDMM_SOP_ONE_MINUS_SIGMOID || ops.sop == kSopValueMinusSigmoid;
  a->sop_c1 = ops.sop == FUSEDMM_SOP_ONE_MINUS_SIGMOID ? 1.4426950408889634f : -1.4426950408889634f;
  a->sop_rcp = a->sop_exp || ops.sop == FUSEDMM_SOP_INV_1P;
  a->sop_lin = ops.sop == FUSEDMM_SOP_SCAL ? ops.alpha : 1.0f;
  a->vop = ops.vop; a->rop = ops.rop; a->sop = ops.sop; a->mop = ops.mop;
  a->mean = ops.aop == FUSEDMM_AOP_MEAN;  // accumulated as a sum; whole rows are scaled at the store, split rows in the merge
  a->aop = a->mean ? FUSEDMM_AOP_SUM : ops.aop;
}

}  // namespace

extern "C" {

int fusedmm_version(void) { return FUSEDMM_VERSION; }

const char* fusedmm_status_string(int status) {
  switch (status) {
    case FUSEDMM_OK: return "ok";
    case FUSEDMM_ERR_INVALID_ARG: return "invalid argument";
    case FUSEDMM_ERR_UNSUPPORTED_OPS: return "unsupported op tuple";
    case FUSEDMM_ERR_UNSUPPORTED_DIM: return "unsupported feature dimension";
    case FUSEDMM_ERR_ALIAS: return "output overlaps an input";
    case FUSEDMM_ERR_ALLOC: return "allocation failed";
    case FUSEDMM_ERR_HIP: return "HIP runtime error";
    case FUSEDMM_ERR_NOT_RESERVED: return "scratch not reserved for this dimension (call fusedmm_plan_reserve first)";
    case FUSEDMM_ERR_SCRATCH_LIMIT: return "the partial rows of this call exceed the fixed scratch of fusedmm_execute_static_scratch";
    default: return "unknown status";
  }
}

int fusedmm_ops_preset(int pattern, fusedmm_ops_t* out) {
  if (!out) return FUSEDMM_ERR_INVALID_ARG;
  fusedmm_ops_t o;
  o.aop = FUSEDMM_AOP_SUM;
  o.alpha = 1.0f;
  switch (pattern) {
    case FUSEDMM_PATTERN_SIGMOID_EMBED:
      o.vop = FUSEDMM_VOP_MUL; o.rop = FUSEDMM_ROP_RSUM; o.sop = FUSEDMM_SOP_SIGMOID; o.mop = FUSEDMM_MOP_MUL_Y; break;
    case FUSEDMM_PATTERN_ONE_MINUS_SIGMOID_EMBED:
      o.vop = FUSEDMM_VOP_MUL; o.rop = FUSEDMM_ROP_RSUM; o.sop = FUSEDMM_SOP_ONE_MINUS_SIGMOID; o.mop = FUSEDMM_MOP_MUL_Y; break;
    case FUSEDMM_PATTERN_GCN_SUM:
      o.vop = FUSEDMM_VOP_SEL2ND; o.rop = FUSEDMM_ROP_NOOP; o.sop = FUSEDMM_SOP_EDGE_VALUE; o.mop = FUSEDMM_MOP_MUL_Y; break;
    case FUSEDMM_PATTERN_TDIST:
      o.vop = FUSEDMM_VOP_SUB; o.rop = FUSEDMM_ROP_SUMSQ; o.sop = FUSEDMM_SOP_INV_1P; o.mop = FUSEDMM_MOP_MUL_T; break;
    case FUSEDMM_PATTERN_FR:
      o.vop = FUSEDMM_VOP_SUB; o.rop = FUSEDMM_ROP_NORM2; o.sop = FUSEDMM_SOP_SCAL; o.mop = FUSEDMM_MOP_MUL_T; break;
    default: return FUSEDMM_ERR_INVALID_ARG;
  }
  *out = o;
  return FUSEDMM_OK;
}

int fusedmm_plan_create(fusedmm_plan_t** out, int64_t m, int64_t n, int64_t nnz, const int64_t* d_rowptr,
                        const int32_t* d_colidx, const fusedmm_plan_options_t* options, void* stream_) {
  if (!out) return FUSEDMM_ERR_INVALID_ARG;
  *out = nullptr;
  if (m < 0 || n < 0 || nnz < 0 || m >= INT32_MAX || n >= INT32_MAX) return FUSEDMM_ERR_INVALID_ARG;
  if (!d_rowptr || (nnz > 0 && (!d_colidx || n == 0 || m == 0))) return FUSEDMM_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(stream_);

  int32_t small_max = kDefaultSmallRowMax, split_min = kDefaultSplitRowMin, chunk = kDefaultChunkEdges;
  if (options && options->feature_dim_hint > 0 && options->feature_dim_hint <= 16) {
    // very short feature vectors (one lane per stored entry): a work item's fixed cost -- its descriptor, the
    // reduction across lanes, the store -- is spread over more entries
    small_max = kShortDimSmallRowMax; split_min = kShortDimSplitRowMin; chunk = kShortDimChunkEdges;
  }
  if (options) {
    if (options->small_row_max < 0 || options->split_row_min < 0 || options->chunk_edges < 0) return FUSEDMM_ERR_INVALID_ARG;
    if (options->small_row_max > 0) small_max = options->small_row_max;
    if (options->split_row_min > 0) split_min = options->split_row_min;
    if (options->chunk_edges > 0) chunk = options->chunk_edges;
  }
  int32_t n_classes = 0, tile_min = 0, d_hint = 128;
  if (options) {
    if (options->column_classes < 0 || options->tile_row_min < 0 || options->feature_dim_hint < 0) return FUSEDMM_ERR_INVALID_ARG;
    n_classes = options->column_classes;
    tile_min = options->tile_row_min;
    if (options->feature_dim_hint > 0) d_hint = options->feature_dim_hint;
  }
  if (n_classes == 0) {
    // automatic: off while Y (n rows of the hinted dimension) is small; else as many finest classes as
    // bring a class slice of Y down to the size that pays for the pattern's density, at most 64
    const int64_t y_bytes = n * (int64_t)d_hint * (int64_t)sizeof(float);
    const bool dense = m > 0 && nnz / m >= kDenseEntriesPerRow;
    n_classes = 1;
    if (y_bytes >= (dense ? kTilingMinYBytesDense : kTilingMinYBytes)) {
      n_classes = kNumXcd;
      const int64_t slice = dense ? kTilingSliceBytesDense : kTilingSliceBytesSparse;
      while (n_classes < kAutoMaxColumnClasses && y_bytes / n_classes > slice) n_classes *= 2;
    }
  }
  if (n_classes > 1) {  // levels are nested: 8, 16, 32, ... classes
    int32_t c = kNumXcd;
    while (c < n_classes && c < kMaxColumnClasses) c *= 2;
    n_classes = c;
  }
  // a row needs 16 entries per class on average for a partial row per class to be worth it; 8 on dense patterns,
  // where nearly every row is tiled anyway and the shorter ones gain more from their classes' L2 than their partial
  // rows cost (c3: 3.99 -> 3.90 ms; the sparse workloads lose 1-6 % with it)
  if (tile_min <= 0)
    tile_min = ((m > 0 && nnz / m >= kDenseEntriesPerRow) ? kDenseTileEdgesPerClass : kDefaultTileEdgesPerClass) * kNumXcd;
  const int64_t tile_edges_per_class = std::max<int64_t>(1, tile_min / kNumXcd);
  small_max = std::min(small_max, 1 << 16);
  split_min = std::min(std::max(split_min, small_max), 1 << 20);
  chunk = std::min(std::max((chunk + 255) / 256 * 256, 256), 1 << 24);

  // row pointers to the host: O(m) scan, like Part1D
  std::vector<int64_t> rp;
  try {
    rp.resize((size_t)m + 1);
  } catch (const std::bad_alloc&) {
    return FUSEDMM_ERR_ALLOC;
  }
  if (hipStreamSynchronize(stream) != hipSuccess) return FUSEDMM_ERR_HIP;
  if (hipMemcpy(rp.data(), d_rowptr, ((size_t)m + 1) * sizeof(int64_t), hipMemcpyDeviceToHost) != hipSuccess)
    return FUSEDMM_ERR_HIP;
  if (rp[0] != 0 || rp[m] != nnz) return FUSEDMM_ERR_INVALID_ARG;
  for (int64_t u = 0; u < m; ++u)
    if (rp[u + 1] < rp[u]) return FUSEDMM_ERR_INVALID_ARG;

  // column indices must address rows of Y: checked on the device, once
  if (nnz > 0) {
    int32_t* d_flag = nullptr;
    if (hipMalloc(reinterpret_cast<void**>(&d_flag), sizeof(int32_t)) != hipSuccess) return FUSEDMM_ERR_ALLOC;
    int32_t flag = 0;
    hipError_t e = hipMemcpy(d_flag, &flag, sizeof(flag), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = launch_validate_colidx(d_colidx, nnz, n, d_flag, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e == hipSuccess) e = hipMemcpy(&flag, d_flag, sizeof(flag), hipMemcpyDeviceToHost);
    (void)hipFree(d_flag);
    if (e != hipSuccess) return FUSEDMM_ERR_HIP;
    if (flag != 0) return FUSEDMM_ERR_INVALID_ARG;
  }

  fusedmm_plan* p = new (std::nothrow) fusedmm_plan();
  if (!p) return FUSEDMM_ERR_ALLOC;
  p->m = m; p->n = n; p->nnz = nnz;
  p->d_rowptr = d_rowptr; p->d_colidx = d_colidx;
  p->small_row_max = small_max; p->split_row_min = split_min; p->chunk_edges = chunk; p->tile_row_min = tile_min;
  p->general_only = options && options->general_kernel_only != 0;

  std::vector<int32_t> order;
  std::vector<ChunkDesc> chunks, tile_descs;
  std::vector<MergeDesc> merges;
  std::vector<BlockItem> items;
  int st = FUSEDMM_OK;
  int32_t* d_class_start = nullptr;  // column-class boundaries on the device while the tile bounds are computed
  try {
    // ---- which rows are cut into column-class tiles, and how finely ---------------------
    // Level of a row = number of classes it is cut into: the largest of 8, 16, ..., n_classes
    // that leaves it tile_edges_per_class entries per class on average.  Classes are nested
    // contiguous column ranges: a class of level L is n_classes / L finest classes.
    std::vector<int32_t> tiled_rows, tiled_level;
    std::vector<int64_t> bnd_off;  // per tiled row: where its level + 1 boundaries start in bounds[]
    std::vector<int32_t> bounds;
    // The finest classes are contiguous column ranges that hold about the same number of stored entries each
    // (from a histogram of the column indices over kClassBuckets buckets, every stride-th entry), not the same
    // number of columns: where the often-gathered columns sit side by side -- vertex orders that keep hubs
    // together -- equal widths would give one XCD most of the work.
    std::vector<int32_t> class_start;
    if (n_classes > 1 && nnz > 0) {
      const int32_t nbk = (int32_t)std::min<int64_t>(kClassBuckets, n);
      const int64_t stride = std::max<int64_t>(1, nnz / kClassSamples);
      std::vector<uint32_t> hist((size_t)nbk);
      uint32_t* d_hist = nullptr;
      hipError_t e = hipMalloc(reinterpret_cast<void**>(&d_hist), (size_t)nbk * sizeof(uint32_t));
      if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&d_class_start), ((size_t)n_classes + 1) * sizeof(int32_t));
      if (e != hipSuccess) {
        (void)hipGetLastError();
        st = FUSEDMM_ERR_ALLOC;
      } else {
        e = hipMemsetAsync(d_hist, 0, (size_t)nbk * sizeof(uint32_t), stream);
        if (e == hipSuccess) e = launch_column_histogram(d_colidx, nnz, stride, n, nbk, d_hist, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e == hipSuccess) e = hipMemcpy(hist.data(), d_hist, (size_t)nbk * sizeof(uint32_t), hipMemcpyDeviceToHost);
        if (e == hipSuccess) {
          uint64_t total = 0;
          for (uint32_t h : hist) total += h;
          class_start.assign((size_t)n_classes + 1, 0);
          class_start[(size_t)n_classes] = (int32_t)n;
          // A class's weight is 3/4 its share of the stored entries + 1/4 its share of the columns: a class of
          // often-gathered columns is served from the L2 and can take more entries than a wide class of rarely
          // gathered ones, whose rows of Y mostly come from memory.  (Where entries are spread evenly over the
          // columns both shares are the same.)  Measured on the workloads in their as-generated vertex order,
          // weights of the width 0 / 0.25 / 0.5 / 1: c3 5.5 / 4.9 / 5.0 / 8.8 ms, c5 15.3 / 14.6 / 15.7 / 26.7 ms.
          const double wfrac = kClassWidthWeight;
          double acc = 0.0;
          int32_t c = 1;
          for (int32_t b = 0; b < nbk && c < n_classes; ++b) {
            acc += (1.0 - wfrac) * (total ? (double)hist[(size_t)b] / (double)total : 0.0) + wfrac / (double)nbk;
            // bucket b ends class c - 1 (and any class it fills on its own) once the classes before c hold their share
            while (c < n_classes && acc * (double)n_classes >= (double)c * (1.0 - 1e-12)) {
              const int64_t first_col_after = ((int64_t)(b + 1) * n + nbk - 1) / nbk;  // first column of bucket b + 1
              class_start[(size_t)c++] = (int32_t)std::min<int64_t>(first_col_after, n);
            }
          }
          for (; c < n_classes; ++c) class_start[(size_t)c] = (int32_t)n;
          e = hipMemcpy(d_class_start, class_start.data(), class_start.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        }
        if (e != hipSuccess) st = FUSEDMM_ERR_HIP;
      }
      if (d_hist) (void)hipFree(d_hist);
      if (st != FUSEDMM_OK) {
        if (d_class_start) (void)hipFree(d_class_start);
        delete p;
        return st;
      }
    }
    if (n_classes > 1 && nnz > 0) {
      int64_t nb = 0;
      for (int64_t u = 0; u < m; ++u) {
        const int64_t deg = rp[u + 1] - rp[u];
        if (deg < tile_min) continue;
        int32_t level = kNumXcd;
        while (level < n_classes && deg >= tile_edges_per_class * 2 * level) level *= 2;
        tiled_rows.push_back((int32_t)u);
        tiled_level.push_back(level);
        bnd_off.push_back(nb);
        nb += level + 1;
      }
      if (!tiled_rows.empty()) {
        int32_t *d_rows = nullptr, *d_level = nullptr, *d_bounds = nullptr, *d_flag = nullptr;
        int64_t* d_off = nullptr;
        const size_t nt = tiled_rows.size();
        bounds.resize((size_t)nb);
        int32_t flag = 0;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&d_rows), nt * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&d_level), nt * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&d_off), nt * sizeof(int64_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&d_bounds), (size_t)nb * sizeof(int32_t));
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&d_flag), sizeof(int32_t));
        if (e != hipSuccess) {
          (void)hipGetLastError();
          st = FUSEDMM_ERR_ALLOC;
        } else {
          e = hipMemcpy(d_rows, tiled_rows.data(), nt * sizeof(int32_t), hipMemcpyHostToDevice);
          if (e == hipSuccess) e = hipMemcpy(d_level, tiled_level.data(), nt * sizeof(int32_t), hipMemcpyHostToDevice);
          if (e == hipSuccess) e = hipMemcpy(d_off, bnd_off.data(), nt * sizeof(int64_t), hipMemcpyHostToDevice);
          if (e == hipSuccess) e = hipMemcpy(d_flag, &flag, sizeof(flag), hipMemcpyHostToDevice);
          if (e == hipSuccess)
            e = launch_tile_bounds(d_rowptr, d_colidx, d_rows, d_level, d_off, (int32_t)nt, n_classes, d_class_start,
                                   d_bounds, d_flag, stream);
          if (e == hipSuccess) e = hipStreamSynchronize(stream);
          if (e == hipSuccess) e = hipMemcpy(bounds.data(), d_bounds, (size_t)nb * sizeof(int32_t), hipMemcpyDeviceToHost);
          if (e == hipSuccess) e = hipMemcpy(&flag, d_flag, sizeof(flag), hipMemcpyDeviceToHost);
          if (e != hipSuccess) st = FUSEDMM_ERR_HIP;
        }
        if (d_rows) (void)hipFree(d_rows);
        if (d_level) (void)hipFree(d_level);
        if (d_off) (void)hipFree(d_off);
        if (d_bounds) (void)hipFree(d_bounds);
        if (d_flag) (void)hipFree(d_flag);
        if (st != FUSEDMM_OK) { (void)hipFree(d_class_start); delete p; return st; }
        if (flag != 0) tiled_rows.clear();  // some long row has unsorted columns: no tiling for this pattern
      }
    }
    if (d_class_start) { (void)hipFree(d_class_start); d_class_start = nullptr; }
    const bool tiling = !tiled_rows.empty();
    const int64_t tiled_from = tiling ? tile_min : INT64_MAX;

    // length of a workgroup chunk when `count` entries are cut into chunks of at most chunk_edges:
    // equal shares, rounded up to whole batches of 64 entries for each of the 4 wavefronts
    auto chunk_len = [&](int64_t count) {
      const int64_t nc = (count + chunk - 1) / chunk;
      return ((count + nc - 1) / nc + 255) / 256 * 256;
    };

    // ---- the rows are walked twice, by T host threads over contiguous row ranges: first counted, then placed.
    // What a thread counts in the first pass becomes, by prefix sums over the threads in row order, the positions
    // it writes to in the second, so the lists are the ones a single thread walking the rows in order produces:
    // short rows sorted by length (longest first, row order kept among equals); the segments of the tiled rows
    // class by class ([chunks][wavefront segments][lane-group segments], longest first within each); partial-row
    // slots handed out in row order, so the merge order of a row is fixed by (class, chunk) and does not depend
    // on how the descriptors are arranged.  All memory is allocated here, before the threads start.
    const size_t ncls = tiling ? (size_t)n_classes : 0;
    const size_t hw = (size_t)split_min + 1;
    const int asked_threads = options ? options->host_threads : 0;
    const int T = asked_threads > 0
                      ? std::min(asked_threads, kPlanThreadsLimit)
                      : (int)std::max<int64_t>(1, std::min<int64_t>({(int64_t)kPlanThreads, (int64_t)std::thread::hardware_concurrency(),
                                                                      m / kPlanRowsPerThread}));
    struct ThreadCounts {
      std::vector<int64_t> bucket;                // short rows by length; after the prefix sums: where the next one goes
      std::vector<int64_t> cls_nchunk, cls_hist;  // tile chunks per class, shorter segments per (class, length); likewise
      int64_t n_long = 0, n_chunk_descs = 0, n_merges = 0, n_parts = 0, n_tiled = 0;
      size_t ti0 = 0;  // index in tiled_rows of the thread's first tiled row
    };
    std::vector<ThreadCounts> tc((size_t)T);
    for (int t = 0; t < T; ++t) {
      tc[(size_t)t].bucket.assign((size_t)split_min + 1, 0);
      tc[(size_t)t].cls_nchunk.assign(ncls, 0);
      tc[(size_t)t].cls_hist.assign(ncls * hw, 0);
      tc[(size_t)t].ti0 = (size_t)(std::lower_bound(tiled_rows.begin(), tiled_rows.end(), (int32_t)(m * t / T)) - tiled_rows.begin());
    }
    auto on_threads = [&](auto&& body) {
      if (T == 1) { body(0); return; }
      std::vector<std::thread> workers;
      workers.reserve((size_t)T);
      for (int t = 0; t < T; ++t) workers.emplace_back([&body, t]() { body(t); });
      for (auto& w : workers) w.join();
    };

    // first pass: count
    on_threads([&](int t) {
      ThreadCounts& c = tc[(size_t)t];
      size_t ti = c.ti0;
      for (int64_t u = m * t / T; u < m * (t + 1) / T; ++u) {
        const int64_t deg = rp[u + 1] - rp[u];
        if (deg >= tiled_from) {
          const int32_t* bnd = bounds.data() + bnd_off[ti];
          const size_t level = (size_t)tiled_level[ti], stride = ncls / level;
          ++ti;
          for (size_t k = 0; k < level; ++k) {
            const int64_t cnt = (int64_t)bnd[k + 1] - bnd[k];
            if (cnt <= 0) continue;
            const size_t cl = k * stride;  // the tile is filed under the first finest class it covers
            if (cnt > split_min) {
              const int64_t per = chunk_len(cnt);
              c.cls_nchunk[cl] += (cnt + per - 1) / per;
              c.n_parts += (cnt + per - 1) / per;
            } else {
              ++c.cls_hist[cl * hw + (size_t)cnt];
              ++c.n_parts;
            }
          }
          ++c.n_long; ++c.n_tiled; ++c.n_merges;
        } else if (deg <= split_min) {
          ++c.bucket[(size_t)deg];
        } else {
          const int64_t per = chunk_len(deg);
          const int64_t nc = (deg + per - 1) / per;
          ++c.n_long;
          c.n_chunk_descs += nc;
          if (nc > 1) { ++c.n_merges; c.n_parts += nc; }
        }
      }
    });

    // totals, the layout of the lists, and every thread's starting positions in them
    std::vector<int64_t> bucket((size_t)split_min + 1, 0), cls_nchunk(ncls, 0), cls_hist(ncls * hw, 0);
    int64_t n_long = 0, n_chunk_descs = 0, n_merge_descs = 0, n_part_slots = 0;
    for (const ThreadCounts& c : tc) {
      for (size_t i = 0; i < bucket.size(); ++i) bucket[i] += c.bucket[i];
      for (size_t i = 0; i < cls_nchunk.size(); ++i) cls_nchunk[i] += c.cls_nchunk[i];
      for (size_t i = 0; i < cls_hist.size(); ++i) cls_hist[i] += c.cls_hist[i];
      n_long += c.n_long; n_chunk_descs += c.n_chunk_descs; n_merge_descs += c.n_merges; n_part_slots += c.n_parts;
      p->n_tiled_rows += (int32_t)c.n_tiled;
    }
    if (n_part_slots >= (int64_t)INT32_MAX || n_chunk_descs >= (int64_t)INT32_MAX) { delete p; return FUSEDMM_ERR_INVALID_ARG; }
    std::vector<int64_t> start((size_t)split_min + 1, 0);
    int64_t pos = 0;
    for (int64_t deg = split_min; deg >= 0; --deg) { start[(size_t)deg] = pos; pos += bucket[(size_t)deg]; }
    int64_t n_wave = 0;
    for (int64_t deg = split_min; deg > small_max; --deg) n_wave += bucket[(size_t)deg];
    // descriptor layout: class by class, [chunks][wavefront segments][lane-group segments]
    std::vector<int64_t> cls_base(ncls + 1, 0), cls_nwave(ncls, 0), cls_nshort(ncls, 0), cls_chunk_cursor(ncls, 0);
    for (size_t c = 0; c < ncls; ++c) {
      int64_t at = cls_base[c] + cls_nchunk[c];
      cls_chunk_cursor[c] = cls_base[c];
      for (int64_t len = split_min; len >= 1; --len) {
        const int64_t h = cls_hist[c * hw + (size_t)len];
        cls_hist[c * hw + (size_t)len] = at;  // from now on: where the first segment of this length goes
        at += h;
        (len > small_max ? cls_nwave : cls_nshort)[c] += h;
      }
      cls_base[c + 1] = at;
    }
    if (ncls > 0 && cls_base[ncls] >= (int64_t)INT32_MAX) { delete p; return FUSEDMM_ERR_INVALID_ARG; }
    std::vector<int64_t> part0((size_t)T, 0), merge0((size_t)T, 0), chunk0((size_t)T, 0);
    {
      int64_t parts = 0, mrg = 0, chk = 0;
      for (int t = 0; t < T; ++t) {
        ThreadCounts& c = tc[(size_t)t];
        part0[(size_t)t] = parts; merge0[(size_t)t] = mrg; chunk0[(size_t)t] = chk;
        parts += c.n_parts; mrg += c.n_merges; chk += c.n_chunk_descs;
        // counts -> positions: what the earlier threads' rows take comes first
        for (size_t i = 0; i < start.size(); ++i) { const int64_t k = c.bucket[i]; c.bucket[i] = start[i]; start[i] += k; }
        for (size_t i = 0; i < cls_chunk_cursor.size(); ++i) {
          const int64_t k = c.cls_nchunk[i]; c.cls_nchunk[i] = cls_chunk_cursor[i]; cls_chunk_cursor[i] += k;
        }
        for (size_t i = 0; i < cls_hist.size(); ++i) { const int64_t k = c.cls_hist[i]; c.cls_hist[i] = cls_hist[i]; cls_hist[i] += k; }
      }
    }
    order.resize((size_t)(m - n_long));
    chunks.resize((size_t)n_chunk_descs);
    merges.resize((size_t)n_merge_descs);
    tile_descs.resize(ncls > 0 ? (size_t)cls_base[ncls] : 0);

    // second pass: place
    on_threads([&](int t) {
      ThreadCounts& c = tc[(size_t)t];
      size_t ti = c.ti0;
      int32_t next_part = (int32_t)part0[(size_t)t];
      int64_t next_merge = merge0[(size_t)t], next_chunk = chunk0[(size_t)t];
      for (int64_t u = m * t / T; u < m * (t + 1) / T; ++u) {
        const int64_t deg = rp[u + 1] - rp[u];
        if (deg >= tiled_from) {
          const int32_t* bnd = bounds.data() + bnd_off[ti];
          const size_t level = (size_t)tiled_level[ti], stride = ncls / level;
          ++ti;
          const int32_t first_part = next_part;
          for (size_t k = 0; k < level; ++k) {
            const int64_t cnt = (int64_t)bnd[k + 1] - bnd[k];
            if (cnt <= 0) continue;
            const size_t cl = k * stride;
            const int64_t e_begin = rp[u] + bnd[k];
            if (cnt > split_min) {
              const int64_t per = chunk_len(cnt);
              for (int64_t off = 0; off < cnt; off += per)
                tile_descs[(size_t)c.cls_nchunk[cl]++] =
                    ChunkDesc{e_begin + off, (int32_t)std::min<int64_t>(per, cnt - off), (int32_t)u, next_part++, 0};
            } else {
              tile_descs[(size_t)c.cls_hist[cl * hw + (size_t)cnt]++] = ChunkDesc{e_begin, (int32_t)cnt, (int32_t)u, next_part++, 0};
            }
          }
          merges[(size_t)next_merge++] = MergeDesc{(int32_t)u, first_part, next_part - first_part, 0};
        } else if (deg <= split_min) {
          order[(size_t)c.bucket[(size_t)deg]++] = (int32_t)u;
        } else {
          const int64_t per = chunk_len(deg);
          const int32_t nc = (int32_t)((deg + per - 1) / per);
          if (nc > 1) merges[(size_t)next_merge++] = MergeDesc{(int32_t)u, next_part, nc, 0};
          for (int64_t off = 0; off < deg; off += per)
            chunks[(size_t)next_chunk++] = ChunkDesc{rp[u] + off, (int32_t)std::min<int64_t>(per, deg - off), (int32_t)u,
                                                     nc > 1 ? next_part++ : -1, 0};
        }
      }
    });
    const int32_t next_part = (int32_t)n_part_slots;

    // ---- deal the classes to the XCDs: XCD k owns the k-th eighth of the column range and works
    // through its finest classes in order; coarser tiles sit where their first finest class is ----
    if (tiling) {
      std::vector<std::vector<BlockItem>> xcd_items(kNumXcd);
      for (size_t c = 0; c < ncls; ++c) {
        auto& lst = xcd_items[c / (ncls / kNumXcd)];
        int64_t at = cls_base[c];
        for (int64_t k = 0; k < cls_nchunk[c]; ++k) lst.push_back(BlockItem{kItemChunk, (int32_t)(at++), 1, 0});
        for (int64_t k = 0; k < cls_nwave[c]; k += kWavesPerBlock) {
          const int32_t cnt = (int32_t)std::min<int64_t>(kWavesPerBlock, cls_nwave[c] - k);
          lst.push_back(BlockItem{kItemWave, (int32_t)at, cnt, 0});
          at += cnt;
        }
        for (int64_t k = 0; k < cls_nshort[c]; k += kPackedSegsPerItem) {
          const int32_t cnt = (int32_t)std::min<int64_t>(kPackedSegsPerItem, cls_nshort[c] - k);
          lst.push_back(BlockItem{kItemPacked, (int32_t)at, cnt, 0});
          at += cnt;
        }
      }
      size_t longest = 0;
      for (const auto& lst : xcd_items) longest = std::max(longest, lst.size());
      items.assign(longest * kNumXcd, BlockItem{kItemNone, 0, 0, 0});
      for (int k = 0; k < kNumXcd; ++k)
        for (size_t j = 0; j < xcd_items[(size_t)k].size(); ++j) items[j * kNumXcd + (size_t)k] = xcd_items[(size_t)k][j];
      p->n_classes = n_classes;
    }
    if (tile_descs.size() >= (size_t)INT32_MAX || items.size() >= (size_t)INT32_MAX) { delete p; return FUSEDMM_ERR_INVALID_ARG; }
    p->n_wave = (int32_t)n_wave;
    p->n_empty = (int32_t)bucket[0];  // they sort last: zero-filled by workgroups of their own
    p->n_packed = (int32_t)((m - n_long) - n_wave - bucket[0]);
    p->n_chunks = (int32_t)chunks.size();
    p->n_merges = (int32_t)merges.size();
    p->n_parts = next_part;
    p->n_items = (int32_t)items.size();
    p->n_tile_descs = (int32_t)tile_descs.size();
  } catch (const std::bad_alloc&) {
    if (d_class_start) (void)hipFree(d_class_start);
    delete p;
    return FUSEDMM_ERR_ALLOC;
  }

  // ---- the general kernel's segments: rows longer than kGenericSplit, cut into runs of that length
  std::vector<ChunkDesc> gen_segs;
  std::vector<MergeDesc> gen_merges;
  try {
    for (int64_t u = 0; u < m; ++u) {
      const int64_t deg = rp[u + 1] - rp[u];
      if (deg <= kGenericSplit) continue;
      const int32_t first = (int32_t)gen_segs.size();
      for (int64_t off = 0; off < deg; off += kGenericSplit)
        gen_segs.push_back(ChunkDesc{rp[u] + off, (int32_t)std::min<int64_t>(kGenericSplit, deg - off), (int32_t)u,
                                     (int32_t)gen_segs.size(), 0});
      gen_merges.push_back(MergeDesc{(int32_t)u, first, (int32_t)gen_segs.size() - first, 0});
      if (gen_segs.size() >= (size_t)INT32_MAX / 2) { delete p; return FUSEDMM_ERR_INVALID_ARG; }
    }
  } catch (const std::bad_alloc&) {
    delete p;
    return FUSEDMM_ERR_ALLOC;
  }
  p->n_gen_segs = (int32_t)gen_segs.size();
  p->n_gen_merges = (int32_t)gen_merges.size();

  st = upload(&p->d_order, order, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_gen_segs, gen_segs, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_gen_merges, gen_merges, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_chunks, chunks, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_merges, merges, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_items, items, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_tile_descs, tile_descs, stream);
  if (st == FUSEDMM_OK && hipStreamSynchronize(stream) != hipSuccess) st = FUSEDMM_ERR_HIP;
  // the address of the static scratch on this device is looked up here, once, so that
  // fusedmm_execute_static_scratch finds it in place (its own first call would look it up otherwise)
  if (st == FUSEDMM_OK) {
    void* unused = nullptr;
    (void)static_scratch_for_current_device(&unused);  // a failure is reported by that entry point, not here
  }
  // the scratch of the hinted dimension, so that execute never has to allocate
  if (st == FUSEDMM_OK) st = fusedmm_plan_reserve(p, std::min<int32_t>(d_hint, FUSEDMM_MAX_D));
  if (st != FUSEDMM_OK) {
    free_plan_device(p);
    delete p;
    return st;
  }
  *out = p;
  return FUSEDMM_OK;
}

int fusedmm_plan_reserve(fusedmm_plan_t* plan, int32_t d) {
  if (!plan) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  // every dimension <= d: the largest instance size one of them runs on, and the general kernel's rows of d elements
  int st = ensure_partials(plan, partial_floats_f32(d));
  if (st == FUSEDMM_OK) st = ensure_gen_partials(plan, d, sizeof(float));
  return st;
}

int fusedmm_plan_reserve_f64(fusedmm_plan_t* plan, int32_t d) {
  if (!plan) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  int st = ensure_partials(plan, partial_floats_f64(d));
  if (st == FUSEDMM_OK) st = ensure_gen_partials(plan, d, sizeof(double));
  return st;
}

int fusedmm_plan_workspace_bytes(const fusedmm_plan_t* plan, int32_t d, size_t* out) {
  if (!plan || !out) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  size_t b = (size_t)(plan->n_wave + plan->n_packed + plan->n_empty) * sizeof(int32_t) + (size_t)plan->n_chunks * sizeof(ChunkDesc) +
             (size_t)plan->n_merges * sizeof(MergeDesc) + (size_t)plan->n_items * sizeof(BlockItem) +
             (size_t)plan->n_tile_descs * sizeof(ChunkDesc);
  b += (size_t)plan->n_gen_segs * sizeof(ChunkDesc) + (size_t)plan->n_gen_merges * sizeof(MergeDesc);
  // what the plan holds once fusedmm_plan_reserve(plan, d) has run: partial rows of both kernels
  b += (size_t)plan->n_parts * (size_t)std::max(partial_floats_f32(d), plan->partials_d) * sizeof(float);
  b += std::max((size_t)plan->n_gen_segs * (size_t)d * sizeof(float), plan->gen_partials_bytes);
  *out = b;
  return FUSEDMM_OK;
}

int fusedmm_plan_stats(const fusedmm_plan_t* plan, int64_t* n_packed_rows, int64_t* n_wave_rows, int64_t* n_chunks,
                       int64_t* n_split_rows, int64_t* n_partials, int64_t* n_tiled_rows, int64_t* n_tile_segments,
                       int64_t* n_column_classes) {
  if (!plan) return FUSEDMM_ERR_INVALID_ARG;
  if (n_packed_rows) *n_packed_rows = plan->n_packed + plan->n_empty;
  if (n_wave_rows) *n_wave_rows = plan->n_wave;
  if (n_chunks) *n_chunks = plan->n_chunks;
  if (n_split_rows) *n_split_rows = plan->n_merges;
  if (n_partials) *n_partials = plan->n_parts;
  if (n_tiled_rows) *n_tiled_rows = plan->n_tiled_rows;
  if (n_tile_segments) *n_tile_segments = plan->n_tile_descs;
  if (n_column_classes) *n_column_classes = plan->n_classes;
  return FUSEDMM_OK;
}

namespace {

// Shared body of fusedmm_execute, fusedmm_execute_bf16y and fusedmm_execute_f16y.  y_format other than
// kYF32: d_Y points at rows of 2-byte elements (ldy in elements); only the fast instances exist for those.
// static_scratch: null = the partial rows live in the plan's own scratch; else they go to this buffer of
// FUSEDMM_STATIC_SCRATCH_BYTES (fusedmm_execute_static_scratch), whatever the plan has reserved.
int execute_impl(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d, const float* d_values, const float* d_X,
                 int64_t ldx, const void* d_Y, int y_format, int64_t ldy, float* d_Z, int64_t ldz, void* stream_,
                 bool allow_private = false, void* static_scratch = nullptr) {
  const bool y_bf16 = y_format != kYF32;  // any 2-byte storage
  if (!plan || !ops) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  if (!ops_valid(*ops, allow_private)) return FUSEDMM_ERR_UNSUPPORTED_OPS;
  const bool uses_x = ops->vop != FUSEDMM_VOP_SEL2ND;
  const bool uses_val = ops->sop == FUSEDMM_SOP_EDGE_VALUE || ops->sop == kSopValueMinusSigmoid;
  if (plan->m == 0) return FUSEDMM_OK;
  if (!d_Z || ldz < d) return FUSEDMM_ERR_INVALID_ARG;
  if (plan->nnz > 0) {
    if (!d_Y || ldy < d) return FUSEDMM_ERR_INVALID_ARG;
    if (uses_val && !d_values) return FUSEDMM_ERR_INVALID_ARG;
  }
  if (uses_x && (!d_X || ldx < d)) return FUSEDMM_ERR_INVALID_ARG;
  // Z against Y: compare byte ranges (a bfloat16 row is half as long)
  {
    const uintptr_t z0 = reinterpret_cast<uintptr_t>(d_Z);
    const uintptr_t z1 = z0 + (uintptr_t)((plan->m - 1) * ldz + d) * sizeof(float);
    const uintptr_t y0 = reinterpret_cast<uintptr_t>(d_Y);
    const uintptr_t y1 = y0 + (uintptr_t)((plan->n > 0 ? plan->n - 1 : 0) * ldy + d) * (y_bf16 ? 2u : 4u);
    if (d_Y && plan->n > 0 && z0 < y1 && y0 < z1) return FUSEDMM_ERR_ALIAS;
  }
  if (uses_x && overlaps(d_Z, plan->m, ldz, d_X, plan->m, ldx, d)) return FUSEDMM_ERR_ALIAS;
  if (uses_val && plan->nnz > 0) {  // the edge values are read while Z is written
    const uintptr_t z0 = reinterpret_cast<uintptr_t>(d_Z);
    const uintptr_t z1 = z0 + (uintptr_t)((plan->m - 1) * ldz + d) * sizeof(float);
    const uintptr_t v0 = reinterpret_cast<uintptr_t>(d_values), v1 = v0 + (uintptr_t)plan->nnz * sizeof(float);
    if (z0 < v1 && v0 < z1) return FUSEDMM_ERR_ALIAS;
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);

  // d = 2, 3, 4, 8, 16: the one-lane-per-entry kernels; 9 ... 1024: the wide kernels, on the instance of d itself
  // or the next larger one (choose_pattern says in which form); everything else, and every call of a plan that
  // asks for it: the general kernel.  2-byte storage of Y exists on the wide kernels only (d = 8, 16, 24 ... 512).
  const bool small = !y_bf16 && is_small_dim(d) && !plan->general_only;  // one lane per stored entry
  const int32_t D = y_bf16 ? instance_dim_2byte(d) : instance_dim(d);
  const int recognised = recognise(*ops);
  const int family = recognise_family(*ops);
  const int pattern = choose_pattern(recognised, family, d, D);
  // fp32 rows may start anywhere (the kernels read and write them as element-aligned vectors); rows of 2-byte
  // elements are read 16 bytes at a time and have to be aligned to that
  const bool y_ok = plan->nnz == 0 || !y_bf16 || (aligned16(d_Y) && ldy % 8 == 0);
  // the fast kernels address a row of Y by a 32-bit pitch in bytes
  const bool fast = D != 0 && ldy < (int64_t(1) << 29) && y_ok && (y_bf16 || !plan->general_only);
  if (y_bf16 && !fast) return D != 0 ? FUSEDMM_ERR_INVALID_ARG : FUSEDMM_ERR_UNSUPPORTED_DIM;

  hipEvent_t ev0 = nullptr, ev1 = nullptr, ev2 = nullptr;
  if (plan->profiling && plan->events_used < plan->events.size()) {
    ev0 = plan->events[plan->events_used].before;
    ev1 = plan->events[plan->events_used].after;
    ev2 = plan->events[plan->events_used].after2;
  }

  hipError_t e = hipSuccess;
  if (small && ldy < (int64_t(1) << 29)) {
    if (static_scratch) {
      if ((size_t)plan->n_parts * kSmallPartialStride * sizeof(float) > (size_t)FUSEDMM_STATIC_SCRATCH_BYTES) return FUSEDMM_ERR_SCRATCH_LIMIT;
    } else if (plan->n_parts > 0 && kSmallPartialStride > plan->partials_d) {
      return FUSEDMM_ERR_NOT_RESERVED;
    }
    float* partials = static_scratch ? static_cast<float*>(static_scratch) : plan->d_partials;
    KernelArgs a;
    fill_schedule_args(plan, d, kYF32, &a);
    a.partials = partials;
    a.d_pieces = a.d_full = a.d_tail = 0;
    a.values = d_values; a.X = d_X; a.Y = d_Y; a.Z = d_Z;
    a.ldx = ldx; a.ldy = ldy; a.ldz = ldz;
    a.alpha = ops->alpha;
    a.vop = ops->vop; a.rop = ops->rop; a.sop = ops->sop; a.mop = ops->mop;
    a.mean = ops->aop == FUSEDMM_AOP_MEAN;
    a.aop = a.mean ? FUSEDMM_AOP_SUM : ops->aop;
    if (ev0) (void)hipEventRecord(ev0, stream);
    e = launch_small(recognised, d, a, stream);
    if (ev0) { (void)hipEventRecord(ev1, stream); (void)hipEventRecord(ev2, stream); ++plan->events_used; }
    if (e == hipSuccess)
      e = launch_small_merge(plan->d_merges, plan->n_merges, partials, d, ops->aop, plan->d_rowptr, d_Z, ldz, stream);
  } else if (fast) {
    if (static_scratch) {
      if ((size_t)plan->n_parts * (size_t)D * sizeof(float) > (size_t)FUSEDMM_STATIC_SCRATCH_BYTES) return FUSEDMM_ERR_SCRATCH_LIMIT;
    } else if (plan->n_parts > 0 && D > plan->partials_d) {
      return FUSEDMM_ERR_NOT_RESERVED;
    }
    float* partials = static_scratch ? static_cast<float*>(static_scratch) : plan->d_partials;
    KernelArgs a;
    fill_schedule_args(plan, D, y_format, &a);
    a.partials = partials;
    a.d_full = d / 4; a.d_tail = d % 4; a.d_pieces = (d + 3) / 4;
    a.values = d_values; a.X = d_X; a.Y = d_Y; a.Z = d_Z;
    a.ldx = ldx; a.ldy = ldy; a.ldz = ldz;
    fill_op_args(*ops, &a);
    if (ev0) (void)hipEventRecord(ev0, stream);
    e = launch_fast(pattern, D, y_format, a, stream);
    if (ev0) { (void)hipEventRecord(ev1, stream); (void)hipEventRecord(ev2, stream); ++plan->events_used; }
    // partial rows are stored with the instance size as their stride, whatever the scratch capacity is
    if (e == hipSuccess)
      e = launch_merge(plan->d_merges, plan->n_merges, partials, d, D, ops->aop, plan->d_rowptr, d_Z, ldz, stream);
  } else {
    GenericArgs g;
    g.rowptr = plan->d_rowptr; g.colidx = plan->d_colidx; g.values = d_values;
    g.X = d_X; g.Y = static_cast<const float*>(d_Y); g.Z = d_Z;
    g.ldx = ldx; g.ldy = ldy; g.ldz = ldz;
    g.m = plan->m; g.d = d;
    g.vop = ops->vop; g.rop = ops->rop; g.sop = ops->sop; g.mop = ops->mop; g.aop = ops->aop;
    g.alpha = ops->alpha;
    g.visit_counts = nullptr;
    const size_t gen_need = (size_t)plan->n_gen_segs * (size_t)d * sizeof(float);
    if (static_scratch) {
      if (gen_need > (size_t)FUSEDMM_STATIC_SCRATCH_BYTES) return FUSEDMM_ERR_SCRATCH_LIMIT;
    } else if (gen_need > plan->gen_partials_bytes) {
      return FUSEDMM_ERR_NOT_RESERVED;
    }
    fill_generic_segments(plan, &g);
    if (static_scratch) g.partials = static_cast<float*>(static_scratch);
    if (ev0) (void)hipEventRecord(ev0, stream);
    e = launch_generic(g, stream);
    if (ev0) { (void)hipEventRecord(ev1, stream); (void)hipEventRecord(ev2, stream); ++plan->events_used; }
  }
  return e == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
}

}  // namespace

}  // extern "C"

int fusedmm_execute_private_ops(fusedmm_plan* plan, const fusedmm_ops* ops, int32_t d, const float* d_values,
                                const float* d_X, int64_t ldx, const float* d_Y, int64_t ldy, float* d_Z, int64_t ldz,
                                void* stream) {
  return execute_impl(plan, ops, d, d_values, d_X, ldx, d_Y, kYF32, ldy, d_Z, ldz, stream, true);
}

extern "C" {

int fusedmm_execute(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d, const float* d_values, const float* d_X,
                    int64_t ldx, const float* d_Y, int64_t ldy, float* d_Z, int64_t ldz, void* stream_) {
  return execute_impl(plan, ops, d, d_values, d_X, ldx, d_Y, kYF32, ldy, d_Z, ldz, stream_);
}

int fusedmm_execute_static_scratch(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d, const float* d_values,
                                   const float* d_X, int64_t ldx, const float* d_Y, int64_t ldy, float* d_Z, int64_t ldz,
                                   void* stream_) {
  void* ptr = nullptr;
  const int st = static_scratch_for_current_device(&ptr);
  if (st != FUSEDMM_OK) return st;
  // nothing in the scratch has to start at zero: every partial row a merge reads was written by this call
  return execute_impl(plan, ops, d, d_values, d_X, ldx, d_Y, kYF32, ldy, d_Z, ldz, stream_, false, ptr);
}

int fusedmm_execute_bf16y(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d, const float* d_values,
                          const float* d_X, int64_t ldx, const uint16_t* d_Y_bf16, int64_t ldy, float* d_Z, int64_t ldz,
                          void* stream_) {
  return execute_impl(plan, ops, d, d_values, d_X, ldx, d_Y_bf16, kYBf16, ldy, d_Z, ldz, stream_);
}

int fusedmm_execute_f16y(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d, const float* d_values,
                         const float* d_X, int64_t ldx, const uint16_t* d_Y_f16, int64_t ldy, float* d_Z, int64_t ldz,
                         void* stream_) {
  return execute_impl(plan, ops, d, d_values, d_X, ldx, d_Y_f16, kYF16, ldy, d_Z, ldz, stream_);
}

int fusedmm_execute_f64(fusedmm_plan_t* plan, const fusedmm_ops_t* ops, int32_t d, const double* d_values,
                        const double* d_X, int64_t ldx, const double* d_Y, int64_t ldy, double* d_Z, int64_t ldz,
                        void* stream_) {
  if (!plan || !ops) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  if (!ops_valid(*ops)) return FUSEDMM_ERR_UNSUPPORTED_OPS;
  const bool uses_x = ops->vop != FUSEDMM_VOP_SEL2ND;
  if (plan->m == 0) return FUSEDMM_OK;
  if (!d_Z || ldz < d) return FUSEDMM_ERR_INVALID_ARG;
  if (plan->nnz > 0) {
    if (!d_Y || ldy < d) return FUSEDMM_ERR_INVALID_ARG;
    if (ops->sop == FUSEDMM_SOP_EDGE_VALUE && !d_values) return FUSEDMM_ERR_INVALID_ARG;
  }
  if (uses_x && (!d_X || ldx < d)) return FUSEDMM_ERR_INVALID_ARG;
  auto range = [d](const double* p, int64_t rows, int64_t ld, uintptr_t* lo, uintptr_t* hi) {
    *lo = reinterpret_cast<uintptr_t>(p);
    *hi = *lo + (uintptr_t)((rows > 0 ? rows - 1 : 0) * ld + d) * sizeof(double);
  };
  uintptr_t z0, z1, o0, o1;
  range(d_Z, plan->m, ldz, &z0, &z1);
  if (d_Y && plan->n > 0) {
    range(d_Y, plan->n, ldy, &o0, &o1);
    if (z0 < o1 && o0 < z1) return FUSEDMM_ERR_ALIAS;
  }
  if (uses_x) {
    range(d_X, plan->m, ldx, &o0, &o1);
    if (z0 < o1 && o0 < z1) return FUSEDMM_ERR_ALIAS;
  }
  if (ops->sop == FUSEDMM_SOP_EDGE_VALUE && plan->nnz > 0) {
    o0 = reinterpret_cast<uintptr_t>(d_values);
    o1 = o0 + (uintptr_t)plan->nnz * sizeof(double);
    if (z0 < o1 && o0 < z1) return FUSEDMM_ERR_ALIAS;
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // the specialised schedule in double precision: the same dispatch as fp32 (a recognised pattern at an instance
  // size, else its tuple family, else the ops at run time) on row registers of four doubles
  const int32_t D = instance_dim_f64(d);
  const bool fast = D != 0 && ldy < (int64_t(1) << 28) && !plan->general_only;
  if (fast) {
    if (plan->n_parts > 0 && 2 * D > plan->partials_d) return FUSEDMM_ERR_NOT_RESERVED;
    const int recognised = recognise(*ops);
    const int family = recognise_family(*ops);
    const int pattern = choose_pattern(recognised, family, d, D);
    KernelArgs a;
    fill_schedule_args(plan, D, kYF64, &a);
    fill_op_args(*ops, &a);
    a.d_full = d / 4; a.d_tail = d % 4; a.d_pieces = (d + 3) / 4;
    a.values = d_values; a.X = d_X; a.Y = d_Y; a.Z = d_Z;
    a.ldx = ldx; a.ldy = ldy; a.ldz = ldz;
    hipEvent_t ev0 = nullptr, ev1 = nullptr, ev2 = nullptr;
    if (plan->profiling && plan->events_used < plan->events.size()) {
      ev0 = plan->events[plan->events_used].before;
      ev1 = plan->events[plan->events_used].after;
      ev2 = plan->events[plan->events_used].after2;
    }
    if (ev0) (void)hipEventRecord(ev0, stream);
    hipError_t e = launch_fast(pattern, D, kYF64, a, stream);
    if (ev0) { (void)hipEventRecord(ev1, stream); (void)hipEventRecord(ev2, stream); ++plan->events_used; }
    if (e == hipSuccess)
      e = launch_merge(plan->d_merges, plan->n_merges, reinterpret_cast<const double*>(plan->d_partials), d, D, ops->aop,
                       plan->d_rowptr, d_Z, ldz, stream);
    return e == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
  }
  GenericArgsT<double> g;
  g.rowptr = plan->d_rowptr; g.colidx = plan->d_colidx; g.values = d_values;
  g.X = d_X; g.Y = d_Y; g.Z = d_Z;
  g.ldx = ldx; g.ldy = ldy; g.ldz = ldz;
  g.m = plan->m; g.d = d;
  g.vop = ops->vop; g.rop = ops->rop; g.sop = ops->sop; g.mop = ops->mop; g.aop = ops->aop;
  g.alpha = (double)ops->alpha;
  g.visit_counts = nullptr;
  if ((size_t)plan->n_gen_segs * (size_t)d * sizeof(double) > plan->gen_partials_bytes) return FUSEDMM_ERR_NOT_RESERVED;
  fill_generic_segments(plan, &g);
  return launch_generic(g, stream) == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
}

int fusedmm_to_f16(uint16_t* d_dst, const float* d_src, size_t count, void* stream_) {
  if (count > 0 && (!d_dst || !d_src)) return FUSEDMM_ERR_INVALID_ARG;
  return launch_to_f16(d_dst, d_src, count, static_cast<hipStream_t>(stream_)) == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
}

int fusedmm_to_bf16(uint16_t* d_dst, const float* d_src, size_t count, void* stream_) {
  if (count == 0) return FUSEDMM_OK;
  if (!d_dst || !d_src) return FUSEDMM_ERR_INVALID_ARG;
  return launch_to_bf16(d_dst, d_src, count, static_cast<hipStream_t>(stream_)) == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
}

int fusedmm_debug_edge_visits(fusedmm_plan_t* plan, int32_t d, int32_t fast_path, uint32_t* d_counts, void* stream_) {
  if (!plan) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  if (fast_path < 0 || fast_path > 2) return FUSEDMM_ERR_INVALID_ARG;
  if (fast_path == 1 && !instance_dim(d) && !is_small_dim(d)) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  if (fast_path == 2 && !instance_dim_f64(d)) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  if (plan->m == 0 || plan->nnz == 0) return FUSEDMM_OK;
  if (!d_counts) return FUSEDMM_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  hipError_t e;
  if (fast_path) {
    KernelArgs a;
    const int fmt = fast_path == 2 ? kYF64 : kYF32;
    const int32_t D = fast_path == 2 ? instance_dim_f64(d)
                                     : (is_small_dim(d) ? 0 : instance_dim(d));  // 0: the kernels for very short feature vectors
    fill_schedule_args(plan, D ? D : d, fmt, &a);
    a.values = nullptr; a.X = nullptr; a.Y = nullptr; a.Z = nullptr;
    a.ldx = a.ldy = a.ldz = d;
    a.alpha = 0.f;
    a.vop = a.rop = a.sop = a.mop = a.aop = a.mean = 0;
    a.d_full = d / 4; a.d_tail = d % 4; a.d_pieces = (d + 3) / 4;
    a.visit_counts = d_counts;
    e = D == 0 ? launch_small(PAT_VISIT, d, a, stream) : launch_fast(PAT_VISIT, D, fmt, a, stream);
  } else {
    GenericArgs g = {};
    g.rowptr = plan->d_rowptr; g.colidx = plan->d_colidx;
    g.m = plan->m; g.d = d;
    g.visit_counts = d_counts;
    fill_generic_segments(plan, &g);  // the same cut of the long rows as an execute (no partial rows are written)
    e = launch_generic(g, stream);
  }
  return e == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
}

int fusedmm_plan_set_profiling(fusedmm_plan_t* plan, int32_t enabled) {
  if (!plan) return FUSEDMM_ERR_INVALID_ARG;
  plan->profiling = enabled != 0;
  plan->events_used = 0;
  if (plan->profiling && plan->events.empty()) {
    try {
      plan->events.reserve(kMaxProfiledCalls);
    } catch (const std::bad_alloc&) {
      return FUSEDMM_ERR_ALLOC;
    }
    for (size_t i = 0; i < kMaxProfiledCalls; ++i) {
      hipEvent_t a, b, c;
      if (hipEventCreate(&a) != hipSuccess) return FUSEDMM_ERR_HIP;
      if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return FUSEDMM_ERR_HIP; }
      if (hipEventCreate(&c) != hipSuccess) { (void)hipEventDestroy(a); (void)hipEventDestroy(b); return FUSEDMM_ERR_HIP; }
      plan->events.push_back(fusedmm_plan::EventTriple{a, b, c});
    }
  }
  return FUSEDMM_OK;
}

int fusedmm_plan_read_profile(fusedmm_plan_t* plan, double* main_kernel_ms_sum, double* empty_bracket_ms_sum,
                              int64_t* calls) {
  if (!plan || !main_kernel_ms_sum || !empty_bracket_ms_sum || !calls) return FUSEDMM_ERR_INVALID_ARG;
  double sum = 0.0, empty = 0.0;
  for (size_t i = 0; i < plan->events_used; ++i) {
    const auto& ev = plan->events[i];
    if (hipEventSynchronize(ev.after2) != hipSuccess) return FUSEDMM_ERR_HIP;
    float ms = 0.f, ms0 = 0.f;
    if (hipEventElapsedTime(&ms, ev.before, ev.after) != hipSuccess) return FUSEDMM_ERR_HIP;
    if (hipEventElapsedTime(&ms0, ev.after, ev.after2) != hipSuccess) return FUSEDMM_ERR_HIP;
    sum += ms;
    empty += ms0;
  }
  *main_kernel_ms_sum = sum;
  *empty_bracket_ms_sum = empty;
  *calls = (int64_t)plan->events_used;
  plan->events_used = 0;
  return FUSEDMM_OK;
}

int fusedmm_plan_read_profile_samples(fusedmm_plan_t* plan, double* main_kernel_ms, double* empty_bracket_ms,
                                      int64_t capacity, int64_t* calls) {
  if (!plan || !main_kernel_ms || !empty_bracket_ms || !calls || capacity < 0) return FUSEDMM_ERR_INVALID_ARG;
  const size_t n = plan->events_used < (size_t)capacity ? plan->events_used : (size_t)capacity;
  for (size_t i = 0; i < n; ++i) {
    const auto& ev = plan->events[i];
    if (hipEventSynchronize(ev.after2) != hipSuccess) return FUSEDMM_ERR_HIP;
    float ms = 0.f, ms0 = 0.f;
    if (hipEventElapsedTime(&ms, ev.before, ev.after) != hipSuccess) return FUSEDMM_ERR_HIP;
    if (hipEventElapsedTime(&ms0, ev.after, ev.after2) != hipSuccess) return FUSEDMM_ERR_HIP;
    main_kernel_ms[i] = ms;
    empty_bracket_ms[i] = ms0;
  }
  *calls = (int64_t)n;
  plan->events_used = 0;
  return FUSEDMM_OK;
}

int fusedmm_plan_create_tuned(fusedmm_plan_t** out, int64_t m, int64_t n, int64_t nnz, const int64_t* d_rowptr,
                              const int32_t* d_colidx, const fusedmm_ops_t* ops, int32_t d, const float* d_values,
                              const float* d_X, int64_t ldx, const float* d_Y, int64_t ldy, float* d_Z, int64_t ldz,
                              void* stream_, fusedmm_plan_options_t* chosen, float* best_ms) {
  if (!out || !ops) return FUSEDMM_ERR_INVALID_ARG;
  *out = nullptr;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  constexpr int kMaxTimed = 11;
  hipEvent_t ev[kMaxTimed + 1] = {};
  for (auto& e : ev)
    if (hipEventCreate(&e) != hipSuccess) {
      for (auto& f : ev) if (f) (void)hipEventDestroy(f);
      return FUSEDMM_ERR_HIP;
    }

  // Median time of one execute under a plan built with `opt`; the plan is returned in *made.
  auto measure = [&](const fusedmm_plan_options_t& opt, fusedmm_plan_t** made, float* median_ms) -> int {
    *made = nullptr;
    fusedmm_plan_t* p = nullptr;
    int st = fusedmm_plan_create(&p, m, n, nnz, d_rowptr, d_colidx, &opt, stream_);
    if (st != FUSEDMM_OK) return st;
    // two untimed executes, the second one timed to size the sample: 11 executes, fewer for kernels of several ms
    float first_ms = 0.f;
    for (int it = 0; it < 2 && st == FUSEDMM_OK; ++it) {
      if (hipEventRecord(ev[0], stream) != hipSuccess) st = FUSEDMM_ERR_HIP;
      if (st == FUSEDMM_OK) st = fusedmm_execute(p, ops, d, d_values, d_X, ldx, d_Y, ldy, d_Z, ldz, stream_);
      if (st == FUSEDMM_OK && (hipEventRecord(ev[1], stream) != hipSuccess || hipEventSynchronize(ev[1]) != hipSuccess ||
                               hipEventElapsedTime(&first_ms, ev[0], ev[1]) != hipSuccess))
        st = FUSEDMM_ERR_HIP;
    }
    const int timed = first_ms > 20.f ? 3 : (first_ms > 5.f ? 5 : kMaxTimed);
    for (int it = 0; it < timed && st == FUSEDMM_OK; ++it) {
      if (it == 0 && hipEventRecord(ev[0], stream) != hipSuccess) st = FUSEDMM_ERR_HIP;
      if (st == FUSEDMM_OK) st = fusedmm_execute(p, ops, d, d_values, d_X, ldx, d_Y, ldy, d_Z, ldz, stream_);
      if (st == FUSEDMM_OK && hipEventRecord(ev[it + 1], stream) != hipSuccess) st = FUSEDMM_ERR_HIP;
    }
    if (st == FUSEDMM_OK && hipEventSynchronize(ev[timed]) != hipSuccess) st = FUSEDMM_ERR_HIP;
    float ms[kMaxTimed];
    for (int it = 0; it < timed && st == FUSEDMM_OK; ++it)
      if (hipEventElapsedTime(&ms[it], ev[it], ev[it + 1]) != hipSuccess) st = FUSEDMM_ERR_HIP;
    if (st != FUSEDMM_OK) {
      (void)fusedmm_plan_destroy(p);
      return st;
    }
    std::sort(ms, ms + timed);
    *median_ms = ms[timed / 2];
    *made = p;
    return FUSEDMM_OK;
  };

  // The incumbent starts as the default plan, so the result is never slower than fusedmm_plan_create's
  // (beyond timing noise: a candidate has to win by 1 %).  Then one knob at a time is varied around the
  // incumbent, in the order of their measured influence: column classes, shortest tiled row, chunk length,
  // and the two row-length thresholds of the bins.
  fusedmm_plan_options_t best_opt = {};
  best_opt.feature_dim_hint = d;
  fusedmm_plan_t* best = nullptr;
  float best_time = 0.f;
  int st = measure(best_opt, &best, &best_time);
  auto consider = [&](fusedmm_plan_options_t opt) {
    if (st != FUSEDMM_OK) return;
    fusedmm_plan_t* p = nullptr;
    float t = 0.f;
    st = measure(opt, &p, &t);
    if (st != FUSEDMM_OK) return;
    if (t < 0.99f * best_time) {
      (void)fusedmm_plan_destroy(best);
      best = p; best_time = t; best_opt = opt;
    } else {
      (void)fusedmm_plan_destroy(p);
    }
  };
  if (st == FUSEDMM_OK) {
    const int32_t default_classes = best->n_classes;
    for (int32_t c : {1, 8, 16, 32, 64, 128}) {
      if (c == default_classes) continue;
      fusedmm_plan_options_t o = best_opt;
      o.column_classes = c;
      consider(o);
    }
    if (st == FUSEDMM_OK && best->n_classes > 1)
      for (int32_t t : {64, 256}) {
        fusedmm_plan_options_t o = best_opt;
        o.column_classes = best->n_classes;
        o.tile_row_min = t;
        consider(o);
      }
    for (int32_t c : {512, 2048}) { fusedmm_plan_options_t o = best_opt; o.chunk_edges = c; consider(o); }
    for (int32_t v : {256, 1024}) { fusedmm_plan_options_t o = best_opt; o.split_row_min = v; consider(o); }
    for (int32_t v : {32, 128}) { fusedmm_plan_options_t o = best_opt; o.small_row_max = v; consider(o); }
  }
  for (auto& e : ev) (void)hipEventDestroy(e);
  if (st != FUSEDMM_OK) {
    if (best) (void)fusedmm_plan_destroy(best);
    return st;
  }
  *out = best;
  if (chosen) {
    *chosen = best_opt;  // what was asked of fusedmm_plan_create, with the values the plan resolved them to
    chosen->small_row_max = best->small_row_max;
    chosen->split_row_min = best->split_row_min;
    chosen->chunk_edges = best->chunk_edges;
    chosen->column_classes = best->n_classes;
    chosen->tile_row_min = best->tile_row_min;
  }
  if (best_ms) *best_ms = best_time;
  return FUSEDMM_OK;
}

int fusedmm_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* stream_) {
  if (bytes == 0) return FUSEDMM_OK;
  if (!d_dst || !d_src || bytes % 16 != 0 || !aligned16(d_dst) || !aligned16(d_src)) return FUSEDMM_ERR_INVALID_ARG;
  const uintptr_t a = reinterpret_cast<uintptr_t>(d_dst), b = reinterpret_cast<uintptr_t>(d_src);
  if (a < b + bytes && b < a + bytes) return FUSEDMM_ERR_ALIAS;
  return launch_copy(d_dst, d_src, bytes, static_cast<hipStream_t>(stream_)) == hipSuccess ? FUSEDMM_OK : FUSEDMM_ERR_HIP;
}

int fusedmm_plan_destroy(fusedmm_plan_t* plan) {
  if (!plan) return FUSEDMM_OK;
  free_plan_device(plan);
  delete plan;
  return FUSEDMM_OK;
}

}  // extern "C"
