// Host side of libfusedmm.so: the C ABI of include/fusedmm.h apart from fusedmm_plan_create (fusedmm_plan.hip) --
// argument validation, pattern recognition, dispatch to the kernels, scratch, profiling, the tuned plan.
#include "fusedmm_plan.h"

#include <algorithm>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

using namespace fmm;

// Fixed scratch of fusedmm_execute_static_scratch: partial rows of split rows, for callers that cannot
// allocate.  One copy per GPU the library runs on, held until the process ends.  In host code the array's
// name only stands for the symbol: its device address is looked up once per device
// (static_scratch_for_current_device) and that pointer is what kernels, copies and fills are given.
static __device__ __align__(256) unsigned char scratch[FUSEDMM_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxScratchDevices = 64;
void* g_scratch_ptr[kMaxScratchDevices] = {};
std::mutex g_scratch_mutex;

}  // namespace

// The address of `scratch` on the current device (every GPU holds its own copy at its own address).
int fmm::static_scratch_for_current_device(void** out) {
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

namespace {

constexpr size_t kMaxProfiledCalls = 4096;

// The instance size a dimension runs on: itself if it has instances of its own, else the next larger one (the
// masked instances skip what lies beyond d, element by element in the last piece when d is not a multiple of 4),
// else 0.  fp32: the powers of two from 32 to 2048 and the sizes halfway between them (96 ... 1536: a dimension
// such as 300 or 768 would leave 40 % or 25 % of the lanes of the next power of two idle); Y stored in 2-byte
// elements: the same sizes up to 1024; double precision: the powers of two.
constexpr int32_t kMaxWideDim = 2048;
constexpr int32_t kMaxWideDim2Byte = 1024;
static_assert(kMaxWideDim == FUSEDMM_MAX_D, "every accepted dimension has an instance to run on");
int32_t instance_dim(int32_t d) {
  if (d < 1 || d > kMaxWideDim) return 0;
  int32_t D = 32;
  while (D < d) D *= 2;
  return (D >= 128 && d <= D / 4 * 3) ? D / 4 * 3 : D;
}

// Double precision: the powers of two.
int32_t instance_dim_f64(int32_t d) {
  if (d < 1 || d > kMaxWideDim) return 0;
  int32_t D = 32;
  while (D < d) D *= 2;
  return D;
}

// Y stored in 2-byte elements: rows are read 16 bytes = 8 elements at a time, so d is a multiple of 8, from 8 up
// to 1024.
int32_t instance_dim_2byte(int32_t d) {
  if (d < 8 || d % 8 != 0 || d > kMaxWideDim2Byte) return 0;
  return instance_dim(d);
}

// How many floats a partial row of the specialised schedule takes when the plan serves dimensions up to d in
// fp32 (the largest instance size among them, and the short-vector kernels' fixed stride) ...
int32_t partial_floats_f32(int32_t d) {
  return std::max<int32_t>(d >= kMaxWideDim ? kMaxWideDim : instance_dim(d), kSmallPartialStride);
}
// ... and in fp64 (two floats per element)
int32_t partial_floats_f64(int32_t d) { return 2 * (d >= kMaxWideDim ? kMaxWideDim : instance_dim_f64(d)); }

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

// The ragged instances (d not a multiple of 4) gather the piece a row of Y ends in with one 4-element load, which
// reads 4 - d % 4 elements beyond the row; from the row returned here on, that would reach beyond the last element
// of the matrix, and the kernels move the load back to end with the row.  -1 when such a load of the first of those
// rows would begin before the matrix (a matrix of fewer than four elements before that row's end): then the wide
// kernels cannot take the call.
int32_t first_back_row(int64_t n, int64_t ldy, int32_t d) {
  if (d % 4 == 0 || n <= 0) return (int32_t)std::max<int64_t>(n, 0);
  const int64_t beyond = 4 - d % 4;
  const int64_t first = std::max<int64_t>(0, n - (beyond + ldy - 1) / ldy);
  if (first * ldy + d - 4 < 0) return -1;
  return (int32_t)first;
}

bool overlaps(const float* a, int64_t rows_a, int64_t ld_a, const float* b, int64_t rows_b, int64_t ld_b, int32_t d) {
  if (!a || !b || rows_a <= 0 || rows_b <= 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  const uintptr_t a1 = a0 + (uintptr_t)((rows_a - 1) * ld_a + d) * sizeof(float);
  const uintptr_t b1 = b0 + (uintptr_t)((rows_b - 1) * ld_b + d) * sizeof(float);
  return a0 < b1 && b0 < a1;
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

// d: the instance size of a wide kernel (pattern: the instance launch_fast will be given), or the dimension itself
// for the kernels for very short feature vectors
void fill_schedule_args(const fusedmm_plan* p, int pattern, int32_t d, int y_format, KernelArgs* a) {
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
  const int rpb = (is_small_dim(d) && y_format != kYF64) ? small_packed_rows_per_block(d) : packed_rows_per_block(pattern, d, y_format);
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

  // d = 2, 3, 4, 8, 16: the one-lane-per-entry kernels; every other d: the wide kernels, on the instance of d
  // itself or the next larger one (choose_pattern says in which form); every call of a plan that asks for it: the
  // general kernel.  2-byte storage of Y exists on the wide kernels only (d = 8, 16, 24 ... 1024).
  const bool small = !y_bf16 && is_small_dim(d) && !plan->general_only;  // one lane per stored entry
  const int32_t D = y_bf16 ? instance_dim_2byte(d) : instance_dim(d);
  const int recognised = recognise(*ops);
  const int family = recognise_family(*ops);
  const int pattern = choose_pattern(recognised, family, d, D);
  // fp32 rows may start anywhere (the kernels read and write them as element-aligned vectors); rows of 2-byte
  // elements are read 16 bytes at a time and have to be aligned to that
  const bool y_ok = plan->nnz == 0 || !y_bf16 || (aligned16(d_Y) && ldy % 8 == 0);
  // the fast kernels address a row of Y by a 32-bit pitch in bytes
  // (and a ragged d needs four elements of Y before the end of the first row it reads backwards: see first_back_row)
  const bool fast = D != 0 && ldy < (int64_t(1) << 29) && y_ok && (y_bf16 || !plan->general_only) &&
                    (plan->nnz == 0 || first_back_row(plan->n, ldy, d) >= 0);
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
    fill_schedule_args(plan, recognised, d, kYF32, &a);
    a.partials = partials;
    a.d_pieces = a.d_full = a.d_tail = 0;
    a.y_first_back_row = 0;
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
    fill_schedule_args(plan, pattern, D, y_format, &a);
    a.partials = partials;
    a.d_full = d / 4; a.d_tail = d % 4; a.d_pieces = (d + 3) / 4;
    a.y_first_back_row = first_back_row(plan->n, ldy, d);
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
  const bool fast = D != 0 && ldy < (int64_t(1) << 28) && !plan->general_only &&
                    (plan->nnz == 0 || first_back_row(plan->n, ldy, d) >= 0);
  if (fast) {
    if (plan->n_parts > 0 && 2 * D > plan->partials_d) return FUSEDMM_ERR_NOT_RESERVED;
    const int recognised = recognise(*ops);
    const int family = recognise_family(*ops);
    const int pattern = choose_pattern(recognised, family, d, D);
    KernelArgs a;
    fill_schedule_args(plan, pattern, D, kYF64, &a);
    fill_op_args(*ops, &a);
    a.d_full = d / 4; a.d_tail = d % 4; a.d_pieces = (d + 3) / 4;
    a.y_first_back_row = first_back_row(plan->n, ldy, d);
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
    // a dimension that is not a multiple of 4 runs the ragged instances, which may have lane groups of their own
    const int visit = (D != 0 && d % 4 != 0) ? (PAT_VISIT | kPatRagged) : PAT_VISIT;
    fill_schedule_args(plan, visit, D ? D : d, fmt, &a);
    a.values = nullptr; a.X = nullptr; a.Y = nullptr; a.Z = nullptr;
    a.ldx = a.ldy = a.ldz = d;
    a.alpha = 0.f;
    a.vop = a.rop = a.sop = a.mop = a.aop = a.mean = 0;
    a.d_full = d / 4; a.d_tail = d % 4; a.d_pieces = (d + 3) / 4;
    a.y_first_back_row = 0;  // no Y is read
    a.visit_counts = d_counts;
    e = D == 0 ? launch_small(PAT_VISIT, d, a, stream) : launch_fast(visit, D, fmt, a, stream);
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

int fusedmm_debug_kernel_size(int32_t d, int32_t storage) {
  if (d < 1 || d > FUSEDMM_MAX_D) return 0;
  switch (storage) {
    case 0: return is_small_dim(d) ? d : instance_dim(d);
    case 1: return instance_dim_2byte(d);
    case 2: return instance_dim_f64(d);
    default: return 0;
  }
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
