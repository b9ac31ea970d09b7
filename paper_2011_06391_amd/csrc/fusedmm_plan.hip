// fusedmm_plan_create: the degree-binned plan, the GPU counterpart of Part1D in Algorithm 1 (Section III-C:
// balance by stored entries, rows never write-shared).  Host code; the three small kernels it uses
// (column-index check, column histogram, class boundaries inside the long rows) are in fusedmm_generic.hip.
//
// Steps, one function each:
//   resolve_settings        options and defaults -> bin thresholds, number of column classes
//   rowptr_to_host          the O(m) scan of Part1D works on a host copy of the row pointers
//   check_column_indices    so that no kernel can index outside Y
//   cut_rows_into_tiles     which rows are cut by column class, and where each class begins inside them
//   build_work_lists        the rows walked twice by host threads: counted, then placed
//   deal_classes_to_xcds    the tiled segments as per-XCD lists of workgroup items
//   general_segments        the general kernel's own cut of the long rows
// and fusedmm_plan_create uploads the lists and reserves the scratch of the hinted dimension.
#include "fusedmm_plan.h"

#include <algorithm>
#include <new>
#include <system_error>
#include <thread>
#include <vector>

using namespace fmm;

namespace {

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
// the passes over the rows run on up to this many host threads, each on at least this many rows
constexpr int kPlanThreads = 16;
constexpr int kPlanThreadsLimit = 64;  // for an explicit fusedmm_plan_options_t::host_threads
constexpr int64_t kPlanRowsPerThread = 1 << 16;

// Device memory for the length of a scope.
struct DeviceBuffer {
  void* ptr = nullptr;
  DeviceBuffer() = default;
  DeviceBuffer(const DeviceBuffer&) = delete;
  DeviceBuffer& operator=(const DeviceBuffer&) = delete;
  ~DeviceBuffer() {
    if (ptr) (void)hipFree(ptr);
  }
  hipError_t alloc(size_t bytes) { return hipMalloc(&ptr, bytes); }
  template <class T>
  T* as() const { return static_cast<T*>(ptr); }
};

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

// ---------------------------------------------------------------------------------------------------------
struct Settings {
  int32_t small_max = 0, split_min = 0, chunk = 0;  // the three bins: packed <= small_max < wave <= split_min < chunks
  int32_t n_classes = 1;                             // finest number of column classes; 1 = no tiling
  int32_t tile_min = 0;                              // rows with at least this many entries are tiled
  int64_t tile_edges_per_class = 1;
  int32_t d_hint = 128;
  int host_threads = 0;  // 0 = automatic
  bool general_only = false;
};

int resolve_settings(int64_t m, int64_t n, int64_t nnz, const fusedmm_plan_options_t* options, Settings* out) {
  Settings s;
  s.small_max = kDefaultSmallRowMax; s.split_min = kDefaultSplitRowMin; s.chunk = kDefaultChunkEdges;
  if (options && options->feature_dim_hint > 0 && options->feature_dim_hint <= 16) {
    // very short feature vectors (one lane per stored entry): a work item's fixed cost -- its descriptor, the
    // reduction across lanes, the store -- is spread over more entries
    s.small_max = kShortDimSmallRowMax; s.split_min = kShortDimSplitRowMin; s.chunk = kShortDimChunkEdges;
  }
  s.n_classes = 0;
  if (options) {
    if (options->small_row_max < 0 || options->split_row_min < 0 || options->chunk_edges < 0) return FUSEDMM_ERR_INVALID_ARG;
    if (options->column_classes < 0 || options->tile_row_min < 0 || options->feature_dim_hint < 0) return FUSEDMM_ERR_INVALID_ARG;
    if (options->small_row_max > 0) s.small_max = options->small_row_max;
    if (options->split_row_min > 0) s.split_min = options->split_row_min;
    if (options->chunk_edges > 0) s.chunk = options->chunk_edges;
    s.n_classes = options->column_classes;
    s.tile_min = options->tile_row_min;
    if (options->feature_dim_hint > 0) s.d_hint = options->feature_dim_hint;
    s.host_threads = options->host_threads;
    s.general_only = options->general_kernel_only != 0;
  }
  const bool dense = m > 0 && nnz / m >= kDenseEntriesPerRow;
  if (s.n_classes == 0) {
    // automatic: off while Y (n rows of the hinted dimension) is small; else as many finest classes as
    // bring a class slice of Y down to the size that pays for the pattern's density, at most 64
    const int64_t y_bytes = n * (int64_t)s.d_hint * (int64_t)sizeof(float);
    s.n_classes = 1;
    if (y_bytes >= (dense ? kTilingMinYBytesDense : kTilingMinYBytes)) {
      s.n_classes = kNumXcd;
      const int64_t slice = dense ? kTilingSliceBytesDense : kTilingSliceBytesSparse;
      while (s.n_classes < kAutoMaxColumnClasses && y_bytes / s.n_classes > slice) s.n_classes *= 2;
    }
  }
  if (s.n_classes > 1) {  // levels are nested: 8, 16, 32, ... classes
    int32_t c = kNumXcd;
    while (c < s.n_classes && c < kMaxColumnClasses) c *= 2;
    s.n_classes = c;
  }
  // a row needs 16 entries per class on average for a partial row per class to be worth it; 8 on dense patterns,
  // where nearly every row is tiled anyway and the shorter ones gain more from their classes' L2 than their partial
  // rows cost (c3: 3.99 -> 3.90 ms; the sparse workloads lose 1-6 % with it)
  if (s.tile_min <= 0) s.tile_min = (dense ? kDenseTileEdgesPerClass : kDefaultTileEdgesPerClass) * kNumXcd;
  s.tile_edges_per_class = std::max<int64_t>(1, s.tile_min / kNumXcd);
  s.small_max = std::min(s.small_max, 1 << 16);
  s.split_min = std::min(std::max(s.split_min, s.small_max), 1 << 20);
  s.chunk = std::min(std::max((s.chunk + 255) / 256 * 256, 256), 1 << 24);
  *out = s;
  return FUSEDMM_OK;
}

// Row pointers to the host (the O(m) scan of Part1D reads them there), checked: from 0 to nnz, never decreasing.
int rowptr_to_host(const int64_t* d_rowptr, int64_t m, int64_t nnz, hipStream_t stream, std::vector<int64_t>* rp) {
  rp->resize((size_t)m + 1);
  if (hipStreamSynchronize(stream) != hipSuccess) return FUSEDMM_ERR_HIP;
  if (hipMemcpy(rp->data(), d_rowptr, ((size_t)m + 1) * sizeof(int64_t), hipMemcpyDeviceToHost) != hipSuccess)
    return FUSEDMM_ERR_HIP;
  if ((*rp)[0] != 0 || (*rp)[(size_t)m] != nnz) return FUSEDMM_ERR_INVALID_ARG;
  for (int64_t u = 0; u < m; ++u)
    if ((*rp)[(size_t)u + 1] < (*rp)[(size_t)u]) return FUSEDMM_ERR_INVALID_ARG;
  return FUSEDMM_OK;
}

// Column indices must address rows of Y: checked on the device, once.
int check_column_indices(const int32_t* d_colidx, int64_t nnz, int64_t n, hipStream_t stream) {
  if (nnz == 0) return FUSEDMM_OK;
  DeviceBuffer d_flag;
  if (d_flag.alloc(sizeof(int32_t)) != hipSuccess) return FUSEDMM_ERR_ALLOC;
  int32_t flag = 0;
  hipError_t e = hipMemcpy(d_flag.ptr, &flag, sizeof(flag), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = launch_validate_colidx(d_colidx, nnz, n, d_flag.as<int32_t>(), stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e == hipSuccess) e = hipMemcpy(&flag, d_flag.ptr, sizeof(flag), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return FUSEDMM_ERR_HIP;
  return flag != 0 ? FUSEDMM_ERR_INVALID_ARG : FUSEDMM_OK;
}

// ---------------------------------------------------------------------------------------------------------
// Which rows are cut into column-class tiles, and how finely.  Level of a row = number of classes it is cut
// into: the largest of 8, 16, ..., n_classes that leaves it tile_edges_per_class entries per class on average.
// Classes are nested contiguous column ranges: a class of level L is n_classes / L finest classes.
struct TiledRows {
  std::vector<int32_t> rows, level;  // in row order; empty = the pattern is not tiled
  std::vector<int64_t> bnd_off;      // per tiled row: where its level + 1 boundaries start in bounds[]
  std::vector<int32_t> bounds;       // offsets, within the row, where each of its classes begins
};

// The finest classes are contiguous column ranges that hold about the same number of stored entries each
// (from a histogram of the column indices over kClassBuckets buckets, every stride-th entry), not the same
// number of columns: where the often-gathered columns sit side by side -- vertex orders that keep hubs
// together -- equal widths would give one XCD most of the work.  class_start: n_classes + 1 column numbers.
int class_boundaries(const int32_t* d_colidx, int64_t nnz, int64_t n, int32_t n_classes, hipStream_t stream,
                     std::vector<int32_t>* class_start) {
  const int32_t nbk = (int32_t)std::min<int64_t>(kClassBuckets, n);
  const int64_t stride = std::max<int64_t>(1, nnz / kClassSamples);
  std::vector<uint32_t> hist((size_t)nbk);
  DeviceBuffer d_hist;
  if (d_hist.alloc((size_t)nbk * sizeof(uint32_t)) != hipSuccess) {
    (void)hipGetLastError();
    return FUSEDMM_ERR_ALLOC;
  }
  hipError_t e = hipMemsetAsync(d_hist.ptr, 0, (size_t)nbk * sizeof(uint32_t), stream);
  if (e == hipSuccess) e = launch_column_histogram(d_colidx, nnz, stride, n, nbk, d_hist.as<uint32_t>(), stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e == hipSuccess) e = hipMemcpy(hist.data(), d_hist.ptr, (size_t)nbk * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return FUSEDMM_ERR_HIP;
  uint64_t total = 0;
  for (uint32_t h : hist) total += h;
  class_start->assign((size_t)n_classes + 1, 0);
  (*class_start)[(size_t)n_classes] = (int32_t)n;
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
      (*class_start)[(size_t)c++] = (int32_t)std::min<int64_t>(first_col_after, n);
    }
  }
  for (; c < n_classes; ++c) (*class_start)[(size_t)c] = (int32_t)n;
  return FUSEDMM_OK;
}

int cut_rows_into_tiles(const std::vector<int64_t>& rp, int64_t m, int64_t n, int64_t nnz, const int64_t* d_rowptr,
                        const int32_t* d_colidx, const Settings& s, hipStream_t stream, TiledRows* t) {
  if (s.n_classes <= 1 || nnz == 0) return FUSEDMM_OK;
  std::vector<int32_t> class_start;
  int st = class_boundaries(d_colidx, nnz, n, s.n_classes, stream, &class_start);
  if (st != FUSEDMM_OK) return st;

  int64_t nb = 0;
  for (int64_t u = 0; u < m; ++u) {
    const int64_t deg = rp[(size_t)u + 1] - rp[(size_t)u];
    if (deg < s.tile_min) continue;
    int32_t level = kNumXcd;
    while (level < s.n_classes && deg >= s.tile_edges_per_class * 2 * level) level *= 2;
    t->rows.push_back((int32_t)u);
    t->level.push_back(level);
    t->bnd_off.push_back(nb);
    nb += level + 1;
  }
  if (t->rows.empty()) return FUSEDMM_OK;

  // where each class begins inside each tiled row: a binary search per boundary, on the device where the
  // column indices are; the same kernel reports rows whose columns are not sorted
  const size_t nt = t->rows.size();
  t->bounds.resize((size_t)nb);
  DeviceBuffer d_class_start, d_rows, d_level, d_off, d_bounds, d_flag;
  hipError_t e = d_class_start.alloc(class_start.size() * sizeof(int32_t));
  if (e == hipSuccess) e = d_rows.alloc(nt * sizeof(int32_t));
  if (e == hipSuccess) e = d_level.alloc(nt * sizeof(int32_t));
  if (e == hipSuccess) e = d_off.alloc(nt * sizeof(int64_t));
  if (e == hipSuccess) e = d_bounds.alloc((size_t)nb * sizeof(int32_t));
  if (e == hipSuccess) e = d_flag.alloc(sizeof(int32_t));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return FUSEDMM_ERR_ALLOC;
  }
  int32_t flag = 0;
  e = hipMemcpy(d_class_start.ptr, class_start.data(), class_start.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d_rows.ptr, t->rows.data(), nt * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d_level.ptr, t->level.data(), nt * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d_off.ptr, t->bnd_off.data(), nt * sizeof(int64_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d_flag.ptr, &flag, sizeof(flag), hipMemcpyHostToDevice);
  if (e == hipSuccess)
    e = launch_tile_bounds(d_rowptr, d_colidx, d_rows.as<int32_t>(), d_level.as<int32_t>(), d_off.as<int64_t>(), (int32_t)nt,
                           s.n_classes, d_class_start.as<int32_t>(), d_bounds.as<int32_t>(), d_flag.as<int32_t>(), stream);
  if (e == hipSuccess) e = hipStreamSynchronize(stream);
  if (e == hipSuccess) e = hipMemcpy(t->bounds.data(), d_bounds.ptr, (size_t)nb * sizeof(int32_t), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(&flag, d_flag.ptr, sizeof(flag), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return FUSEDMM_ERR_HIP;
  if (flag != 0) t->rows.clear();  // some long row has unsorted columns: no tiling for this pattern
  return FUSEDMM_OK;
}

// ---------------------------------------------------------------------------------------------------------
struct WorkLists {
  std::vector<int32_t> order;      // rows that are not split: sorted by length, longest first
  std::vector<ChunkDesc> chunks;   // workgroup chunks of the long rows that are not tiled
  std::vector<ChunkDesc> tile_descs;  // segments of the tiled rows, class by class
  std::vector<MergeDesc> merges;   // rows that were split: where their partial rows are
  std::vector<BlockItem> items;    // the tiled segments as workgroup items, dealt to the XCDs
  int64_t n_wave = 0, n_empty = 0, n_long = 0, n_parts = 0, n_tiled_rows = 0;
  bool tiled = false;  // some rows are cut by column class
};

// The classes are dealt to the XCDs: XCD k owns the k-th eighth of the column range and works through its
// finest classes in order; coarser tiles sit where their first finest class is.  Workgroup b runs on XCD
// b % 8, so the lists are interleaved, padded with empty items to the longest.
void deal_classes_to_xcds(size_t ncls, const std::vector<int64_t>& cls_base, const std::vector<int64_t>& cls_nchunk,
                          const std::vector<int64_t>& cls_nwave, const std::vector<int64_t>& cls_nshort,
                          std::vector<BlockItem>* items) {
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
  items->assign(longest * kNumXcd, BlockItem{kItemNone, 0, 0, 0});
  for (int k = 0; k < kNumXcd; ++k)
    for (size_t j = 0; j < xcd_items[(size_t)k].size(); ++j) (*items)[j * kNumXcd + (size_t)k] = xcd_items[(size_t)k][j];
}

// The rows are walked twice, by T host threads over contiguous row ranges: first counted, then placed.
// What a thread counts in the first pass becomes, by prefix sums over the threads in row order, the positions
// it writes to in the second, so the lists are the ones a single thread walking the rows in order produces:
// short rows sorted by length (longest first, row order kept among equals); the segments of the tiled rows
// class by class ([chunks][wavefront segments][lane-group segments], longest first within each); partial-row
// slots handed out in row order, so the merge order of a row is fixed by (class, chunk) and does not depend
// on how the descriptors are arranged.  All memory is allocated before the threads start.
int build_work_lists(const std::vector<int64_t>& rp, int64_t m, const Settings& s, const TiledRows& tiles, WorkLists* w) {
  const int64_t small_max = s.small_max, split_min = s.split_min, chunk = s.chunk;
  const bool tiling = !tiles.rows.empty();
  const int64_t tiled_from = tiling ? s.tile_min : INT64_MAX;

  // length of a workgroup chunk when `count` entries are cut into chunks of at most chunk_edges:
  // equal shares, rounded up to whole batches of 64 entries for each of the 4 wavefronts
  auto chunk_len = [&](int64_t count) {
    const int64_t nc = (count + chunk - 1) / chunk;
    return ((count + nc - 1) / nc + 255) / 256 * 256;
  };

  const size_t ncls = tiling ? (size_t)s.n_classes : 0;
  const size_t hw = (size_t)split_min + 1;
  const int T = s.host_threads > 0
                    ? std::min(s.host_threads, kPlanThreadsLimit)
                    : (int)std::max<int64_t>(1, std::min<int64_t>({(int64_t)kPlanThreads, (int64_t)std::thread::hardware_concurrency(),
                                                                    m / kPlanRowsPerThread}));
  struct ThreadCounts {
    std::vector<int64_t> bucket;                // short rows by length; after the prefix sums: where the next one goes
    std::vector<int64_t> cls_nchunk, cls_hist;  // tile chunks per class, shorter segments per (class, length); likewise
    int64_t n_long = 0, n_chunk_descs = 0, n_merges = 0, n_parts = 0, n_tiled = 0;
    size_t ti0 = 0;  // index in tiles.rows of the thread's first tiled row
  };
  std::vector<ThreadCounts> tc((size_t)T);
  for (int t = 0; t < T; ++t) {
    tc[(size_t)t].bucket.assign((size_t)split_min + 1, 0);
    tc[(size_t)t].cls_nchunk.assign(ncls, 0);
    tc[(size_t)t].cls_hist.assign(ncls * hw, 0);
    tc[(size_t)t].ti0 = (size_t)(std::lower_bound(tiles.rows.begin(), tiles.rows.end(), (int32_t)(m * t / T)) - tiles.rows.begin());
  }
  // body(t) for every row range t: range 0 on the calling thread, the others on threads of their own; a range
  // whose thread cannot be started (the process is at its limit) is walked by the calling thread as well.  The
  // bodies allocate nothing and throw nothing.
  auto on_threads = [&](auto&& body) {
    std::vector<std::thread> workers;
    workers.reserve((size_t)T);
    int started = 1;
    try {
      for (; started < T; ++started) workers.emplace_back([&body, t = started]() { body(t); });
    } catch (const std::system_error&) {
    }
    body(0);
    for (int t = started; t < T; ++t) body(t);
    for (auto& worker : workers) worker.join();
  };

  // first pass: count
  on_threads([&](int t) {
    ThreadCounts& c = tc[(size_t)t];
    size_t ti = c.ti0;
    for (int64_t u = m * t / T; u < m * (t + 1) / T; ++u) {
      const int64_t deg = rp[(size_t)u + 1] - rp[(size_t)u];
      if (deg >= tiled_from) {
        const int32_t* bnd = tiles.bounds.data() + tiles.bnd_off[ti];
        const size_t level = (size_t)tiles.level[ti], stride = ncls / level;
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
  int64_t n_chunk_descs = 0, n_merge_descs = 0;
  for (const ThreadCounts& c : tc) {
    for (size_t i = 0; i < bucket.size(); ++i) bucket[i] += c.bucket[i];
    for (size_t i = 0; i < cls_nchunk.size(); ++i) cls_nchunk[i] += c.cls_nchunk[i];
    for (size_t i = 0; i < cls_hist.size(); ++i) cls_hist[i] += c.cls_hist[i];
    w->n_long += c.n_long; n_chunk_descs += c.n_chunk_descs; n_merge_descs += c.n_merges; w->n_parts += c.n_parts;
    w->n_tiled_rows += c.n_tiled;
  }
  if (w->n_parts >= (int64_t)INT32_MAX || n_chunk_descs >= (int64_t)INT32_MAX) return FUSEDMM_ERR_INVALID_ARG;
  std::vector<int64_t> start((size_t)split_min + 1, 0);
  int64_t pos = 0;
  for (int64_t deg = split_min; deg >= 0; --deg) { start[(size_t)deg] = pos; pos += bucket[(size_t)deg]; }
  for (int64_t deg = split_min; deg > small_max; --deg) w->n_wave += bucket[(size_t)deg];
  w->n_empty = bucket[0];  // they sort last: zero-filled by workgroups of their own
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
  if (ncls > 0 && cls_base[ncls] >= (int64_t)INT32_MAX) return FUSEDMM_ERR_INVALID_ARG;
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
  w->order.resize((size_t)(m - w->n_long));
  w->chunks.resize((size_t)n_chunk_descs);
  w->merges.resize((size_t)n_merge_descs);
  w->tile_descs.resize(ncls > 0 ? (size_t)cls_base[ncls] : 0);

  // second pass: place
  on_threads([&](int t) {
    ThreadCounts& c = tc[(size_t)t];
    size_t ti = c.ti0;
    int32_t next_part = (int32_t)part0[(size_t)t];
    int64_t next_merge = merge0[(size_t)t], next_chunk = chunk0[(size_t)t];
    for (int64_t u = m * t / T; u < m * (t + 1) / T; ++u) {
      const int64_t deg = rp[(size_t)u + 1] - rp[(size_t)u];
      if (deg >= tiled_from) {
        const int32_t* bnd = tiles.bounds.data() + tiles.bnd_off[ti];
        const size_t level = (size_t)tiles.level[ti], stride = ncls / level;
        ++ti;
        const int32_t first_part = next_part;
        for (size_t k = 0; k < level; ++k) {
          const int64_t cnt = (int64_t)bnd[k + 1] - bnd[k];
          if (cnt <= 0) continue;
          const size_t cl = k * stride;
          const int64_t e_begin = rp[(size_t)u] + bnd[k];
          if (cnt > split_min) {
            const int64_t per = chunk_len(cnt);
            for (int64_t off = 0; off < cnt; off += per)
              w->tile_descs[(size_t)c.cls_nchunk[cl]++] =
                  ChunkDesc{e_begin + off, (int32_t)std::min<int64_t>(per, cnt - off), (int32_t)u, next_part++, 0};
          } else {
            w->tile_descs[(size_t)c.cls_hist[cl * hw + (size_t)cnt]++] = ChunkDesc{e_begin, (int32_t)cnt, (int32_t)u, next_part++, 0};
          }
        }
        w->merges[(size_t)next_merge++] = MergeDesc{(int32_t)u, first_part, next_part - first_part, 0};
      } else if (deg <= split_min) {
        w->order[(size_t)c.bucket[(size_t)deg]++] = (int32_t)u;
      } else {
        const int64_t per = chunk_len(deg);
        const int32_t nc = (int32_t)((deg + per - 1) / per);
        if (nc > 1) w->merges[(size_t)next_merge++] = MergeDesc{(int32_t)u, next_part, nc, 0};
        for (int64_t off = 0; off < deg; off += per)
          w->chunks[(size_t)next_chunk++] = ChunkDesc{rp[(size_t)u] + off, (int32_t)std::min<int64_t>(per, deg - off), (int32_t)u,
                                                      nc > 1 ? next_part++ : -1, 0};
      }
    }
  });

  w->tiled = tiling;
  if (tiling) deal_classes_to_xcds(ncls, cls_base, cls_nchunk, cls_nwave, cls_nshort, &w->items);
  if (w->tile_descs.size() >= (size_t)INT32_MAX || w->items.size() >= (size_t)INT32_MAX) return FUSEDMM_ERR_INVALID_ARG;
  return FUSEDMM_OK;
}

// The general kernel's segments: rows longer than kGenericSplit, cut into runs of that length.
int general_segments(const std::vector<int64_t>& rp, int64_t m, std::vector<ChunkDesc>* segs, std::vector<MergeDesc>* merges) {
  for (int64_t u = 0; u < m; ++u) {
    const int64_t deg = rp[(size_t)u + 1] - rp[(size_t)u];
    if (deg <= kGenericSplit) continue;
    const int32_t first = (int32_t)segs->size();
    for (int64_t off = 0; off < deg; off += kGenericSplit)
      segs->push_back(ChunkDesc{rp[(size_t)u] + off, (int32_t)std::min<int64_t>(kGenericSplit, deg - off), (int32_t)u,
                                (int32_t)segs->size(), 0});
    merges->push_back(MergeDesc{(int32_t)u, first, (int32_t)segs->size() - first, 0});
    if (segs->size() >= (size_t)INT32_MAX / 2) return FUSEDMM_ERR_INVALID_ARG;
  }
  return FUSEDMM_OK;
}

}  // namespace

namespace fmm {

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
  p->d_order = nullptr; p->d_chunks = nullptr; p->d_merges = nullptr; p->d_items = nullptr; p->d_tile_descs = nullptr;
  p->d_partials = nullptr; p->d_gen_segs = nullptr; p->d_gen_merges = nullptr; p->d_gen_partials = nullptr;
}

}  // namespace fmm

extern "C" int fusedmm_plan_create(fusedmm_plan_t** out, int64_t m, int64_t n, int64_t nnz, const int64_t* d_rowptr,
                                   const int32_t* d_colidx, const fusedmm_plan_options_t* options, void* stream_) {
  if (!out) return FUSEDMM_ERR_INVALID_ARG;
  *out = nullptr;
  if (m < 0 || n < 0 || nnz < 0 || m >= INT32_MAX || n >= INT32_MAX) return FUSEDMM_ERR_INVALID_ARG;
  if (!d_rowptr || (nnz > 0 && (!d_colidx || n == 0 || m == 0))) return FUSEDMM_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(stream_);

  Settings s;
  int st = resolve_settings(m, n, nnz, options, &s);
  if (st != FUSEDMM_OK) return st;

  WorkLists w;
  std::vector<ChunkDesc> gen_segs;
  std::vector<MergeDesc> gen_merges;
  fusedmm_plan* p = nullptr;
  try {
    std::vector<int64_t> rp;
    st = rowptr_to_host(d_rowptr, m, nnz, stream, &rp);
    if (st == FUSEDMM_OK) st = check_column_indices(d_colidx, nnz, n, stream);
    TiledRows tiles;
    if (st == FUSEDMM_OK) st = cut_rows_into_tiles(rp, m, n, nnz, d_rowptr, d_colidx, s, stream, &tiles);
    if (st == FUSEDMM_OK) st = build_work_lists(rp, m, s, tiles, &w);
    if (st == FUSEDMM_OK) st = general_segments(rp, m, &gen_segs, &gen_merges);
    if (st != FUSEDMM_OK) return st;
    p = new fusedmm_plan();
  } catch (const std::bad_alloc&) {
    return FUSEDMM_ERR_ALLOC;
  }

  p->m = m; p->n = n; p->nnz = nnz;
  p->d_rowptr = d_rowptr; p->d_colidx = d_colidx;
  p->small_row_max = s.small_max; p->split_row_min = s.split_min; p->chunk_edges = s.chunk; p->tile_row_min = s.tile_min;
  p->general_only = s.general_only;
  p->n_wave = (int32_t)w.n_wave;
  p->n_empty = (int32_t)w.n_empty;
  p->n_packed = (int32_t)((m - w.n_long) - w.n_wave - w.n_empty);
  p->n_chunks = (int32_t)w.chunks.size();
  p->n_merges = (int32_t)w.merges.size();
  p->n_parts = (int32_t)w.n_parts;
  p->n_items = (int32_t)w.items.size();
  p->n_tile_descs = (int32_t)w.tile_descs.size();
  p->n_tiled_rows = (int32_t)w.n_tiled_rows;
  p->n_classes = w.tiled ? s.n_classes : 1;
  p->n_gen_segs = (int32_t)gen_segs.size();
  p->n_gen_merges = (int32_t)gen_merges.size();

  st = upload(&p->d_order, w.order, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_gen_segs, gen_segs, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_gen_merges, gen_merges, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_chunks, w.chunks, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_merges, w.merges, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_items, w.items, stream);
  if (st == FUSEDMM_OK) st = upload(&p->d_tile_descs, w.tile_descs, stream);
  if (st == FUSEDMM_OK && hipStreamSynchronize(stream) != hipSuccess) st = FUSEDMM_ERR_HIP;
  // the address of the static scratch on this device is looked up here, once, so that
  // fusedmm_execute_static_scratch finds it in place (its own first call would look it up otherwise)
  if (st == FUSEDMM_OK) {
    void* unused = nullptr;
    (void)static_scratch_for_current_device(&unused);  // a failure is reported by that entry point, not here
  }
  // the scratch of the hinted dimension, so that execute never has to allocate
  if (st == FUSEDMM_OK) st = fusedmm_plan_reserve(p, std::min<int32_t>(s.d_hint, FUSEDMM_MAX_D));
  if (st != FUSEDMM_OK) {
    free_plan_device(p);
    delete p;
    return st;
  }
  *out = p;
  return FUSEDMM_OK;
}
