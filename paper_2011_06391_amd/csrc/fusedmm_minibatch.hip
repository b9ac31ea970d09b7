// Minibatch embedding epoch on top of the C ABI (Section V, end-to-end training, Table VIII;
// Section III-C: minibatching belongs to the application layer).  A batch is a rectangular
// slice A[B, :] of the adjacency matrix; per batch two FusedMM calls (attraction over the
// stored entries with 1 - sigmoid, repulsion from the batch's negative samples with sigmoid)
// and one update of the batch's rows.  Every batch has its own plans, built once; an epoch is
// a sequence of asynchronous launches on one stream, issued from this file without going
// back to the caller in between.
#include "../../include/fusedmm.h"
#include "fusedmm_internal.h"

#include <new>
#include <vector>

struct fusedmm_minibatch {
  int64_t n = 0;
  int32_t batch_rows = 0, n_negative = 0, n_batches = 0;
  std::vector<fusedmm_plan_t*> pos, neg;
  int64_t* d_rowptrs = nullptr;     // rebased row pointers of all batches, back to back
  int64_t* d_neg_rowptr = nullptr;  // 0, s, 2s, ...: every row of a batch holds the same s samples
  int32_t* d_neg_colidx = nullptr;  // n_batches x batch_rows x s
  float* d_z = nullptr;             // Zpos then Zneg, batch_rows x z_d each
  int32_t z_d = 0;
};

namespace {

// out[(b * batch_rows + r) * s + j] = negatives[b * s + j]
__global__ __launch_bounds__(256) void tile_negatives_kernel(const int32_t* negatives, int64_t total, int32_t batch_rows,
                                                             int32_t s, int32_t* out) {
  const int64_t per_batch = (int64_t)batch_rows * s;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t b = i / per_batch;
    const int32_t j = (int32_t)((i - b * per_batch) % s);
    out[i] = negatives[b * s + j];
  }
}

// X[r, k] += lr * (Zpos[r, k] - Zneg[r, k]); Zneg may be null (no negative samples)
__global__ __launch_bounds__(256) void embedding_update_kernel(int64_t rows, int32_t d, float lr, const float* zpos,
                                                               const float* zneg, float* X, int64_t ldx) {
  const int64_t total = rows * d;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / d;
    const int32_t k = (int32_t)(i - r * d);
    const float g = zneg ? zpos[i] - zneg[i] : zpos[i];
    X[r * ldx + k] = X[r * ldx + k] + lr * g;
  }
}

unsigned grid_for(int64_t total) {
  const int64_t blocks = (total + 255) / 256;
  return (unsigned)(blocks < 1 ? 1 : (blocks > 65535 ? 65535 : blocks));
}

void release(fusedmm_minibatch* h) {
  for (fusedmm_plan_t* p : h->pos) (void)fusedmm_plan_destroy(p);
  for (fusedmm_plan_t* p : h->neg) (void)fusedmm_plan_destroy(p);
  if (h->d_rowptrs) (void)hipFree(h->d_rowptrs);
  if (h->d_neg_rowptr) (void)hipFree(h->d_neg_rowptr);
  if (h->d_neg_colidx) (void)hipFree(h->d_neg_colidx);
  if (h->d_z) (void)hipFree(h->d_z);
  delete h;
}

}  // namespace

extern "C" {

int fusedmm_minibatch_create(fusedmm_minibatch_t** out, int64_t n, int64_t nnz, const int64_t* d_rowptr,
                             const int32_t* d_colidx, int32_t batch_rows, int32_t n_negative,
                             const int32_t* d_negatives, void* stream_) {
  if (!out) return FUSEDMM_ERR_INVALID_ARG;
  *out = nullptr;
  if (n < 1 || n >= INT32_MAX || nnz < 0 || !d_rowptr || (nnz > 0 && !d_colidx)) return FUSEDMM_ERR_INVALID_ARG;
  if (batch_rows < 1 || n_negative < 0 || (n_negative > 0 && !d_negatives)) return FUSEDMM_ERR_INVALID_ARG;
  if ((int64_t)batch_rows * n_negative >= INT32_MAX) return FUSEDMM_ERR_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(stream_);

  std::vector<int64_t> rp, rebased;
  try {
    rp.resize((size_t)n + 1);
  } catch (const std::bad_alloc&) {
    return FUSEDMM_ERR_ALLOC;
  }
  if (hipStreamSynchronize(stream) != hipSuccess) return FUSEDMM_ERR_HIP;
  if (hipMemcpy(rp.data(), d_rowptr, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyDeviceToHost) != hipSuccess)
    return FUSEDMM_ERR_HIP;
  if (rp[0] != 0 || rp[n] != nnz) return FUSEDMM_ERR_INVALID_ARG;
  for (int64_t u = 0; u < n; ++u)
    if (rp[u + 1] < rp[u]) return FUSEDMM_ERR_INVALID_ARG;

  fusedmm_minibatch* h = new (std::nothrow) fusedmm_minibatch();
  if (!h) return FUSEDMM_ERR_ALLOC;
  h->n = n;
  h->batch_rows = batch_rows;
  h->n_negative = n_negative;
  h->n_batches = (int32_t)((n + batch_rows - 1) / batch_rows);
  const int32_t nb = h->n_batches;
  const int32_t s = n_negative;

  // rebased row pointers: batch b occupies [b * (batch_rows + 1), ...) with rows_b + 1 entries
  std::vector<int64_t> neg_rp;
  try {
    rebased.assign((size_t)nb * ((size_t)batch_rows + 1), 0);
    neg_rp.resize((size_t)batch_rows + 1);
    h->pos.reserve(nb);
    h->neg.reserve(nb);
  } catch (const std::bad_alloc&) {
    release(h);
    return FUSEDMM_ERR_ALLOC;
  }
  for (int32_t b = 0; b < nb; ++b) {
    const int64_t b0 = (int64_t)b * batch_rows;
    const int64_t b1 = b0 + batch_rows < n ? b0 + batch_rows : n;
    for (int64_t r = 0; r <= b1 - b0; ++r) rebased[(size_t)b * (batch_rows + 1) + r] = rp[b0 + r] - rp[b0];
  }
  for (int32_t r = 0; r <= batch_rows; ++r) neg_rp[r] = (int64_t)r * s;

  int status = FUSEDMM_OK;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&h->d_rowptrs), rebased.size() * sizeof(int64_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_neg_rowptr), neg_rp.size() * sizeof(int64_t));
  if (e == hipSuccess && s > 0)
    e = hipMalloc(reinterpret_cast<void**>(&h->d_neg_colidx), (size_t)nb * batch_rows * s * sizeof(int32_t));
  if (e != hipSuccess) {
    release(h);
    return FUSEDMM_ERR_ALLOC;
  }
  e = hipMemcpy(h->d_rowptrs, rebased.data(), rebased.size() * sizeof(int64_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(h->d_neg_rowptr, neg_rp.data(), neg_rp.size() * sizeof(int64_t), hipMemcpyHostToDevice);
  if (e == hipSuccess && s > 0) {
    const int64_t total = (int64_t)nb * batch_rows * s;
    hipLaunchKernelGGL(tile_negatives_kernel, dim3(grid_for(total)), dim3(256), 0, stream, d_negatives, total, batch_rows,
                       s, h->d_neg_colidx);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
  }
  if (e != hipSuccess) {
    release(h);
    return FUSEDMM_ERR_HIP;
  }

  for (int32_t b = 0; b < nb && status == FUSEDMM_OK; ++b) {
    const int64_t b0 = (int64_t)b * batch_rows;
    const int64_t b1 = b0 + batch_rows < n ? b0 + batch_rows : n;
    const int64_t rows = b1 - b0;
    fusedmm_plan_t* p = nullptr;
    status = fusedmm_plan_create(&p, rows, n, rp[b1] - rp[b0], h->d_rowptrs + (size_t)b * (batch_rows + 1),
                                 d_colidx ? d_colidx + rp[b0] : nullptr, nullptr, stream_);
    if (status != FUSEDMM_OK) break;
    h->pos.push_back(p);
    if (s > 0) {
      p = nullptr;
      // out-of-range samples are rejected here, by the plan's own check of the column indices
      status = fusedmm_plan_create(&p, rows, n, rows * s, h->d_neg_rowptr, h->d_neg_colidx + (size_t)b * batch_rows * s,
                                   nullptr, stream_);
      if (status != FUSEDMM_OK) break;
      h->neg.push_back(p);
    }
  }
  if (status != FUSEDMM_OK) {
    release(h);
    return status;
  }
  *out = h;
  return FUSEDMM_OK;
}

int fusedmm_minibatch_reserve(fusedmm_minibatch_t* h, int32_t d) {
  if (!h || d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_INVALID_ARG;
  for (fusedmm_plan_t* p : h->pos) {
    const int st = fusedmm_plan_reserve(p, d);
    if (st != FUSEDMM_OK) return st;
  }
  for (fusedmm_plan_t* p : h->neg) {
    const int st = fusedmm_plan_reserve(p, d);
    if (st != FUSEDMM_OK) return st;
  }
  if (h->z_d < d) {
    if (hipDeviceSynchronize() != hipSuccess) return FUSEDMM_ERR_HIP;  // earlier epochs may still read the old buffer
    if (h->d_z) (void)hipFree(h->d_z);
    h->d_z = nullptr;
    h->z_d = 0;
    if (hipMalloc(reinterpret_cast<void**>(&h->d_z), (size_t)2 * h->batch_rows * d * sizeof(float)) != hipSuccess)
      return FUSEDMM_ERR_ALLOC;
    h->z_d = d;
  }
  return FUSEDMM_OK;
}

int fusedmm_minibatch_epoch(fusedmm_minibatch_t* h, int32_t d, float lr, float* d_X, int64_t ldx, void* stream_) {
  if (!h || !d_X || ldx < d) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  const int st = fusedmm_minibatch_reserve(h, d);  // allocates on the first call for a larger d only
  if (st != FUSEDMM_OK) return st;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  fusedmm_ops_t attract, repel;
  (void)fusedmm_ops_preset(FUSEDMM_PATTERN_ONE_MINUS_SIGMOID_EMBED, &attract);
  (void)fusedmm_ops_preset(FUSEDMM_PATTERN_SIGMOID_EMBED, &repel);
  float* zpos = h->d_z;
  float* zneg = h->n_negative > 0 ? h->d_z + (size_t)h->batch_rows * d : nullptr;
  for (int32_t b = 0; b < h->n_batches; ++b) {
    const int64_t b0 = (int64_t)b * h->batch_rows;
    const int64_t rows = b0 + h->batch_rows < h->n ? h->batch_rows : h->n - b0;
    float* xb = d_X + b0 * ldx;
    int s = fusedmm_execute(h->pos[b], &attract, d, nullptr, xb, ldx, d_X, ldx, zpos, d, stream_);
    if (s != FUSEDMM_OK) return s;
    if (zneg) {
      s = fusedmm_execute(h->neg[b], &repel, d, nullptr, xb, ldx, d_X, ldx, zneg, d, stream_);
      if (s != FUSEDMM_OK) return s;
    }
    hipLaunchKernelGGL(embedding_update_kernel, dim3(grid_for(rows * d)), dim3(256), 0, stream, rows, d, lr, zpos, zneg,
                       xb, ldx);
    if (hipGetLastError() != hipSuccess) return FUSEDMM_ERR_HIP;
  }
  return FUSEDMM_OK;
}

int fusedmm_minibatch_info(const fusedmm_minibatch_t* h, int32_t* n_batches, int64_t* launches_per_epoch) {
  if (!h) return FUSEDMM_ERR_INVALID_ARG;
  if (n_batches) *n_batches = h->n_batches;
  if (launches_per_epoch) {
    int64_t total = 0;
    for (const fusedmm_plan_t* p : h->pos) {
      int64_t split = 0;
      (void)fusedmm_plan_stats(p, nullptr, nullptr, nullptr, &split, nullptr, nullptr, nullptr, nullptr);
      total += 2 + (split > 0 ? 1 : 0);  // execute (+ merge of split rows) and the update
    }
    total += (int64_t)h->neg.size();
    *launches_per_epoch = total;
  }
  return FUSEDMM_OK;
}

int fusedmm_minibatch_destroy(fusedmm_minibatch_t* h) {
  if (!h) return FUSEDMM_OK;
  (void)hipDeviceSynchronize();
  release(h);
  return FUSEDMM_OK;
}

}  // extern "C"
