// Minibatch embedding epoch on top of the C ABI (Section V, end-to-end training, Table VIII;
// Section III-C: minibatching belongs to the application layer).  A batch is a rectangular
// slice A[B, :] of the adjacency matrix; per batch two FusedMM calls (attraction over the
// stored entries with 1 - sigmoid, repulsion from the batch's negative samples with sigmoid)
// and one update of the batch's rows.  The two calls are issued as one: over the concatenated
// pattern [A[B, :] | N_B] with the scaling step h = a_uv - sigmoid(s) (the paper's SOP is
// user-definable), a_uv = 1 on stored entries and 0 on samples, the sum is Zpos - Zneg.  Every
// batch has its own plan, built once; an epoch is a sequence of asynchronous launches on one
// stream, issued from this file without going back to the caller in between.
#include "../../include/fusedmm.h"
#include "fusedmm_internal.h"

#include <new>
#include <vector>

struct fusedmm_minibatch {
  int64_t n = 0;
  int32_t batch_rows = 0, n_negative = 0, n_batches = 0;
  // one plan per batch over the concatenated pattern [A[B, :] | N_B]: row r holds its stored
  // entries (edge value 1) followed by the batch's negative samples (edge value 0)
  std::vector<fusedmm_plan_t*> plans;
  std::vector<int64_t> e_off;       // first entry of batch b in d_colidx / d_values
  int64_t* d_rowptrs = nullptr;     // rebased row pointers of all batches, back to back
  int32_t* d_colidx = nullptr;      // all batches, back to back
  float* d_values = nullptr;
  float* d_z = nullptr;             // batch_rows x z_d
  int32_t z_d = 0;
};

namespace {

// X[r, k] += lr * Z[r, k]
__global__ __launch_bounds__(256) void embedding_update_kernel(int64_t rows, int32_t d, float lr, const float* z, float* X,
                                                               int64_t ldx) {
  const int64_t total = rows * d;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / d;
    const int32_t k = (int32_t)(i - r * d);
    X[r * ldx + k] = X[r * ldx + k] + lr * z[i];
  }
}

unsigned grid_for(int64_t total) {
  const int64_t blocks = (total + 255) / 256;
  return (unsigned)(blocks < 1 ? 1 : (blocks > 65535 ? 65535 : blocks));
}

void release(fusedmm_minibatch* h) {
  for (fusedmm_plan_t* p : h->plans) (void)fusedmm_plan_destroy(p);
  if (h->d_rowptrs) (void)hipFree(h->d_rowptrs);
  if (h->d_colidx) (void)hipFree(h->d_colidx);
  if (h->d_values) (void)hipFree(h->d_values);
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
  const int32_t nb = (int32_t)((n + batch_rows - 1) / batch_rows);
  const int32_t s = n_negative;

  // the pattern and the samples come to the host once; the concatenated per-batch patterns go back
  std::vector<int64_t> rp, rebased;
  std::vector<int32_t> ci, neg, cat;
  std::vector<float> val;
  try {
    rp.resize((size_t)n + 1);
    ci.resize((size_t)nnz);
    neg.resize((size_t)nb * s);
  } catch (const std::bad_alloc&) {
    return FUSEDMM_ERR_ALLOC;
  }
  if (hipStreamSynchronize(stream) != hipSuccess) return FUSEDMM_ERR_HIP;
  if (hipMemcpy(rp.data(), d_rowptr, ((size_t)n + 1) * sizeof(int64_t), hipMemcpyDeviceToHost) != hipSuccess)
    return FUSEDMM_ERR_HIP;
  if (rp[0] != 0 || rp[n] != nnz) return FUSEDMM_ERR_INVALID_ARG;
  for (int64_t u = 0; u < n; ++u)
    if (rp[u + 1] < rp[u]) return FUSEDMM_ERR_INVALID_ARG;
  if (nnz > 0 && hipMemcpy(ci.data(), d_colidx, (size_t)nnz * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
    return FUSEDMM_ERR_HIP;
  if (!neg.empty() && hipMemcpy(neg.data(), d_negatives, neg.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
    return FUSEDMM_ERR_HIP;

  fusedmm_minibatch* h = new (std::nothrow) fusedmm_minibatch();
  if (!h) return FUSEDMM_ERR_ALLOC;
  h->n = n;
  h->batch_rows = batch_rows;
  h->n_negative = n_negative;
  h->n_batches = nb;
  try {
    rebased.assign((size_t)nb * ((size_t)batch_rows + 1), 0);
    cat.reserve((size_t)nnz + (size_t)n * s);
    val.reserve((size_t)nnz + (size_t)n * s);
    h->plans.reserve(nb);
    h->e_off.reserve((size_t)nb + 1);
    for (int32_t b = 0; b < nb; ++b) {
      const int64_t b0 = (int64_t)b * batch_rows;
      const int64_t b1 = b0 + batch_rows < n ? b0 + batch_rows : n;
      h->e_off.push_back((int64_t)cat.size());
      int64_t* brp = rebased.data() + (size_t)b * (batch_rows + 1);
      for (int64_t u = b0; u < b1; ++u) {
        cat.insert(cat.end(), ci.begin() + rp[u], ci.begin() + rp[u + 1]);
        val.insert(val.end(), (size_t)(rp[u + 1] - rp[u]), 1.0f);
        cat.insert(cat.end(), neg.begin() + (size_t)b * s, neg.begin() + (size_t)(b + 1) * s);
        val.insert(val.end(), (size_t)s, 0.0f);
        brp[u - b0 + 1] = (int64_t)cat.size() - h->e_off.back();
      }
    }
    h->e_off.push_back((int64_t)cat.size());
  } catch (const std::bad_alloc&) {
    release(h);
    return FUSEDMM_ERR_ALLOC;
  }

  hipError_t e = hipMalloc(reinterpret_cast<void**>(&h->d_rowptrs), rebased.size() * sizeof(int64_t));
  if (e == hipSuccess && !cat.empty()) e = hipMalloc(reinterpret_cast<void**>(&h->d_colidx), cat.size() * sizeof(int32_t));
  if (e == hipSuccess && !cat.empty()) e = hipMalloc(reinterpret_cast<void**>(&h->d_values), val.size() * sizeof(float));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    release(h);
    return FUSEDMM_ERR_ALLOC;
  }
  e = hipMemcpy(h->d_rowptrs, rebased.data(), rebased.size() * sizeof(int64_t), hipMemcpyHostToDevice);
  if (e == hipSuccess && !cat.empty()) e = hipMemcpy(h->d_colidx, cat.data(), cat.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess && !cat.empty()) e = hipMemcpy(h->d_values, val.data(), val.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    release(h);
    return FUSEDMM_ERR_HIP;
  }

  int status = FUSEDMM_OK;
  for (int32_t b = 0; b < nb; ++b) {
    const int64_t b0 = (int64_t)b * batch_rows;
    const int64_t rows = (b0 + batch_rows < n ? b0 + batch_rows : n) - b0;
    const int64_t cnt = h->e_off[(size_t)b + 1] - h->e_off[(size_t)b];
    fusedmm_plan_t* p = nullptr;
    // columns outside [0, n), stored or sampled, are rejected here by the plan's own check
    status = fusedmm_plan_create(&p, rows, n, cnt, h->d_rowptrs + (size_t)b * (batch_rows + 1),
                                 cnt > 0 ? h->d_colidx + h->e_off[(size_t)b] : nullptr, nullptr, stream_);
    if (status != FUSEDMM_OK) break;
    h->plans.push_back(p);
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
  for (fusedmm_plan_t* p : h->plans) {
    const int st = fusedmm_plan_reserve(p, d);
    if (st != FUSEDMM_OK) return st;
  }
  if (h->z_d < d) {
    if (hipDeviceSynchronize() != hipSuccess) return FUSEDMM_ERR_HIP;  // earlier epochs may still read the old buffer
    if (h->d_z) (void)hipFree(h->d_z);
    h->d_z = nullptr;
    h->z_d = 0;
    if (hipMalloc(reinterpret_cast<void**>(&h->d_z), (size_t)h->batch_rows * d * sizeof(float)) != hipSuccess)
      return FUSEDMM_ERR_ALLOC;
    h->z_d = d;
  }
  return FUSEDMM_OK;
}

int fusedmm_minibatch_epoch(fusedmm_minibatch_t* h, int32_t d, float lr, float* d_X, int64_t ldx, void* stream_) {
  if (!h || !d_X || ldx < d) return FUSEDMM_ERR_INVALID_ARG;
  if (d < 1 || d > FUSEDMM_MAX_D) return FUSEDMM_ERR_UNSUPPORTED_DIM;
  if (h->z_d < d) return FUSEDMM_ERR_NOT_RESERVED;  // fusedmm_minibatch_reserve(h, d) allocates; an epoch never does
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  // attraction and repulsion in one call: h = a_uv - sigmoid(x_u . x_v), a_uv = 1 on stored entries
  // (1 - sigmoid) and 0 on negative samples (-sigmoid)
  fusedmm_ops_t ops;
  (void)fusedmm_ops_preset(FUSEDMM_PATTERN_SIGMOID_EMBED, &ops);
  ops.sop = fmm::kSopValueMinusSigmoid;
  for (int32_t b = 0; b < h->n_batches; ++b) {
    const int64_t b0 = (int64_t)b * h->batch_rows;
    const int64_t rows = b0 + h->batch_rows < h->n ? h->batch_rows : h->n - b0;
    float* xb = d_X + b0 * ldx;
    const int s = fusedmm_execute_private_ops(h->plans[b], &ops, d, h->d_values ? h->d_values + h->e_off[(size_t)b] : nullptr,
                                              xb, ldx, d_X, ldx, h->d_z, d, stream_);
    if (s != FUSEDMM_OK) return s;
    hipLaunchKernelGGL(embedding_update_kernel, dim3(grid_for(rows * d)), dim3(256), 0, stream, rows, d, lr, h->d_z, xb, ldx);
    if (hipGetLastError() != hipSuccess) return FUSEDMM_ERR_HIP;
  }
  return FUSEDMM_OK;
}

int fusedmm_minibatch_info(const fusedmm_minibatch_t* h, int32_t* n_batches, int64_t* launches_per_epoch) {
  if (!h) return FUSEDMM_ERR_INVALID_ARG;
  if (n_batches) *n_batches = h->n_batches;
  if (launches_per_epoch) {
    int64_t total = 0;
    for (const fusedmm_plan_t* p : h->plans) {
      int64_t split = 0;
      (void)fusedmm_plan_stats(p, nullptr, nullptr, nullptr, &split, nullptr, nullptr, nullptr, nullptr);
      total += 2 + (split > 0 ? 1 : 0);  // execute (+ merge of split rows) and the update
    }
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
