// General FusedMM kernel (any 1 <= d <= 2048, any supported op tuple, any alignment),
// the split-row merge kernel, the colidx validator and the (pattern, d) dispatcher.
#include "fusedmm_internal.h"
#include "../../include/fusedmm.h"

namespace fmm {

typedef float v4f __attribute__((ext_vector_type(4)));

template <class T>
__device__ __forceinline__ T vop_apply(int vop, T x, T y) {
  switch (vop) {
    case FUSEDMM_VOP_MUL: return x * y;
    case FUSEDMM_VOP_SEL2ND: return y;
    case FUSEDMM_VOP_SUB: return x - y;
    default: return x + y;  // ADD
  }
}

// fp32 uses the hardware's exp2 / reciprocal / square root (1 ulp each, as the specialised kernels do);
// fp64 the library routines.  e^big = inf gives 1/(1+inf) = 0, never NaN.
__device__ __forceinline__ float exp_of(float v) { return __builtin_amdgcn_exp2f(v * 1.4426950408889634f); }
__device__ __forceinline__ double exp_of(double v) { return exp(v); }
__device__ __forceinline__ float sqrt_of(float v) { return __builtin_amdgcn_sqrtf(v); }
__device__ __forceinline__ double sqrt_of(double v) { return sqrt(v); }
__device__ __forceinline__ float recip_of(float v) { return __builtin_amdgcn_rcpf(v); }
__device__ __forceinline__ double recip_of(double v) { return 1.0 / v; }

template <class T>
__device__ __forceinline__ T sop_apply(int sop, T s, T alpha) {
  switch (sop) {
    case FUSEDMM_SOP_SIGMOID: return recip_of(T(1) + exp_of(-s));
    case FUSEDMM_SOP_ONE_MINUS_SIGMOID: return recip_of(T(1) + exp_of(s));
    case FUSEDMM_SOP_INV_1P: return recip_of(T(1) + s);
    case FUSEDMM_SOP_SCAL: return alpha * s;
    default: return s;  // NOOP
  }
}

// Algorithm 1, UpdateU, one wavefront per row (or per segment of a long row).  The five steps run per
// stored entry in the paper's order.  A group of G lanes works on one stored entry and owns z_u (lane g of
// the group: elements g, g+G, ... ; NP of them, in registers); rows of up to 32 elements use groups of
// 2 ... 32 lanes, so that a wavefront works on 64/G entries at once, and the groups' results are combined at
// the end (exchange by lane index in a fixed order: reproducible).  Column indices are read 64 at a time;
// x_u is read once; U entries per group are in flight, and the row of Y read for VOP/ROP is kept for MOP.
// Covers every op of Table II: scalar messages (after a reduction, or the edge value) and vector
// messages (no reduction: SOP acts on each element of t); SUM / MAX / MIN accumulation from a
// zero-initialised z_u, and MEAN (the sum divided by the row length).  T is float or double (Section V: the
// method is not tied to single precision).
// Sum (or product) over each aligned group of G lanes, result in every lane of the group.  fp32 takes
// the data-parallel-primitive moves inside a row of 16 lanes (neighbour, quad halves, mirror within 8,
// mirror within 16) and a lane exchange beyond; fp64 exchanges lanes all the way.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <class T, int G>
__device__ __forceinline__ T group_allreduce(T v, bool product) {
  if constexpr (sizeof(T) == 4) {
    float o;
    o = dpp_lane<0xB1>(v);  // quad_perm [1,0,3,2]
    v = product ? v * o : v + o;
    if constexpr (G >= 4) { o = dpp_lane<0x4E>(v); v = product ? v * o : v + o; }   // quad_perm [2,3,0,1]
    if constexpr (G >= 8) { o = dpp_lane<0x141>(v); v = product ? v * o : v + o; }  // row_half_mirror
    if constexpr (G >= 16) { o = dpp_lane<0x140>(v); v = product ? v * o : v + o; } // row_mirror
    if constexpr (G >= 32) { o = __shfl_xor(v, 16); v = product ? v * o : v + o; }
    if constexpr (G >= 64) { o = __shfl_xor(v, 32); v = product ? v * o : v + o; }
    return v;
  } else {
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) {
      const T o = __shfl_xor(v, off);
      v = product ? v * o : v + o;
    }
    return v;
  }
}

template <class T>
__device__ __forceinline__ T aop_apply(int aop, T acc, T w) {
  if (aop == FUSEDMM_AOP_SUM || aop == FUSEDMM_AOP_MEAN) return acc + w;
  if (aop == FUSEDMM_AOP_MAX) return w > acc ? w : acc;  // a NaN message is skipped, as by fmax
  return w < acc ? w : acc;
}

template <class T, int NP, int G, int U>
__global__ __launch_bounds__(kBlockThreads) void fusedmm_generic_kernel(const GenericArgsT<T> a) {
  static_assert(G == 64 || NP == 1, "lane groups narrower than a wavefront hold one element per lane");
  constexpr int S = 64 / G;  // stored entries a wavefront works on at once
  const int lane = threadIdx.x & 63;
  const int slot = lane / G, g = lane % G;
  // wavefronts [0, m): one row each (rows longer than kGenericSplit are left to the segment
  // wavefronts that follow); wavefronts [m, m + n_segs): one segment of a long row each
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (w >= a.m + a.n_segs) return;
  int64_t row, e0, e1;
  T* zr;
  bool whole_row;  // the wavefront stores z_u itself (mean pooling divides here)
  if (w < a.m) {
    row = w;
    e0 = a.rowptr[row];
    e1 = a.rowptr[row + 1];
    if (e1 - e0 > kGenericSplit) return;
    zr = a.Z + row * a.ldz;
    whole_row = true;
  } else {
    const ChunkDesc sg = a.segs[w - a.m];
    row = sg.row;
    e0 = sg.e_begin;
    e1 = sg.e_begin + sg.e_count;
    zr = a.partials + (int64_t)sg.part * a.d;
    whole_row = false;
  }
  const int d = a.d;
  if (a.visit_counts) {
    for (int64_t e = e0 + lane; e < e1; e += 64) atomicAdd(a.visit_counts + e, 1u);
    return;
  }
  const bool uses_x = a.vop != FUSEDMM_VOP_SEL2ND;
  const bool scalar_h = a.sop == FUSEDMM_SOP_EDGE_VALUE || a.rop != FUSEDMM_ROP_NOOP;
  const bool reads_val = a.sop == FUSEDMM_SOP_EDGE_VALUE || a.sop == kSopValueMinusSigmoid;
  const bool product = a.rop == FUSEDMM_ROP_RMUL;
  T x[NP], acc[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    const int k = g + G * i;
    x[i] = (uses_x && k < d) ? a.X[row * a.ldx + k] : T(0);
    acc[i] = T(0);  // z_u <- 0
  }

  for (int64_t base = e0; base < e1; base += 64) {
    const int cnt = (int)((e1 - base) < 64 ? (e1 - base) : 64);  // wave-uniform
    int colb = 0;
    T valb = T(0);
    if (lane < cnt) {
      colb = a.colidx[base + lane];
      if (reads_val) valb = a.values[base + lane];
    }
    for (int k0 = 0; k0 < cnt; k0 += S * U) {
      bool ok[U];
      T av[U];
      T y[U][NP];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = k0 + u * S + slot;
        ok[u] = j < cnt;
        const int c = __shfl(colb, j & 63);
        av[u] = __shfl(valb, j & 63);
        const T* yr = a.Y + (int64_t)c * a.ldy;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
          const int k = g + G * i;
          y[u][i] = (ok[u] && k < d) ? yr[k] : T(0);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (k0 + u * S >= cnt) break;  // wave-uniform: no group has an entry in this step
        T h = T(0);
        if (a.sop == FUSEDMM_SOP_EDGE_VALUE) {
          h = av[u];
        } else if (a.rop != FUSEDMM_ROP_NOOP) {
          T p = product ? T(1) : T(0);
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            const T t = vop_apply<T>(a.vop, x[i], y[u][i]);  // VOP (0 beyond d: x and y are 0 there)
            if (a.rop == FUSEDMM_ROP_RSUM) p += t;            // ROP (per-lane share)
            else if (product) p *= (g + G * i < d) ? t : T(1);
            else p += t * t;
          }
          T s = group_allreduce<T, G>(p, product);
          if (a.rop == FUSEDMM_ROP_NORM2) s = sqrt_of(s);
          h = a.sop == kSopValueMinusSigmoid ? av[u] - sop_apply<T>(FUSEDMM_SOP_SIGMOID, s, a.alpha)
                                             : sop_apply<T>(a.sop, s, a.alpha);  // SOP on the scalar
        }
#pragma unroll
        for (int i = 0; i < NP; ++i) {
          if (ok[u] && g + G * i < d) {
            const T yk = y[u][i];
            const T t = vop_apply<T>(a.vop, x[i], yk);
            const T hk = scalar_h ? h : sop_apply<T>(a.sop, t, a.alpha);  // SOP on the element
            T wk;                                                           // MOP
            if (a.mop == FUSEDMM_MOP_SEL2ND) wk = yk;
            else if (a.mop == FUSEDMM_MOP_MUL_Y) wk = hk * yk;
            else wk = hk * t;
            acc[i] = aop_apply<T>(a.aop, acc[i], wk);                       // AOP
          }
        }
      }
    }
  }
  if constexpr (S > 1) {  // the groups' shares of z_u
#pragma unroll
    for (int off = G; off < 64; off <<= 1) acc[0] = aop_apply<T>(a.aop, acc[0], __shfl_xor(acc[0], off));
  }
  const T post = (whole_row && a.aop == FUSEDMM_AOP_MEAN && e1 > e0) ? T(1) / (T)(e1 - e0) : T(1);  // mean pooling
  if (slot == 0) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int k = g + G * i;
      if (k < d) zr[k] = acc[i] * post;
    }
  }
}

// z_u of a row that the general kernel cut into segments: its partial rows combined in segment
// order (SUM / MAX / MIN; MEAN: summed, then divided by the row length).  One wavefront per row.
template <class T>
__global__ __launch_bounds__(kBlockThreads) void fusedmm_generic_merge_kernel(const GenericArgsT<T> a) {
  const int lane = threadIdx.x & 63;
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (w >= a.n_merges) return;
  const MergeDesc md = a.merges[w];
  const T* src = a.partials + (int64_t)md.first_part * a.d;
  const T post = a.aop == FUSEDMM_AOP_MEAN ? T(1) / (T)(a.rowptr[md.row + 1] - a.rowptr[md.row]) : T(1);
  for (int k = lane; k < a.d; k += 64) {
    T s = src[k];
    for (int p = 1; p < md.n_parts; ++p) {
      const T v = src[(int64_t)p * a.d + k];
      if (a.aop == FUSEDMM_AOP_SUM || a.aop == FUSEDMM_AOP_MEAN) s += v;
      else if (a.aop == FUSEDMM_AOP_MAX) s = v > s ? v : s;
      else s = v < s ? v : s;
    }
    a.Z[(int64_t)md.row * a.ldz + k] = s * post;
  }
}

template <class T>
static hipError_t launch_generic_t(const GenericArgsT<T>& a, hipStream_t stream) {
  if (a.m <= 0) return hipSuccess;
  const int64_t waves = a.m + a.n_segs;
  const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
  static_assert(FUSEDMM_MAX_D == 64 * 32, "the widest instance holds 32 elements per lane");
#define FMM_GENERIC(NP, G, U) \
  hipLaunchKernelGGL((fusedmm_generic_kernel<T, NP, G, U>), dim3((unsigned)blocks), dim3(kBlockThreads), 0, stream, a)
  if (a.d <= 2) FMM_GENERIC(1, 2, 4);
  else if (a.d <= 4) FMM_GENERIC(1, 4, 4);
  else if (a.d <= 8) FMM_GENERIC(1, 8, 4);
  else if (a.d <= 16) FMM_GENERIC(1, 16, 4);
  else if (a.d <= 32) FMM_GENERIC(1, 32, 4);
  else if (a.d <= 64) FMM_GENERIC(1, 64, 4);
  else if (a.d <= 128) FMM_GENERIC(2, 64, 4);
  else if (a.d <= 256) FMM_GENERIC(4, 64, 2);
  else if (a.d <= 512) FMM_GENERIC(8, 64, 2);
  else FMM_GENERIC(32, 64, 1);
#undef FMM_GENERIC
  hipError_t e = hipGetLastError();
  if (e == hipSuccess && a.n_merges > 0 && !a.visit_counts) {
    const int64_t mblocks = ((int64_t)a.n_merges + kWavesPerBlock - 1) / kWavesPerBlock;
    hipLaunchKernelGGL(fusedmm_generic_merge_kernel<T>, dim3((unsigned)mblocks), dim3(kBlockThreads), 0, stream, a);
    e = hipGetLastError();
  }
  return e;
}
hipError_t launch_generic(const GenericArgsT<float>& a, hipStream_t stream) { return launch_generic_t(a, stream); }
hipError_t launch_generic(const GenericArgsT<double>& a, hipStream_t stream) { return launch_generic_t(a, stream); }

// z_u = sum of the row's partial rows, in slot order (fixed order => run-to-run deterministic).
// A workgroup covers 256 / (d/4) rows; a thread owns one 16-byte column of one row and keeps
// eight partial-row loads in flight.
template <class V4>
__device__ __forceinline__ V4 merge_two(int aop, V4 s, V4 t) {
  if (aop == FUSEDMM_AOP_SUM || aop == FUSEDMM_AOP_MEAN) return s + t;
  if (aop == FUSEDMM_AOP_MAX) return V4{fmax(s.x, t.x), fmax(s.y, t.y), fmax(s.z, t.z), fmax(s.w, t.w)};
  return V4{fmin(s.x, t.x), fmin(s.y, t.y), fmin(s.z, t.z), fmin(s.w, t.w)};
}

// E: float, or double (a thread then owns a 32-byte column).  d need not be a multiple of 4 (the last column of
// a row then holds d % 4 elements, stored one by one) and the rows of Z may start at any element.
template <class E>
__global__ __launch_bounds__(256) void fusedmm_merge_kernel(const MergeDesc* merges, int32_t n_merges,
                                                           const E* partials, int32_t d, int32_t pstride,
                                                           int32_t aop, const int64_t* rowptr, E* Z, int64_t ldz) {
  typedef E V4 __attribute__((ext_vector_type(4)));
  typedef E V4G __attribute__((ext_vector_type(4), aligned(sizeof(E))));
  const int cols = (d + 3) >> 2;
  const int cols_here = cols < 256 ? cols : 256;  // rows of more than 256 columns take gridDim.y workgroups each
  const int rows_per_block = 256 / cols_here;
  const int r = threadIdx.x / cols_here, c = blockIdx.y * 256 + (threadIdx.x - r * cols_here);
  const int64_t mi = (int64_t)blockIdx.x * rows_per_block + r;
  if (r >= rows_per_block || mi >= n_merges || c >= cols) return;
  const MergeDesc md = merges[mi];
  const E* src = partials + (int64_t)md.first_part * pstride + 4 * c;  // partial rows are pstride >= 4 * cols apart
  V4 s = {0, 0, 0, 0};
  int p = 0;
  for (; p + 8 <= md.n_parts; p += 8) {
    V4 t[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) t[k] = __builtin_nontemporal_load(reinterpret_cast<const V4*>(src + (int64_t)(p + k) * pstride));
#pragma unroll
    for (int k = 0; k < 8; ++k) s = merge_two(aop, s, t[k]);
  }
  for (; p < md.n_parts; ++p)
    s = merge_two(aop, s, __builtin_nontemporal_load(reinterpret_cast<const V4*>(src + (int64_t)p * pstride)));
  if (aop == FUSEDMM_AOP_MEAN) s *= (E)1 / (E)(rowptr[md.row + 1] - rowptr[md.row]);  // split rows are never empty
  E* dst = Z + (int64_t)md.row * ldz + 4 * c;
  const int left = d - 4 * c;
  if (left >= 4) {
    __builtin_nontemporal_store(static_cast<V4G>(s), reinterpret_cast<V4G*>(dst));
  } else {  // the row ends inside this column (what the partial rows hold beyond it was never written)
    __builtin_nontemporal_store(s.x, dst);
    if (left > 1) __builtin_nontemporal_store(s.y, dst + 1);
    if (left > 2) __builtin_nontemporal_store(s.z, dst + 2);
  }
}

template <class E>
static hipError_t launch_merge_t(const MergeDesc* merges, int32_t n_merges, const E* partials, int32_t d, int32_t pstride,
                                 int32_t aop, const int64_t* rowptr, E* Z, int64_t ldz, hipStream_t stream) {
  if (n_merges <= 0) return hipSuccess;
  const int cols = (d + 3) >> 2;
  const int rows_per_block = 256 / (cols < 256 ? cols : 256);
  const int64_t blocks = ((int64_t)n_merges + rows_per_block - 1) / rows_per_block;
  hipLaunchKernelGGL(fusedmm_merge_kernel<E>, dim3((unsigned)blocks, (unsigned)((cols + 255) / 256)), dim3(256), 0, stream, merges,
                     n_merges, partials, d, pstride, aop, rowptr, Z, ldz);
  return hipGetLastError();
}
hipError_t launch_merge(const MergeDesc* merges, int32_t n_merges, const float* partials, int32_t d, int32_t pstride,
                        int32_t aop, const int64_t* rowptr, float* Z, int64_t ldz, hipStream_t stream) {
  return launch_merge_t(merges, n_merges, partials, d, pstride, aop, rowptr, Z, ldz, stream);
}
hipError_t launch_merge(const MergeDesc* merges, int32_t n_merges, const double* partials, int32_t d, int32_t pstride,
                        int32_t aop, const int64_t* rowptr, double* Z, int64_t ldz, hipStream_t stream) {
  return launch_merge_t(merges, n_merges, partials, d, pstride, aop, rowptr, Z, ldz, stream);
}

__global__ __launch_bounds__(256) void validate_colidx_kernel(const int32_t* colidx, int64_t nnz, int64_t n, int32_t* flag) {
  bool bad = false;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nnz; i += (int64_t)gridDim.x * blockDim.x) {
    const int32_t c = colidx[i];
    bad |= (c < 0) || ((int64_t)c >= n);
  }
  if (bad) atomicOr(flag, 1);
}

hipError_t launch_validate_colidx(const int32_t* colidx, int64_t nnz, int64_t n, int32_t* flag, hipStream_t stream) {
  if (nnz <= 0) return hipSuccess;
  int64_t blocks = (nnz + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(validate_colidx_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, colidx, nnz, n, flag);
  return hipGetLastError();
}

// hist[b] += 1 for every `stride`-th stored entry, b the bucket of its column (column * n_buckets / n): where
// the stored entries lie along the column range, for class boundaries that balance them.
__global__ __launch_bounds__(256) void column_histogram_kernel(const int32_t* colidx, int64_t nnz, int64_t stride, int64_t n,
                                                               int32_t n_buckets, uint32_t* hist) {
  const int64_t samples = (nnz + stride - 1) / stride;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < samples; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t c = colidx[i * stride];
    atomicAdd(hist + (int32_t)(c * n_buckets / n), 1u);
  }
}

hipError_t launch_column_histogram(const int32_t* colidx, int64_t nnz, int64_t stride, int64_t n, int32_t n_buckets,
                                   uint32_t* hist, hipStream_t stream) {
  if (nnz <= 0) return hipSuccess;
  const int64_t samples = (nnz + stride - 1) / stride;
  int64_t blocks = (samples + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(column_histogram_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, colidx, nnz, stride, n, n_buckets, hist);
  return hipGetLastError();
}

// One wavefront per tiled row: is the row sorted by column, and where does each of its column
// classes start?  A row of level L has L classes, each n_classes / L finest classes wide.
__global__ __launch_bounds__(kBlockThreads) void tile_bounds_kernel(const int64_t* rowptr, const int32_t* colidx,
                                                                    const int32_t* rows, const int32_t* level,
                                                                    const int64_t* out_off, int32_t n_rows,
                                                                    int32_t n_classes, const int32_t* class_start,
                                                                    int32_t* bounds, int32_t* unsorted) {
  const int lane = threadIdx.x & 63;
  const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  if (w >= n_rows) return;
  const int32_t row = rows[w];
  const int32_t L = level[w];
  const int stride = n_classes / L;  // finest classes per class of this row
  const int64_t e0 = rowptr[row];
  const int64_t len = rowptr[row + 1] - e0;
  bool bad = false;
  for (int64_t i = lane; i + 1 < len; i += 64) bad |= colidx[e0 + i] > colidx[e0 + i + 1];
  if (bad) atomicOr(unsorted, 1);
  int32_t* out = bounds + out_off[w];
  for (int c = lane; c <= L; c += 64) {
    const int64_t target = class_start[c * stride];  // first column id of class c
    int64_t lo = 0, hi = len;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if ((int64_t)colidx[e0 + mid] < target) lo = mid + 1; else hi = mid;
    }
    out[c] = (int32_t)lo;
  }
}

hipError_t launch_tile_bounds(const int64_t* rowptr, const int32_t* colidx, const int32_t* rows, const int32_t* level,
                              const int64_t* out_off, int32_t n_rows, int32_t n_classes, const int32_t* class_start,
                              int32_t* bounds, int32_t* unsorted, hipStream_t stream) {
  if (n_rows <= 0) return hipSuccess;
  const int blocks = (n_rows + kWavesPerBlock - 1) / kWavesPerBlock;
  hipLaunchKernelGGL(tile_bounds_kernel, dim3((unsigned)blocks), dim3(kBlockThreads), 0, stream, rowptr, colidx, rows,
                     level, out_off, n_rows, n_classes, class_start, bounds, unsorted);
  return hipGetLastError();
}

// Plain streaming copy, 16 bytes per thread per step (counter calibration).
__global__ __launch_bounds__(256) void fusedmm_copy_kernel(v4f* dst, const v4f* src, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(fusedmm_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<v4f*>(dst),
                     static_cast<const v4f*>(src), n16);
  return hipGetLastError();
}

// ---- dispatcher over the per-dimension translation units --------------------------------
#define FMM_DECL(D)                                                                   \
  hipError_t launch_fast##D(int pattern, int y_format, const KernelArgs& a, hipStream_t stream); \
  int packed_rows_per_block##D(int pattern, int y_format);
FMM_DECL(_d32) FMM_DECL(_d64) FMM_DECL(_d128) FMM_DECL(_d256) FMM_DECL(_d512) FMM_DECL(_d1024) FMM_DECL(_d2048)
FMM_DECL(_d96) FMM_DECL(_d192) FMM_DECL(_d384) FMM_DECL(_d768) FMM_DECL(_d1536)
FMM_DECL(_f64_d32) FMM_DECL(_f64_d64) FMM_DECL(_f64_d128) FMM_DECL(_f64_d256) FMM_DECL(_f64_d512)
FMM_DECL(_f64_d1024) FMM_DECL(_f64_d2048)
#undef FMM_DECL

int packed_rows_per_block(int pattern, int d, int y_format) {
  if (y_format == kYF64) {
    switch (d) {
      case 32: return packed_rows_per_block_f64_d32(pattern, kYF32);
      case 64: return packed_rows_per_block_f64_d64(pattern, kYF32);
      case 128: return packed_rows_per_block_f64_d128(pattern, kYF32);
      case 256: return packed_rows_per_block_f64_d256(pattern, kYF32);
      case 512: return packed_rows_per_block_f64_d512(pattern, kYF32);
      case 1024: return packed_rows_per_block_f64_d1024(pattern, kYF32);
      case 2048: return packed_rows_per_block_f64_d2048(pattern, kYF32);
      default: return 0;
    }
  }
  switch (d) {
    case 32: return packed_rows_per_block_d32(pattern, y_format);
    case 64: return packed_rows_per_block_d64(pattern, y_format);
    case 128: return packed_rows_per_block_d128(pattern, y_format);
    case 256: return packed_rows_per_block_d256(pattern, y_format);
    case 512: return packed_rows_per_block_d512(pattern, y_format);
    case 1024: return packed_rows_per_block_d1024(pattern, y_format);
    case 2048: return packed_rows_per_block_d2048(pattern, y_format);
    case 96: return packed_rows_per_block_d96(pattern, y_format);
    case 192: return packed_rows_per_block_d192(pattern, y_format);
    case 384: return packed_rows_per_block_d384(pattern, y_format);
    case 768: return packed_rows_per_block_d768(pattern, y_format);
    case 1536: return packed_rows_per_block_d1536(pattern, y_format);
    default: return 0;
  }
}

hipError_t launch_fast(int pattern, int d, int y_format, const KernelArgs& a, hipStream_t stream) {
  if (y_format == kYF64) {
    switch (d) {
      case 32: return launch_fast_f64_d32(pattern, kYF32, a, stream);
      case 64: return launch_fast_f64_d64(pattern, kYF32, a, stream);
      case 128: return launch_fast_f64_d128(pattern, kYF32, a, stream);
      case 256: return launch_fast_f64_d256(pattern, kYF32, a, stream);
      case 512: return launch_fast_f64_d512(pattern, kYF32, a, stream);
      case 1024: return launch_fast_f64_d1024(pattern, kYF32, a, stream);
      case 2048: return launch_fast_f64_d2048(pattern, kYF32, a, stream);
      default: return hipErrorInvalidValue;
    }
  }
  switch (d) {
    case 32: return launch_fast_d32(pattern, y_format, a, stream);
    case 64: return launch_fast_d64(pattern, y_format, a, stream);
    case 128: return launch_fast_d128(pattern, y_format, a, stream);
    case 256: return launch_fast_d256(pattern, y_format, a, stream);
    case 512: return launch_fast_d512(pattern, y_format, a, stream);
    case 1024: return launch_fast_d1024(pattern, y_format, a, stream);
    case 2048: return launch_fast_d2048(pattern, y_format, a, stream);
    case 96: return launch_fast_d96(pattern, y_format, a, stream);
    case 192: return launch_fast_d192(pattern, y_format, a, stream);
    case 384: return launch_fast_d384(pattern, y_format, a, stream);
    case 768: return launch_fast_d768(pattern, y_format, a, stream);
    case 1536: return launch_fast_d1536(pattern, y_format, a, stream);
    default: return hipErrorInvalidValue;
  }
}

// fp32 -> bfloat16, round to nearest even on the discarded 16 bits; a NaN keeps a set mantissa bit.
__global__ __launch_bounds__(256) void to_bf16_kernel(uint16_t* dst, const float* src, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, src[i]);
    uint32_t r;
    if ((u & 0x7fffffffu) > 0x7f800000u) r = (u >> 16) | 0x0040u;  // NaN
    else r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    dst[i] = (uint16_t)r;
  }
}

// fp32 -> IEEE half, round to nearest even (the hardware conversion); overflow gives infinity.
__global__ __launch_bounds__(256) void to_f16_kernel(uint16_t* dst, const float* src, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = __builtin_bit_cast(uint16_t, (_Float16)src[i]);
}

hipError_t launch_to_f16(uint16_t* dst, const float* src, size_t count, hipStream_t stream) {
  if (count == 0) return hipSuccess;
  size_t blocks = (count + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dst, src, count);
  return hipGetLastError();
}

hipError_t launch_to_bf16(uint16_t* dst, const float* src, size_t count, hipStream_t stream) {
  if (count == 0) return hipSuccess;
  size_t blocks = (count + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(to_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, dst, src, count);
  return hipGetLastError();
}

}  // namespace fmm
