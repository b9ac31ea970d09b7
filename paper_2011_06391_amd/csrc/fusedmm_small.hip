// FusedMM for very short feature vectors: d = 2, 3, 4, 8 or 16 (the layout application of Table III row 1
// runs in 2 or 3 dimensions).  A lane group of the wide kernels holds d/4 floats per lane along the feature
// dimension; here the whole vector fits one lane, so the roles turn round: one lane per stored entry.  A lane
// keeps x_u and its own partial z_u (d floats each) in registers, gathers y_v with one short load, runs
// VOP / ROP / SOP / MOP without any cross-lane step (Algorithm 1's UpdateU, all five steps lane-local), and
// AOP is finished by a reduction across the lanes that share a row.  The schedule is the plan's own: the same
// bins (packed rows, one-wavefront rows, workgroup chunks, column-class tiles, rows without entries), the same
// descriptors and block ranges as the wide kernels, so no stored entry is visited twice and results are
// reproducible bit for bit (fixed order of every sum).
#include "fusedmm_device.h"

namespace fmm {

namespace {

// AOP of a compile-time pattern is SUM; the run-time-ops instance reads it from the arguments.
template <int P>
__device__ __forceinline__ float small_aop(const KernelArgs& a, float z, float w) {
  if constexpr (P == PAT_RUNTIME) return aop_apply(a.aop, z, w); else return z + w;
}

// The five steps for one stored entry, all in one lane: acc = AOP(acc, MOP(SOP(ROP(VOP(x, y))), .)).
template <int P, int D>
__device__ __forceinline__ void small_entry(const KernelArgs& a, const float (&x)[D], const float (&y)[D], float aval,
                                            bool valid, float (&acc)[D]) {
  constexpr float kLog2e = 1.4426950408889634f;
  float w[D];
  if constexpr (P == PAT_RUNTIME) {
    float t[D];
#pragma unroll
    for (int i = 0; i < D; ++i) t[i] = rt_vop(a.vop, x[i], y[i]);
    const bool scalar_h = a.sop == FUSEDMM_SOP_EDGE_VALUE || a.rop != FUSEDMM_ROP_NOOP;
    float h = aval;
    if (a.sop != FUSEDMM_SOP_EDGE_VALUE && a.rop != FUSEDMM_ROP_NOOP) {
      float s;
      if (a.rop == FUSEDMM_ROP_RMUL) {
        s = 1.f;
#pragma unroll
        for (int i = 0; i < D; ++i) s *= t[i];
      } else if (a.rop == FUSEDMM_ROP_RSUM) {
        s = 0.f;
#pragma unroll
        for (int i = 0; i < D; ++i) s += t[i];
      } else {
        s = 0.f;
#pragma unroll
        for (int i = 0; i < D; ++i) s = __builtin_fmaf(t[i], t[i], s);
        if (a.rop == FUSEDMM_ROP_NORM2) s = __builtin_amdgcn_sqrtf(s);
      }
      h = a.sop == kSopValueMinusSigmoid ? aval - rt_sop(FUSEDMM_SOP_SIGMOID, s, a.alpha) : rt_sop(a.sop, s, a.alpha);
    }
#pragma unroll
    for (int i = 0; i < D; ++i) {
      const float hi = scalar_h ? h : rt_sop(a.sop, t[i], a.alpha);  // vector message: SOP on every element of t
      w[i] = a.mop == FUSEDMM_MOP_SEL2ND ? y[i] : (a.mop == FUSEDMM_MOP_MUL_Y ? hi * y[i] : hi * t[i]);
    }
  } else if constexpr (P == PAT_GCN) {
#pragma unroll
    for (int i = 0; i < D; ++i) w[i] = aval * y[i];
  } else if constexpr (P == PAT_SIGMOID || P == PAT_ONE_MINUS_SIGMOID) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) s = __builtin_fmaf(x[i], y[i], s);
    const float h = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(P == PAT_ONE_MINUS_SIGMOID ? s * kLog2e : -s * kLog2e));
#pragma unroll
    for (int i = 0; i < D; ++i) w[i] = h * y[i];
  } else {  // PAT_TDIST, PAT_FR
    float t[D], s = 0.f;
#pragma unroll
    for (int i = 0; i < D; ++i) {
      t[i] = x[i] - y[i];
      s = __builtin_fmaf(t[i], t[i], s);
    }
    const float h = (P == PAT_TDIST) ? __builtin_amdgcn_rcpf(1.0f + s) : a.alpha * __builtin_amdgcn_sqrtf(s);
#pragma unroll
    for (int i = 0; i < D; ++i) w[i] = h * t[i];
  }
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = small_aop<P>(a, acc[i], valid ? w[i] : 0.f);  // 0 is neutral from the zero start
}

// d consecutive floats that are only known to be 4-byte aligned (any leading dimension)
template <int D>
__device__ __forceinline__ void load_vec(const float* p, float (&v)[D]) {
  typedef float vec __attribute__((ext_vector_type(D == 3 ? 3 : (D >= 4 ? 4 : 2)), aligned(4)));
  if constexpr (D <= 4) {
    const vec r = *reinterpret_cast<const vec*>(p);
#pragma unroll
    for (int i = 0; i < D; ++i) v[i] = r[i];
  } else {
#pragma unroll
    for (int j = 0; j < D / 4; ++j) {
      const vec r = *reinterpret_cast<const vec*>(p + 4 * j);
#pragma unroll
      for (int i = 0; i < 4; ++i) v[4 * j + i] = r[i];
    }
  }
}

// One lane's share of the entries [e0, e0 + cnt): entries l, l + W, l + 2W, ... (W lanes work on the run),
// U of them in flight.
template <int P, int D, int W, int U>
__device__ __forceinline__ void small_accumulate(const KernelArgs& a, int64_t e0, int cnt, int l, const float (&x)[D],
                                                 float (&acc)[D]) {
  using T = PatTraits<P>;
  const bool use_val = reads_values<P>(a);
  const float* Y = static_cast<const float*>(a.Y);
  for (int k = l; k < cnt; k += W * U) {
    bool ok[U];
    int c[U];
    float av[U];
    float y[U][D];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      ok[u] = k + u * W < cnt;
      c[u] = ok[u] ? a.colidx[e0 + k + u * W] : 0;
      av[u] = (ok[u] && use_val) ? values_of(a)[e0 + k + u * W] : 0.f;
    }
    if constexpr (T::loads_y) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int i = 0; i < D; ++i) y[u][i] = 0.f;
        if (ok[u]) load_vec<D>(Y + (int64_t)c[u] * a.ldy, y[u]);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) small_entry<P, D>(a, x, y[u], av[u], ok[u], acc);
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (ok[u]) atomicAdd(a.visit_counts + (e0 + k + u * W), 1u);
    }
  }
}

// AOP across the W lanes that worked on one run, fixed order; every lane ends up with the result.
template <int P, int D, int W>
__device__ __forceinline__ void small_reduce(const KernelArgs& a, float (&acc)[D]) {
#pragma unroll
  for (int i = 0; i < D; ++i) {
    float v = acc[i];
    v = small_aop<P>(a, v, lane_xor<1>(v));
    v = small_aop<P>(a, v, lane_xor<2>(v));
    v = small_aop<P>(a, v, lane_xor<4>(v));
    if constexpr (W >= 16) v = small_aop<P>(a, v, lane_xor<8>(v));
    if constexpr (W >= 32) v = small_aop<P>(a, v, lane_xor<16>(v));
    if constexpr (W >= 64) v = small_aop<P>(a, v, lane_xor<32>(v));
    acc[i] = v;
  }
}

template <int D>
__device__ __forceinline__ void store_vec(float* dst, const float (&v)[D], float scale) {
#pragma unroll
  for (int i = 0; i < D; ++i) dst[i] = v[i] * scale;
}

}  // namespace

// G: lanes per packed row (entries taken per step); UW / UP: entries per lane in flight in the one-wavefront
// and chunk runs / in the longer packed rows.
template <int P, int D, int G, int UW, int UP>
__global__ __launch_bounds__(kBlockThreads) void fusedmm_small_kernel(const KernelArgs a) {
  using T = PatTraits<P>;
  constexpr int S = 64 / G;
  constexpr int kRowsPerRound = kWavesPerBlock * S;  // rows (or tile segments) the workgroup's lane groups hold at once
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int b = blockIdx.x;
  __shared__ float stage[kWavesPerBlock][D];

  int kind, first, count;
  bool from_desc;
  if (b < a.nb_tiled) {
    const BlockItem it = a.items[b];
    kind = it.kind; first = it.first; count = it.count; from_desc = true;
  } else if (b < a.nb_tiled + a.nb_chunk) {
    kind = kItemChunk; first = b - a.nb_tiled; count = 1; from_desc = false;
  } else if (b < a.nb_tiled + a.nb_chunk + a.nb_wave) {
    kind = kItemWave; first = (b - a.nb_tiled - a.nb_chunk) * kWavesPerBlock;
    count = a.n_wave - first < kWavesPerBlock ? a.n_wave - first : kWavesPerBlock; from_desc = false;
  } else if (b < a.nb_tiled + a.nb_chunk + a.nb_wave + a.nb_packed) {
    constexpr int kRows = kRowsPerRound;
    kind = kItemPacked; first = (b - a.nb_tiled - a.nb_chunk - a.nb_wave) * kRows;
    count = a.n_packed - first < kRows ? a.n_packed - first : kRows; from_desc = false;
  } else {
    kind = kItemZero; first = (b - a.nb_tiled - a.nb_chunk - a.nb_wave - a.nb_packed) * kZeroRowsPerBlock;
    count = a.n_empty - first < kZeroRowsPerBlock ? a.n_empty - first : kZeroRowsPerBlock; from_desc = false;
  }

  float x[D], acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) { x[i] = 0.f; acc[i] = 0.f; }  // z_u <- 0

  if (kind == kItemChunk) {
    const ChunkDesc ch = from_desc ? a.tile_descs[first] : a.chunks[first];
    const int per = ((ch.e_count + kWavesPerBlock * 64 - 1) / (kWavesPerBlock * 64)) * 64;
    const int lo = wave * per < ch.e_count ? wave * per : ch.e_count;
    const int hi = (wave + 1) * per < ch.e_count ? (wave + 1) * per : ch.e_count;
    if (reads_x<P>(a)) load_vec<D>(X_of(a) + (int64_t)ch.row * a.ldx, x);
    small_accumulate<P, D, 64, UW>(a, ch.e_begin + lo, hi - lo, lane, x, acc);
    if constexpr (T::loads_y) {
      small_reduce<P, D, 64>(a, acc);
      if (lane == 0) {
#pragma unroll
        for (int i = 0; i < D; ++i) stage[wave][i] = acc[i];
      }
      __syncthreads();
      if (threadIdx.x < D) {
        float s = stage[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) s = small_aop<P>(a, s, stage[w][threadIdx.x]);
        if (a.mean && ch.part < 0) s *= 1.0f / (float)ch.e_count;  // the chunk is the whole row
        float* dst = ch.part < 0 ? Z_of(a) + (int64_t)ch.row * a.ldz : partials_of(a) + (int64_t)ch.part * kSmallPartialStride;
        dst[threadIdx.x] = s;
      }
    }
  } else if (kind == kItemWave) {
    if (wave >= count) return;
    int row;
    int64_t e0, e1;
    float* dst;
    if (from_desc) {
      const ChunkDesc td = a.tile_descs[first + wave];
      row = td.row; e0 = td.e_begin; e1 = td.e_begin + td.e_count;
      dst = partials_of(a) + (int64_t)td.part * kSmallPartialStride;
    } else {
      row = __builtin_amdgcn_readfirstlane(a.order[first + wave]);
      e0 = a.rowptr[row]; e1 = a.rowptr[row + 1];
      dst = Z_of(a) + (int64_t)row * a.ldz;
    }
    if (reads_x<P>(a)) load_vec<D>(X_of(a) + (int64_t)row * a.ldx, x);
    small_accumulate<P, D, 64, UW>(a, e0, (int)(e1 - e0), lane, x, acc);
    if constexpr (T::loads_y) {
      small_reduce<P, D, 64>(a, acc);
      if (lane == 0) store_vec<D>(dst, acc, (a.mean && !from_desc) ? 1.0f / (float)(e1 - e0) : 1.0f);
    }
  } else if (kind == kItemPacked) {
    const int slot = lane / G;
    const int g = lane % G;
    for (int round = 0; round < count; round += kRowsPerRound) {
      const int idx = round + wave * S + slot;
      const bool has_seg = idx < count;
      int64_t row = 0, e0 = 0;
      int deg = 0;
      float* dst = nullptr;
      if (has_seg) {
        if (from_desc) {
          const ChunkDesc td = a.tile_descs[first + idx];
          row = td.row; e0 = td.e_begin; deg = td.e_count;
          dst = partials_of(a) + (int64_t)td.part * kSmallPartialStride;
        } else {
          row = a.order[a.n_wave + first + idx];
          e0 = a.rowptr[row];
          deg = (int)(a.rowptr[row + 1] - e0);
          dst = Z_of(a) + row * a.ldz;
        }
      }
#pragma unroll
      for (int i = 0; i < D; ++i) { x[i] = 0.f; acc[i] = 0.f; }
      if (reads_x<P>(a)) {
        if (deg > 0) load_vec<D>(X_of(a) + row * a.ldx, x);
      }
      // rows come sorted by length, so the lane groups of a wavefront hold rows of about the same length:
      // the number of entries per lane taken at once follows the longest of them (wave-uniform)
      int maxdeg = deg;
      maxdeg = max(maxdeg, __shfl_xor(maxdeg, 8));
      maxdeg = max(maxdeg, __shfl_xor(maxdeg, 16));
      maxdeg = max(maxdeg, __shfl_xor(maxdeg, 32));
      maxdeg = __builtin_amdgcn_readfirstlane(maxdeg);
      if (maxdeg <= G) small_accumulate<P, D, G, 1>(a, e0, deg, g, x, acc);
      else if (maxdeg <= 2 * G) small_accumulate<P, D, G, 2>(a, e0, deg, g, x, acc);
      else small_accumulate<P, D, G, UP>(a, e0, deg, g, x, acc);
      if constexpr (T::loads_y) {
        small_reduce<P, D, G>(a, acc);
        if (has_seg && g == 0) store_vec<D>(dst, acc, (a.mean && !from_desc && deg > 0) ? 1.0f / (float)deg : 1.0f);
      }
    }
  } else if (kind == kItemZero) {
    if constexpr (T::loads_y) {
      const int32_t* rows = a.order + a.n_wave + a.n_packed + first;
      for (int i = threadIdx.x; i < count * D; i += kBlockThreads) Z_of(a)[(int64_t)rows[i / D] * a.ldz + (i % D)] = 0.f;
    }
  }
}

// z_u of the rows cut into pieces: their partial rows combined in slot order.  One thread per output element.
__global__ __launch_bounds__(256) void fusedmm_small_merge_kernel(const MergeDesc* merges, int32_t n_merges,
                                                                 const float* partials, int32_t d, int32_t aop,
                                                                 const int64_t* rowptr, float* Z, int64_t ldz) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= (int64_t)n_merges * d) return;
  const MergeDesc md = merges[t / d];
  const int k = (int)(t % d);
  const float* src = partials + (int64_t)md.first_part * kSmallPartialStride + k;
  float s = src[0];
  for (int p = 1; p < md.n_parts; ++p) {
    const float v = src[(int64_t)p * kSmallPartialStride];
    s = (aop == FUSEDMM_AOP_SUM || aop == FUSEDMM_AOP_MEAN) ? s + v : (aop == FUSEDMM_AOP_MAX ? fmaxf(s, v) : fminf(s, v));
  }
  if (aop == FUSEDMM_AOP_MEAN) s *= 1.0f / (float)(rowptr[md.row + 1] - rowptr[md.row]);
  Z[(int64_t)md.row * ldz + k] = s;
}

namespace {

// The entries in flight shrink with d so that the gathered vectors stay in registers.
constexpr int kSmallG = 8;

template <int P, int D>
hipError_t launch_small_one(const KernelArgs& a, hipStream_t stream) {
  const int64_t blocks = (int64_t)a.nb_tiled + a.nb_chunk + a.nb_wave + a.nb_packed + a.nb_zero;
  if (blocks <= 0) return hipSuccess;
  constexpr int UW = D <= 4 ? 8 : (D <= 8 ? 4 : 2), UP = D <= 8 ? 4 : 2;
  hipLaunchKernelGGL((fusedmm_small_kernel<P, D, kSmallG, UW, UP>), dim3((unsigned)blocks), dim3(kBlockThreads), 0, stream, a);
  return hipGetLastError();
}

template <int D>
hipError_t launch_small_d(int pattern, const KernelArgs& a, hipStream_t stream) {
  switch (pattern) {
    case PAT_SIGMOID: return launch_small_one<PAT_SIGMOID, D>(a, stream);
    case PAT_ONE_MINUS_SIGMOID: return launch_small_one<PAT_ONE_MINUS_SIGMOID, D>(a, stream);
    case PAT_GCN: return launch_small_one<PAT_GCN, D>(a, stream);
    case PAT_TDIST: return launch_small_one<PAT_TDIST, D>(a, stream);
    case PAT_FR: return launch_small_one<PAT_FR, D>(a, stream);
    case PAT_VISIT: return launch_small_one<PAT_VISIT, D>(a, stream);
    default: return launch_small_one<PAT_RUNTIME, D>(a, stream);  // every other tuple, read at run time
  }
}

}  // namespace

int small_packed_rows_per_block(int) { return kWavesPerBlock * (64 / kSmallG); }

hipError_t launch_small(int pattern, int d, const KernelArgs& a, hipStream_t stream) {
  switch (d) {
    case 2: return launch_small_d<2>(pattern, a, stream);
    case 3: return launch_small_d<3>(pattern, a, stream);
    case 4: return launch_small_d<4>(pattern, a, stream);
    case 8: return launch_small_d<8>(pattern, a, stream);
    case 16: return launch_small_d<16>(pattern, a, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_small_merge(const MergeDesc* merges, int32_t n_merges, const float* partials, int32_t d, int32_t aop,
                              const int64_t* rowptr, float* Z, int64_t ldz, hipStream_t stream) {
  if (n_merges <= 0) return hipSuccess;
  const int64_t blocks = ((int64_t)n_merges * d + 255) / 256;
  hipLaunchKernelGGL(fusedmm_small_merge_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, merges, n_merges, partials, d,
                     aop, rowptr, Z, ldz);
  return hipGetLastError();
}

}  // namespace fmm
