// Measurement aid, not part of libfusedmm.so: how many bytes per clock a CU is handed by the caches for the
// access pattern of the gathers (Algorithm 1: y_v <- Y[v, :] for every stored entry), with no arithmetic and
// no index traffic around it.  Every wavefront issues 16-byte loads, four in flight, over a buffer of a
// power-of-two size:
//   stream    64 consecutive lanes read 1 KB of consecutive bytes, load after load through consecutive KBs
//   rows R    groups of R/16 lanes read R-byte rows (R = 128 ... 1024) at pseudo-random row numbers
// A buffer of 1-2 MiB stays in every XCD's L2 (and is far larger than a 32 KB L1): the L2 -> L1 rate.  A
// buffer of 64 MiB exceeds the L2s and stays in the 256 MB Infinity Cache: the fabric rate.  1 GiB: HBM.
//
//   python -m paper_2011_06391_amd.build microbench && ./paper_2011_06391_amd/bench_l2_delivery
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef float v4f __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                   \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      return 1;                                                                    \
    }                                                                              \
  } while (0)

// n16: buffer length in 16-byte pieces, a power of two.  lanes_per_row: 64 = stream, else 8 ... 64 lanes per row.
// sequential != 0: the wavefront walks through consecutive rows from a start of its own instead.
__global__ __launch_bounds__(256) void delivery_kernel(const v4f* buf, unsigned n16, int lanes_per_row, int sequential,
                                                       int steps, float* sink) {
  const unsigned lane = threadIdx.x & 63;
  const unsigned wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const unsigned in_row = lane % lanes_per_row, row_of_lane = lane / lanes_per_row;
  const unsigned rows_per_load = 64 / lanes_per_row;
  const unsigned n_rows = n16 / lanes_per_row;  // power of two
  unsigned state = wave * 2654435761u + 12345u;
  v4f acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < steps; ++s) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      state = sequential ? state + 1u : state * 1664525u + 1013904223u;  // wave-uniform
      const unsigned row = ((sequential ? state : state >> 7) * rows_per_load + row_of_lane) & (n_rows - 1);
      acc += buf[row * lanes_per_row + in_row];
    }
  }
  if (acc.x == 123.456f) sink[0] = acc.y + acc.z + acc.w;  // never true for a zeroed buffer: keeps the loads
}

int main() {
  const double clock_hz = 2.4e9;
  const int n_cu = 256, blocks = n_cu * 8, steps = 2000;
  float* sink = nullptr;
  CHECK(hipMalloc(&sink, sizeof(float)));
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  const size_t sizes_mib[] = {1, 2, 64, 1024};
  const int row_bytes[] = {1024, 128, 256, 512, 1024};  // first entry: the stream (64 lanes, consecutive)
  for (size_t mib : sizes_mib) {
    v4f* buf = nullptr;
    const size_t bytes = mib << 20;
    CHECK(hipMalloc(&buf, bytes));
    CHECK(hipMemset(buf, 0, bytes));
    for (int k = 0; k < 5; ++k) {
      const int lanes = row_bytes[k] / 16;
      float best = 1e30f;
      for (int rep = 0; rep < 4; ++rep) {
        CHECK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(delivery_kernel, dim3(blocks), dim3(256), 0, 0, buf, (unsigned)(bytes / 16), lanes, k == 0 ? 1 : 0, steps,
                           sink);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(e1, 0));
        CHECK(hipEventSynchronize(e1));
        float ms = 0.f;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        if (rep > 0 && ms < best) best = ms;
      }
      const double total = (double)blocks * 4 * steps * 4 * 1024.0;  // bytes loaded per launch
      std::printf("buffer %5zu MiB  %-22s %8.3f ms  %6.2f TB/s  %5.1f B/clk/CU\n", mib,
                  k == 0 ? "stream (1 KB per load)" : (row_bytes[k] == 128 ? "rows of 128 B, random" : row_bytes[k] == 256 ? "rows of 256 B, random" : row_bytes[k] == 512 ? "rows of 512 B, random" : "rows of 1 KB, random"),
                  best, total / best / 1e9, total / (best * 1e-3) / n_cu / clock_hz);
      std::fflush(stdout);
    }
    CHECK(hipFree(buf));
  }
  return 0;
}
