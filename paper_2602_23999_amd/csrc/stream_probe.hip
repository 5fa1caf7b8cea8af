// Stand-alone driver of the code scan in the streaming regime, for counter runs under rocprofv3 (no Python in the
// process).  It builds an index of N vectors (D = 128, N / 1024 lists, 1-bit codes unless told otherwise) with the
// library, takes the first vector of every list as a query, so that every query probes a list of its own
// (nprobe = 1) and the scan reads every list from memory once, and runs rabitq_search a few times.  Before and
// after, a plain kernel that reads 256 MiB and writes 256 MiB runs once: what the counters show for it is the scale
// for what they show for the scan.  Data: N / 1024 centres N(0, 16 I); a point is its centre plus a scatter inside one
// of 64 eight-dimensional subspaces (std 3) plus isotropic noise (std 0.3), from a counter-based generator.
//
//   stream_probe [N = 33554432] [bits = 1] [searches = 5] [longest_first = 1] [scan_segment_tiles = 0] [kmeans_iters = 4]
//
// Prints the kernel-relevant sizes (lists probed, vectors scanned, algorithmic bytes at 24 or 28 bytes per vector) and
// the mean time of a whole search; the scan kernel's own time is in the profiler's trace.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "rabitq.h"

#define CK(x)                                                                    \
  do {                                                                           \
    hipError_t e_ = (x);                                                         \
    if (e_ != hipSuccess) {                                                      \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 1;                                                                  \
    }                                                                            \
  } while (0)
#define RQ(x)                                                                        \
  do {                                                                               \
    int rc_ = (x);                                                                   \
    if (rc_ != 0) {                                                                  \
      std::printf("rabitq error %d (%s) at line %d\n", rc_, rabitq_last_error(), __LINE__); \
      return 1;                                                                      \
    }                                                                                \
  } while (0)

namespace {

constexpr int D = 128, SUB = 64, SUBDIM = 8;

__host__ __device__ inline uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// standard normal from two counters (Box-Muller)
__host__ __device__ inline float gauss(uint32_t a, uint32_t b) {
  const float u1 = ((float)(mix(a * 2654435761u + b) >> 8) + 1.0f) * (1.0f / 16777217.0f);
  const float u2 = (float)(mix(b * 2246822519u + a + 0x9e3779b9u) >> 8) * (1.0f / 16777216.0f);
  return sqrtf(-2.0f * logf(u1)) * cosf(6.2831853f * u2);
}

// one wavefront per vector (four to a workgroup): lane d and d + 64 are its dimensions
__global__ __launch_bounds__(256) void make_points(float* __restrict__ x, int64_t n, int nlist, const float* __restrict__ basis) {
  for (int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); i < n; i += (int64_t)gridDim.x * 4) {
    const uint32_t own = mix((uint32_t)i * 747796405u + 12345u) % (uint32_t)nlist;
    float z[SUBDIM];
    for (int t = 0; t < SUBDIM; ++t) z[t] = 3.0f * gauss((uint32_t)i, 1000u + t);
    const float* b = basis + (size_t)(own % SUB) * D * SUBDIM;
    for (int d = threadIdx.x & 63; d < D; d += 64) {
      float v = 4.0f * gauss(own, 77u + d) + 0.3f * gauss((uint32_t)i, 5000u + d);
      for (int t = 0; t < SUBDIM; ++t) v += z[t] * b[d * SUBDIM + t];
      x[i * D + d] = v;
    }
  }
}

__global__ __launch_bounds__(64) void gather_rows(const float* __restrict__ x, const int32_t* __restrict__ rows, int nq,
                                                  float* __restrict__ q) {
  const int i = blockIdx.x;
  if (i >= nq) return;
  for (int d = threadIdx.x; d < D; d += 64) q[(int64_t)i * D + d] = x[(int64_t)rows[i] * D + d];
}

// the scale of the counters: reads n floats, writes n floats
__global__ __launch_bounds__(256) void calibration_add(const float* __restrict__ in, float* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) out[i] = in[i] + 1.0f;
}

}  // namespace

int main(int argc, char** argv) {
  const int64_t n = argc > 1 ? std::atoll(argv[1]) : 33554432;
  const int bits = argc > 2 ? std::atoi(argv[2]) : 1;
  const int searches = argc > 3 ? std::atoi(argv[3]) : 5;
  const int longest_first = argc > 4 ? std::atoi(argv[4]) : 1, seg_tiles = argc > 5 ? std::atoi(argv[5]) : 0;
  const int kmeans_iters = argc > 6 ? std::atoi(argv[6]) : 4;  // (fewer iterations: fewer launches for a counter run to sit through)
  const int nlist = (int)(n / 1024), k = 10;
  if (n < 65536 || n > ((int64_t)1 << 28) || bits < 1 || bits > 8 || searches < 1 || searches > 100 || seg_tiles < 0 ||
      seg_tiles > 4096 || kmeans_iters < 0 || kmeans_iters > 50) {
    std::printf("usage: stream_probe [N in 65536 .. 2^28] [bits 1 .. 8] [searches 1 .. 100] [longest_first 0|1] [segment tiles] [k-means iterations 0 .. 50]\n");
    return 1;
  }
  // rotation: Gram-Schmidt on a Gaussian matrix; subspace bases the same way
  auto orthonormal = [](std::vector<float>& m, int rows, int cols, uint32_t seed) {  // rows x cols, columns orthonormal
    for (int j = 0; j < cols; ++j) {
      for (int i = 0; i < rows; ++i) m[(size_t)i * cols + j] = gauss(seed + (uint32_t)i, 31u * (uint32_t)j + 7u);
      for (int p = 0; p < j; ++p) {
        double dot = 0;
        for (int i = 0; i < rows; ++i) dot += (double)m[(size_t)i * cols + j] * m[(size_t)i * cols + p];
        for (int i = 0; i < rows; ++i) m[(size_t)i * cols + j] -= (float)dot * m[(size_t)i * cols + p];
      }
      double nn = 0;
      for (int i = 0; i < rows; ++i) nn += (double)m[(size_t)i * cols + j] * m[(size_t)i * cols + j];
      const float inv = (float)(1.0 / std::sqrt(nn));
      for (int i = 0; i < rows; ++i) m[(size_t)i * cols + j] *= inv;
    }
  };
  std::vector<float> P((size_t)D * D), basis((size_t)SUB * D * SUBDIM);
  orthonormal(P, D, D, 99u);
  for (int s = 0; s < SUB; ++s) {
    std::vector<float> b((size_t)D * SUBDIM);
    orthonormal(b, D, SUBDIM, 1000u * (uint32_t)(s + 1));
    for (size_t i = 0; i < b.size(); ++i) basis[(size_t)s * D * SUBDIM + i] = b[i];
  }
  float *d_basis = nullptr, *x = nullptr, *cal_in = nullptr, *cal_out = nullptr;
  CK(hipMalloc(&d_basis, basis.size() * sizeof(float)));
  CK(hipMemcpy(d_basis, basis.data(), basis.size() * sizeof(float), hipMemcpyHostToDevice));
  CK(hipMalloc(&x, (size_t)n * D * sizeof(float)));
  hipLaunchKernelGGL(make_points, dim3((unsigned)std::min<int64_t>((n + 3) / 4, 1 << 20)), dim3(256), 0, 0, x, n, nlist, d_basis);
  CK(hipGetLastError());
  const size_t cal_n = (size_t)64 << 20;  // 256 MiB each way
  CK(hipMalloc(&cal_in, cal_n * sizeof(float)));
  CK(hipMalloc(&cal_out, cal_n * sizeof(float)));
  CK(hipMemset(cal_in, 0, cal_n * sizeof(float)));
  CK(hipDeviceSynchronize());

  rabitq_build_params prm{};
  prm.dim = D; prm.nlist = nlist; prm.n = n; prm.total_bits = bits; prm.metric = RABITQ_L2; prm.kmeans_iters = kmeans_iters;
  prm.train_size = n / 10; prm.epsilon0 = 1.9f; prm.rotation = P.data(); prm.center = 0;
  rabitq_index_t ix = nullptr;
  RQ(rabitq_index_build(&prm, x, &ix, nullptr));
  CK(hipDeviceSynchronize());
  const int64_t n_slots = rabitq_index_info(ix, "n_slots");
  std::vector<int64_t> offsets((size_t)nlist + 1);
  std::vector<int32_t> ids((size_t)n_slots);
  RQ(rabitq_index_export(ix, nullptr, nullptr, offsets.data(), nullptr, nullptr, nullptr, nullptr, ids.data(), nullptr));
  // the first vector of every non-empty list is that list's query
  std::vector<int32_t> rows;
  int64_t slot = 0, scanned = 0;
  for (int c = 0; c < nlist; ++c) {
    const int64_t nc = offsets[c + 1] - offsets[c];
    if (nc > 0) {
      rows.push_back(ids[(size_t)slot]);
      scanned += nc;
    }
    slot += (nc + 63) / 64 * 64;
  }
  const int nq = (int)rows.size();
  int32_t* d_rows = nullptr;
  float *q = nullptr, *out_d = nullptr;
  int64_t* out_ids = nullptr;
  CK(hipMalloc(&d_rows, (size_t)nq * sizeof(int32_t)));
  CK(hipMemcpy(d_rows, rows.data(), (size_t)nq * sizeof(int32_t), hipMemcpyHostToDevice));
  CK(hipMalloc(&q, (size_t)nq * D * sizeof(float)));
  hipLaunchKernelGGL(gather_rows, dim3((unsigned)nq), dim3(64), 0, 0, x, d_rows, nq, q);
  CK(hipGetLastError());
  CK(hipDeviceSynchronize());
  CK(hipFree(x));
  CK(hipMalloc(&out_ids, (size_t)nq * k * sizeof(int64_t)));
  CK(hipMalloc(&out_d, (size_t)nq * k * sizeof(float)));
  RQ(rabitq_set_option(ix, "scan_impl", 0));
  RQ(rabitq_set_option(ix, "longest_first", longest_first != 0));
  RQ(rabitq_set_option(ix, "scan_segment_tiles", seg_tiles));

  hipLaunchKernelGGL(calibration_add, dim3(8192), dim3(256), 0, 0, cal_in, cal_out, cal_n);
  RQ(rabitq_search(ix, q, nq, k, 1, out_ids, out_d, nullptr));  // (grows the workspace)
  CK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  CK(hipEventRecord(e0, nullptr));
  for (int i = 0; i < searches; ++i) RQ(rabitq_search(ix, q, nq, k, 1, out_ids, out_d, nullptr));
  CK(hipEventRecord(e1, nullptr));
  CK(hipEventSynchronize(e1));
  float ms = 0;
  CK(hipEventElapsedTime(&ms, e0, e1));
  hipLaunchKernelGGL(calibration_add, dim3(8192), dim3(256), 0, 0, cal_in, cal_out, cal_n);
  CK(hipDeviceSynchronize());
  // how many queries found themselves (their own id first): a check that the search did what it is timed for
  std::vector<int64_t> h_ids((size_t)nq * k);
  CK(hipMemcpy(h_ids.data(), out_ids, h_ids.size() * sizeof(int64_t), hipMemcpyDeviceToHost));
  int64_t self = 0;
  for (int i = 0; i < nq; ++i) self += h_ids[(size_t)i * k] == rows[i];
  const int per_vec = D / 8 + (bits == 1 ? 8 : 12);
  std::printf("stream_probe: N=%lld lists=%d bits=%d queries=%d (one per non-empty list) vectors_scanned=%lld "
              "algorithmic_bytes=%lld (%d per vector) stream=%lld search_ms=%.4f self_first=%lld\n",
              (long long)n, nlist, bits, nq, (long long)scanned, (long long)(scanned * per_vec), per_vec,
              (long long)rabitq_index_info(ix, "last_scan_stream"), ms / searches, (long long)self);
  RQ(rabitq_index_free(ix));
  return 0;
}
