// fp32 MFMA GEMM for the two dense contractions of the search path:
//   query rotation  Q' = Q P            (Section 3.3.1)
//   coarse scores   s_q 1^T + 1 s_c^T - 2 Q' C^T   (Section 3.3.2)
// fp32 inputs are kept (v_mfma_f32_32x32x2_f32): the rotated query feeds an integer
// quantisation and the estimator, so reduced-precision inputs are not an option.
#include "rq_internal.h"

namespace rq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 64, BK = 16;

// Block: 256 threads = 4 wavefronts; wavefront w owns rows [32w, 32w+32) x 64 columns
// of the block tile as two 32x32 MFMA accumulators.
template <int MODE>
__global__ __launch_bounds__(256) void gemm_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                   float* __restrict__ C, int64_t M, int N, int K,
                                                   const float* __restrict__ rowv, const float* __restrict__ colv) {
  __shared__ float As[BK][BM];  // k-major so that the 32 lanes of an MFMA operand read consecutive words
  __shared__ float Bs[BK][BN];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;
  floatx16 acc0 = {0}, acc1 = {0};

  const int a_row = tid >> 1, a_half = tid & 1;        // A tile: 128 rows x 16 k, 8 floats per thread
  const int b_k = tid >> 4, b_n = (tid & 15) * 4;      // B tile: 16 k x 64 n, 4 floats per thread
  const bool a_ok = (m0 + a_row) < M;
  const float* a_ptr = A + (m0 + a_row) * (int64_t)K + a_half * 8;
  const bool n_vec = ((N & 3) == 0) && (n0 + b_n + 3 < N);

  // operands of one k step as this thread loads them
  float4 a0, a1, b;
  auto fetch = [&](int k0) {
    a0 = make_float4(0, 0, 0, 0);
    a1 = a0;
    if (a_ok) {
      a0 = *reinterpret_cast<const float4*>(a_ptr + k0);
      a1 = *reinterpret_cast<const float4*>(a_ptr + k0 + 4);
    }
    b = make_float4(0, 0, 0, 0);
    const float* b_ptr = B + (int64_t)(k0 + b_k) * N + n0 + b_n;
    if (n_vec) {
      b = *reinterpret_cast<const float4*>(b_ptr);
    } else {
      if (n0 + b_n + 0 < N) b.x = b_ptr[0];
      if (n0 + b_n + 1 < N) b.y = b_ptr[1];
      if (n0 + b_n + 2 < N) b.z = b_ptr[2];
      if (n0 + b_n + 3 < N) b.w = b_ptr[3];
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += BK) {
    __syncthreads();  // previous tile fully consumed
    const int kk = a_half * 8;
    As[kk + 0][a_row] = a0.x; As[kk + 1][a_row] = a0.y; As[kk + 2][a_row] = a0.z; As[kk + 3][a_row] = a0.w;
    As[kk + 4][a_row] = a1.x; As[kk + 5][a_row] = a1.y; As[kk + 6][a_row] = a1.z; As[kk + 7][a_row] = a1.w;
    *reinterpret_cast<float4*>(&Bs[b_k][b_n]) = b;
    __syncthreads();
    if (k0 + BK < K) fetch(k0 + BK);  // the next step's operands travel while this step's products run
#pragma unroll
    for (int k = 0; k < BK; k += 2) {
      const int kr = k + (lane >> 5);
      const float a = As[kr][wave * 32 + (lane & 31)];
      const float b0 = Bs[kr][lane & 31];
      const float b1 = Bs[kr][32 + (lane & 31)];
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc1, 0, 0, 0);
    }
  }
  // accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int64_t m = m0 + wave * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (m >= M) continue;
    float rv = 0.f;
    if (MODE == 1) rv = rowv[m];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + 32 * j + (lane & 31);
      if (n >= N) continue;
      float v = j == 0 ? acc0[r] : acc1[r];
      if (MODE == 1) v = rv + colv[n] - 2.0f * v;
      if (MODE == 2) v = -v;
      if (MODE == 3) v = colv[n] - 2.0f * v;
      if (MODE == 4) v = v - colv[n];
      C[m * (int64_t)N + n] = v;
    }
  }
}

int launch_gemm(const float* A, const float* B, float* C, int64_t M, int N, int K, int mode, const float* rowv,
                const float* colv, hipStream_t st) {
  if (M <= 0) return RABITQ_OK;
  if (K % BK != 0 || N <= 0) {
    set_error("gemm: K must be a multiple of 16 and N positive");
    return RABITQ_EINVAL;
  }
  if ((M + BM - 1) / BM > 0x7fffffff || (N + BN - 1) / BN > 65535) {
    set_error("gemm: matrix too large");
    return RABITQ_EINVAL;
  }
  dim3 grid((unsigned)((M + BM - 1) / BM), (unsigned)((N + BN - 1) / BN));
  switch (mode) {
    case 0: hipLaunchKernelGGL(gemm_kernel<0>, grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 1: hipLaunchKernelGGL(gemm_kernel<1>, grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 2: hipLaunchKernelGGL(gemm_kernel<2>, grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 3: hipLaunchKernelGGL(gemm_kernel<3>, grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 4: hipLaunchKernelGGL(gemm_kernel<4>, grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    default: set_error("gemm: bad mode"); return RABITQ_EINVAL;
  }
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

}  // namespace rq
