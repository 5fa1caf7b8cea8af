// fp32 MFMA GEMM for the two dense contractions of the search path:
//   query rotation  Q' = Q P            (Section 3.3.1)
//   coarse scores   s_q 1^T + 1 s_c^T - 2 Q' C^T   (Section 3.3.2)
// fp32 inputs are kept (v_mfma_f32_32x32x2_f32): the rotated query feeds an integer
// quantisation and the estimator, so reduced-precision inputs are not an option.
#include "rq_device.h"

namespace rq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;

// Block: 256 threads = 4 wavefronts in a 2 x 2 arrangement; a wavefront owns 32 TM rows x 32 TN columns of the block
// tile (64 TM x 64 TN) as TM x TN 32x32 MFMA accumulators, so with TM = TN = 2 every operand word read from LDS feeds
// two matrix instructions.  The LDS tiles are double buffered: the next k-step's operands travel from memory to
// registers while this step's products run and are stored to the other buffer afterwards, one barrier per k-step.
// Every output element is accumulated over k = 0, 2, 4, ... by v_mfma_f32_32x32x2_f32 in that order, whatever the tile
// shape (the small-batch kernel below relies on it).  The launcher picks the tile from the problem's shape.
template <int MODE, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                   float* __restrict__ C, int64_t M, int N, int K,
                                                   const float* __restrict__ rowv, const float* __restrict__ colv) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int AF = 4 * TM, BF = 4 * TN;  // floats of the A / B tile each thread moves per k-step
  __shared__ float As[2][BK][BM];  // k-major so that the 32 lanes of an MFMA operand read consecutive words
  __shared__ float Bs[2][BK][BN];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = floatx16{0};

  const int a_row = tid / (BK / AF), a_k = (tid % (BK / AF)) * AF;  // A tile: BM rows x 16 k
  const int b_k = tid / (BN / BF), b_n = (tid % (BN / BF)) * BF;    // B tile: 16 k x BN columns
  const bool a_ok = (m0 + a_row) < M;
  const float* a_ptr = A + (m0 + a_row) * (int64_t)K + a_k;
  const bool n_vec = ((N & 3) == 0) && (n0 + b_n + BF - 1 < N);

  // operands of one k step as this thread loads them
  float4 av[TM], bv[TN];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < TM; ++i) av[i] = a_ok ? *reinterpret_cast<const float4*>(a_ptr + k0 + 4 * i) : make_float4(0, 0, 0, 0);
    const float* b_ptr = B + (int64_t)(k0 + b_k) * N + n0 + b_n;
    if (n_vec) {
#pragma unroll
      for (int j = 0; j < TN; ++j) bv[j] = *reinterpret_cast<const float4*>(b_ptr + 4 * j);
    } else {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        float t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = (n0 + b_n + 4 * j + i < N) ? b_ptr[4 * j + i] : 0.f;
        bv[j] = make_float4(t[0], t[1], t[2], t[3]);
      }
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      As[buf][a_k + 4 * i + 0][a_row] = av[i].x; As[buf][a_k + 4 * i + 1][a_row] = av[i].y;
      As[buf][a_k + 4 * i + 2][a_row] = av[i].z; As[buf][a_k + 4 * i + 3][a_row] = av[i].w;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) *reinterpret_cast<float4*>(&Bs[buf][b_k][b_n + 4 * j]) = bv[j];
  };
  fetch(0);
  stash(0);
  __syncthreads();
  int buf = 0;
  for (int k0 = 0; k0 < K; k0 += BK, buf ^= 1) {
    const bool more = k0 + BK < K;
    if (more) fetch(k0 + BK);  // the next step's operands travel while this step's products run
#pragma unroll
    for (int k = 0; k < BK; k += 2) {
      const int kr = k + (lane >> 5);
      float a_[TM], b_[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a_[i] = As[buf][kr][wm * 32 * TM + 32 * i + (lane & 31)];
#pragma unroll
      for (int j = 0; j < TN; ++j) b_[j] = Bs[buf][kr][wn * 32 * TN + 32 * j + (lane & 31)];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_[i], b_[j], acc[i][j], 0, 0, 0);
    }
    if (more) stash(buf ^ 1);  // (the other buffer was last read before the previous barrier)
    __syncthreads();
  }
  // accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t m = m0 + wm * 32 * TM + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (m >= M) continue;
      float rv = 0.f;
      if (MODE == 1) rv = rowv[m];
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * 32 * TN + 32 * j + (lane & 31);
        if (n >= N) continue;
        float v = acc[i][j][r];
        if (MODE == 1) v = rv + colv[n] - 2.0f * v;
        if (MODE == 2) v = -v;
        if (MODE == 3) v = colv[n] - 2.0f * v;
        if (MODE == 4) v = v - colv[n];
        if (MODE == 1 || MODE == 2) __builtin_nontemporal_store(v, &C[m * (int64_t)N + n]);  // coarse scores: read once, by the selection
        else C[m * (int64_t)N + n] = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// Small batches (Section 4.2.2: latency at small batch sizes): rotation, per-query representation and coarse scores
// in ONE launch.  A workgroup takes 32 queries and 128 lists.  Every workgroup first rotates its 32 queries itself
// (each wavefront a 32 x 32 block of Q' at a time, operands straight from memory) and keeps Q' in LDS; the
// workgroups of the first list group also store Q', and the list groups share the queries' representation.  Then each wavefront
// contracts Q' with 32 centroids.  Both contractions issue v_mfma_f32_32x32x2_f32 over k = 0, 2, 4, ... exactly as
// gemm_kernel does and finish with the same expressions, so every number is the one the three separate kernels
// produce, bit for bit.
// ---------------------------------------------------------------------------------
template <int F>
__global__ __launch_bounds__(256) void small_front_kernel(const float* __restrict__ queries, int nq, int D, int nlist,
                                                          const float* __restrict__ P, const float* __restrict__ mean_rot,
                                                          const float* __restrict__ ct, const float* __restrict__ csq,
                                                          int metric, float* __restrict__ q_rot, rabitq_query_repr o,
                                                          float* __restrict__ scores) {
  extern __shared__ float qs[];  // [32][D + 1] rotated queries, then [32] squared norms
  const int ld = D + 1;
  float* s_sq = qs + 32 * ld;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m0 = 32 * blockIdx.y;
  const int half = lane >> 5, l32 = lane & 31;
  // rotation: block cb of Q' = rows m0.. x columns 32cb..
  for (int cb = wave; cb < D / 32; cb += 4) {
    floatx16 acc = {0};
    const bool row_ok = m0 + l32 < nq;
    const float* a_ptr = queries + (int64_t)(row_ok ? m0 + l32 : 0) * D + half;  // (an absent row reads row 0, unused)
    const float* b_ptr = P + (int64_t)half * D + 32 * cb + l32;
    // (a small batch waits for memory round trips, not for the matrix cores: the operands of the next 32 values of
    // k are requested before the current 32 are multiplied; D is a multiple of 32)
    constexpr int KU = 16;
    auto load = [&](float (&a_)[KU], float (&b_)[KU], int k0) {
#pragma unroll
      for (int u = 0; u < KU; ++u) {
        a_[u] = a_ptr[k0 + 2 * u];
        b_[u] = b_ptr[(int64_t)(k0 + 2 * u) * D];
      }
    };
    auto mma = [&](float (&a_)[KU], float (&b_)[KU]) {
#pragma unroll
      for (int u = 0; u < KU; ++u) {
        a_[u] = pinned(a_[u]);
        b_[u] = pinned(b_[u]);
      }
#pragma unroll
      for (int u = 0; u < KU; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(row_ok ? a_[u] : 0.f, b_[u], acc, 0, 0, 0);
    };
    float a0[KU], b0[KU], a1[KU], b1[KU];
    load(a0, b0, 0);
    for (int k0 = 0;;) {
      if (k0 + 32 < D) load(a1, b1, k0 + 32);
      mma(a0, b0);
      k0 += 32;
      if (k0 >= D) break;
      if (k0 + 32 < D) load(a0, b0, k0 + 32);
      mma(a1, b1);
      k0 += 32;
      if (k0 >= D) break;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + 4 * half + (r & 3), col = 32 * cb + l32;
      float v = acc[r];
      if (mean_rot != nullptr) v = v - mean_rot[col];
      qs[row * ld + col] = v;
      if (blockIdx.x == 0 && m0 + row < nq) q_rot[(int64_t)(m0 + row) * D + col] = v;
    }
  }
  __syncthreads();
  // squared norms of the queries that exist (every workgroup, for its scores); the representation of query r is
  // stored by the workgroup of list group r mod gridDim.x, so that the list groups share that work
  const int nrows = min(32, nq - m0);
  for (int row = wave; row < nrows; row += 4) {
    float amax, s1, s2;
    prep_reduce(qs + row * ld, D, lane, amax, s1, s2);
    if (lane == 0) s_sq[row] = s2;
  }
  for (int row = (int)blockIdx.x + (int)gridDim.x * wave; row < nrows; row += (int)gridDim.x * 4)
    query_prep_row<F>(qs + row * ld, m0 + row, D, o, lane);
  __syncthreads();
  // coarse scores: this wavefront's 32 lists
  {
    const int c0 = 128 * blockIdx.x + 32 * wave;
    if (c0 >= nlist) return;
    floatx16 acc = {0};
    const int col = c0 + l32;
    const bool col_ok = col < nlist;
    const float* b_ptr = ct + (int64_t)half * nlist + min(col, nlist - 1);
    const float* a_ptr = qs + l32 * ld + half;
    constexpr int KU = 16;
    auto load = [&](float (&b_)[KU], int k0) {
#pragma unroll
      for (int u = 0; u < KU; ++u) b_[u] = b_ptr[(int64_t)(k0 + 2 * u) * nlist];
    };
    auto mma = [&](float (&b_)[KU], int k0) {
#pragma unroll
      for (int u = 0; u < KU; ++u) b_[u] = pinned(b_[u]);
#pragma unroll
      for (int u = 0; u < KU; ++u)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a_ptr[k0 + 2 * u], col_ok ? b_[u] : 0.f, acc, 0, 0, 0);
    };
    float b0[KU], b1[KU];
    load(b0, 0);
    for (int k0 = 0;;) {
      if (k0 + 32 < D) load(b1, k0 + 32);
      mma(b0, k0);
      k0 += 32;
      if (k0 >= D) break;
      if (k0 + 32 < D) load(b0, k0 + 32);
      mma(b1, k0);
      k0 += 32;
      if (k0 >= D) break;
    }
    const float cv = col_ok ? csq[col] : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + 4 * half + (r & 3);
      if (m0 + row >= nq || !col_ok) continue;
      float v = acc[r];
      if (metric == RABITQ_L2) {
        const float rv = s_sq[row];
        v = rv + cv - 2.0f * v;
      } else {
        v = -v;
      }
      scores[(int64_t)(m0 + row) * nlist + col] = v;
    }
  }
}

int launch_small_front(const rabitq_index* ix, const float* queries, int64_t nq, float* q_rot, const rabitq_query_repr& o,
                       float* scores, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  const int D = ix->dim;
  const size_t smem = (size_t)(32 * (D + 1) + 32) * sizeof(float);
  dim3 grid((unsigned)((ix->nlist + 127) / 128), (unsigned)((nq + 31) / 32));
#define RQ_SF(F_)                                                                                                        \
  {                                                                                                                      \
    if (smem > 64 * 1024) RQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(small_front_kernel<F_>),             \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));            \
    hipLaunchKernelGGL(small_front_kernel<F_>, grid, dim3(256), smem, st, queries, (int)nq, D, ix->nlist, ix->rotation,  \
                       ix->mean_rot, ix->centroids_t, ix->centroid_sq, ix->metric, q_rot, o, scores);                    \
  }
  switch (ix->F) {
    case 0: RQ_SF(0) break;
    case 2: RQ_SF(2) break;
    case 4: RQ_SF(4) break;
    default: RQ_SF(8) break;
  }
#undef RQ_SF
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

template <int TM, int TN>
static int launch_gemm_tile(const float* A, const float* B, float* C, int64_t M, int N, int K, int mode, const float* rowv,
                            const float* colv, hipStream_t st) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  if ((M + BM - 1) / BM > 0x7fffffff || (N + BN - 1) / BN > 65535) {
    set_error("gemm: matrix too large");
    return RABITQ_EINVAL;
  }
  dim3 grid((unsigned)((M + BM - 1) / BM), (unsigned)((N + BN - 1) / BN));
  switch (mode) {
    case 0: hipLaunchKernelGGL((gemm_kernel<0, TM, TN>), grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 1: hipLaunchKernelGGL((gemm_kernel<1, TM, TN>), grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 2: hipLaunchKernelGGL((gemm_kernel<2, TM, TN>), grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 3: hipLaunchKernelGGL((gemm_kernel<3, TM, TN>), grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    case 4: hipLaunchKernelGGL((gemm_kernel<4, TM, TN>), grid, dim3(256), 0, st, A, B, C, M, N, K, rowv, colv); break;
    default: set_error("gemm: bad mode"); return RABITQ_EINVAL;
  }
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

int launch_gemm(const float* A, const float* B, float* C, int64_t M, int N, int K, int mode, const float* rowv,
                const float* colv, hipStream_t st) {
  if (M <= 0) return RABITQ_OK;
  if (K % BK != 0 || N <= 0) {
    set_error("gemm: K must be a multiple of 16 and N positive");
    return RABITQ_EINVAL;
  }
  // Tile by shape: the 128 x 128 tile reuses every LDS word twice and pays off when the contraction is long
  // (measured 0.72 of the fp32 matrix peak at K = 768 against 0.45 for 128 x 64); a short contraction is bound by
  // its prologue, epilogue and the write of C, where more and smaller workgroups do better; and a small problem
  // needs small tiles to give every compute unit a workgroup at all.
  auto tiles = [&](int bm, int bn) { return ((M + bm - 1) / bm) * (int64_t)((N + bn - 1) / bn); };
  if (K >= 256 && tiles(128, 128) >= 384) return launch_gemm_tile<2, 2>(A, B, C, M, N, K, mode, rowv, colv, st);
  // (64 x 128 rather than 128 x 64: a wavefront then stores 256 contiguous bytes of a row of C)
  if (tiles(64, 128) >= 512) return launch_gemm_tile<1, 2>(A, B, C, M, N, K, mode, rowv, colv, st);
  return launch_gemm_tile<1, 1>(A, B, C, M, N, K, mode, rowv, colv, st);
}

}  // namespace rq
