// Device-side index construction (Section 3.2): k-means in the rotated space, assignment,
// normalisation with respect to the centroid, RaBitQ quantisation by the two-phase grid
// search over the rescaling factor, factors, and the tiled index layout.
#include <vector>

#include "rq_device.h"

namespace rq {

__device__ inline float wave_sum_f32(float v) {
  const uint32_t r = wave_reduce_u32(__builtin_bit_cast(uint32_t, v), [](uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b));
  });
  return __builtin_bit_cast(float, r);
}
__device__ inline float wave_max_f32(float v) {
  const uint32_t r = wave_reduce_u32(__builtin_bit_cast(uint32_t, v), [](uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b)));
  });
  return __builtin_bit_cast(float, r);
}

// rows[i] = src[(i * stride_num) / stride_den]  (strided training subset / initial centroids)
__global__ void gather_rows_kernel(const float* __restrict__ src, int64_t n_src, int64_t n_dst, int D,
                                   float* __restrict__ dst) {
  const int64_t total = n_dst * D;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / D;
    const int64_t s = (r * n_src) / n_dst;
    dst[i] = src[s * D + (i - r * D)];
  }
}

// ct[d][c] = c_rows[c][d], csq[c] = ||c||^2
__global__ void transpose_centroids_kernel(const float* __restrict__ c_rows, int nlist, int D, float* __restrict__ ct,
                                           float* __restrict__ csq) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= nlist) return;
  float s = 0.f;
  for (int d = 0; d < D; ++d) {
    const float v = c_rows[(int64_t)c * D + d];
    ct[(int64_t)d * nlist + c] = v;
    s += v * v;
  }
  csq[c] = s;
}

// nearest centroid of each row of a score chunk (scores = ||c||^2 - 2<x,c>), ties to the lower id
__global__ __launch_bounds__(256) void argmin_rows_kernel(const float* __restrict__ scores, int64_t rows, int nlist,
                                                         int32_t* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const float* row = scores + r * nlist;
  uint64_t best = KEY_NONE;
  // eight requests in flight (clamped indices, so that no load sits under a condition)
  for (int c0 = lane; c0 < nlist; c0 += 8 * 64) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = row[min(c0 + u * 64, nlist - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = pinned(v[u]);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c = c0 + u * 64;
      const uint64_t key = c < nlist ? make_key(v[u], (uint32_t)c) : KEY_NONE;
      best = key < best ? key : best;
    }
  }
  best = wave_reduce_u64(best, [](uint64_t a, uint64_t b) { return a < b ? a : b; });
  if (lane == 0) out[r] = (int32_t)(uint32_t)best;
}

// Lloyd update: one workgroup per cluster sums its members in list order (deterministic);
// an empty cluster keeps its centroid.
__global__ __launch_bounds__(256) void centroid_update_kernel(const float* __restrict__ x, const int32_t* __restrict__ off,
                                                             const int32_t* __restrict__ members, int D,
                                                             float* __restrict__ c_rows) {
  const int c = blockIdx.x;
  const int s = off[c], e = off[c + 1];
  if (e == s) return;
  const float inv = 1.0f / (float)(e - s);
  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    float acc = 0.f;
    for (int i = s; i < e; ++i) acc += x[(int64_t)members[i] * D + d];
    c_rows[(int64_t)c * D + d] = acc * inv;
  }
}

__global__ void cluster_layout_kernel(const int32_t* __restrict__ off, int nlist, int32_t* __restrict__ csize) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < nlist) csize[c] = off[c + 1] - off[c];
}

__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

// f_add planes of the short factors start at +inf (padding), everything else at 0
__global__ void init_short_factors_kernel(float* p, int64_t n_tiles) {
  const int64_t total = n_tiles * 3 * TILE;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = ((i / TILE) % 3 == 0) ? INFINITY : 0.f;
}

struct EncodeArgs {
  const float* xr;          // [N][D] rotated vectors
  const float* c_rows;      // [nlist][D] rotated centroids
  const int32_t* off;       // [nlist+1] CSR over stored vectors
  const int32_t* members;   // [N] vector ids in cluster order
  const int32_t* tile_off;  // [nlist+1]
  int64_t n;
  int64_t p0;               // first position of this launch
  int D, B, F, LW, nlist, metric;
  float eps0;
  uint32_t* short_codes;
  float* short_factors;
  uint32_t* long_codes;
  float* long_factors;
  int32_t* ids;
};

// ---------------------------------------------------------------------------------
// One wavefront per stored vector (Section 3.2.2 maps a thread block to a vector; a
// 64-wide wavefront is that block here).  Phase 1: lanes = dimensions (residual, norm,
// |o'|).  Phase 2: lanes = sampled rescaling factors — every lane walks all dimensions for
// its own t, so the N_coarse = 64 samples need no cross-lane reduction until the arg-max;
// then N_fine = 32 samples around the best one (plus the coarse winner itself).  Phase 3:
// lanes = dimensions again (codes, factor sums, packing).
// ---------------------------------------------------------------------------------
template <int DPL>  // dimensions per lane = ceil(D / 64)
__global__ __launch_bounds__(256) void encode_kernel(EncodeArgs a) {
  extern __shared__ unsigned char smem_raw[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* ybuf = reinterpret_cast<float*>(smem_raw) + (size_t)wave * a.D;                          // [D] |o'|
  unsigned char* ubuf = smem_raw + 4 * (size_t)a.D * sizeof(float) + (size_t)wave * a.D;         // [D] codes
  const int64_t p = a.p0 + (int64_t)blockIdx.x * 4 + wave;  // position in cluster order
  if (p >= a.n) return;
  // cluster of this position: largest c with off[c] <= p
  int lo = 0, hi = a.nlist;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (a.off[mid] <= p) lo = mid; else hi = mid;
  }
  const int c = lo;
  const int32_t vid = a.members[p];
  const int64_t slot = (int64_t)a.tile_off[c] * TILE + (p - a.off[c]);
  const int D = a.D, B = a.B;
  const int half = 1 << (B - 1), L = half - 1;

  float res[DPL], cr[DPL];
  float r2 = 0.f, cdotres = 0.f;
#pragma unroll
  for (int k = 0; k < DPL; ++k) {
    const int d = k * 64 + lane;
    res[k] = 0.f;
    cr[k] = 0.f;
    if (d < D) {
      cr[k] = a.c_rows[(int64_t)c * D + d];
      res[k] = a.xr[(int64_t)vid * D + d] - cr[k];
    }
    r2 += res[k] * res[k];
    cdotres += cr[k] * res[k];
  }
  r2 = wave_sum_f32(r2);
  cdotres = wave_sum_f32(cdotres);
  const float r = sqrtf(r2);
  const bool ok = r > 0.f;
  const float inv_r = ok ? 1.0f / r : 0.f;
  float o[DPL], ymax = 0.f;
#pragma unroll
  for (int k = 0; k < DPL; ++k) {
    o[k] = res[k] * inv_r;
    const int d = k * 64 + lane;
    if (d < D) ybuf[d] = fabsf(o[k]);
    ymax = fmaxf(ymax, fabsf(o[k]));
  }
  ymax = wave_max_f32(ymax);
  float t_best = 0.f;
  if (L > 0 && ok) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // search range: the best factor lies below range_mult * 2^(B-1) / max|o'| (the fewer
    // levels, the further the bulk of the coordinates may be pushed past the largest one)
    const float range_mult = (B >= 5) ? 1.5f : (B == 4 ? 2.5f : (B == 3 ? 4.5f : 6.0f));
    const float t_end = range_mult * (float)half / ymax;
    const float Lf = (float)L;
    auto objective = [&](float t) -> float {
      float num = 0.f, den = 0.f;
      for (int d = 0; d < D; d += 4) {
        const float4 y = *reinterpret_cast<const float4*>(ybuf + d);
        const float m0 = fminf(floorf(t * y.x), Lf) + 0.5f, m1 = fminf(floorf(t * y.y), Lf) + 0.5f;
        const float m2 = fminf(floorf(t * y.z), Lf) + 0.5f, m3 = fminf(floorf(t * y.w), Lf) + 0.5f;
        num += m0 * y.x + m1 * y.y + m2 * y.z + m3 * y.w;
        den += m0 * m0 + m1 * m1 + m2 * m2 + m3 * m3;
      }
      return num * rsqrtf(den);
    };
    // coarse: t_k = (k+1)/64 * t_end, one sample per lane; ties go to the smaller t
    const float tc = (float)(lane + 1) * (1.0f / 64.0f) * t_end;
    uint64_t key = ((uint64_t)f2ord(objective(tc)) << 32) | (uint32_t)(63 - lane);
    key = wave_reduce_u64(key, [](uint64_t x, uint64_t y) { return x > y ? x : y; });
    const int kc = 63 - (int)(uint32_t)key;
    const float t_c = (float)(kc + 1) * (1.0f / 64.0f) * t_end;
    // fine: 32 samples uniform over t_c -+ t_end/64 (lanes 0..31), lane 32 re-evaluates t_c
    const float width = t_end * (1.0f / 64.0f);
    float tf = t_c;
    if (lane < 32) tf = fmaxf(t_c + width * (-1.0f + 2.0f * (float)lane * (1.0f / 31.0f)), 0.f);
    uint64_t key2 = 0ull;
    if (lane <= 32) key2 = ((uint64_t)f2ord(objective(tf)) << 32) | (uint32_t)(63 - lane);
    key2 = wave_reduce_u64(key2, [](uint64_t x, uint64_t y) { return x > y ? x : y; });
    const int kf = 63 - (int)(uint32_t)key2;
    t_best = __shfl(tf, kf, 64);
  }
  // codes and factor sums (lanes = dimensions)
  const float cB = (float)((1 << B) - 1) * 0.5f;
  float xo = 0.f, xc = 0.f, xx = 0.f, bo = 0.f, bc = 0.f;
  uint32_t u[DPL];
#pragma unroll
  for (int k = 0; k < DPL; ++k) {
    const int d = k * 64 + lane;
    const float y = fabsf(o[k]);
    const int m = (L > 0 && ok) ? (int)fminf(floorf(t_best * y), (float)L) : 0;
    const bool pos = o[k] >= 0.f;
    u[k] = ok ? (uint32_t)(pos ? half + m : half - 1 - m) : (uint32_t)half;
    if (d < D) {
      ubuf[d] = (unsigned char)u[k];
      const float x = (float)u[k] - cB;
      const float xb = (float)(u[k] >> (B - 1)) - 0.5f;
      xo += x * o[k]; xc += x * cr[k]; xx += x * x;
      bo += xb * o[k]; bc += xb * cr[k];
    }
  }
  xo = wave_sum_f32(xo); xc = wave_sum_f32(xc); xx = wave_sum_f32(xx);
  bo = wave_sum_f32(bo); bc = wave_sum_f32(bc);
  // short code: sign bits, 64 dimensions per ballot
  const int W = D >> 5;
  const int64_t tile = slot >> 6;
  const int ln = (int)(slot & 63);
#pragma unroll
  for (int k = 0; k < DPL; ++k) {
    const int d = k * 64 + lane;
    const uint64_t m = __ballot(d < D && ((u[k] >> (B - 1)) & 1u));
    if (lane == 0) {
      const int w = 2 * k;
      if (w < W) a.short_codes[(tile * W + w) * TILE + ln] = (uint32_t)m;
      if (w + 1 < W) a.short_codes[(tile * W + w + 1) * TILE + ln] = (uint32_t)(m >> 32);
    }
  }
  if (lane == 0) {
    const float Df = (float)D;
    float f1[3] = {0.f, 0.f, 0.f}, fB[2] = {0.f, 0.f};
    if (ok) {
      const float scale = (a.metric == RABITQ_L2) ? 2.0f : 1.0f;
      const float lead = (a.metric == RABITQ_L2) ? r2 : -cdotres;
      const float a1 = fminf(fmaxf(bo / (0.5f * sqrtf(Df)), 0.f), 1.f);
      f1[0] = lead + scale * r * bc / bo;
      f1[1] = -scale * r / bo;
      f1[2] = scale * r * a.eps0 * sqrtf(fmaxf(1.f - a1 * a1, 0.f)) / (a1 * sqrtf(Df - 1.f));
      fB[0] = lead + scale * r * xc / xo;
      fB[1] = -scale * r / xo;
    }
    a.short_factors[(tile * 3 + 0) * TILE + ln] = f1[0];
    a.short_factors[(tile * 3 + 1) * TILE + ln] = f1[1];
    a.short_factors[(tile * 3 + 2) * TILE + ln] = f1[2];
    if (B > 1) {
      a.long_factors[2 * slot] = fB[0];
      a.long_factors[2 * slot + 1] = fB[1];
    }
    a.ids[slot] = vid;
  }
  if (B > 1) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int per = 32 / a.F;
    for (int w = lane; w < a.LW; w += 64) {
      uint32_t word = 0;
      for (int j = 0; j < per; ++j) word |= (uint32_t)ubuf[w * per + j] << (a.F * j);
      a.long_codes[slot * a.LW + w] = word;
    }
  }
}

template <typename T>
struct DevBuf {
  T* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  int alloc(int64_t count) {
    if (count <= 0) count = 1;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&p), (size_t)count * sizeof(T));
    if (e != hipSuccess) {
      (void)hipGetLastError();
      p = nullptr;
      set_error("index build: hipMalloc failed: " + std::string(hipGetErrorString(e)));
      return RABITQ_ENOMEM;
    }
    return RABITQ_OK;
  }
  T* release() { T* r = p; p = nullptr; return r; }
};

// Column means of a row-major [n][D] matrix in two fixed-order passes (deterministic): every
// workgroup sums its own block of rows per column in fp64, then one workgroup adds the
// partial sums in block order.
constexpr int MEAN_BLOCKS = 1024;
__global__ __launch_bounds__(256) void column_partial_kernel(const float* __restrict__ x, int64_t n, int D,
                                                            double* __restrict__ partial) {
  const int64_t rows_per = (n + MEAN_BLOCKS - 1) / MEAN_BLOCKS;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per, r1 = r0 + rows_per < n ? r0 + rows_per : n;
  for (int d = threadIdx.x; d < D; d += 256) {
    double acc = 0.0;
    for (int64_t r = r0; r < r1; ++r) acc += (double)x[r * D + d];
    partial[(int64_t)blockIdx.x * D + d] = acc;
  }
}
__global__ __launch_bounds__(256) void column_mean_kernel(const double* __restrict__ partial, int64_t n, int D,
                                                         float* __restrict__ mean) {
  for (int d = threadIdx.x; d < D; d += 256) {
    double acc = 0.0;
    for (int b = 0; b < MEAN_BLOCKS; ++b) acc += partial[(int64_t)b * D + d];
    mean[d] = (float)(acc / (double)n);
  }
}

static unsigned grid_for(int64_t n, int block = 256, int64_t cap = 65535) {
  return (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + block - 1) / block, cap));
}

// ---- rows grouped by cluster -------------------------------------------------------------------
// A stable counting sort of row ids by cluster id whose memory grows with rows + blocks * nlist (the
// search path's builder keeps one bit per (cluster, query), which is right for 10^4 queries and far
// too much for 10^7 vectors).  The rows are cut into `nb` contiguous blocks; a workgroup counts its
// block per cluster, the counts are scanned block-major per cluster, and the same workgroup then places
// its rows tile by tile in row order, so every list holds its rows in ascending order whatever the
// scheduling.
constexpr int GROUP_TILE = 256;
struct GroupPlan {
  int nb;       // workgroups = row blocks
  int64_t ch;   // rows per block, a multiple of GROUP_TILE
};
static GroupPlan group_plan(int64_t rows) {
  GroupPlan g;
  const int64_t want = std::max<int64_t>(1, std::min<int64_t>((rows + 4095) / 4096, 1024));
  g.ch = ((rows + want - 1) / want + GROUP_TILE - 1) / GROUP_TILE * GROUP_TILE;
  if (g.ch < GROUP_TILE) g.ch = GROUP_TILE;
  g.nb = (int)std::max<int64_t>(1, (rows + g.ch - 1) / g.ch);
  return g;
}

__global__ __launch_bounds__(GROUP_TILE) void group_count_kernel(const int32_t* __restrict__ asg, int64_t rows, int64_t ch,
                                                                 int nlist, int32_t* __restrict__ hist) {
  const int64_t r0 = (int64_t)blockIdx.x * ch, r1 = r0 + ch < rows ? r0 + ch : rows;
  int32_t* h = hist + (int64_t)blockIdx.x * nlist;
  for (int64_t i = r0 + threadIdx.x; i < r1; i += GROUP_TILE) atomicAdd(&h[asg[i]], 1);
}

// per cluster: counts of the row blocks -> exclusive prefix over the blocks (in place) and the list length
__global__ void group_block_prefix_kernel(int32_t* __restrict__ hist, int nb, int nlist, int32_t* __restrict__ total) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= nlist) return;
  int32_t run = 0;
  for (int b = 0; b < nb; ++b) {
    const int32_t v = hist[(int64_t)b * nlist + c];
    hist[(int64_t)b * nlist + c] = run;
    run += v;
  }
  total[c] = run;
}

// off[c] = sum of total[0..c), off[nlist] = rows; one workgroup walks the lists in order
__global__ __launch_bounds__(1024) void group_offsets_kernel(const int32_t* __restrict__ total, int nlist,
                                                             int32_t* __restrict__ off) {
  __shared__ int32_t s_part[1024];
  __shared__ int32_t s_base;
  if (threadIdx.x == 0) s_base = 0;
  __syncthreads();
  for (int c0 = 0; c0 < nlist; c0 += 1024) {
    const int c = c0 + threadIdx.x;
    const int32_t v = c < nlist ? total[c] : 0;
    s_part[threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {  // inclusive scan of the 1024 values
      const int32_t add = threadIdx.x >= d ? s_part[threadIdx.x - d] : 0;
      __syncthreads();
      s_part[threadIdx.x] += add;
      __syncthreads();
    }
    if (c < nlist) off[c] = s_base + s_part[threadIdx.x] - v;
    __syncthreads();
    if (threadIdx.x == 1023) s_base += s_part[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0) off[nlist] = s_base;
}

__global__ __launch_bounds__(GROUP_TILE) void group_scatter_kernel(const int32_t* __restrict__ asg, int64_t rows, int64_t ch,
                                                                   int nlist, int32_t* __restrict__ hist,
                                                                   const int32_t* __restrict__ off,
                                                                   int32_t* __restrict__ members) {
  __shared__ int32_t s_key[GROUP_TILE];
  const int64_t r0 = (int64_t)blockIdx.x * ch, r1 = r0 + ch < rows ? r0 + ch : rows;
  int32_t* h = hist + (int64_t)blockIdx.x * nlist;  // rows of this cluster placed so far, by earlier blocks and tiles
  const int tid = threadIdx.x;
  for (int64_t t0 = r0; t0 < r1; t0 += GROUP_TILE) {
    const int64_t i = t0 + tid;
    const bool valid = i < r1;
    const int32_t key = valid ? asg[i] : -1;
    s_key[tid] = key;
    __syncthreads();
    int before = 0, same = 0;  // rows of the tile in the same list: ahead of this one, and in all
    for (int j = 0; j < GROUP_TILE; ++j) {
      const bool eq = s_key[j] == key;
      same += eq;
      before += eq && j < tid;
    }
    if (valid) {
      // the counter is only ever changed by atomics of this workgroup; read it where they are performed
      const int32_t base = __hip_atomic_load(&h[key], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      members[off[key] + base + before] = (int32_t)i;
    }
    __syncthreads();  // every row of the tile has read its counter
    if (valid && before == same - 1) atomicAdd(&h[key], same);
    __syncthreads();  // and the next tile sees the advanced counters
  }
}

// rows [0, rows) grouped by asg[] into off[nlist + 1] / members[rows]; hist holds group_plan(rows).nb * nlist words
static int launch_group_rows(const int32_t* asg, int64_t rows, int nlist, int32_t* off, int32_t* members, int32_t* hist,
                             int32_t* total, hipStream_t st) {
  const GroupPlan g = group_plan(rows);
  const int64_t hw = (int64_t)g.nb * nlist;
  hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(hw)), dim3(256), 0, st, hist, hw, 0);
  if (rows > 0)
    hipLaunchKernelGGL(group_count_kernel, dim3(g.nb), dim3(GROUP_TILE), 0, st, asg, rows, g.ch, nlist, hist);
  hipLaunchKernelGGL(group_block_prefix_kernel, dim3((nlist + 255) / 256), dim3(256), 0, st, hist, g.nb, nlist, total);
  hipLaunchKernelGGL(group_offsets_kernel, dim3(1), dim3(1024), 0, st, total, nlist, off);
  if (rows > 0)
    hipLaunchKernelGGL(group_scatter_kernel, dim3(g.nb), dim3(GROUP_TILE), 0, st, asg, rows, g.ch, nlist, hist, off, members);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

// nearest rotated centroid of every row of `x` [rows][D]; `scores` holds chunk x nlist floats
static int assign_rows(const float* x, int64_t rows, int D, int nlist, const float* ct, const float* csq, float* scores,
                       int64_t chunk, int32_t* out, hipStream_t st) {
  for (int64_t s = 0; s < rows; s += chunk) {
    const int64_t m = std::min(chunk, rows - s);
    int rc = launch_gemm(x + s * D, ct, scores, m, nlist, D, 3, nullptr, csq, st);
    if (rc) return rc;
    hipLaunchKernelGGL(argmin_rows_kernel, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, st, scores, m, nlist, out + s);
  }
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

int build_index_device(rabitq_index* ix, const float* data, const float* rotation_host, int kmeans_iters,
                       int64_t train_size, float eps0, int center, hipStream_t st) {
  const int D = ix->dim, nlist = ix->nlist, B = ix->total_bits;
  const int64_t N = ix->n;
  int rc;
#define RQ_TRY(x) do { if ((rc = (x)) != RABITQ_OK) return rc; } while (0)
  // rotation to the device, rotate all vectors once (distances are rotation invariant, so
  // clustering and residuals are taken in the rotated space)
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->rotation), (size_t)D * D * sizeof(float)));
  RQ_HIP(hipMemcpyAsync(ix->rotation, rotation_host, (size_t)D * D * sizeof(float), hipMemcpyHostToDevice, st));
  DevBuf<float> xr, tr, c_rows, scores;
  DevBuf<int32_t> asg, off, members, hist, total;
  RQ_TRY(xr.alloc(N * D));
  if (center && N > 0) {
    // mean of the raw vectors; every later step sees (x - mean) P = x P - mean P
    DevBuf<double> partial;
    DevBuf<float> mean_dev;
    RQ_TRY(partial.alloc((int64_t)MEAN_BLOCKS * D));
    RQ_TRY(mean_dev.alloc(D));
    hipLaunchKernelGGL(column_partial_kernel, dim3(MEAN_BLOCKS), dim3(256), 0, st, data, N, D, partial.p);
    hipLaunchKernelGGL(column_mean_kernel, dim3(1), dim3(256), 0, st, partial.p, N, D, mean_dev.p);
    std::vector<float> mean(D);
    RQ_HIP(hipMemcpyAsync(mean.data(), mean_dev.p, (size_t)D * sizeof(float), hipMemcpyDeviceToHost, st));
    RQ_HIP(hipStreamSynchronize(st));
    RQ_TRY(set_index_mean(ix, mean.data(), rotation_host, st));
  }
  RQ_TRY(launch_rotate(ix, data, xr.p, N, st));
  const int64_t nt = std::max<int64_t>(nlist, std::min<int64_t>(train_size > 0 ? train_size : N, N));
  RQ_TRY(tr.alloc(nt * D));
  RQ_TRY(c_rows.alloc((int64_t)nlist * D));
  hipLaunchKernelGGL(gather_rows_kernel, dim3(grid_for(nt * D)), dim3(256), 0, st, xr.p, N, nt, D, tr.p);
  hipLaunchKernelGGL(gather_rows_kernel, dim3(grid_for((int64_t)nlist * D)), dim3(256), 0, st, tr.p, nt, (int64_t)nlist,
                     D, c_rows.p);
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->centroids_t), (size_t)D * nlist * sizeof(float)));
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->centroid_sq), (size_t)nlist * sizeof(float)));
  const int64_t chunk = std::max<int64_t>(1024, (int64_t)(64 << 20) / nlist);
  RQ_TRY(scores.alloc(std::min<int64_t>(chunk, std::max(N, nt)) * nlist));
  RQ_TRY(asg.alloc(std::max(N, nt)));
  RQ_TRY(off.alloc(nlist + 1));
  RQ_TRY(members.alloc(std::max(N, nt)));
  RQ_TRY(hist.alloc((int64_t)std::max(group_plan(N).nb, group_plan(nt).nb) * nlist));
  RQ_TRY(total.alloc(nlist));
  for (int it = 0; it < kmeans_iters; ++it) {
    hipLaunchKernelGGL(transpose_centroids_kernel, dim3((nlist + 255) / 256), dim3(256), 0, st, c_rows.p, nlist, D,
                       ix->centroids_t, ix->centroid_sq);
    RQ_TRY(assign_rows(tr.p, nt, D, nlist, ix->centroids_t, ix->centroid_sq, scores.p, chunk, asg.p, st));
    RQ_TRY(launch_group_rows(asg.p, nt, nlist, off.p, members.p, hist.p, total.p, st));
    hipLaunchKernelGGL(centroid_update_kernel, dim3(nlist), dim3(256), 0, st, tr.p, off.p, members.p, D, c_rows.p);
  }
  hipLaunchKernelGGL(transpose_centroids_kernel, dim3((nlist + 255) / 256), dim3(256), 0, st, c_rows.p, nlist, D,
                     ix->centroids_t, ix->centroid_sq);
  RQ_TRY(assign_rows(xr.p, N, D, nlist, ix->centroids_t, ix->centroid_sq, scores.p, chunk, asg.p, st));
  RQ_TRY(launch_group_rows(asg.p, N, nlist, off.p, members.p, hist.p, total.p, st));
  // layout: cluster sizes, tile offsets (the total is needed on the host to size the arrays)
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->cluster_size), (size_t)nlist * sizeof(int32_t)));
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->tile_off), (size_t)tile_off_words(nlist) * sizeof(int32_t)));
  RQ_HIP(hipMemsetAsync(ix->tile_off, 0, (size_t)tile_off_words(nlist) * sizeof(int32_t), st));
  hipLaunchKernelGGL(cluster_layout_kernel, dim3((nlist + 255) / 256), dim3(256), 0, st, off.p, nlist, ix->cluster_size);
  std::vector<int32_t> h_off(nlist + 1), h_tile(nlist + 1);
  RQ_HIP(hipMemcpyAsync(h_off.data(), off.p, (size_t)(nlist + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, st));
  RQ_HIP(hipStreamSynchronize(st));
  int64_t tiles = 0;
  for (int c = 0; c < nlist; ++c) {
    h_tile[c] = (int32_t)tiles;
    tiles += (h_off[c + 1] - h_off[c] + TILE - 1) / TILE;
  }
  h_tile[nlist] = (int32_t)tiles;
  ix->host_tiles.resize(nlist);
  for (int c = 0; c < nlist; ++c) ix->host_tiles[c] = h_tile[c + 1] - h_tile[c];
  if (tiles > (0x7fffffff / TILE)) { set_error("index build: too many slots"); return RABITQ_EINVAL; }
  ix->n_tiles = tiles;
  ix->n_slots = tiles * TILE;
  RQ_HIP(hipMemcpyAsync(ix->tile_off, h_tile.data(), (size_t)(nlist + 1) * sizeof(int32_t), hipMemcpyHostToDevice, st));
  const int W = ix->W, LW = ix->LW;
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->short_codes), (size_t)std::max<int64_t>(1, tiles * W * TILE) * 4));
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->short_factors), (size_t)std::max<int64_t>(1, tiles * 3 * TILE) * 4));
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->ids), (size_t)std::max<int64_t>(1, tiles * TILE) * 4));
  hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(tiles * W * TILE)), dim3(256), 0, st,
                     reinterpret_cast<int32_t*>(ix->short_codes), tiles * W * TILE, 0);
  hipLaunchKernelGGL(init_short_factors_kernel, dim3(grid_for(tiles * 3 * TILE)), dim3(256), 0, st, ix->short_factors, tiles);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(tiles * TILE)), dim3(256), 0, st, ix->ids, tiles * TILE, -1);
  if (B > 1) {
    RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->long_codes), (size_t)std::max<int64_t>(1, tiles * TILE * LW) * 4));
    RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->long_factors), (size_t)std::max<int64_t>(1, tiles * TILE * 2) * 4));
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(tiles * TILE * LW)), dim3(256), 0, st,
                       reinterpret_cast<int32_t*>(ix->long_codes), tiles * TILE * LW, 0);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(tiles * TILE * 2)), dim3(256), 0, st,
                       reinterpret_cast<int32_t*>(ix->long_factors), tiles * TILE * 2, 0);
  }
  EncodeArgs a{};
  a.xr = xr.p; a.c_rows = c_rows.p; a.off = off.p; a.members = members.p; a.tile_off = ix->tile_off;
  a.n = N; a.D = D; a.B = B; a.F = ix->F; a.LW = LW; a.nlist = nlist; a.metric = ix->metric; a.eps0 = eps0;
  a.short_codes = ix->short_codes; a.short_factors = ix->short_factors; a.long_codes = ix->long_codes;
  a.long_factors = ix->long_factors; a.ids = ix->ids;
  // (a launch may hold fewer than 2^32 work-items: the positions are encoded in slices)
  constexpr int64_t SLICE = (int64_t)1 << 24;
  for (int64_t p0 = 0; p0 < N; p0 += SLICE) {
    a.p0 = p0;
    const unsigned grid = (unsigned)((std::min(SLICE, N - p0) + 3) / 4);
    const size_t smem = 4 * (size_t)D * (sizeof(float) + 1);
    const int dpl = (D + 63) / 64;
    if (dpl <= 2) hipLaunchKernelGGL(encode_kernel<2>, dim3(grid), dim3(256), smem, st, a);
    else if (dpl <= 4) hipLaunchKernelGGL(encode_kernel<4>, dim3(grid), dim3(256), smem, st, a);
    else if (dpl <= 8) hipLaunchKernelGGL(encode_kernel<8>, dim3(grid), dim3(256), smem, st, a);
    else if (dpl <= 16) hipLaunchKernelGGL(encode_kernel<16>, dim3(grid), dim3(256), smem, st, a);
    else hipLaunchKernelGGL(encode_kernel<32>, dim3(grid), dim3(256), smem, st, a);
  }
  RQ_HIP(hipGetLastError());
  RQ_HIP(hipStreamSynchronize(st));  // temporaries are freed on return
#undef RQ_TRY
  return RABITQ_OK;
}

}  // namespace rq
