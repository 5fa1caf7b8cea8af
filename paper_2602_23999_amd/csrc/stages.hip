// Small stages of the search path: per-query representation, probe selection,
// probe-list regrouping and the per-query merge.
#include "rq_device.h"

namespace rq {


// ---------------------------------------------------------------------------------
// Section 3.3.3 / 3.4.1(2): 4-bit signed quantisation of q' and its bit-planes, once
// per query.  One wavefront per query.  delta = max|q'|/7 and q'/delta use IEEE fp32
// division and round-half-even, because they decide integers.
// ---------------------------------------------------------------------------------
template <int F>
__global__ __launch_bounds__(256) void query_prep_kernel(const float* __restrict__ q_rot, int64_t nq, int D,
                                                        rabitq_query_repr o) {
  const int lane = threadIdx.x & 63;
  const int64_t q = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (q >= nq) return;
  query_prep_row<F>(q_rot + q * D, q, D, o, lane);
}

int launch_query_prep(const float* q_rot, int64_t nq, int D, int F, const rabitq_query_repr& out, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  const unsigned grid = (unsigned)((nq + 3) / 4);
  switch (F) {
    case 0: hipLaunchKernelGGL(query_prep_kernel<0>, dim3(grid), dim3(256), 0, st, q_rot, nq, D, out); break;
    case 2: hipLaunchKernelGGL(query_prep_kernel<2>, dim3(grid), dim3(256), 0, st, q_rot, nq, D, out); break;
    case 4: hipLaunchKernelGGL(query_prep_kernel<4>, dim3(grid), dim3(256), 0, st, q_rot, nq, D, out); break;
    default: hipLaunchKernelGGL(query_prep_kernel<8>, dim3(grid), dim3(256), 0, st, q_rot, nq, D, out); break;
  }
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

// ---------------------------------------------------------------------------------
// Section 3.3.2: the nprobe best clusters of one score row, best first, ties to the
// lower cluster id (the key's low word).  One workgroup per query.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void select_probes_kernel(const float* __restrict__ scores,
                                                           const float* __restrict__ sq_norm,
                                                           const float* __restrict__ centroid_sq, int nlist,
                                                           int nprobe, int npad, int metric,
                                                           int32_t* __restrict__ probe_ids,
                                                           float* __restrict__ probe_G,
                                                           float* __restrict__ probe_E) {
  extern __shared__ uint64_t sel_out[];  // [npad]
  __shared__ SelectScratch sh;
  const int64_t q = blockIdx.x;
  const float* row = scores + q * nlist;
  auto key_at = [&](int i) -> uint64_t { return make_key(row[i], (uint32_t)i); };
  block_select_smallest(nlist, nprobe, npad, key_at, sel_out, &sh);
  for (int r = threadIdx.x; r < nprobe; r += blockDim.x) {
    const uint64_t key = sel_out[r];
    const int c = (int)(uint32_t)key;
    const float s = ord2f((uint32_t)(key >> 32));
    probe_ids[q * nprobe + r] = c;
    probe_G[q * nprobe + r] = s;
    const float d2 = (metric == RABITQ_L2) ? s : (sq_norm[q] + centroid_sq[c] + 2.0f * s);
    probe_E[q * nprobe + r] = sqrtf(fmaxf(d2, 0.f));
  }
}

// The same selection with one wavefront per query and the whole score row in registers
// (nlist <= 64*R): no LDS histogram, no workgroup barriers.
template <int R>
__global__ __launch_bounds__(64) void select_probes_wave_kernel(const float* __restrict__ scores,
                                                               const float* __restrict__ sq_norm,
                                                               const float* __restrict__ centroid_sq, int nlist,
                                                               int nprobe, int npad, int metric,
                                                               int32_t* __restrict__ probe_ids,
                                                               float* __restrict__ probe_G,
                                                               float* __restrict__ probe_E) {
  extern __shared__ uint64_t sel_out[];  // [npad]
  const int lane = threadIdx.x;
  const int64_t q = blockIdx.x;
  const float* row = scores + q * nlist;
  uint64_t key[R];
  float sv[R];
#pragma unroll
  for (int r = 0; r < R; ++r) sv[r] = row[min(r * 64 + lane, nlist - 1)];  // unconditional: R requests in flight together
#pragma unroll
  for (int r = 0; r < R; ++r) sv[r] = pinned(sv[r]);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int i = r * 64 + lane;
    key[r] = (i < nlist) ? make_key(sv[r], (uint32_t)i) : KEY_NONE;
  }
  const uint64_t bound = wave_kth_bound<R>(key, nprobe);
  wave_gather_selected<R>(key, bound, sel_out, npad);
  block_bitonic_sort(sel_out, npad);
  for (int r = lane; r < nprobe; r += 64) {
    const uint64_t k2 = sel_out[r];
    const int c = (int)(uint32_t)k2;
    const float s = ord2f((uint32_t)(k2 >> 32));
    probe_ids[q * nprobe + r] = c;
    probe_G[q * nprobe + r] = s;
    const float d2 = (metric == RABITQ_L2) ? s : (sq_norm[q] + centroid_sq[c] + 2.0f * s);
    probe_E[q * nprobe + r] = sqrtf(fmaxf(d2, 0.f));
  }
}

// The selection for nprobe <= 64 and any nlist, one wavefront per query: the score row is read
// once through a register-resident sorted list of the best.
__global__ __launch_bounds__(256) void select_probes_stream_kernel(const float* __restrict__ scores,
                                                                  const float* __restrict__ sq_norm,
                                                                  const float* __restrict__ centroid_sq, int64_t nq,
                                                                  int nlist, int nprobe, int metric,
                                                                  int32_t* __restrict__ probe_ids,
                                                                  float* __restrict__ probe_G,
                                                                  float* __restrict__ probe_E) {
  const int lane = threadIdx.x & 63;
  const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (q >= nq) return;
  const float* row = scores + q * nlist;
  const WaveTopK top = stream_select_smallest(row, nlist, nprobe, lane);
  if (lane < nprobe) {
    const uint64_t key = top.v;
    const int c = (int)(uint32_t)key;
    const float s = ord2f((uint32_t)(key >> 32));
    probe_ids[q * nprobe + lane] = c;
    probe_G[q * nprobe + lane] = s;
    const float d2 = (metric == RABITQ_L2) ? s : (sq_norm[q] + centroid_sq[c] + 2.0f * s);
    probe_E[q * nprobe + lane] = sqrtf(fmaxf(d2, 0.f));
  }
}

// Which selection kernel a given (nlist, nprobe) takes: 0 = one wavefront per query streaming the score row through
// a register-resident sorted list (nprobe <= 64, any nlist); 1, 2, 3 = one wavefront per query with the whole row
// in registers, 8 / 16 / 32 scores per lane (nprobe > 64, nlist <= 512 / 1024 / 2048); 4 = one workgroup per
// query, radix select in LDS (nprobe > 64, nlist > 2048).
int probe_select_variant(int nlist, int nprobe) {
  if (nprobe <= 64) return 0;
  if (nlist <= 64 * 8) return 1;
  if (nlist <= 64 * 16) return 2;
  if (nlist <= 64 * 32) return 3;
  return 4;
}

int launch_select_probes(const float* scores, const float* sq_norm, const float* centroid_sq, int64_t nq, int nlist,
                         int nprobe, int metric, int32_t* probe_ids, float* probe_G, float* probe_E, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  const int npad = next_pow2(nprobe);
  const size_t smem = npad * sizeof(uint64_t);
  switch (probe_select_variant(nlist, nprobe)) {
    case 0:
      hipLaunchKernelGGL(select_probes_stream_kernel, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, st, scores, sq_norm,
                         centroid_sq, nq, nlist, nprobe, metric, probe_ids, probe_G, probe_E);
      break;
    case 1:
      hipLaunchKernelGGL(select_probes_wave_kernel<8>, dim3((unsigned)nq), dim3(64), smem, st, scores, sq_norm,
                         centroid_sq, nlist, nprobe, npad, metric, probe_ids, probe_G, probe_E);
      break;
    case 2:
      hipLaunchKernelGGL(select_probes_wave_kernel<16>, dim3((unsigned)nq), dim3(64), smem, st, scores, sq_norm,
                         centroid_sq, nlist, nprobe, npad, metric, probe_ids, probe_G, probe_E);
      break;
    case 3:
      hipLaunchKernelGGL(select_probes_wave_kernel<32>, dim3((unsigned)nq), dim3(64), smem, st, scores, sq_norm,
                         centroid_sq, nlist, nprobe, npad, metric, probe_ids, probe_G, probe_E);
      break;
    default:
      hipLaunchKernelGGL(select_probes_kernel, dim3((unsigned)nq), dim3(256), smem, st, scores, sq_norm, centroid_sq,
                         nlist, nprobe, npad, metric, probe_ids, probe_G, probe_E);
  }
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

// ---------------------------------------------------------------------------------
// Section 3.3.3: regroup (query, cluster) pairs by cluster, stable in query id.
// A query probes a cluster at most once, so membership is one bit per (cluster, query):
//   1. clear and set the bitmap  M[c][q]
//   2. per cluster: running popcount of its bitmap row -> rank of every 32-query word
//   3. exclusive scan of the cluster totals -> pair_off
//   4. every pair computes its own destination: pair_off[c] + rank of q in row c
// All integer, no order-dependent atomics: the output is unique.
// scratch: bitmap [nlist][QWORDS] | word_rank [nlist][QWORDS] | total [nlist]
// ---------------------------------------------------------------------------------
__global__ void fill_u32_kernel(uint32_t* p, int64_t n, uint32_t v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void bitmap_set_kernel(const int32_t* __restrict__ probe_ids, int64_t npairs, int nprobe, int qwords,
                                  uint32_t* __restrict__ bitmap) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < npairs; p += (int64_t)gridDim.x * blockDim.x) {
    const int c = probe_ids[p];
    const int64_t q = p / nprobe;
    atomicOr(&bitmap[(int64_t)c * qwords + (q >> 5)], 1u << (q & 31));
  }
}

__global__ __launch_bounds__(64) void row_rank_kernel(const uint32_t* __restrict__ bitmap, int qwords,
                                                      uint32_t* __restrict__ word_rank,
                                                      uint32_t* __restrict__ total) {
  const int c = blockIdx.x, lane = threadIdx.x;
  const uint32_t* row = bitmap + (int64_t)c * qwords;
  uint32_t* out = word_rank + (int64_t)c * qwords;
  uint32_t carry = 0;
  for (int base = 0; base < qwords; base += 64) {
    const int w = base + lane;
    const uint32_t pc = (w < qwords) ? __popc(row[w]) : 0u;
    uint32_t incl = pc;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t o = __shfl_up(incl, d, 64);
      if (lane >= d) incl += o;
    }
    if (w < qwords) out[w] = carry + incl - pc;
    carry += __shfl(incl, 63, 64);
  }
  if (lane == 0) total[c] = carry;
}

// out[0] = 0, out[i+1] = sum_{j<=i} f(in[j]); f = identity (div == 1) or ceil(x/div).  One workgroup.
__global__ __launch_bounds__(256) void exclusive_scan_kernel(const uint32_t* __restrict__ in, int n, int div,
                                                            int32_t* __restrict__ out) {
  __shared__ uint32_t part[256];
  const int tid = threadIdx.x;
  const int per = (n + 255) / 256;
  const int s = tid * per, e = min(n, s + per);
  uint32_t sum = 0;
  for (int i = s; i < e; ++i) sum += (in[i] + div - 1) / div;
  part[tid] = sum;
  __syncthreads();
  for (int d = 1; d < 256; d <<= 1) {
    const uint32_t o = (tid >= d) ? part[tid - d] : 0u;
    __syncthreads();
    part[tid] += o;
    __syncthreads();
  }
  uint32_t run = part[tid] - sum;
  for (int i = s; i < e; ++i) {
    out[i] = (int32_t)run;
    run += (in[i] + div - 1) / div;
  }
  if (tid == 255) out[n] = (int32_t)part[255];
}

__global__ void scatter_pairs_kernel(const int32_t* __restrict__ probe_ids, int64_t npairs, int nprobe, int qwords,
                                     const uint32_t* __restrict__ bitmap, const uint32_t* __restrict__ word_rank,
                                     const int32_t* __restrict__ pair_off, int32_t* __restrict__ pair_ids) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < npairs; p += (int64_t)gridDim.x * blockDim.x) {
    const int c = probe_ids[p];
    const int64_t q = p / nprobe;
    const int64_t wi = (int64_t)c * qwords + (q >> 5);
    const uint32_t below = bitmap[wi] & ((1u << (q & 31)) - 1u);
    pair_ids[pair_off[c] + word_rank[wi] + __popc(below)] = (int32_t)p;
  }
}

int64_t probe_list_scratch_words(int32_t nlist, int64_t nq) {
  const int64_t qwords = (nq + 31) / 32;
  return 2 * (int64_t)nlist * qwords + nlist;
}

// step 1 on its own: it needs no probes, so a search can clear the bitmap while the probes are still being computed
int launch_clear_list_bitmap(int64_t nq, int nlist, uint32_t* scratch, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  const int64_t bm_words = (int64_t)nlist * ((nq + 31) / 32);
  const unsigned g1 = (unsigned)std::min<int64_t>((bm_words + 255) / 256, 4096);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(g1), dim3(256), 0, st, scratch, bm_words, 0u);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

int launch_build_lists(const int32_t* probe_ids, int64_t nq, int nprobe, int nlist, int32_t* pair_off,
                       int32_t* pair_ids, uint32_t* scratch, hipStream_t st, bool bitmap_is_clear) {
  if (nq <= 0) return RABITQ_OK;
  const int qwords = (int)((nq + 31) / 32);
  const int64_t npairs = nq * nprobe;
  uint32_t* bitmap = scratch;
  uint32_t* word_rank = scratch + (int64_t)nlist * qwords;
  uint32_t* total = word_rank + (int64_t)nlist * qwords;
  if (!bitmap_is_clear) {
    if (int rc = launch_clear_list_bitmap(nq, nlist, scratch, st)) return rc;
  }
  const unsigned g2 = (unsigned)std::min<int64_t>((npairs + 255) / 256, 8192);
  hipLaunchKernelGGL(bitmap_set_kernel, dim3(g2), dim3(256), 0, st, probe_ids, npairs, nprobe, qwords, bitmap);
  hipLaunchKernelGGL(row_rank_kernel, dim3(nlist), dim3(64), 0, st, bitmap, qwords, word_rank, total);
  hipLaunchKernelGGL(exclusive_scan_kernel, dim3(1), dim3(256), 0, st, total, nlist, 1, pair_off);
  hipLaunchKernelGGL(scatter_pairs_kernel, dim3(g2), dim3(256), 0, st, probe_ids, npairs, nprobe, qwords, bitmap,
                     word_rank, pair_off, pair_ids);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

// ---------------------------------------------------------------------------------
// Section 3.3.5: merge the nprobe cluster-local lists of one query into its top-k.
// The lists (cnt[j] keys at stride `cap`) are first packed into LDS; the selection then
// runs on the packed keys.  A query with more candidates than the LDS buffer holds is
// selected straight from global memory instead.
// ---------------------------------------------------------------------------------
constexpr int MERGE_LDS_KEYS = 3072;

__global__ __launch_bounds__(256) void merge_kernel(const uint64_t* __restrict__ cand_keys,
                                                   const int32_t* __restrict__ cand_cnt, int k, int kpad, int cap,
                                                   int nprobe, int metric, int64_t* __restrict__ out_ids,
                                                   float* __restrict__ out_dists) {
  extern __shared__ uint64_t sel_out[];  // [kpad]
  __shared__ uint64_t buf[MERGE_LDS_KEYS];
  __shared__ int offs[RABITQ_MAX_NPROBE + 1];
  __shared__ SelectScratch sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t q = blockIdx.x;
  const uint64_t* keys = cand_keys + q * nprobe * (int64_t)cap;
  const int32_t* cnt = cand_cnt + q * nprobe;
  // exclusive scan of the list lengths (nprobe <= 1024: four per thread)
  int loc[4], sum = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = tid * 4 + i;
    loc[i] = (j < nprobe) ? cnt[j] : 0;
    sum += loc[i];
  }
  int incl = sum;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  __shared__ int wsum[4];
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  int base = incl - sum;
  for (int w2 = 0; w2 < wave; ++w2) base += wsum[w2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = tid * 4 + i;
    if (j < nprobe) offs[j] = base;
    base += loc[i];
  }
  if (tid == 255) offs[nprobe] = base;
  __syncthreads();
  const int total = offs[nprobe];
  if (total <= MERGE_LDS_KEYS) {
    for (int j = wave; j < nprobe; j += 4) {
      const int n = offs[j + 1] - offs[j];
      for (int e = lane; e < n; e += 64) buf[offs[j] + e] = keys[(int64_t)j * cap + e];
    }
    __syncthreads();
    auto key_at = [&](int i) -> uint64_t { return buf[i]; };
    block_select_smallest(total, k, kpad, key_at, sel_out, &sh);
  } else {
    auto key_at = [&](int i) -> uint64_t {
      const int j = i / cap, e = i - j * cap;
      return (e < cnt[j]) ? keys[i] : KEY_NONE;
    };
    block_select_smallest(nprobe * cap, k, kpad, key_at, sel_out, &sh);
  }
  for (int r = tid; r < k; r += blockDim.x) {
    const uint64_t key = sel_out[r];
    int64_t id = -1;
    float d = (metric == RABITQ_L2) ? INFINITY : -INFINITY;
    if (key != KEY_NONE) {
      id = (int64_t)(int32_t)(uint32_t)key;
      d = ord2f((uint32_t)(key >> 32));
      if (metric == RABITQ_IP) d = -d;
    }
    out_ids[q * k + r] = id;
    out_dists[q * k + r] = d;
  }
}

// The same merge with one wavefront per query (k <= 64): the candidate lists stream through
// a register-resident sorted list, G lanes per list, four entries per lane in flight.
__global__ __launch_bounds__(256) void merge_wave_kernel(const uint64_t* __restrict__ cand_keys,
                                                        const int32_t* __restrict__ cand_cnt, int64_t nq, int k,
                                                        int cap, int nprobe, int metric,
                                                        int64_t* __restrict__ out_ids, float* __restrict__ out_dists) {
  const int lane = threadIdx.x & 63;
  const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (q >= nq) return;
  const uint64_t* keys = cand_keys + q * nprobe * (int64_t)cap;
  const int32_t* cnt = cand_cnt + q * nprobe;
  int G = 1;  // lanes per list: the largest power of two with G * nprobe <= 64
  while (2 * G * nprobe <= 64) G <<= 1;
  const int ppc = 64 / G, g = lane % G;
  WaveTopK top;
  top.v = KEY_NONE;
  bool first = true;
  for (int jb = 0; jb < nprobe; jb += ppc) {
    const int j = jb + lane / G;
    const int n = (j < nprobe) ? min(cnt[j], cap) : 0;
    const int nmax = (int)wave_reduce_u32((uint32_t)n, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
    const uint64_t* row = keys + (int64_t)min(j, nprobe - 1) * cap;
    for (int e0 = 0; e0 < nmax; e0 += 4 * G) {
      uint64_t kk[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = e0 + u * G + g;
        kk[u] = (e < n) ? row[e] : KEY_NONE;  // (lists differ in length: reading past a short one would only add traffic)
      }
      if (first) {
        // the lanes' smallest keys start the sorted list; the other keys are then offered to it
        uint64_t mn = kk[0];
        int mu = 0;
#pragma unroll
        for (int u = 1; u < 4; ++u)
          if (kk[u] < mn) { mn = kk[u]; mu = u; }
        top.init_sorted(mn, lane);
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (e0 + u * G < nmax) top.push_tile(u == mu ? KEY_NONE : kk[u], k, lane);
        first = false;
        continue;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (e0 + u * G < nmax) top.push_tile(kk[u], k, lane);
      }
    }
  }
  if (lane < k) {
    const uint64_t key = top.v;
    int64_t id = -1;
    float d = (metric == RABITQ_L2) ? INFINITY : -INFINITY;
    if (key != KEY_NONE) {
      id = (int64_t)(int32_t)(uint32_t)key;
      d = ord2f((uint32_t)(key >> 32));
      if (metric == RABITQ_IP) d = -d;
    }
    out_ids[q * k + lane] = id;
    out_dists[q * k + lane] = d;
  }
}

int launch_merge(const uint64_t* cand_keys, const int32_t* cand_cnt, int64_t nq, int k, int nprobe, int metric,
                 int64_t* out_ids, float* out_dists, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  const int kpad = next_pow2(k);
  const int cap = next_pow2(k + TILE);
  if (k <= 64)
    hipLaunchKernelGGL(merge_wave_kernel, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, st, cand_keys, cand_cnt, nq, k,
                       cap, nprobe, metric, out_ids, out_dists);
  else
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)nq), dim3(256), kpad * sizeof(uint64_t), st, cand_keys, cand_cnt, k,
                       kpad, cap, nprobe, metric, out_ids, out_dists);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

__global__ void fill_f32_kernel(float* p, int64_t n, float v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

int launch_fill_f32(float* p, int64_t n, float v, hipStream_t st) {
  if (n <= 0) return RABITQ_OK;
  const unsigned g = (unsigned)std::min<int64_t>((n + 255) / 256, 4096);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(g), dim3(256), 0, st, p, n, v);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

}  // namespace rq
