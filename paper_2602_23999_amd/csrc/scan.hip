// Threshold seeding and the fused cluster-local search kernel (Sections 3.3.4, 3.4.1(2), 3.4.2).
#include <algorithm>

#include "rq_device.h"
#include "rq_scan_args.h"
#include "rq_small_batch.h"

namespace rq {

// 1-bit estimate of one lane's vector for one query (Section 3.4.1(2) + factors):
// est1 = G + f_add + f_rescale * (delta * I - delta * S / 2).
template <int W>
__device__ inline float est1_of(const uint32_t (&cw)[W], const_u32_ptr pl, float fa, float fr, float G, float dl,
                                float be, int* I_out) {
  const int I = ip_bitplanes<W>(cw, pl);
  *I_out = I;
  return G + fa + fr * fmaf(dl, (float)I, -be);  // dl = delta, be = delta * S / 2 (one fused step per vector)
}

// Lookup-table variant (Section 3.4.1(1), U = 4): <x_b, q'> as the fp32 sum, in ascending
// block order, of one binary16 entry per 4 dimensions; `lut` points at the query's tables
// [8W][16] in LDS.  The order and the types are part of the variant's definition.
template <int W>
__device__ inline float ip_lut_of(const uint32_t (&cw)[W], const _Float16* lut) {
  float acc = 0.f;
#pragma unroll
  for (int w = 0; w < W; ++w) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t nib = (cw[w] >> (4 * i)) & 15u;
      acc += (float)lut[(w * 8 + i) * 16 + nib];
    }
  }
  return acc;
}

// copy one query's tables (W * 64 words) into LDS
__device__ inline void stage_lut(_Float16* dst, const uint16_t* __restrict__ src, int W, int tid, int nt) {
  const uint32_t* s32 = reinterpret_cast<const uint32_t*>(src);
  uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
  for (int i = tid; i < W * 64; i += nt) d32[i] = s32[i];
}

// copy one rotated query (already in refinement order) into LDS
__device__ inline void stage_query(float* dst, const float* __restrict__ src, int D, int tid, int nt) {
  for (int i = tid; i < D; i += nt) dst[i] = src[i];
}

// ---------------------------------------------------------------------------------
// Seeding: one workgroup (256 threads) per query.  In the nearest probed cluster with
// at least k vectors: the m = max(k, SEED_M) smallest (est1, position) -> refine -> tau = k-th
// smallest refined estimate (B == 1: the k-th smallest est1).
// ---------------------------------------------------------------------------------
constexpr int SEED_CHUNK_TILES = 32;  // 2048 keys per selection round

template <int W, int F, int M>  // M = 1: lookup-table inner product
__global__ __launch_bounds__(256) void seed_kernel(ScanArgs a) {
  extern __shared__ unsigned char smem_raw[];
  // layout: chunk keys [2048] u64 | best [kpad] u64 | out [kpad] u64 | qf [D] f32 | tables [8W][16] f16 (M = 1)
  const int m = max(a.k, SEED_M);
  const int kpad = next_pow2(m);
  uint64_t* chunk = reinterpret_cast<uint64_t*>(smem_raw);
  uint64_t* best = chunk + SEED_CHUNK_TILES * TILE;
  uint64_t* out = best + kpad;
  float* qf = reinterpret_cast<float*>(out + kpad);
  _Float16* lut_s = reinterpret_cast<_Float16*>(qf + a.D);
  __shared__ SelectScratch sh;
  __shared__ int s_rank, s_t0, s_t1;
  __shared__ float s_G;
  __shared__ uint32_t s_max;

  const int64_t q = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (wave == 0) {
    // lane j looks at probe j: size, coarse term and tile range of all probes are fetched at once and the first
    // probe with at least k vectors is taken from its lane
    int r = -1, to0_ = 0, to1_ = 0;
    float g_ = 0.f;
    for (int b = 0; b < a.nprobe && r < 0; b += 64) {
      const int j = b + lane;
      const bool in = j < a.nprobe;
      const int pid = in ? a.probe_ids[q * a.nprobe + j] : 0;
      const float g = in ? a.probe_G[q * a.nprobe + j] : 0.f;
      const int sz = in ? a.cluster_size[pid] : 0;
      const int to0 = in ? a.tile_off[pid] : 0, to1 = in ? a.tile_off[pid + 1] : 0;
      const uint64_t mk = __ballot(in && sz >= a.k);
      if (mk != 0ull) {
        const int l = __ffsll((unsigned long long)mk) - 1;
        r = b + l;
        g_ = __shfl(g, l, 64);
        to0_ = __shfl(to0, l, 64);
        to1_ = __shfl(to1, l, 64);
      }
    }
    if (lane == 0) {
      s_rank = r;
      s_G = g_;
      s_t0 = to0_;
      s_t1 = to1_;
      s_max = 0u;
    }
  }
  for (int i = tid; i < kpad; i += 256) best[i] = KEY_NONE;
  if (F > 0) stage_query(qf, a.q_stage + q * a.D, a.D, tid, 256);
  if (M == 1) stage_lut(lut_s, a.lut + q * (int64_t)W * 128, W, tid, 256);
  __syncthreads();
  const int rank = s_rank;
  if (rank < 0) {
    if (tid == 0) a.tau_out[q] = 3.402823466e+38f;
    return;
  }
  const float G = s_G;
  const float dl = a.delta[q];
  const float be = 0.5f * dl * (float)a.sum_qhat[q];
  const float hsq = 0.5f * a.sum_q[q];
  const_u32_ptr pl = (const_u32_ptr)(a.planes + q * 4 * W);
  const int t0 = s_t0, t1 = s_t1;

  for (int tb = t0; tb < t1; tb += SEED_CHUNK_TILES) {
    const int nt = min(SEED_CHUNK_TILES, t1 - tb);
    for (int tl = wave; tl < nt; tl += 4) {
      const int tile = tb + tl;
      uint32_t cw[W];
#pragma unroll
      for (int w = 0; w < W; ++w) cw[w] = a.short_codes[((int64_t)tile * W + w) * TILE + lane];
      const float fa = a.short_factors[((int64_t)tile * 3 + 0) * TILE + lane];
      const float fr = a.short_factors[((int64_t)tile * 3 + 1) * TILE + lane];
      int I;
      const float e1 = (M == 1) ? G + fa + fr * (ip_lut_of<W>(cw, lut_s) - hsq) : est1_of<W>(cw, pl, fa, fr, G, dl, be, &I);
      const bool real = a.ids[(int64_t)tile * TILE + lane] >= 0;
      chunk[tl * TILE + lane] = real ? make_key(e1, (uint32_t)((tile - t0) * TILE + lane)) : KEY_NONE;
    }
    __syncthreads();
    const int nc = nt * TILE;
    auto key_at = [&](int i) -> uint64_t { return i < nc ? chunk[i] : best[i - nc]; };
    block_select_smallest(nc + kpad, m, kpad, key_at, out, &sh);
    for (int i = tid; i < kpad; i += 256) best[i] = out[i];
    __syncthreads();
  }
  if (F == 0) {
    if (tid == 0) a.tau_out[q] = ord2f((uint32_t)(best[a.k - 1] >> 32));
    return;
  }
  // refine the m seeds (fewer if the cluster is smaller), GL lanes per seed; their keys replace `out`
  constexpr int FF = (F > 0 ? F : 8), LW = W * FF, GL = RefineShape<LW>::G;
  const int grp = tid / GL, t = tid % GL;
  for (int i = tid; i < kpad; i += 256) out[i] = KEY_NONE;
  __syncthreads();
  for (int base = 0; base < m; base += 256 / GL) {
    const int sidx = base + grp;
    const bool valid = sidx < m && best[min(sidx, kpad - 1)] != KEY_NONE;
    float part = 0.f;
    int64_t slot = 0;
    if (valid) {
      slot = (int64_t)t0 * TILE + (uint32_t)best[sidx];
      part = refine_lane<FF, LW>(a.long_codes + slot * LW, qf, t);
    }
    const float ip = group_sum<GL>(part);
    if (valid && t == 0) {
      const float eB = G + a.long_factors[2 * slot] + a.long_factors[2 * slot + 1] * (ip - a.cB * a.sum_q[q]);
      out[sidx] = make_key(eB, (uint32_t)sidx);
    }
  }
  __syncthreads();
  block_bitonic_sort(out, kpad);
  if (tid == 0) a.tau_out[q] = fminf(ord2f((uint32_t)(out[a.k - 1] >> 32)), 3.402823466e+38f);
}

// ---------------------------------------------------------------------------------
// Seeding with one wavefront per query (k <= 64, popcount inner products): the same
// selection and refinement as seed_kernel, but the m <= 64 smallest (est1, position) keys are
// kept in registers while the cluster streams by, so there is no LDS and no barrier.
// ---------------------------------------------------------------------------------
// SPLIT (small batches): the four wavefronts of a workgroup share one query, each streaming a quarter of the
// cluster; their sorted lists meet in LDS and the first wavefront finishes alone.
// The work of one query (SPLIT: of the four wavefronts that share it; every one of them must call, and they meet
// at one barrier unless no probed cluster has k vectors, which all four find alike).
template <int W, int F, bool SPLIT>
__device__ inline void seed_wave_body(const ScanArgs& a, int64_t q, int lane, int wave, uint64_t* s_lists) {
  // Lane j looks at probe j: everything the chosen probe contributes (cluster, coarse term, tile range) is fetched
  // for all probes at once and read from the chosen lane, so the walk to the first tile is two dependent loads deep.
  int rank = -1, t0 = 0, t1 = 0, n_c = 0;
  float G = 0.f;
  for (int b = 0; b < a.nprobe && rank < 0; b += 64) {
    const int j = b + lane;
    const bool in = j < a.nprobe;
    const int pid = in ? a.probe_ids[q * a.nprobe + j] : 0;
    const float g = in ? a.probe_G[q * a.nprobe + j] : 0.f;
    const int sz = in ? a.cluster_size[pid] : 0;
    const int to0 = in ? a.tile_off[pid] : 0, to1 = in ? a.tile_off[pid + 1] : 0;
    const uint64_t m = __ballot(in && sz >= a.k);
    if (m != 0ull) {
      const int l = __ffsll((unsigned long long)m) - 1;
      rank = b + l;
      G = __shfl(g, l, 64);
      t0 = __shfl(to0, l, 64);  // positions in the keys are relative to the cluster's first tile
      t1 = __shfl(to1, l, 64);
      n_c = __shfl(sz, l, 64);
    }
  }
  if (rank < 0) {
    if (lane == 0) a.tau_out[q] = 3.402823466e+38f;
    return;
  }
  // (the same in all lanes)
  t0 = __builtin_amdgcn_readfirstlane(t0);
  t1 = __builtin_amdgcn_readfirstlane(t1);
  n_c = __builtin_amdgcn_readfirstlane(n_c);
  G = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(G)));
  const float dl = a.delta[q];
  const float be = 0.5f * dl * (float)a.sum_qhat[q];
  const_u32_ptr pl = (const_u32_ptr)(a.planes + q * 4 * W);
  int tw0 = t0;
  if (SPLIT) {  // this wavefront's quarter of the tiles (possibly empty)
    const int per = (t1 - t0 + 3) >> 2;
    tw0 = min(t0 + wave * per, t1);
    t1 = min(tw0 + per, t1);
  }
  const int m = max(a.k, SEED_M);  // <= 64
  WaveTopK top;
  top.v = KEY_NONE;
  // U tiles are requested together so that their load latencies overlap (tiles past the end
  // re-read the last tile and contribute no key)
  constexpr int U = (W <= 4) ? 4 : (W <= 8 ? 2 : 1);
  // est1 of U tiles starting at tb, as order-preserving words (all ones where there is no vector)
  auto estimate = [&](int tb, uint32_t (&ord)[U]) {
    uint32_t cw[U][W];
    float fa[U], fr[U];
    bool real[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int tile = min(tb + u, t1 - 1);
#pragma unroll
      for (int w = 0; w < W; ++w) cw[u][w] = a.short_codes[((int64_t)tile * W + w) * TILE + lane];
      fa[u] = a.short_factors[((int64_t)tile * 3 + 0) * TILE + lane];
      fr[u] = a.short_factors[((int64_t)tile * 3 + 1) * TILE + lane];
      real[u] = tb + u < t1 && (tile - t0) * TILE + lane < n_c;  // slots past the cluster's last vector are padding
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int I;
      const float e1 = est1_of<W>(cw[u], pl, fa[u], fr[u], G, dl, be, &I);
      ord[u] = real[u] ? f2ord(e1) : 0xffffffffu;
    }
  };
  // The first R tiles are estimated before anything is selected: the 64 per-lane minima (distinct vectors) start
  // the sorted list, so its m-th key is small from the outset and few of the remaining keys have to be inserted.
  constexpr int R = (W <= 4) ? 16 : (W <= 8 ? 8 : 4);
  if (tw0 < t1) {
    const uint32_t pos0 = (uint32_t)(tw0 - t0) * TILE + lane;
    uint32_t ord[R];
#pragma unroll
    for (int c2 = 0; c2 < R; c2 += U) {
      uint32_t o[U];
      estimate(tw0 + c2, o);
#pragma unroll
      for (int u = 0; u < U; ++u) ord[c2 + u] = (tw0 + c2 + u < t1) ? o[u] : 0xffffffffu;
    }
    uint32_t mo = ord[0];
    int mr = 0;
#pragma unroll
    for (int r = 1; r < R; ++r)
      if (ord[r] < mo) { mo = ord[r]; mr = r; }  // ties keep the lower position, as the key order does
    top.init_sorted(mo == 0xffffffffu ? KEY_NONE : (((uint64_t)mo << 32) | (pos0 + (uint32_t)(mr * TILE))), lane);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const bool take = r != mr && ord[r] != 0xffffffffu;
      top.push_tile(take ? (((uint64_t)ord[r] << 32) | (pos0 + (uint32_t)(r * TILE))) : KEY_NONE, m, lane);
    }
    for (int tb = tw0 + R; tb < t1; tb += U) {
      uint32_t o[U];
      estimate(tb, o);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t key = o[u] != 0xffffffffu ? (((uint64_t)o[u] << 32) | (uint32_t)((tb + u - t0) * TILE + lane)) : KEY_NONE;
        top.push_tile(key, m, lane);
      }
    }
  }
  if (SPLIT) {  // the other wavefronts hand their lists to the first and leave
    if (wave > 0) s_lists[(wave - 1) * 64 + lane] = top.v;
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w2 = 0; w2 < 3; ++w2) top.push_tile(s_lists[w2 * 64 + lane], m, lane);
  }
  if (F == 0) {
    const uint64_t kth = readlane_u64(top.v, a.k - 1);
    if (lane == 0) a.tau_out[q] = ord2f((uint32_t)(kth >> 32));
    return;
  }
  // refine the m seeds (fewer if the cluster is smaller), GL lanes per seed; lane i ends up with the
  // refined key of seed i, and the k-th smallest of those is tau
  constexpr int FF = (F > 0 ? F : 8), LW = W * FF, GL = RefineShape<LW>::G, NS = RefineShape<LW>::NS;
  const int grp = lane / GL, t = lane % GL;
  const float csq = a.cB * a.sum_q[q];
  uint64_t rkey = KEY_NONE;
  for (int base = 0; base < m; base += NS) {
    const int sidx = base + grp;
    const uint64_t skey = shfl_u64(top.v, min(sidx, 63));
    const bool valid = sidx < m && skey != KEY_NONE;
    // nothing here is fetched under a condition (an absent seed reads the cluster's first slot instead), so the
    // code words and the factors of a round are requested together
    const int64_t slot = (int64_t)t0 * TILE + (valid ? (uint32_t)skey : 0u);
    const float2 lf = *reinterpret_cast<const float2*>(a.long_factors + 2 * slot);
    const float part = refine_lane<FF, LW>(a.long_codes + slot * LW, a.q_stage + q * a.D, t);
    const float ip = group_sum<GL>(part);
    const float eB = G + lf.x + lf.y * (ip - csq);
    // seed base + g was refined by lanes g*GL ..; hand its estimate to lane base + g
    const int g = (lane - base) & (NS - 1);
    const float mine = __shfl(eB, g * GL, 64);
    const bool mine_valid = __shfl((int)valid, g * GL, 64) != 0;
    if (lane >= base && lane < base + NS && mine_valid) rkey = make_key(mine, (uint32_t)lane);
  }
  WaveTopK fin;
  fin.init_sorted(rkey, lane);
  const uint64_t kth = readlane_u64(fin.v, a.k - 1);
  if (lane == 0) a.tau_out[q] = fminf(ord2f((uint32_t)(kth >> 32)), 3.402823466e+38f);
}

template <int W, int F, bool SPLIT>
__global__ __launch_bounds__(256) void seed_wave_kernel(ScanArgs a, int64_t nq) {
  __shared__ uint64_t s_lists[SPLIT ? 3 * 64 : 1];
  // (the wavefront index is the same in all lanes: saying so lets everything indexed by the query be fetched
  // through the scalar cache)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous range of queries, so that
  // neighbouring queries (which the caller may have grouped by nearest list) share one L2
  // (the grid is the number of workgroups rounded up to a multiple of 8)
  const int per = (int)(gridDim.x >> 3);
  const int blk = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  const int64_t q = SPLIT ? (int64_t)blk : (int64_t)blk * 4 + wave;
  if (q >= nq) return;
  seed_wave_body<W, F, SPLIT>(a, q, lane, wave, s_lists);
}

// ---------------------------------------------------------------------------------
// Small batches: cluster selection (Section 3.3.2) and threshold seeding (Section 3.3.4) of one query by one
// workgroup, and, by the workgroup that finishes last, the pair lists and the scan's work-item table of the whole
// batch.  Nobody waits for anybody: a workgroup takes a ticket when it is done, and the holder of the last ticket
// knows that every other workgroup's probes are in memory.  The code of each step is the general kernels' own.
// ---------------------------------------------------------------------------------
template <int W, int F>
__global__ __launch_bounds__(256) void small_select_seed_kernel(ScanArgs a, SmallSelectArgs b) {
  __shared__ uint64_t s_lists[3 * 64];
  __shared__ uint32_t s_pairs[256], s_items[256];
  __shared__ int s_last;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane((int)(tid >> 6));
  const int64_t q = blockIdx.x;
  const int nprobe = a.nprobe;
  if (wave == 0) {
    const WaveTopK top = stream_select_smallest(b.scores + q * a.nlist, a.nlist, nprobe, lane);
    if (lane < nprobe) {
      const uint64_t key = top.v;
      const int c = (int)(uint32_t)key;
      const float sc = ord2f((uint32_t)(key >> 32));
      b.probe_ids[q * nprobe + lane] = c;
      b.probe_G[q * nprobe + lane] = sc;
      const float d2 = (b.metric == RABITQ_L2) ? sc : (b.sq_norm[q] + b.centroid_sq[c] + 2.0f * sc);
      b.probe_E[q * nprobe + lane] = sqrtf(fmaxf(d2, 0.f));
    }
  }
  __syncthreads();  // the probes are in memory for the other wavefronts of the workgroup
  if (b.do_seed) {
    seed_wave_body<W, F, true>(a, q, lane, wave, s_lists);
  } else if (tid == 0) {
    a.tau_out[q] = 3.402823466e+38f;
  }
  __syncthreads();
  if (tid == 0) {
    __threadfence();  // this workgroup's probes are visible to the device before its ticket is
    s_last = atomicAdd(b.ticket, 1) == (int)gridDim.x - 1;
  }
  __syncthreads();
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // and the last workgroup reads everybody's probes from memory
  small_lists_body<256>(b.lists, s_pairs, s_items);
  if (tid == 0) *b.ticket = 0;  // ready for the next launch
}

// ---------------------------------------------------------------------------------
// Fused cluster-local search.  One wavefront (= one 64-thread workgroup) per work item:
// QW pairs of the same cluster.  Lane l owns vector l of the current 64-vector tile; its
// code words stay in registers while the plane words of the QW queries come through the
// scalar cache.  Survivors of the filter are appended to a list in LDS; a full list (and
// the list left at the end) is refined NS candidates per round, G lanes per candidate, and
// the refined keys go to a per-query pool in LDS.  A pool that fills up is cut back to its
// k best (exact: it only compares final keys) and its k-th key then rejects later keys.
// Output: the surviving keys of each pair, unsorted, at most `pool` = next_pow2(k + 64) of them.
// ---------------------------------------------------------------------------------
constexpr int LIST_CAP = 512;
// MASKED: MASK_BATCH words of survivor bits are turned into list entries at a time, at most 16 each
constexpr int MASK_BATCH = 32;
constexpr int LIST_CAP_MASKED = 256 + 16 * MASK_BATCH;
constexpr int REFINE_AHEAD_MASKED = 2;  // refinement rounds whose loads are in flight (1 in the fused kernel)

#ifdef RQ_TIMELINE  // development: when each work item of the popcount kernel started, began to scan and ended
__device__ unsigned long long g_timeline[1 << 16][4];
#define RQ_TL(i, slot, v) do { if (threadIdx.x == 0 && (i) < (1 << 16)) g_timeline[i][slot] = (unsigned long long)(v); } while (0)
#else
#define RQ_TL(i, slot, v) do { } while (0)
#endif
#ifdef RQ_STATS  // development counters: survivors, refine rounds, compactions, flushes
__device__ unsigned long long g_scan_stats[8];
#define RQ_STAT(i, v) do { if (threadIdx.x == 0) atomicAdd(&g_scan_stats[i], (unsigned long long)(v)); } while (0)
#else
#define RQ_STAT(i, v) do { } while (0)
#endif

__device__ inline int pool_compact(uint64_t* pool, int pool_n, int cnt, int k) {
  __syncthreads();
  for (int i = cnt + (int)threadIdx.x; i < pool_n; i += 64) pool[i] = KEY_NONE;
  block_bitonic_sort(pool, pool_n);
  return min(cnt, k);
}

// PFD > 0 (streaming regime, few pairs per list): the codes and factors of the next tiles are requested ahead, because
// there the kernel waits for memory, not for the vector ALUs.
// MASKED: the first stage has been done by estimate_mfma_kernel; the survivors of a (pair, tile) are read as one bit
// per vector and only refinement, pools and output happen here.
template <int W, int F, bool DBG, int M, int PFD = 0, bool MASKED = false>  // M = 1: lookup-table inner product (tables of the QW queries in LDS)
__device__ __forceinline__ void scan_item(const ScanArgs& a, const int item) {
  // pairs per work item: QW, or one where every list is read about once (each pair then streams its list by itself,
  // with a quarter of the scalar state, which is what lets eight wavefronts share a SIMD)
  constexpr int QN = PFD > 0 ? 1 : QW;
  constexpr int FF = (F > 0 ? F : 8), LW = W * FF;
  constexpr int G = RefineShape<LW>::G, NS = RefineShape<LW>::NS;
  extern __shared__ unsigned char smem_raw[];
  uint64_t* pools = reinterpret_cast<uint64_t*>(smem_raw);             // [QN][pool]
  uint64_t* pool_kth = pools + (size_t)QN * a.pool;                    // [QN] k-th best key so far
  float* qs = reinterpret_cast<float*>(pool_kth + QN);                 // [QN][2]: G, cB*sum(q')
  int* pool_cnt = reinterpret_cast<int*>(qs + 2 * QN);                 // [QN]
  constexpr int LCAP = MASKED ? LIST_CAP_MASKED : LIST_CAP, AHEAD = MASKED ? REFINE_AHEAD_MASKED : 1;
  uint32_t* list = reinterpret_cast<uint32_t*>(pool_cnt + QN);         // [LCAP] (F > 0)
  // The queries in LDS, padded: a lane of the refinement reads a chunk of QCH = D / G consecutive floats, 16 bytes at
  // a time, and the chunks of one row (and the rows) would all start in the same banks; QPAD floats after every
  // chunk spread them over the banks.  Element e of row j sits at j * QROW + e + QPAD * (e / QCH).
  constexpr int QCH = RefineShape<LW>::WPL * (32 / FF), QPAD = 4, QROW = 32 * W + QPAD * G;
  float* qf = reinterpret_cast<float*>(list + (F > 0 ? LCAP : 0));     // [QN][QROW] (F > 0)
  _Float16* lut_s = reinterpret_cast<_Float16*>(qf + (F > 0 ? QN * QROW : 0));  // [QN][8W][16] (M = 1)
  const int lane = threadIdx.x;

  RQ_TL(item, 0, wall_clock64());
  int t0, nseg, ts, te, pbeg, np;
  // MASKED: blocks of survivor bits of this item's group of 16 pairs (its 4 pairs are lane group `mg` of every word)
  int mg = 0;
  const uint16_t* mblk = nullptr;
  typedef const StreamDesc __attribute__((address_space(4)))* const_sdesc_ptr;
  const_sdesc_ptr sdp = (const_sdesc_ptr)(a.stream_desc + (PFD > 0 ? item : 0));  // (read only where PFD > 0)
  if (MASKED) {
    // (everything about the item was laid down by item_desc_kernel: one load instead of a chain of dependent ones,
    // which is what a kernel that only refines would spend its time waiting for)
    typedef const ItemDesc __attribute__((address_space(4)))* const_desc_ptr;
    const_desc_ptr d = (const_desc_ptr)(a.item_desc + item);
    pbeg = d->pbeg;
    np = d->np_mg & 255;
    mg = d->np_mg >> 8;
    t0 = d->t0;
    ts = d->ts;
    te = d->te;
    nseg = d->nseg;
    mblk = reinterpret_cast<const uint16_t*>(a.surv_mask + (int64_t)d->mblock * 16);
  } else if (PFD > 0) {
    // (one load, as above: this variant waits for memory, and a chain of look-ups before the first tile is requested
    // is time in which the wavefront has nothing in flight)
    t0 = sdp->t0;
    ts = sdp->ts;
    te = sdp->te;
    nseg = sdp->nseg;
    pbeg = sdp->ppos;
    np = 1;
  } else {
    // cluster of this item: largest c with item_off[c] <= item
    const int c = wave_upper_cluster(a.item_off, a.nlist, item, lane);
    // a long cluster is scanned in nseg segments by separate work items
    t0 = a.tile_off[c];
    const int tc1 = a.tile_off[c + 1];
    nseg = seg_count(tc1 - t0, a.tseg, a.segmax);
    const int local = item - a.item_off[c];
    const int grp = local / nseg, sidx = local - grp * nseg;
    const int seglen = (tc1 - t0 + nseg - 1) / nseg;
    ts = t0 + sidx * seglen;
    te = min(tc1, ts + seglen);
    pbeg = a.pair_off[c] + grp * QN;
    np = __builtin_amdgcn_readfirstlane(min(QN, a.pair_off[c + 1] - pbeg));  // the same in all lanes
  }

  constexpr int PD = PFD > 0 ? (W <= 8 ? 2 : 1) : 0;  // tiles requested ahead (three and four: no faster)
  uint32_t pw[PD > 0 ? PD : 1][W];
  float pf[PD > 0 ? PD : 1][3];
  // (the prefetching variant reads every tile once and never again: with the streaming hint its codes and factors do
  // not displace one another, the descriptors, the plane words and the ids in the L2 - the largest single gain of that
  // variant; everywhere else a tile is shared by the pairs of its cluster and wants to stay cached)
  auto fetch = [&](uint32_t (&w_)[W], float (&f_)[3], int tile) {
#pragma unroll
    for (int w = 0; w < W; ++w) {
      const uint32_t* p = a.short_codes + ((int64_t)tile * W + w) * TILE + lane;
      w_[w] = PFD > 0 ? __builtin_nontemporal_load(p) : *p;
    }
#pragma unroll
    for (int f = 0; f < 3; ++f) {
      const float* p = a.short_factors + ((int64_t)tile * 3 + f) * TILE + lane;
      f_[f] = PFD > 0 ? __builtin_nontemporal_load(p) : *p;
    }
  };
  // (requested here, before the scalars of the pairs are fetched, so that the two waits overlap)
  if (PD > 0 && ts < te) {
#pragma unroll
    for (int d = 0; d < PD; ++d) fetch(pw[PD > 0 ? d : 0], pf[PD > 0 ? d : 0], min(ts + d, te - 1));
  }

  int pj[QN], Sj[QN], cnt[QN];
  float Gj[QN], Ej[QN], dlj[QN], bej[QN], tauj[QN], hsqj[QN];
  int64_t qj[QN];
#pragma unroll
  for (int j = 0; j < QN; ++j) {
    // (the prefetching variant has its pair's scalars in the descriptor; only the threshold, which the seeding writes
    // while the descriptors are being made, is fetched here)
    const int pp = PFD > 0 ? sdp->pp : a.pair_ids[pbeg + min(j, np - 1)];
    const int64_t q = PFD > 0 ? (int64_t)sdp->q : (int64_t)pair_query(a, pp);
    pj[j] = pp;
    qj[j] = q;
    Gj[j] = PFD > 0 ? sdp->G : a.probe_G[pp];
    dlj[j] = PFD > 0 ? sdp->delta : a.delta[q];
    {  // radius of the bound: ||q'-c'|| widened by the rounding error of the 4-bit query
      const float e = PFD > 0 ? sdp->E : a.probe_E[pp];
      Ej[j] = sqrtf(fmaf(a.qerr, dlj[j] * dlj[j], e * e));
    }
    Sj[j] = PFD > 0 ? sdp->S : a.sum_qhat[q];
    const float sumq = PFD > 0 ? sdp->sumq : a.sum_q[q];
    bej[j] = 0.5f * dlj[j] * (float)Sj[j];
    hsqj[j] = 0.5f * sumq;
    // (the prefetching variant reads it through the scalar cache: as a vector load it would be the youngest load in
    // flight when the tile loop starts, and every tile's wait for its own loads would become a wait for all of them)
    typedef const float __attribute__((address_space(4)))* const_f32_sptr;
    const float tau_q = PFD > 0 ? *(const_f32_sptr)(a.tau + q) : a.tau[q];
    tauj[j] = (j < np) ? tau_q : -3.402823466e+38f;  // an absent pair lets nothing through
    cnt[j] = 0;
    if (lane == 0) {
      pool_kth[j] = KEY_NONE;
      pool_cnt[j] = 0;
      qs[2 * j] = Gj[j];
      qs[2 * j + 1] = a.cB * sumq;
    }
  }
  if (M == 1) {
    // the lookup tables of the QN queries (W * 64 dwords each) go to LDS, all words of a batch requested before the
    // first one is stored
    constexpr int JB = (W * QN <= 16) ? QN : 1;
    uint32_t* d32 = reinterpret_cast<uint32_t*>(lut_s);
#pragma unroll
    for (int j0 = 0; j0 < QN; j0 += JB) {
      uint32_t tv[JB][W];
#pragma unroll
      for (int jj = 0; jj < JB; ++jj) {
        const uint32_t* s32 = reinterpret_cast<const uint32_t*>(a.lut + qj[j0 + jj] * (int64_t)W * 128);
#pragma unroll
        for (int u = 0; u < W; ++u) tv[jj][u] = s32[u * 64 + lane];
      }
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int u = 0; u < W; ++u) d32[(j0 + jj) * W * 64 + u * 64 + lane] = tv[jj][u];
    }
  }
  if (F > 0) {
    // the rotated queries go to LDS for the refinement: every word is requested before the first one is stored
    // (copied one after the other, each word would wait for its own round trip, 2 QN of them for D = 128)
    constexpr int DD = 32 * W, PER = (DD + 63) / 64, JB = (PER * QN <= 16) ? QN : 1;
#pragma unroll
    for (int j0 = 0; j0 < QN; j0 += JB) {
      float sv[JB][PER];
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int u = 0; u < PER; ++u) sv[jj][u] = a.q_stage[qj[j0 + jj] * DD + min(u * 64 + lane, DD - 1)];
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int u = 0; u < PER; ++u) sv[jj][u] = pinned(sv[jj][u]);
#pragma unroll
      for (int jj = 0; jj < JB; ++jj)
#pragma unroll
        for (int u = 0; u < PER; ++u)
          if (u * 64 + lane < DD) qf[(j0 + jj) * QROW + (u * 64 + lane) + QPAD * ((u * 64 + lane) / QCH)] = sv[jj][u];
    }
  }
  __syncthreads();
  RQ_TL(item, 1, wall_clock64());
  RQ_TL(item, 3, te - ts);

  int list_cnt = 0;
  // Streaming variant with 1-bit codes and k <= 64: the k best keys of each pair are kept in registers (lane l holds
  // the l-th smallest), so a list that is read once is also selected from in one pass, without the LDS pools and their
  // sorts; its k-th key tightens the filter as the pools' compaction does.
  constexpr bool REGK_VARIANT = (F == 0 && PFD > 0);
  const bool regk = REGK_VARIANT && a.k <= 64;
  WaveTopK top[QN];
  bool started[QN];
#pragma unroll
  for (int j = 0; j < QN; ++j) {
    top[j].v = KEY_NONE;
    started[j] = false;
  }

  // refine everything in the list (F > 0 only); wave-uniform control flow throughout.  Nothing is fetched under a
  // condition: a lane without a candidate repeats the list's last one, so a round's code words, factors and id are
  // requested together, and the next round's are requested before the current round is worked on.
  struct Cand {
    uint32_t w[RefineShape<LW>::WPL];
    float2 lf;
    int id, j;
    bool valid;
  };
  auto request = [&](int base, Cand& c_) {
    const int idx = base + lane / G;
    c_.valid = idx < list_cnt;
    const uint32_t e = list[min(idx, list_cnt - 1)];
    c_.j = (int)(e >> 30);
    const int64_t slot = (int64_t)t0 * TILE + (e & 0x3fffffffu);
    refine_load<FF, LW>(a.long_codes + slot * LW, lane % G, c_.w);
    c_.lf = *reinterpret_cast<const float2*>(a.long_factors + 2 * slot);
    c_.id = a.ids[slot];
  };
  auto flush = [&]() {
    __syncthreads();
    RQ_STAT(0, list_cnt);
    RQ_STAT(3, 1);
    // (AHEAD rounds are in flight: where this kernel only refines, nothing else covers the latency of the scattered
    // long-code reads)
    Cand ring[AHEAD];
#pragma unroll
    for (int d = 0; d < AHEAD; ++d)
      if (d * NS < list_cnt) request(d * NS, ring[d]);
    for (int base = 0; base < list_cnt; base += AHEAD * NS) {
#pragma unroll
      for (int d = 0; d < AHEAD; ++d) {
        const int rb = base + d * NS;
        if (rb >= list_cnt) break;
        RQ_STAT(1, 1);
        const Cand cur = ring[d];
        if (rb + AHEAD * NS < list_cnt) request(rb + AHEAD * NS, ring[d]);
        const int t = lane % G, j = cur.j;
        const float ip = group_sum<G>(refine_dot<FF, LW>(cur.w, qf + j * QROW + t * QPAD, t));
        if (cur.valid && t == 0) {
          const float eB = qs[2 * j] + cur.lf.x + cur.lf.y * (ip - qs[2 * j + 1]);
          const uint64_t key = make_key(eB, (uint32_t)cur.id);
          if (key <= pool_kth[j]) {
            const int pos = atomicAdd(&pool_cnt[j], 1);
            pools[(size_t)j * a.pool + pos] = key;
          }
        }
      }
      // a pool that could not take the keys of another AHEAD rounds is cut to its k best (pool >= k + 64 >= k + AHEAD * NS)
      __syncthreads();
#pragma unroll
      for (int jj = 0; jj < QN; ++jj) {
        const int cj = pool_cnt[jj];
        if (cj + AHEAD * NS > a.pool) {
          RQ_STAT(2, 1);
          uint64_t* pool = pools + (size_t)jj * a.pool;
          const int nc = pool_compact(pool, a.pool, cj, a.k);
          if (lane == 0) {
            pool_cnt[jj] = nc;
            if (nc >= a.k) pool_kth[jj] = pool[a.k - 1];
          }
          __syncthreads();
        }
      }
    }
    list_cnt = 0;
  };

  if (MASKED) {
    // The first stage is done: the survivor bits of MASK_BATCH / 16 tiles are turned into list entries at a time.  A
    // block holds, for each of the 4 groups of 4 pairs and each lj = 0..15, a 16-bit word about vectors 16 cb + lj and
    // pairs r of the group: bit 4 cb + r set = does not survive.  Lane l < MASK_BATCH takes word (tile wb / 16 + l / 16,
    // this item's group mg, lj = l % 16).
    const int nwords = (te - ts) * 16;
    const uint32_t present = 0x1111u * ((1u << np) - 1u);  // bits of the pairs this item has (r < np)
    auto word_at = [&](int wi) -> uint32_t {
      return (lane < MASK_BATCH && wi < nwords) ? (uint32_t)mblk[(int64_t)(wi >> 4) * TILE + 16 * mg + (wi & 15)] : 0xffffu;
    };
    uint32_t wnext = word_at(lane);
    for (int wb = 0; wb < nwords; wb += MASK_BATCH) {
      const uint32_t wcur = wnext;
      wnext = word_at(wb + MASK_BATCH + lane);
      const int wi = wb + lane;
      uint32_t field = ~wcur & present;
      if (__ballot(field != 0u) == 0ull) continue;
      const int mine_n = __popc(field);
      int incl = mine_n;  // inclusive scan over the lanes that carry words
#pragma unroll
      for (int d = 1; d < MASK_BATCH; d <<= 1) {
        const int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
      }
      const int total = __builtin_amdgcn_readlane(incl, MASK_BATCH - 1);
      if (list_cnt + total > LCAP) flush();
      int pos = list_cnt + incl - mine_n;
      const uint32_t pos0 = (uint32_t)((ts - t0 + (wi >> 4)) * TILE + (wi & 15));
      while (field != 0u) {
        const int b = __ffs(field) - 1;  // bit 4 cb + r
        list[pos++] = ((uint32_t)(b & 3) << 30) | (pos0 + 16u * (uint32_t)(b >> 2));
        field &= field - 1u;
      }
      list_cnt += total;
    }
  }
  // one 64-vector tile: first stage for the item's pairs, survivors filed (or, 1-bit codes, kept)
  auto scan_tile = [&](const uint32_t (&cw)[W], const float (&fq)[3], const int tile) {
    const float fa = fq[0], fr = fq[1], fe = fq[2];
    // The plane words are re-read through the scalar cache for every (tile, query): an
    // opaque zero keeps the compiler from hoisting QN*4*W scalar registers out of the loop.
    // (the streaming variant runs one or two queries per item and waits for memory, not for registers: there the
    // plane words may stay in scalar registers across tiles)
    int opaque0 = 0;
    if (!(PFD > 0 && W <= 4)) asm volatile("s_mov_b32 %0, 0" : "=s"(opaque0));
#pragma unroll
    for (int j = 0; j < QN; ++j) {
      // pairs the item does not have (the last group of a list; most groups when a list is probed by one or two
      // queries only) are not estimated at all
      if (j >= np) break;
      const_u32_ptr pl = (const_u32_ptr)(a.planes + qj[j] * 4 * W + opaque0);
      int I;
      float e1;
      if (M == 1) {
        const float ipf = ip_lut_of<W>(cw, lut_s + j * W * 128);
        I = __float_as_int(ipf);
        e1 = Gj[j] + fa + fr * (ipf - hsqj[j]);
      } else {
        e1 = est1_of<W>(cw, pl, fa, fr, Gj[j], dlj[j], bej[j], &I);
      }
      if (DBG) {
        if (j < np) a.dbg_ip[a.dbg_off[pbeg + j] + (int64_t)(tile - t0) * TILE + lane] = I;
      }
      const float filt = (F > 0) ? (e1 - fe * Ej[j]) : e1;
      const bool surv = filt <= tauj[j];
      const uint64_t m = __ballot(surv);
      if (m == 0ull) continue;
      const int ns = __popcll(m);
      const int before = __popcll(m & ((1ull << lane) - 1ull));
      if (REGK_VARIANT && regk) {
        const uint64_t key = surv ? make_key(e1, (uint32_t)((tile - t0) * TILE + lane)) : KEY_NONE;
        if (!started[j]) {
          top[j].init_sorted(key, lane);
          started[j] = true;
        } else {
          top[j].push_tile(key, a.k, lane);
        }
        const uint64_t kth = readlane_u64(top[j].v, a.k - 1);
        if (kth != KEY_NONE) tauj[j] = fminf(tauj[j], ord2f((uint32_t)(kth >> 32)));
        continue;
      }
      if (F == 0) {
        // B == 1: the 1-bit estimate is the final key
        uint64_t* pool = pools + (size_t)j * a.pool;
        if (cnt[j] + TILE > a.pool) {
          cnt[j] = pool_compact(pool, a.pool, cnt[j], a.k);
          // exact tightening: keys above the k-th best of this pair cannot be in its top-k
          if (cnt[j] >= a.k) tauj[j] = fminf(tauj[j], ord2f((uint32_t)(pool[a.k - 1] >> 32)));
        }
        // (the key's low word is the vector's position in its list, which needs no load; the id replaces it when the
        // pool is written out.  Lists hold their vectors in ascending id order, so equal estimates rank alike.)
        if (surv) pool[cnt[j] + before] = make_key(e1, (uint32_t)((tile - t0) * TILE + lane));
        cnt[j] += ns;
      } else {
        if (list_cnt + ns > LCAP) flush();
        if (surv) list[list_cnt + before] = ((uint32_t)j << 30) | (uint32_t)((tile - t0) * TILE + lane);
        list_cnt += ns;
      }
    }
  };
  if (!MASKED && PD >= 2) {
    // PD tiles ahead, in PD sets of registers that take turns: a set is requested again as soon as its tile is done
    // (rotating the sets instead would make every tile wait for the loads of the next one too), and every tile of the
    // main loop is scanned unconditionally.  Only a request past the item's end is left out: these loads carry the
    // streaming hint, so a clamped re-read of the last tile would come from memory a second time.
    int tile = ts;
    for (; tile + PD <= te; tile += PD) {
#pragma unroll
      for (int d = 0; d < PD; ++d) {
        scan_tile(pw[PD > 0 ? d : 0], pf[PD > 0 ? d : 0], tile + d);
        if (tile + d + PD < te) fetch(pw[PD > 0 ? d : 0], pf[PD > 0 ? d : 0], tile + d + PD);
      }
    }
    // the last tiles (fewer than PD) are in their sets already
#pragma unroll
    for (int d = 0; d + 1 < PD; ++d)
      if (tile + d < te) scan_tile(pw[PD > 0 ? d : 0], pf[PD > 0 ? d : 0], tile + d);
  }
  for (int tile = ts; !MASKED && PD < 2 && tile < te; ++tile) {
    uint32_t cw[W];
    float fq[3];
    if (PD > 0) {
#pragma unroll
      for (int w = 0; w < W; ++w) cw[w] = pw[0][w];
#pragma unroll
      for (int f = 0; f < 3; ++f) fq[f] = pf[0][f];
      fetch(pw[0], pf[0], min(tile + PD, te - 1));  // (PD == 1)
    } else {
      fetch(cw, fq, tile);
    }
    scan_tile(cw, fq, tile);
  }
  if (F > 0) {
    flush();
#pragma unroll
    for (int j = 0; j < QN; ++j) cnt[j] = pool_cnt[j];
  }
  // every key still in a pool goes out, unsorted; the per-query merge selects among them.
  // The segments of a split cluster share the pair's region (cand_cnt starts at 0 and is
  // advanced atomically), each contributing at most k keys so that the region cannot overflow.
  if (REGK_VARIANT && regk) {
    // the register lists go out through the pools' memory, so that one output path serves both
#pragma unroll
    for (int j = 0; j < QN; ++j) {
      if (j >= np) break;
      const bool have = lane < a.k && top[j].v != KEY_NONE;
      cnt[j] = __popcll(__ballot(have));
      if (have) pools[(size_t)j * a.pool + lane] = top[j].v;  // sorted: the present keys are the first cnt lanes
    }
  }
#pragma unroll
  for (int j = 0; j < QN; ++j) {
    if (j >= np) break;
    if (nseg > 1 && cnt[j] > a.k) cnt[j] = pool_compact(pools + (size_t)j * a.pool, a.pool, cnt[j], a.k);
  }
  __syncthreads();
  // lane j reserves pair j's part of its candidate region: the atomics of the work item are in flight together
  int mine = 0, base_l = 0;
#pragma unroll
  for (int j = 0; j < QN; ++j)
    if (lane == j && j < np) mine = cnt[j];
  if (mine > 0) {
    int pp = pj[0];
#pragma unroll
    for (int j = 1; j < QN; ++j)
      if (lane == j) pp = pj[j];
    if (nseg > 1) base_l = atomicAdd(&a.cand_cnt[pp], mine);
    else a.cand_cnt[pp] = mine;  // the only work item of this pair: its region starts at 0 and nobody else counts
  }
#pragma unroll
  for (int j = 0; j < QN; ++j) {
    if (j >= np) break;
    const uint64_t* pool = pools + (size_t)j * a.pool;
    const int base = __builtin_amdgcn_readlane(base_l, j);
    for (int e = lane; e < cnt[j]; e += 64) {
      uint64_t key = pool[e];
      if (F == 0) key = (key & 0xffffffff00000000ull) | (uint32_t)a.ids[(int64_t)t0 * TILE + (uint32_t)key];
      a.cand_keys[(int64_t)pj[j] * a.cand_stride + base + e] = key;
    }
  }
  RQ_TL(item, 2, wall_clock64());
}

template <int W, int F, bool DBG, int M, int PFD = 0, bool MASKED = false>
__global__ __launch_bounds__(64) void scan_kernel(ScanArgs a) {
  // XCD-aware order: workgroups are dealt round-robin to the 8 XCDs, so give each XCD a
  // contiguous range of work items; items of one cluster then share one L2.
  // (the grid is an upper bound of the number of work items; the ranges are cut from the true count)
  const int n_items = a.item_off[a.nlist];
  const int per = (n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per || item >= n_items) return;
  scan_item<W, F, DBG, M, PFD, MASKED>(a, item);
}

// The prefetching variant (few pairs per list: every list is read from memory about once) as a kernel of its own: one
// pair per work item.  It waits for memory, so what it needs is wavefronts in flight, and the scalar state of four
// pairs (their plane words above all) costs more than 100 scalar registers, which admits six wavefronts per SIMD.
// One workgroup per item, in the order of the descriptors (longest list first when the host has that order, so that
// the short items come last and the launch ends everywhere at about the same time).  The number of items is only known
// on the device and its upper bound is several times the usual count (all queries might probe the longest list), so
// the grid is sized for the usual case and a workgroup goes on to item + grid size while there is one: a grid sized
// from the bound would end in empty workgroups that cost more dispatch time than the scan takes.
template <int W, int F, bool DBG>
__device__ __forceinline__ void scan_stream_items(const ScanArgs& a) {
  const int n_items = a.item_off[a.nlist];
  for (int item = (int)blockIdx.x; item < n_items; item += (int)gridDim.x) {
    scan_item<W, F, DBG, 0, 1, false>(a, item);
    __syncthreads();  // (a further item starts by overwriting what this one read from LDS last)
  }
}
// (1-bit codes: the kernel is held to the registers with which eight wavefronts share a SIMD; with a long code the
// refinement's registers would spill to memory under that limit, so that form is left to the compiler)
template <int W, bool DBG>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(8))) void scan_stream_kernel(ScanArgs a) {
  scan_stream_items<W, 0, DBG>(a);
}
template <int W, int F, bool DBG>
__global__ __launch_bounds__(64) void scan_stream_long_kernel(ScanArgs a) {
  scan_stream_items<W, F, DBG>(a);
}

// ---------------------------------------------------------------------------------
// Matrix-core variant of the fused cluster-local search.  The integer inner product
// <x_b, qhat> of Section 3.4.1(2) is a dense contraction once the batch is grouped by
// cluster: (queries probing the cluster) x (vectors of the cluster) over D.  One wavefront
// takes QM = 16 pairs of one cluster; per 64-vector tile it expands the sign bits to int8
// once ((word >> s) & 0x01010101, four dimensions per two instructions) and issues
// v_mfma_i32_16x16x64_i8 with the 16 queries' qhat bytes held in registers.  Accumulator
// r of lane l is query 4*(l/16)+r, vector 16*cb + l%16 of the tile, so a lane keeps the
// factors of its four vectors and the scalars of its four queries.  Everything after the
// inner product (filter, survivor list, refinement, pools, output) is shared in form with
// the popcount kernel; integer results are identical.
// ---------------------------------------------------------------------------------
// wavefronts per work item (they split its tiles and own QM / n of its queries each): four for short codes, two for
// wide ones, where a tile keeps a wavefront busy for longer and the barrier after every round of tiles weighs more
// (D = 960: 0.97 ms with four, 0.86 ms with two, 0.86 ms with one; D = 128: 0.32 / 0.38 / 0.45 ms)
__host__ __device__ constexpr int mfma_waves(int W) { return W >= 16 ? 2 : 4; }
constexpr int MLIST_FLUSH = 128;              // an owner list longer than this is refined before the next tiles
// + what one round of tiles can add: every wavefront a tile, 64 vectors x QM / n queries per owner
__host__ __device__ constexpr int mlist_cap(int n) { return MLIST_FLUSH + n * TILE * (QM / n); }

// A decision every wavefront of the workgroup must take alike, although each of them computes it from LDS counters
// that faster wavefronts may already be advancing: the first wavefront to arrive fixes the value in `slot` (which
// holds AGREE_UNSET) and the others adopt it.  Whoever advances a counter has taken the decision first, so the
// value that wins was computed before any counter moved.  `mine` is wave-uniform and never AGREE_UNSET.
constexpr uint32_t AGREE_UNSET = 0xffffffffu;
__device__ inline uint32_t wave_agree(uint32_t* slot, uint32_t mine, int lane) {
  uint32_t v = 0;
  if (lane == 0) {
    const uint32_t old = atomicCAS(slot, AGREE_UNSET, mine);
    v = (old == AGREE_UNSET) ? mine : old;
  }
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}

__device__ inline int block_pool_compact(uint64_t* pool, int pool_n, int cnt, int k) {
  __syncthreads();
  for (int i = cnt + (int)threadIdx.x; i < pool_n; i += (int)blockDim.x) pool[i] = KEY_NONE;
  block_bitonic_sort(pool, pool_n);
  return min(cnt, k);
}

// Work split inside the workgroup of n = mfma_waves(W) wavefronts: every wavefront scans every n-th tile for all 16
// queries, but survivors are filed by OWNER: query j belongs to wavefront j % n, which alone
// refines them and keeps that query's pool.  Refinement therefore needs no workgroup
// barrier; the wavefronts only meet once per round of tiles.
template <int W, int F, bool DBG>
__global__ __launch_bounds__(64 * mfma_waves(W)) void scan_mfma_kernel(ScanArgs a) {
  constexpr int FF = (F > 0 ? F : 8), LW = W * FF, KC = (W + 1) / 2;
  constexpr int MWAVES = mfma_waves(W), MLIST_CAP = mlist_cap(MWAVES);
  constexpr int G = RefineShape<LW>::G, NS = RefineShape<LW>::NS;
  extern __shared__ unsigned char smem_raw[];
  uint64_t* pools = reinterpret_cast<uint64_t*>(smem_raw);          // [QM][pool]
  uint64_t* pool_kth = pools + (size_t)QM * a.pool;                 // [QM]
  float* qs = reinterpret_cast<float*>(pool_kth + QM);              // [QM][2]: G, cB*sum(q')
  int* pool_cnt = reinterpret_cast<int*>(qs + 2 * QM);              // [QM]
  int* qidx = pool_cnt + QM;                                        // [QM] query of each pair
  int* s_list_cnt = qidx + QM;                                      // [MWAVES] entries in each owner list
  int* s_out = s_list_cnt + MWAVES;                                 // [QM] first output slot of each pair
  uint32_t* s_agree = reinterpret_cast<uint32_t*>(s_out + QM);      // [2] per-round decisions (wave_agree), by round parity
  uint32_t* lists = s_agree + 2;                                    // [MWAVES][MLIST_CAP] (F > 0)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lj = lane & 15, g = lane >> 4;

  const int n_items = a.item_off[a.nlist];
  const int per = (n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per || item >= n_items) return;
  const int c = wave_upper_cluster(a.item_off, a.nlist, item, lane);
  const int t0 = a.tile_off[c], tc1 = a.tile_off[c + 1];
  const int nseg = seg_count(tc1 - t0, a.tseg, a.segmax);
  const int local = item - a.item_off[c];
  const int grp = local / nseg, sidx = local - grp * nseg;
  const int seglen = (tc1 - t0 + nseg - 1) / nseg;
  const int ts = t0 + sidx * seglen, t1 = min(tc1, ts + seglen);
  const int pbeg = a.pair_off[c] + grp * QM;
  const int np = min(QM, a.pair_off[c + 1] - pbeg);

  // query operand: lane (row lj, k-group g) holds bytes 16g .. 16g+15 of every 64-dimension chunk of qhat8, which
  // is stored in the order the expansion of the code words produces (qhat_mfma_pos)
  v4i qa[KC];
  {
    const int pp = a.pair_ids[pbeg + min(lj, np - 1)];
    const int64_t q = pair_query(a, pp);
    const int8_t* src = a.qhat8 + q * a.Dp + 16 * g;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      qa[kc] = *reinterpret_cast<const v4i*>(src + 64 * kc);
      if (lj >= np) qa[kc] = v4i{0, 0, 0, 0};
    }
    if (tid < QM) {  // one thread per pair fills the shared per-pair state
      qidx[lj] = (int)q;
      qs[2 * lj] = a.probe_G[pp];
      qs[2 * lj + 1] = a.cB * a.sum_q[q];
      pool_kth[lj] = KEY_NONE;
      pool_cnt[lj] = 0;
    }
    if (tid < MWAVES) s_list_cnt[tid] = 0;
    if (tid < 2) s_agree[tid] = AGREE_UNSET;
  }
  // scalars of this lane's four queries (rows 4g .. 4g+3; query 4g+r is owned by wavefront r)
  float al[4], be[4], Gr[4], Er[4], tr[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qi = 4 * g + r;
    const int pp = a.pair_ids[pbeg + min(qi, np - 1)];
    const int64_t q = pair_query(a, pp);
    const float dl = a.delta[q];
    al[r] = dl;
    be[r] = 0.5f * dl * (float)a.sum_qhat[q];
    Gr[r] = a.probe_G[pp];
    {  // radius of the bound: ||q'-c'|| widened by the rounding error of the 4-bit query
      const float e = a.probe_E[pp];
      Er[r] = sqrtf(fmaf(a.qerr, dl * dl, e * e));
    }
    tr[r] = (qi < np) ? a.tau[q] : -3.402823466e+38f;
  }
  __syncthreads();

  // Cuts the pools named by `mask` (bit jj = pool jj; the same in every wavefront) back to their k best.
  // No wavefront may be adding to those pools meanwhile.
  auto block_compact = [&](uint32_t mask) {
#pragma unroll 1
    for (int jj = 0; jj < QM; ++jj) {
      if ((mask >> jj) & 1u) {
        const int cj = pool_cnt[jj];
        uint64_t* pool = pools + (size_t)jj * a.pool;
        const int nc = block_pool_compact(pool, a.pool, cj, a.k);
        if (tid == 0) {
          pool_cnt[jj] = nc;
          if (nc >= a.k) pool_kth[jj] = pool[a.k - 1];
        }
        __syncthreads();
      }
    }
  };

  // F > 0: this wavefront refines its own list (queries j with j % MWAVES == wave) into its own pools
  // (nothing is fetched under a condition: a lane without a candidate repeats the list's last one, so a round's code
  // words, factors and id are requested together, and the next round's before the current round is worked on)
  struct Cand {
    uint32_t w[RefineShape<LW>::WPL];
    float2 lf;
    int id, j;
    bool valid;
  };
  auto flush_own = [&]() {
    uint32_t* list = lists + (size_t)wave * MLIST_CAP;
    const int list_cnt = s_list_cnt[wave];
    auto request = [&](int base, Cand& c_) {
      const int idx = base + lane / G;
      c_.valid = idx < list_cnt;
      const uint32_t e = list[min(idx, list_cnt - 1)];
      c_.j = (int)(e >> 28);
      const int64_t slot = (int64_t)t0 * TILE + (e & 0x0fffffffu);
      refine_load<FF, LW>(a.long_codes + slot * LW, lane % G, c_.w);
      c_.lf = *reinterpret_cast<const float2*>(a.long_factors + 2 * slot);
      c_.id = a.ids[slot];
    };
    Cand nxt;
    if (list_cnt > 0) request(0, nxt);
    for (int base = 0; base < list_cnt; base += NS) {
      const Cand cur = nxt;
      if (base + NS < list_cnt) request(base + NS, nxt);
      const int t = lane % G, j = cur.j;
      const float* qrow = a.q_stage + (int64_t)qidx[j] * a.D;
      const float ip = group_sum<G>(refine_dot<FF, LW>(cur.w, qrow, t));
      if (cur.valid && t == 0) {
        const float eB = qs[2 * j] + cur.lf.x + cur.lf.y * (ip - qs[2 * j + 1]);
        const uint64_t key = make_key(eB, (uint32_t)cur.id);
        if (key <= pool_kth[j]) {
          const int pos = atomicAdd(&pool_cnt[j], 1);
          pools[(size_t)j * a.pool + pos] = key;
        }
      }
      wave_sync();
#pragma unroll
      for (int rr = 0; rr < QM / MWAVES; ++rr) {  // the pools this wavefront owns
        const int jj = MWAVES * rr + wave;
        const int cj = pool_cnt[jj];
        if (cj + NS > a.pool) {
          uint64_t* pool = pools + (size_t)jj * a.pool;
          const int nc = wave_pool_compact(pool, a.pool, cj, a.k, lane);
          if (lane == 0) {
            pool_cnt[jj] = nc;
            if (nc >= a.k) pool_kth[jj] = pool[a.k - 1];
          }
          wave_sync();
        }
      }
    }
    wave_sync();
    if (lane == 0) s_list_cnt[wave] = 0;
  };

  // pools that could not take `room` more keys (lane jj looks at pool jj); wave-uniform
  auto full_pools = [&](int room) -> uint32_t {
    return (uint32_t)__ballot(lane < QM && pool_cnt[min(lane, QM - 1)] + room > a.pool);
  };
  int round = 0;
  for (int tb = ts; tb < t1; tb += MWAVES, round ^= 1) {
    // Every wavefront is past the previous round's barrier here, but a faster one may already be filing this
    // round's survivors, so the counters a slower one reads can be ahead of what its siblings saw: the decision to
    // flush / compact (which contains barriers) is therefore agreed upon, not taken by each wavefront for itself.
    // The slot of the other parity was last read before the previous barrier and is reset for the next round.
    if (tid == 0) s_agree[round ^ 1] = AGREE_UNSET;
    if (F > 0) {
      int longest = 0;
      for (int ww = 0; ww < MWAVES; ++ww) longest = max(longest, s_list_cnt[ww]);
      if (wave_agree(&s_agree[round], longest > MLIST_FLUSH ? 1u : 0u, lane)) {
        flush_own();
        __syncthreads();
      }
    } else {
      const uint32_t mask = wave_agree(&s_agree[round], full_pools(MWAVES * TILE), lane);
      if (mask) block_compact(mask);
    }
    const int tile = tb + wave;
    if (tile < t1) {
      // the factors of the lane's four vectors are requested with the code words, ahead of the matrix
      // instructions (fetched where they are used, each column block would wait for its own three loads)
      float fa4[4], fr4[4], fe4[4];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int v = 16 * cb + lj;
        fa4[cb] = a.short_factors[((int64_t)tile * 3 + 0) * TILE + v];
        fr4[cb] = a.short_factors[((int64_t)tile * 3 + 1) * TILE + v];
        fe4[cb] = a.short_factors[((int64_t)tile * 3 + 2) * TILE + v];
      }
      // inner products: 4 column blocks of 16 vectors x 16 queries
      v4i acc[4];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        acc[cb] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          const int w = 2 * kc + (g >> 1);
          uint32_t word = 0u;
          if (w < W) word = a.short_codes[((int64_t)tile * W + w) * TILE + 16 * cb + lj];
          const v4i xb = expand_half(word, g & 1);
          acc[cb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa[kc], xb, acc[cb], 0, 0, 0);
        }
      }
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        fa4[cb] = pinned(fa4[cb]);
        fr4[cb] = pinned(fr4[cb]);
        fe4[cb] = pinned(fe4[cb]);
      }
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int v = 16 * cb + lj;
        const float fa = fa4[cb], fr = fr4[cb], fe = fe4[cb];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int I = acc[cb][r];
          if (DBG) {
            if (4 * g + r < np) a.dbg_ip[a.dbg_off[pbeg + 4 * g + r] + (int64_t)(tile - t0) * TILE + v] = I;
          }
          const float x = fmaf(al[r], (float)I, -be[r]);  // delta * (I - S/2)
          const float e1 = fmaf(fr, x, fa + Gr[r]);
          const float filt = (F > 0) ? fmaf(-fe, Er[r], e1) : e1;
          if (filt <= tr[r]) {
            const int j = 4 * g + r;
            if (F == 0) {  // B == 1: the 1-bit estimate is the final key
              const uint64_t key = make_key(e1, (uint32_t)a.ids[(int64_t)tile * TILE + v]);
              if (key <= pool_kth[j]) pools[(size_t)j * a.pool + atomicAdd(&pool_cnt[j], 1)] = key;
            } else {       // file the survivor with the owner of query j (= wavefront r % MWAVES)
              const int pos = atomicAdd(&s_list_cnt[r % MWAVES], 1);
              lists[(size_t)(r % MWAVES) * MLIST_CAP + pos] = ((uint32_t)j << 28) | (uint32_t)((tile - t0) * TILE + v);
            }
          }
        }
      }
    }
    __syncthreads();
  }
  if (F > 0) {
    flush_own();
    __syncthreads();
  }
  // a pool larger than the output region, or any pool of a split cluster, is cut to its k best
  // (every wavefront is past a barrier and nothing is being added any more: all see the same counters)
  block_compact(full_pools(nseg > 1 ? a.pool - a.k : a.pool - a.cand_stride));
  // every pair reserves its part of the candidate region at once (one atomic per pair, all in flight together);
  // the wavefronts then copy the pools out, a pair each
  if (tid < np) {
    const int cj = pool_cnt[tid];
    const int pp = a.pair_ids[pbeg + tid];
    qidx[tid] = pp;  // the query indices are no longer needed
    s_out[tid] = cj > 0 ? atomicAdd(&a.cand_cnt[pp], cj) : 0;
  }
  __syncthreads();
  for (int j = wave; j < np; j += MWAVES) {
    const uint64_t* pool = pools + (size_t)j * a.pool;
    const int cj = pool_cnt[j], base = s_out[j];
    const int64_t pp = qidx[j];
    for (int e = lane; e < cj; e += 64) a.cand_keys[pp * a.cand_stride + base + e] = pool[e];
  }
}

// ---------------------------------------------------------------------------------
// Instantiations.  This file is compiled once per RQ_PART; each part holds the kernels
// of a few code widths W = dim/32 so that the parts build in parallel.
// ---------------------------------------------------------------------------------
#ifndef RQ_PART
#error "compile with -DRQ_PART=0..2"
#endif
#if RQ_PART == 0
#define RQ_W_LIST(X) X(1) X(2) X(3) X(4)
#define RQ_PART_NAME(f) f##_part0
#elif RQ_PART == 1
#define RQ_W_LIST(X) X(8) X(16) X(24)
#define RQ_PART_NAME(f) f##_part1
#else
#define RQ_W_LIST(X) X(30) X(32)
#define RQ_PART_NAME(f) f##_part2
#endif

template <int W, int F>
static void launch_seed_wf(const ScanArgs& a, int impl, int64_t nq, hipStream_t st) {
  const int kpad = next_pow2(std::max(a.k, SEED_M));
  const size_t smem = (size_t)(SEED_CHUNK_TILES * TILE + 2 * kpad) * sizeof(uint64_t) + (size_t)a.D * sizeof(float);
  if (impl == 2)
    hipLaunchKernelGGL((seed_kernel<W, F, 1>), dim3((unsigned)nq), dim3(256), smem + (size_t)W * 256, st, a);
  else if (a.k <= 64 && nq <= 2048)  // few queries: four wavefronts per query
    hipLaunchKernelGGL((seed_wave_kernel<W, F, true>), dim3((unsigned)((nq + 7) / 8 * 8)), dim3(256), 0, st, a, nq);
  else if (a.k <= 64)
    hipLaunchKernelGGL((seed_wave_kernel<W, F, false>), dim3((unsigned)(((nq + 3) / 4 + 7) / 8 * 8)), dim3(256), 0, st, a,
                       nq);
  else
    hipLaunchKernelGGL((seed_kernel<W, F, 0>), dim3((unsigned)nq), dim3(256), smem, st, a);
}

template <int W, int F>
static void launch_scan_mfma_wf(const ScanArgs& a, unsigned grid, bool dbg, hipStream_t st) {
  constexpr int MWAVES = mfma_waves(W), MLIST_CAP = mlist_cap(MWAVES);
  const size_t smem = (size_t)QM * a.pool * sizeof(uint64_t) +
                      QM * (sizeof(uint64_t) + 2 * sizeof(float) + 2 * sizeof(int)) + (MWAVES + QM + 2) * sizeof(int) +
                      (F > 0 ? (size_t)MWAVES * MLIST_CAP * sizeof(uint32_t) : 0);
  if (dbg)
    hipLaunchKernelGGL((scan_mfma_kernel<W, F, true>), dim3(grid), dim3(64 * MWAVES), smem, st, a);
  else
    hipLaunchKernelGGL((scan_mfma_kernel<W, F, false>), dim3(grid), dim3(64 * MWAVES), smem, st, a);
}

template <int W, int F, int M>
static void launch_scan_wf(const ScanArgs& a, unsigned grid, bool dbg, hipStream_t st) {
  const bool masked = M == 0 && F > 0 && a.surv_mask != nullptr;  // second half of the split search
  const bool stream = M == 0 && a.streaming && !masked;
  const int qn = stream ? 1 : QW;  // pairs per work item
  const size_t smem = (size_t)qn * a.pool * sizeof(uint64_t) + qn * (sizeof(uint64_t) + 2 * sizeof(float) + sizeof(int)) +
                      (F > 0 ? (masked ? LIST_CAP_MASKED : LIST_CAP) * sizeof(uint32_t) +
                                   (size_t)qn * (a.D + 4 * RefineShape<W * (F > 0 ? F : 8)>::G) * sizeof(float) : 0) +
                      (M == 1 ? (size_t)qn * W * 256 : 0);
  if (masked)  // (estimate_mfma_kernel ran)
    hipLaunchKernelGGL((scan_kernel<W, F, false, M, 0, (M == 0 && F > 0)>), dim3(grid), dim3(64), smem, st, a);
  else if (stream && F == 0 && dbg)
    hipLaunchKernelGGL((scan_stream_kernel<W, true>), dim3(grid), dim3(64), smem, st, a);
  else if (stream && F == 0)
    hipLaunchKernelGGL((scan_stream_kernel<W, false>), dim3(grid), dim3(64), smem, st, a);
  else if (stream && dbg)
    hipLaunchKernelGGL((scan_stream_long_kernel<W, F, true>), dim3(grid), dim3(64), smem, st, a);
  else if (stream)
    hipLaunchKernelGGL((scan_stream_long_kernel<W, F, false>), dim3(grid), dim3(64), smem, st, a);
  else if (dbg)
    hipLaunchKernelGGL((scan_kernel<W, F, true, M>), dim3(grid), dim3(64), smem, st, a);
  else
    hipLaunchKernelGGL((scan_kernel<W, F, false, M>), dim3(grid), dim3(64), smem, st, a);
}

template <int W>
static void seed_by_f(const ScanArgs& a, int F, int impl, int64_t nq, hipStream_t st) {
  switch (F) {
    case 0: launch_seed_wf<W, 0>(a, impl, nq, st); break;
    case 2: launch_seed_wf<W, 2>(a, impl, nq, st); break;
    case 4: launch_seed_wf<W, 4>(a, impl, nq, st); break;
    default: launch_seed_wf<W, 8>(a, impl, nq, st); break;
  }
}

template <int W>
static void scan_by_f(const ScanArgs& a, int F, int impl, unsigned grid, bool dbg, hipStream_t st) {
  if (impl == 1) {
    switch (F) {
      case 0: launch_scan_mfma_wf<W, 0>(a, grid, dbg, st); break;
      case 2: launch_scan_mfma_wf<W, 2>(a, grid, dbg, st); break;
      case 4: launch_scan_mfma_wf<W, 4>(a, grid, dbg, st); break;
      default: launch_scan_mfma_wf<W, 8>(a, grid, dbg, st); break;
    }
    return;
  }
  if (impl == 2) {
    switch (F) {
      case 0: launch_scan_wf<W, 0, 1>(a, grid, dbg, st); break;
      case 2: launch_scan_wf<W, 2, 1>(a, grid, dbg, st); break;
      case 4: launch_scan_wf<W, 4, 1>(a, grid, dbg, st); break;
      default: launch_scan_wf<W, 8, 1>(a, grid, dbg, st); break;
    }
    return;
  }
  switch (F) {
    case 0: launch_scan_wf<W, 0, 0>(a, grid, dbg, st); break;
    case 2: launch_scan_wf<W, 2, 0>(a, grid, dbg, st); break;
    case 4: launch_scan_wf<W, 4, 0>(a, grid, dbg, st); break;
    default: launch_scan_wf<W, 8, 0>(a, grid, dbg, st); break;
  }
}

// Return false when W is not one of this part's widths.
bool RQ_PART_NAME(seed)(const ScanArgs& a, int W, int F, int impl, int64_t nq, hipStream_t st) {
  switch (W) {
#define RQ_X(W_) case W_: seed_by_f<W_>(a, F, impl, nq, st); return true;
    RQ_W_LIST(RQ_X)
#undef RQ_X
    default: return false;
  }
}

template <int W>
static void small_by_f(const ScanArgs& a, const SmallSelectArgs& b, int F, hipStream_t st) {
  const dim3 grid((unsigned)b.lists.nq), blk(256);
  switch (F) {
    case 0: hipLaunchKernelGGL((small_select_seed_kernel<W, 0>), grid, blk, 0, st, a, b); break;
    case 2: hipLaunchKernelGGL((small_select_seed_kernel<W, 2>), grid, blk, 0, st, a, b); break;
    case 4: hipLaunchKernelGGL((small_select_seed_kernel<W, 4>), grid, blk, 0, st, a, b); break;
    default: hipLaunchKernelGGL((small_select_seed_kernel<W, 8>), grid, blk, 0, st, a, b); break;
  }
}

bool RQ_PART_NAME(small)(const ScanArgs& a, const SmallSelectArgs& b, int W, int F, hipStream_t st) {
  switch (W) {
#define RQ_X(W_) case W_: small_by_f<W_>(a, b, F, st); return true;
    RQ_W_LIST(RQ_X)
#undef RQ_X
    default: return false;
  }
}

bool RQ_PART_NAME(scan)(const ScanArgs& a, int W, int F, int impl, unsigned grid, bool dbg, hipStream_t st) {
  switch (W) {
#define RQ_X(W_) case W_: scan_by_f<W_>(a, F, impl, grid, dbg, st); return true;
    RQ_W_LIST(RQ_X)
#undef RQ_X
    default: return false;
  }
}

#if defined(RQ_TIMELINE)
extern "C" int RQ_PART_NAME(rabitq_debug_timeline)(unsigned long long* out) {
  return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_timeline), sizeof(g_timeline)) == hipSuccess ? 0 : -3;
}
#endif
#if defined(RQ_STATS)
// development only: one counter block per translation unit (part), summed by the caller
extern "C" int RQ_PART_NAME(rabitq_debug_scan_stats)(unsigned long long* out, int reset) {
  if (hipMemcpyFromSymbol(out, HIP_SYMBOL(g_scan_stats), sizeof(g_scan_stats)) != hipSuccess) return -3;
  if (reset) {
    unsigned long long z[8] = {0};
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_scan_stats), z, sizeof(z)) != hipSuccess) return -3;
  }
  return 0;
}
#endif

}  // namespace rq
