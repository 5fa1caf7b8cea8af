// Host-side launchers of the seeding and scan kernels: argument block, work-item
// offsets, and routing to the translation unit that holds the kernels for W = dim/32.
#include <algorithm>
#include <functional>

#include "rq_internal.h"
#include "rq_scan_args.h"
#include "rq_small_batch.h"

namespace rq {

// ---------------------------------------------------------------------------------
// item_off[c] = first work item of cluster c; a work item is qw consecutive pairs of
// one cluster times one segment of its tiles.  (One workgroup.)
// ---------------------------------------------------------------------------------
__global__ void zero_i32_kernel(int32_t* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// item16 != nullptr (split search): also item16[c] = first work item of cluster c when an item is 16 pairs times one
// segment, and mask_off[c] = first block of survivor bits of cluster c (a block per group of 16 pairs and tile).
__global__ __launch_bounds__(256) void item_offsets_kernel(const int32_t* __restrict__ pair_off,
                                                          const int32_t* __restrict__ tile_off,
                                                          const int32_t* __restrict__ order, int n, int qw, int tseg,
                                                          int segmax, int32_t* __restrict__ item_off,
                                                          int32_t* __restrict__ item16, uint32_t* __restrict__ mask_off) {
  __shared__ uint32_t part[3][256];
  const int tid = threadIdx.x;
  const int per = (n + 255) / 256;
  const int s = tid * per, e = min(n, s + per);
  // (entry i is about cluster i, or about the i-th longest cluster when an order is given)
  auto counts = [&](int r, uint32_t& it, uint32_t& i16, uint32_t& mb) {
    const int i = order ? order[r] : r;
    const uint32_t pairs = (uint32_t)(pair_off[i + 1] - pair_off[i]), tiles = (uint32_t)(tile_off[i + 1] - tile_off[i]);
    const uint32_t nseg = (uint32_t)seg_count((int)tiles, tseg, segmax), groups = (pairs + QM - 1) / QM;
    it = ((pairs + qw - 1) / qw) * nseg;
    i16 = groups * nseg;
    mb = groups * tiles;
  };
  uint32_t sum[3] = {0, 0, 0};
  for (int i = s; i < e; ++i) {
    uint32_t a, b, c;
    counts(i, a, b, c);
    sum[0] += a; sum[1] += b; sum[2] += c;
  }
  const int nscan = item16 ? 3 : 1;
  for (int v = 0; v < nscan; ++v) part[v][tid] = sum[v];
  __syncthreads();
  for (int d = 1; d < 256; d <<= 1) {
    uint32_t o[3];
    for (int v = 0; v < nscan; ++v) o[v] = (tid >= d) ? part[v][tid - d] : 0u;
    __syncthreads();
    for (int v = 0; v < nscan; ++v) part[v][tid] += o[v];
    __syncthreads();
  }
  uint32_t run[3];
  for (int v = 0; v < nscan; ++v) run[v] = part[v][tid] - sum[v];
  for (int i = s; i < e; ++i) {
    uint32_t a, b, c;
    counts(i, a, b, c);
    item_off[i] = (int32_t)run[0];
    run[0] += a;
    if (item16) {
      item16[i] = (int32_t)run[1];
      mask_off[i] = run[2];
      run[1] += b; run[2] += c;
    }
  }
  if (tid == 255) {
    item_off[n] = (int32_t)part[0][255];
    if (item16) {
      item16[n] = (int32_t)part[1][255];
      mask_off[n] = part[2][255];
    }
  }
}

// One wavefront per cluster writes the descriptors of its work items of QW pairs (split search).
__global__ __launch_bounds__(64) void item_desc_kernel(const int32_t* __restrict__ pair_off, const int32_t* __restrict__ tile_off,
                                                      const int32_t* __restrict__ item_off, const uint32_t* __restrict__ mask_off,
                                                      int tseg, int segmax, ItemDesc* __restrict__ desc) {
  const int c = blockIdx.x;
  const int i0 = item_off[c], n = item_off[c + 1] - i0;
  if (n <= 0) return;
  const int t0 = tile_off[c], tiles = tile_off[c + 1] - t0;
  const int p0 = pair_off[c], cnt = pair_off[c + 1] - p0;
  const int nseg = seg_count(tiles, tseg, segmax);
  const int seglen = (tiles + nseg - 1) / nseg;
  const uint32_t m0 = mask_off[c];
  for (int it = threadIdx.x; it < n; it += 64) {
    const int grp = it / nseg, sidx = it - grp * nseg;
    ItemDesc d;
    d.pbeg = p0 + grp * QW;
    d.np_mg = min(QW, cnt - grp * QW) | ((grp & 3) << 8);
    d.t0 = t0;
    d.ts = t0 + sidx * seglen;
    d.te = min(t0 + tiles, d.ts + seglen);
    d.nseg = nseg;
    d.mblock = m0 + (uint32_t)((grp >> 2) * tiles + sidx * seglen);
    d.pad = 0;
    desc[i0 + it] = d;
  }
}

// One wavefront per entry r of the item table (cluster order[r], or cluster r without an order) writes the descriptors
// of its work items of one pair (prefetching variant of the popcount kernel).
__global__ __launch_bounds__(64) void stream_desc_kernel(ScanArgs a, StreamDesc* __restrict__ desc) {
  const int r = blockIdx.x;
  const int i0 = a.item_off[r], n = a.item_off[r + 1] - i0;
  if (n <= 0) return;
  const int c = a.order ? a.order[r] : r;
  const int t0 = a.tile_off[c], tiles = a.tile_off[c + 1] - t0;
  const int p0 = a.pair_off[c];
  const int nseg = seg_count(tiles, a.tseg, a.segmax);
  const int seglen = (tiles + nseg - 1) / nseg;
  for (int it = threadIdx.x; it < n; it += 64) {
    const int pi = it / nseg, sidx = it - pi * nseg;
    const int pp = a.pair_ids[p0 + pi];
    const int q = pair_query(a, pp);
    StreamDesc d{};
    d.pp = pp;
    d.q = q;
    d.t0 = t0;
    d.ts = t0 + sidx * seglen;
    d.te = min(t0 + tiles, d.ts + seglen);
    d.nseg = nseg;
    d.ppos = p0 + pi;
    d.S = a.sum_qhat[q];
    d.G = a.probe_G[pp];
    d.E = a.probe_E[pp];
    d.delta = a.delta[q];
    d.sumq = a.sum_q[q];
    desc[i0 + it] = d;
  }
}

// segments per cluster, sorted, for the work-item bound of a launch (cached per segment length and limit)
static void update_seg_cache(const rabitq_index* ix, int tseg, int segmax) {
  std::vector<int>& nseg = ix->seg_sorted;
  if (ix->seg_sorted_max == segmax && ix->seg_sorted_tseg == tseg) return;
  nseg.resize(ix->host_tiles.size());
  for (size_t c = 0; c < nseg.size(); ++c) nseg[c] = seg_count(ix->host_tiles[c], tseg, segmax);
  std::sort(nseg.begin(), nseg.end(), std::greater<int>());
  ix->seg_sorted_max = segmax;
  ix->seg_sorted_tseg = tseg;
  ix->seg_total = 0;
  for (int v : nseg) ix->seg_total += v;
}

// Work-item bound.  Cluster c with cnt_c pairs and nseg_c segments has ceil(cnt_c / per_item) * nseg_c work items, at
// most (cnt_c / per_item + 1) * nseg_c.  Every query probes nprobe distinct clusters, so cnt_c <= nq and sum cnt_c =
// nq * nprobe: the sum is largest when the nprobe clusters with the most segments are probed by every query.
static int64_t item_bound(const rabitq_index* ix, int64_t nq, int nprobe, int per_item) {
  const std::vector<int>& nseg = ix->seg_sorted;
  int64_t top = 0;
  for (int i = 0; i < nprobe && i < (int)nseg.size(); ++i) top += nseg[i];
  const int64_t m = ix->seg_total + (nq * top + per_item - 1) / per_item;
  return ((m + 7) / 8) * 8;
}

int64_t split_mask_blocks(rabitq_index* ix, int64_t nq, int nprobe) {
  if (ix->tiles_prefix.empty()) {
    std::vector<int> t(ix->host_tiles.begin(), ix->host_tiles.end());
    std::sort(t.begin(), t.end(), std::greater<int>());
    ix->tiles_prefix.assign(t.size() + 1, 0);
    for (size_t i = 0; i < t.size(); ++i) ix->tiles_prefix[i + 1] = ix->tiles_prefix[i] + t[i];
  }
  const size_t top = std::min<size_t>((size_t)nprobe, ix->tiles_prefix.size() - 1);
  return (nq * ix->tiles_prefix[top] + QM - 1) / QM + ix->n_tiles;
}

// few pairs per list, popcount kernel, not split: the shape the prefetching variant is for
static bool stream_shape(const rabitq_index* ix, int64_t nq, int nprobe) {
  return effective_impl(ix) == 0 && nq * nprobe <= 4 * (int64_t)ix->nlist && !split_wanted(ix, nq, nprobe);
}
static ScanPlan plan_for(const rabitq_index* ix, int64_t nq, int nprobe, int k, bool streaming);
// descriptor slots (of sizeof(ItemDesc)) the prefetching variant needs for (nq, nprobe, k)
// work items of one pair: a pair has as many as its list has segments, at most those of the longest list
static int64_t stream_item_bound(const rabitq_index* ix, int64_t nq, int nprobe, const ScanPlan& plan) {
  const int64_t m = nq * nprobe * seg_count(ix->max_tiles, plan.tseg, plan.segmax);
  return ((m + 7) / 8) * 8;
}
static int64_t stream_desc_slots(const rabitq_index* ix, int64_t nq, int nprobe, int k) {
  return stream_item_bound(ix, nq, nprobe, plan_for(ix, nq, nprobe, k, true)) *
         (int64_t)(sizeof(StreamDesc) / sizeof(ItemDesc));
}

int ensure_stream_buffers(rabitq_index* ix, int64_t nq, int nprobe, int k) {
  if (!stream_shape(ix, nq, nprobe)) return RABITQ_OK;
  const int64_t slots = stream_desc_slots(ix, nq, nprobe, k);
  if (slots <= ix->item_desc_cap || slots > 0x7fffffff) return RABITQ_OK;
  RQ_HIP(hipDeviceSynchronize());
  if (ix->item_desc) (void)hipFree(ix->item_desc);
  ix->item_desc = nullptr;
  ix->item_desc_cap = 0;
  RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->item_desc), (size_t)slots * sizeof(ItemDesc)));
  ix->item_desc_cap = slots;
  return RABITQ_OK;
}

int ensure_split_buffers(rabitq_index* ix, int64_t nq, int nprobe, int k) {
  const int64_t need = split_mask_blocks(ix, nq, nprobe);
  const ScanPlan plan = scan_plan(ix, nq, nprobe, k);
  update_seg_cache(ix, plan.tseg, plan.segmax);
  const int64_t items = item_bound(ix, nq, nprobe, QW);
  if (need <= ix->surv_mask_blocks && items <= ix->item_desc_cap) return RABITQ_OK;
  if (need >= ((int64_t)1 << 32) || items > 0x7fffffff) return RABITQ_OK;  // beyond 32-bit offsets: the search is not split
  RQ_HIP(hipDeviceSynchronize());
  if (need > ix->surv_mask_blocks) {
    if (ix->surv_mask) (void)hipFree(ix->surv_mask);
    ix->surv_mask = nullptr;
    ix->surv_mask_blocks = 0;
    RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->surv_mask), (size_t)need * 16 * sizeof(uint64_t)));
    ix->surv_mask_blocks = need;
  }
  if (items > ix->item_desc_cap) {
    if (ix->item_desc) (void)hipFree(ix->item_desc);
    ix->item_desc = nullptr;
    ix->item_desc_cap = 0;
    RQ_HIP(hipMalloc(reinterpret_cast<void**>(&ix->item_desc), (size_t)items * sizeof(ItemDesc)));
    ix->item_desc_cap = items;
  }
  return RABITQ_OK;
}

__global__ __launch_bounds__(1024) void small_batch_lists_kernel(SmallListArgs b) {
  __shared__ uint32_t s_pairs[1024], s_items[1024];
  small_lists_body<1024>(b, s_pairs, s_items);
}

static int field_bits(int B) {  // long-code field width: B rounded up to 2, 4, 8 (0: no long code)
  if (B <= 1) return 0;
  if (B <= 2) return 2;
  if (B <= 4) return 4;
  return 8;
}

static int next_pow2_host(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

static ScanArgs base_args(const rabitq_index* ix) {
  ScanArgs a{};
  a.short_codes = ix->short_codes;
  a.short_factors = ix->short_factors;
  a.long_codes = ix->long_codes;
  a.long_factors = ix->long_factors;
  a.ids = ix->ids;
  a.tile_off = ix->tile_off;
  a.cluster_size = ix->cluster_size;
  a.D = ix->dim;
  a.B = ix->total_bits;
  a.LW = ix->LW;
  a.nlist = ix->nlist;
  a.cB = (float)(((1 << ix->total_bits) - 1) * 0.5);
  a.qerr = effective_impl(ix) == 2 ? 0.f : (float)((ix->dim - 1.0) / (12.0 * (1.0 - 2.0 / 3.14159265358979323846)));
  return a;
}

static int bad_width() {
  set_error("dim/32 must be one of 1,2,3,4,8,16,24,30,32 in this build");
  return RABITQ_EINVAL;
}

static void set_repr(ScanArgs& a, const rabitq_index* ix, const rabitq_query_repr& r) {
  a.q_stage = r.q_stage; a.qhat8 = r.qhat8; a.Dp = qhat_stride(ix->dim);
  a.planes = r.planes; a.delta = r.delta; a.sum_qhat = r.sum_qhat; a.sum_q = r.sum_q; a.lut = r.lut;
}

static int need_lut(const rabitq_index* ix, const rabitq_query_repr& r) {
  if (ix->scan_impl == 2 && r.lut == nullptr) {
    set_error("scan_impl 2 needs the lookup tables (rabitq_query_repr.lut)");
    return RABITQ_EINVAL;
  }
  return RABITQ_OK;
}

int launch_clear_counters(int32_t* cand_cnt, int64_t n, hipStream_t st) {
  if (n <= 0) return RABITQ_OK;
  hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 4096)), dim3(256), 0, st, cand_cnt, n);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

int launch_seed(const rabitq_index* ix, const rabitq_query_repr& repr, const int32_t* probe_ids, const float* probe_G,
                const float* probe_E, int64_t nq, int k, int nprobe, float* tau, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  if (int rc = need_lut(ix, repr)) return rc;
  ScanArgs a = base_args(ix);
  set_repr(a, ix, repr);
  a.probe_ids = probe_ids; a.probe_G = probe_G; a.probe_E = probe_E;
  set_nprobe(a, nprobe); a.k = k; a.tau_out = tau;
  const int W = ix->W, F = field_bits(ix->total_bits);
  const int impl = effective_impl(ix);
  if (!(seed_part0(a, W, F, impl, nq, st) || seed_part1(a, W, F, impl, nq, st) || seed_part2(a, W, F, impl, nq, st)))
    return bad_width();
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

// Long clusters are scanned in segments of about tseg tiles by separate work items; each segment of a split cluster
// contributes at most k keys to the pair's region of cand_stride keys (cand_cnt is advanced atomically).  The segment
// length adapts to the batch: a large batch has more work items than the chip has wavefront slots and keeps long
// segments (32 tiles); a small batch is cut finer, down to 2 tiles, so that about 4096 items exist.
static ScanPlan plan_for(const rabitq_index* ix, int64_t nq, int nprobe, int k, bool streaming) {
  ScanPlan p;
  p.streaming = streaming;
  p.qw = effective_impl(ix) == 1 ? QM : (p.streaming ? 1 : QW);
  const int64_t np_all = nq * nprobe;
  const int64_t est_items = std::min<int64_t>(np_all, (np_all + p.qw - 1) / p.qw + ix->nlist);
  const int64_t avg_tiles = std::max<int64_t>(1, ix->n_tiles / std::max(1, ix->nlist));
  p.tseg = (int)std::min<int64_t>(32, std::max<int64_t>(2, est_items * avg_tiles / 4096));
  if (ix->seg_tiles > 0) p.tseg = ix->seg_tiles;
  p.segmax = std::max(1, next_pow2_host(k + TILE) / k);
  return p;
}

// Few pairs per list: every list is read from memory about once, by the prefetching variant of the popcount kernel,
// whose work items are single pairs with a descriptor each (never together with the split search, whose items are
// groups of pairs).  Taken when the handle's descriptor memory is large enough (ensure_stream_buffers, called by the
// entry points that may allocate); otherwise the general kernel does the same work.
ScanPlan scan_plan(const rabitq_index* ix, int64_t nq, int nprobe, int k) {
  const bool streaming = stream_shape(ix, nq, nprobe) && ix->item_desc != nullptr &&
                         stream_desc_slots(ix, nq, nprobe, k) <= ix->item_desc_cap;
  return plan_for(ix, nq, nprobe, k, streaming);
}

static SmallListArgs small_list_args(const rabitq_index* ix, const int32_t* probe_ids, int64_t nq, int nprobe, int k,
                                     int32_t* pair_off, int32_t* pair_ids, uint32_t* scratch, int32_t* cand_cnt) {
  const ScanPlan p = scan_plan(ix, nq, nprobe, k);
  SmallListArgs b{};
  b.probe_ids = probe_ids; b.nq = (int)nq; b.nprobe = nprobe; b.nlist = ix->nlist; b.tile_off = ix->tile_off;
  b.qw = p.qw; b.tseg = p.tseg; b.segmax = p.segmax; b.mask = scratch; b.pair_off = pair_off; b.pair_ids = pair_ids;
  b.item_off = ix->tile_off + (ix->nlist + 1); b.cand_cnt = cand_cnt;
  b.desc = nullptr;
  return b;
}

int launch_small_batch_lists(const rabitq_index* ix, const int32_t* probe_ids, int64_t nq, int nprobe, int k,
                             int32_t* pair_off, int32_t* pair_ids, uint32_t* scratch, int32_t* cand_cnt, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  if (nq > SMALL_BATCH_MAX) { set_error("small-batch list builder: more than 64 queries"); return RABITQ_EINVAL; }
  const SmallListArgs b = small_list_args(ix, probe_ids, nq, nprobe, k, pair_off, pair_ids, scratch, cand_cnt);
  hipLaunchKernelGGL(small_batch_lists_kernel, dim3(1), dim3(1024), 0, st, b);
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

int launch_small_select_seed(const rabitq_index* ix, const rabitq_query_repr& repr, const float* scores, int64_t nq, int k,
                             int nprobe, int32_t* probe_ids, float* probe_G, float* probe_E, float* tau, int32_t* pair_off,
                             int32_t* pair_ids, uint32_t* scratch, int32_t* cand_cnt, hipStream_t st) {
  if (nq <= 0) return RABITQ_OK;
  if (nq > SMALL_BATCH_MAX || nprobe > 64 || k > 64 || effective_impl(ix) == 2) {
    set_error("fused selection + seeding: needs at most 64 queries, nprobe <= 64, k <= 64 and a bitwise scan");
    return RABITQ_EINVAL;
  }
  ScanArgs a = base_args(ix);
  set_repr(a, ix, repr);
  a.probe_ids = probe_ids; a.probe_G = probe_G; a.probe_E = probe_E;
  set_nprobe(a, nprobe); a.k = k; a.tau_out = tau;
  SmallSelectArgs b{};
  b.scores = scores; b.sq_norm = repr.sq_norm; b.centroid_sq = ix->centroid_sq; b.metric = ix->metric;
  // (with one probed list and 1-bit codes the scan's own top-k selects what a seeded threshold would: no seeding)
  b.do_seed = (ix->prune && !(nprobe == 1 && ix->total_bits == 1)) ? 1 : 0;
  b.probe_ids = probe_ids; b.probe_G = probe_G; b.probe_E = probe_E;
  b.ticket = ix->tile_off + 2 * (ix->nlist + 1);
  b.lists = small_list_args(ix, probe_ids, nq, nprobe, k, pair_off, pair_ids, scratch, cand_cnt);
  if (scan_plan(ix, nq, nprobe, k).streaming) {
    // (the workgroup that builds the lists also writes the descriptors of the prefetching scan's work items)
    b.lists.desc = reinterpret_cast<StreamDesc*>(ix->item_desc);
    b.lists.probe_G = probe_G; b.lists.probe_E = probe_E;
    b.lists.delta = repr.delta; b.lists.sum_q = repr.sum_q; b.lists.sum_qhat = repr.sum_qhat;
  }
  const int W = ix->W, F = field_bits(ix->total_bits);
  if (!(small_part0(a, b, W, F, st) || small_part1(a, b, W, F, st) || small_part2(a, b, W, F, st))) return bad_width();
  RQ_HIP(hipGetLastError());
  return RABITQ_OK;
}

int launch_scan(const rabitq_index* ix, const rabitq_query_repr& repr, const float* probe_G, const float* probe_E,
                const int32_t* pair_off, const int32_t* pair_ids, const float* tau, int64_t nq, int k, int nprobe,
                uint64_t* cand_keys, int32_t* cand_cnt, int32_t* dbg_ip, const int64_t* dbg_off, const ScanStreams& ss) {
  if (nq <= 0) return RABITQ_OK;
  const hipStream_t st = ss.main, sst = ss.setup;
  if (int rc = need_lut(ix, repr)) return rc;
  ScanArgs a = base_args(ix);
  set_repr(a, ix, repr);
  const int impl = effective_impl(ix);
  const ScanPlan plan = scan_plan(ix, nq, nprobe, k);
  const int qw = plan.qw;
  a.probe_G = probe_G; a.probe_E = probe_E; a.pair_off = pair_off; a.pair_ids = pair_ids; a.tau = tau;
  set_nprobe(a, nprobe); a.k = k;
  a.cand_stride = next_pow2_host(k + TILE);
  // LDS pool entries per pair: the popcount kernel may append a whole tile at once
  // (the matrix-core kernel's four wavefronts may together append 4 x 16 refined keys per round, or four whole
  // tiles when there is no long code)
  a.pool = next_pow2_host(k + TILE);
  if (impl == 1 && ix->total_bits == 1) a.pool = next_pow2_host(k + 4 * TILE);

  a.cand_keys = cand_keys; a.cand_cnt = cand_cnt; a.dbg_ip = dbg_ip; a.dbg_off = dbg_off;
  // work-item offsets live in the second half of the tile_off allocation (owned by the handle)
  int32_t* item_off = ix->tile_off + (ix->nlist + 1);
  a.item_off = item_off;
  a.tseg = plan.tseg;
  a.segmax = plan.segmax;
  a.streaming = plan.streaming ? 1 : 0;
  // Few pairs per list: the lists are read from memory about once each and a work item lasts as long as its list is
  // long, so the launch ends when its last long item does.  Handing the items out longest list first leaves the short
  // ones for the end (the popcount kernel's own item table only: the small-batch builder and the split search keep
  // cluster order, where items of one cluster share a cache).
  if (a.streaming && !ss.setup_done && ix->longest_first && ix->cluster_order != nullptr) a.order = ix->cluster_order;
  // Split search: the estimates of groups of 16 pairs on the matrix cores, then this kernel's refinement only.
  // Chosen when asked for (scan_impl 4), built for the index, worth it for the batch, and the handle's buffer of
  // survivor bits is large enough (ensure_split_buffers, called by the entry points that may allocate).
  if (!a.streaming) update_seg_cache(ix, a.tseg, a.segmax);
  const int64_t max_items = a.streaming ? stream_item_bound(ix, nq, nprobe, plan) : item_bound(ix, nq, nprobe, qw);
  const bool split = split_wanted(ix, nq, nprobe) && ix->surv_mask != nullptr && ix->item_desc != nullptr &&
                     split_mask_blocks(const_cast<rabitq_index*>(ix), nq, nprobe) <= ix->surv_mask_blocks &&
                     max_items <= ix->item_desc_cap;
  ss.split = split;
  ss.streamed = a.streaming != 0;
  int32_t* item16 = ix->tile_off + 2 * (ix->nlist + 1) + TICKET_WORDS;
  uint32_t* mask_off = reinterpret_cast<uint32_t*>(item16 + (ix->nlist + 1));
  if (ss.setup_b) RQ_HIP(hipEventRecord(ss.setup_b, sst));
  // (one launch for the item table and, when the search is split, the two tables of its first half; a small batch's
  // list builder has written the item table already, with the same values)
  if (!ss.setup_done || split)
    hipLaunchKernelGGL(item_offsets_kernel, dim3(1), dim3(256), 0, sst, pair_off, ix->tile_off, a.order, ix->nlist, qw,
                       a.tseg, a.segmax, item_off, split ? item16 : nullptr, split ? mask_off : nullptr);
  if (!ss.setup_done && !ss.counters_clear) {
    if (int rc = launch_clear_counters(cand_cnt, nq * nprobe, sst)) return rc;
  }
  if (a.streaming) a.stream_desc = reinterpret_cast<const StreamDesc*>(ix->item_desc);
  if (a.streaming && !ss.desc_done) {
    hipLaunchKernelGGL(stream_desc_kernel, dim3((unsigned)ix->nlist), dim3(64), 0, sst, a,
                       reinterpret_cast<StreamDesc*>(ix->item_desc));
  }
  if (split) {
    hipLaunchKernelGGL(item_desc_kernel, dim3((unsigned)ix->nlist), dim3(64), 0, sst, pair_off, ix->tile_off, item_off,
                       mask_off, a.tseg, a.segmax, ix->item_desc);
    a.item_off16 = item16;
    a.mask_off = mask_off;
    a.surv_mask = ix->surv_mask;
    a.item_desc = ix->item_desc;
    // (the refinement-only kernel lives on wavefronts in flight: smaller pools, checked every second round of 16 keys)
    a.pool = std::max(64, next_pow2_host(k + 32));
  }
  if (ss.setup_e) RQ_HIP(hipEventRecord(ss.setup_e, sst));
  if (sst != st) {
    RQ_HIP(hipEventRecord(ss.join, sst));
    RQ_HIP(hipStreamWaitEvent(st, ss.join, 0));
  }
  if (ss.scan_b) RQ_HIP(hipEventRecord(ss.scan_b, st));
  if (max_items > 0x7fffffff) {
    set_error("scan: too many work items");
    return RABITQ_EINVAL;
  }
  // (the prefetching variant's grid: the usual number of items, three for every two pairs, when the bound is larger;
  // its workgroups go on to further items if there are more)
  const unsigned grid = (unsigned)(a.streaming ? std::min<int64_t>(max_items, nq * nprobe + nq * nprobe / 2 + 1024) : max_items);
  const bool dbg = dbg_ip != nullptr;
  const int W = ix->W, F = field_bits(ix->total_bits);
  if (split) {
    const int64_t items16 = item_bound(ix, nq, nprobe, QM);  // the same bound with 16 pairs per item
    if (ss.est_b) RQ_HIP(hipEventRecord(ss.est_b, st));
    if (!estimate_mfma(a, W, (unsigned)items16, dbg, st)) return bad_width();
    RQ_HIP(hipGetLastError());
    if (ss.est_e) RQ_HIP(hipEventRecord(ss.est_e, st));
  }
  if (!(scan_part0(a, W, F, impl, grid, dbg, st) || scan_part1(a, W, F, impl, grid, dbg, st) ||
        scan_part2(a, W, F, impl, grid, dbg, st)))
    return bad_width();
  RQ_HIP(hipGetLastError());
  if (ss.scan_e) RQ_HIP(hipEventRecord(ss.scan_e, st));
  return RABITQ_OK;
}

}  // namespace rq
