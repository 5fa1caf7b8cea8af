// Small batches (at most 64 queries): pair lists, the scan's work-item offsets and cleared candidate counters,
// computed by ONE workgroup of NT threads.  Shared by the stand-alone kernel and by the fused
// selection + seeding kernel, whose last workgroup runs it.
#pragma once
#include "rq_device.h"
#include "rq_scan_args.h"

namespace rq {

struct SmallListArgs {
  const int32_t* probe_ids;  // [nq][nprobe]
  int nq, nprobe, nlist;
  const int32_t* tile_off;   // [nlist + 1]
  int qw, tseg, segmax;      // the scan's plan: pairs per work item, tiles per segment, segments per list at most
  uint32_t* mask;            // [nlist][2] scratch
  int32_t* pair_off;         // [nlist + 1] out
  int32_t* pair_ids;         // [nq * nprobe] out
  int32_t* item_off;         // [nlist + 1] out
  int32_t* cand_cnt;         // [nq * nprobe] out: zeros
  // work items of one pair (qw == 1): their descriptors for the prefetching scan, nullptr = not written here
  StreamDesc* desc;
  const float *probe_G, *probe_E, *delta, *sum_q;
  const int32_t* sum_qhat;
};

// A query probes a list at most once, so the queries of a list are one 64-bit mask; a pair's place in its list is
// the number of lower queries in the mask (the regrouping is stable in query id, as in the large-batch builder), a
// list's length is the mask's popcount, and the exclusive scans over the lists give pair_off and item_off.
// s_pairs / s_items: NT words of LDS each.  All NT threads of the workgroup must call it.
template <int NT>
__device__ inline void small_lists_body(const SmallListArgs& b, uint32_t* s_pairs, uint32_t* s_items) {
  const int tid = threadIdx.x, npairs = b.nq * b.nprobe, nlist = b.nlist;
  // (the masks are built by atomics, which act in the L2: they are read back from there, past the L1)
  auto mask_at = [&](int i) { return __hip_atomic_load(&b.mask[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  for (int i = tid; i < 2 * nlist; i += NT) b.mask[i] = 0u;
  for (int i = tid; i < npairs; i += NT) b.cand_cnt[i] = 0;
  __syncthreads();
  for (int p = tid; p < npairs; p += NT) {
    const int c = b.probe_ids[p], q = p / b.nprobe;
    atomicOr(&b.mask[2 * c + (q >> 5)], 1u << (q & 31));
  }
  __syncthreads();
  // every thread takes a run of consecutive lists; the runs' sums are scanned across the workgroup
  const int per = (nlist + NT - 1) / NT;
  const int c0 = min(tid * per, nlist), c1 = min(c0 + per, nlist);
  auto items_of = [&](int c, uint32_t cnt) {
    return ((cnt + b.qw - 1) / b.qw) * (uint32_t)seg_count(b.tile_off[c + 1] - b.tile_off[c], b.tseg, b.segmax);
  };
  uint32_t sp = 0, si = 0;
  for (int c = c0; c < c1; ++c) {
    const uint32_t cnt = __popc(mask_at(2 * c)) + __popc(mask_at(2 * c + 1));
    sp += cnt;
    si += items_of(c, cnt);
  }
  s_pairs[tid] = sp;
  s_items[tid] = si;
  __syncthreads();
  for (int d = 1; d < NT; d <<= 1) {
    const uint32_t op = tid >= d ? s_pairs[tid - d] : 0u, oi = tid >= d ? s_items[tid - d] : 0u;
    __syncthreads();
    s_pairs[tid] += op;
    s_items[tid] += oi;
    __syncthreads();
  }
  uint32_t rp = s_pairs[tid] - sp, ri = s_items[tid] - si;
  for (int c = c0; c < c1; ++c) {
    const uint32_t cnt = __popc(mask_at(2 * c)) + __popc(mask_at(2 * c + 1));
    b.pair_off[c] = (int32_t)rp;
    b.item_off[c] = (int32_t)ri;
    rp += cnt;
    ri += items_of(c, cnt);
  }
  if (tid == NT - 1) {
    b.pair_off[nlist] = (int32_t)s_pairs[NT - 1];
    b.item_off[nlist] = (int32_t)s_items[NT - 1];
  }
  __syncthreads();  // pair_off is read below by other threads than those that wrote it
  for (int p = tid; p < npairs; p += NT) {
    const int c = b.probe_ids[p], q = p / b.nprobe;
    const uint32_t lo = mask_at(2 * c), hi = mask_at(2 * c + 1);
    const int below = q < 32 ? __popc(lo & ((1u << q) - 1u)) : __popc(lo) + __popc(hi & ((1u << (q - 32)) - 1u));
    b.pair_ids[b.pair_off[c] + below] = p;
    if (b.desc) {
      const int t0 = b.tile_off[c], tiles = b.tile_off[c + 1] - t0;
      const int nseg = seg_count(tiles, b.tseg, b.segmax), seglen = (tiles + nseg - 1) / nseg;
      StreamDesc d{};
      d.pp = p;
      d.q = q;
      d.t0 = t0;
      d.nseg = nseg;
      d.ppos = b.pair_off[c] + below;
      d.S = b.sum_qhat[q];
      d.G = b.probe_G[p];
      d.E = b.probe_E[p];
      d.delta = b.delta[q];
      d.sumq = b.sum_q[q];
      for (int sidx = 0; sidx < nseg; ++sidx) {
        d.ts = t0 + sidx * seglen;
        d.te = min(t0 + tiles, d.ts + seglen);
        b.desc[b.item_off[c] + below * nseg + sidx] = d;
      }
    }
  }
}

// Everything the fused selection + seeding kernel needs beyond ScanArgs.
struct SmallSelectArgs {
  const float* scores;       // [nq][nlist]
  const float* sq_norm;      // [nq]
  const float* centroid_sq;  // [nlist]
  int metric, do_seed;
  int32_t* probe_ids;        // [nq][nprobe] out
  float* probe_G;            // out
  float* probe_E;            // out
  int32_t* ticket;           // one word, zero between launches
  SmallListArgs lists;
};

bool small_part0(const ScanArgs& a, const SmallSelectArgs& b, int W, int F, hipStream_t st);
bool small_part1(const ScanArgs& a, const SmallSelectArgs& b, int W, int F, hipStream_t st);
bool small_part2(const ScanArgs& a, const SmallSelectArgs& b, int W, int F, hipStream_t st);

}  // namespace rq
