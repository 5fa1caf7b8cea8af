// Argument block of the seeding and scan kernels (plain data, passed by value).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rq {

// Threshold seeding (Section 3.3.4): the max(k, SEED_M) best 1-bit candidates of the nearest cluster are refined
// and tau is the k-th smallest refined estimate.
constexpr int SEED_M = 32;

// What the refinement-only kernel of the split search needs to know about a work item, looked up once by a kernel of
// its own instead of by every item through a chain of dependent loads (item -> cluster -> offsets -> ...).
struct ItemDesc {
  int32_t pbeg;     // first pair of the item
  int32_t np_mg;    // pairs of the item | (group of 4 inside its group of 16) << 8
  int32_t t0;       // first tile of the cluster
  int32_t ts, te;   // tiles of the item's segment
  int32_t nseg;     // segments the cluster is scanned in
  uint32_t mblock;  // block of survivor bits of (group of 16, tile ts)
  int32_t pad;
};

// The same for the prefetching variant of the popcount kernel (one pair per work item, lists read from memory about
// once): the item's tiles and the scalars of its pair, 64 bytes that one scalar load brings in.
struct StreamDesc {
  int32_t pp, q;    // the pair and its query
  int32_t t0;       // first tile of the cluster
  int32_t ts, te;   // tiles of the item's segment
  int32_t nseg;     // segments the cluster is scanned in
  int32_t ppos;     // position of the pair in the pair list
  int32_t S;        // sum of the query's 4-bit digits
  float G, E;       // coarse score of the pair and ||q' - c'||
  float delta;      // step of the query's 4-bit grid
  float sumq;       // sum of the rotated query
  int32_t pad[4];
};

struct ScanArgs {
  // index
  const uint32_t* short_codes;
  const float* short_factors;
  const uint32_t* long_codes;
  const float* long_factors;
  const int32_t* ids;
  const int32_t* tile_off;
  const int32_t* cluster_size;
  int D, B, LW, nlist;
  float cB;  // (2^B - 1) / 2
  // The 1-bit bound of a 4-bit query multiplies f_err by sqrt(E^2 + qerr * delta^2) instead of E = ||q'-c'||: the
  // query's rounding errors add variance (D-1) delta^2 / (12 (1-a^2)) in the units of the code's own error, with
  // a^2 = 2/pi for 1-bit codes; qerr = (D-1) / (12 (1 - 2/pi)), 0 for the lookup-table scheme (no rounded query).
  float qerr;
  // per query
  const float* q_stage;   // [nq][D] rotated query in refinement order
  const int8_t* qhat8;    // [nq][Dp] 4-bit query as bytes (matrix-core scan)
  int Dp;
  const uint32_t* planes;
  const uint16_t* lut;    // [nq][D/4][16] binary16 lookup tables (lookup-table scan only)
  const float* delta;
  const int32_t* sum_qhat;
  const float* sum_q;
  const float* tau;
  // per pair
  const float* probe_G;
  const float* probe_E;
  const int32_t* probe_ids;
  const int32_t* pair_off;
  const int32_t* pair_ids;
  const int32_t* item_off;
  // nullptr: item_off[c] is the first work item of cluster c.  Otherwise item_off[r] is the first work item of cluster
  // order[r], the clusters being handed out longest first (a launch whose lists are each read about once)
  const int32_t* order;
  // split search (estimates by estimate_mfma_kernel, refinement by the popcount kernel): work items of 16 pairs,
  // first block of survivor bits of every cluster, the bits themselves (nullptr: not split)
  const int32_t* item_off16;
  const uint32_t* mask_off;
  uint64_t* surv_mask;
  ItemDesc* item_desc;  // [work items of 4 pairs]
  const StreamDesc* stream_desc;  // [work items of one pair] (prefetching variant; the same memory as item_desc)
  int nprobe, k, pool, cand_stride;
  // pair / nprobe without a division: (pair * nprobe_mul) >> nprobe_shift is exact for pair < 2^31 when nprobe_mul =
  // ceil(2^(31 + L) / nprobe), nprobe_shift = 31 + L and 2^L >= nprobe (set_nprobe)
  uint64_t nprobe_mul;
  int nprobe_shift;
  int streaming;     // few pairs per list: every list is read from memory about once (prefetching scan variant)
  int tseg, segmax;  // a cluster of more than tseg tiles is scanned in up to segmax segments (separate work items)
  // outputs
  uint64_t* cand_keys;
  int32_t* cand_cnt;
  float* tau_out;
  int32_t* dbg_ip;
  const int64_t* dbg_off;
};

inline void set_nprobe(ScanArgs& a, int nprobe) {
  int L = 0;
  while ((1 << L) < nprobe) ++L;
  a.nprobe = nprobe;
  a.nprobe_shift = 31 + L;
  a.nprobe_mul = (((uint64_t)1 << (31 + L)) + (uint64_t)nprobe - 1) / (uint64_t)nprobe;  // L <= 31: no overflow
}
// query of a pair (pairs are numbered query * nprobe + rank)
__host__ __device__ inline int pair_query(const ScanArgs& a, int pair) {
  return (int)(((uint64_t)(uint32_t)pair * a.nprobe_mul) >> a.nprobe_shift);
}

// number of segments a cluster of `tiles` tiles is split into
__host__ __device__ inline int seg_count(int tiles, int tseg, int segmax) {
  const int n = (tiles + tseg - 1) / tseg;
  return n < 1 ? 1 : (n > segmax ? segmax : n);
}

// impl 4: the estimates of QM pairs per wavefront on the matrix cores, leaving survivor bits for the popcount kernel;
// false for a width it is not built for
bool estimate_mfma(const ScanArgs& a, int W, unsigned grid, bool dbg, hipStream_t st);

// impl 0: popcount kernel (QW pairs per wavefront); impl 1: matrix-core kernel (QM pairs; seeds by popcount);
// impl 2: lookup-table kernel (QW pairs)
bool seed_part0(const ScanArgs& a, int W, int F, int impl, int64_t nq, hipStream_t st);
bool seed_part1(const ScanArgs& a, int W, int F, int impl, int64_t nq, hipStream_t st);
bool seed_part2(const ScanArgs& a, int W, int F, int impl, int64_t nq, hipStream_t st);
bool scan_part0(const ScanArgs& a, int W, int F, int impl, unsigned grid, bool dbg, hipStream_t st);
bool scan_part1(const ScanArgs& a, int W, int F, int impl, unsigned grid, bool dbg, hipStream_t st);
bool scan_part2(const ScanArgs& a, int W, int F, int impl, unsigned grid, bool dbg, hipStream_t st);

}  // namespace rq
