// Internal declarations shared by the translation units of librabitq_hip.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "rabitq.h"

namespace rq {

constexpr int TILE = RABITQ_TILE;
constexpr int QW = 4;        // queries handled by one wavefront of the popcount scan
constexpr int QM = 16;       // queries handled by one wavefront of the matrix-core scan
inline int qhat_stride(int D) { return (D + 63) / 64 * 64; }

struct Workspace {
  // per query
  float* q_rot = nullptr;
  rabitq_query_repr repr = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  int64_t cap_lut = 0;  // queries the lookup tables were sized for (allocated on first use of scan_impl 2)
  float* tau = nullptr;
  // coarse
  float* scores = nullptr;
  int32_t* probe_ids = nullptr;
  float* probe_G = nullptr;
  float* probe_E = nullptr;
  // lists
  int32_t* pair_off = nullptr;
  int32_t* pair_ids = nullptr;
  uint32_t* list_scratch = nullptr;
  // candidates
  uint64_t* cand_keys = nullptr;
  int32_t* cand_cnt = nullptr;
  // capacities the buffers were sized for
  int64_t cap_nq = 0;
  int64_t cap_pairs = 0;
  int64_t cap_cand = 0;
  int64_t cap_scratch = 0;
};

}  // namespace rq

namespace rq { struct ItemDesc; }

struct rabitq_index {
  int32_t dim = 0, W = 0, nlist = 0, total_bits = 0, metric = 0, F = 0, LW = 0;  // LW = long words per slot
  int64_t n = 0, n_tiles = 0, n_slots = 0;
  int device = 0;
  // device arrays
  float* rotation = nullptr;        // [D][D]
  float* mean_rot = nullptr;        // [D] mean * P of a centred index (nullptr: not centred)
  std::vector<float> host_mean;     // [D] the mean itself (empty: not centred)
  float* centroids_t = nullptr;     // [D][nlist]  (transposed c')
  float* centroid_sq = nullptr;     // [nlist]
  int32_t* tile_off = nullptr;      // [nlist+1] tile offsets | [nlist+1] scan work-item offsets | [TICKET_WORDS] zeroed ticket
                                    // | [nlist+1] work items of 16 pairs | [nlist+1] first survivor block (split search)
  int32_t* cluster_size = nullptr;  // [nlist]
  int32_t* cluster_order = nullptr; // [nlist] clusters by descending tile count, equal counts by ascending id
  uint32_t* short_codes = nullptr;
  float* short_factors = nullptr;
  uint32_t* long_codes = nullptr;
  float* long_factors = nullptr;
  int32_t* ids = nullptr;
  std::vector<int32_t> host_tiles;  // tiles per cluster (host copy, sizes the scan grid)
  int32_t max_tiles = 0;            // the longest list's
  // segments per cluster in descending order for the segment limit seg_sorted_max and length seg_sorted_tseg, and their sum (scan grid bound)
  mutable std::vector<int> seg_sorted;
  mutable int seg_sorted_max = -1, seg_sorted_tseg = -1;
  mutable int64_t seg_total = 0;
  // options
  int prune = 1;
  int scan_impl = 3;  // 0 popcount, 1 matrix cores, 2 lookup tables, 3 chosen by code width (see effective_impl),
                      // 4 estimates on the matrix cores + refinement by the popcount kernel (split search)
  // survivor bits of the split search: blocks of 16 words; grown on demand by ensure_split_buffers, kept by the handle
  int last_scan_split = 0;   // the scan of the latest rabitq_search / rabitq_scan was split (rabitq_index_info)
  int last_scan_stream = 0;  // ... was the prefetching variant of the popcount kernel (one pair per work item)
  int split_min_pairs = 32;  // pairs per list, on average, from which scan_impl 3 / 4 split the search
  uint64_t* surv_mask = nullptr;
  int64_t surv_mask_blocks = 0;
  rq::ItemDesc* item_desc = nullptr;  // descriptors of the refinement kernel's work items (split search), grown with the bits
  int64_t item_desc_cap = 0;
  std::vector<int64_t> tiles_prefix;  // [i] = tiles of the i largest lists (host; filled on first use)
  int overlap = 1;  // list building and scan set-up run beside the seeding on `side`
  int64_t max_batch = 0;  // queries per pass of rabitq_search; 0 = from the workspace budget
  int small_batch = 1;    // batches of at most SMALL_BATCH_MAX queries take the fused low-launch-count kernels
  int longest_first = 1;  // a scan that reads every list about once hands out its work items longest list first
  int seg_tiles = 0;      // tiles per scan work item of a long list; 0 = chosen from the batch (see launch_scan)
  // second stream of a search (default priority) and the events that fork it from and join it to the caller's
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  static constexpr int N_STAGES = 10;
  // begin / end of every stage, on the stream it ran on; bit s of `rec`: stage s was recorded in this search (a
  // small batch runs several stages as one kernel, recorded under the first of them)
  struct EventSet { hipEvent_t b[N_STAGES], e[N_STAGES]; unsigned rec; };
  std::vector<EventSet> prof_sets;  // one per recorded search
  int prof_used = 0, prof_limit = 0;
  unsigned prof_mask = 0x3ffu;  // stages whose events are recorded (bit s = stage s)
  rq::Workspace ws;
};

namespace rq {

// The scan the handle's option selects: "by code width" takes the matrix-core kernel from D = 960 on, where it was
// measured 3.2x faster than the popcount kernel (0.86 against 2.79 ms), and the popcount kernel below (D = 128: 0.28
// against 0.32 ms; at D = 768 the matrix-core kernel wins where the filter works, 4.2 against 5.8 ms, and loses where
// nearly every vector has to be refined, 32 against 22 ms).
// (4 is the popcount kernel everywhere except in launch_scan, which splits the search when it can: see split_search)
inline int effective_impl(const rabitq_index* ix) {
  const int impl = ix->scan_impl == 3 ? (ix->W >= 30 ? 1 : 0) : ix->scan_impl;
  return impl == 4 ? 0 : impl;
}

void set_error(const std::string& s);
int hip_fail(hipError_t e, const char* what);

#define RQ_HIP(call)                                  \
  do {                                                \
    hipError_t e__ = (call);                          \
    if (e__ != hipSuccess) return rq::hip_fail(e__, #call); \
  } while (0)

// order-preserving map float -> uint32 (ascending floats give ascending unsigned ints)
__host__ __device__ inline uint32_t f2ord(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__host__ __device__ inline float ord2f(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
  return __builtin_bit_cast(float, u);
}

// ---- launchers (each returns a rabitq_status) ----
// C[M,N] = A[M,K] * B[K,N], row-major fp32.  mode 0: plain.  mode 1 (L2 coarse):
// C = rowv[m] + colv[n] - 2*acc.  mode 2 (IP coarse): C = -acc.  mode 3 (assignment): C = colv[n] - 2*acc.
// mode 4 (rotation of a centred index): C = acc - colv[n].
int launch_gemm(const float* A, const float* B, float* C, int64_t M, int N, int K, int mode, const float* rowv,
                const float* colv, hipStream_t st);
// small batches: Q' = (Q - mean) P, the queries' representation and the coarse scores [nq][nlist] from one launch,
// bit-identical to launch_rotate + launch_query_prep + launch_gemm (mode 1 / 2)
int launch_small_front(const rabitq_index* ix, const float* queries, int64_t nq, float* q_rot, const rabitq_query_repr& o,
                       float* scores, hipStream_t st);
int launch_query_prep(const float* q_rot, int64_t nq, int D, int F, const rabitq_query_repr& out, hipStream_t st);
int launch_select_probes(const float* scores, const float* sq_norm, const float* centroid_sq, int64_t nq, int nlist,
                         int nprobe, int metric, int32_t* probe_ids, float* probe_G, float* probe_E, hipStream_t st);
int probe_select_variant(int nlist, int nprobe);  // which selection kernel launch_select_probes takes (see stages.hip)
int64_t probe_list_scratch_words(int32_t nlist, int64_t nq);
int launch_clear_list_bitmap(int64_t nq, int nlist, uint32_t* scratch, hipStream_t st);
int launch_build_lists(const int32_t* probe_ids, int64_t nq, int nprobe, int nlist, int32_t* pair_off,
                       int32_t* pair_ids, uint32_t* scratch, hipStream_t st, bool bitmap_is_clear = false);
int launch_seed(const rabitq_index* ix, const rabitq_query_repr& repr, const int32_t* probe_ids, const float* probe_G,
                const float* probe_E, int64_t nq, int k, int nprobe, float* tau, hipStream_t st);
// Streams and events of one scan launch: the set-up kernels (work-item offsets, counter clearing) run on `setup`
// and the scan kernel on `main`; when the two differ, `join` is recorded on `setup` and awaited on `main`.  The
// four profiling events may be null.
struct ScanStreams {
  hipStream_t main = nullptr, setup = nullptr;
  hipEvent_t join = nullptr;
  hipEvent_t setup_b = nullptr, setup_e = nullptr, scan_b = nullptr, scan_e = nullptr;
  hipEvent_t est_b = nullptr, est_e = nullptr;  // around the estimate kernel of a split search
  mutable bool split = false;                  // out: the search was split
  mutable bool streamed = false;               // out: the prefetching variant of the popcount kernel ran
  bool counters_clear = false;  // cand_cnt was already zeroed by launch_clear_counters
  bool desc_done = false;       // ... and so were the descriptors of the prefetching scan's work items (launch_small_select_seed)
  bool setup_done = false;      // work-item offsets and counters were already prepared (launch_small_batch_lists)
};
// How a scan launch cuts its work: pairs per work item, tiles per segment of a long list, segments per list at most.
struct ScanPlan { int qw, tseg, segmax; bool streaming; };
ScanPlan scan_plan(const rabitq_index* ix, int64_t nq, int nprobe, int k);
// Batches of at most SMALL_BATCH_MAX queries: pair lists, the scan's work-item offsets and the cleared candidate
// counters from ONE single-workgroup kernel (instead of the seven launches of launch_build_lists + the scan set-up).
// `scratch` holds at least 2 * nlist words.  Same pair_off / pair_ids as launch_build_lists.
constexpr int SMALL_BATCH_MAX = 64;
constexpr int TICKET_WORDS = 4;  // words behind the two offset arrays of rabitq_index::tile_off (zero between launches)
inline int64_t tile_off_words(int nlist) { return 4 * (int64_t)(nlist + 1) + TICKET_WORDS; }
// Split search (scan_impl 4): the first stage runs on the matrix cores for groups of 16 pairs and hands one survivor
// bit per (pair, vector) to the popcount kernel.  Built for every code with a long part (B > 1); taken on request (4) and,
// by default (3), below D = 960 (there the four-wavefront matrix-core kernel is faster) from split_min_pairs pairs per
// list on average.  split_mask_blocks bounds the blocks of survivor bits a search of
// (nq, nprobe) can need: sum_c ceil(cnt_c / 16) tiles_c <= (nq * tiles of the nprobe largest lists) / 16 + all tiles,
// because every query probes nprobe distinct lists.
inline bool split_built(const rabitq_index* ix) { return ix->total_bits > 1; }
inline bool split_wanted(const rabitq_index* ix, int64_t nq, int nprobe) {
  return (ix->scan_impl == 4 || (ix->scan_impl == 3 && ix->W < 30)) && split_built(ix) &&
         nq * nprobe >= (int64_t)ix->split_min_pairs * ix->nlist;
}
int64_t split_mask_blocks(rabitq_index* ix, int64_t nq, int nprobe);
// makes the handle's survivor-bit buffer large enough for (nq, nprobe); may allocate (then it synchronises the device)
int ensure_split_buffers(rabitq_index* ix, int64_t nq, int nprobe, int k);
// makes the handle's descriptor memory large enough for the prefetching scan of (nq, nprobe, k), when that is the shape;
// may allocate (then it synchronises the device)
int ensure_stream_buffers(rabitq_index* ix, int64_t nq, int nprobe, int k);
// The same for nprobe <= 64, k <= 64 and a bitwise scan, preceded in the same kernel by the selection of the probes
// from the coarse scores and the seeding of the thresholds (one workgroup per query; the last one to finish builds the
// lists): everything between the coarse scores and the scan in one launch.
int launch_small_select_seed(const rabitq_index* ix, const rabitq_query_repr& repr, const float* scores, int64_t nq, int k,
                             int nprobe, int32_t* probe_ids, float* probe_G, float* probe_E, float* tau, int32_t* pair_off,
                             int32_t* pair_ids, uint32_t* scratch, int32_t* cand_cnt, hipStream_t st);
int launch_small_batch_lists(const rabitq_index* ix, const int32_t* probe_ids, int64_t nq, int nprobe, int k,
                             int32_t* pair_off, int32_t* pair_ids, uint32_t* scratch, int32_t* cand_cnt, hipStream_t st);
int launch_clear_counters(int32_t* cand_cnt, int64_t n, hipStream_t st);
int launch_scan(const rabitq_index* ix, const rabitq_query_repr& repr, const float* probe_G, const float* probe_E,
                const int32_t* pair_off, const int32_t* pair_ids, const float* tau, int64_t nq, int k, int nprobe,
                uint64_t* cand_keys, int32_t* cand_cnt, int32_t* dbg_ip, const int64_t* dbg_off, const ScanStreams& ss);
int launch_merge(const uint64_t* cand_keys, const int32_t* cand_cnt, int64_t nq, int k, int nprobe, int metric,
                 int64_t* out_ids, float* out_dists, hipStream_t st);
int launch_fill_f32(float* p, int64_t n, float v, hipStream_t st);
int build_index_device(rabitq_index* ix, const float* data, const float* rotation_host, int kmeans_iters,
                       int64_t train_size, float eps0, int center, hipStream_t st);
// stores `mean` [D] (host) in the handle together with mean * P on the device
int set_index_mean(rabitq_index* ix, const float* mean, const float* rotation_host, hipStream_t st);
// Q' = (Q - mean) P for the handle's rotation
int launch_rotate(const rabitq_index* ix, const float* q, float* q_rot, int64_t nq, hipStream_t st);

}  // namespace rq
