/*
 * rabitq.h — C ABI of the MI355X (gfx950) IVF-RaBitQ batched-search library.
 *
 * The calls follow the paper's problem statement (Section 2.1: a batch of
 * queries Q in R^{nq x D}, return the K approximate nearest neighbours of each
 * among N indexed vectors) and its search pipeline (Section 3.3).  All entry
 * points are plain C: pointers, sizes and an opaque handle.  No entry point
 * throws or aborts; each returns RABITQ_OK (0) or a negative rabitq_status, and
 * rabitq_last_error() describes the last failure of the calling thread.
 *
 * Pointer kinds are stated per argument: "host" = ordinary host memory,
 * "device" = memory of the current HIP device (for example the data_ptr() of a
 * torch tensor).  `stream` is a hipStream_t passed as void* (NULL = the default
 * stream).  Unless stated otherwise a call only enqueues work on `stream` and
 * returns; outputs are valid once the caller has synchronised the stream.
 * A handle supports one in-flight rabitq_search at a time (the workspace it owns
 * is reused); the stage-level calls use only caller-provided buffers.  A handle belongs
 * to the device that was current when it was created; calls made with another current
 * device are rejected (RABITQ_EINVAL).
 */
#ifndef RABITQ_H
#define RABITQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RABITQ_TILE 64        /* vectors per tile of the code layout (one wavefront)   */
#define RABITQ_MAX_K 128      /* largest supported K                                    */
#define RABITQ_QUERY_BITS 4   /* B_q of the bitwise scheme (Section 3.4.1(2))           */
#define RABITQ_MAX_NPROBE 1024
#define RABITQ_NOALLOC_SCRATCH_BYTES (64u << 20) /* static workspace of rabitq_search_noalloc, per device */

typedef enum {
  RABITQ_OK = 0,
  RABITQ_EINVAL = -1, /* null pointer, size out of range, dim not a multiple of 32 ... */
  RABITQ_ENOMEM = -2, /* device or host allocation failed                              */
  RABITQ_EHIP = -3    /* a HIP runtime call or kernel launch failed                    */
} rabitq_status;

typedef enum { RABITQ_L2 = 0, RABITQ_IP = 1 } rabitq_metric;

typedef struct rabitq_index* rabitq_index_t; /* opaque; owns device copies of the index */

/*
 * Index description (Section 3.4.3: flattened CSR-like arrays, one offset array
 * shared by all of them).  All pointers are HOST pointers owned by the caller;
 * rabitq_index_upload copies them and the caller may free them afterwards.
 *
 * Interleaving unit: the paper interleaves the packed 1-bit words of a whole
 * cluster per 32-dimension group; here the unit is a tile of 64 vectors (one
 * wavefront).  Cluster c holds n_c = offsets[c+1]-offsets[c] vectors in
 * ceil(n_c/64) tiles; tiles of consecutive clusters follow each other, and the
 * slot of the j-th vector of cluster c is 64*first_tile(c) + j.  Slots past n_c
 * in the last tile of a cluster are padding: code words 0, f_add = +inf, other
 * factors 0, id = -1.  n_tiles = sum_c ceil(n_c/64), n_slots = 64*n_tiles.
 * W = dim/32.  Bit i (LSB = 0) of word w is dimension 32*w+i, for codes and for
 * query bit-planes alike.
 */
typedef struct {
  int32_t dim;        /* D: 32, 64, 96, 128, 256, 512, 768, 960 or 1024 (the scan kernels are
                         instantiated per D/32; other values are rejected)              */
  int32_t nlist;      /* n_k, number of inverted lists                                 */
  int64_t n;          /* N, number of stored vectors                                   */
  int32_t total_bits; /* B in 1..8: 1 sign bit + (B-1) ex bits per dimension           */
  int32_t metric;     /* rabitq_metric                                                 */
  const float* rotation;      /* [D*D] row-major P; rotated query q' = q P             */
  const float* centroids;     /* [nlist*D] rotated centroids c'                         */
  const int64_t* offsets;     /* [nlist+1] CSR over stored vectors, offsets[nlist]==n   */
  const uint32_t* short_codes;  /* [n_tiles][W][64]  1-bit (sign) codes                 */
  const float* short_factors;   /* [n_tiles][3][64]  f_add, f_rescale, f_err planes     */
  const uint32_t* long_codes;   /* [n_slots][D*F/32] the whole B-bit code of each dimension
                                   in F-bit little-endian fields, F = B rounded up to
                                   2, 4 or 8 (dimension i sits in word i/(32/F) at bit
                                   F*(i mod 32/F)); NULL when B == 1                    */
  const float* long_factors;    /* [n_slots][2] f_add, f_rescale of the B-bit code;
                                   NULL when B == 1                                     */
  const int32_t* ids;           /* [n_slots] original id (Pid) of each stored vector    */
  const float* mean;            /* [D] or NULL: a translation the index was built under (L2 only):
                                   codes, factors and centroids describe the vectors minus `mean`,
                                   and the search rotates (q - mean).  Squared distances do not
                                   change; the rotated query, which Section 3.4.1(2) quantises to
                                   4 bits, loses the offset all vectors share                */
} rabitq_index_desc;

/* Estimator read by the search (Section 2.2 leaves the expressions to an external
 * document; these follow from Eq. (1)-(3)).  With G the coarse term of the probed
 * cluster (L2: ||q'-c'||^2, IP: -<q',c'>), E = ||q'-c'||, the 4-bit query qhat with
 * scale delta and S = sum(qhat), and I = <x_b, qhat> by AND+popcount:
 *   est1 = G + f_add1 + f_rescale1 * delta * (2I - S)/2,
 *   lb1 = est1 - f_err1 * sqrt(E^2 + (D-1) delta^2 / (12 (1 - 2/pi)))   (the second term under the root is the
 *         variance the 4-bit query's rounding adds, in the units of the code's own error; the lookup-table
 *         scheme rounds no query and uses lb1 = est1 - f_err1 * E)
 *   estB = G + f_addB + f_rescaleB * (<u, q'> - (2^B-1)/2 * sum(q'))
 * Keys are "smaller is better" for both metrics (IP keys are negated products). */

/* Copies the index to the current device.  Synchronises `stream` before returning.
 * Errors: RABITQ_EINVAL (null pointer, bad dim/bits/metric, offsets not monotone or
 * offsets[nlist] != n), RABITQ_ENOMEM, RABITQ_EHIP.  *out is untouched on error. */
int rabitq_index_upload(const rabitq_index_desc* desc, rabitq_index_t* out, void* stream);

/*
 * Index build on the device (Section 3.2): the vectors are rotated by P, k-means (plain
 * Lloyd) runs in the rotated space on a training subset, every vector is assigned to its
 * nearest centroid, normalised with respect to it, and quantised by the two-phase grid
 * search over the rescaling factor (N_coarse = 64 samples over [0, m_B*2^(B-1)/max|o'|] with
 * m_B = 6, 4.5, 2.5 for B = 2, 3, 4 and 1.5 above, then N_fine = 32 around the best); codes,
 * factors and ids are written in the layout above, every list in ascending id order.
 * Deterministic: no order-dependent atomics anywhere.  Temporary device memory, freed before
 * the call returns: a rotated copy of the data (n*D floats), the training subset, 3n words
 * of assignments and list members and at most 1024*nlist counters.
 *   data: device, [n*D] fp32 row-major raw vectors (not modified)
 * The training subset is taken at a fixed stride through the data and the initial centroids
 * at a fixed stride through the training subset (shuffle the data first if its order is not
 * random).  Synchronises `stream`.  Errors as for rabitq_index_upload.
 */
typedef struct {
  int32_t dim, nlist;
  int64_t n;
  int32_t total_bits, metric;
  int32_t kmeans_iters;  /* Lloyd iterations, >= 0                                        */
  int64_t train_size;    /* vectors used for k-means; <= 0 or > n: all of them            */
  float epsilon0;        /* multiplier of the 1-bit error bound stored as f_err (e.g. 1.9) */
  const float* rotation; /* host, [D*D] row-major orthogonal P                            */
  int32_t center;        /* 1: build on the vectors minus their mean (see rabitq_index_desc.mean;
                            L2 only), 0: on the vectors as given                          */
} rabitq_build_params;
int rabitq_index_build(const rabitq_build_params* params, const float* data, rabitq_index_t* out, void* stream);

/* Copies the arrays of an index back to HOST buffers laid out as in rabitq_index_desc (sizes
 * from rabitq_index_info: n_tiles, n_slots, long_field_bits).  Any pointer may be NULL to
 * skip that array.  Device-synchronising.  Errors: RABITQ_EINVAL, RABITQ_EHIP. */
int rabitq_index_export(rabitq_index_t index, float* rotation, float* centroids, int64_t* offsets,
                        uint32_t* short_codes, float* short_factors, uint32_t* long_codes, float* long_factors,
                        int32_t* ids, float* mean /* [D], zeros if the index is not centred */);

/* Frees the handle and everything it owns (device-synchronising).  NULL is allowed. */
int rabitq_index_free(rabitq_index_t index);

/*
 * Batched search (Sections 2.1, 3.3).
 *   queries   device, [nq*D] fp32 row-major, unrotated
 *   out_ids   device, [nq*k] int64: original ids, best first; -1 where fewer than k
 *             candidates survived
 *   out_dists device, [nq*k] fp32: L2 -> estimated squared distance ascending (not
 *             clamped at 0); IP -> estimated inner product descending; +inf / -inf
 *             beside id -1
 * The handle's workspace grows on demand (growth synchronises the device).  A batch whose
 * workspace would exceed 16 GiB (or the "max_batch" option) is searched in consecutive
 * sub-batches on `stream` through one workspace; results do not depend on the split.
 * Errors: RABITQ_EINVAL (null pointer with nq > 0, nq < 0, k < 1 or k > RABITQ_MAX_K,
 * nprobe < 1 or > min(nlist, RABITQ_MAX_NPROBE)), RABITQ_ENOMEM, RABITQ_EHIP.
 * nq == 0 succeeds and does nothing.
 */
int rabitq_search(rabitq_index_t index, const float* queries, int64_t nq, int32_t k, int32_t nprobe,
                  int64_t* out_ids, float* out_dists, void* stream);

/*
 * The same search for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Arguments, results and kernels are those of rabitq_search;
 * the workspace (rotated queries and their representation, coarse scores [nq][nlist], probes, pair lists,
 * list-builder bitmap, candidate keys [nq*nprobe][cap] and counters) is laid out in a static device array of
 * RABITQ_NOALLOC_SCRATCH_BYTES (64 MiB) that every device the library runs on holds until the process ends.
 * The call allocates and frees nothing, on the device or through any library, and never splits the batch:
 * a (nq, k, nprobe) whose workspace does not fit is rejected with RABITQ_EINVAL and a message that names the
 * bytes needed.  Roughly nq * (4 nlist + nprobe * (8 cap + 20) + 10 D + nlist / 4) bytes, cap = rabitq_cand_capacity(k):
 * about 7000 queries at nlist 1024, D 128, k 10, nprobe 16.
 * All calls on one device share that device's array, which keeps the previous call's contents; the call clears
 * what must start at zero itself (with kernels).  Calls that overlap in time on one device (other streams, other
 * handles, other threads) race on the array: the caller must order them.  rabitq_search is not affected: it
 * uses the handle's own workspace.
 */
int rabitq_search_noalloc(rabitq_index_t index, const float* queries, int64_t nq, int32_t k, int32_t nprobe,
                          int64_t* out_ids, float* out_dists, void* stream);

/* Options (host call, takes effect for later searches):
 *   "prune"   1 (default): filter with the per-query seeded threshold (Section 3.3.4);
 *             0: refine every vector of every probed cluster (the unpruned definition).
 *   "profile" n: see rabitq_stage_ms.
 *   "profile_stages" m: bit s of m (1..1023, default all) selects whether stage s of rabitq_stage_ms is
 *             recorded; unrecorded stages report 0.  Recording costs two event records per stage and search.
 *   "overlap" 1 (default): inside a search of 256 or more queries the pair lists and the scan's work-item table
 *             are built on a second stream owned by the handle (default priority), beside the threshold seeding;
 *             the scan kernel waits for both and everything joins the caller's stream again before the call
 *             returns to it.  Smaller batches stay on one stream.  0: always one stream.
 *   "max_batch" n: rabitq_search passes at most n queries through the pipeline at a time (0, the default:
 *             as many as keep the workspace under 16 GiB, at least 256).
 *   "small_batch" 1 (default): a batch of at most 64 queries goes through fused kernels that do the same work in fewer
 *             launches (Section 4.2.2: latency at small batch sizes is launch-bound): the pair lists, the scan's
 *             work-item table and the cleared counters come from one single-workgroup kernel, probe selection and
 *             threshold seeding run in one kernel.  Results are identical to those of the general kernels.
 *             0: always the general kernels.
 *   "scan_segment_tiles" n: a list longer than n tiles of 64 vectors is scanned by several work items of about n tiles
 *             each (at most cand_capacity(k) / k of them); 0 (default): chosen from the batch size, 2..32.
 *   "longest_first" 1 (default): when a batch has at most four pairs per list on average, so that every probed list
 *             is read from memory about once (Section 3.4.2's coalesced cluster reads are then what bounds the scan),
 *             the popcount kernel takes one pair per work item and is handed the lists longest first, so that its
 *             launch ends everywhere at about the same time.  0: in cluster order.  Same results.
 *   "scan_impl" 0: bit-plane AND + popcount inner products (Section 3.4.1(2)), 4 queries per
 *             wavefront; 1: the same integer inner products on the matrix cores (the sign
 *             bits of a tile are expanded to int8 once and contracted against 16 queries'
 *             qhat with v_mfma_i32_16x16x64_i8).  Results of 0 and 1 are identical; only speed differs.
 *             4: split search: the estimates and the filter run on the matrix cores as a kernel of their own (one
 *             wavefront per 16 pairs of a cluster, next tile requested ahead, no LDS) and leave one bit per (pair,
 *             vector); the kernel of 0 then only refines the survivors.  Taken for B > 1 and at least
 *             "split_min_pairs" (an option; default 32) pairs per list on average, otherwise as 0.  Same results.  The
 *             survivor bits and the work-item descriptors live in buffers the handle grows on demand (rabitq_search
 *             and rabitq_scan may allocate when a larger batch arrives; rabitq_search_noalloc never does and splits
 *             only if the buffers are already large enough).
 *             3 (default): the faster in measurements: 1 for D >= 960; below that 4 where it is taken (see above), else 0.
 *             2: the lookup-table scheme of Section 3.4.1(1) instead of the quantised query:
 *             <x_b, q'> is the fp32 sum, in ascending block order, of one binary16 table entry per
 *             4 dimensions (tables in LDS, 4 queries per wavefront).  Used by the threshold
 *             seeding and the scan; its estimates differ from those of 0/1 by the query
 *             quantisation error.
 * Errors: RABITQ_EINVAL for an unknown name or value. */
int rabitq_set_option(rabitq_index_t index, const char* name, int64_t value);

/* Host-visible sizes of an uploaded index: name in {"n","n_tiles","n_slots","dim","nlist",
 * "total_bits","long_field_bits","metric"}, or "last_scan_split": 1 if the scan of the latest rabitq_search /
 * rabitq_scan on the handle was split ("scan_impl" 4), else 0; "last_scan_stream": 1 if it was the popcount kernel's
 * one-pair-per-work-item form (see "longest_first"), else 0.  Returns the value, or a negative status. */
int64_t rabitq_index_info(rabitq_index_t index, const char* name);

/* Per-stage timing.  The option "profile" = n (0..4096) makes the next n searches record
 * HIP events on the caller's stream around every stage (no synchronisation is added to the
 * search itself); setting it again restarts the recording.  rabitq_stage_ms waits for the
 * last recorded search and returns the MEAN duration in milliseconds of each stage over
 * the recorded searches.
 *   out_ms: host, [10]: rotate, query_prep, coarse GEMM, probe select, list build, seed,
 *           scan set-up (work-item offsets), scan (all its kernels), merge, and the estimate kernel of a split scan
 *           ("scan_impl" 4; part of the scan's time, 0 when the scan was not split); each is the time between two events on the
 *           stream the stage ran on, so with "overlap" their sum exceeds the duration of the search
 *   out_calls: host, number of searches the means were taken over (may be NULL)
 * Errors: RABITQ_EINVAL (null pointer, nothing recorded), RABITQ_EHIP. */
int rabitq_stage_ms(rabitq_index_t index, float* out_ms, int32_t* out_calls);

/* ---- Stage-level entry points: the same kernels rabitq_search chains, with every
 * buffer supplied by the caller (device pointers).  They exist so that each stage can
 * be checked and profiled with the previous stage's reference output injected. ---- */

/* Section 3.3.1: q_rot [nq*D] = (queries [nq*D] - mean) x P (fp32 MFMA; mean = 0 unless the index is centred). */
int rabitq_rotate(rabitq_index_t index, const float* queries, int64_t nq, float* q_rot, void* stream);

/* Section 3.3.3 / 3.4.1(2): the per-query representation, computed once per query and
 * reused by all of its cluster scans.  All members are DEVICE pointers supplied by the caller.
 *   planes   [nq][4][W] u32 two's-complement bit-planes of qhat (plane 3 weighs -8)
 *   delta    [nq] fp32  = max|q'|/7 (1 if q' == 0);  qhat = clamp(rint(q'/delta),-7,7)
 *   sum_qhat [nq] i32   = S;   sum_q [nq] fp32 = sum(q');   sq_norm [nq] fp32 = ||q'||^2
 *   qhat8    [nq][rabitq_qhat_stride(D)] i8: qhat as bytes, zero padded to a multiple of 64 dimensions (the
 *            operand of the matrix-core variant of the scan), in the order that variant's expansion of the sign bits
 *            produces: within every chunk of 64 dimensions, dimension 32 w + 8 b + 4 h + i (w, h in 0..1, b, i in
 *            0..3) sits at byte 16 (2 w + h) + 4 i + b
 *   q_stage  [nq][D] fp32: q' in the order the refinement reads it (within each long-code
 *            word, dimension b*(8/F)+s of the word sits at position 4*s+b; identity if B == 1)
 *   lut      [nq][D/4][16] binary16 bit patterns, or NULL (then not written; required by
 *            "scan_impl" 2): the lookup tables of Section 3.4.1(1) with U = 4,
 *            L_j(b) = sum of the q'[4j+i] whose bit i of b is set, summed in fp32 in ascending
 *            i and rounded to binary16 */
typedef struct {
  uint32_t* planes;
  float* delta;
  int32_t* sum_qhat;
  float* sum_q;
  float* sq_norm;
  int8_t* qhat8;
  float* q_stage;
  uint16_t* lut;
} rabitq_query_repr;
int32_t rabitq_qhat_stride(int32_t dim); /* = dim rounded up to a multiple of 64 */
int rabitq_query_prep(rabitq_index_t index, const float* q_rot, int64_t nq, const rabitq_query_repr* out,
                      void* stream);

/* Section 3.3.2: coarse scores by one GEMM (s_q 1^T + 1 s_c^T - 2 Q'C^T for L2, -Q'C^T
 * for IP) and the nprobe best clusters per query, best first, ties to the lower id.
 *   scores    [nq*nlist] fp32 scratch (the full score matrix)
 *   probe_ids [nq*nprobe] i32, probe_G [nq*nprobe] fp32 (the score), probe_E fp32 (||q'-c'||) */
int rabitq_coarse_probe(rabitq_index_t index, const float* q_rot, const float* sq_norm, int64_t nq,
                        int32_t nprobe, float* scores, int32_t* probe_ids, float* probe_G, float* probe_E,
                        void* stream);
/* The top-nprobe selection of Section 3.3.2 has several kernels; this names the one rabitq_coarse_probe and
 * rabitq_search launch for an index of nlist lists (so that tests can show each of them was exercised):
 * 0 = one wavefront per query streams the score row through a register-resident sorted list (nprobe <= 64);
 * 1, 2, 3 = one wavefront per query, whole row in registers, nlist <= 512 / 1024 / 2048 (nprobe > 64);
 * 4 = one workgroup per query, radix select in LDS (nprobe > 64, nlist > 2048).  Negative status if out of range. */
int32_t rabitq_probe_select_variant(int32_t nlist, int32_t nprobe);

/* Section 3.3.3: regroup the (query, cluster) pairs by cluster (stable in query id).
 *   pair_off [nlist+1] i32: pairs of cluster c are pair_ids[pair_off[c] .. pair_off[c+1])
 *   pair_ids [nq*nprobe] i32: pair p = query*nprobe + rank
 *   scratch  u32, at least rabitq_probe_list_scratch_words(nlist, nq) words */
int64_t rabitq_probe_list_scratch_words(int32_t nlist, int64_t nq);
int rabitq_build_probe_lists(rabitq_index_t index, const int32_t* probe_ids, int64_t nq, int32_t nprobe,
                             int32_t* pair_off, int32_t* pair_ids, uint32_t* scratch, void* stream);

/* Section 3.3.4 threshold: tau [nq] fp32.  In the query's nearest probed cluster with at
 * least k vectors, the max(k, 32) vectors with the smallest 1-bit estimates (ties: lower
 * position; all vectors if the cluster has fewer) are refined and tau is the k-th smallest
 * refined estimate (B == 1: the k-th smallest 1-bit estimate); FLT_MAX when no probed
 * cluster has k vectors. */
int rabitq_seed_threshold(rabitq_index_t index, const rabitq_query_repr* repr, const int32_t* probe_ids,
                          const float* probe_G, const float* probe_E, int64_t nq, int32_t k, int32_t nprobe,
                          float* tau, void* stream);

/* Sections 3.3.4, 3.4.1(2), 3.4.2: the fused cluster-local search over all pairs.
 * For every pair: 1-bit estimate of every vector of the cluster (see option "scan_impl"), filter
 * (B > 1: lb1 <= tau, B == 1: est1 <= tau), refinement of survivors, cluster-local top-k.
 *   tau        [nq] fp32 (pass FLT_MAX everywhere to disable the filter)
 *   cand_keys  [nq*nprobe*cap] u64, cap = rabitq_cand_capacity(k): (order-preserving bits of
 *              the key << 32) | id.  Pair p owns the cap-slot region starting at p*cap.
 *   cand_cnt   [nq*nprobe] i32: valid entries of each pair's region (unsorted).  A region
 *              holds every surviving key of the pair unless more than cap-16 survived, in
 *              which case it holds at least the k best of them.
 *   dbg_ip     optional (may be NULL) [sum over pairs, in pair_ids order, of 64*tiles(c)] i32:
 *              raw integer <x_b, qhat> of every slot (scan_impl 2: the bits of the fp32 table sum
 *              <x_b, q'>); dbg_off [nq*nprobe+1] i64 gives each
 *              pair's first entry (indexed by position in pair_ids).  For small inputs. */
int32_t rabitq_cand_capacity(int32_t k); /* = smallest power of two >= k + 64; negative status if k is out of range */
int rabitq_scan(rabitq_index_t index, const rabitq_query_repr* repr, const float* probe_G, const float* probe_E,
                const int32_t* pair_off, const int32_t* pair_ids, const float* tau, int64_t nq, int32_t k,
                int32_t nprobe, uint64_t* cand_keys, int32_t* cand_cnt, int32_t* dbg_ip, const int64_t* dbg_off,
                void* stream);

/* Section 3.3.5: per-query merge of the nprobe local lists into the final top-k. */
int rabitq_merge(rabitq_index_t index, const uint64_t* cand_keys, const int32_t* cand_cnt, int64_t nq, int32_t k,
                 int32_t nprobe, int64_t* out_ids, float* out_dists, void* stream);

/* Text of the last error raised on the calling thread ("" if none). */
const char* rabitq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RABITQ_H */
