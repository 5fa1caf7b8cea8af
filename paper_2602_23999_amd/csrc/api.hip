// C ABI of librabitq_hip.so: handle management, argument checks, workspace, and the
// chaining of the stage kernels on the caller's stream.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "rq_internal.h"

namespace rq {

static thread_local std::string g_err;

// Search workspace of rabitq_search_noalloc: one array per device, held until the process ends.  The name is a
// host-side stand-in; the device address is looked up once per device (noalloc_scratch) and only that address is
// ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[RABITQ_NOALLOC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static unsigned char* g_scratch_ptr[MAX_DEVICES] = {nullptr};
static std::mutex g_scratch_mu;

void set_error(const std::string& s) { g_err = s; }

int hip_fail(hipError_t e, const char* what) {
  g_err = std::string(what) + ": " + hipGetErrorString(e);
  return RABITQ_EHIP;
}

static int field_bits_of(int B) {  // long-code field width: B rounded up to 2, 4, 8 (0: no long code)
  if (B <= 1) return 0;
  if (B <= 2) return 2;
  if (B <= 4) return 4;
  return 8;
}

template <typename T>
static int dev_alloc(T** p, int64_t count) {
  *p = nullptr;
  if (count <= 0) count = 1;
  hipError_t e = hipMalloc(reinterpret_cast<void**>(p), (size_t)count * sizeof(T));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    set_error("hipMalloc failed: " + std::string(hipGetErrorString(e)));
    return RABITQ_ENOMEM;
  }
  return RABITQ_OK;
}

template <typename T>
static void dev_free(T*& p) {
  if (p) (void)hipFree(p);
  p = nullptr;
}

static void free_workspace(Workspace& w) {
  dev_free(w.q_rot); dev_free(w.repr.planes); dev_free(w.repr.delta); dev_free(w.repr.sum_qhat);
  dev_free(w.repr.sum_q); dev_free(w.repr.sq_norm); dev_free(w.repr.qhat8); dev_free(w.repr.q_stage); dev_free(w.repr.lut); dev_free(w.tau); dev_free(w.scores); dev_free(w.probe_ids); dev_free(w.probe_G);
  dev_free(w.probe_E); dev_free(w.pair_off); dev_free(w.pair_ids); dev_free(w.list_scratch);
  dev_free(w.cand_keys); dev_free(w.cand_cnt);
  w.cap_nq = w.cap_pairs = w.cap_cand = w.cap_scratch = w.cap_lut = 0;
}

static void free_index(rabitq_index* ix) {
  if (!ix) return;
  dev_free(ix->rotation); dev_free(ix->mean_rot); dev_free(ix->centroids_t); dev_free(ix->centroid_sq); dev_free(ix->tile_off); dev_free(ix->surv_mask); dev_free(ix->item_desc);
  dev_free(ix->cluster_size); dev_free(ix->cluster_order); dev_free(ix->short_codes); dev_free(ix->short_factors); dev_free(ix->long_codes);
  dev_free(ix->long_factors); dev_free(ix->ids);
  free_workspace(ix->ws);
  for (auto& set : ix->prof_sets) {
    for (auto& e : set.b)
      if (e) (void)hipEventDestroy(e);
    for (auto& e : set.e)
      if (e) (void)hipEventDestroy(e);
  }
  if (ix->ev_fork) (void)hipEventDestroy(ix->ev_fork);
  if (ix->ev_join) (void)hipEventDestroy(ix->ev_join);
  if (ix->side) (void)hipStreamDestroy(ix->side);
  delete ix;
}

// Grow the handle's workspace for (nq, nprobe, k).  Growth frees and reallocates
// (device-synchronising); steady-state calls allocate nothing.
static int ensure_workspace(rabitq_index* ix, int64_t nq, int nprobe, int k) {
  Workspace& w = ix->ws;
  const int64_t pairs = nq * nprobe;
  int cap = 1;
  while (cap < k + TILE) cap <<= 1;
  const int64_t cand = pairs * cap;
  const int64_t scratch = probe_list_scratch_words(ix->nlist, nq);
  const bool want_lut = ix->scan_impl == 2;  // lookup tables only exist once the lookup-table scan is selected
  if (nq <= w.cap_nq && pairs <= w.cap_pairs && cand <= w.cap_cand && scratch <= w.cap_scratch &&
      (!want_lut || nq <= w.cap_lut))
    return RABITQ_OK;
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) return hip_fail(e, "hipDeviceSynchronize");
  const int64_t c_nq = std::max(nq, w.cap_nq), c_pairs = std::max(pairs, w.cap_pairs);
  const int64_t c_cand = std::max(cand, w.cap_cand), c_scr = std::max(scratch, w.cap_scratch);
  free_workspace(w);
  int rc;
#define RQ_A(ptr, cnt) if ((rc = dev_alloc(&(ptr), (cnt))) != RABITQ_OK) { free_workspace(w); return rc; }
  RQ_A(w.q_rot, c_nq * ix->dim);
  RQ_A(w.repr.planes, c_nq * 4 * ix->W);
  RQ_A(w.repr.delta, c_nq);
  RQ_A(w.repr.sum_qhat, c_nq);
  RQ_A(w.repr.sum_q, c_nq);
  RQ_A(w.repr.sq_norm, c_nq);
  RQ_A(w.repr.qhat8, c_nq * qhat_stride(ix->dim));
  RQ_A(w.repr.q_stage, c_nq * ix->dim);
  if (want_lut) RQ_A(w.repr.lut, c_nq * ix->dim * 4);
  RQ_A(w.tau, c_nq);
  RQ_A(w.scores, c_nq * ix->nlist);
  RQ_A(w.probe_ids, c_pairs);
  RQ_A(w.probe_G, c_pairs);
  RQ_A(w.probe_E, c_pairs);
  RQ_A(w.pair_off, ix->nlist + 1);
  RQ_A(w.pair_ids, c_pairs);
  RQ_A(w.list_scratch, c_scr);
  RQ_A(w.cand_keys, c_cand);
  RQ_A(w.cand_cnt, c_pairs);
#undef RQ_A
  w.cap_nq = c_nq; w.cap_pairs = c_pairs; w.cap_cand = c_cand; w.cap_scratch = c_scr;
  w.cap_lut = want_lut ? c_nq : 0;
  return RABITQ_OK;
}

// Largest number of queries one pass may take: the "max_batch" option, else as many as keep the per-query part
// of the workspace (coarse scores, pair arrays, candidate keys, query representation) under WORKSPACE_BUDGET
// bytes, and never so many that the pair index leaves 31 bits.
constexpr int64_t WORKSPACE_BUDGET = (int64_t)16 << 30;
static int64_t search_batch_limit(const rabitq_index* ix, int k, int nprobe) {
  int cap = 1;
  while (cap < k + TILE) cap <<= 1;
  const int64_t per_query = (int64_t)ix->nlist * 4 + (int64_t)nprobe * ((int64_t)cap * 8 + 20) +
                            (int64_t)ix->dim * 10 + (int64_t)ix->nlist / 4 + 64;
  int64_t lim = std::max<int64_t>(256, WORKSPACE_BUDGET / per_query);
  if (ix->max_batch > 0) lim = ix->max_batch;
  return std::max<int64_t>(1, std::min<int64_t>(lim, 0x7fffffff / nprobe));
}


// Address of the current device's copy of `scratch`; `dev` must be the current device.  Looked up once per device.
static int noalloc_scratch(int dev, unsigned char** out) {
  if (dev < 0 || dev >= MAX_DEVICES) { set_error("device index out of range"); return RABITQ_EINVAL; }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p) { set_error("hipGetSymbolAddress(scratch) returned a null address"); return RABITQ_EHIP; }
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return RABITQ_OK;
}

// Lays the buffers of one search of (nq, nprobe, k) out behind `base`, each at a multiple of 256 bytes, and
// returns the bytes they take; base == nullptr only measures.  Nothing is allocated.
static size_t carve_workspace(const rabitq_index* ix, int64_t nq, int nprobe, int k, unsigned char* base, Workspace* w) {
  size_t off = 0;
  auto take = [&](auto** p, int64_t count) {
    using T = std::remove_pointer_t<std::remove_pointer_t<decltype(p)>>;
    if (base && p) *p = reinterpret_cast<T*>(base + off);
    off += (((size_t)std::max<int64_t>(count, 1) * sizeof(T)) + 255) / 256 * 256;
  };
  const int64_t pairs = nq * nprobe;
  int cap = 1;
  while (cap < k + TILE) cap <<= 1;
  Workspace dummy;
  Workspace& x = w ? *w : dummy;
  take(&x.q_rot, nq * ix->dim);
  take(&x.repr.planes, nq * 4 * ix->W);
  take(&x.repr.delta, nq);
  take(&x.repr.sum_qhat, nq);
  take(&x.repr.sum_q, nq);
  take(&x.repr.sq_norm, nq);
  take(&x.repr.qhat8, nq * qhat_stride(ix->dim));
  take(&x.repr.q_stage, nq * ix->dim);
  if (ix->scan_impl == 2) take(&x.repr.lut, nq * ix->dim * 4);
  take(&x.tau, nq);
  take(&x.scores, nq * ix->nlist);
  take(&x.probe_ids, pairs);
  take(&x.probe_G, pairs);
  take(&x.probe_E, pairs);
  take(&x.pair_off, (int64_t)ix->nlist + 1);
  take(&x.pair_ids, pairs);
  take(&x.list_scratch, probe_list_scratch_words(ix->nlist, nq));
  take(&x.cand_keys, pairs * cap);
  take(&x.cand_cnt, pairs);
  return off;
}

// second stream (default priority) and fork / join events of a handle; called once when the handle is made,
// with the handle's device current
static int init_streams(rabitq_index* ix) {
  RQ_HIP(hipStreamCreateWithFlags(&ix->side, hipStreamNonBlocking));
  RQ_HIP(hipEventCreateWithFlags(&ix->ev_fork, hipEventDisableTiming));
  RQ_HIP(hipEventCreateWithFlags(&ix->ev_join, hipEventDisableTiming));
  ix->seg_sorted.reserve(ix->host_tiles.size());  // so that a search never grows a host vector either
  {
    // clusters by descending length: the order in which a scan that reads every list once hands them out (launch_scan)
    ix->max_tiles = 0;
    for (int32_t t : ix->host_tiles) ix->max_tiles = std::max(ix->max_tiles, t);
    std::vector<int32_t> order(ix->host_tiles.size());
    for (size_t c = 0; c < order.size(); ++c) order[c] = (int32_t)c;
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t x, int32_t y) { return ix->host_tiles[x] > ix->host_tiles[y]; });
    if (int rc = dev_alloc(&ix->cluster_order, (int64_t)order.size())) return rc;
    if (!order.empty())
      RQ_HIP(hipMemcpy(ix->cluster_order, order.data(), order.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  }
  unsigned char* sp = nullptr;  // the allocation-free search's workspace on this device
  return noalloc_scratch(ix->device, &sp);
}

int set_index_mean(rabitq_index* ix, const float* mean, const float* rotation_host, hipStream_t st) {
  const int D = ix->dim;
  bool any = false;
  for (int i = 0; i < D; ++i) any = any || mean[i] != 0.f;
  if (!any) return RABITQ_OK;
  if (ix->metric != RABITQ_L2) { set_error("a centred index needs the L2 metric"); return RABITQ_EINVAL; }
  ix->host_mean.assign(mean, mean + D);
  std::vector<float> mr(D);
  for (int j = 0; j < D; ++j) {
    double s = 0.0;
    for (int i = 0; i < D; ++i) s += (double)mean[i] * (double)rotation_host[(size_t)i * D + j];
    mr[j] = (float)s;
  }
  int rc = dev_alloc(&ix->mean_rot, (int64_t)D);
  if (rc != RABITQ_OK) return rc;
  RQ_HIP(hipMemcpyAsync(ix->mean_rot, mr.data(), (size_t)D * sizeof(float), hipMemcpyHostToDevice, st));
  RQ_HIP(hipStreamSynchronize(st));  // mr dies at return
  return RABITQ_OK;
}

int launch_rotate(const rabitq_index* ix, const float* q, float* q_rot, int64_t nq, hipStream_t st) {
  return launch_gemm(q, ix->rotation, q_rot, nq, ix->dim, ix->dim, ix->mean_rot ? 4 : 0, nullptr, ix->mean_rot, st);
}

}  // namespace rq

using namespace rq;

extern "C" {

const char* rabitq_last_error(void) { return g_err.c_str(); }

// the scan kernels are instantiated for these code widths (dim / 32)
static bool width_supported(int dim) {
  const int W = dim / 32;
  return W == 1 || W == 2 || W == 3 || W == 4 || W == 8 || W == 16 || W == 24 || W == 30 || W == 32;
}
static const char* kWidthMsg = "dim must be one of 32, 64, 96, 128, 256, 512, 768, 960, 1024 in this build";

int rabitq_index_upload(const rabitq_index_desc* d, rabitq_index_t* out, void* stream) {
  if (!d || !out) { set_error("upload: null argument"); return RABITQ_EINVAL; }
  if (d->dim < 32 || d->dim > 2048 || (d->dim % 32) != 0) { set_error("upload: dim must be a multiple of 32 in 32..2048"); return RABITQ_EINVAL; }
  if (!width_supported(d->dim)) { set_error(std::string("upload: ") + kWidthMsg); return RABITQ_EINVAL; }
  if (d->nlist < 1 || d->n < 0) { set_error("upload: bad nlist or n"); return RABITQ_EINVAL; }
  if (d->total_bits < 1 || d->total_bits > 8) { set_error("upload: total_bits must be 1..8"); return RABITQ_EINVAL; }
  if (d->metric != RABITQ_L2 && d->metric != RABITQ_IP) { set_error("upload: bad metric"); return RABITQ_EINVAL; }
  if (!d->rotation || !d->centroids || !d->offsets || !d->short_codes || !d->short_factors || !d->ids) {
    set_error("upload: null array"); return RABITQ_EINVAL;
  }
  if (d->total_bits > 1 && (!d->long_codes || !d->long_factors)) { set_error("upload: long arrays required when total_bits > 1"); return RABITQ_EINVAL; }
  const int D = d->dim, nlist = d->nlist, W = D / 32;
  if (d->offsets[0] != 0 || d->offsets[nlist] != d->n) { set_error("upload: offsets[0] must be 0 and offsets[nlist] == n"); return RABITQ_EINVAL; }
  std::vector<int32_t> tile_off(nlist + 1), csize(nlist);
  int64_t tiles = 0;
  for (int c = 0; c < nlist; ++c) {
    const int64_t nc = d->offsets[c + 1] - d->offsets[c];
    if (nc < 0 || nc > 0x7fffffff) { set_error("upload: offsets not monotone"); return RABITQ_EINVAL; }
    tile_off[c] = (int32_t)tiles;
    csize[c] = (int32_t)nc;
    tiles += (nc + TILE - 1) / TILE;
    if (tiles > (0x7fffffff / TILE)) { set_error("upload: too many slots for 32-bit slot indices"); return RABITQ_EINVAL; }
  }
  tile_off[nlist] = (int32_t)tiles;

  rabitq_index* ix = new (std::nothrow) rabitq_index();
  if (!ix) { set_error("upload: out of host memory"); return RABITQ_ENOMEM; }
  ix->dim = D; ix->W = W; ix->nlist = nlist; ix->n = d->n; ix->total_bits = d->total_bits; ix->metric = d->metric;
  ix->F = field_bits_of(d->total_bits);
  ix->LW = D * ix->F / 32;
  ix->n_tiles = tiles; ix->n_slots = tiles * TILE;
  ix->host_tiles.resize(nlist);
  for (int c = 0; c < nlist; ++c) ix->host_tiles[c] = tile_off[c + 1] - tile_off[c];
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = RABITQ_OK;
  hipError_t he = hipGetDevice(&ix->device);
  if (he != hipSuccess) { rc = hip_fail(he, "hipGetDevice"); free_index(ix); return rc; }

  // transposed centroids [D][nlist] and their squared norms
  std::vector<float> ct((size_t)D * nlist), csq(nlist);
  for (int c = 0; c < nlist; ++c) {
    double s = 0.0;
    for (int i = 0; i < D; ++i) {
      const float v = d->centroids[(size_t)c * D + i];
      ct[(size_t)i * nlist + c] = v;
      s += (double)v * (double)v;
    }
    csq[c] = (float)s;
  }
#define RQ_UP(dst, src, cnt, T)                                                                     \
  if (rc == RABITQ_OK) rc = dev_alloc(&(dst), (int64_t)(cnt));                                       \
  if (rc == RABITQ_OK && (cnt) > 0) {                                                                \
    he = hipMemcpyAsync((dst), (src), (size_t)(cnt) * sizeof(T), hipMemcpyHostToDevice, st);         \
    if (he != hipSuccess) rc = hip_fail(he, "hipMemcpyAsync");                                       \
  }
  RQ_UP(ix->rotation, d->rotation, (int64_t)D * D, float);
  RQ_UP(ix->centroids_t, ct.data(), (int64_t)D * nlist, float);
  RQ_UP(ix->centroid_sq, csq.data(), nlist, float);
  if (rc == RABITQ_OK) rc = dev_alloc(&ix->tile_off, tile_off_words(nlist));  // + scan work-item offsets + ticket
  if (rc == RABITQ_OK) {
    he = hipMemsetAsync(ix->tile_off, 0, (size_t)tile_off_words(nlist) * sizeof(int32_t), st);
    if (he == hipSuccess)
      he = hipMemcpyAsync(ix->tile_off, tile_off.data(), (size_t)(nlist + 1) * sizeof(int32_t), hipMemcpyHostToDevice, st);
    if (he != hipSuccess) rc = hip_fail(he, "hipMemcpyAsync");
  }
  RQ_UP(ix->cluster_size, csize.data(), nlist, int32_t);
  RQ_UP(ix->short_codes, d->short_codes, tiles * W * TILE, uint32_t);
  RQ_UP(ix->short_factors, d->short_factors, tiles * 3 * TILE, float);
  RQ_UP(ix->ids, d->ids, tiles * TILE, int32_t);
  if (d->total_bits > 1) {
    RQ_UP(ix->long_codes, d->long_codes, tiles * TILE * ix->LW, uint32_t);
    RQ_UP(ix->long_factors, d->long_factors, tiles * TILE * 2, float);
  }
#undef RQ_UP
  if (rc == RABITQ_OK) {
    he = hipStreamSynchronize(st);  // host staging vectors die at return
    if (he != hipSuccess) rc = hip_fail(he, "hipStreamSynchronize");
  } else {
    (void)hipStreamSynchronize(st);
  }
  if (rc == RABITQ_OK && d->mean) rc = set_index_mean(ix, d->mean, d->rotation, st);
  if (rc == RABITQ_OK) rc = init_streams(ix);
  if (rc != RABITQ_OK) { free_index(ix); return rc; }
  *out = ix;
  return RABITQ_OK;
}

int rabitq_index_build(const rabitq_build_params* p, const float* data, rabitq_index_t* out, void* stream) {
  if (!p || !out) { set_error("build: null argument"); return RABITQ_EINVAL; }
  if (p->dim < 32 || p->dim > 2048 || (p->dim % 32) != 0) { set_error("build: dim must be a multiple of 32 in 32..2048"); return RABITQ_EINVAL; }
  if (!width_supported(p->dim)) { set_error(std::string("build: ") + kWidthMsg); return RABITQ_EINVAL; }
  if (p->nlist < 1 || p->n < 0 || p->n > 0x7fffffff) { set_error("build: bad nlist or n"); return RABITQ_EINVAL; }
  if (p->total_bits < 1 || p->total_bits > 8) { set_error("build: total_bits must be 1..8"); return RABITQ_EINVAL; }
  if (p->metric != RABITQ_L2 && p->metric != RABITQ_IP) { set_error("build: bad metric"); return RABITQ_EINVAL; }
  if (p->kmeans_iters < 0 || !(p->epsilon0 >= 0.f)) { set_error("build: bad kmeans_iters or epsilon0"); return RABITQ_EINVAL; }
  if (!p->rotation || (!data && p->n > 0)) { set_error("build: null array"); return RABITQ_EINVAL; }
  if (p->center != 0 && p->center != 1) { set_error("build: center must be 0 or 1"); return RABITQ_EINVAL; }
  if (p->center && p->metric != RABITQ_L2) { set_error("build: a centred index needs the L2 metric"); return RABITQ_EINVAL; }
  rabitq_index* ix = new (std::nothrow) rabitq_index();
  if (!ix) { set_error("build: out of host memory"); return RABITQ_ENOMEM; }
  ix->dim = p->dim; ix->W = p->dim / 32; ix->nlist = p->nlist; ix->n = p->n; ix->total_bits = p->total_bits;
  ix->metric = p->metric; ix->F = field_bits_of(p->total_bits); ix->LW = p->dim * ix->F / 32;
  hipError_t he = hipGetDevice(&ix->device);
  int rc = (he == hipSuccess) ? RABITQ_OK : hip_fail(he, "hipGetDevice");
  if (rc == RABITQ_OK)
    rc = build_index_device(ix, data, p->rotation, p->kmeans_iters, p->train_size, p->epsilon0, p->center,
                            (hipStream_t)stream);
  if (rc == RABITQ_OK) rc = init_streams(ix);
  if (rc != RABITQ_OK) {
    (void)hipDeviceSynchronize();
    free_index(ix);
    return rc;
  }
  *out = ix;
  return RABITQ_OK;
}

int rabitq_index_export(rabitq_index_t ix, float* rotation, float* centroids, int64_t* offsets, uint32_t* short_codes,
                        float* short_factors, uint32_t* long_codes, float* long_factors, int32_t* ids, float* mean) {
  if (!ix) { set_error("export: null index"); return RABITQ_EINVAL; }
  if (mean)
    for (int i = 0; i < ix->dim; ++i) mean[i] = ix->host_mean.empty() ? 0.f : ix->host_mean[i];
  RQ_HIP(hipDeviceSynchronize());
  const int D = ix->dim, nlist = ix->nlist;
  const int64_t slots = ix->n_slots, tiles = ix->n_tiles;
  if (rotation) RQ_HIP(hipMemcpy(rotation, ix->rotation, (size_t)D * D * sizeof(float), hipMemcpyDeviceToHost));
  if (centroids) {
    std::vector<float> ct((size_t)D * nlist);
    RQ_HIP(hipMemcpy(ct.data(), ix->centroids_t, ct.size() * sizeof(float), hipMemcpyDeviceToHost));
    for (int c = 0; c < nlist; ++c)
      for (int i = 0; i < D; ++i) centroids[(size_t)c * D + i] = ct[(size_t)i * nlist + c];
  }
  if (offsets) {
    std::vector<int32_t> cs(nlist);
    RQ_HIP(hipMemcpy(cs.data(), ix->cluster_size, (size_t)nlist * sizeof(int32_t), hipMemcpyDeviceToHost));
    offsets[0] = 0;
    for (int c = 0; c < nlist; ++c) offsets[c + 1] = offsets[c] + cs[c];
  }
  if (short_codes && tiles) RQ_HIP(hipMemcpy(short_codes, ix->short_codes, (size_t)tiles * ix->W * TILE * 4, hipMemcpyDeviceToHost));
  if (short_factors && tiles) RQ_HIP(hipMemcpy(short_factors, ix->short_factors, (size_t)tiles * 3 * TILE * 4, hipMemcpyDeviceToHost));
  if (ids && slots) RQ_HIP(hipMemcpy(ids, ix->ids, (size_t)slots * 4, hipMemcpyDeviceToHost));
  if (ix->total_bits > 1) {
    if (long_codes && slots) RQ_HIP(hipMemcpy(long_codes, ix->long_codes, (size_t)slots * ix->LW * 4, hipMemcpyDeviceToHost));
    if (long_factors && slots) RQ_HIP(hipMemcpy(long_factors, ix->long_factors, (size_t)slots * 2 * 4, hipMemcpyDeviceToHost));
  }
  return RABITQ_OK;
}

int rabitq_index_free(rabitq_index_t ix) {
  if (!ix) return RABITQ_OK;
  (void)hipDeviceSynchronize();
  free_index(ix);
  return RABITQ_OK;
}

int rabitq_set_option(rabitq_index_t ix, const char* name, int64_t value) {
  if (!ix || !name) { set_error("set_option: null argument"); return RABITQ_EINVAL; }
  if (!std::strcmp(name, "prune") && (value == 0 || value == 1)) { ix->prune = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "scan_impl") && value >= 0 && value <= 4) { ix->scan_impl = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "split_min_pairs") && value >= 0 && value <= 0x7fffffff) { ix->split_min_pairs = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "overlap") && (value == 0 || value == 1)) { ix->overlap = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "max_batch") && value >= 0 && value <= 0x7fffffff) { ix->max_batch = value; return RABITQ_OK; }
  if (!std::strcmp(name, "small_batch") && (value == 0 || value == 1)) { ix->small_batch = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "longest_first") && (value == 0 || value == 1)) { ix->longest_first = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "scan_segment_tiles") && value >= 0 && value <= 4096) { ix->seg_tiles = (int)value; return RABITQ_OK; }
  if (!std::strcmp(name, "profile_stages") && value >= 1 && value <= 0x3ff) {
    ix->prof_mask = (unsigned)value;
    ix->prof_used = 0;
    return RABITQ_OK;
  }
  if (!std::strcmp(name, "profile") && value >= 0 && value <= 4096) {
    const size_t have = ix->prof_sets.size();
    if ((size_t)value > have) {
      ix->prof_sets.resize((size_t)value);
      for (size_t i = have; i < (size_t)value; ++i)
        for (int s2 = 0; s2 < rabitq_index::N_STAGES; ++s2) ix->prof_sets[i].b[s2] = ix->prof_sets[i].e[s2] = nullptr;
      for (size_t i = have; i < (size_t)value; ++i) ix->prof_sets[i].rec = 0;
      for (size_t i = have; i < (size_t)value; ++i)
        for (int s2 = 0; s2 < rabitq_index::N_STAGES; ++s2) {
          RQ_HIP(hipEventCreate(&ix->prof_sets[i].b[s2]));
          RQ_HIP(hipEventCreate(&ix->prof_sets[i].e[s2]));
        }
    }
    ix->prof_used = 0;
    ix->prof_limit = (int)value;
    return RABITQ_OK;
  }
  set_error("set_option: unknown option or value");
  return RABITQ_EINVAL;
}

int64_t rabitq_index_info(rabitq_index_t ix, const char* name) {
  if (!ix || !name) { set_error("index_info: null argument"); return RABITQ_EINVAL; }
  if (!std::strcmp(name, "n")) return ix->n;
  if (!std::strcmp(name, "n_tiles")) return ix->n_tiles;
  if (!std::strcmp(name, "n_slots")) return ix->n_slots;
  if (!std::strcmp(name, "dim")) return ix->dim;
  if (!std::strcmp(name, "nlist")) return ix->nlist;
  if (!std::strcmp(name, "total_bits")) return ix->total_bits;
  if (!std::strcmp(name, "long_field_bits")) return ix->F;
  if (!std::strcmp(name, "metric")) return ix->metric;
  if (!std::strcmp(name, "last_scan_split")) return ix->last_scan_split;
  if (!std::strcmp(name, "last_scan_stream")) return ix->last_scan_stream;
  set_error("index_info: unknown name");
  return RABITQ_EINVAL;
}

int rabitq_stage_ms(rabitq_index_t ix, float* out_ms, int32_t* out_calls) {
  if (!ix || !out_ms) { set_error("stage_ms: null argument"); return RABITQ_EINVAL; }
  const int n = ix->prof_used;
  if (n <= 0) { set_error("stage_ms: no search was recorded (set the option \"profile\" first)"); return RABITQ_EINVAL; }
  double acc[rabitq_index::N_STAGES] = {0};
  for (int s = 0; s < rabitq_index::N_STAGES; ++s) {
    if (!((ix->prof_mask >> s) & 1u)) continue;  // not recorded: reported as 0
    for (int i = 0; i < n; ++i) {
      if (!((ix->prof_sets[i].rec >> s) & 1u)) continue;  // this search ran the stage inside another one's kernel
      RQ_HIP(hipEventSynchronize(ix->prof_sets[i].e[s]));
      float ms = 0.f;
      RQ_HIP(hipEventElapsedTime(&ms, ix->prof_sets[i].b[s], ix->prof_sets[i].e[s]));
      acc[s] += ms;
    }
  }
  for (int s = 0; s < rabitq_index::N_STAGES; ++s) out_ms[s] = (float)(acc[s] / n);
  if (out_calls) *out_calls = n;
  return RABITQ_OK;
}

static int check_common(rabitq_index_t ix, int64_t nq, const char* who) {
  if (!ix) { set_error(std::string(who) + ": null index"); return RABITQ_EINVAL; }
  if (nq < 0) { set_error(std::string(who) + ": nq < 0"); return RABITQ_EINVAL; }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != ix->device) {  // the handle's arrays live on one device
    set_error(std::string(who) + ": the current device is not the one the index was created on");
    return RABITQ_EINVAL;
  }
  return RABITQ_OK;
}

static int check_k_nprobe(rabitq_index_t ix, int k, int nprobe, const char* who) {
  if (k < 1 || k > RABITQ_MAX_K) { set_error(std::string(who) + ": k must be in 1..128"); return RABITQ_EINVAL; }
  if (nprobe < 1 || nprobe > ix->nlist || nprobe > RABITQ_MAX_NPROBE) {
    set_error(std::string(who) + ": nprobe must be in 1..min(nlist,1024)");
    return RABITQ_EINVAL;
  }
  return RABITQ_OK;
}

int rabitq_rotate(rabitq_index_t ix, const float* queries, int64_t nq, float* q_rot, void* stream) {
  int rc = check_common(ix, nq, "rotate");
  if (rc) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!queries || !q_rot) { set_error("rotate: null pointer"); return RABITQ_EINVAL; }
  return launch_rotate(ix, queries, q_rot, nq, (hipStream_t)stream);
}

static bool repr_ok(const rabitq_query_repr* r) {
  return r && r->planes && r->delta && r->sum_qhat && r->sum_q && r->sq_norm && r->qhat8 && r->q_stage;
}

int32_t rabitq_qhat_stride(int32_t dim) { return dim < 1 ? RABITQ_EINVAL : qhat_stride(dim); }

int rabitq_query_prep(rabitq_index_t ix, const float* q_rot, int64_t nq, const rabitq_query_repr* out, void* stream) {
  int rc = check_common(ix, nq, "query_prep");
  if (rc) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!q_rot || !repr_ok(out)) { set_error("query_prep: null pointer"); return RABITQ_EINVAL; }
  return launch_query_prep(q_rot, nq, ix->dim, ix->F, *out, (hipStream_t)stream);
}

int rabitq_coarse_probe(rabitq_index_t ix, const float* q_rot, const float* sq_norm, int64_t nq, int32_t nprobe,
                        float* scores, int32_t* probe_ids, float* probe_G, float* probe_E, void* stream) {
  int rc = check_common(ix, nq, "coarse_probe");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, 1, nprobe, "coarse_probe"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!q_rot || !sq_norm || !scores || !probe_ids || !probe_G || !probe_E) { set_error("coarse_probe: null pointer"); return RABITQ_EINVAL; }
  hipStream_t st = (hipStream_t)stream;
  rc = launch_gemm(q_rot, ix->centroids_t, scores, nq, ix->nlist, ix->dim, ix->metric == RABITQ_L2 ? 1 : 2, sq_norm,
                   ix->centroid_sq, st);
  if (rc) return rc;
  return launch_select_probes(scores, sq_norm, ix->centroid_sq, nq, ix->nlist, nprobe, ix->metric, probe_ids, probe_G,
                              probe_E, st);
}

int32_t rabitq_probe_select_variant(int32_t nlist, int32_t nprobe) {
  if (nlist < 1 || nprobe < 1 || nprobe > nlist || nprobe > RABITQ_MAX_NPROBE) return RABITQ_EINVAL;
  return probe_select_variant(nlist, nprobe);
}

int32_t rabitq_cand_capacity(int32_t k) {
  if (k < 1 || k > RABITQ_MAX_K) return RABITQ_EINVAL;
  int cap = 1;
  while (cap < k + TILE) cap <<= 1;
  return cap;
}

int64_t rabitq_probe_list_scratch_words(int32_t nlist, int64_t nq) {
  if (nlist < 1 || nq < 0) return RABITQ_EINVAL;
  return probe_list_scratch_words(nlist, nq);
}

int rabitq_build_probe_lists(rabitq_index_t ix, const int32_t* probe_ids, int64_t nq, int32_t nprobe,
                             int32_t* pair_off, int32_t* pair_ids, uint32_t* scratch, void* stream) {
  int rc = check_common(ix, nq, "build_probe_lists");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, 1, nprobe, "build_probe_lists"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!probe_ids || !pair_off || !pair_ids || !scratch) { set_error("build_probe_lists: null pointer"); return RABITQ_EINVAL; }
  if (nq * nprobe > 0x7fffffff) { set_error("build_probe_lists: nq*nprobe exceeds 2^31-1"); return RABITQ_EINVAL; }
  return launch_build_lists(probe_ids, nq, nprobe, ix->nlist, pair_off, pair_ids, scratch, (hipStream_t)stream);
}

int rabitq_seed_threshold(rabitq_index_t ix, const rabitq_query_repr* repr, const int32_t* probe_ids,
                          const float* probe_G, const float* probe_E, int64_t nq, int32_t k, int32_t nprobe,
                          float* tau, void* stream) {
  int rc = check_common(ix, nq, "seed_threshold");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, k, nprobe, "seed_threshold"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!repr_ok(repr) || !probe_ids || !probe_G || !probe_E || !tau) { set_error("seed_threshold: null pointer"); return RABITQ_EINVAL; }
  return launch_seed(ix, *repr, probe_ids, probe_G, probe_E, nq, k, nprobe, tau, (hipStream_t)stream);
}

int rabitq_scan(rabitq_index_t ix, const rabitq_query_repr* repr, const float* probe_G, const float* probe_E,
                const int32_t* pair_off, const int32_t* pair_ids, const float* tau, int64_t nq, int32_t k,
                int32_t nprobe, uint64_t* cand_keys, int32_t* cand_cnt, int32_t* dbg_ip, const int64_t* dbg_off,
                void* stream) {
  int rc = check_common(ix, nq, "scan");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, k, nprobe, "scan"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!repr_ok(repr) || !probe_G || !probe_E || !pair_off || !pair_ids || !tau || !cand_keys || !cand_cnt ||
      (dbg_ip && !dbg_off)) {
    set_error("scan: null pointer"); return RABITQ_EINVAL;
  }
  if (nq * nprobe > 0x7fffffff) { set_error("scan: nq*nprobe exceeds 2^31-1"); return RABITQ_EINVAL; }
  if (split_wanted(ix, nq, nprobe))
    if ((rc = ensure_split_buffers(ix, nq, nprobe, k))) return rc;
  if ((rc = ensure_stream_buffers(ix, nq, nprobe, k))) return rc;
  ScanStreams ss;
  ss.main = ss.setup = (hipStream_t)stream;
  rc = launch_scan(ix, *repr, probe_G, probe_E, pair_off, pair_ids, tau, nq, k, nprobe, cand_keys, cand_cnt, dbg_ip,
                   dbg_off, ss);
  ix->last_scan_split = ss.split ? 1 : 0;
  ix->last_scan_stream = ss.streamed ? 1 : 0;
  return rc;
}

int rabitq_merge(rabitq_index_t ix, const uint64_t* cand_keys, const int32_t* cand_cnt, int64_t nq, int32_t k,
                 int32_t nprobe, int64_t* out_ids, float* out_dists, void* stream) {
  int rc = check_common(ix, nq, "merge");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, k, nprobe, "merge"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!cand_keys || !cand_cnt || !out_ids || !out_dists) { set_error("merge: null pointer"); return RABITQ_EINVAL; }
  return launch_merge(cand_keys, cand_cnt, nq, k, nprobe, ix->metric, out_ids, out_dists, (hipStream_t)stream);
}

}  // extern "C"

// One pass of the whole path over the queries `w` was sized for.  `forked` tells the caller whether the handle's
// second stream has work that the caller's stream has not waited for yet (only possible when an error is returned).
static int search_batch_body(rabitq_index* ix, Workspace& w, const float* queries, int64_t nq, int32_t k, int32_t nprobe,
                             int64_t* out_ids, float* out_dists, hipStream_t st, bool* forked) {
  int rc;
  rabitq_index::EventSet* ev = nullptr;  // event set of this call when it is being recorded
  if (ix->prof_used < ix->prof_limit) {
    ev = &ix->prof_sets[ix->prof_used++];
    ev->rec = 0;
  }
  // stage s runs between its begin and end events, both recorded on the stream the stage is put on
#define RQ_STAGE(s, stream_, call)                                              \
  do {                                                                          \
    const bool on_ = ev && ((ix->prof_mask >> (s)) & 1u);                       \
    if (on_) RQ_HIP(hipEventRecord(ev->b[s], (stream_)));                       \
    if (on_) ev->rec |= 1u << (s);                                              \
    if ((rc = (call)) != RABITQ_OK) return rc;                                  \
    if (on_) RQ_HIP(hipEventRecord(ev->e[s], (stream_)));                       \
  } while (0)
  // What needs no probes is cleared on the second stream while the probes are being computed (a large batch only:
  // for a small one the clears take no time and the extra dependency between the streams would only add latency).
  // The second stream pays off when the kernels are long enough: its events cost the host about 0.08 ms per search,
  // more than a whole search of a few queries takes on the GPU.
  const bool side_stream = ix->overlap && nq >= 256;
  const bool early_clear = side_stream && nq >= 2048;
  if (early_clear) {
    RQ_HIP(hipEventRecord(ix->ev_fork, st));
    RQ_HIP(hipStreamWaitEvent(ix->side, ix->ev_fork, 0));
    *forked = true;
    if ((rc = launch_clear_list_bitmap(nq, ix->nlist, w.list_scratch, ix->side)) != RABITQ_OK) return rc;
    if ((rc = launch_clear_counters(w.cand_cnt, nq * nprobe, ix->side)) != RABITQ_OK) return rc;
  }
  rabitq_query_repr repr = w.repr;
  if (ix->scan_impl != 2) repr.lut = nullptr;  // tables are only built for the scan that reads them
  // a small batch is bound by the number of dependent launches (Section 4.2.2): it takes fused kernels
  const bool small = ix->small_batch && nq <= SMALL_BATCH_MAX;
  if (small) {
    RQ_STAGE(0, st, launch_small_front(ix, queries, nq, w.q_rot, repr, w.scores, st));
  } else {
    RQ_STAGE(0, st, launch_rotate(ix, queries, w.q_rot, nq, st));
    RQ_STAGE(1, st, launch_query_prep(w.q_rot, nq, ix->dim, ix->F, repr, st));
    RQ_STAGE(2, st, launch_gemm(w.q_rot, ix->centroids_t, w.scores, nq, ix->nlist, ix->dim,
                                ix->metric == RABITQ_L2 ? 1 : 2, w.repr.sq_norm, ix->centroid_sq, st));
  }
  // ... and, when the per-query selections fit one wavefront, everything up to the scan from a second one
  const bool small_fused = small && nprobe <= 64 && k <= 64 && effective_impl(ix) != 2;
  if (small_fused) {
    RQ_STAGE(3, st, launch_small_select_seed(ix, w.repr, w.scores, nq, k, nprobe, w.probe_ids, w.probe_G, w.probe_E, w.tau,
                                             w.pair_off, w.pair_ids, w.list_scratch, w.cand_cnt, st));
  } else {
    RQ_STAGE(3, st, launch_select_probes(w.scores, w.repr.sq_norm, ix->centroid_sq, nq, ix->nlist, nprobe, ix->metric,
                                         w.probe_ids, w.probe_G, w.probe_E, st));
  }
  // The pair lists and the scan's work-item table depend on the probes only, and so does the threshold seeding:
  // the former run on the handle's second stream beside the latter, and the scan kernel waits for both.
  hipStream_t lst = st;
  if (side_stream) {
    lst = ix->side;
    RQ_HIP(hipEventRecord(ix->ev_fork, st));
    RQ_HIP(hipStreamWaitEvent(lst, ix->ev_fork, 0));
    *forked = true;
  }
  // a small batch takes its lists, work-item offsets and cleared counters from one single-workgroup kernel
  if (small_fused) {
    // lists, thresholds, work-item table and counters are already there
  } else if (small) {
    RQ_STAGE(4, lst, launch_small_batch_lists(ix, w.probe_ids, nq, nprobe, k, w.pair_off, w.pair_ids, w.list_scratch,
                                              w.cand_cnt, lst));
  } else {
    RQ_STAGE(4, lst, launch_build_lists(w.probe_ids, nq, nprobe, ix->nlist, w.pair_off, w.pair_ids, w.list_scratch, lst,
                                        early_clear));
  }
  // With one probed list and 1-bit codes the threshold would be the k-th smallest estimate of that very list: the
  // scan's own top-k selects the same vectors, so the seeding pass (a second read of the list) is left out.
  const bool seed = ix->prune && !(nprobe == 1 && ix->total_bits == 1);
  if (small_fused) {
  } else if (seed) {
    RQ_STAGE(5, st, launch_seed(ix, w.repr, w.probe_ids, w.probe_G, w.probe_E, nq, k, nprobe, w.tau, st));
  } else {
    RQ_STAGE(5, st, launch_fill_f32(w.tau, nq, 3.402823466e+38f, st));
  }
  ScanStreams ss;
  ss.main = st; ss.setup = lst; ss.join = ix->ev_join;
  ss.counters_clear = early_clear;
  ss.setup_done = small;
  ss.desc_done = small_fused;
  if (ev && ((ix->prof_mask >> 6) & 1u)) { ss.setup_b = ev->b[6]; ss.setup_e = ev->e[6]; ev->rec |= 1u << 6; }
  if (ev && ((ix->prof_mask >> 7) & 1u)) { ss.scan_b = ev->b[7]; ss.scan_e = ev->e[7]; ev->rec |= 1u << 7; }
  if (ev && ((ix->prof_mask >> 9) & 1u)) { ss.est_b = ev->b[9]; ss.est_e = ev->e[9]; }
  if ((rc = launch_scan(ix, w.repr, w.probe_G, w.probe_E, w.pair_off, w.pair_ids, w.tau, nq, k, nprobe, w.cand_keys,
                        w.cand_cnt, nullptr, nullptr, ss)) != RABITQ_OK)
    return rc;
  if (ss.est_b && ss.split) ev->rec |= 1u << 9;
  ix->last_scan_split = ss.split ? 1 : 0;
  ix->last_scan_stream = ss.streamed ? 1 : 0;
  RQ_STAGE(8, st, launch_merge(w.cand_keys, w.cand_cnt, nq, k, nprobe, ix->metric, out_ids, out_dists, st));
#undef RQ_STAGE
  return RABITQ_OK;
}

static int search_batch(rabitq_index* ix, Workspace& w, const float* queries, int64_t nq, int32_t k, int32_t nprobe,
                        int64_t* out_ids, float* out_dists, hipStream_t st) {
  bool forked = false;
  const int rc = search_batch_body(ix, w, queries, nq, k, nprobe, out_ids, out_dists, st, &forked);
  if (rc != RABITQ_OK && forked) {
    // An error left the second stream forked from the caller's: join it again, so that the caller's stream (and a
    // stream capture it may be part of) ends with no work outstanding elsewhere.  The first error is the one reported.
    const std::string first = g_err;
    if (hipEventRecord(ix->ev_join, ix->side) == hipSuccess) (void)hipStreamWaitEvent(st, ix->ev_join, 0);
    (void)hipGetLastError();
    g_err = first;
  }
  return rc;
}

extern "C" {

int rabitq_search(rabitq_index_t ix, const float* queries, int64_t nq, int32_t k, int32_t nprobe, int64_t* out_ids,
                  float* out_dists, void* stream) {
  int rc = check_common(ix, nq, "search");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, k, nprobe, "search"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!queries || !out_ids || !out_dists) { set_error("search: null pointer"); return RABITQ_EINVAL; }
  // Queries are independent of one another, so a batch whose workspace would be large is searched in
  // consecutive sub-batches through one workspace; the results do not depend on the split.
  const int64_t step = std::min(nq, search_batch_limit(ix, k, nprobe));
  if ((rc = ensure_workspace(ix, step, nprobe, k))) return rc;
  if (split_wanted(ix, step, nprobe))
    if ((rc = ensure_split_buffers(ix, step, nprobe, k))) return rc;
  if ((rc = ensure_stream_buffers(ix, step, nprobe, k))) return rc;
  for (int64_t s0 = 0; s0 < nq; s0 += step) {
    const int64_t m = std::min(step, nq - s0);
    if ((rc = search_batch(ix, ix->ws, queries + s0 * ix->dim, m, k, nprobe, out_ids + s0 * k, out_dists + s0 * k,
                           (hipStream_t)stream)))
      return rc;
  }
  return RABITQ_OK;
}

int rabitq_search_noalloc(rabitq_index_t ix, const float* queries, int64_t nq, int32_t k, int32_t nprobe,
                          int64_t* out_ids, float* out_dists, void* stream) {
  int rc = check_common(ix, nq, "search_noalloc");
  if (rc) return rc;
  if ((rc = check_k_nprobe(ix, k, nprobe, "search_noalloc"))) return rc;
  if (nq == 0) return RABITQ_OK;
  if (!queries || !out_ids || !out_dists) { set_error("search_noalloc: null pointer"); return RABITQ_EINVAL; }
  if (nq > 0x7fffffff / nprobe) { set_error("search_noalloc: nq*nprobe exceeds 2^31-1"); return RABITQ_EINVAL; }
  const size_t need = carve_workspace(ix, nq, nprobe, k, nullptr, nullptr);
  if (need > (size_t)RABITQ_NOALLOC_SCRATCH_BYTES) {
    set_error("search_noalloc: this (nq, k, nprobe) needs " + std::to_string(need) + " bytes of workspace, the static "
              "scratch holds " + std::to_string((size_t)RABITQ_NOALLOC_SCRATCH_BYTES) + "; use rabitq_search or a smaller batch");
    return RABITQ_EINVAL;
  }
  unsigned char* base = nullptr;
  if ((rc = noalloc_scratch(ix->device, &base))) return rc;
  Workspace w;
  carve_workspace(ix, nq, nprobe, k, base, &w);
  return search_batch(ix, w, queries, nq, k, nprobe, out_ids, out_dists, (hipStream_t)stream);
}

}  // extern "C"
