// Device-side building blocks shared by the selection, seeding, scan and merge kernels.
#pragma once
#include "rq_internal.h"

namespace rq {

constexpr uint64_t KEY_NONE = ~0ull;

__device__ inline uint64_t make_key(float v, uint32_t lo) { return ((uint64_t)f2ord(v) << 32) | lo; }

// ---------------------------------------------------------------------------------
// Bitonic sort (ascending) of n = 2^m u64 keys in LDS by the whole workgroup.
// Ends with a barrier.
// ---------------------------------------------------------------------------------
__device__ inline void block_bitonic_sort(uint64_t* keys, int n) {
  const int tid = threadIdx.x, nt = blockDim.x;
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      __syncthreads();
      for (int t = tid; t < (n >> 1); t += nt) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int l = i | j;
        const uint64_t a = keys[i], b = keys[l];
        const bool up = (i & k) == 0;
        if ((a > b) == up) {
          keys[i] = b;
          keys[l] = a;
        }
      }
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------
// Workgroup-wide selection of the K smallest of n u64 keys produced by key_at(i),
// written in ascending order to out[0..Kpad) (Kpad = power of two >= K, the tail is
// KEY_NONE).  key_at may return KEY_NONE for an absent entry.  Keys are distinct (their
// low word is an index or id), so the result is unique.
//
// MSB-first radix select that (1) skips the bits all keys share (estimates of one query lie
// in a narrow range, so their exponent bits are equal and would all hit one histogram bin),
// (2) stops as soon as the bucket holding the K-th key is taken whole, and (3) finishes a
// bucket of at most 64 keys inside one wavefront by ranking them against each other.
// blockDim.x must be a multiple of 64, at most 1024.
// ---------------------------------------------------------------------------------
// Wavefront reductions on the VALU's data-parallel primitives (no LDS round trips).
// After the four row steps every lane of a 16-lane row holds the row's result; the four
// rows are then combined through scalar lane reads.
template <typename Op>
__device__ inline uint32_t wave_reduce_u32(uint32_t v, Op op) {
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));  // row_half_mirror
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));  // row_mirror
  const uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
  return op(op(a, b), op(c, d));
}

template <typename Op>
__device__ inline uint64_t wave_reduce_u64(uint64_t v, Op op) {
  auto step = [&](int ctrl_id) {
    int lo = (int)(uint32_t)v, hi = (int)(uint32_t)(v >> 32);
    int olo, ohi;
    switch (ctrl_id) {
      case 0: olo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, true); ohi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, true); break;
      case 1: olo = __builtin_amdgcn_update_dpp(0, lo, 0x4E, 0xF, 0xF, true); ohi = __builtin_amdgcn_update_dpp(0, hi, 0x4E, 0xF, 0xF, true); break;
      case 2: olo = __builtin_amdgcn_update_dpp(0, lo, 0x141, 0xF, 0xF, true); ohi = __builtin_amdgcn_update_dpp(0, hi, 0x141, 0xF, 0xF, true); break;
      default: olo = __builtin_amdgcn_update_dpp(0, lo, 0x140, 0xF, 0xF, true); ohi = __builtin_amdgcn_update_dpp(0, hi, 0x140, 0xF, 0xF, true); break;
    }
    v = op(v, ((uint64_t)(uint32_t)ohi << 32) | (uint32_t)olo);
  };
  step(0); step(1); step(2); step(3);
  auto rd = [&](int l) {
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l) << 32) |
           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
  };
  return op(op(rd(0), rd(16)), op(rd(32), rd(48)));
}

struct SelectScratch {
  uint64_t lo, hi, bound;
  uint64_t small[64];
  uint64_t wlo[16], whi[16];
  uint32_t hist[256];
  uint32_t wcnt[16];
  uint32_t digit, need, bucket, cnt, nvalid;
};

template <typename KeyFn>
__device__ inline void block_select_smallest(int n, int K, int Kpad, KeyFn key_at, uint64_t* out, SelectScratch* sh) {
  const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
  // range and count of the present keys
  uint64_t lo = KEY_NONE, hi = 0ull;
  uint32_t nv = 0;
  for (int i = tid; i < n; i += nt) {
    const uint64_t key = key_at(i);
    if (key != KEY_NONE) {
      lo = key < lo ? key : lo;
      hi = key > hi ? key : hi;
      ++nv;
    }
  }
  lo = wave_reduce_u64(lo, [](uint64_t a, uint64_t b) { return a < b ? a : b; });
  hi = wave_reduce_u64(hi, [](uint64_t a, uint64_t b) { return a > b ? a : b; });
  nv = wave_reduce_u32(nv, [](uint32_t a, uint32_t b) { return a + b; });
  if (lane == 0) {
    sh->wlo[wave] = lo;
    sh->whi[wave] = hi;
    sh->wcnt[wave] = nv;
  }
  __syncthreads();
  if (tid == 0) {
    uint64_t l = KEY_NONE, h = 0ull;
    uint32_t c = 0;
    for (int w = 0; w < nw; ++w) {
      l = sh->wlo[w] < l ? sh->wlo[w] : l;
      h = sh->whi[w] > h ? sh->whi[w] : h;
      c += sh->wcnt[w];
    }
    sh->lo = l;
    sh->hi = h;
    sh->nvalid = c;
  }
  __syncthreads();
  uint64_t bound = KEY_NONE;  // select present keys <= bound
  if (sh->nvalid > (uint32_t)K && sh->lo != sh->hi) {
    lo = sh->lo;
    hi = sh->hi;
    const int top = 63 - __clzll((long long)(lo ^ hi));  // highest bit in which two keys differ
    int width = min(8, top + 1);
    int shift = top + 1 - width;
    uint64_t pmask = (top == 63) ? 0ull : (~0ull << (top + 1));
    uint64_t prefix = lo & pmask;
    uint32_t need = (uint32_t)K;
    while (true) {
      for (int i = tid; i < 256; i += nt) sh->hist[i] = 0;
      __syncthreads();
      const uint32_t dmask = (1u << width) - 1u;
      for (int i = tid; i < n; i += nt) {
        const uint64_t key = key_at(i);
        if (key != KEY_NONE && (key & pmask) == prefix) atomicAdd(&sh->hist[(uint32_t)(key >> shift) & dmask], 1u);
      }
      __syncthreads();
      if (tid < 64) {
        const uint32_t c0 = sh->hist[4 * tid], c1 = sh->hist[4 * tid + 1], c2 = sh->hist[4 * tid + 2],
                       c3 = sh->hist[4 * tid + 3];
        const uint32_t s = c0 + c1 + c2 + c3;
        uint32_t incl = s;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const uint32_t o = __shfl_up(incl, d, 64);
          if (tid >= d) incl += o;
        }
        const uint32_t excl = incl - s;
        if (excl < need && need <= incl) {
          uint32_t rem = need - excl, digit, cnt;
          if (rem <= c0) { digit = 0; cnt = c0; }
          else if (rem <= c0 + c1) { digit = 1; cnt = c1; rem -= c0; }
          else if (rem <= c0 + c1 + c2) { digit = 2; cnt = c2; rem -= c0 + c1; }
          else { digit = 3; cnt = c3; rem -= c0 + c1 + c2; }
          sh->digit = 4 * tid + digit;
          sh->need = rem;
          sh->bucket = cnt;
          sh->cnt = 0;
        }
      }
      __syncthreads();
      prefix |= (uint64_t)sh->digit << shift;
      pmask |= (uint64_t)dmask << shift;
      need = sh->need;
      const uint32_t bucket = sh->bucket;
      if (bucket == need || shift == 0) {  // the whole bucket is selected
        bound = prefix | (shift == 0 ? 0ull : ((1ull << shift) - 1ull));
        break;
      }
      if (bucket <= 64u) {  // rank the bucket's keys against each other in one wavefront
        for (int i = tid; i < n; i += nt) {
          const uint64_t key = key_at(i);
          if (key != KEY_NONE && (key & pmask) == prefix) sh->small[atomicAdd(&sh->cnt, 1u)] = key;
        }
        __syncthreads();
        if (tid < (int)bucket) {
          const uint64_t mine = sh->small[tid];
          uint32_t rank = 0;
          for (uint32_t m = 0; m < bucket; ++m) rank += (sh->small[m] < mine) ? 1u : 0u;
          if (rank == need - 1u) sh->bound = mine;
        }
        __syncthreads();
        bound = sh->bound;
        break;
      }
      width = min(8, shift);
      shift -= width;
      __syncthreads();
    }
  }
  __syncthreads();
  if (tid == 0) sh->cnt = 0;
  for (int i = tid; i < Kpad; i += nt) out[i] = KEY_NONE;
  __syncthreads();
  for (int i = tid; i < n; i += nt) {
    const uint64_t key = key_at(i);
    if (key <= bound && key != KEY_NONE) {
      const uint32_t pos = atomicAdd(&sh->cnt, 1u);
      if (pos < (uint32_t)Kpad) out[pos] = key;
    }
  }
  block_bitonic_sort(out, Kpad);
}

// ---------------------------------------------------------------------------------
// Wavefront-wide selection with the keys in registers: every lane holds R keys (KEY_NONE =
// absent).  Returns a bound such that exactly min(K, #present) present keys are <= bound.
// MSB-first bisection: one bit per step, counting the keys of the current bucket whose
// next bit is 0; the bits all keys share are skipped and the search stops as soon as the
// bucket holding the K-th key is taken whole.  No LDS, no barriers.
// ---------------------------------------------------------------------------------
template <int R>
__device__ inline uint64_t wave_kth_bound(const uint64_t (&key)[R], int K) {
  uint64_t lo = KEY_NONE, hi = 0ull;
  uint32_t nv = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    if (key[r] != KEY_NONE) {
      lo = key[r] < lo ? key[r] : lo;
      hi = key[r] > hi ? key[r] : hi;
      ++nv;
    }
  }
  lo = wave_reduce_u64(lo, [](uint64_t a, uint64_t b) { return a < b ? a : b; });
  hi = wave_reduce_u64(hi, [](uint64_t a, uint64_t b) { return a > b ? a : b; });
  nv = wave_reduce_u32(nv, [](uint32_t a, uint32_t b) { return a + b; });
  if (nv <= (uint32_t)K) return KEY_NONE - 1ull;
  if (lo == hi) return hi;
  const int top = 63 - __clzll((long long)(lo ^ hi));
  uint64_t prefix = (top == 63) ? 0ull : (hi & (~0ull << (top + 1)));
  uint32_t need = (uint32_t)K, cmatch = nv;
  for (int b = top; b >= 0; --b) {
    const uint64_t mask_hi = ~0ull << b;
    uint32_t c0 = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) c0 += ((key[r] & mask_hi) == prefix) ? 1u : 0u;
    c0 = wave_reduce_u32(c0, [](uint32_t a, uint32_t x) { return a + x; });
    if (need <= c0) {
      cmatch = c0;
    } else {
      need -= c0;
      cmatch -= c0;
      prefix |= 1ull << b;
    }
    if (cmatch == need) return prefix | ((b == 0) ? 0ull : ((1ull << b) - 1ull));
  }
  return prefix;
}

// Packs the keys <= bound of every lane into out[0..) in LDS (any order) and pads the rest
// of out[0..Kpad) with KEY_NONE.  For a single-wavefront workgroup.  Returns the count.
template <int R>
__device__ inline int wave_gather_selected(const uint64_t (&key)[R], uint64_t bound, uint64_t* out, int Kpad) {
  const int lane = threadIdx.x & 63;
  for (int i = lane; i < Kpad; i += 64) out[i] = KEY_NONE;
  __syncthreads();
  int base = 0;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const bool sel = key[r] <= bound && key[r] != KEY_NONE;
    const uint64_t m = __ballot(sel);
    if (sel) {
      const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
      if (pos < Kpad) out[pos] = key[r];
    }
    base += __popcll(m);
  }
  __syncthreads();
  return base;
}

// ---------------------------------------------------------------------------------
// Streaming selection of the K <= 64 smallest 64-bit keys by one wavefront, entirely in
// registers: lane l holds the l-th smallest key seen so far.  The first 64 keys are sorted
// across the lanes (bitonic network); afterwards a tile of 64 keys is compared with the
// current K-th key and only the few that beat it are inserted, one at a time.  Keys are
// unique (their low word is an index), so the result does not depend on the order of
// arrival.  All control flow is wave-uniform.
// ---------------------------------------------------------------------------------
__device__ inline uint64_t shfl_u64(uint64_t v, int src) {
  const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)v, src, 64);
  const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)(v >> 32), src, 64);
  return ((uint64_t)hi << 32) | lo;
}
__device__ inline uint64_t readlane_u64(uint64_t v, int src) {  // src must be wave-uniform
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, src);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), src);
  return ((uint64_t)hi << 32) | lo;
}

// Keeps a loaded value where it is: without it the compiler moves a load whose value is only used under a
// condition back under that condition, into a block of its own, and then waits for every such load before it
// issues the next one.
__device__ inline float pinned(float v) {
  asm volatile("" : "+v"(v));
  return v;
}
__device__ inline uint64_t pinned(uint64_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

struct WaveTopK {
  uint64_t v;  // lane l: l-th smallest key so far (KEY_NONE where there is none yet)

  // the first tile: ascending bitonic sort of one key per lane
  __device__ inline void init_sorted(uint64_t key, int lane) {
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1) {
#pragma unroll
      for (int j = k >> 1; j > 0; j >>= 1) {
        const uint64_t other = shfl_u64(key, lane ^ j);
        const bool asc = (lane & k) == 0;
        const bool low = (lane & j) == 0;
        const bool take_min = (asc == low);
        const uint64_t mn = key < other ? key : other, mx = key < other ? other : key;
        key = take_min ? mn : mx;
      }
    }
    v = key;
  }

  // a further tile: one key per lane
  __device__ inline void push_tile(uint64_t key, int K, int lane) {
    uint64_t kth = readlane_u64(v, K - 1);
    uint64_t m = __ballot(key < kth);
    while (m != 0ull) {
      const int src = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)m) - 1);
      m &= m - 1ull;
      const uint64_t x = readlane_u64(key, src);
      if (x < kth) {  // the K-th key may have dropped since the ballot
        const int p = __popcll(__ballot(v < x));  // keys below x; x goes to position p (< K)
        // every lane's left neighbour through the data-parallel primitive that shifts the whole wavefront by one
        // lane (lane 0 keeps its own value, which it never needs: it takes x or stays)
        const uint32_t ulo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)v, (int)(uint32_t)v, 0x138, 0xF, 0xF, false);
        const uint32_t uhi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(v >> 32), (int)(uint32_t)(v >> 32), 0x138, 0xF, 0xF, false);
        const uint64_t up = ((uint64_t)uhi << 32) | ulo;
        v = lane < p ? v : (lane == p ? x : up);
        kth = readlane_u64(v, K - 1);
      }
    }
  }
};

template <int F>
__host__ __device__ inline int stage_index(int d);  // position of dimension d in the refinement's query order (below)

// Position of dimension d in the qhat8 array (the matrix-core scan's query operand).  Within every chunk of 64
// dimensions, dimension r = 32 w + 8 b + 4 h + i (w: word of the chunk, b = 0..3, h = 0..1, i = 0..3) sits at byte
// 16 (2 w + h) + 4 i + b: the order in which (word >> (4h + i)) & 0x01010101 delivers the sign bits of a code word.
__host__ __device__ inline int qhat_mfma_pos(int d) {
  const int c = d >> 6, r = d & 63, w = r >> 5, x = r & 31;
  return 64 * c + 16 * (2 * w + ((x >> 2) & 1)) + 4 * (x & 3) + (x >> 3);
}

// ---------------------------------------------------------------------------------
// Section 3.3.3 / 3.4.1(2): the per-query representation of one rotated query x[0..D), by one wavefront:
// 4-bit signed quantisation and its bit-planes, sums, the query in refinement order, lookup tables.
// delta = max|q'|/7 and q'/delta use IEEE fp32 division and round-half-even, because they decide integers.
// prep_reduce is the first half on its own (max |x|, sum, squared norm, each the same in every lane afterwards);
// whoever needs only the squared norm calls it and gets the very bits query_prep_row stores.
// ---------------------------------------------------------------------------------
__device__ inline void prep_reduce(const float* x, int D, int lane, float& amax, float& s1, float& s2) {
  amax = 0.f; s1 = 0.f; s2 = 0.f;
  for (int i = lane; i < D; i += 64) {
    const float v = x[i];
    amax = fmaxf(amax, fabsf(v));
    s1 += v;
    s2 += v * v;
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) {
    amax = fmaxf(amax, __shfl_xor(amax, d, 64));
    s1 += __shfl_xor(s1, d, 64);
    s2 += __shfl_xor(s2, d, 64);
  }
}

template <int F>
__device__ inline void query_prep_row(const float* x, int64_t q, int D, const rabitq_query_repr& o, int lane) {
  const int W = D >> 5;
  const int Dp = (D + 63) / 64 * 64;
  float amax, s1, s2;
  prep_reduce(x, D, lane, amax, s1, s2);
  for (int i = lane; i < D; i += 64) o.q_stage[q * D + (F == 0 ? i : stage_index<(F == 0 ? 8 : F)>(i))] = x[i];
  const float dl = (amax == 0.f) ? 1.0f : __fdiv_rn(amax, 7.0f);
  int S = 0;
  uint32_t* pl = o.planes + q * 4 * W;
  for (int base = 0; base < Dp; base += 64) {
    const int i = base + lane;
    int qh = 0;
    if (i < D && amax != 0.f) {
      const float t = rintf(__fdiv_rn(x[i], dl));
      qh = (int)fminf(fmaxf(t, -7.f), 7.f);
    }
    S += qh;
    o.qhat8[q * Dp + qhat_mfma_pos(i)] = (int8_t)qh;
    const uint32_t tc = (uint32_t)qh & 15u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint64_t m = __ballot((tc >> j) & 1u);
      const int w = base >> 5;
      if (lane == 0 && w < W) pl[j * W + w] = (uint32_t)m;
      if (lane == 0 && w + 1 < W) pl[j * W + w + 1] = (uint32_t)(m >> 32);
    }
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) S += __shfl_xor(S, d, 64);
  // Section 3.4.1(1): lookup tables, one entry per (block of 4 dimensions, 4-bit pattern); the sum runs in
  // fp32 over the set bits in ascending dimension order and is rounded to binary16
  if (o.lut != nullptr) {
    _Float16* lut = reinterpret_cast<_Float16*>(o.lut) + q * (int64_t)D * 4;
    for (int e = lane; e < D * 4; e += 64) {
      const int j = e >> 4, b = e & 15;
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if ((b >> i) & 1) acc += x[4 * j + i];
      lut[e] = (_Float16)acc;
    }
  }
  if (lane == 0) {
    o.delta[q] = dl;
    o.sum_qhat[q] = S;
    o.sum_q[q] = s1;
    o.sq_norm[q] = s2;
  }
}

// ---------------------------------------------------------------------------------
// Section 3.3.2: the K <= 64 smallest of row[0..n) as (order-preserving score bits << 32 | index), by one
// wavefront that reads the row once through a register-resident sorted list.
// ---------------------------------------------------------------------------------
__device__ inline WaveTopK stream_select_smallest(const float* __restrict__ row, int nlist, int nprobe, int lane) {
  WaveTopK top;
  // The first 16 tiles (1024 scores) are held in registers: the 64 per-lane minima start the sorted list, so
  // its nprobe-th key is small from the outset and few of the remaining scores have to be inserted.
  constexpr int R = 16;
  {
    // (unconditional loads of clamped indices, all requested before the first value is touched: a load whose value
    // is only used under a condition would otherwise be waited for before the next one is issued)
    float sv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) sv[r] = __builtin_nontemporal_load(row + min(r * 64 + lane, nlist - 1));
#pragma unroll
    for (int r = 0; r < R; ++r) sv[r] = pinned(sv[r]);
    uint32_t ord[R];
#pragma unroll
    for (int r = 0; r < R; ++r) ord[r] = (r * 64 + lane < nlist) ? f2ord(sv[r]) : 0xffffffffu;
    uint32_t mo = ord[0];
    int mr = 0;
#pragma unroll
    for (int r = 1; r < R; ++r)
      if (ord[r] < mo) { mo = ord[r]; mr = r; }  // ties keep the lower index, as the key order does
    top.init_sorted(mo == 0xffffffffu ? KEY_NONE : (((uint64_t)mo << 32) | (uint32_t)(mr * 64 + lane)), lane);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (r * 64 < nlist) {
        const bool take = r != mr && ord[r] != 0xffffffffu;
        top.push_tile(take ? (((uint64_t)ord[r] << 32) | (uint32_t)(r * 64 + lane)) : KEY_NONE, nprobe, lane);
      }
    }
  }
  // the rest of the row, eight tiles of scores in flight; a tile is only looked at closely when its smallest
  // score beats the current nprobe-th key
  for (int tb = R * 64; tb < nlist; tb += 512) {
    float sc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) sc[u] = __builtin_nontemporal_load(row + min(tb + u * 64 + lane, nlist - 1));
#pragma unroll
    for (int u = 0; u < 8; ++u) sc[u] = pinned(sc[u]);
#pragma unroll
    for (int u = 0; u < 8; ++u) sc[u] = (tb + u * 64 + lane < nlist) ? sc[u] : INFINITY;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (tb + u * 64 < nlist) {
        const int i = tb + u * 64 + lane;
        top.push_tile((i < nlist) ? make_key(sc[u], (uint32_t)i) : KEY_NONE, nprobe, lane);
      }
    }
  }
  return top;
}

// Largest c in [0, n) with off[c] <= v, for a non-decreasing array off[0..n] with off[0] <= v < off[n]
// (any v >= off[n] gives n - 1).  One wavefront, 64-ary: every level is a single coalesced load and a ballot,
// so the chain of dependent loads is ceil(log64(n + 1)) long.  Every index read is within [0, n].
__device__ inline int wave_upper_cluster(const int32_t* __restrict__ off, int n, int v, int lane) {
  int stride = 1;
  while ((int64_t)stride * 64 < (int64_t)n + 1) stride *= 64;
  int base = 0;
  for (; stride >= 1; stride >>= 6) {
    const int64_t idx = (int64_t)base + (int64_t)lane * stride;
    const bool in = idx < n;
    const int val = off[in ? idx : n];
    const uint64_t m = __ballot(in && val <= v);
    const int cnt = __popcll(m);
    base += (cnt > 0 ? cnt - 1 : 0) * stride;
  }
  return base;
}

__host__ __device__ inline int next_pow2(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

// ---------------------------------------------------------------------------------
// Section 3.4.1(2): <x_b, qhat> = -8 pc(x&q3) + 4 pc(x&q2) + 2 pc(x&q1) + pc(x&q0),
// 32 dimensions per AND + popcount.  `pl` points at the query's planes [4][W]; it is
// wave-uniform, so the compiler keeps the plane words in scalar registers.
// ---------------------------------------------------------------------------------
typedef const uint32_t __attribute__((address_space(4)))* const_u32_ptr;
typedef const uint64_t __attribute__((address_space(4)))* const_u64_ptr;

// popcount(x) + acc in one VALU instruction (the compiler otherwise splits the add off)
__device__ inline uint32_t bcnt_acc(uint32_t x, uint32_t acc) {
  uint32_t d;
  asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(acc));
  return d;
}

template <int W>
__device__ inline int ip_bitplanes(const uint32_t (&cw)[W], const_u32_ptr pl) {
  uint32_t p0 = 0, p1 = 0, p2 = 0, p3 = 0;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    p0 = bcnt_acc(cw[w] & pl[0 * W + w], p0);
    p1 = bcnt_acc(cw[w] & pl[1 * W + w], p1);
    p2 = bcnt_acc(cw[w] & pl[2 * W + w], p2);
    p3 = bcnt_acc(cw[w] & pl[3 * W + w], p3);
  }
  // p0 + 2 p1 + 4 p2 - 8 p3 in three instructions
  uint32_t t;
  asm("v_lshl_add_u32 %0, %1, 1, %2" : "=v"(t) : "v"(p1), "v"(p0));
  asm("v_lshl_add_u32 %0, %1, 2, %2" : "=v"(t) : "v"(p2), "v"(t));
  int r;
  asm("v_mad_i32_i24 %0, %1, -8, %2" : "=v"(r) : "v"(p3), "v"(t));
  return r;
}

// ---------------------------------------------------------------------------------
// Refinement (Section 3.4.2: lanes cooperate on one candidate).  The long code holds the
// whole B-bit code of every dimension in F-bit fields (F = 2, 4, 8), LW = D*F/32 words per
// vector.  G lanes share one candidate; lane t takes the words [t*WPL, (t+1)*WPL).
//
// A word is decoded byte-lane-wise: for each of the 8/F field positions s inside a byte,
// (word >> s*F) & mask leaves one field in each of the four bytes, and a byte converts to
// float in one instruction.  Byte b, position s of word w is dimension
// w*(32/F) + b*(8/F) + s; the query is staged in LDS in that order (stage_index) so that
// the four floats matching one masked word are one 16-byte read.
// ---------------------------------------------------------------------------------
template <int F>
__host__ __device__ inline int stage_index(int d) {
  constexpr int DPW = 32 / F, SPB = 8 / F;
  const int w = d / DPW, r = d % DPW;
  return w * DPW + (r % SPB) * 4 + (r / SPB);
}

template <int F>
__device__ inline float dot_word(uint32_t word, const float* qw) {
  constexpr int SPB = 8 / F;
  constexpr uint32_t MASK = (F == 8) ? 0xffffffffu : (((1u << F) - 1u) * 0x01010101u);
  float acc = 0.f;
#pragma unroll
  for (int s = 0; s < SPB; ++s) {
    uint32_t m = (word >> (s * F)) & MASK;
    // (kept opaque: otherwise the compiler undoes the shared mask and extracts every field on its own, two
    // instructions per dimension instead of one byte-to-float conversion)
    if (F < 8) asm volatile("" : "+v"(m));
    const float4 q = *reinterpret_cast<const float4*>(qw + 4 * s);
    acc += (float)(m & 255u) * q.x + (float)((m >> 8) & 255u) * q.y + (float)((m >> 16) & 255u) * q.z +
           (float)(m >> 24) * q.w;
  }
  return acc;
}

template <int LW>
struct RefineShape {
  static constexpr int G = (LW > 32) ? 16 : 4;          // lanes per candidate
  static constexpr int WPL = (LW + G - 1) / G;          // words per lane
  static constexpr int NS = 64 / G;                     // candidates per wavefront round
};

// partial <u, q'> of lane t (0..G-1) of a candidate whose long-code row starts at `row`
template <int F, int LW>
__device__ inline float refine_lane(const uint32_t* __restrict__ row, const float* qf, int t) {
  constexpr int WPL = RefineShape<LW>::WPL, DPW = 32 / F;
  float acc = 0.f;
  const int w0 = t * WPL;
  if (w0 >= LW) return 0.f;
  if (WPL % 4 == 0 && LW % 4 == 0) {
#pragma unroll
    for (int c = 0; c < WPL / 4; ++c) {
      const uint4 v = *reinterpret_cast<const uint4*>(row + w0 + 4 * c);
      const float* q = qf + (w0 + 4 * c) * DPW;
      acc += dot_word<F>(v.x, q) + dot_word<F>(v.y, q + DPW) + dot_word<F>(v.z, q + 2 * DPW) +
             dot_word<F>(v.w, q + 3 * DPW);
    }
  } else {
#pragma unroll
    for (int i = 0; i < WPL; ++i) {
      const int w = w0 + i;
      if (w < LW) acc += dot_word<F>(row[w], qf + w * DPW);
    }
  }
  return acc;
}

// The same in two steps, so that the words of the next candidate can be requested before the current one is
// worked on: refine_load only issues loads (every address is inside the row, whatever t), refine_dot consumes them.
template <int F, int LW>
__device__ inline void refine_load(const uint32_t* __restrict__ row, int t, uint32_t (&w)[RefineShape<LW>::WPL]) {
  constexpr int WPL = RefineShape<LW>::WPL;
  const int w0 = t * WPL;
  if (WPL % 4 == 0 && LW % 4 == 0) {
#pragma unroll
    for (int c = 0; c < WPL / 4; ++c) {
      const uint4 v = *reinterpret_cast<const uint4*>(row + min(w0 + 4 * c, LW - 4));
      w[4 * c] = v.x; w[4 * c + 1] = v.y; w[4 * c + 2] = v.z; w[4 * c + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int i = 0; i < WPL; ++i) w[i] = row[min(w0 + i, LW - 1)];
  }
}

template <int F, int LW>
__device__ inline float refine_dot(const uint32_t (&w)[RefineShape<LW>::WPL], const float* qf, int t) {
  constexpr int WPL = RefineShape<LW>::WPL, DPW = 32 / F;
  const int w0 = t * WPL;
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < WPL; ++i)
    if (w0 + i < LW) acc += dot_word<F>(w[i], qf + (w0 + i) * DPW);
  return acc;
}

// sum over the G = 4 or 16 adjacent lanes of a candidate, in every one of them; data-parallel moves inside a row of
// 16 lanes (rotate by 8 and by 4, then the quad permutations [2,3,0,1] and [1,0,3,2]), no LDS round trips
template <int CTRL>
__device__ inline float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int G>
__device__ inline float group_sum(float v) {
  if (G >= 16) {
    v += dpp_move<0x128>(v);
    v += dpp_move<0x124>(v);
  }
  v += dpp_move<0x4E>(v);
  v += dpp_move<0xB1>(v);
  return v;
}

// ---------------------------------------------------------------------------------
// Shared by the matrix-core variants of the scan.
// ---------------------------------------------------------------------------------
typedef int v4i __attribute__((ext_vector_type(4)));

// 16 sign bits of a code word -> 16 bytes of 0/1 for the matrix instruction's B operand, at two instructions per
// four bytes: (word >> s) & 0x01010101 leaves bits s, s+8, s+16, s+24 of the word in the four bytes.  The lane
// group with half h (0 / 1) of a word takes the shifts s = 4h .. 4h+3, so byte b of its i-th operand word is dimension
// 4h + i + 8b of the code word, and the query's qhat bytes are stored in that same order (qhat_mfma_pos).
__device__ inline v4i expand_half(uint32_t word, int h) {
  const uint32_t v = word >> (4 * h);
  v4i x;
  x.x = (int)(v & 0x01010101u);
  x.y = (int)((v >> 1) & 0x01010101u);
  x.z = (int)((v >> 2) & 0x01010101u);
  x.w = (int)((v >> 3) & 0x01010101u);
  return x;
}

__device__ inline void wave_sync() {  // orders LDS traffic among the lanes of one wavefront
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// bitonic sort of n = 2^m keys in LDS by ONE wavefront of a larger workgroup (no workgroup barrier)
__device__ inline void wave_bitonic_sort(uint64_t* keys, int n, int lane) {
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      wave_sync();
      for (int t = lane; t < (n >> 1); t += 64) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int l = i | j;
        const uint64_t x = keys[i], y = keys[l];
        const bool up = (i & k) == 0;
        if ((x > y) == up) {
          keys[i] = y;
          keys[l] = x;
        }
      }
    }
  }
  wave_sync();
}

__device__ inline int wave_pool_compact(uint64_t* pool, int pool_n, int cnt, int k, int lane) {
  wave_sync();
  for (int i = cnt + lane; i < pool_n; i += 64) pool[i] = KEY_NONE;
  wave_bitonic_sort(pool, pool_n, lane);
  return min(cnt, k);
}

}  // namespace rq
