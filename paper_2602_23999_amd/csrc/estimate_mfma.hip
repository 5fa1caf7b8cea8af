// First stage of the cluster-local search (Sections 3.3.4, 3.4.1(2)) on the matrix cores, as a kernel of its own:
// 1-bit estimates and the filter for 16 pairs of one cluster per wavefront, one 64-vector tile at a time.  What it
// leaves behind is one bit per (pair, vector): "survives the filter".  The refinement of the survivors, the pools and
// the output are the popcount kernel's, which in this mode reads those bits instead of estimating (scan.hip, MASKED).
// Splitting the stages lets each run at its own occupancy: this kernel needs registers and no LDS, the refinement
// needs LDS and many wavefronts in flight to hide the scattered long-code reads.
//
// Survivor bits.  A block of 128 bytes belongs to (cluster, group of 16 pairs, tile); the blocks of cluster c start at
// mask_off[c] and are ordered [group][tile].  A block is what the 64 lanes of the wavefront hold after the tile: lane
// 16 g + lj writes 16 bits about vectors 16 cb + lj (cb = 0..3) and pairs 4 g + r (r = 0..3) of the group; bit
// 4 cb + r is SET when that vector does NOT survive for that pair (the sign of tau minus the bound, shifted in as the
// comparisons are made).
#include "rq_device.h"
#include "rq_scan_args.h"

namespace rq {

template <int W, bool DBG>
__device__ __forceinline__ void estimate_body(const ScanArgs& a) {
  constexpr int KC = (W + 1) / 2;
  const int lane = threadIdx.x, lj = lane & 15, g = lane >> 4;

  // XCD-aware order, as in the popcount kernel: each XCD gets a contiguous range of the true item count
  const int n_items = a.item_off16[a.nlist];
  const int per = (n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= per || item >= n_items) return;
  const int c = wave_upper_cluster(a.item_off16, a.nlist, item, lane);
  const int t0 = a.tile_off[c], tc1 = a.tile_off[c + 1];
  const int nseg = seg_count(tc1 - t0, a.tseg, a.segmax);
  const int local = item - a.item_off16[c];
  const int grp = local / nseg, sidx = local - grp * nseg;
  const int seglen = (tc1 - t0 + nseg - 1) / nseg;
  const int ts = t0 + sidx * seglen, te = min(tc1, ts + seglen);
  const int pbeg = a.pair_off[c] + grp * QM;
  const int np = __builtin_amdgcn_readfirstlane(min(QM, a.pair_off[c + 1] - pbeg));
  // first block of this group's tiles
  uint16_t* blocks = reinterpret_cast<uint16_t*>(a.surv_mask + ((int64_t)a.mask_off[c] + (int64_t)grp * (tc1 - t0)) * 16);

  // query operand: lane (row lj, k-group g) holds bytes 16g .. 16g+15 of every 64-dimension chunk of qhat8, which
  // is stored in the order the expansion of the code words produces (qhat_mfma_pos)
  // (both are fetched by load_pairs, which each branch below calls after it has requested its first codes, so that
  // the two waits overlap)
  v4i qa[KC];
  float al[4], be[4], Gr[4], Er[4], tr[4];
  auto load_pairs = [&]() __attribute__((always_inline)) {
    const int pp = a.pair_ids[pbeg + min(lj, np - 1)];
    const int64_t q = pair_query(a, pp);
    const int8_t* src = a.qhat8 + q * a.Dp + 16 * g;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      qa[kc] = *reinterpret_cast<const v4i*>(src + 64 * kc);
      if (lj >= np) qa[kc] = v4i{0, 0, 0, 0};
    }
    // scalars of this lane's four queries (accumulator r of lane (lj, g) is query 4g + r)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int qi = 4 * g + r;
      const int pp2 = a.pair_ids[pbeg + min(qi, np - 1)];
      const int64_t q2 = pair_query(a, pp2);
      const float dl = a.delta[q2];
      al[r] = dl;
      be[r] = 0.5f * dl * (float)a.sum_qhat[q2];
      Gr[r] = a.probe_G[pp2];
      {  // radius of the bound: ||q'-c'|| widened by the rounding error of the 4-bit query
        const float e = a.probe_E[pp2];
        Er[r] = sqrtf(fmaf(a.qerr, dl * dl, e * e));
      }
      tr[r] = (qi < np) ? a.tau[q2] : -3.402823466e+38f;  // an absent pair lets nothing through
    }
  };

  // estimate, bound and comparison of the lane's four values of one column block; one instruction per comparison:
  // the sign bit of tau - bound (set: the bound is above the threshold; minus infinity for padding, whose f_add is
  // +inf) is shifted into the lane's word.  No operand can be a NaN: the radius Er is positive, so an infinite error
  // factor gives a bound of minus infinity, not inf * 0.  Column blocks are taken 3, 2, 1, 0 and accumulators 3 .. 0:
  // the last comparison ends up in bit 0, which leaves (cb, r) in bit 4 cb + r.
  auto compare = [&](const v4i& acc, float fa, float fr, float fe, int tile, int cb, uint32_t& bits) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 3; r >= 0; --r) {
      const int I = acc[r];
      if (DBG) {
        if (4 * g + r < np) a.dbg_ip[a.dbg_off[pbeg + 4 * g + r] + (int64_t)(tile - t0) * TILE + 16 * cb + lj] = I;
      }
      const float x = fmaf(al[r], (float)I, -be[r]);  // delta * (I - S/2)
      const float e1 = fmaf(fr, x, fa + Gr[r]);
      const float filt = fmaf(-fe, Er[r], e1);
      bits = __builtin_amdgcn_alignbit(bits, __float_as_uint(tr[r] - filt), 31);  // (bits << 1) | sign
    }
  };

  if constexpr (KC <= 2) {
    // Short codes: a whole tile in registers.  Lane (lj, g) holds, for each of the 4 column blocks of 16 vectors, word
    // 2 kc + g/2 of vector 16 cb + lj (it expands half g % 2 of it) and that vector's three factors; the next tile is
    // requested before this one is worked on, two tiles per iteration so that the two register sets swap roles.
    struct TileRegs {
      uint32_t cw[4][KC];
      float fa[4], fr[4], fe[4];
    };
    auto fetch = [&](TileRegs& t, int tile) __attribute__((always_inline)) {
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          const int w = min(2 * kc + (g >> 1), W - 1);
          t.cw[cb][kc] = a.short_codes[((int64_t)tile * W + w) * TILE + 16 * cb + lj];
        }
      }
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int v = 16 * cb + lj;
        t.fa[cb] = a.short_factors[((int64_t)tile * 3 + 0) * TILE + v];
        t.fr[cb] = a.short_factors[((int64_t)tile * 3 + 1) * TILE + v];
        t.fe[cb] = a.short_factors[((int64_t)tile * 3 + 2) * TILE + v];
      }
    };
    auto process = [&](const TileRegs& t, int tile) __attribute__((always_inline)) {
      v4i acc[4];
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        acc[cb] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          uint32_t word = t.cw[cb][kc];
          if ((W & 1) && kc == KC - 1 && (g >> 1)) word = 0u;  // odd W: the last chunk has one word only
          acc[cb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa[kc], expand_half(word, g & 1), acc[cb], 0, 0, 0);
        }
      }
      uint32_t bits = 0u;
#pragma unroll
      for (int cb = 3; cb >= 0; --cb) compare(acc[cb], t.fa[cb], t.fr[cb], t.fe[cb], tile, cb, bits);
      blocks[(int64_t)(tile - t0) * TILE + lane] = (uint16_t)bits;
    };
    TileRegs ta, tb;
    if (ts < te) fetch(ta, ts);
    load_pairs();
    for (int tile = ts; tile < te; tile += 2) {
      fetch(tb, min(tile + 1, te - 1));  // past the end: a harmless re-read
      process(ta, tile);
      if (tile + 1 < te) {
        fetch(ta, min(tile + 2, te - 1));
        process(tb, tile + 1);
      }
    }
  } else {
    // Long codes: the query operand alone takes 4 KC registers, so a column block (16 vectors) at a time: step s of
    // the segment is column block 3 - s % 4 of tile ts + s / 4; the words of the next step are requested before this
    // one is worked on.
    struct CbRegs {
      uint32_t cw[KC];
      float fa, fr, fe;
    };
    const int nstep = (te - ts) * 4;
    auto fetch = [&](CbRegs& t, int s) __attribute__((always_inline)) {
      const int tile = ts + (s >> 2), v = 16 * (3 - (s & 3)) + lj;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const int w = min(2 * kc + (g >> 1), W - 1);
        t.cw[kc] = a.short_codes[((int64_t)tile * W + w) * TILE + v];
      }
      t.fa = a.short_factors[((int64_t)tile * 3 + 0) * TILE + v];
      t.fr = a.short_factors[((int64_t)tile * 3 + 1) * TILE + v];
      t.fe = a.short_factors[((int64_t)tile * 3 + 2) * TILE + v];
    };
    uint32_t bits = 0u;
    auto process = [&](const CbRegs& t, int s) __attribute__((always_inline)) {
      const int tile = ts + (s >> 2), cb = 3 - (s & 3);
      v4i acc = v4i{0, 0, 0, 0};
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        uint32_t word = t.cw[kc];
        if ((W & 1) && kc == KC - 1 && (g >> 1)) word = 0u;
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa[kc], expand_half(word, g & 1), acc, 0, 0, 0);
      }
      compare(acc, t.fa, t.fr, t.fe, tile, cb, bits);
      if (cb == 0) {
        blocks[(int64_t)(tile - t0) * TILE + lane] = (uint16_t)bits;
        bits = 0u;
      }
    };
    CbRegs ca, cb_;
    if (nstep > 0) fetch(ca, 0);
    load_pairs();
    for (int s = 0; s < nstep; s += 2) {  // nstep is a multiple of 4
      fetch(cb_, s + 1);
      process(ca, s);
      fetch(ca, min(s + 2, nstep - 1));
      process(cb_, s + 1);
    }
  }
}

// (two entry points for the register budget: four wavefronts per SIMD for codes of up to 512 bits, three beyond, where
// the query operand alone takes 48 to 64 registers)
template <int W, bool DBG>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(4))) void estimate_mfma_kernel(ScanArgs a) {
  estimate_body<W, DBG>(a);
}
template <int W, bool DBG>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(3))) void estimate_mfma_wide_kernel(ScanArgs a) {
  estimate_body<W, DBG>(a);
}

template <int W>
static void launch_w(const ScanArgs& a, unsigned grid, bool dbg, hipStream_t st) {
  if (W > 16) {
    if (dbg)
      hipLaunchKernelGGL((estimate_mfma_wide_kernel<W, true>), dim3(grid), dim3(64), 0, st, a);
    else
      hipLaunchKernelGGL((estimate_mfma_wide_kernel<W, false>), dim3(grid), dim3(64), 0, st, a);
  } else if (dbg) {
    hipLaunchKernelGGL((estimate_mfma_kernel<W, true>), dim3(grid), dim3(64), 0, st, a);
  } else {
    hipLaunchKernelGGL((estimate_mfma_kernel<W, false>), dim3(grid), dim3(64), 0, st, a);
  }
}

// Returns false when the kernel is not built for the code width W.
bool estimate_mfma(const ScanArgs& a, int W, unsigned grid, bool dbg, hipStream_t st) {
  switch (W) {
    case 1: launch_w<1>(a, grid, dbg, st); return true;
    case 2: launch_w<2>(a, grid, dbg, st); return true;
    case 3: launch_w<3>(a, grid, dbg, st); return true;
    case 4: launch_w<4>(a, grid, dbg, st); return true;
    case 8: launch_w<8>(a, grid, dbg, st); return true;
    case 16: launch_w<16>(a, grid, dbg, st); return true;
    case 24: launch_w<24>(a, grid, dbg, st); return true;
    case 30: launch_w<30>(a, grid, dbg, st); return true;
    case 32: launch_w<32>(a, grid, dbg, st); return true;
    default: return false;
  }
}

}  // namespace rq
