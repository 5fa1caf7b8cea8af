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
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(4))) void estimate_mfma_kernel(ScanArgs a) {
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

  // One tile as the matrix instruction wants it: lane (lj, g) holds, for each of the 4 column blocks of 16 vectors,
  // word 2 kc + g/2 of vector 16 cb + lj (it expands half g % 2 of it) and that vector's three factors.
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
  TileRegs ta, tb;
  if (ts < te) fetch(ta, ts);  // requested before the pairs' scalars, so that the two waits overlap

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
  }
  // scalars of this lane's four queries (accumulator r of lane (lj, g) is query 4g + r)
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
    tr[r] = (qi < np) ? a.tau[q] : -3.402823466e+38f;  // an absent pair lets nothing through
  }

  auto process = [&](const TileRegs& t, int tile) __attribute__((always_inline)) {
    // inner products: 4 column blocks of 16 vectors x 16 queries
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
    // one instruction per comparison: the sign bit of tau - bound (set: the bound is above the threshold; minus
    // infinity for padding, whose f_add is +inf) is shifted into the lane's word.  No operand can be a NaN: the
    // radius Er is positive, so an infinite error factor gives a bound of minus infinity, not inf * 0.
    // (the last comparison ends up in bit 0: descending order leaves (cb, r) in bit 4 cb + r)
    uint32_t bits = 0u;
#pragma unroll
    for (int cb = 3; cb >= 0; --cb) {
      const int v = 16 * cb + lj;
      const float fa = t.fa[cb], fr = t.fr[cb], fe = t.fe[cb];
#pragma unroll
      for (int r = 3; r >= 0; --r) {
        const int I = acc[cb][r];
        if (DBG) {
          if (4 * g + r < np) a.dbg_ip[a.dbg_off[pbeg + 4 * g + r] + (int64_t)(tile - t0) * TILE + v] = I;
        }
        const float x = fmaf(al[r], (float)I, -be[r]);  // delta * (I - S/2)
        const float e1 = fmaf(fr, x, fa + Gr[r]);
        const float filt = fmaf(-fe, Er[r], e1);
        bits = __builtin_amdgcn_alignbit(bits, __float_as_uint(tr[r] - filt), 31);  // (bits << 1) | sign
      }
    }
    blocks[(int64_t)(tile - t0) * TILE + lane] = (uint16_t)bits;
  };

  // two tiles per iteration, so that the registers of the tile in flight and of the tile in work swap roles
  for (int tile = ts; tile < te; tile += 2) {
    fetch(tb, min(tile + 1, te - 1));  // past the end: a harmless re-read
    process(ta, tile);
    if (tile + 1 < te) {
      fetch(ta, min(tile + 2, te - 1));
      process(tb, tile + 1);
    }
  }
}

template <int W>
static void launch_w(const ScanArgs& a, unsigned grid, bool dbg, hipStream_t st) {
  if (dbg)
    hipLaunchKernelGGL((estimate_mfma_kernel<W, true>), dim3(grid), dim3(64), 0, st, a);
  else
    hipLaunchKernelGGL((estimate_mfma_kernel<W, false>), dim3(grid), dim3(64), 0, st, a);
}

// Returns false when the kernel is not built for the code width W.
bool estimate_mfma(const ScanArgs& a, int W, unsigned grid, bool dbg, hipStream_t st) {
  switch (W) {
    case 1: launch_w<1>(a, grid, dbg, st); return true;
    case 2: launch_w<2>(a, grid, dbg, st); return true;
    case 3: launch_w<3>(a, grid, dbg, st); return true;
    case 4: launch_w<4>(a, grid, dbg, st); return true;
    default: return false;
  }
}

}  // namespace rq
