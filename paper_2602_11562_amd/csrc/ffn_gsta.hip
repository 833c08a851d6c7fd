// Segment FFN + LayerNorm (paper Sec. 3.4.2, s <- LN(FFN(s) + s)) feeding the GSTA layer (Sec. 3.4.3) from one pass
// over H': the normalised segment vectors of a pair are scored against r = W_k (t0 W_q)^T / sqrt(d) and pooled with
// their softmax weights while they are still on chip, so the transformed H' is neither written nor read back
// (it is written as well when the caller wants it). One layer, bf16, d = 128, d_ff in {64, 128}.
//
// Three launches, the outer two shared with the split form of GSTA (gsta_tiled.hip):
//   gsta_r_kernel     r = (t0 W_q) W_k^T / sqrt(d)   tiles of 32 pairs, MFMA                       -> z rows
//   ffn_pool_kernel   below: a wave per pair          H' rows -> s rows (on chip), z rows (r) -> z rows (p)
//   gsta_out_kernel   z = t0 + p W_v                  tiles of 32 pairs, MFMA             z rows -> z rows
// with p = sum_i a_i s_i, a = softmax over the segments that hold a valid item of r . s_i (the attention equation
// with its products re-associated, which is exact).
//
// ffn_pool_kernel: the FFN tile of segment_ffn_tile.h on the rows of one pair at a time (tiles of 32 rows over the
// pair's first nv segments, the ones that hold a valid item; rows past them repeat the last one and count as empty;
// the rows of the remaining segments are never read). A wave walks pairs with a grid stride; the rows of its next
// tile, of this pair or the next, and the next pair's r are in flight while it multiplies. After LayerNorm a lane
// holds, in the accumulator layout, 64 of the 128 components of row l32: the rounded values (what a stored s would
// hold) are multiplied with the same components of r, read from a wave-private LDS copy, and one exchange with
// lane ^ 32 gives the row's score. Maximum and sum over the tile's rows are wave reductions; tiles of a pair are
// merged with the running maximum (online softmax). The weighted sum over rows is taken from the LDS patch the
// rounded rows are parked in: lane l owns components 2 l and 2 l + 1 and reads one word per row, with the row's
// weight from v_readlane. Rows of segments without a valid item are never read (whatever H' holds there is not
// trusted): inside a tile they are copies of the last valid row with weight zero, and they leave as zeros.
// p / sum of weights replaces r in the pair's z row.
#include "segment_ffn_tile.h"

namespace laser {

// MR: also the two other views of Sec. 3.4.4 of the transformed rows: pool [P, D] bf16, the component-wise maximum
// over the segments that hold a valid item (zeros when there is none), taken in the weighted-sum loop from the same
// words (rows past the last valid segment are copies of it, so they leave the maximum alone); recent [P, r, D] bf16,
// the first r rows as they would be stored. Either may be null.
template <int DFF, bool MR>
__global__ __launch_bounds__(FM_THREADS) void ffn_pool_kernel(
    const unsigned short* seg, const int32_t* __restrict__ lens, const unsigned short* __restrict__ w1,
    const float* __restrict__ b1, const unsigned short* __restrict__ w2, const float* __restrict__ b2,
    const float* __restrict__ ln_g, const float* __restrict__ ln_b, const int32_t* __restrict__ cand_off, int U, int P,
    int C, int L, int w, int S, float eps,
    unsigned short* out,   // s rows [P, S, D], may be null (not wanted), may be seg
    float* z,              // [P, D]: r on entry, p on exit
    unsigned* pool, unsigned short* recent, int r) {
  constexpr int D = FM_D, KSTEPS = D / 16, DB = D / 32, OP = FM_OP;
  constexpr int RVB = 1024;   // bytes per copy of r: the 512 bytes twice (a fetch moves 16 bytes per lane, 64 lanes)
  __shared__ __attribute__((aligned(1024))) unsigned char W1L[FM_W1B];
  __shared__ __attribute__((aligned(1024))) unsigned char W2L[DFF * FM_ROWB];
  __shared__ __attribute__((aligned(1024))) unsigned char patch[FM_WAVES * FM_PATCH];
  __shared__ __attribute__((aligned(1024))) unsigned char rvec[FM_WAVES * 2 * RVB];   // r of the wave's pair and of its next
  __shared__ __attribute__((aligned(16))) float vecs[DFF + 3 * D];                    // b1, b2, ln_g, ln_b

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char* opatch = patch + wave * FM_PATCH;
  const unsigned land = __builtin_amdgcn_readfirstlane(ffn_lds_addr(opatch));
  unsigned char* rmine = rvec + wave * 2 * RVB;
  const unsigned rland = __builtin_amdgcn_readfirstlane(ffn_lds_addr(rmine));
  const int stride = gridDim.x * FM_WAVES;
  int pr = blockIdx.x * FM_WAVES + wave;
  // segments of pair p that hold a valid item (the first ones)
  auto valid_segments = [&](int p) {
    const int n = (valid_len(lens, pair_user(cand_off, U, C, p), L) + w - 1) / w;
    return __builtin_amdgcn_readfirstlane(n < S ? n : S);
  };
  // rows i0 .. i0 + 31 of pair p into the landing area (rows past the last valid segment repeat it), r of pair p
  // into copy rb
  auto fetch_rows = [&](int p, int i0, int nvp) {
    ffn_fetch_rows(seg + ((size_t)p * S + i0) * D, nvp - i0 - 1 < FM_ROWS - 1 ? nvp - i0 - 1 : FM_ROWS - 1, land, lane);
  };
  auto fetch_r = [&](int p, int rb) { ffn_dma16(z + (size_t)p * D, (unsigned)((lane & 31) << 4), rland + rb * RVB); };

  int nv = pr < P ? valid_segments(pr) : 0;
  int rb = 0;
  ffn_park_weights<DFF>(__builtin_amdgcn_readfirstlane(ffn_lds_addr(W1L)), __builtin_amdgcn_readfirstlane(ffn_lds_addr(W2L)),
                        vecs, w1, w2, b1, b2, ln_g, ln_b, tid);
  if (nv > 0) {
    fetch_rows(pr, 0, nv);
    fetch_r(pr, 0);
  }
  ffn_wait_fetches();
  __syncthreads();
  const float* b1s = vecs;
  const float* b2s = vecs + DFF;
  const float* gs = vecs + DFF + D;
  const float* bs = vecs + DFF + 2 * D;
  FfnLane ln;
  ln.init(lane);
  constexpr int LPR = D / 8, RPI = 64 / LPR;
  const unsigned char* opr = opatch + (lane / LPR) * OP + (lane % LPR) * 16;
  const unsigned char* pcol = opatch + lane * 4;   // components 2 lane, 2 lane + 1 of row 0

  bf16x8 xreg[KSTEPS];
  if (nv > 0) ffn_read_rows(opatch, l32, h, xreg);
  for (; pr < P; pr += stride) {
    const int prn = pr + stride;
    const int nvn = prn < P ? valid_segments(prn) : 0;
    unsigned short* O = out ? out + (size_t)pr * S * D : nullptr;
    const float* rw = reinterpret_cast<const float*>(rmine + rb * RVB);
    unsigned short* R = (MR && recent) ? recent + (size_t)pr * r * D : nullptr;
    const int nr = R ? r : 0;
    float m = -INFINITY, den = 0.0f, p0 = 0.0f, p1 = 0.0f;
    float mx0 = -INFINITY, mx1 = -INFINITY;
    for (int i0 = 0; i0 < nv; i0 += FM_ROWS) {
      // the next tile with a valid segment: of this pair, else the first of the next pair (with its r)
      const bool same = i0 + FM_ROWS < nv;
      const bool more = same || nvn > 0;
      if (same) {
        fetch_rows(pr, i0 + FM_ROWS, nv);
      } else if (nvn > 0) {
        fetch_rows(prn, 0, nvn);
        fetch_r(prn, rb ^ 1);
      }
      const bool ok = i0 + l32 < nv;
      f32x16 acc[DB];
      ffn_tile_products<DFF>(xreg, ln, W1L, W2L, b1s, b2s, l32, h, acc);
      if (more) {   // the next tile's rows move into the registers of this one's before the patch is written
        ffn_wait_fetches();
        ffn_read_rows(opatch, l32, h, xreg);
      }
      float rstd, nmr;
      ffn_row_stats(acc, eps, rstd, nmr);
      // normalise, round (the value a stored s holds), park; the row's score against r from the rounded values.
      // Rows past the pair's last valid segment hold copies of it (see fetch_rows): finite like it, with weight
      // zero below, and replaced by zeros on their way out.
      float sdot = 0.0f;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        __builtin_amdgcn_sched_barrier(0);   // a column block at a time: hoisted together, the LDS reads of all four spill
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c0 = db * 32 + 8 * g + 4 * h;
          const f32x4 gg = *reinterpret_cast<const f32x4*>(gs + c0);
          const f32x4 bb = *reinterpret_cast<const f32x4*>(bs + c0);
          const f32x4 rr = *reinterpret_cast<const f32x4*>(rw + c0);
          u32x2 bits;
#pragma unroll
          for (int e2 = 0; e2 < 2; ++e2) {
            const bf16x2 o = {(__bf16)fmaf(fmaf(acc[db][4 * g + 2 * e2], rstd, nmr), gg[2 * e2], bb[2 * e2]),
                              (__bf16)fmaf(fmaf(acc[db][4 * g + 2 * e2 + 1], rstd, nmr), gg[2 * e2 + 1], bb[2 * e2 + 1])};
            const unsigned wd = __builtin_bit_cast(unsigned, o);
            bits[e2] = wd;
            sdot = fmaf(__uint_as_float(wd << 16), rr[2 * e2], sdot);
            sdot = fmaf(__uint_as_float(wd & 0xffff0000u), rr[2 * e2 + 1], sdot);
          }
          *reinterpret_cast<u32x2*>(opatch + l32 * OP + c0 * 2) = bits;
        }
      }
      sdot = ffn_both_halves_sum(sdot);
      // softmax over the tile's valid rows, merged into the pair's running sums (the tile has at least one). Row
      // reductions by lane permutations; the two rows of a half meet through scalar registers
      float mt = ffn_row_max(ok ? sdot : -INFINITY);
      {
        const int b = __float_as_int(mt);
        mt = fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16)));
      }
      const float m_new = fmaxf(m, mt);
      const float sc = __expf(m - m_new);   // 0 for the first tile (m = -inf)
      const float a = ok ? __expf(sdot - m_new) : 0.0f;
      float asum = row_sum<16>(a);
      {
        const int b = __float_as_int(asum);
        asum = __int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16));
      }
      den = fmaf(den, sc, asum);
      p0 *= sc;
      p1 *= sc;
      m = m_new;
      const int abits = __float_as_int(a);
#pragma unroll
      for (int row = 0; row < FM_ROWS; ++row) {
        const float ar = __int_as_float(__builtin_amdgcn_readlane(abits, row));
        const unsigned wd = *reinterpret_cast<const unsigned*>(pcol + row * OP);
        p0 = fmaf(ar, __uint_as_float(wd << 16), p0);
        p1 = fmaf(ar, __uint_as_float(wd & 0xffff0000u), p1);
        if (MR) {
          mx0 = fmaxf(mx0, __uint_as_float(wd << 16));
          mx1 = fmaxf(mx1, __uint_as_float(wd & 0xffff0000u));
        }
      }
      if (O) {   // rows leave as whole 256-byte rows (LDS operations of a wave execute in order: no barrier needed)
#pragma unroll
        for (int b = 0; b < FM_ROWS / RPI; ++b) {
          const int ii = i0 + b * RPI + lane / LPR;
          u32x4 val = *reinterpret_cast<const u32x4*>(opr + b * RPI * OP);
          if (ii >= nv) val = u32x4{0u, 0u, 0u, 0u};
          if (ii < S) *reinterpret_cast<u32x4*>(O + (size_t)ii * D + (lane % LPR) * 8) = val;
        }
      }
      if (MR && i0 < nr) {   // the same rows into the most recent segments' view
#pragma unroll
        for (int b = 0; b < FM_ROWS / RPI; ++b) {
          const int ii = i0 + b * RPI + lane / LPR;
          u32x4 val = *reinterpret_cast<const u32x4*>(opr + b * RPI * OP);
          if (ii >= nv) val = u32x4{0u, 0u, 0u, 0u};
          if (ii < nr) *reinterpret_cast<u32x4*>(R + (size_t)ii * D + (lane % LPR) * 8) = val;
        }
      }
    }
    if (MR && nr > 0) {   // its rows in the tiles without a valid segment: zeros
      for (int i0 = ((nv + FM_ROWS - 1) / FM_ROWS) * FM_ROWS; i0 < nr; i0 += FM_ROWS) {
#pragma unroll
        for (int b = 0; b < FM_ROWS / RPI; ++b) {
          const int ii = i0 + b * RPI + lane / LPR;
          if (ii < nr) *reinterpret_cast<u32x4*>(R + (size_t)ii * D + (lane % LPR) * 8) = u32x4{0u, 0u, 0u, 0u};
        }
      }
    }
    if (MR && pool) {   // maxima of stored values: their bits pass through
      pool[(size_t)pr * (D / 2) + lane] = nv > 0 ? ((__float_as_uint(mx0) >> 16) | (__float_as_uint(mx1) & 0xffff0000u)) : 0u;
    }
    if (O) {   // the rows of the tiles without a valid segment: zeros
      for (int i0 = ((nv + FM_ROWS - 1) / FM_ROWS) * FM_ROWS; i0 < S; i0 += FM_ROWS) {
#pragma unroll
        for (int b = 0; b < FM_ROWS / RPI; ++b) {
          const int ii = i0 + b * RPI + lane / LPR;
          if (ii < S) *reinterpret_cast<u32x4*>(O + (size_t)ii * D + (lane % LPR) * 8) = u32x4{0u, 0u, 0u, 0u};
        }
      }
    }
    const float inv = nv > 0 ? 1.0f / den : 0.0f;
    *reinterpret_cast<f32x2*>(z + (size_t)pr * D + 2 * lane) = f32x2{p0 * inv, p1 * inv};
    if (nv == 0 && nvn > 0) {   // nothing was multiplied for this pair, so nothing was requested for the next one
      fetch_rows(prn, 0, nvn);
      fetch_r(prn, rb ^ 1);
      ffn_wait_fetches();
      ffn_read_rows(opatch, l32, h, xreg);
    }
    if (nvn > 0) rb ^= 1;   // (a copy of r is only replaced by a fetch, and a fetch goes to the copy not in use)
    nv = nvn;
  }
}

// (the views come from the same pass: g.pool_out, g.recent_out and g.r as for the GSTA launchers)
bool ffn_gsta_fused_supports(const FfnArgs& f, const GstaArgs& g) {
  if (f.dt != LASER_BF16 || g.dt != LASER_BF16) return false;
  if (f.d != 128 || g.d != 128 || !(f.d_ff == 64 || f.d_ff == 128)) return false;
  return g.M == 1;
}

laser_status ffn_gsta_fused_launch(const FfnArgs& f, const GstaArgs& g) {
  if (!ffn_gsta_fused_supports(f, g)) return LASER_ERR_UNSUPPORTED;
  laser_status s = gsta_r_launch(g);
  if (s != LASER_OK) return s;
  const int P = f.cand_off ? f.P : f.U * f.C;
  long long blocks = ((long long)P + FM_WAVES - 1) / FM_WAVES;
  if (blocks > 256) blocks = 256;   // one workgroup per compute unit (LDS), each wave walking several pairs
  const bool views = g.pool_out != nullptr || g.recent_out != nullptr;
#define LASER_FFN_POOL(FF, MRF)                                                                                       \
  hipLaunchKernelGGL((ffn_pool_kernel<FF, MRF>), dim3((unsigned)blocks), dim3(FM_THREADS), 0, f.stream,               \
                     (const unsigned short*)f.seg, f.lens, (const unsigned short*)f.w1, f.b1,                        \
                     (const unsigned short*)f.w2, f.b2, f.ln_g, f.ln_b, f.cand_off, f.U, P, f.C, f.L, f.w, f.S, f.eps, \
                     (unsigned short*)f.seg_out, g.z_out, (unsigned*)g.pool_out, (unsigned short*)g.recent_out, g.r)
  if (f.d_ff == 64) { if (views) LASER_FFN_POOL(64, true); else LASER_FFN_POOL(64, false); }
  else { if (views) LASER_FFN_POOL(128, true); else LASER_FFN_POOL(128, false); }
#undef LASER_FFN_POOL
  s = launch_status();
  if (s != LASER_OK) return s;
  return gsta_out_launch(g);
}

}  // namespace laser
