// Segment FFN + LayerNorm (paper Sec. 3.4.2, s <- LN(FFN(s) + s)) feeding the GSTA layer (Sec. 3.4.3) from one pass
// over H': the normalised segment vectors of a pair are scored against r = W_k (t0 W_q)^T / sqrt(d) and pooled with
// their softmax weights while they are still on chip, so the transformed H' is neither written nor read back
// (it is written as well when the caller wants it). One layer, bf16, d = 128, d_ff in {64, 128}.
//
// Three launches, the outer two shared with the split form of GSTA (gsta_tiled.hip):
//   gsta_r_kernel     r = (t0 W_q) W_k^T / sqrt(d)   tiles of 32 pairs, MFMA                       -> z rows
//   ffn_pool_kernel   below: a wave walks pairs       H' rows -> s rows (on chip), z rows (r) -> z rows (p)
//   gsta_out_kernel   z = t0 + p W_v                  tiles of 32 pairs, MFMA             z rows -> z rows
// with p = sum_i a_i s_i, a = softmax over the segments that hold a valid item of r . s_i (the attention equation
// with its products re-associated, which is exact).
//
// ffn_pool_kernel: the FFN tile of segment_ffn_tile.h on the valid rows (the first nv segments, the ones that hold a
// valid item) of the pairs a wave walks with a grid stride, one pair after the other, cut into tiles of 32 as one
// stream: a tile holds rows of one pair, or the last rows of one followed by the first of the next, so that only the
// wave's last tile is padded (with copies of its last row, which count as empty). The rows of the remaining segments
// are never read (whatever H' holds there is not trusted): they, and the results of a pair without any valid
// segment, are written by a pass of their own before the first tile. The rows of the wave's next tile and r of the
// pairs that start in it are in flight while it multiplies. After LayerNorm a lane holds, in the accumulator layout,
// 64 of the 128 components of row l32: the rounded values (what a stored s would hold) are multiplied with the same
// components of its pair's r, read from a wave-private LDS copy, and one exchange with lane ^ 32 gives the row's
// score. Maximum and sum over the rows of a pair in the tile are wave reductions; tiles of a pair are merged with the
// running maximum (online softmax). The weighted sum over rows is taken from the LDS patch the rounded rows are
// parked in: lane l owns components 2 l and 2 l + 1 and reads one word per row, with the row's weight from
// v_readlane. p / sum of weights replaces r in the pair's z row.
#include "segment_ffn_tile.h"

namespace laser {

// Request a tile that holds rows of two pairs: rows a0 .. a0 + na - 1 of the pair whose row 0 is at `rowsA`, then rows
// 0 .. nb - 1 of the pair whose row 0 lies dB bytes further (nb >= 1); tile rows past the last one repeat it.
__device__ __forceinline__ void ffn_fetch_rows_two(const unsigned short* rowsA, int a0, int na, unsigned dB, int nb,
                                                   unsigned land, int lane) {
  asm volatile("" : "+v"(lane));   // (as in ffn_fetch_rows)
  const int q = lane >> 4, pos = lane & 15;
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  const int last = na + nb - 1;
#pragma unroll
  for (int j = 0; j < FM_ROWS / 4; ++j) {
    const int row = 4 * j + q;
    const int src = row < last ? row : last;
    const unsigned off = src < na ? (unsigned)(a0 + src) * FM_ROWB : dB + (unsigned)(src - na) * FM_ROWB;
    ffn_dma16(rowsA, off + ((pos ^ (row & 15)) << 4), land + j * 1024);
  }
}

// MR: also the two other views of Sec. 3.4.4 of the transformed rows: pool [P, D] bf16, the component-wise maximum
// over the segments that hold a valid item (zeros when there is none), taken in the weighted-sum loop from the same
// words (tile rows past the last one are copies of it, so they leave the maximum alone); recent [P, r, D] bf16,
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
  constexpr int RVB = 512, RSLOTS = 4;   // copies of r per wave: the pairs of the tile in work and of the next one
  __shared__ __attribute__((aligned(1024))) unsigned char W1L[FM_W1B];
  __shared__ __attribute__((aligned(1024))) unsigned char W2L[DFF * FM_ROWB];
  __shared__ __attribute__((aligned(1024))) unsigned char patch[FM_WAVES * FM_PATCH];
  __shared__ __attribute__((aligned(1024))) unsigned char rvec[FM_WAVES * RSLOTS * RVB];
  __shared__ __attribute__((aligned(16))) float vecs[DFF + 3 * D];                    // b1, b2, ln_g, ln_b

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char* opatch = patch + wave * FM_PATCH;
  const unsigned land = __builtin_amdgcn_readfirstlane(ffn_lds_addr(opatch));
  unsigned char* rmine = rvec + wave * RSLOTS * RVB;
  const unsigned rland = __builtin_amdgcn_readfirstlane(ffn_lds_addr(rmine));
  const int stride = gridDim.x * FM_WAVES;
  const int pr0 = blockIdx.x * FM_WAVES + wave;   // the wave's k-th pair is pr0 + k * stride
  // segments of pair p that hold a valid item (the first ones)
  auto valid_segments = [&](int p) {
    const int n = (valid_len(lens, pair_user(cand_off, U, C, p), L) + w - 1) / w;
    return __builtin_amdgcn_readfirstlane(n < S ? n : S);
  };
  constexpr int LPR = D / 8, RPI = 64 / LPR;
  const int nr = (MR && recent) ? (r < S ? r : S) : 0;
  // The wave's first pair at or after its k-th that has a valid segment (nvk > 0), else nvk = 0. Every pair of the
  // wave is looked at here exactly once, in order, and gets what the tiles never touch: the rows of its segments
  // without a valid item leave as zeros, and a pair without any has p = 0 and a pooled maximum of zeros.
  auto next_pair = [&](int k, int& nvk) {
    nvk = 0;
    while (pr0 + k * stride < P) {
      const int p = pr0 + k * stride;
      nvk = valid_segments(p);
      if (out)
        for (int i = nvk + lane / LPR; i < S; i += RPI)
          *reinterpret_cast<u32x4*>(out + ((size_t)p * S + i) * D + (lane % LPR) * 8) = u32x4{0u, 0u, 0u, 0u};
      if (MR && recent)
        for (int i = nvk + lane / LPR; i < nr; i += RPI)
          *reinterpret_cast<u32x4*>(recent + ((size_t)p * r + i) * D + (lane % LPR) * 8) = u32x4{0u, 0u, 0u, 0u};
      if (nvk > 0) break;
      if (MR && pool) pool[(size_t)p * (D / 2) + lane] = 0u;
      *reinterpret_cast<f32x2*>(z + (size_t)p * D + 2 * lane) = f32x2{0.0f, 0.0f};
      ++k;
    }
    return k;
  };
  // The valid rows of the wave's pairs, one pair after the other, are cut into tiles of 32: a tile holds rows
  // a0 .. a0 + na - 1 of pair A and, when A ends inside it and there is room, the first nb rows of the next pair
  // with a valid segment, B (which may end inside the tile too). ord counts the pairs with a valid segment.
  struct Tile {
    bool some;
    int kA, nvA, a0, na;
    int kB, nvB, nb;   // with A ending in the tile: the next pair (nvB == 0: there is none) and its rows in the tile
    int ord;
  };
  auto make_tile = [&](int k, int nvk, int off, int ord) {
    Tile t;
    t.some = nvk > 0;
    t.kA = k; t.nvA = nvk; t.a0 = off; t.ord = ord;
    t.na = nvk - off < FM_ROWS ? nvk - off : FM_ROWS;
    t.kB = k; t.nvB = 0; t.nb = 0;
    if (t.some && off + t.na == nvk) {
      t.kB = next_pair(k + 1, t.nvB);
      const int room = FM_ROWS - t.na;
      t.nb = t.nvB < room ? t.nvB : room;
    }
    return t;
  };
  auto tile_after = [&](const Tile& t) {
    if (t.a0 + t.na < t.nvA) return make_tile(t.kA, t.nvA, t.a0 + t.na, t.ord);   // A goes on
    if (t.nb < t.nvB) return make_tile(t.kB, t.nvB, t.nb, t.ord + 1);             // B goes on (or starts)
    int nvn = 0, kn = t.kB;
    if (t.nvB > 0) kn = next_pair(t.kB + 1, nvn);                                  // B ended here as well
    return make_tile(kn, nvn, 0, t.ord + 2);
  };
  auto fetch_r = [&](int p, int slot) {   // 512 bytes: 16 per lane of the lower half of the wave
    if (lane < 32) ffn_dma16(z + (size_t)p * D, (unsigned)(lane << 4), rland + (slot & (RSLOTS - 1)) * RVB);
  };
  // the rows of tile t into the landing area, and r of the pairs that start in it
  auto fetch_tile = [&](const Tile& t) {
    const int pA = pr0 + t.kA * stride;
    const unsigned short* rowsA = seg + (size_t)pA * S * D;
    if (t.nb == 0) {
      ffn_fetch_rows(rowsA + (size_t)t.a0 * D, t.na - 1, land, lane);
    } else {
      const unsigned dB = (unsigned)(t.kB - t.kA) * (unsigned)stride * (unsigned)S * (unsigned)(D * 2);
      ffn_fetch_rows_two(rowsA, t.a0, t.na, dB, t.nb, land, lane);
      fetch_r(pr0 + t.kB * stride, t.ord + 1);
    }
    if (t.a0 == 0) fetch_r(pA, t.ord);
  };

  int nv0 = 0;
  const int k0 = next_pair(0, nv0);
  Tile cur = make_tile(k0, nv0, 0, 0);
  ffn_park_weights<DFF>(__builtin_amdgcn_readfirstlane(ffn_lds_addr(W1L)), __builtin_amdgcn_readfirstlane(ffn_lds_addr(W2L)),
                        vecs, w1, w2, b1, b2, ln_g, ln_b, tid);
  if (cur.some) fetch_tile(cur);

  ffn_wait_fetches();
  __syncthreads();
  const float* b1s = vecs;
  const float* b2s = vecs + DFF;
  const float* gs = vecs + DFF + D;
  const float* bs = vecs + DFF + 2 * D;
  FfnLane ln;
  ln.init(lane);
  const unsigned char* opr = opatch + (lane / LPR) * OP + (lane % LPR) * 16;
  const unsigned char* pcol = opatch + lane * 4;   // components 2 lane, 2 lane + 1 of row 0

  // maximum over the wave's rows (the value of a row sits in its 16-lane group's lanes l32 and l32 + 32)
  auto rows_max = [&](float v) {
    const int b = __float_as_int(ffn_row_max(v));
    return fmaxf(__int_as_float(__builtin_amdgcn_readlane(b, 0)), __int_as_float(__builtin_amdgcn_readlane(b, 16)));
  };
  auto rows_sum = [&](float v) {
    const int b = __float_as_int(row_sum<16>(v));
    return __int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16));
  };
  // a finished pair: its pooled maximum (bits of stored values pass through) and p / sum of weights in place of r
  auto finish_pair = [&](int p, float den, float p0, float p1, float mx0, float mx1) {
    if (MR && pool) pool[(size_t)p * (D / 2) + lane] = (__float_as_uint(mx0) >> 16) | (__float_as_uint(mx1) & 0xffff0000u);
    const float inv = 1.0f / den;
    *reinterpret_cast<f32x2*>(z + (size_t)p * D + 2 * lane) = f32x2{p0 * inv, p1 * inv};
  };

  bf16x8 xreg[KSTEPS];
  if (cur.some) ffn_read_rows(opatch, l32, h, xreg);
  // running sums of pair A (online softmax over its tiles)
  float m = -INFINITY, den = 0.0f, p0 = 0.0f, p1 = 0.0f, mx0 = -INFINITY, mx1 = -INFINITY;
  while (cur.some) {
    const Tile nxt = tile_after(cur);
    if (nxt.some) fetch_tile(nxt);
    const int na = cur.na, nb = cur.nb, ntot = na + nb;
    const int pA = pr0 + cur.kA * stride, pB = pr0 + cur.kB * stride;
    const bool ok = l32 < ntot;
    const bool isB = nb > 0 && l32 >= na;
    const float* rw = reinterpret_cast<const float*>(rmine + ((cur.ord + (isB ? 1 : 0)) & (RSLOTS - 1)) * RVB);
    f32x16 acc[DB];
    ffn_tile_products<DFF>(xreg, ln, W1L, W2L, b1s, b2s, l32, h, acc);
    if (nxt.some) {   // the next tile's rows move into the registers of this one's before the patch is written
      ffn_wait_fetches();
      ffn_read_rows(opatch, l32, h, xreg);
    }
    float rstd, nmr;
    ffn_row_stats(acc, eps, rstd, nmr);
    // normalise, round (the value a stored s holds), park; the row's score against its pair's r from the rounded
    // values. Tile rows past the last one hold copies of it: finite like it, with weight zero below.
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
    // softmax over the tile's rows, merged into the pair's running sums. Row reductions by lane permutations; the
    // two rows of a half meet through scalar registers. The weighted sum over rows is taken from the parked words
    // (LDS operations of a wave execute in order: no barrier needed), a row's weight from v_readlane.
    if (nb == 0) {   // one pair in the tile
      const float m_new = fmaxf(m, rows_max(ok ? sdot : -INFINITY));
      const float sc = __expf(m - m_new);   // 0 for the pair's first tile (m = -inf)
      const float a = ok ? __expf(sdot - m_new) : 0.0f;
      den = fmaf(den, sc, rows_sum(a));
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
    }
    float q0 = 0.0f, q1 = 0.0f, nx0 = -INFINITY, nx1 = -INFINITY, mB = -INFINITY, denB = 0.0f;   // pair B's sums
    if (nb > 0) {    // A's last rows, then B's first
      const float m_new = fmaxf(m, rows_max(isB ? -INFINITY : sdot));
      mB = rows_max(isB && ok ? sdot : -INFINITY);
      const float sc = __expf(m - m_new);
      const float a = ok ? __expf(sdot - (isB ? mB : m_new)) : 0.0f;
      den = fmaf(den, sc, rows_sum(isB ? 0.0f : a));
      denB = rows_sum(isB ? a : 0.0f);
      p0 *= sc;
      p1 *= sc;
      const int abits = __float_as_int(a);
#pragma unroll
      for (int row = 0; row < FM_ROWS; ++row) {
        const bool rowA = row < na;   // uniform: the selects below are scalar
        const float ar = __int_as_float(__builtin_amdgcn_readlane(abits, row));
        const float arA = rowA ? ar : 0.0f, arB = rowA ? 0.0f : ar;
        const unsigned wd = *reinterpret_cast<const unsigned*>(pcol + row * OP);
        const float lo = __uint_as_float(wd << 16), hi = __uint_as_float(wd & 0xffff0000u);
        p0 = fmaf(arA, lo, p0);
        p1 = fmaf(arA, hi, p1);
        q0 = fmaf(arB, lo, q0);
        q1 = fmaf(arB, hi, q1);
        if (MR) {
          mx0 = fmaxf(mx0, rowA ? lo : -INFINITY);
          mx1 = fmaxf(mx1, rowA ? hi : -INFINITY);
          nx0 = fmaxf(nx0, rowA ? -INFINITY : lo);
          nx1 = fmaxf(nx1, rowA ? -INFINITY : hi);
        }
      }
    }
    // rows on their way out, as whole 256-byte rows: tile row j is row a0 + j of A or row j - na of B. Without the
    // transformed rows wanted, only the tile rows that belong to the first r of their pair leave (jr: one past the
    // last of them), four at a time.
    {
      const unsigned dBpairs = (unsigned)(cur.kB - cur.kA) * (unsigned)stride;   // pairs between A and B
      auto rows_out = [&](int b) {
        const int j = b * RPI + lane / LPR;
        const u32x4 val = *reinterpret_cast<const u32x4*>(opr + b * RPI * OP);
        const bool jb = j >= na;
        const int i = jb ? j - na : cur.a0 + j;              // segment index inside its pair
        const unsigned pj = jb ? dBpairs : 0u;               // pair, counted from A
        if (j < ntot) {
          if (out) *reinterpret_cast<u32x4*>(out + ((size_t)pA * S + (size_t)pj * S + i) * D + (lane % LPR) * 8) = val;
          if (MR && i < nr)
            *reinterpret_cast<u32x4*>(recent + ((size_t)pA * r + (size_t)pj * r + i) * D + (lane % LPR) * 8) = val;
        }
      };
      if (out) {
#pragma unroll
        for (int b = 0; b < FM_ROWS / RPI; ++b) rows_out(b);
      } else if (MR) {
        int jr = nr == 0 ? 0 : (nb > 0 ? na + nr : nr - cur.a0);
        jr = jr < ntot ? jr : ntot;
#pragma unroll 1
        for (int b = 0; b * RPI < jr; ++b) rows_out(b);
      }
    }
    if (nb > 0) {   // A ended; B's sums become the running ones, unless B ended here too
      finish_pair(pA, den, p0, p1, mx0, mx1);
      if (nb == cur.nvB) {
        finish_pair(pB, denB, q0, q1, nx0, nx1);
        m = -INFINITY; den = 0.0f; p0 = 0.0f; p1 = 0.0f; mx0 = -INFINITY; mx1 = -INFINITY;
      } else {
        m = mB; den = denB; p0 = q0; p1 = q1; mx0 = nx0; mx1 = nx1;
      }
    } else if (cur.a0 + na == cur.nvA) {
      finish_pair(pA, den, p0, p1, mx0, mx1);
      m = -INFINITY; den = 0.0f; p0 = 0.0f; p1 = 0.0f; mx0 = -INFINITY; mx1 = -INFINITY;
    }
    cur = nxt;
  }
}

// (the views come from the same pass: g.pool_out, g.recent_out and g.r as for the GSTA launchers)
bool ffn_gsta_fused_supports(const FfnArgs& f, const GstaArgs& g) {
  if (f.dt != LASER_BF16 || g.dt != LASER_BF16) return false;
  if (f.d != 128 || g.d != 128 || !(f.d_ff == 64 || f.d_ff == 128)) return false;
  // a tile's rows are addressed by 32-bit byte offsets from the row 0 of its first pair
  const long long P = f.cand_off ? f.P : (long long)f.U * f.C;
  if (P * f.S * f.d * 2 >= (1LL << 32)) return false;
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
