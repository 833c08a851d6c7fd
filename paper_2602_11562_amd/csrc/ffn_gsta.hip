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
// ffn_pool_kernel: the FFN tile of segment_ffn_tile.h on the rows of one pair at a time (ceil(S / 32) tiles of 32
// rows; rows past S repeat the last one and count as empty). After LayerNorm a lane holds, in the accumulator layout,
// 64 of the 128 components of row l32: the rounded values (what a stored s would hold) are multiplied with the same
// components of r, read from a wave-private LDS copy, and one exchange with lane ^ 32 gives the row's score. Maximum
// and sum over the tile's rows are wave reductions; tiles of a pair are merged with the running maximum (online
// softmax). The weighted sum over rows is taken from the LDS patch the rounded rows are parked in: lane l owns
// components 2 l and 2 l + 1 and reads one word per row, with the row's weight from v_readlane. Rows of segments
// without a valid item are parked as zeros: they carry weight zero, and whatever H' holds there (it is never
// trusted) cannot reach the sums. p / sum of weights replaces r in the pair's z row.
#include "segment_ffn_tile.h"

namespace laser {

template <int DFF>
__global__ __launch_bounds__(FM_THREADS) void ffn_pool_kernel(
    const unsigned short* seg, const int32_t* __restrict__ lens, const unsigned short* __restrict__ w1,
    const float* __restrict__ b1, const unsigned short* __restrict__ w2, const float* __restrict__ b2,
    const float* __restrict__ ln_g, const float* __restrict__ ln_b, const int32_t* __restrict__ cand_off, int U, int P,
    int C, int L, int w, int S, float eps,
    unsigned short* out,   // s rows [P, S, D], may be null (not wanted), may be seg
    float* z) {            // [P, D]: r on entry, p on exit
  constexpr int D = FM_D, KSTEPS = D / 16, DB = D / 32, OP = FM_OP;
  __shared__ __attribute__((aligned(1024))) unsigned char W2L[DFF * FM_ROWB];
  __shared__ __attribute__((aligned(16))) unsigned char W1T[DFF * FM_W1P];
  __shared__ __attribute__((aligned(16))) unsigned char patch[FM_WAVES * FM_ROWS * OP];
  __shared__ __attribute__((aligned(16))) float vecs[DFF + 3 * D];             // b1, b2, ln_g, ln_b
  __shared__ __attribute__((aligned(16))) float rvec[FM_WAVES][D];             // r of the wave's pair

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  ffn_park_weights<DFF>(W1T, W2L, vecs, w1, w2, b1, b2, ln_g, ln_b, tid);
  __syncthreads();
  const float* b1s = vecs;
  const float* b2s = vecs + DFF;
  const float* gs = vecs + DFF + D;
  const float* bs = vecs + DFF + 2 * D;
  FfnLane ln;
  ln.init(W1T, lane);
  unsigned char* opatch = patch + wave * FM_ROWS * OP;
  constexpr int LPR = D / 8, RPI = 64 / LPR;
  const unsigned char* opr = opatch + (lane / LPR) * OP + (lane % LPR) * 16;
  const unsigned char* pcol = opatch + lane * 4;   // components 2 lane, 2 lane + 1 of row 0
  float* rw = rvec[wave];
  const int tpp = (S + FM_ROWS - 1) / FM_ROWS;     // tiles per pair

  for (int pr = blockIdx.x * FM_WAVES + wave; pr < P; pr += gridDim.x * FM_WAVES) {
    const int u = pair_user(cand_off, U, C, pr);
    int nv = (valid_len(lens, u, L) + w - 1) / w;   // segments with a valid item (the first nv)
    nv = __builtin_amdgcn_readfirstlane(nv < S ? nv : S);
    *reinterpret_cast<f32x2*>(rw + 2 * lane) = *reinterpret_cast<const f32x2*>(z + (size_t)pr * D + 2 * lane);
    const unsigned short* H = seg + (size_t)pr * S * D;
    unsigned short* O = out ? out + (size_t)pr * S * D : nullptr;
    float m = -INFINITY, den = 0.0f, p0 = 0.0f, p1 = 0.0f;
    for (int t = 0; t < tpp; ++t) {
      const int i0 = t * FM_ROWS;
      if (i0 >= nv) {   // no valid segment in this tile (wave-uniform): nothing to add; the rows are zeros
        if (O) {
#pragma unroll
          for (int b = 0; b < FM_ROWS / RPI; ++b) {
            const int i = i0 + b * RPI + lane / LPR;
            if (i < S) *reinterpret_cast<u32x4*>(O + (size_t)i * D + (lane % LPR) * 8) = u32x4{0u, 0u, 0u, 0u};
          }
        }
        continue;
      }
      const int i = i0 + l32;
      const bool ok = i < nv;
      bf16x8 xreg[KSTEPS];
      {
        const unsigned short* xr = H + (size_t)(i < S ? i : S - 1) * D + h * 8;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) xreg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xr + ks * 16));
      }
      f32x16 acc[DB];
      ffn_tile_products<DFF>(xreg, ln, W2L, b1s, b2s, h, acc);
      float rstd, nmr;
      ffn_row_stats(acc, eps, rstd, nmr);
      // normalise, round (the value a stored s holds), park; the row's score against r from the rounded values
      float sdot = 0.0f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c0 = db * 32 + 8 * g + 4 * h;
          const f32x4 gg = *reinterpret_cast<const f32x4*>(gs + c0);
          const f32x4 bb = *reinterpret_cast<const f32x4*>(bs + c0);
          const f32x4 rr = *reinterpret_cast<const f32x4*>(rw + c0);
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = (__bf16)fmaf(fmaf(acc[db][4 * g + e], rstd, nmr), gg[e], bb[e]);
            sdot = fmaf((float)o[e], rr[e], sdot);
          }
          u32x2 bits = __builtin_bit_cast(u32x2, o);
          if (!ok) bits = u32x2{0u, 0u};
          *reinterpret_cast<u32x2*>(opatch + l32 * OP + c0 * 2) = bits;
        }
      sdot += __shfl_xor(sdot, 32, 64);
      // softmax over the tile's valid rows, merged into the pair's running sums (the tile has at least one)
      float mt = ok ? sdot : -INFINITY;
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) mt = fmaxf(mt, __shfl_xor(mt, off, 64));
      const float m_new = fmaxf(m, mt);
      const float sc = __expf(m - m_new);   // 0 for the first tile (m = -inf)
      const float a = ok ? __expf(sdot - m_new) : 0.0f;
      float asum = a;
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) asum += __shfl_xor(asum, off, 64);
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
      }
      if (O) {   // rows leave as whole 256-byte rows (LDS operations of a wave execute in order: no barrier needed)
#pragma unroll
        for (int b = 0; b < FM_ROWS / RPI; ++b) {
          const int ii = i0 + b * RPI + lane / LPR;
          const u32x4 val = *reinterpret_cast<const u32x4*>(opr + b * RPI * OP);
          if (ii < S) *reinterpret_cast<u32x4*>(O + (size_t)ii * D + (lane % LPR) * 8) = val;
        }
      }
    }
    const float inv = nv > 0 ? 1.0f / den : 0.0f;
    *reinterpret_cast<f32x2*>(z + (size_t)pr * D + 2 * lane) = f32x2{p0 * inv, p1 * inv};
  }
}

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
#define LASER_FFN_POOL(FF)                                                                                            \
  hipLaunchKernelGGL((ffn_pool_kernel<FF>), dim3((unsigned)blocks), dim3(FM_THREADS), 0, f.stream,                    \
                     (const unsigned short*)f.seg, f.lens, (const unsigned short*)f.w1, f.b1,                        \
                     (const unsigned short*)f.w2, f.b2, f.ln_g, f.ln_b, f.cand_off, f.U, P, f.C, f.L, f.w, f.S, f.eps, \
                     (unsigned short*)f.seg_out, g.z_out)
  if (f.d_ff == 64) LASER_FFN_POOL(64);
  else LASER_FFN_POOL(128);
#undef LASER_FFN_POOL
  s = launch_status();
  if (s != LASER_OK) return s;
  return gsta_out_launch(g);
}

}  // namespace laser
