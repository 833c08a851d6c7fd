// s_i <- LN(FFN(s_i) + s_i) on every segment vector of H' (paper Sec. 3.4.2, the equation that follows the STA
// paragraph), FFN(s) = relu(s W1 + b1) W2 + b2, LN over the d components with gain, bias and epsilon.
// Segments without a valid item are written as zeros.
//
// Two kernels. segment_ffn_generic_kernel: fp32 arithmetic, any d and d_ff, either storage type; a workgroup takes
// eight rows so that the weights, which it reads from L2, are used eight times. segment_ffn_mfma_kernel (below):
// bf16 storage, d = 128, d_ff in {64, 128}, both products on the matrix cores with the weights resident in LDS.
#include "segment_ffn_tile.h"

namespace laser {

constexpr int FG_ROWS = 8, FG_THREADS = 256;

template <typename T>
__global__ __launch_bounds__(FG_THREADS) void segment_ffn_generic_kernel(
    const T* seg, const int32_t* __restrict__ lens, const T* __restrict__ w1, const float* __restrict__ b1,
    const T* __restrict__ w2, const float* __restrict__ b2, const float* __restrict__ ln_g,
    const float* __restrict__ ln_b, const int32_t* __restrict__ cand_off, int U, long long rows, int C, int L, int d,
    int d_ff, int w, int S, float eps,
    T* out) {   // out may be seg: a workgroup has read its rows before it writes them
  extern __shared__ float sm[];            // x [FG_ROWS][d], hidden [FG_ROWS][d_ff], y [FG_ROWS][d], stats [FG_ROWS][2]
  float* x = sm;
  float* hid = x + FG_ROWS * d;
  float* y = hid + FG_ROWS * d_ff;
  float* stats = y + FG_ROWS * d;
  __shared__ int valid[FG_ROWS];
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * FG_ROWS;
  if (tid < FG_ROWS) {
    const long long r = row0 + tid;
    int ok = 0;
    if (r < rows) {
      const int i = (int)(r % S);
      const int u = pair_user(cand_off, U, C, (int)(r / S));
      ok = (long long)i * w < valid_len(lens, u, L);
    }
    valid[tid] = ok;
  }
  for (int e = tid; e < FG_ROWS * d; e += FG_THREADS) {
    const int rr = e / d, c = e - rr * d;
    const long long r = row0 + rr;
    x[e] = r < rows ? load_as_f32(seg, (size_t)r * d + c) : 0.0f;
  }
  __syncthreads();
  for (int j = tid; j < d_ff; j += FG_THREADS) {   // hidden unit j of the eight rows
    float acc[FG_ROWS];
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = b1[j];
    for (int e = 0; e < d; ++e) {
      const float wv = load_as_f32(w1, (size_t)e * d_ff + j);
#pragma unroll
      for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = fmaf(x[rr * d + e], wv, acc[rr]);
    }
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) hid[rr * d_ff + j] = fmaxf(acc[rr], 0.0f);
  }
  __syncthreads();
  for (int e = tid; e < d; e += FG_THREADS) {      // output component e of the eight rows, residual included
    float acc[FG_ROWS];
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = b2[e] + x[rr * d + e];
    for (int j = 0; j < d_ff; ++j) {
      const float wv = load_as_f32(w2, (size_t)j * d + e);
#pragma unroll
      for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = fmaf(hid[rr * d_ff + j], wv, acc[rr]);
    }
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) y[rr * d + e] = acc[rr];
  }
  __syncthreads();
  // mean and variance of each row: one wave per two rows, fixed order
  {
    const int wave = tid >> 6, lane = tid & 63;
    for (int rr = wave; rr < FG_ROWS; rr += FG_THREADS / 64) {
      float s = 0.0f;
      for (int e = lane; e < d; e += 64) s += y[rr * d + e];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
      const float mean = s / (float)d;
      float q = 0.0f;
      for (int e = lane; e < d; e += 64) {
        const float t = y[rr * d + e] - mean;
        q = fmaf(t, t, q);
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off, 64);
      if (lane == 0) {
        stats[rr * 2] = mean;
        stats[rr * 2 + 1] = 1.0f / sqrtf(q / (float)d + eps);
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < FG_ROWS * d; e += FG_THREADS) {
    const int rr = e / d, c = e - rr * d;
    const long long r = row0 + rr;
    if (r < rows) {
      const float o = valid[rr] ? (y[e] - stats[rr * 2]) * stats[rr * 2 + 1] * ln_g[c] + ln_b[c] : 0.0f;
      store_from_f32(out, (size_t)r * d + c, o);
    }
  }
}

bool segment_ffn_generic_supports(const FfnArgs& a) {
  const size_t lds = (size_t)FG_ROWS * (2 * a.d + a.d_ff + 2) * sizeof(float);
  return lds <= 150 * 1024;
}

laser_status segment_ffn_generic_launch(const FfnArgs& a) {
  if (!segment_ffn_generic_supports(a)) return LASER_ERR_UNSUPPORTED;
  const long long rows = (long long)(a.cand_off ? a.P : a.U * a.C) * a.S;
  const long long blocks = (rows + FG_ROWS - 1) / FG_ROWS;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  const size_t lds = (size_t)FG_ROWS * (2 * a.d + a.d_ff + 2) * sizeof(float);
  if (a.dt == LASER_BF16) {
    auto kern = segment_ffn_generic_kernel<unsigned short>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(FG_THREADS), lds, a.stream, (const unsigned short*)a.seg,
                       a.lens, (const unsigned short*)a.w1, a.b1, (const unsigned short*)a.w2, a.b2, a.ln_g, a.ln_b,
                       a.cand_off, a.U, rows, a.C, a.L, a.d, a.d_ff, a.w, a.S, a.eps, (unsigned short*)a.seg_out);
  } else {
    auto kern = segment_ffn_generic_kernel<float>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(FG_THREADS), lds, a.stream, (const float*)a.seg, a.lens,
                       (const float*)a.w1, a.b1, (const float*)a.w2, a.b2, a.ln_g, a.ln_b, a.cand_off, a.U, rows, a.C, a.L, a.d,
                       a.d_ff, a.w, a.S, a.eps, (float*)a.seg_out);
  }
  return launch_status();
}

}  // namespace laser

namespace laser {

// ------------------------------------------------------------------------------------------ matrix-core form
// The tile itself (operand scheme, weights and rows fetched straight into LDS, products, LayerNorm statistics) is in
// segment_ffn_tile.h. Here the rows are the flat [pairs * S] row space of H' in tiles of 32; 256 workgroups of 8
// waves walk the tiles with a grid stride, each wave with the rows of its next tile in flight while it multiplies.
// Normalised rows are rounded and leave through the wave's LDS patch as whole 256-byte rows. In place is safe: a
// wave's requests for a tile are complete before it writes that tile, and no other wave touches it.
template <int DFF>
__global__ __launch_bounds__(FM_THREADS) void segment_ffn_mfma_kernel(
    const unsigned short* seg, const int32_t* __restrict__ lens, const unsigned short* __restrict__ w1,
    const float* __restrict__ b1, const unsigned short* __restrict__ w2, const float* __restrict__ b2,
    const float* __restrict__ ln_g, const float* __restrict__ ln_b, const int32_t* __restrict__ cand_off, int U,
    long long rows, int C, int L, int w, int S, float eps,
    unsigned short* out) {
  constexpr int D = FM_D, KSTEPS = D / 16, DB = D / 32, OP = FM_OP;
  __shared__ __attribute__((aligned(1024))) unsigned char W1L[FM_W1B];
  __shared__ __attribute__((aligned(1024))) unsigned char W2L[DFF * FM_ROWB];
  __shared__ __attribute__((aligned(1024))) unsigned char patch[FM_WAVES * FM_PATCH];
  __shared__ __attribute__((aligned(16))) float vecs[DFF + 3 * D];             // b1, b2, ln_g, ln_b

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char* opatch = patch + wave * FM_PATCH;
  const unsigned land = __builtin_amdgcn_readfirstlane(ffn_lds_addr(opatch));
  const long long ntiles = (rows + FM_ROWS - 1) / FM_ROWS;
  const long long stride = (long long)gridDim.x * FM_WAVES;
  long long t = (long long)blockIdx.x * FM_WAVES + wave;
  // rows of tile tt into the landing area (rows past the end repeat the last one; never stored)
  auto fetch_tile = [&](long long tt) {
    const long long r0 = tt * FM_ROWS;
    const long long left = rows - r0 - 1;
    ffn_fetch_rows(seg + (size_t)r0 * D, left < FM_ROWS - 1 ? (int)left : FM_ROWS - 1, land, lane);
  };
  ffn_park_weights<DFF>(__builtin_amdgcn_readfirstlane(ffn_lds_addr(W1L)), __builtin_amdgcn_readfirstlane(ffn_lds_addr(W2L)),
                        vecs, w1, w2, b1, b2, ln_g, ln_b, tid);
  if (t < ntiles) fetch_tile(t);
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

  // Does this lane's row of tile tt belong to a segment with a valid item: first item of the segment and the user's
  // valid length. The length of the next tile's row is requested ahead of that tile's fetch and compared after the
  // products (a vector load awaited while the fetch is in flight would wait for the fetch as well).
  struct RowLen { long long first; int len; };
  auto row_len = [&](long long tt) {
    const long long r = tt * FM_ROWS + l32;
    RowLen o{1, 0};
    if (r < rows) {   // (rows < 2^31: 32-bit division)
      const unsigned pr = (unsigned)r / (unsigned)S;
      o.first = (long long)((unsigned)r - pr * (unsigned)S) * w;
      o.len = valid_len(lens, pair_user(cand_off, U, C, (int)pr), L);
    }
    return o;
  };
  bf16x8 xreg[KSTEPS];
  bool ok = false;
  if (t < ntiles) {
    ffn_read_rows(opatch, l32, h, xreg);
    const RowLen rl = row_len(t);
    ok = rl.first < rl.len;
  }
  for (; t < ntiles; t += stride) {
    const long long r0 = t * FM_ROWS;
    const bool more = t + stride < ntiles;
    RowLen nxt{1, 0};
    if (more) {
      nxt = row_len(t + stride);
      fetch_tile(t + stride);   // the patch is idle: the previous tile's rows have left it
    }
    f32x16 acc[DB];
    ffn_tile_products<DFF>(xreg, ln, W1L, W2L, b1s, b2s, l32, h, acc);
    if (more) {   // the next tile's rows move into the registers of this one's before the patch is written
      ffn_wait_fetches();
      ffn_read_rows(opatch, l32, h, xreg);
    }
    // ---- LayerNorm over d, gain, bias: two multiply-adds per value; rows of segments without a valid item are zeros
    float rstd, nmr;
    ffn_row_stats(acc, eps, rstd, nmr);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      __builtin_amdgcn_sched_barrier(0);   // a column block at a time (register pressure)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 gg = *reinterpret_cast<const f32x4*>(gs + db * 32 + 8 * g + 4 * h);
        const f32x4 bb = *reinterpret_cast<const f32x4*>(bs + db * 32 + 8 * g + 4 * h);
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (__bf16)fmaf(fmaf(acc[db][4 * g + e], rstd, nmr), gg[e], bb[e]);
        u32x2 bits = __builtin_bit_cast(u32x2, o);
        if (!ok) bits = u32x2{0u, 0u};
        *reinterpret_cast<u32x2*>(opatch + l32 * OP + (db * 32 + g * 8 + h * 4) * 2) = bits;
      }
    }
    // ---- rows leave as whole 256-byte rows (LDS operations of a wave execute in order: no barrier needed)
#pragma unroll
    for (int b = 0; b < FM_ROWS / RPI; ++b) {
      const int rr = b * RPI + lane / LPR;
      const u32x4 val = *reinterpret_cast<const u32x4*>(opr + b * RPI * OP);
      if (r0 + rr < rows) *reinterpret_cast<u32x4*>(out + (size_t)(r0 + rr) * D + (lane % LPR) * 8) = val;
    }
    ok = nxt.first < nxt.len;
  }
}

bool segment_ffn_mfma_supports(const FfnArgs& a) {
  return a.dt == LASER_BF16 && a.d == 128 && (a.d_ff == 64 || a.d_ff == 128);
}

laser_status segment_ffn_mfma_launch(const FfnArgs& a) {
  if (!segment_ffn_mfma_supports(a)) return LASER_ERR_UNSUPPORTED;
  const long long rows = (long long)(a.cand_off ? a.P : a.U * a.C) * a.S;
  const long long ntiles = (rows + FM_ROWS - 1) / FM_ROWS;
  long long blocks = (ntiles + FM_WAVES - 1) / FM_WAVES;
  if (blocks > 256) blocks = 256;   // one workgroup per compute unit (LDS), each walking several tiles per wave
#define LASER_FFN_LAUNCH(FF)                                                                                          \
  hipLaunchKernelGGL((segment_ffn_mfma_kernel<FF>), dim3((unsigned)blocks), dim3(FM_THREADS), 0, a.stream,            \
                     (const unsigned short*)a.seg, a.lens, (const unsigned short*)a.w1, a.b1,                        \
                     (const unsigned short*)a.w2, a.b2, a.ln_g, a.ln_b, a.cand_off, a.U, rows, a.C, a.L, a.w, a.S, a.eps, \
                     (unsigned short*)a.seg_out)
  if (a.d_ff == 64) LASER_FFN_LAUNCH(64);
  else LASER_FFN_LAUNCH(128);
#undef LASER_FFN_LAUNCH
  return launch_status();
}

}  // namespace laser
