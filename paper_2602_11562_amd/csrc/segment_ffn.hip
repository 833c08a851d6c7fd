// s_i <- LN(FFN(s_i) + s_i) on every segment vector of H' (paper Sec. 3.4.2, the equation that follows the STA
// paragraph), FFN(s) = relu(s W1 + b1) W2 + b2, LN over the d components with gain, bias and epsilon.
// Segments without a valid item are written as zeros.
//
// Two kernels. segment_ffn_generic_kernel: fp32 arithmetic, any d and d_ff, either storage type; a workgroup takes
// eight rows so that the weights, which it reads from L2, are used eight times. segment_ffn_mfma_kernel (below):
// bf16 storage, d = 128, d_ff in {64, 128}, both products on the matrix cores with the weights resident in LDS.
#include "laser_internal.h"

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
// Same operand scheme as the STA kernels (sta_mfma.hip), with the first-layer weights in the place of the keys and
// the second-layer weights in the place of the values. A wave owns 32 rows of H' at a time (its B operand, read
// once into registers) and walks the hidden layer in tiles of 32 units:
//   hid^T [32 units x 32 rows] = W1^T tile . X^T      (v_mfma_f32_32x32x16_bf16, A from LDS 16 bytes per lane)
//   + b1, relu, rounded to bf16: the accumulator layout is, per 16 units, a valid B operand of
//   Y^T [d x 32 rows] += W2 tile^T . hid             (A fetched by ds_read_b64_tr_b16 from W2 rows as stored)
// The residual enters as one more product, identity x X^T (exact), so that it needs no other copy of X. Then b2,
// LayerNorm (a row's d values sit in one lane pair: a sum per lane and one exchange), rounding, and the rows leave
// through a wave-private LDS patch as whole 256-byte rows. Weights are parked once per workgroup (W1 transposed on
// the way, padded rows; W2 in 32-row tiles with the XOR swizzle of the STA value tiles); workgroups walk the row
// tiles with a grid stride. In place is safe: a wave has its 32 rows in registers before it writes them.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int FM_WAVES = 8, FM_THREADS = 64 * FM_WAVES, FM_ROWS = 32;

__device__ __forceinline__ bf16x8 ffn_lds_tr(const unsigned char* p) {   // see lds_read_tr in sta_mfma.hip
  typedef __attribute__((address_space(3))) s16x4* lds4;
  const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4)(size_t)(unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p);
  const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4)(size_t)(unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)(p + 2048));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
}

template <int DFF>
__global__ __launch_bounds__(FM_THREADS) void segment_ffn_mfma_kernel(
    const unsigned short* seg, const int32_t* __restrict__ lens, const unsigned short* __restrict__ w1,
    const float* __restrict__ b1, const unsigned short* __restrict__ w2, const float* __restrict__ b2,
    const float* __restrict__ ln_g, const float* __restrict__ ln_b, const int32_t* __restrict__ cand_off, int U,
    long long rows, int C, int L, int w, int S, float eps,
    unsigned short* out) {
  constexpr int D = 128, KSTEPS = D / 16, DB = D / 32, HT = DFF / 32;
  constexpr int W1P = D * 2 + 16;            // W1^T row pitch: 16-byte reads of 32 consecutive rows hit all banks
  constexpr int OP = D * 2 + 16;             // output patch row pitch
  constexpr int ROWB = D * 2;
  __shared__ __attribute__((aligned(1024))) unsigned char W2L[DFF * ROWB];   // tiles of 32 rows, chunk c of row r at c ^ 4 (r & 3)
  __shared__ __attribute__((aligned(16))) unsigned char W1T[DFF * W1P];
  __shared__ __attribute__((aligned(16))) unsigned char patch[FM_WAVES * FM_ROWS * OP];
  __shared__ __attribute__((aligned(16))) float vecs[DFF + 3 * D];             // b1, b2, ln_g, ln_b
  __shared__ int rowok[FM_WAVES][FM_ROWS];

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- park the weights
  // W1 [D][DFF]: 16 bytes = 8 hidden units of one k. Consecutive threads take consecutive k, so that their 2-byte
  // writes into the transposed rows fall next to each other (with consecutive unit blocks per thread instead, the
  // writes of a wave are 8 rows apart and share two banks)
  for (int e = tid; e < D * DFF / 8; e += FM_THREADS) {
    const int kk = e % D, n0 = (e / D) * 8;
    const u32x4 raw = *reinterpret_cast<const u32x4*>(w1 + (size_t)kk * DFF + n0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned short val = (unsigned short)((raw[j >> 1] >> ((j & 1) * 16)) & 0xffffu);
      *reinterpret_cast<unsigned short*>(W1T + (n0 + j) * W1P + kk * 2) = val;
    }
  }
  for (int e = tid; e < DFF * (ROWB / 16); e += FM_THREADS) {    // W2 [DFF][D]: 16-byte chunks, swizzled inside each tile
    const int row = e / (ROWB / 16), c = e % (ROWB / 16);
    const u32x4 raw = *reinterpret_cast<const u32x4*>(w2 + (size_t)row * D + c * 8);
    *reinterpret_cast<u32x4*>(W2L + row * ROWB + ((c ^ (4 * (row & 3))) << 4)) = raw;
  }
  for (int e = tid; e < DFF + 3 * D; e += FM_THREADS)
    vecs[e] = e < DFF ? b1[e] : (e < DFF + D ? b2[e - DFF] : (e < DFF + 2 * D ? ln_g[e - DFF - D] : ln_b[e - DFF - 2 * D]));
  __syncthreads();
  const float* b1s = vecs;
  const float* b2s = vecs + DFF;
  const float* gs = vecs + DFF + D;
  const float* bs = vecs + DFF + 2 * D;

  // ---- per-lane constants
  const unsigned char* w1a = W1T + l32 * W1P + h * 16;            // + tile * 32 * W1P + ks * 32
  unsigned vofs[DB];                                              // as in the STA direct-to-LDS kernel (value tiles)
  {
    const int i16 = lane & 15;
    const int rr = h * 4 + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int c16 = db * 4 + 2 * (l32 >> 4) + ((i16 & 3) >> 1);
      vofs[db] = rr * ROWB + ((c16 ^ (4 * (rr & 3))) << 4) + (i16 & 1) * 8;
    }
  }
  bf16x8 idA[2];   // identity block for the residual product: row l32 of a 32 x 16 slice, k = 16 s + 8 h + e
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
    for (int e = 0; e < 8; ++e) idA[s2][e] = (l32 == 16 * s2 + 8 * h + e) ? (__bf16)1.0f : (__bf16)0.0f;
  unsigned char* opatch = patch + wave * FM_ROWS * OP;
  constexpr int LPR = D / 8, RPI = 64 / LPR;
  const unsigned char* opr = opatch + (lane / LPR) * OP + (lane % LPR) * 16;

  const long long ntiles = (rows + FM_ROWS - 1) / FM_ROWS;
  for (long long t = (long long)blockIdx.x * FM_WAVES + wave; t < ntiles; t += (long long)gridDim.x * FM_WAVES) {
    const long long r0 = t * FM_ROWS;
    // the wave's rows as the B operand (rows past the end repeat the last one; never stored)
    bf16x8 xreg[KSTEPS];
    {
      const long long r = (r0 + l32) < rows ? (r0 + l32) : (rows - 1);
      const unsigned short* xr = seg + (size_t)r * D + h * 8;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) xreg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xr + ks * 16));
    }
    if (lane < FM_ROWS) {   // which rows belong to a segment with a valid item
      const long long r = r0 + lane;
      int ok = 0;
      if (r < rows) {
        const int i = (int)(r % S);
        const int u = pair_user(cand_off, U, C, (int)(r / S));
        ok = (long long)i * w < valid_len(lens, u, L);
      }
      rowok[wave][lane] = ok;
    }
    f32x16 acc[DB];
    {
      // the biases enter as the initial value of the accumulators (the same LDS reads as adding them afterwards,
      // without the additions): b2 here, b1 below
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 bb = *reinterpret_cast<const f32x4*>(b2s + db * 32 + 8 * g + 4 * h);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[db][4 * g + e] = bb[e];
        }
#pragma unroll
      for (int db = 0; db < DB; ++db) {   // residual: Y^T = b2 + I . X^T
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(idA[0], xreg[2 * db], acc[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(idA[1], xreg[2 * db + 1], acc[db], 0, 0, 0);
      }
      // Operand reads run ahead of their use: the second layer's weights of a hidden tile are requested before its
      // first-layer products start, the first layer's weights of the next tile as soon as those products are
      // issued; the fences keep that placement (reads are only awaited where their registers are used).
      bf16x8 w1r[KSTEPS], w2r[2][DB];
      auto read_w1 = [&](int j) {
        const unsigned char* a1 = w1a + j * 32 * W1P;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) w1r[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(a1 + ks * 32));
      };
      read_w1(0);
#pragma unroll 1
      for (int j = 0; j < HT; ++j) {
        const unsigned char* a2 = W2L + j * 32 * ROWB;
        f32x16 hid;   // starts at b1: hidden unit of element r is 32 j + 8 (r >> 2) + 4 h + (r & 3)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 bb = *reinterpret_cast<const f32x4*>(b1s + j * 32 + 8 * g + 4 * h);
#pragma unroll
          for (int e = 0; e < 4; ++e) hid[4 * g + e] = bb[e];
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          w2r[0][db] = ffn_lds_tr(a2 + vofs[db]);
          w2r[1][db] = ffn_lds_tr(a2 + vofs[db] + 4096);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) hid = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1r[ks], xreg[ks], hid, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        read_w1(j + 1 < HT ? j + 1 : j);
        __builtin_amdgcn_sched_barrier(0);
        // relu, round
        u32x4 p0, p1;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float v4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v4[e] = fmaxf(hid[4 * g + e], 0.0f);
          const bf16x2 c0 = {(__bf16)v4[0], (__bf16)v4[1]}, c1 = {(__bf16)v4[2], (__bf16)v4[3]};
          if (g < 2) { p0[2 * g] = __builtin_bit_cast(unsigned, c0); p0[2 * g + 1] = __builtin_bit_cast(unsigned, c1); }
          else { p1[2 * (g - 2)] = __builtin_bit_cast(unsigned, c0); p1[2 * (g - 2) + 1] = __builtin_bit_cast(unsigned, c1); }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2r[0][db], __builtin_bit_cast(bf16x8, p0), acc[db], 0, 0, 0);
          acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2r[1][db], __builtin_bit_cast(bf16x8, p1), acc[db], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // ---- LayerNorm over d (this lane holds 64 of the row's 128 values, lane ^ 32 the others), gain, bias.
    // One pass for the sum and the sum of squares (values of order one, 128 terms, fp32: the cancellation in
    // E[x^2] - mean^2 costs ~1e-6), two multiply-adds per value for the normalisation.
    float sum = 0.0f, sq = 0.0f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float xv = acc[db][r];
        sum += xv;
        sq = fmaf(xv, xv, sq);
      }
    sum += __shfl_xor(sum, 32, 64);
    sq += __shfl_xor(sq, 32, 64);
    const float mean = sum * (1.0f / D);
    const float var = fmaxf(sq * (1.0f / D) - mean * mean, 0.0f);
    const float rstd = 1.0f / sqrtf(var + eps);
    const float nmr = -mean * rstd;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 gg = *reinterpret_cast<const f32x4*>(gs + db * 32 + 8 * g + 4 * h);
        const f32x4 bb = *reinterpret_cast<const f32x4*>(bs + db * 32 + 8 * g + 4 * h);
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (__bf16)fmaf(fmaf(acc[db][4 * g + e], rstd, nmr), gg[e], bb[e]);
        *reinterpret_cast<u32x2*>(opatch + l32 * OP + (db * 32 + g * 8 + h * 4) * 2) = __builtin_bit_cast(u32x2, o);
      }
    // ---- rows leave as whole 256-byte rows (LDS operations of a wave execute in order: no barrier needed)
#pragma unroll
    for (int b = 0; b < FM_ROWS / RPI; ++b) {
      const int rr = b * RPI + lane / LPR;
      u32x4 val = *reinterpret_cast<const u32x4*>(opr + b * RPI * OP);
      if (!rowok[wave][rr]) val = u32x4{0u, 0u, 0u, 0u};
      if (r0 + rr < rows) *reinterpret_cast<u32x4*>(out + (size_t)(r0 + rr) * D + (lane % LPR) * 8) = val;
    }
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
