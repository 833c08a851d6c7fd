// The matrix-core tile of the segment FFN + LayerNorm step (paper Sec. 3.4.2, s <- LN(FFN(s) + s)), shared by the
// stand-alone kernel (segment_ffn.hip) and the kernel that feeds the result straight into the GSTA layer
// (ffn_gsta.hip). bf16 storage, d = 128, d_ff a multiple of 32.
//
// Same operand scheme as the STA kernels (sta_mfma.hip), with the first-layer weights in the place of the keys and
// the second-layer weights in the place of the values. A wave owns 32 rows of H' at a time (its B operand, read
// once into registers) and walks the hidden layer in tiles of 32 units:
//   hid^T [32 units x 32 rows] = W1^T tile . X^T      (v_mfma_f32_32x32x16_bf16, A from LDS 16 bytes per lane)
//   + b1, relu, rounded to bf16: the accumulator layout is, per 16 units, a valid B operand of
//   Y^T [d x 32 rows] += W2 tile^T . hid             (A fetched by ds_read_b64_tr_b16 from W2 rows as stored)
// The residual enters as one more product, identity x X^T (exact), so that it needs no other copy of X. Then b2 and
// LayerNorm (a row's d values sit in one lane pair: a sum per lane and one exchange).
#pragma once

#include "laser_internal.h"

namespace laser {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int FM_WAVES = 8, FM_THREADS = 64 * FM_WAVES, FM_ROWS = 32;
constexpr int FM_D = 128;
constexpr int FM_W1P = FM_D * 2 + 16;   // W1^T row pitch: 16-byte reads of 32 consecutive rows hit all banks
constexpr int FM_OP = FM_D * 2 + 16;    // output patch row pitch
constexpr int FM_ROWB = FM_D * 2;

__device__ __forceinline__ bf16x8 ffn_lds_tr(const unsigned char* p) {   // see lds_read_tr in sta_mfma.hip
  typedef __attribute__((address_space(3))) s16x4* lds4;
  const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4)(size_t)(unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p);
  const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4)(size_t)(unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)(p + 2048));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Park the weights for the life of the workgroup: W1 [D][DFF] transposed into W1T (rows of pitch FM_W1P), W2 [DFF][D]
// in tiles of 32 rows with chunk c of row r at c ^ 4 (r & 3), and b1, b2, ln_g, ln_b behind one another in vecs.
// The caller puts a barrier behind it.
template <int DFF>
__device__ __forceinline__ void ffn_park_weights(unsigned char* W1T, unsigned char* W2L, float* vecs,
                                                 const unsigned short* __restrict__ w1,
                                                 const unsigned short* __restrict__ w2, const float* __restrict__ b1,
                                                 const float* __restrict__ b2, const float* __restrict__ ln_g,
                                                 const float* __restrict__ ln_b, int tid) {
  constexpr int D = FM_D;
  // W1: 16 bytes = 8 hidden units of one k. Consecutive threads take consecutive k, so that their 2-byte writes into
  // the transposed rows fall next to each other (with consecutive unit blocks per thread instead, the writes of a
  // wave are 8 rows apart and share two banks)
  for (int e = tid; e < D * DFF / 8; e += FM_THREADS) {
    const int kk = e % D, n0 = (e / D) * 8;
    const u32x4 raw = *reinterpret_cast<const u32x4*>(w1 + (size_t)kk * DFF + n0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned short val = (unsigned short)((raw[j >> 1] >> ((j & 1) * 16)) & 0xffffu);
      *reinterpret_cast<unsigned short*>(W1T + (n0 + j) * FM_W1P + kk * 2) = val;
    }
  }
  for (int e = tid; e < DFF * (FM_ROWB / 16); e += FM_THREADS) {    // W2: 16-byte chunks, swizzled inside each tile
    const int row = e / (FM_ROWB / 16), c = e % (FM_ROWB / 16);
    const u32x4 raw = *reinterpret_cast<const u32x4*>(w2 + (size_t)row * D + c * 8);
    *reinterpret_cast<u32x4*>(W2L + row * FM_ROWB + ((c ^ (4 * (row & 3))) << 4)) = raw;
  }
  for (int e = tid; e < DFF + 3 * D; e += FM_THREADS)
    vecs[e] = e < DFF ? b1[e] : (e < DFF + D ? b2[e - DFF] : (e < DFF + 2 * D ? ln_g[e - DFF - D] : ln_b[e - DFF - 2 * D]));
}

// Per-lane constants of the tile: where the lane reads W1^T and W2 from, and its piece of the identity.
struct FfnLane {
  const unsigned char* w1a;   // + tile * 32 * FM_W1P + ks * 32
  unsigned vofs[FM_D / 32];   // as in the STA direct-to-LDS kernel (value tiles)
  bf16x8 idA[2];              // identity block for the residual product: row l32 of a 32 x 16 slice, k = 16 s + 8 h + e
  __device__ __forceinline__ void init(const unsigned char* W1T, int lane) {
    const int l32 = lane & 31, h = lane >> 5;
    w1a = W1T + l32 * FM_W1P + h * 16;
    const int i16 = lane & 15;
    const int rr = h * 4 + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < FM_D / 32; ++db) {
      const int c16 = db * 4 + 2 * (l32 >> 4) + ((i16 & 3) >> 1);
      vofs[db] = rr * FM_ROWB + ((c16 ^ (4 * (rr & 3))) << 4) + (i16 & 1) * 8;
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int e = 0; e < 8; ++e) idA[s2][e] = (l32 == 16 * s2 + 8 * h + e) ? (__bf16)1.0f : (__bf16)0.0f;
  }
};

// y^T = b2 + X^T + W2^T relu(W1^T X^T + b1) for the wave's 32 rows: acc[db][r] of lane (l32, h) is component
// 32 db + 8 (r / 4) + 4 h + r % 4 of row l32.
template <int DFF>
__device__ __forceinline__ void ffn_tile_products(const bf16x8 (&xreg)[FM_D / 16], const FfnLane& ln,
                                                  const unsigned char* W2L, const float* b1s, const float* b2s, int h,
                                                  f32x16 (&acc)[FM_D / 32]) {
  constexpr int KSTEPS = FM_D / 16, DB = FM_D / 32, HT = DFF / 32;
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
    acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ln.idA[0], xreg[2 * db], acc[db], 0, 0, 0);
    acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ln.idA[1], xreg[2 * db + 1], acc[db], 0, 0, 0);
  }
  // Operand reads run ahead of their use: the second layer's weights of a hidden tile are requested before its
  // first-layer products start, the first layer's weights of the next tile as soon as those products are
  // issued; the fences keep that placement (reads are only awaited where their registers are used).
  bf16x8 w1r[KSTEPS], w2r[2][DB];
  auto read_w1 = [&](int j) {
    const unsigned char* a1 = ln.w1a + j * 32 * FM_W1P;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) w1r[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(a1 + ks * 32));
  };
  read_w1(0);
#pragma unroll 1
  for (int j = 0; j < HT; ++j) {
    const unsigned char* a2 = W2L + j * 32 * FM_ROWB;
    f32x16 hid;   // starts at b1: hidden unit of element r is 32 j + 8 (r >> 2) + 4 h + (r & 3)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 bb = *reinterpret_cast<const f32x4*>(b1s + j * 32 + 8 * g + 4 * h);
#pragma unroll
      for (int e = 0; e < 4; ++e) hid[4 * g + e] = bb[e];
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      w2r[0][db] = ffn_lds_tr(a2 + ln.vofs[db]);
      w2r[1][db] = ffn_lds_tr(a2 + ln.vofs[db] + 4096);
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

// LayerNorm statistics of the wave's rows from the accumulator layout (this lane holds 64 of its row's 128 values,
// lane ^ 32 the others): normalised value = x * rstd + nmr. One pass for the sum and the sum of squares (values of
// order one, 128 terms, fp32: the cancellation in E[x^2] - mean^2 costs ~1e-6).
__device__ __forceinline__ void ffn_row_stats(const f32x16 (&acc)[FM_D / 32], float eps, float& rstd, float& nmr) {
  float sum = 0.0f, sq = 0.0f;
#pragma unroll
  for (int db = 0; db < FM_D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float xv = acc[db][r];
      sum += xv;
      sq = fmaf(xv, xv, sq);
    }
  sum += __shfl_xor(sum, 32, 64);
  sq += __shfl_xor(sq, 32, 64);
  const float mean = sum * (1.0f / FM_D);
  const float var = fmaxf(sq * (1.0f / FM_D) - mean * mean, 0.0f);
  rstd = 1.0f / sqrtf(var + eps);
  nmr = -mean * rstd;
}

}  // namespace laser
