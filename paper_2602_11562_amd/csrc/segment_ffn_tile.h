// The matrix-core tile of the segment FFN + LayerNorm step (paper Sec. 3.4.2, s <- LN(FFN(s) + s)), shared by the
// stand-alone kernel (segment_ffn.hip) and the kernel that feeds the result straight into the GSTA layer
// (ffn_gsta.hip). bf16 storage, d = 128, d_ff a multiple of 32, at most 128.
//
// Same operand scheme as the STA kernels (sta_mfma.hip), with the first-layer weights in the place of the keys and
// the second-layer weights in the place of the values. A wave owns 32 rows of H' at a time (its B operand, read
// once into registers) and walks the hidden layer in tiles of 32 units:
//   hid^T [32 units x 32 rows] = W1^T tile . X^T      (v_mfma_f32_32x32x16_bf16)
//   + b1, relu, rounded to bf16: the accumulator layout is, per 16 units, a valid B operand of
//   Y^T [d x 32 rows] += W2 tile^T . hid
// Both weight matrices are stored with the contraction index as their row (W1 [d][d_ff], W2 [d_ff][d]), so both A
// operands come from ds_read_b64_tr_b16 on the rows as stored. The residual enters as one more product, identity x
// X^T (exact), so that it needs no other copy of X. Then b2 and LayerNorm (a row's d values sit in one lane pair:
// a sum per lane and one exchange).
//
// Everything reaches LDS by global_load_lds_dwordx4 (each lane names a 16-byte global chunk, the 64 chunks of a wave
// land contiguously): no register or VALU work is spent on staging, and a wave's next 32 rows are in flight while
// it multiplies the current ones. Rows are unpadded (256 bytes); bank conflicts are avoided by an XOR swizzle of the
// 16-byte chunk index that the fetching lane applies when it picks its global chunk:
//   weights   chunk c of row r at position c ^ 4 (r & 3)   (conflict-free for the 4-rows-by-64-bytes transpose loads)
//   H' rows   chunk c of row r at position c ^ (r & 15)    (conflict-free for the 16-rows-by-16-bytes operand reads)
// The transpose load hands a lane the contraction indices {4 h .. 4 h + 3, 8 + 4 h .. 8 + 4 h + 3} of a 16-row group
// where the operand read of the H' rows hands it 8 h .. 8 h + 7: W1's rows are parked in the matching order (row
// 8 h + 4 g + j of a group at position 8 g + 4 h + j). The fetches are inline assembly the compiler's wait-count
// pass does not see; their completion is awaited explicitly (s_waitcnt vmcnt(0)).
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
constexpr int FM_OP = FM_D * 2 + 16;    // output patch row pitch
constexpr int FM_ROWB = FM_D * 2;       // bytes per parked row (W1 rows are padded to it when d_ff < 128)
constexpr int FM_W1B = FM_D * FM_ROWB;  // W1 in LDS
// A wave's patch: the landing area of its next 32 rows (8 KB, unpadded, swizzled) and, once those are in registers,
// the normalised rows on their way out (pitch FM_OP). 1 KB-aligned like every fetch destination.
constexpr int FM_PATCH = ((FM_ROWS * FM_OP + 1023) / 1024) * 1024;

// 16 bytes per lane from global (uniform base + per-lane byte offset) to LDS (uniform address + 16 * lane)
__device__ __forceinline__ void ffn_dma16(const void* gbase, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(lds_addr), "v"(voff), "s"(gbase)
               : "memory");
}
// every fetch of this wave has landed (and every store it issued has left)
__device__ __forceinline__ void ffn_wait_fetches() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ unsigned ffn_lds_addr(const void* p) {
  return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// Request the 32 rows of 256 bytes that start at `rows0` (a uniform pointer to row 0 of the tile) into the landing
// area at LDS address `land`; rows past `last` (>= 0, uniform) repeat row `last`.
__device__ __forceinline__ void ffn_fetch_rows(const unsigned short* rows0, int last, unsigned land, int lane) {
  // (the offsets are worked out here, from a lane number the compiler cannot tell from a fresh value: computed once
  // per loop and kept, they are spilled, and every reload waits for the fetch before it)
  asm volatile("" : "+v"(lane));
  const int q = lane >> 4, pos = lane & 15;
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own reads of the landing area have been served
#pragma unroll
  for (int j = 0; j < FM_ROWS / 4; ++j) {
    const int row = 4 * j + q;
    const int src = row < last ? row : last;
    ffn_dma16(rows0, (unsigned)(src * FM_ROWB + ((pos ^ (row & 15)) << 4)), land + j * 1024);
  }
}

// The wave's 32 rows from the landing area as the B operand of the first product: lane (l32, h) holds components
// 16 ks + 8 h .. + 7 of row l32.
__device__ __forceinline__ void ffn_read_rows(const unsigned char* land, int l32, int h, bf16x8 (&xreg)[FM_D / 16]) {
  const unsigned char* row = land + l32 * FM_ROWB;
#pragma unroll
  for (int ks = 0; ks < FM_D / 16; ++ks)
    xreg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(row + (((2 * ks + h) ^ (l32 & 15)) << 4)));
}

// The compiler folds "lane offset + tile offset + constant" into one three-operand add per read; hiding the sum of
// the first two behind an empty asm leaves "register + constant", which becomes the read's immediate offset.
__device__ __forceinline__ const unsigned char* ffn_opaque(const unsigned char* p) {
  unsigned a = ffn_lds_addr(p);
  asm volatile("" : "+v"(a));
  return (const unsigned char*)(__attribute__((address_space(3))) const unsigned char*)(size_t)a;
}

__device__ __forceinline__ bf16x8 ffn_lds_tr(const unsigned char* p) {   // see lds_read_tr in sta_mfma.hip
  typedef __attribute__((address_space(3))) s16x4* lds4;
  const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4)(size_t)(unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p);
  const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4)(size_t)(unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)(p + 2048));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Park the weights for the life of the workgroup: W1 [D][DFF] (rows in the order the transpose load wants, see the
// file header; padded to 256-byte rows) and W2 [DFF][D], both with chunk c of row r at position c ^ 4 (r & 3), and
// b1, b2, ln_g, ln_b behind one another in vecs. The caller awaits the fetches and puts a barrier behind them.
template <int DFF>
__device__ __forceinline__ void ffn_park_weights(unsigned w1l, unsigned w2l, float* vecs,
                                                 const unsigned short* __restrict__ w1,
                                                 const unsigned short* __restrict__ w2, const float* __restrict__ b1,
                                                 const float* __restrict__ b2, const float* __restrict__ ln_g,
                                                 const float* __restrict__ ln_b, int tid) {
  constexpr int D = FM_D;
  static_assert(DFF % 32 == 0 && DFF <= 128, "hidden tiles of 32 units, rows of at most 256 bytes");
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int q = lane >> 4, pos = lane & 15;
  const int c = pos ^ (4 * q);                        // the chunk this lane fetches: rows 4 g + q, and (4 g + q) & 3 = q
#pragma unroll
  for (int it = 0; it < D / 4 / FM_WAVES; ++it) {     // W1: groups of four rows
    const int g = it * FM_WAVES + wave;
    const int row = 4 * g + q;                        // position; holds row 8 h + 4 g2 + j of its 16-row group
    const int src = (row & ~15) + 8 * ((row >> 2) & 1) + 4 * ((row >> 3) & 1) + (row & 3);
    ffn_dma16(w1, (unsigned)(src * (DFF * 2) + ((c & (DFF / 8 - 1)) << 4)), w1l + g * 1024);   // (chunks past the row: never read)
  }
#pragma unroll
  for (int it = 0; it < (DFF / 4 + FM_WAVES - 1) / FM_WAVES; ++it) {   // W2
    const int g = it * FM_WAVES + wave;
    if (g < DFF / 4) ffn_dma16(w2, (unsigned)((4 * g + q) * FM_ROWB + (c << 4)), w2l + g * 1024);
  }
  for (int e = tid; e < DFF + 3 * D; e += FM_THREADS)
    vecs[e] = e < DFF ? b1[e] : (e < DFF + D ? b2[e - DFF] : (e < DFF + 2 * D ? ln_g[e - DFF - D] : ln_b[e - DFF - 2 * D]));
}

// Per-lane constants of the transpose loads (as in the STA direct-to-LDS kernel's value tiles): the lane addresses
// row rr = 4 h + (lane & 15) / 4 of a 16-row group, and of column block db the 8 bytes at chunk
// c = 4 db + 2 (l32 / 16) + ((lane & 3) / 2), half (lane & 1), which sits at position c ^ 4 (rr & 3), i.e. block
// db ^ (rr & 3) of the row with the rest of c unchanged.
struct FfnLane {
  unsigned vbase;   // byte offset for block 0 before the swizzle
  unsigned q;       // rr & 3
  __device__ __forceinline__ void init(int lane) {
    const int l32 = lane & 31, h = lane >> 5;
    const int i16 = lane & 15;
    const int rr = h * 4 + (i16 >> 2);
    q = rr & 3;
    vbase = rr * FM_ROWB + ((2 * (l32 >> 4) + ((i16 & 3) >> 1)) << 4) + (i16 & 1) * 8;
  }
  __device__ __forceinline__ unsigned vofs(int db) const { return vbase + (((unsigned)db ^ q) << 6); }
};

// y^T = b2 + X^T + W2^T relu(W1^T X^T + b1) for the wave's 32 rows: acc[db][r] of lane (l32, h) is component
// 32 db + 8 (r / 4) + 4 h + r % 4 of row l32.
template <int DFF>
__device__ __forceinline__ void ffn_tile_products(const bf16x8 (&xreg)[FM_D / 16], const FfnLane& ln,
                                                  const unsigned char* W1L, const unsigned char* W2L,
                                                  const float* b1s, const float* b2s, int lane32, int h,
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
  {   // residual: Y^T = b2 + I . X^T. The identity block (row l32 of a 32 x 16 slice, k = 16 s + 8 h + e) is built
      // here, from a lane number the compiler cannot tell from a fresh value: kept across the tile loop it would
      // cost eight registers that the products need
    int l32 = lane32;
    asm volatile("" : "+v"(l32));
    u32x4 id[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const int e0 = l32 - 16 * s2 - 8 * h;   // the slot of this lane's one, if it has one in this slice
      const unsigned one = (e0 & 1) ? 0x3f800000u : 0x3f80u;
      const int word = e0 >> 1;               // (negative or >= 4: none)
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) id[s2][e2] = word == e2 ? one : 0u;
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, id[0]), xreg[2 * db], acc[db], 0, 0, 0);
      acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, id[1]), xreg[2 * db + 1], acc[db], 0, 0, 0);
    }
  }
  // Operand reads run ahead of their use: the second layer's weights of a hidden tile are requested before its
  // first-layer products start, the first layer's weights of the next tile between the two halves of the second
  // product; the fences keep that placement (reads are only awaited where their registers are used).
  bf16x8 w1r[KSTEPS], w2r[2][DB];
  auto read_w1 = [&](int j) {   // units 32 j .. 32 j + 31: column block j of W1's rows, 16 rows per k-step
    const unsigned char* a1 = ffn_opaque(W1L + ln.vofs(j));
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) w1r[ks] = ffn_lds_tr(a1 + ks * 16 * FM_ROWB);
  };
  read_w1(0);
#pragma unroll 1
  for (int j = 0; j < HT; ++j) {
    const unsigned char* a2 = ffn_opaque(W2L + j * 32 * FM_ROWB + ln.vbase);
    f32x16 hid;   // starts at b1: hidden unit of element r is 32 j + 8 (r >> 2) + 4 h + (r & 3)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 bb = *reinterpret_cast<const f32x4*>(b1s + j * 32 + 8 * g + 4 * h);
#pragma unroll
      for (int e = 0; e < 4; ++e) hid[4 * g + e] = bb[e];
    }
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      // block db ^ q: with q < 4 known only at run time the four blocks are visited in the lane's own order, and
      // the offset is a select between constants
      const unsigned blk = ((unsigned)db ^ ln.q) << 6;
      w2r[0][db] = ffn_lds_tr(a2 + blk);
      w2r[1][db] = ffn_lds_tr(a2 + blk + 4096);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) hid = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1r[ks], xreg[ks], hid, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    // relu, round
    u32x4 p0, p1;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float v4[4];   // relu as a signed-integer maximum with 0: negative values (sign bit set) become +0 in one instruction
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int b = __float_as_int(hid[4 * g + e]);
        v4[e] = __int_as_float(b > 0 ? b : 0);
      }
      const bf16x2 c0 = {(__bf16)v4[0], (__bf16)v4[1]}, c1 = {(__bf16)v4[2], (__bf16)v4[3]};
      if (g < 2) { p0[2 * g] = __builtin_bit_cast(unsigned, c0); p0[2 * g + 1] = __builtin_bit_cast(unsigned, c1); }
      else { p1[2 * (g - 2)] = __builtin_bit_cast(unsigned, c0); p1[2 * (g - 2) + 1] = __builtin_bit_cast(unsigned, c1); }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2r[0][db], __builtin_bit_cast(bf16x8, p0), acc[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_w1(j + 1 < HT ? j + 1 : j);   // into the registers the first half of W2's tile has just left
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2r[1][db], __builtin_bit_cast(bf16x8, p1), acc[db], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// x + the value of lane ^ 32 (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float ffn_both_halves_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Maximum over the 16 lanes of a row, in every lane of the row (lane permutations as in row_sum, laser_internal.h)
__device__ __forceinline__ float ffn_row_max(float v) {
#define LASER_DPP_MAX(ctrl) \
  v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, false)))
  LASER_DPP_MAX(0xB1);    // quad_perm [1,0,3,2]
  LASER_DPP_MAX(0x4E);    // quad_perm [2,3,0,1]
  LASER_DPP_MAX(0x141);   // row_half_mirror
  LASER_DPP_MAX(0x140);   // row_mirror
#undef LASER_DPP_MAX
  return v;
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
  sum = ffn_both_halves_sum(sum);
  sq = ffn_both_halves_sum(sq);
  const float mean = sum * (1.0f / FM_D);
  const float var = fmaxf(sq * (1.0f / FM_D) - mean * mean, 0.0f);
  rstd = 1.0f / sqrtf(var + eps);
  nmr = -mean * rstd;
}

}  // namespace laser
