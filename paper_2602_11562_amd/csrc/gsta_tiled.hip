// GSTA for bf16 storage: a tile of 32 (user, candidate) pairs per workgroup.
//
// Per layer (Sec. 3.4.3): a = softmax((t W_q)(H' W_k)^T / sqrt(d)), o = a (H' W_v), t += o, with the two
// products with H' re-associated (exact up to rounding): scores = H' (W_k (t W_q)^T), o = (a H') W_v.
//
//   step 1  q' = T W_q            [32 x d].[d x d]   bf16 MFMA, one 32-column block per wave
//   step 2  r  = q' W_k^T / sqrt(d)                   bf16 MFMA
//   step 3  per pair: e_i = H'_i . r, softmax over the valid segments, p = sum_i a_i H'_i
//           one wave per pair at a time; the pair's whole S x d block of H' is read from HBM ONCE into
//           registers (16 B per lane, rows spread over lane groups) and used for both passes
//   step 4  o = p W_v, t += o     bf16 MFMA
//
// fp32 operands of the MFMA steps (t, q', p) are split into a bf16 head and a bf16 remainder and multiplied
// in two passes, so the products carry ~16 significant bits; weights and H' are bf16 by storage. The running
// target t stays in fp32 registers in accumulator layout. W_q and W_v (contraction index = row index, the slow
// one in memory) are staged in LDS with coalesced loads and read with the LDS transpose load; W_k is read in
// operand order straight from global memory (L2 resident). Two fp32 [32 x d] LDS buffers carry the operands
// between steps. The H' block of a wave's next pair is requested before the current pair is reduced, and the
// first one before the projection steps, so the HBM stream runs behind the arithmetic.
#include <cstdlib>

#include "laser_internal.h"

namespace laser {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int GT_ROWS = 32;     // MFMA row block; a workgroup owns PT <= 32 pairs, the other rows are padding
constexpr int GT_WAVES = 8;     // waves per workgroup: all of them stream H', the first d/32 also run the MFMA steps
constexpr int GT_THREADS = 64 * GT_WAVES;

struct HiLo {
  bf16x8 hi, lo;
};

// 8 consecutive fp32 values of one LDS row -> bf16 head and remainder
__device__ __forceinline__ HiLo split8(const float* p) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
  HiLo o;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o.hi[i] = (__bf16)a[i];
    o.lo[i] = (__bf16)(a[i] - (float)o.hi[i]);
    o.hi[4 + i] = (__bf16)b[i];
    o.lo[4 + i] = (__bf16)(b[i] - (float)o.hi[4 + i]);
  }
  return o;
}

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

template <int D> struct WPitch { static constexpr int v = (D * 2) % 256 == 64 ? D * 2 : D * 2 + 64; };

// B operand of X.W^T: lane n needs W[n][k] for 8 consecutive k: one 16-byte load per k-step
template <int D>
__device__ __forceinline__ void load_b_rows(const unsigned short* __restrict__ W, int nb, int l32, int h,
                                            bf16x8 (&b)[D / 16]) {
  const int n = nb * 32 + l32;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks)
    b[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(W + (size_t)n * D + ks * 16 + h * 8));
}

// [32 x D] (LDS, fp32, pitch FP) times W^T with W bf16 [D][D] -> a 32 x 32 block: out[p][n] = sum_k X[p][k] W[n][k],
// with the B operands (k contiguous per lane: one 16-byte load per step, load_b_rows) already in registers,
// requested early by the caller
template <int D>
__device__ __forceinline__ f32x16 tile_gemm_breg(const float* X, int FP, const bf16x8 (&b)[D / 16], int l32, int h) {
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    const HiLo a = split8(X + l32 * FP + ks * 16 + h * 8);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b[ks], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b[ks], acc, 0, 0, 0);
  }
  return acc;
}

// [32 x D] (LDS, fp32, pitch FP) times W with W bf16 [D][D] staged row-major in LDS (pitch WPitch) ->
// 32 x 32 block `nb`: out[p][n] = sum_k X[p][k] W[k][n]. The B operand wants k contiguous per lane, i.e. a
// column of W: fetched with the LDS transpose load (lane i of a 16-lane group supplies the address of
// W[k0 + i/4][n0 + 4 (i%4)] and receives W[k0 .. k0+3][n0 + i]).
template <int D>
__device__ __forceinline__ f32x16 tile_gemm_lds(const float* X, int FP, const unsigned char* Wl, int nb, int lane,
                                                int l32, int h) {
  constexpr int WP = WPitch<D>::v;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  const int i16 = lane & 15;
  const unsigned char* base = Wl + (h * 8 + (i16 >> 2)) * WP + (nb * 32 + (l32 & 16) + 4 * (i16 & 3)) * 2;
#pragma unroll 2
  for (int ks = 0; ks < D / 16; ++ks) {
    const unsigned char* src = base + ks * 16 * WP;
    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 4 * WP));
    const bf16x8 b = __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
    const HiLo a = split8(X + l32 * FP + ks * 16 + h * 8);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b, acc, 0, 0, 0);
  }
  return acc;
}

// W [D][D] bf16: global -> registers (coalesced 16-byte chunks) and registers -> LDS, split so that the loads can
// be in flight across other work
template <int D>
struct WStage {
  static constexpr int IT = (D * (D / 8) + GT_THREADS - 1) / GT_THREADS;
  static constexpr bool EXACT = (D * (D / 8)) % GT_THREADS == 0;
  u32x4 r[IT];
  __device__ __forceinline__ void load(const unsigned short* __restrict__ W, int tid) {
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      int e = tid + it * GT_THREADS;
      if (!EXACT) e = e < D * (D / 8) ? e : D * (D / 8) - 1;
      r[it] = *reinterpret_cast<const u32x4*>(W + (size_t)e * 8);
    }
  }
  __device__ __forceinline__ void store(unsigned char* Wl, int tid) const {
    constexpr int WP = WPitch<D>::v, CH = D / 8;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int e = tid + it * GT_THREADS, row = e / CH, ch = e % CH;
      if (EXACT || e < D * CH) *reinterpret_cast<u32x4*>(Wl + row * WP + ch * 16) = r[it];
    }
  }
};

// accumulator layout: lane = column nb*32 + l32, register r = row 8 (r/4) + 4 h + r % 4
__device__ __forceinline__ void store_acc(float* X, int FP, const f32x16& acc, int nb, int l32, int h, float scale) {
#pragma unroll
  for (int r = 0; r < 16; ++r) X[(8 * (r >> 2) + 4 * h + (r & 3)) * FP + nb * 32 + l32] = acc[r] * scale;
}

template <int D, int ROWS, int PT>
__global__ __launch_bounds__(GT_THREADS) void gsta_tiled_kernel(const unsigned short* __restrict__ seg,
                                                         const unsigned short* __restrict__ t0,
                                                         const unsigned short* __restrict__ wq,
                                                         const unsigned short* __restrict__ wk,
                                                         const unsigned short* __restrict__ wv,
                                                         const int32_t* __restrict__ lens, const int32_t* __restrict__ cand_off, int U, int P, int C, int L, int w,
                                                         int S, int M, float* __restrict__ z) {
  constexpr int FP = D + 4;          // fp32 row pitch: 16 B mod 256 B, conflict-free 16-byte row reads
  constexpr int DB = D / 32;         // 32-column blocks; waves >= DB idle in the MFMA steps
  constexpr int LPR = D / 8;         // lanes per H' row (16 B each)
  constexpr int RPW = 64 / LPR;      // rows per wave-wide load
  constexpr int WP = WPitch<D>::v;
  constexpr int PPW = PT / GT_WAVES;  // pairs per wave in step 3
  __shared__ __attribute__((aligned(16))) float bufA[GT_ROWS * FP];
  __shared__ __attribute__((aligned(16))) float bufB[GT_ROWS * FP];
  __shared__ __attribute__((aligned(16))) unsigned char Wl[D * WP];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: the valid lengths become scalar loads
  const int l32 = lane & 31, h = lane >> 5;
  const int pbase = blockIdx.x * PT;
  const float scale = 1.0f / sqrtf((float)D);
  const int grp = lane / LPR, gl = lane % LPR;   // row group and position inside the row

  WStage<D> ws;
  ws.load(wq, tid);
  // W_k of the layer as the B operand of step 2, straight from memory in operand order and a layer ahead: requested
  // inside the product it put a round trip to L2 into every layer's chain
  bf16x8 bk[D / 16];
  if (wave < DB) load_b_rows<D>(wk, wave, l32, h, bk);

  // valid segments of the wave's pairs (independent loads, one round trip)
  int nvs[PPW];
#pragma unroll
  for (int it = 0; it < PPW; ++it) {
    const int pr = pbase + wave + it * GT_WAVES;
    nvs[it] = 0;
    if (pr < P) nvs[it] = (valid_len(lens, pair_user(cand_off, U, C, pr), L) + w - 1) / w;
  }
  // H' block of one pair: rows j*RPW + grp, 16 bytes per lane; rows of invalid segments are not read.
  // DEPTH blocks are kept in flight per wave (a ring of register sets).
  constexpr int DEPTH_WANT = ROWS <= 4 ? 4 : 2;
  constexpr int DEPTH = DEPTH_WANT < PPW ? DEPTH_WANT : PPW;   // H' blocks in flight per wave (register sets)
  u32x4 hring[DEPTH][ROWS];
  auto load_pair = [&](int pi, int nv, u32x4 (&hreg)[ROWS]) {
    const unsigned short* H = seg + (size_t)(pbase + pi) * S * D;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const int i = j * RPW + grp;
      hreg[j] = u32x4{0u, 0u, 0u, 0u};
      if (i < nv) hreg[j] = *reinterpret_cast<const u32x4*>(H + (size_t)i * D + gl * 8);
    }
  };
#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd) load_pair(wave + dd * GT_WAVES, nvs[dd], hring[dd]);   // in flight during steps 1-2

  // running target t in accumulator layout (wave = column block)
  f32x16 ts;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = 8 * (r >> 2) + 4 * h + (r & 3);
    const int pr = pbase + row;
    ts[r] = (wave < DB && row < PT && pr < P) ? bf16_bits_to_f32(t0[(size_t)pr * D + wave * 32 + l32]) : 0.0f;
  }

  for (int layer = 0; layer < M; ++layer) {
    const unsigned short* Wv = wv + (size_t)layer * D * D;

    ws.store(Wl, tid);                                 // W_q of this layer
    if (wave < DB) store_acc(bufA, FP, ts, wave, l32, h, 1.0f);
    __syncthreads();
    if (wave < DB) {                                   // step 1: q' = t W_q
      const f32x16 qp = tile_gemm_lds<D>(bufA, FP, Wl, wave, lane, l32, h);
      store_acc(bufB, FP, qp, wave, l32, h, 1.0f);
    }
    __syncthreads();
    ws.load(Wv, tid);                                  // W_v: in flight during step 2, W_q is no longer needed
    if (wave < DB) {                                   // step 2: r = q' W_k^T / sqrt(d)
      const f32x16 rr = tile_gemm_breg<D>(bufB, FP, bk, l32, h);
      store_acc(bufA, FP, rr, wave, l32, h, scale);
      if (layer + 1 < M) load_b_rows<D>(wk + (size_t)(layer + 1) * D * D, wave, l32, h, bk);
    }
    ws.store(Wl, tid);
    __syncthreads();

    // step 3: one pair per wave at a time; its H' block goes through registers once
    // (H' is the same in every layer, Sec. 3.4.3: when the ring holds all of the wave's blocks they stay where they
    // are; otherwise the first ones are requested again, from the caches)
    if (layer > 0 && PPW > DEPTH) {
#pragma unroll
      for (int dd = 0; dd < DEPTH; ++dd) load_pair(wave + dd * GT_WAVES, nvs[dd], hring[dd]);
    }
    auto reduce_pair = [&](int pi, int nv, u32x4 (&hcur)[ROWS], int refill_pi, int refill_nv) {
      float rs[8];
      {
        const f32x4 a = *reinterpret_cast<const f32x4*>(bufA + pi * FP + gl * 8);
        const f32x4 b = *reinterpret_cast<const f32x4*>(bufA + pi * FP + gl * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { rs[e] = a[e]; rs[4 + e] = b[e]; }
      }
      // one pass with a running maximum (per lane group, merged across groups afterwards): each row's values
      // are converted once and used for both the score and the weighted sum
      float m = -INFINITY, den = 0.0f;
      float pacc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pacc[e] = 0.0f;
#pragma unroll
      for (int j = 0; j < ROWS; ++j) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          x[2 * e] = __uint_as_float(hcur[j][e] << 16);
          x[2 * e + 1] = __uint_as_float(hcur[j][e] & 0xffff0000u);
        }
        float sdot = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sdot = fmaf(x[e], rs[e], sdot);
        sdot = row_sum<LPR>(sdot);
        const bool ok = (j * RPW + grp) < nv;
        const float m_new = ok ? fmaxf(m, sdot) : m;
        const float sc = (m == m_new) ? 1.0f : __expf(m - m_new);
        const float a = ok ? __expf(sdot - m_new) : 0.0f;
        den = fmaf(den, sc, a);
#pragma unroll
        for (int e = 0; e < 8; ++e) pacc[e] = fmaf(pacc[e], sc, a * x[e]);
        m = m_new;
      }
      if (refill_pi >= 0) load_pair(refill_pi, refill_nv, hcur);   // refill the slot: next block in flight
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) {
        const float m_o = __shfl_xor(m, off, 64);
        const float den_o = __shfl_xor(den, off, 64);
        const float M2 = fmaxf(m, m_o);
        const float f = (m == M2) ? 1.0f : __expf(m - M2);
        const float f_o = (m_o == M2) ? 1.0f : __expf(m_o - M2);
        den = den * f + den_o * f_o;
#pragma unroll
        for (int e = 0; e < 8; ++e) pacc[e] = pacc[e] * f + __shfl_xor(pacc[e], off, 64) * f_o;
        m = M2;
      }
      if (grp == 0) {
        const float inv = nv > 0 ? 1.0f / den : 0.0f;
        f32x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) { a[e] = pacc[e] * inv; b[e] = pacc[4 + e] * inv; }
        *reinterpret_cast<f32x4*>(bufB + pi * FP + gl * 8) = a;
        *reinterpret_cast<f32x4*>(bufB + pi * FP + gl * 8 + 4) = b;
      }
    };
    if constexpr (DEPTH > 1) {
#pragma unroll
      for (int it = 0; it < PPW; ++it) {
        const bool more = it + DEPTH < PPW;
        reduce_pair(wave + it * GT_WAVES, nvs[it], hring[it % DEPTH], more ? wave + (it + DEPTH) * GT_WAVES : -1,
                    more ? nvs[(it + DEPTH) % PPW] : 0);
      }
    } else {
#pragma unroll 1
      for (int it = 0; it < PPW; ++it) {
        const int pr = pbase + wave + it * GT_WAVES;
        int nv = 0;
        if (pr < P) nv = (valid_len(lens, pair_user(cand_off, U, C, pr), L) + w - 1) / w;
        if (it > 0) load_pair(wave + it * GT_WAVES, nv, hring[0]);
        reduce_pair(wave + it * GT_WAVES, nv, hring[0], -1, 0);
      }
    }
    __syncthreads();
    if (wave < DB) {                                   // step 4: o = p W_v ; t += o
      const f32x16 o = tile_gemm_lds<D>(bufB, FP, Wl, wave, lane, l32, h);
#pragma unroll
      for (int r = 0; r < 16; ++r) ts[r] += o[r];
    }
    if (layer + 1 < M) ws.load(wq + (size_t)(layer + 1) * D * D, tid);
    __syncthreads();   // W_v and bufB fully consumed before the next layer overwrites them
  }

  // z: through LDS for coalesced fp32 rows
  if (wave < DB) store_acc(bufA, FP, ts, wave, l32, h, 1.0f);
  __syncthreads();
  for (int e = tid; e < PT * (D / 4); e += GT_THREADS) {
    const int row = e / (D / 4), c4 = e - row * (D / 4);
    if (pbase + row < P)
      *reinterpret_cast<f32x4*>(z + (size_t)(pbase + row) * D + c4 * 4) =
          *reinterpret_cast<const f32x4*>(bufA + row * FP + c4 * 4);
  }
}

// ------------------------------------------------------------------------------------------ split form (M = 1)
// One GSTA layer as three kernels that each have the shape their work wants; the fp32 output buffer z doubles as
// the only scratch (r, then p, then z live in the same [P x d] fp32 rows, each written by the reader of the last):
//   gsta_r_kernel     r = (t0 W_q) W_k^T / sqrt(d)        tiles of 32 pairs, MFMA                 -> z rows
//   gsta_pool_kernel  p = softmax_i(H'_i . r) H'          one wave per pair, H' streamed once     z rows -> z rows
//   gsta_out_kernel   z = t0 + p W_v                      tiles of 32 pairs, MFMA                 z rows -> z rows
// The streaming kernel needs ~120 registers and no LDS, so a compute unit holds 16 waves of it and HBM latency is
// covered by occupancy. The two projection kernels are pure latency chains (one tile per compute unit at the
// benchmark size), so they are written to need one round trip to memory: every operand is requested in MFMA
// operand order straight from global memory before anything is waited for.
constexpr int GS_THREADS = 256;

// B operand of X.W for column block nb: lane n = nb*32 + l32 needs W[k][n] for 8 consecutive k, i.e. a column
// piece of the row-major matrix: eight 2-byte loads per k-step (consecutive lanes read consecutive addresses).
template <int D>
__device__ __forceinline__ void load_b_cols(const unsigned short* __restrict__ W, int nb, int l32, int h,
                                            bf16x8 (&b)[D / 16]) {
  const int n = nb * 32 + l32;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
    for (int i = 0; i < 8; ++i) b[ks][i] = __builtin_bit_cast(__bf16, W[(size_t)(ks * 16 + h * 8 + i) * D + n]);
}

template <int D>
__global__ __launch_bounds__(GS_THREADS) void gsta_r_kernel(const unsigned short* __restrict__ t0,
                                                            const unsigned short* __restrict__ wq,
                                                            const unsigned short* __restrict__ wk, int P,
                                                            float* __restrict__ z) {
  constexpr int FP = D + 4, DB = D / 32;
  __shared__ __attribute__((aligned(16))) float bufB[GT_ROWS * FP];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int pbase = blockIdx.x * GT_ROWS;
  const int nb = wave < DB ? wave : 0;
  // everything the two products read from memory is requested here
  bf16x8 bq[D / 16], bk[D / 16], at[D / 16];
  load_b_cols<D>(wq, nb, l32, h, bq);
  load_b_rows<D>(wk, nb, l32, h, bk);
  {
    const int pr = (pbase + l32) < P ? (pbase + l32) : (P - 1);   // rows past the batch repeat the last pair
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
      at[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(t0 + (size_t)pr * D + ks * 16 + h * 8));
  }
  if (wave < DB) {   // q' = t0 W_q : t0 is bf16 by storage, one pass
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(at[ks], bq[ks], acc, 0, 0, 0);
    store_acc(bufB, FP, acc, wave, l32, h, 1.0f);
  }
  __syncthreads();
  if (wave < DB) {   // r = q' W_k^T / sqrt(d), written from the accumulator layout (64-byte row pieces)
    const f32x16 rr = tile_gemm_breg<D>(bufB, FP, bk, l32, h);
    const float scale = 1.0f / sqrtf((float)D);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int pr = pbase + 8 * (r >> 2) + 4 * h + (r & 3);
      if (pr < P) z[(size_t)pr * D + wave * 32 + l32] = rr[r] * scale;
    }
  }
}

template <int D>
struct WStage4 {   // W [D][D] bf16 global -> LDS for a 256-thread workgroup
  static constexpr int IT = D * (D / 8) / GS_THREADS;
  u32x4 r[IT];
  __device__ __forceinline__ void load(const unsigned short* __restrict__ W, int tid) {
#pragma unroll
    for (int it = 0; it < IT; ++it) r[it] = *reinterpret_cast<const u32x4*>(W + (size_t)(tid + it * GS_THREADS) * 8);
  }
  __device__ __forceinline__ void store(unsigned char* Wl, int tid) const {
    constexpr int WP = WPitch<D>::v, CH = D / 8;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int e = tid + it * GS_THREADS, row = e / CH, ch = e % CH;
      *reinterpret_cast<u32x4*>(Wl + row * WP + ch * 16) = r[it];
    }
  }
};

// rows of a [32 x D] fp32 LDS tile <- global rows (coalesced pieces); rows >= nrows are zero
template <int D, typename SrcT>
__device__ __forceinline__ void tile_load(float* X, int FP, const SrcT* __restrict__ src, int nrows, int tid) {
  for (int e = tid; e < GT_ROWS * (D / 4); e += GS_THREADS) {
    const int row = e / (D / 4), c4 = e - row * (D / 4);
    f32x4 val = {0.0f, 0.0f, 0.0f, 0.0f};
    if (row < nrows) {
      if constexpr (sizeof(SrcT) == 4) {
        val = *reinterpret_cast<const f32x4*>(src + (size_t)row * D + c4 * 4);
      } else {
        const unsigned int* p2 = reinterpret_cast<const unsigned int*>(src + (size_t)row * D + c4 * 4);
        const unsigned int a = p2[0], b = p2[1];
        val = f32x4{__uint_as_float(a << 16), __uint_as_float(a & 0xffff0000u), __uint_as_float(b << 16),
                    __uint_as_float(b & 0xffff0000u)};
      }
    }
    *reinterpret_cast<f32x4*>(X + row * FP + c4 * 4) = val;
  }
}

// z = t0 + p W_v for a tile of 32 pairs: W_v through LDS and the transpose load, p and t0 through LDS tiles, so
// every global access is a coalesced row piece; the tile is read completely before the barrier and written after
template <int D>
__global__ __launch_bounds__(GS_THREADS) void gsta_out_kernel(const unsigned short* __restrict__ t0,
                                                              const unsigned short* __restrict__ wv, int P,
                                                              float* __restrict__ z) {
  constexpr int FP = D + 4, DB = D / 32, WP = WPitch<D>::v;
  __shared__ __attribute__((aligned(16))) float bufA[GT_ROWS * FP];
  __shared__ __attribute__((aligned(16))) float bufB[GT_ROWS * FP];
  __shared__ __attribute__((aligned(16))) unsigned char Wl[D * WP];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int pbase = blockIdx.x * GT_ROWS;
  const int nrows = (P - pbase) < GT_ROWS ? (P - pbase) : GT_ROWS;
  WStage4<D> ws;
  ws.load(wv, tid);
  tile_load<D>(bufB, FP, z + (size_t)pbase * D, nrows, tid);           // p
  tile_load<D>(bufA, FP, t0 + (size_t)pbase * D, nrows, tid);          // t0
  ws.store(Wl, tid);
  __syncthreads();
  if (wave < DB) {   // each accumulator element adds into its own element of the t0 tile
    const f32x16 o = tile_gemm_lds<D>(bufB, FP, Wl, wave, lane, l32, h);
#pragma unroll
    for (int r = 0; r < 16; ++r) bufA[(8 * (r >> 2) + 4 * h + (r & 3)) * FP + wave * 32 + l32] += o[r];
  }
  __syncthreads();
  for (int e = tid; e < nrows * (D / 4); e += GS_THREADS) {
    const int row = e / (D / 4), c4 = e - row * (D / 4);
    *reinterpret_cast<f32x4*>(z + (size_t)(pbase + row) * D + c4 * 4) =
        *reinterpret_cast<const f32x4*>(bufA + row * FP + c4 * 4);
  }
}

// one wave per pair; ROWS register rows of 16 bytes cover the pair's S x D block.
// MR: the two other views of Sec. 3.4.4 from the same registers: the component-wise maximum over the valid segments
// (exact in fp32: stored values are compared and passed through) and a copy of the first r rows as stored. Both leave
// after the pair is reduced, behind the wave's last load.
template <int D, int ROWS, bool MR>
__global__ __launch_bounds__(GS_THREADS) void gsta_pool_kernel(const unsigned short* __restrict__ seg,
                                                               const int32_t* __restrict__ lens, const int32_t* __restrict__ cand_off, int U, int P, int C, int L,
                                                               int w, int S, float* __restrict__ z,
                                                               u32x4* __restrict__ pool, u32x4* __restrict__ recent, int r) {
  constexpr int LPR = D / 8, RPW = 64 / LPR;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: the valid length is a scalar load
  const int pr = blockIdx.x * (GS_THREADS / 64) + wave;
  if (pr >= P) return;
  const int grp = lane / LPR, gl = lane % LPR;
  const int nv = (valid_len(lens, pair_user(cand_off, U, C, pr), L) + w - 1) / w;
  const int nr = (MR && recent != nullptr) ? (r < S ? r : S) : 0;   // rows copied as stored, valid or not
  const unsigned short* H = seg + (size_t)pr * S * D;
  u32x4 hreg[ROWS];
#pragma unroll
  for (int j = 0; j < ROWS; ++j) {
    const int i = j * RPW + grp;
    // rows without a valid item are not read: zeros, or with MR the most negative finite value, which leaves the
    // maximum alone and, multiplied by its weight of zero, the sums too (the loop below stays free of branches, so
    // every row is worked on as soon as it arrives)
    hreg[j] = MR ? u32x4{0xff7fff7fu, 0xff7fff7fu, 0xff7fff7fu, 0xff7fff7fu} : u32x4{0u, 0u, 0u, 0u};
    if (i < nv) hreg[j] = *reinterpret_cast<const u32x4*>(H + (size_t)i * D + gl * 8);
  }
  float rs[8];
  {
    const f32x4 a = *reinterpret_cast<const f32x4*>(z + (size_t)pr * D + gl * 8);
    const f32x4 b = *reinterpret_cast<const f32x4*>(z + (size_t)pr * D + gl * 8 + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) { rs[e] = a[e]; rs[4 + e] = b[e]; }
  }
  float m = -INFINITY, den = 0.0f;
  float pacc[8], pmax[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    pacc[e] = 0.0f;
    pmax[e] = -INFINITY;
  }
#pragma unroll
  for (int j = 0; j < ROWS; ++j) {
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[2 * e] = __uint_as_float(hreg[j][e] << 16);
      x[2 * e + 1] = __uint_as_float(hreg[j][e] & 0xffff0000u);
    }
    float sdot = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) sdot = fmaf(x[e], rs[e], sdot);
    sdot = row_sum<LPR>(sdot);
    const bool ok = (j * RPW + grp) < nv;
    const float m_new = ok ? fmaxf(m, sdot) : m;
    const float sc = (m == m_new) ? 1.0f : __expf(m - m_new);
    const float a = ok ? __expf(sdot - m_new) : 0.0f;
    den = fmaf(den, sc, a);
#pragma unroll
    for (int e = 0; e < 8; ++e) pacc[e] = fmaf(pacc[e], sc, a * x[e]);
    m = m_new;
    if (MR) {
#pragma unroll
      for (int e = 0; e < 8; ++e) pmax[e] = fmaxf(pmax[e], x[e]);
    }
  }
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
    const float m_o = __shfl_xor(m, off, 64);
    const float den_o = __shfl_xor(den, off, 64);
    const float M2 = fmaxf(m, m_o);
    const float f = (m == M2) ? 1.0f : __expf(m - M2);
    const float f_o = (m_o == M2) ? 1.0f : __expf(m_o - M2);
    den = den * f + den_o * f_o;
#pragma unroll
    for (int e = 0; e < 8; ++e) pacc[e] = pacc[e] * f + __shfl_xor(pacc[e], off, 64) * f_o;
    m = M2;
  }
  if (MR && pool != nullptr) {
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
      for (int e = 0; e < 8; ++e) pmax[e] = fmaxf(pmax[e], __shfl_xor(pmax[e], off, 64));
  }
  if (grp == 0) {   // the row's r has been read by these same lanes above: overwrite it with p
    const float inv = nv > 0 ? 1.0f / den : 0.0f;
    f32x4 a, b;
#pragma unroll
    for (int e = 0; e < 4; ++e) { a[e] = pacc[e] * inv; b[e] = pacc[4 + e] * inv; }
    *reinterpret_cast<f32x4*>(z + (size_t)pr * D + gl * 8) = a;
    *reinterpret_cast<f32x4*>(z + (size_t)pr * D + gl * 8 + 4) = b;
    if (MR && pool != nullptr) {   // no valid segment: zeros
      u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = nv > 0 ? ((__float_as_uint(pmax[2 * e]) >> 16) | (__float_as_uint(pmax[2 * e + 1]) & 0xffff0000u)) : 0u;
      pool[(size_t)pr * LPR + gl] = o;
    }
  }
  // the first rows as stored, valid or not: read again (this wave fetched the valid ones a moment ago: cache hits)
  // rather than kept, which would hold every row's registers to the end and cost a wave of occupancy
  if (MR && nr > 0) {
    for (int i = grp; i < nr; i += RPW)
      recent[((size_t)pr * r + i) * LPR + gl] = *reinterpret_cast<const u32x4*>(H + (size_t)i * D + gl * 8);
  }
}

// ------------------------------------------------------------------------------------------ one-kernel form (M = 1)
// The three steps of the split form in one launch, for a tile of 32 pairs per workgroup (8 waves, 5 or 3 pairs each),
// so that the layer costs one launch and about one round trip to memory plus the H' stream:
//   * the lower four waves request the three weight matrices and the t0 tile (coalesced 16-byte pieces, a few
//     registers per lane) and park them in LDS, each matrix in the layout its MFMA operand read wants: W_q and
//     W_v (contraction index = row) padded for the transpose load, W_k (contraction index = column) padded for
//     16-byte row reads; waves 0 .. d/32-1 then run q' = t0 W_q and r = q' W_k^T / sqrt(d) from LDS;
//   * every wave reads the H' blocks of its pairs into registers (all S rows, unconditionally: rows of empty
//     segments are replaced by zeros when they are used, so nothing waits for the valid lengths); when each wave
//     asks for them is explained in the kernel;
//   * each wave reduces its pairs from registers (scores, softmax, weighted sum);
//   * z = t0 + p W_v leaves from the accumulator layout (128-byte row pieces).
template <int D> struct RPitch { static constexpr int v = D * 2 + 16; };   // 16-byte reads of 32 consecutive rows

// [32 x D] (LDS, fp32, pitch FP) times W^T with W bf16 [D][D] in LDS (pitch RPitch): out[p][n] = sum_k X[p][k] W[n][k]
template <int D>
__device__ __forceinline__ f32x16 tile_gemm_lds_rows(const float* X, int FP, const unsigned char* Wl, int nb, int l32,
                                                     int h) {
  constexpr int RP = RPitch<D>::v;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  const unsigned char* base = Wl + (nb * 32 + l32) * RP + h * 16;
#pragma unroll 2
  for (int ks = 0; ks < D / 16; ++ks) {
    const bf16x8 b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(base + ks * 32));
    const HiLo a = split8(X + l32 * FP + ks * 16 + h * 8);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b, acc, 0, 0, 0);
  }
  return acc;
}

// MR: also write max_pool(H') over the valid segments and the first r segments (Sec. 3.4.4) from the blocks held in
// registers (pool [P, D], recent [P, r, D], bf16; either may be null). They are staged in the LDS that held W_q and
// W_k (idle once r exists) and leave at the end, from the waves that have no part in the output product: a store
// issued while the H' stream is in flight waits in the memory pipeline behind every request queued before it, and
// the wave with it (measured: +5 us for a handful of stores per pair). r is limited by the staging space.
template <int D, int ROWS, int PPU, bool MR>
__global__ __launch_bounds__(GT_THREADS) void gsta_one_kernel(const unsigned short* __restrict__ seg,
                                                              const unsigned short* __restrict__ t0,
                                                              const unsigned short* __restrict__ wq,
                                                              const unsigned short* __restrict__ wk,
                                                              const unsigned short* __restrict__ wv,
                                                              const int32_t* __restrict__ lens, const int32_t* __restrict__ cand_off, int U, int P, int C, int L,
                                                              int w, int S, float* __restrict__ z,
                                                              u32x4* __restrict__ pool, u32x4* __restrict__ recent,
                                                              int r, int xcd_ranges) {
  constexpr int FP = D + 4, DB = D / 32, LPR = D / 8, RPW = 64 / LPR;
  constexpr int WP = WPitch<D>::v, RP = RPitch<D>::v, CH = D / 8;
  static_assert(RP == D * 2 + 16 && D * WP >= GT_ROWS * D * 2, "staging space assumed by gsta_one_max_recent / the pooled rows");
  // pairs per wave: PPU for the upper waves, which hold their blocks from the start, PPL for the lower waves, which
  // ask for theirs once the projection chain is done. 5 + 3 when every compute unit has a workgroup (the launch is
  // then a stream of H' at memory speed, and the earlier a block is requested the better), 4 + 4 for small batches
  // (latency-bound: the longest wave decides)
  constexpr int PPL = GT_ROWS / (GT_WAVES / 2) - PPU;
  static_assert((GT_WAVES / 2) * (PPU + PPL) == GT_ROWS, "the pairs of a tile are dealt to the two halves");
  __shared__ __attribute__((aligned(16))) float bufA[GT_ROWS * FP];
  __shared__ __attribute__((aligned(16))) float bufB[GT_ROWS * FP];
  __shared__ __attribute__((aligned(16))) unsigned char Wql[D * WP];
  __shared__ __attribute__((aligned(16))) unsigned char Wvl[D * WP];
  __shared__ __attribute__((aligned(16))) unsigned char Wkl[D * RP];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: the valid lengths become scalar loads
  // Workgroups are dealt to the eight XCDs round-robin by index; with xcd_ranges they are renumbered so that each
  // XCD takes a contiguous range of pair tiles, the same users whose H' the matrix-core STA kernel, which numbers
  // its workgroups the same way, has just written through that XCD's L2
  int tile = blockIdx.x;
  if (xcd_ranges && gridDim.x % 8 == 0) tile = (tile % 8) * (gridDim.x / 8) + tile / 8;
  const int pbase = tile * GT_ROWS;
  const int grp = lane / LPR, gl = lane % LPR;
  // (a vector load of a length here would make the compiler wait for every load in flight, the H' stream included)
  const bool front = wave < GT_WAVES / 2;
  // first pair of this wave inside the tile and how many it has
  const int pfirst = front ? (GT_WAVES / 2) * PPU + wave * PPL : (wave - GT_WAVES / 2) * PPU;
  int nvs[PPU];
#pragma unroll
  for (int it = 0; it < PPU; ++it) {
    const int pr = pbase + pfirst + it;
    nvs[it] = (pr < P && (it < PPL || !front)) ? (valid_len(lens, pair_user(cand_off, U, C, pr), L) + w - 1) / w : 0;
  }

  // One register set per pair. A wave issues in order, and a compute unit's memory pipeline accepts requests only
  // about as fast as the data comes back: a wave that asks for much sits in the issue queue, and would keep its
  // workgroup waiting at every barrier it has not reached. So the roles are split. The upper four waves ask for
  // all their blocks at once and meet the others only when r is needed. The lower four waves fetch and park the
  // small operands and run the projection chain, synchronising among themselves through a counter in LDS (the
  // hardware barrier counts every wave of the workgroup); they ask for their own blocks once r is written, and
  // those stream in while the upper waves, which share their SIMDs, reduce.
  u32x4 hring[PPU][ROWS];
  auto load_pair = [&](int it, u32x4 (&hreg)[ROWS]) {
    const int pr = (pbase + pfirst + it) < P ? (pbase + pfirst + it) : (P - 1);   // past the batch: repeat
    const unsigned short* H = seg + (size_t)pr * S * D;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const int i = j * RPW + grp;
      hreg[j] = *reinterpret_cast<const u32x4*>(H + (size_t)(i < S ? i : S - 1) * D + gl * 8);
    }
  };
  __shared__ unsigned int arrived[2];
  if (tid < 2) arrived[tid] = 0u;
  __syncthreads();   // everyone is here within the first instructions; nothing has been requested yet
  // arrival counter for the lower waves: LDS operations of a wave execute in order, so what it wrote before its
  // increment is visible to whoever reads the new count. The wait ends because the four lower waves of a workgroup
  // are resident together (a workgroup is launched whole), none of them leaves the kernel or waits for an upper wave
  // before its second arrival, and each arrives at each counter exactly once: the count reaches four as soon as the
  // slowest of them gets there, a few microseconds at most. The poll is bounded all the same, so that no edit of
  // the code around it can turn a lost arrival into a hang of the machine: after LOWER_SYNC_SPINS polls (about a
  // tenth of a second, four orders of magnitude beyond any legitimate wait) the wave goes on without the others,
  // the kernel ends normally, and the results of that workgroup are undefined.
  constexpr int LOWER_SYNC_SPINS = 1 << 20;
  auto lower_sync = [&](int idx) {
    if (lane == 0) __hip_atomic_fetch_add(&arrived[idx], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    for (int spin = 0; spin < LOWER_SYNC_SPINS; ++spin) {
      if (__hip_atomic_load(&arrived[idx], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= GT_WAVES / 2) break;
      __builtin_amdgcn_s_sleep(1);
    }
  };
  if (!front) {
#pragma unroll
    for (int it = 0; it < PPU; ++it) load_pair(it, hring[it]);
  } else {
    constexpr int FT = GT_THREADS / 2;
    constexpr int WIT = D * CH / FT;                   // 16-byte pieces per thread and matrix
    constexpr int TIT = GT_ROWS * (D / 4) / FT;        // 8-byte pieces of the t0 tile per thread
    static_assert((D * CH) % FT == 0 && (GT_ROWS * (D / 4)) % FT == 0, "tile sizes divide the loader threads");
    u32x4 rq[WIT], rk[WIT], rv[WIT];
    unsigned int traw[TIT][2];
#pragma unroll
    for (int it = 0; it < WIT; ++it) rq[it] = *reinterpret_cast<const u32x4*>(wq + (size_t)(tid + it * FT) * 8);
#pragma unroll
    for (int it = 0; it < TIT; ++it) {
      const int e = tid + it * FT, row = e / (D / 4), c4 = e % (D / 4);
      const int pr = (pbase + row) < P ? (pbase + row) : (P - 1);
      const unsigned int* p2 = reinterpret_cast<const unsigned int*>(t0 + (size_t)pr * D + c4 * 4);
      traw[it][0] = p2[0];
      traw[it][1] = p2[1];
    }
#pragma unroll
    for (int it = 0; it < WIT; ++it) rk[it] = *reinterpret_cast<const u32x4*>(wk + (size_t)(tid + it * FT) * 8);
#pragma unroll
    for (int it = 0; it < WIT; ++it) rv[it] = *reinterpret_cast<const u32x4*>(wv + (size_t)(tid + it * FT) * 8);
    // park them in LDS, each matrix with the pitch its operand read wants
#pragma unroll
    for (int it = 0; it < WIT; ++it) {
      const int e = tid + it * FT, row = e / CH, ch = e % CH;
      *reinterpret_cast<u32x4*>(Wql + row * WP + ch * 16) = rq[it];
    }
#pragma unroll
    for (int it = 0; it < TIT; ++it) {
      const int e = tid + it * FT, row = e / (D / 4), c4 = e % (D / 4);
      *reinterpret_cast<f32x4*>(bufA + row * FP + c4 * 4) =
          f32x4{__uint_as_float(traw[it][0] << 16), __uint_as_float(traw[it][0] & 0xffff0000u),
                __uint_as_float(traw[it][1] << 16), __uint_as_float(traw[it][1] & 0xffff0000u)};
    }
#pragma unroll
    for (int it = 0; it < WIT; ++it) {
      const int e = tid + it * FT, row = e / CH, ch = e % CH;
      *reinterpret_cast<u32x4*>(Wkl + row * RP + ch * 16) = rk[it];
      *reinterpret_cast<u32x4*>(Wvl + row * WP + ch * 16) = rv[it];
    }
  }
  if (front) lower_sync(0);
  f32x16 ts;
  if (wave < DB) {   // q' = t0 W_q; t0 in accumulator layout is kept for the last step
#pragma unroll
    for (int r = 0; r < 16; ++r) ts[r] = bufA[(8 * (r >> 2) + 4 * h + (r & 3)) * FP + wave * 32 + l32];
    const f32x16 qp = tile_gemm_lds<D>(bufA, FP, Wql, wave, lane, l32, h);
    store_acc(bufB, FP, qp, wave, l32, h, 1.0f);
  }
  if (front) lower_sync(1);
  if (wave < DB) {   // r = q' W_k^T / sqrt(d)
    const f32x16 rr = tile_gemm_lds_rows<D>(bufB, FP, Wkl, wave, l32, h);
    store_acc(bufA, FP, rr, wave, l32, h, 1.0f / sqrtf((float)D));
  }
  __syncthreads();   // r complete in bufA; q' in bufB consumed
  if (front) {
#pragma unroll
    for (int it = 0; it < PPL; ++it) load_pair(it, hring[it]);
  }

  auto reduce_pair = [&](const u32x4 (&hcur)[ROWS], int pi, int nv) __attribute__((always_inline)) {
    if (MR) {
      u32x4* stage_pool = reinterpret_cast<u32x4*>(Wql);
      u32x4* stage_recent = reinterpret_cast<u32x4*>(Wkl);
      if (recent != nullptr) {
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
          const int i = j * RPW + grp;
          if (i < r) stage_recent[(pi * r + i) * LPR + gl] = hcur[j];   // as stored (zeros where no item is valid)
        }
      }
      if (pool != nullptr) {
        // maximum over the valid rows of this lane group, then over the lane groups; bf16 values compared as
        // floats, bits passed through
        float mx[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) mx[e] = -INFINITY;
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
          if ((j * RPW + grp) < nv) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              mx[2 * e] = fmaxf(mx[2 * e], __uint_as_float(hcur[j][e] << 16));
              mx[2 * e + 1] = fmaxf(mx[2 * e + 1], __uint_as_float(hcur[j][e] & 0xffff0000u));
            }
          }
        }
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
          for (int e = 0; e < 8; ++e) mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], off, 64));
        if (grp == 0) {
          u32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const unsigned int lo = nv > 0 ? (__float_as_uint(mx[2 * e]) >> 16) : 0u;
            const unsigned int hi = nv > 0 ? (__float_as_uint(mx[2 * e + 1]) & 0xffff0000u) : 0u;
            o[e] = lo | hi;
          }
          stage_pool[pi * LPR + gl] = o;
        }
      }
    }
    // r of the pair, this lane's eight components, as two bf16 pairs per two components: r = hi + lo up to 2^-17 of
    // its size, so that a score is two dot products of packed pairs (v_dot2c_f32_bf16) per stored word instead of
    // two conversions and two multiply-adds
    bf16x2 rhi[4], rlo[4];
    {
      const f32x4 a = *reinterpret_cast<const f32x4*>(bufA + pi * FP + gl * 8);
      const f32x4 b = *reinterpret_cast<const f32x4*>(bufA + pi * FP + gl * 8 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float r0 = e < 2 ? a[2 * e] : b[2 * e - 4], r1 = e < 2 ? a[2 * e + 1] : b[2 * e - 3];
        rhi[e] = bf16x2{(__bf16)r0, (__bf16)r1};
        rlo[e] = bf16x2{(__bf16)(r0 - (float)rhi[e][0]), (__bf16)(r1 - (float)rhi[e][1])};
      }
    }
    // Rows of empty segments count as zeros whatever they hold: replaced once, for both passes
    // (words kept as scalars: cast to a bf16 pair straight out of a four-word vector, the compiler's lowering picked
    // the vector's first word for all four)
    unsigned int hs[ROWS][4];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const bool ok = (j * RPW + grp) < nv;
#pragma unroll
      for (int e = 0; e < 4; ++e) hs[j][e] = ok ? hcur[j][e] : 0u;
    }
    // Two passes over the register-resident block instead of a running maximum: the rows' scores are independent
    // of each other (eight dot products in flight instead of one chain of dependent rescalings), and the weighted
    // sum then needs no rescaling: the maximum is taken over the whole pair (the four lane groups hold their own in
    // all their lanes: four scalar reads) before the second pass.
    float sd[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      float sdot = 0.0f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bf16x2 x = __builtin_bit_cast(bf16x2, hs[j][e]);
        sdot = __builtin_amdgcn_fdot2_f32_bf16(x, rhi[e], sdot, false);
        sdot = __builtin_amdgcn_fdot2_f32_bf16(x, rlo[e], sdot, false);
      }
      sdot = row_sum<LPR>(sdot);
      sd[j] = (j * RPW + grp) < nv ? sdot : -INFINITY;
    }
    float m = sd[0];
#pragma unroll
    for (int j = 1; j < ROWS; ++j) m = fmaxf(m, sd[j]);
    if constexpr (LPR == 16) {
      const int mb = __float_as_int(m);
      m = fmaxf(fmaxf(__int_as_float(__builtin_amdgcn_readlane(mb, 0)), __int_as_float(__builtin_amdgcn_readlane(mb, 16))),
                fmaxf(__int_as_float(__builtin_amdgcn_readlane(mb, 32)), __int_as_float(__builtin_amdgcn_readlane(mb, 48))));
    } else {
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    }
    const float mref = (m == -INFINITY) ? 0.0f : m;   // no valid row in this pair
    float den = 0.0f;
    float pacc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) pacc[e] = 0.0f;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
      const float a = __expf(sd[j] - mref);   // 0 for the rows of empty segments (their score is -inf)
      den += a;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const unsigned int pk = hs[j][e];
        pacc[2 * e] = fmaf(a, __uint_as_float(pk << 16), pacc[2 * e]);
        pacc[2 * e + 1] = fmaf(a, __uint_as_float(pk & 0xffff0000u), pacc[2 * e + 1]);
      }
    }
    // sums over the lane groups (the same reference in all of them: plain additions), the upper half first
    // (lane ^ 32 by v_permlane32_swap, no LDS round trip)
    auto add_other = [&](float x, int off) {
      if (off == 32) {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
        return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
      }
      return x + __shfl_xor(x, off, 64);
    };
#pragma unroll
    for (int off = 32; off >= LPR; off >>= 1) {
      den = add_other(den, off);
#pragma unroll
      for (int e = 0; e < 8; ++e) pacc[e] = add_other(pacc[e], off);
    }
    if (grp == 0) {
      const float inv = nv > 0 ? 1.0f / den : 0.0f;
      f32x4 a, b;
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = pacc[e] * inv; b[e] = pacc[4 + e] * inv; }
      *reinterpret_cast<f32x4*>(bufB + pi * FP + gl * 8) = a;
      *reinterpret_cast<f32x4*>(bufB + pi * FP + gl * 8 + 4) = b;
    }
  };
#pragma unroll
  for (int it = 0; it < PPL; ++it) reduce_pair(hring[it], pfirst + it, nvs[it]);
  if (!front) {
#pragma unroll
    for (int it = PPL; it < PPU; ++it) reduce_pair(hring[it], pfirst + it, nvs[it]);
  }
  __syncthreads();
  if (MR && wave >= DB) {   // the staged views leave while the other waves run the output product
    constexpr int NT2 = (GT_WAVES - DB) * 64;
    const int t2 = tid - DB * 64;
    const int npair = (P - pbase) < GT_ROWS ? (P - pbase) : GT_ROWS;
    if (recent != nullptr) {
      const u32x4* st = reinterpret_cast<const u32x4*>(Wkl);
      u32x4* dst = recent + (size_t)pbase * r * LPR;   // the tile's rows are contiguous in the output
      for (int e = t2; e < npair * r * LPR; e += NT2) dst[e] = st[e];
    }
    if (pool != nullptr) {
      const u32x4* st = reinterpret_cast<const u32x4*>(Wql);
      u32x4* dst = pool + (size_t)pbase * LPR;
      for (int e = t2; e < npair * LPR; e += NT2) dst[e] = st[e];
    }
  }
  if (wave < DB) {   // z = t0 + p W_v
    const f32x16 o = tile_gemm_lds<D>(bufB, FP, Wvl, wave, lane, l32, h);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int pr = pbase + 8 * (r >> 2) + 4 * h + (r & 3);
      if (pr < P) z[(size_t)pr * D + wave * 32 + l32] = ts[r] + o[r];
    }
  }
}

static int rows_needed(int S, int d) { return (S + (64 / (d / 8)) - 1) / (64 / (d / 8)); }

bool gsta_tiled_supports(const GstaArgs& a) {
  if (a.dt != LASER_BF16) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  return rows_needed(a.S, a.d) <= 10;   // the pair's H' block must fit a wave's registers several times over
}

template <int D, int ROWS, int PT>
static void launch_pt(const GstaArgs& a) {
  const int P = gsta_pairs(a);
  hipLaunchKernelGGL((gsta_tiled_kernel<D, ROWS, PT>), dim3((P + PT - 1) / PT), dim3(GT_THREADS), 0, a.stream,
                     (const unsigned short*)a.seg, (const unsigned short*)a.t0, (const unsigned short*)a.wq,
                     (const unsigned short*)a.wk, (const unsigned short*)a.wv, a.lens, a.cand_off, a.U, P, a.C, a.L, a.w, a.S, a.M,
                     a.z_out);
}

// pairs per workgroup: fewer when the batch is small, so that every compute unit still gets a few workgroups
static int pick_pt(int P) {
  int pt = P >= 8192 ? 32 : 8;   // measured: the per-workgroup set-up cost favours full tiles once every compute unit has one
  const int vv = tuning_int("LASER_GSTA_PT", 0);   // tuning builds only
  if (vv == 8 || vv == 16 || vv == 32) pt = vv;
  return pt;
}

template <int D, int ROWS>
static void launch_rows(const GstaArgs& a) {
  const int pt = pick_pt(gsta_pairs(a));
  if (pt == 32) launch_pt<D, ROWS, 32>(a);
  else if (pt == 16) launch_pt<D, ROWS, 16>(a);
  else launch_pt<D, ROWS, 8>(a);
}

template <int D>
static void launch_d(const GstaArgs& a) {
  const int rows = rows_needed(a.S, a.d);
  if (rows <= 2) launch_rows<D, 2>(a);
  else if (rows <= 4) launch_rows<D, 4>(a);
  else if (rows <= 8) launch_rows<D, 8>(a);
  else launch_rows<D, 10>(a);
}

template <int D>
static void launch_split(const GstaArgs& a) {
  const int P = gsta_pairs(a);
  const unsigned tiles = (unsigned)((P + GT_ROWS - 1) / GT_ROWS);
  const unsigned short* t0 = (const unsigned short*)a.t0;
  hipLaunchKernelGGL((gsta_r_kernel<D>), dim3(tiles), dim3(GS_THREADS), 0, a.stream, t0,
                     (const unsigned short*)a.wq, (const unsigned short*)a.wk, P, a.z_out);
  const int rows = rows_needed(a.S, a.d);
  const unsigned pblocks = (unsigned)((P + GS_THREADS / 64 - 1) / (GS_THREADS / 64));
  const bool views = a.pool_out != nullptr || a.recent_out != nullptr;
#define LASER_POOL(R)                                                                                             \
  do {                                                                                                            \
    if (views)                                                                                                    \
      hipLaunchKernelGGL((gsta_pool_kernel<D, R, true>), dim3(pblocks), dim3(GS_THREADS), 0, a.stream,            \
                         (const unsigned short*)a.seg, a.lens, a.cand_off, a.U, P, a.C, a.L, a.w, a.S, a.z_out,    \
                         (u32x4*)a.pool_out, (u32x4*)a.recent_out, a.r);                                          \
    else                                                                                                          \
      hipLaunchKernelGGL((gsta_pool_kernel<D, R, false>), dim3(pblocks), dim3(GS_THREADS), 0, a.stream,           \
                         (const unsigned short*)a.seg, a.lens, a.cand_off, a.U, P, a.C, a.L, a.w, a.S, a.z_out,    \
                         (u32x4*)nullptr, (u32x4*)nullptr, 0);                                                    \
  } while (0)
  if (rows <= 2) LASER_POOL(2);
  else if (rows <= 4) LASER_POOL(4);
  else if (rows <= 8) LASER_POOL(8);
  else if (rows <= 10) LASER_POOL(10);
  else if (rows <= 16) LASER_POOL(16);
  else LASER_POOL(32);
#undef LASER_POOL
  hipLaunchKernelGGL((gsta_out_kernel<D>), dim3(tiles), dim3(GS_THREADS), 0, a.stream, t0,
                     (const unsigned short*)a.wv, P, a.z_out);
}

bool gsta_split_supports(const GstaArgs& a) {
  if (a.dt != LASER_BF16 || a.M != 1) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  return rows_needed(a.S, a.d) <= 32;
}

laser_status gsta_split_launch(const GstaArgs& a) {
  if (!gsta_split_supports(a)) return LASER_ERR_UNSUPPORTED;
  if (a.d == 64) launch_split<64>(a);
  else launch_split<128>(a);
  return launch_status();
}

// The outer two launches of the split form on their own, for a caller that produces p itself between them
// (ffn_gsta.hip): r = (t0 W_q) W_k^T / sqrt(d) into the z rows, and z = t0 + p W_v from the z rows. bf16, d in {64, 128}.
laser_status gsta_r_launch(const GstaArgs& a) {
  if (a.dt != LASER_BF16 || !(a.d == 64 || a.d == 128)) return LASER_ERR_UNSUPPORTED;
  const int P = gsta_pairs(a);
  const unsigned tiles = (unsigned)((P + GT_ROWS - 1) / GT_ROWS);
  if (a.d == 64)
    hipLaunchKernelGGL((gsta_r_kernel<64>), dim3(tiles), dim3(GS_THREADS), 0, a.stream, (const unsigned short*)a.t0,
                       (const unsigned short*)a.wq, (const unsigned short*)a.wk, P, a.z_out);
  else
    hipLaunchKernelGGL((gsta_r_kernel<128>), dim3(tiles), dim3(GS_THREADS), 0, a.stream, (const unsigned short*)a.t0,
                       (const unsigned short*)a.wq, (const unsigned short*)a.wk, P, a.z_out);
  return launch_status();
}

laser_status gsta_out_launch(const GstaArgs& a) {
  if (a.dt != LASER_BF16 || !(a.d == 64 || a.d == 128)) return LASER_ERR_UNSUPPORTED;
  const int P = gsta_pairs(a);
  const unsigned tiles = (unsigned)((P + GT_ROWS - 1) / GT_ROWS);
  if (a.d == 64)
    hipLaunchKernelGGL((gsta_out_kernel<64>), dim3(tiles), dim3(GS_THREADS), 0, a.stream, (const unsigned short*)a.t0,
                       (const unsigned short*)a.wv, P, a.z_out);
  else
    hipLaunchKernelGGL((gsta_out_kernel<128>), dim3(tiles), dim3(GS_THREADS), 0, a.stream, (const unsigned short*)a.t0,
                       (const unsigned short*)a.wv, P, a.z_out);
  return launch_status();
}

bool gsta_one_supports(const GstaArgs& a) {
  if (a.dt != LASER_BF16 || a.M != 1) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  return rows_needed(a.S, a.d) <= 8;   // five H' blocks per upper wave are held in registers
}

template <int D>
static void launch_one_kernel(const GstaArgs& a) {
  const int P = gsta_pairs(a);
  const unsigned tiles = (unsigned)((P + GT_ROWS - 1) / GT_ROWS);
  const int rows = rows_needed(a.S, a.d);
#define LASER_ONE_MR(R, PU, MRF)                                                                                   \
  hipLaunchKernelGGL((gsta_one_kernel<D, R, PU, MRF>), dim3(tiles), dim3(GT_THREADS), 0, a.stream,                \
                     (const unsigned short*)a.seg, (const unsigned short*)a.t0, (const unsigned short*)a.wq,       \
                     (const unsigned short*)a.wk, (const unsigned short*)a.wv, a.lens, a.cand_off, a.U, P, a.C, a.L, a.w, a.S,      \
                     a.z_out, (u32x4*)a.pool_out, (u32x4*)a.recent_out, a.r, xcd_ranges)
#define LASER_ONE(R, PU)                                                                                           \
  do {                                                                                                             \
    if (views) LASER_ONE_MR(R, PU, true);                                                                          \
    else LASER_ONE_MR(R, PU, false);                                                                               \
  } while (0)
  const bool views = a.pool_out != nullptr || a.recent_out != nullptr;
  const bool fills = tiles >= 256;   // a workgroup for every compute unit
  // pair tiles in contiguous ranges per XCD (measured on 32 users x 256 candidates: the step 52.3 -> 51.2 us; loads
  // of H' with the non-temporal hint change nothing); a tuning build can switch it off
  const int xcd_ranges = tuning_int("LASER_GSTA_XCD", 1);
  if (rows <= 2) { if (fills) LASER_ONE(2, 5); else LASER_ONE(2, 4); }
  else if (rows <= 4) { if (fills) LASER_ONE(4, 5); else LASER_ONE(4, 4); }
  else { if (fills) LASER_ONE(8, 5); else LASER_ONE(8, 4); }
#undef LASER_ONE
#undef LASER_ONE_MR
}

// most recent segments the one-kernel form can stage per pair (the LDS of W_k holds them for a tile of pairs)
int gsta_one_max_recent(int d) { return (d * (d * 2 + 16)) / (GT_ROWS * d * 2); }

laser_status gsta_one_launch(const GstaArgs& a) {
  if (!gsta_one_supports(a)) return LASER_ERR_UNSUPPORTED;
  if (a.recent_out != nullptr && a.r > gsta_one_max_recent(a.d)) return LASER_ERR_UNSUPPORTED;
  if (a.d == 64) launch_one_kernel<64>(a);
  else launch_one_kernel<128>(a);
  return launch_status();
}

laser_status gsta_tiled_launch(const GstaArgs& a) {
  if (!gsta_tiled_supports(a)) return LASER_ERR_UNSUPPORTED;
  if (a.d == 64) launch_d<64>(a);
  else launch_d<128>(a);
  return launch_status();
}

}  // namespace laser
