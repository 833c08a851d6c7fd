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
// target t stays in fp32 registers in accumulator layout. Weight operands come straight from global memory
// (L2 resident, 3 d^2 elements per layer). Two fp32 [32 x d] LDS buffers carry the operands between steps.
#include "laser_internal.h"

namespace laser {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int GT_PAIRS = 32;

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

// [32 x D] (LDS, fp32, pitch FP) times W (global bf16 [D][D]) -> 32 x 32 block `nb` of the product.
// TRANSPOSED = false: out = X W      (B operand k = row of W: eight 2-byte loads per lane per step)
// TRANSPOSED = true : out = X W^T    (B operand k = column of W: one 16-byte load per lane per step)
template <int D, bool TRANSPOSED>
__device__ __forceinline__ f32x16 tile_gemm(const float* X, int FP, const unsigned short* __restrict__ W, int nb,
                                            int l32, int h) {
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  const int n = nb * 32 + l32;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    const int k0 = ks * 16 + h * 8;
    bf16x8 b;
    if (TRANSPOSED) {
      b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(W + (size_t)n * D + k0));
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) b[i] = __builtin_bit_cast(__bf16, W[(size_t)(k0 + i) * D + n]);
    }
    const HiLo a = split8(X + l32 * FP + k0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b, acc, 0, 0, 0);
  }
  return acc;
}

// accumulator layout: lane = column nb*32 + l32, register r = row 8 (r/4) + 4 h + r % 4
__device__ __forceinline__ void store_acc(float* X, int FP, const f32x16& acc, int nb, int l32, int h, float scale) {
#pragma unroll
  for (int r = 0; r < 16; ++r) X[(8 * (r >> 2) + 4 * h + (r & 3)) * FP + nb * 32 + l32] = acc[r] * scale;
}

template <int D, int ROWS>
__global__ __launch_bounds__(256) void gsta_tiled_kernel(const unsigned short* __restrict__ seg,
                                                         const unsigned short* __restrict__ t0,
                                                         const unsigned short* __restrict__ wq,
                                                         const unsigned short* __restrict__ wk,
                                                         const unsigned short* __restrict__ wv,
                                                         const int32_t* __restrict__ lens, int P, int C, int L, int w,
                                                         int S, int M, float* __restrict__ z) {
  constexpr int FP = D + 4;          // fp32 row pitch: 16 B mod 256 B, conflict-free 16-byte row reads
  constexpr int DB = D / 32;         // 32-column blocks; waves >= DB idle in the MFMA steps
  constexpr int LPR = D / 8;         // lanes per H' row (16 B each)
  constexpr int RPW = 64 / LPR;      // rows per wave-wide load
  __shared__ __attribute__((aligned(16))) float bufA[GT_PAIRS * FP];
  __shared__ __attribute__((aligned(16))) float bufB[GT_PAIRS * FP];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;
  const int pbase = blockIdx.x * GT_PAIRS;
  const float scale = 1.0f / sqrtf((float)D);

  // running target t in accumulator layout (wave = column block)
  f32x16 ts;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int pr = pbase + 8 * (r >> 2) + 4 * h + (r & 3);
    ts[r] = (wave < DB && pr < P) ? bf16_bits_to_f32(t0[(size_t)pr * D + wave * 32 + l32]) : 0.0f;
  }

  const int grp = lane / LPR, gl = lane % LPR;   // row group and position inside the row

  for (int layer = 0; layer < M; ++layer) {
    const unsigned short* Wq = wq + (size_t)layer * D * D;
    const unsigned short* Wk = wk + (size_t)layer * D * D;
    const unsigned short* Wv = wv + (size_t)layer * D * D;

    if (wave < DB) store_acc(bufA, FP, ts, wave, l32, h, 1.0f);
    __syncthreads();
    if (wave < DB) {                                   // step 1: q' = t W_q
      const f32x16 qp = tile_gemm<D, false>(bufA, FP, Wq, wave, l32, h);
      store_acc(bufB, FP, qp, wave, l32, h, 1.0f);
    }
    __syncthreads();
    if (wave < DB) {                                   // step 2: r = q' W_k^T / sqrt(d)
      const f32x16 rr = tile_gemm<D, true>(bufB, FP, Wk, wave, l32, h);
      store_acc(bufA, FP, rr, wave, l32, h, scale);
    }
    __syncthreads();

    // step 3: one pair per wave at a time; its H' block goes through registers once
    for (int pi = wave; pi < GT_PAIRS; pi += 4) {
      const int pr = pbase + pi;
      int nv = 0;
      if (pr < P) {
        const int n = valid_len(lens, pr / C, L);
        nv = (n + w - 1) / w;
      }
      u32x4 hreg[ROWS];
      const unsigned short* H = seg + (size_t)pr * S * D;
#pragma unroll
      for (int j = 0; j < ROWS; ++j) {
        const int i = j * RPW + grp;
        hreg[j] = u32x4{0u, 0u, 0u, 0u};
        if (i < nv) hreg[j] = *reinterpret_cast<const u32x4*>(H + (size_t)i * D + gl * 8);
      }
      float rs[8];
      {
        const f32x4 a = *reinterpret_cast<const f32x4*>(bufA + pi * FP + gl * 8);
        const f32x4 b = *reinterpret_cast<const f32x4*>(bufA + pi * FP + gl * 8 + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { rs[e] = a[e]; rs[4 + e] = b[e]; }
      }
      float e_[ROWS];
      float mx = -INFINITY;
#pragma unroll
      for (int j = 0; j < ROWS; ++j) {
        float s = 0.0f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          s = fmaf(__uint_as_float(hreg[j][e] << 16), rs[2 * e], s);
          s = fmaf(__uint_as_float(hreg[j][e] & 0xffff0000u), rs[2 * e + 1], s);
        }
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) s += __shfl_xor(s, off, 64);
        const bool ok = (j * RPW + grp) < nv;
        e_[j] = ok ? s : -INFINITY;
        mx = fmaxf(mx, e_[j]);
      }
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      float den = 0.0f;
      float pacc[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pacc[e] = 0.0f;
#pragma unroll
      for (int j = 0; j < ROWS; ++j) {
        const float a = (e_[j] == -INFINITY) ? 0.0f : __expf(e_[j] - mx);
        den += a;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          pacc[2 * e] = fmaf(a, __uint_as_float(hreg[j][e] << 16), pacc[2 * e]);
          pacc[2 * e + 1] = fmaf(a, __uint_as_float(hreg[j][e] & 0xffff0000u), pacc[2 * e + 1]);
        }
      }
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) {
        den += __shfl_xor(den, off, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e) pacc[e] += __shfl_xor(pacc[e], off, 64);
      }
      if (grp == 0) {
        const float inv = nv > 0 ? 1.0f / den : 0.0f;
        f32x4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) { a[e] = pacc[e] * inv; b[e] = pacc[4 + e] * inv; }
        *reinterpret_cast<f32x4*>(bufB + pi * FP + gl * 8) = a;
        *reinterpret_cast<f32x4*>(bufB + pi * FP + gl * 8 + 4) = b;
      }
    }
    __syncthreads();
    if (wave < DB) {                                   // step 4: o = p W_v ; t += o
      const f32x16 o = tile_gemm<D, false>(bufB, FP, Wv, wave, l32, h);
#pragma unroll
      for (int r = 0; r < 16; ++r) ts[r] += o[r];
    }
    // bufA is next written after this point only by waves that have passed the barrier above; bufB is next
    // written in step 1 of the next layer, after the barrier that follows the bufA store.
  }

  // z: through LDS for coalesced fp32 rows
  __syncthreads();
  if (wave < DB) store_acc(bufA, FP, ts, wave, l32, h, 1.0f);
  __syncthreads();
  for (int e = tid; e < GT_PAIRS * (D / 4); e += 256) {
    const int row = e / (D / 4), c4 = e - row * (D / 4);
    if (pbase + row < P)
      *reinterpret_cast<f32x4*>(z + (size_t)(pbase + row) * D + c4 * 4) =
          *reinterpret_cast<const f32x4*>(bufA + row * FP + c4 * 4);
  }
}

static int rows_needed(int S, int d) { return (S + (64 / (d / 8)) - 1) / (64 / (d / 8)); }

bool gsta_tiled_supports(const GstaArgs& a) {
  if (a.dt != LASER_BF16) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  return rows_needed(a.S, a.d) <= 32;
}

template <int D, int ROWS>
static void launch_rows(const GstaArgs& a) {
  const int P = a.U * a.C;
  hipLaunchKernelGGL((gsta_tiled_kernel<D, ROWS>), dim3((P + GT_PAIRS - 1) / GT_PAIRS), dim3(256), 0, a.stream,
                     (const unsigned short*)a.seg, (const unsigned short*)a.t0, (const unsigned short*)a.wq,
                     (const unsigned short*)a.wk, (const unsigned short*)a.wv, a.lens, P, a.C, a.L, a.w, a.S, a.M,
                     a.z_out);
}

template <int D>
static void launch_d(const GstaArgs& a) {
  const int rows = rows_needed(a.S, a.d);
  if (rows <= 2) launch_rows<D, 2>(a);
  else if (rows <= 4) launch_rows<D, 4>(a);
  else if (rows <= 8) launch_rows<D, 8>(a);
  else if (rows <= 10) launch_rows<D, 10>(a);
  else if (rows <= 16) launch_rows<D, 16>(a);
  else launch_rows<D, 32>(a);
}

laser_status gsta_tiled_launch(const GstaArgs& a) {
  if (!gsta_tiled_supports(a)) return LASER_ERR_UNSUPPORTED;
  if (a.d == 64) launch_d<64>(a);
  else launch_d<128>(a);
  return launch_status();
}

}  // namespace laser
