// Pieces shared by the matrix-core STA kernels (sta_mfma.hip) and the fused STA + GSTA kernel (fused_forward.hip):
// operand vector types, the tile geometry, LDS row pitches, the sigmoid gate, and the register-staged tile loader.
#pragma once

#include "laser_internal.h"

namespace laser {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int TI = 64;    // history items staged per step
constexpr int CW = 32;    // candidates per wave
// output patch row pitch in bytes: one H' row + 16 (keeps 16-byte alignment for the row-wise read-back)
template <int D> struct OPitch { static constexpr int v = D * 2 + 16; };

// LDS row pitches in bytes. K rows are read 16 B per lane by 32 consecutive items: pitch = 16 mod 256 spreads
// them over all banks. V rows are read by the transpose load, four consecutive items x 64 B: pitch = 64 mod 256.
template <int DQ> struct KPitch { static constexpr int v = DQ * 2 + 16; };
template <int D> struct VPitch { static constexpr int v = (D * 2) % 256 == 64 ? D * 2 : D * 2 + 64; };

__device__ __forceinline__ float gate(float score, float neg_scale_log2e) {
  // sigmoid(x) = 1 / (1 + 2^(-x log2 e)); x = score / gamma
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(score * neg_scale_log2e));
}

template <int DQ, int D, int NT>
struct Stage {
  static constexpr int KCH = DQ / 8, VCH = D / 8;   // 16-byte chunks per row
  static constexpr int KIT = (TI * KCH + NT - 1) / NT, VIT = (TI * VCH + NT - 1) / NT;
  static constexpr bool KEXACT = (TI * KCH) % NT == 0, VEXACT = (TI * VCH) % NT == 0;
  u32x4 kr[KIT], vr[VIT];
  int nvalid;   // rows of the tile that hold valid items

  // global -> registers. Straight-line code (no per-lane branches) so that the loads stay in flight while the
  // caller computes: rows at or past `hi` are fetched from the last valid row instead and zeroed in store().
  // Requires t0 < hi.
  __device__ __forceinline__ void load(const unsigned short* kU, const unsigned short* vU, int t0, int hi, int tid) {
    nvalid = hi - t0;
    const int last = nvalid - 1;
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      int e = tid + it * NT;
      if (!KEXACT) e = e < TI * KCH ? e : TI * KCH - 1;
      int r = e / KCH;
      const int ch = e % KCH;
      r = r < last ? r : last;
      kr[it] = *reinterpret_cast<const u32x4*>(kU + (size_t)(t0 + r) * DQ + ch * 8);
    }
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      int e = tid + it * NT;
      if (!VEXACT) e = e < TI * VCH ? e : TI * VCH - 1;
      int r = e / VCH;
      const int ch = e % VCH;
      r = r < last ? r : last;
      vr[it] = *reinterpret_cast<const u32x4*>(vU + (size_t)(t0 + r) * D + ch * 8);
    }
  }
  // registers -> LDS, padding rows as zeros
  __device__ __forceinline__ void store(unsigned char* Ks, unsigned char* Vs, int tid) const {
    constexpr int KP = KPitch<DQ>::v, VP = VPitch<D>::v;
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < KIT; ++it) {
      const int e = tid + it * NT, r = e / KCH, ch = e % KCH;
      if (KEXACT || e < TI * KCH) *reinterpret_cast<u32x4*>(Ks + r * KP + ch * 16) = r < nvalid ? kr[it] : zero;
    }
#pragma unroll
    for (int it = 0; it < VIT; ++it) {
      const int e = tid + it * NT, r = e / VCH, ch = e % VCH;
      if (VEXACT || e < TI * VCH) *reinterpret_cast<u32x4*>(Vs + r * VP + ch * 16) = r < nvalid ? vr[it] : zero;
    }
  }
};

}  // namespace laser
