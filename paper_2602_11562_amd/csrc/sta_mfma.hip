// STA on the bf16 matrix cores (many candidates per user).
//
// Operation (Sec. 3.4.2 STA equation, global-score form of Sec. 3.5.1): for a user, the scores of all
// candidates against all history items are one [C x d_q].[d_q x L] contraction, the gated aggregation is a
// [C x L].[L x d] contraction whose accumulator is flushed at every segment boundary.
//
// Mapping. A workgroup owns (user, tile of 32*NW candidates, a run of consecutive segments); each of its NW
// waves owns 32 candidates (one MFMA column block) and keeps their queries in registers as the B operand for
// the whole run. History items are staged through LDS 64 at a time with coalesced 16-byte global loads shared
// by all waves; rows past the valid length (or past the end of the segment) are stored as zeros, so a padded
// item contributes gate(0) * 0 = 0 and needs no mask in the epilogue, and padding that holds NaN never reaches
// the arithmetic. With NBUF = 2 the loads of the next tile are issued before the current tile is computed and
// land in the other LDS buffer afterwards: one barrier per tile, memory latency behind the MFMA work.
//
// Both products are computed transposed so that nothing has to be shuffled between them:
//   Sc^T[item, cand] = K_tile . Q^T            v_mfma_f32_32x32x16_bf16, A = K rows from LDS (16 B per lane)
//   P^T = bf16(sigmoid(Sc^T / gamma))          in the accumulator registers
//   acc^T[dcol, cand] += V_tile^T . P^T        A = V^T via the LDS transpose load, B = P^T as it already sits
// The accumulator layout of the first product (lane = candidate, registers = items 8(r/4)+4(lane/32)+r%4) is,
// per 16-item step, exactly a B operand whose k-slots are the items {4h..4h+3, 8+4h..8+4h+3}; V^T is fetched
// with the same slot order by two ds_read_b64_tr_b16 per step.
//
// H' leaves through a wave-private LDS patch, 64 value columns at a time, so that global stores are whole
// 128-byte row pieces instead of 8-byte fragments of 32 different rows.
#include <cstdlib>

#include "laser_internal.h"

namespace laser {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
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

template <int DQ, int D, int NW, int NBUF>
__global__ __launch_bounds__(64 * NW) void sta_mfma_kernel(const unsigned short* __restrict__ q,
                                                           const unsigned short* __restrict__ k,
                                                           const unsigned short* __restrict__ v,
                                                           const int32_t* __restrict__ lens, int C, int L, int w,
                                                           int S, int spw, int ctiles, int sruns,
                                                           float neg_scale_log2e, unsigned short* __restrict__ seg_out,
                                                           int32_t* __restrict__ seg_cnt) {
  constexpr int KP = KPitch<DQ>::v, VP = VPitch<D>::v;
  constexpr int NT = 64 * NW;
  constexpr int KSTEPS = DQ / 16, DB = D / 32;
  constexpr int OP = OPitch<D>::v;
  constexpr int KBYTES = TI * KP, VBYTES = TI * VP, OBYTES = CW * OP;
  __shared__ __attribute__((aligned(16))) unsigned char smem[NBUF * (KBYTES + VBYTES) + NW * OBYTES];

  int bid = blockIdx.x;
  const int srun = bid % sruns;
  bid /= sruns;
  const int ct = bid % ctiles;
  const int u = bid / ctiles;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;
  const int cbase = ct * (CW * NW) + wave * CW;     // first candidate of this wave
  const int n = valid_len(lens, u, L);
  if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, NT);
  unsigned char* opatch = smem + NBUF * (KBYTES + VBYTES) + wave * OBYTES;

  // queries: B operand of the score product, lane = candidate, 8 consecutive d_q elements per k-step half
  bf16x8 qreg[KSTEPS];
  {
    const int c = cbase + l32;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (c < C) raw = *reinterpret_cast<const u32x4*>(q + ((size_t)u * C + c) * DQ + ks * 16 + h * 8);
      qreg[ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  const unsigned short* kU = k + (size_t)u * L * DQ;
  const unsigned short* vU = v + (size_t)u * L * D;

  const int seg_lo = srun * spw;
  const int seg_hi = (seg_lo + spw) < S ? (seg_lo + spw) : S;
  // valid items are a prefix of the history, so the non-empty segments of the run are a prefix of the run
  int seg_ne = seg_lo;
  while (seg_ne < seg_hi && seg_ne * w < n) ++seg_ne;

  // tile cursor over the non-empty segments of the run: (segment, first item, end of valid items in the segment)
  auto seg_end = [&](int i) {
    int e = i * w + w;
    if (e > L) e = L;
    if (e > n) e = n;
    return e;
  };

  Stage<DQ, D, NT> st;
  int ci = seg_lo, ct0 = seg_lo * w, chi = seg_ne > seg_lo ? seg_end(seg_lo) : 0;   // current tile
  int buf = 0;
  if (seg_ne > seg_lo) {
    st.load(kU, vU, ct0, chi, tid);
    st.store(smem, smem + KBYTES, tid);
  }
  __syncthreads();

  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.0f;

  // patch -> global: 16 lanes x 16 B = one row; LDS operations of a wave execute in order, so the rows written
  // by this wave above are visible to its own reads here without a barrier
  constexpr int LPR = D / 8, RPI = 64 / LPR;   // lanes per row, rows per instruction
  auto flush = [&](int seg) {
#pragma unroll
    for (int it = 0; it < CW / RPI; ++it) {
      const int row = it * RPI + lane / LPR;
      const u32x4 val = *reinterpret_cast<const u32x4*>(opatch + row * OP + (lane % LPR) * 16);
      const int cr = cbase + row;
      if (cr < C)
        *reinterpret_cast<u32x4*>(seg_out + (((size_t)u * C + cr) * S + seg) * D + (lane % LPR) * 8) = val;
    }
  };
  int out_seg = -1;

  while (ci < seg_ne) {
    // next tile in the run (same segment, or the first tile of the next non-empty segment)
    int ni = ci, nt0 = ct0 + TI, nhi = chi;
    if (nt0 >= chi) {
      ni = ci + 1;
      nt0 = ni * w;
      nhi = ni < seg_ne ? seg_end(ni) : 0;
    }
    const bool has_next = ni < seg_ne;
    unsigned char* Ks = smem + buf * (KBYTES + VBYTES);
    unsigned char* Vs = Ks + KBYTES;
    // in flight during the MFMA work below; with no next tile the current one is read again (in bounds, unused)
    // so that the instruction stream stays free of branches around the loads
    if (NBUF == 2) st.load(kU, vU, has_next ? nt0 : ct0, has_next ? nhi : chi, tid);
    if (out_seg >= 0) {
      flush(out_seg);
      out_seg = -1;
    }

#pragma unroll
    for (int ib = 0; ib < TI / 32; ++ib) {
      if (ct0 + ib * 32 < chi) {   // uniform: otherwise the rest of the tile is padding
        // ---- Sc^T = K . Q^T for 32 items x 32 candidates
        bf16x8 ka[KSTEPS];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
          ka[ks] = *reinterpret_cast<const bf16x8*>(Ks + (ib * 32 + l32) * KP + (ks * 16 + h * 8) * 2);
        f32x16 sc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[ks], sc, 0, 0, 0);
        // ---- gates, rounded to bf16: they become the B operand of the second product as they sit
        bf16x8 p[2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int e = 0; e < 8; ++e) p[s][e] = (__bf16)gate(sc[s * 8 + e], neg_scale_log2e);
        // ---- acc^T += V^T . P^T
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          const int item0 = ib * 32 + s * 16 + h * 4;   // k-slots 0..3; slots 4..7 are 8 items further
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            // transpose load: lane i of a 16-lane group supplies the address of V[item0 + i/4][dc0 + 4 (i%4)]
            // and receives V[item0 + 0..3][dc0 + i]
            const int dc0 = db * 32 + (l32 & 16);
            const int i16 = lane & 15;
            const unsigned char* src = Vs + (item0 + (i16 >> 2)) * VP + (dc0 + 4 * (i16 & 3)) * 2;
            const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
            const s16x4 hi4 =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 8 * VP));
            const s16x8 both = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), p[s], acc[db], 0, 0, 0);
          }
        }
      }
    }

    // the prefetched tile goes to the other buffer first (its loads were issued a whole tile ago), then the
    // finished segment is written out; those global stores drain during the next tile
    if (NBUF == 2 && has_next)
      st.store(smem + (buf ^ 1) * (KBYTES + VBYTES), smem + (buf ^ 1) * (KBYTES + VBYTES) + KBYTES, tid);
    if (ni != ci) {
      // ---- segment finished: H'[u, c, ci, :] is parked in the wave-private patch as bf16 rows; it is written
      // to global memory at the top of the next step, behind that step's prefetch loads, so that waiting for
      // the prefetch never has to wait for these stores first
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[db][g * 4 + e];
          *reinterpret_cast<u32x2*>(opatch + l32 * OP + (db * 32 + g * 8 + h * 4) * 2) = __builtin_bit_cast(u32x2, o);
        }
      out_seg = ci;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.0f;
    }

    if (NBUF == 2) {
      __syncthreads();
      buf ^= 1;
    } else {
      __syncthreads();   // everyone is done reading the tile
      if (has_next) {
        st.load(kU, vU, nt0, nhi, tid);
        st.store(smem, smem + KBYTES, tid);
      }
      __syncthreads();
    }
    ci = ni;
    ct0 = nt0;
    chi = nhi;
  }

  if (out_seg >= 0) flush(out_seg);

  // empty segments of the run: exact zeros, 16 bytes per thread
  if (seg_ne < seg_hi) {
    const int ncand = (C - ct * (CW * NW)) < CW * NW ? (C - ct * (CW * NW)) : CW * NW;
    const int per_row = D / 8;
    const int rows = ncand * (seg_hi - seg_ne);
    for (int e = tid; e < rows * per_row; e += NT) {
      const int row = e / per_row, ch = e - row * per_row;
      const int cc = row / (seg_hi - seg_ne), ii = seg_ne + row % (seg_hi - seg_ne);
      *reinterpret_cast<u32x4*>(seg_out + (((size_t)u * C + ct * (CW * NW) + cc) * S + ii) * D + ch * 8) =
          u32x4{0u, 0u, 0u, 0u};
    }
  }
}

// ------------------------------------------------------------------------------------------ pipelined form
// Same mapping and arithmetic as above, with the two 32-item blocks of a tile software-pipelined inside each
// wave so that the sigmoid work (VALU, transcendental unit) of one block runs in the shadow of the MFMAs of
// another:
//   phase A   Sc(b1) = K.Q^T            ||  P(b0) = sigmoid(Sc(b0))
//   phase B   acc += V^T(b0).P(b0)      ||  P(b1) = sigmoid(Sc(b1))
//   phase C   acc += V^T(b1).P(b1)          then the prefetched tile goes to the other LDS buffer
//   barrier
//   phase D   Sc(b0 of the next tile) = K.Q^T
// Every tile is computed in full (its padding rows are zeros in LDS), so the phases are straight-line code.
template <int DQ, int D, int NW>
__global__ __launch_bounds__(64 * NW) void sta_mfma_pipe_kernel(const unsigned short* __restrict__ q,
                                                                const unsigned short* __restrict__ k,
                                                                const unsigned short* __restrict__ v,
                                                                const int32_t* __restrict__ lens, int C, int L,
                                                                int w, int S, int spw, int ctiles, int sruns,
                                                                float neg_scale_log2e,
                                                                unsigned short* __restrict__ seg_out,
                                                                int32_t* __restrict__ seg_cnt) {
  constexpr int KP = KPitch<DQ>::v, VP = VPitch<D>::v;
  constexpr int NT = 64 * NW;
  constexpr int KSTEPS = DQ / 16, DB = D / 32;
  constexpr int OP = OPitch<D>::v;
  constexpr int KBYTES = TI * KP, VBYTES = TI * VP, OBYTES = CW * OP;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * (KBYTES + VBYTES) + NW * OBYTES];

  int bid = blockIdx.x;
  const int srun = bid % sruns;
  bid /= sruns;
  const int ct = bid % ctiles;
  const int u = bid / ctiles;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;
  const int cbase = ct * (CW * NW) + wave * CW;
  const int n = valid_len(lens, u, L);
  if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, NT);
  unsigned char* opatch = smem + 2 * (KBYTES + VBYTES) + wave * OBYTES;

  bf16x8 qreg[KSTEPS];
  {
    const int c = cbase + l32;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (c < C) raw = *reinterpret_cast<const u32x4*>(q + ((size_t)u * C + c) * DQ + ks * 16 + h * 8);
      qreg[ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  const unsigned short* kU = k + (size_t)u * L * DQ;
  const unsigned short* vU = v + (size_t)u * L * D;

  const int seg_lo = srun * spw;
  const int seg_hi = (seg_lo + spw) < S ? (seg_lo + spw) : S;
  int seg_ne = seg_lo;
  while (seg_ne < seg_hi && seg_ne * w < n) ++seg_ne;
  auto seg_end = [&](int i) {
    int e = i * w + w;
    if (e > L) e = L;
    if (e > n) e = n;
    return e;
  };

  // per-lane LDS offsets that do not change: K operand row (block 0) and the transpose-load source
  const int koff = l32 * KP + h * 16;
  const int voff = (h * 4 + ((lane & 15) >> 2)) * VP + ((l32 & 16) + 4 * (lane & 3)) * 2;

  auto score = [&](const unsigned char* Ks, int ib) {   // Sc^T of block ib: 32 items x 32 candidates
    f32x16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(Ks + ib * 32 * KP + koff + ks * 32);
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sc, 0, 0, 0);
    }
    return sc;
  };
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.0f;
  auto aggregate = [&](const unsigned char* Vs, int ib, const bf16x8 (&p)[2]) {   // acc^T += V^T . P^T
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const unsigned char* src = Vs + (ib * 32 + s * 16) * VP + voff + db * 64;
        const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
        const s16x4 hi4 =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 8 * VP));
        const s16x8 both = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), p[s], acc[db], 0, 0, 0);
      }
  };
  auto gates = [&](const f32x16& sc, bf16x8 (&p)[2]) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) p[s][e] = (__bf16)gate(sc[s * 8 + e], neg_scale_log2e);
  };

  constexpr int LPR = D / 8, RPI = 64 / LPR;
  auto flush = [&](int seg) {
#pragma unroll
    for (int it = 0; it < CW / RPI; ++it) {
      const int row = it * RPI + lane / LPR;
      const u32x4 val = *reinterpret_cast<const u32x4*>(opatch + row * OP + (lane % LPR) * 16);
      const int cr = cbase + row;
      if (cr < C)
        *reinterpret_cast<u32x4*>(seg_out + (((size_t)u * C + cr) * S + seg) * D + (lane % LPR) * 8) = val;
    }
  };

  Stage<DQ, D, NT> st;
  int ci = seg_lo, ct0 = seg_lo * w, chi = seg_ne > seg_lo ? seg_end(seg_lo) : 0;
  int buf = 0, out_seg = -1;
  f32x16 sc0;
  if (seg_ne > seg_lo) {
    st.load(kU, vU, ct0, chi, tid);
    st.store(smem, smem + KBYTES, tid);
  }
  __syncthreads();
  if (seg_ne > seg_lo) sc0 = score(smem, 0);

  while (ci < seg_ne) {
    int ni = ci, nt0 = ct0 + TI, nhi = chi;
    if (nt0 >= chi) {
      ni = ci + 1;
      nt0 = ni * w;
      nhi = ni < seg_ne ? seg_end(ni) : 0;
    }
    const bool has_next = ni < seg_ne;
    const unsigned char* Ks = smem + buf * (KBYTES + VBYTES);
    const unsigned char* Vs = Ks + KBYTES;
    unsigned char* nKs = smem + (buf ^ 1) * (KBYTES + VBYTES);

    st.load(kU, vU, has_next ? nt0 : ct0, has_next ? nhi : chi, tid);   // lands during phases A-C
    if (out_seg >= 0) {
      flush(out_seg);
      out_seg = -1;
    }

    bf16x8 p0[2], p1[2];
    const f32x16 sc1 = score(Ks, 1);   // phase A
    gates(sc0, p0);
    aggregate(Vs, 0, p0);              // phase B
    gates(sc1, p1);
    aggregate(Vs, 1, p1);              // phase C
    if (has_next) st.store(nKs, nKs + KBYTES, tid);

    if (ni != ci) {   // segment finished: park H' rows in the patch, stored to global at the top of the next step
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[db][g * 4 + e];
          *reinterpret_cast<u32x2*>(opatch + l32 * OP + (db * 32 + g * 8 + h * 4) * 2) = __builtin_bit_cast(u32x2, o);
        }
      out_seg = ci;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[db][r] = 0.0f;
    }
    __syncthreads();
    buf ^= 1;
    if (has_next) sc0 = score(nKs, 0);   // phase D
    ci = ni;
    ct0 = nt0;
    chi = nhi;
  }
  if (out_seg >= 0) flush(out_seg);

  if (seg_ne < seg_hi) {   // empty segments of the run: exact zeros
    const int ncand = (C - ct * (CW * NW)) < CW * NW ? (C - ct * (CW * NW)) : CW * NW;
    const int per_row = D / 8;
    const int rows = ncand * (seg_hi - seg_ne);
    for (int e = tid; e < rows * per_row; e += NT) {
      const int row = e / per_row, ch = e - row * per_row;
      const int cc = row / (seg_hi - seg_ne), ii = seg_ne + row % (seg_hi - seg_ne);
      *reinterpret_cast<u32x4*>(seg_out + (((size_t)u * C + ct * (CW * NW) + cc) * S + ii) * D + ch * 8) =
          u32x4{0u, 0u, 0u, 0u};
    }
  }
}

// ------------------------------------------------------------------------------------------ host side
static int pick_nw(int C) { return C > 128 ? 8 : (C > 64 ? 4 : (C > 32 ? 2 : 1)); }

bool sta_mfma_supports(const StaArgs& a) {
  if (a.dt != LASER_BF16) return false;
  if (!(a.d_q == 32 || a.d_q == 64 || a.d_q == 128)) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  if (a.C < 9) return false;   // fewer candidates than that: the streaming kernel's range
  const int nw = pick_nw(a.C);
  const long long ctiles = (a.C + CW * nw - 1) / (CW * nw);
  return (long long)a.U * ctiles * a.S <= 0x7fffffffLL;
}

template <int DQ, int D, int NW, int NBUF>
static void launch_one(const StaArgs& a, int spw, int ctiles, int sruns, float nsl) {
  const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
  hipLaunchKernelGGL((sta_mfma_kernel<DQ, D, NW, NBUF>), dim3(blocks), dim3(64 * NW), 0, a.stream,
                     (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens, a.C,
                     a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
}

template <int DQ, int D>
static void launch_nw(const StaArgs& a, int nw, int spw, int ctiles, int sruns, float nsl) {
  // eight waves fill a compute unit on their own and prefetch through a second LDS buffer; smaller workgroups
  // overlap memory and MFMA work across the several workgroups that share a compute unit
  if (nw == 8) {
    const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
    hipLaunchKernelGGL((sta_mfma_pipe_kernel<DQ, D, 8>), dim3(blocks), dim3(512), 0, a.stream,
                       (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                       a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
  }
  else if (nw == 4) launch_one<DQ, D, 4, 1>(a, spw, ctiles, sruns, nsl);
  else if (nw == 2) launch_one<DQ, D, 2, 1>(a, spw, ctiles, sruns, nsl);
  else launch_one<DQ, D, 1, 1>(a, spw, ctiles, sruns, nsl);
}

laser_status sta_mfma_launch(const StaArgs& a) {
  if (!sta_mfma_supports(a)) return LASER_ERR_UNSUPPORTED;
  const int nw = pick_nw(a.C);
  const int ctiles = (a.C + CW * nw - 1) / (CW * nw);
  // consecutive segments per workgroup (they share the query registers and the prefetch pipeline): as many as
  // still leave one eight-wave workgroup, or two smaller ones, per compute unit
  const long long want = nw == 8 ? 256 : 512;
  int spw = 1;
  while (spw < 8 && (long long)a.U * ctiles * ((a.S + 2 * spw - 1) / (2 * spw)) >= want) spw *= 2;
  if (const char* e = getenv("LASER_STA_SPW")) {   // tuning override
    const int vv = atoi(e);
    if (vv >= 1 && vv <= 64) spw = vv;
  }
  const int sruns = (a.S + spw - 1) / spw;
  const float nsl = -1.4426950408889634f / a.gamma;
  const int key = a.d_q * 1000 + a.d;
  switch (key) {
    case 32064: launch_nw<32, 64>(a, nw, spw, ctiles, sruns, nsl); break;
    case 32128: launch_nw<32, 128>(a, nw, spw, ctiles, sruns, nsl); break;
    case 64064: launch_nw<64, 64>(a, nw, spw, ctiles, sruns, nsl); break;
    case 64128: launch_nw<64, 128>(a, nw, spw, ctiles, sruns, nsl); break;
    case 128064: launch_nw<128, 64>(a, nw, spw, ctiles, sruns, nsl); break;
    case 128128: launch_nw<128, 128>(a, nw, spw, ctiles, sruns, nsl); break;
    default: return LASER_ERR_UNSUPPORTED;
  }
  return launch_status();
}

}  // namespace laser
