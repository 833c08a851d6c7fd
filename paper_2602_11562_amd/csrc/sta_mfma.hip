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
#include <type_traits>

#include "laser_internal.h"
#include "sta_mfma_tile.h"

namespace laser {

// HEADS > 1 (Sec. 4.1.2): head h owns the h-th run of d_q / HEADS columns of q and k, a whole number of 16-wide
// k-steps, and of d / HEADS columns of v and H', a whole number of 32-column blocks; one score block and one gate
// per head, and every column block is aggregated with its own head's gates.
// SOFTMAX (the ablation of Sec. 4.4.1): the gates of a segment are a softmax over its valid items, per candidate and
// head, taken online: a running maximum and denominator per lane (the two lanes of a candidate agree on the maximum
// after every block and add their denominators at the end of the segment), the sums rescaled when the maximum
// moves. Zero-filled padding rows would count in the denominator, so their scores are masked in a partial block.
template <int DQ, int D, int NW, int NBUF, int HEADS = 1, bool SOFTMAX = false>
__global__ __launch_bounds__(64 * NW) void sta_mfma_kernel(const unsigned short* __restrict__ q,
                                                           const unsigned short* __restrict__ k,
                                                           const unsigned short* __restrict__ v,
                                                           const int32_t* __restrict__ lens,
                                                           const int32_t* __restrict__ cand_off, int P, int C_all,
                                                           int L, int w,
                                                           int S, int spw, int ctiles, int sruns,
                                                           float neg_scale_log2e, unsigned short* __restrict__ seg_out,
                                                           int32_t* __restrict__ seg_cnt) {
  constexpr int KP = KPitch<DQ>::v, VP = VPitch<D>::v;
  constexpr int NT = 64 * NW;
  constexpr int KSTEPS = DQ / 16, DB = D / 32;
  constexpr int KH = KSTEPS / HEADS, DBH = DB / HEADS;   // k-steps and column blocks per head
  static_assert(KSTEPS % HEADS == 0 && DB % HEADS == 0, "heads must own whole k-steps and whole column blocks");
  constexpr int OP = OPitch<D>::v;
  constexpr int KBYTES = TI * KP, VBYTES = TI * VP, OBYTES = CW * OP;
  __shared__ __attribute__((aligned(16))) unsigned char smem[NBUF * (KBYTES + VBYTES) + NW * OBYTES];

  int bid = blockIdx.x;
  const int srun = bid % sruns;
  bid /= sruns;
  const int ct = bid % ctiles;
  const int u = bid / ctiles;
  const CandRange crange = cand_range(cand_off, u, C_all, P);
  const int C = crange.count;               // this user's candidates
  const size_t pb = (size_t)crange.first;   // and the index of their first pair
  if (ct * (CW * NW) >= C) {   // a candidate tile past this user's count: nothing to do (the first still writes the counts)
    if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, valid_len(lens, u, L), L, w, S, threadIdx.x, 64 * NW);
    return;
  }

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
      if (c < C) raw = *reinterpret_cast<const u32x4*>(q + (pb + c) * DQ + ks * 16 + h * 8);
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

  constexpr float SM_NEG = -1e30f;
  float sm_m[HEADS], sm_l[HEADS];
#pragma unroll
  for (int hd = 0; hd < HEADS; ++hd) {
    sm_m[hd] = SM_NEG;
    sm_l[hd] = 0.0f;
  }
  auto both_halves = [](float x, bool take_max) {   // x combined with the value of lane ^ 32 (v_permlane32_swap)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float a0 = __uint_as_float(r[0]), a1 = __uint_as_float(r[1]);
    return take_max ? fmaxf(a0, a1) : a0 + a1;
  };

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
        *reinterpret_cast<u32x4*>(seg_out + ((pb + cr) * S + seg) * D + (lane % LPR) * 8) = val;
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
        // ---- gates, rounded to bf16: they become the B operand of the second product as they sit
        bf16x8 p[HEADS][2];
#pragma unroll
        for (int hd = 0; hd < HEADS; ++hd) {
          f32x16 sc;
#pragma unroll
          for (int r = 0; r < 16; ++r) sc[r] = 0.0f;
#pragma unroll
          for (int ks = hd * KH; ks < (hd + 1) * KH; ++ks)
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[ks], sc, 0, 0, 0);
          if constexpr (SOFTMAX) {
            const float sl = -neg_scale_log2e;            // log2(e) / gamma
            const int left = chi - ct0 - ib * 32;         // valid items from the start of this block (>= 1)
            float x[16], bm = SM_NEG;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              x[r] = sc[r] * sl;
              if (left < 32 && 8 * (r >> 2) + 4 * h + (r & 3) >= left) x[r] = SM_NEG;
              bm = fmaxf(bm, x[r]);
            }
            bm = both_halves(bm, true);
            const float m_new = fmaxf(sm_m[hd], bm);
            const float corr = __builtin_amdgcn_exp2f(sm_m[hd] - m_new);   // 0 at the first block of a segment
            float ps = 0.0f;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const float pe = __builtin_amdgcn_exp2f(x[s * 8 + e] - m_new);
                ps += pe;
                p[hd][s][e] = (__bf16)pe;
              }
            sm_l[hd] = fmaf(sm_l[hd], corr, ps);
            sm_m[hd] = m_new;
#pragma unroll
            for (int db = hd * DBH; db < (hd + 1) * DBH; ++db)
#pragma unroll
              for (int r = 0; r < 16; ++r) acc[db][r] *= corr;
          } else {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
              for (int e = 0; e < 8; ++e) p[hd][s][e] = (__bf16)gate(sc[s * 8 + e], neg_scale_log2e);
          }
        }
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
            acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), p[db / DBH][s], acc[db], 0, 0, 0);
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
      if constexpr (SOFTMAX) {   // divide by the denominator (the segment holds a valid item: it is positive)
#pragma unroll
        for (int hd = 0; hd < HEADS; ++hd) {
          const float inv = 1.0f / both_halves(sm_l[hd], false);
#pragma unroll
          for (int db = hd * DBH; db < (hd + 1) * DBH; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][r] *= inv;
          sm_m[hd] = SM_NEG;
          sm_l[hd] = 0.0f;
        }
      }
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
      *reinterpret_cast<u32x4*>(seg_out + ((pb + ct * (CW * NW) + cc) * S + ii) * D + ch * 8) =
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
                                                                const int32_t* __restrict__ lens,
                                                                const int32_t* __restrict__ cand_off, int P, int C_all,
                                                                int L,
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
  const CandRange crange = cand_range(cand_off, u, C_all, P);
  const int C = crange.count;               // this user's candidates
  const size_t pb = (size_t)crange.first;   // and the index of their first pair
  if (ct * (CW * NW) >= C) {   // a candidate tile past this user's count: nothing to do (the first still writes the counts)
    if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, valid_len(lens, u, L), L, w, S, threadIdx.x, 64 * NW);
    return;
  }

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
      if (c < C) raw = *reinterpret_cast<const u32x4*>(q + (pb + c) * DQ + ks * 16 + h * 8);
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
        *reinterpret_cast<u32x4*>(seg_out + ((pb + cr) * S + seg) * D + (lane % LPR) * 8) = val;
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
      *reinterpret_cast<u32x4*>(seg_out + ((pb + ct * (CW * NW) + cc) * S + ii) * D + ch * 8) =
          u32x4{0u, 0u, 0u, 0u};
    }
  }
}

// ------------------------------------------------------------------------------------------ direct-to-LDS form
// d_q = d = 128 and more than 128 candidates per user (the benchmark shape). Same arithmetic and wave mapping as
// the pipelined form; what changes is how history reaches LDS and how little vector-ALU work surrounds the matrix
// instructions (a MFMA blocks VALU issue of its SIMD for about half of its own duration, and the gates already
// need more VALU slots than the MFMAs leave free, so every address computation removed from the loop counts):
//  * tiles of 32 items are fetched with global_load_lds_dwordx4 (each lane names a 16-byte global chunk, the 64
//    chunks of a wave land contiguously in LDS), so no register or VALU work is spent on staging; the global
//    address is a scalar tile base plus a per-lane offset that never changes. Five LDS buffers, up to four tiles
//    requested ahead. The queries take the same road (through the wave's output patch);
//  * rows are unpadded; bank conflicts are avoided by an XOR swizzle of the 16-byte chunk index that the fetching
//    lane applies when it picks its global chunk: K chunk c of row r sits at position c ^ (r & 15), V chunk c at
//    c ^ 4 (r & 3) (conflict-free for the 16-rows-by-16-bytes operand reads and for the 4-rows-by-64-bytes
//    transpose loads respectively);
//  * rows past the valid length cannot be zero-filled by this path: they are fetched from the last valid row and
//    their gates are forced to 0 in the (rare) partial tile;
//  * fetches and H' stores are inline assembly without outputs. The compiler's wait-count pass does not see
//    them, so it never waits for a fetch in flight (a visible load or store would make it wait for everything
//    outstanding at the next use of a register it cannot prove idle); completion is awaited explicitly with
//    s_waitcnt vmcnt(n), n = the number of younger fetches allowed to stay outstanding. Operand reads from LDS
//    are ordinary loads whose waits the compiler places itself;
//  * H' rows leave with the non-temporal hint when the launch stands alone, and cacheable when the caller is the
//    whole path, whose next launch streams them back (measured: about 3 us of the step).
constexpr int DT_TI = 32, DT_NBUF = 5, DT_AHEAD = 4;

// 16 bytes per lane from global (uniform base + per-lane byte offset) to LDS (uniform address + 16 * lane)
__device__ __forceinline__ void dma16(const void* gbase, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(lds_addr), "v"(voff), "s"(gbase)
               : "memory");
}

constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// waits until at most n (rounded down to even, at most 30) of this wave's vector-memory operations are outstanding
__device__ __forceinline__ void wait_vm(int n) {
  switch (n >> 1) {
#define LASER_VM_CASE(i) case i: __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * i)); break;
    LASER_VM_CASE(1) LASER_VM_CASE(2) LASER_VM_CASE(3) LASER_VM_CASE(4) LASER_VM_CASE(5) LASER_VM_CASE(6)
    LASER_VM_CASE(7) LASER_VM_CASE(8) LASER_VM_CASE(9) LASER_VM_CASE(10) LASER_VM_CASE(11) LASER_VM_CASE(12)
    LASER_VM_CASE(13) LASER_VM_CASE(14)
#undef LASER_VM_CASE
    default:
      if (n >= 30) __builtin_amdgcn_s_waitcnt(vmcnt_imm(30));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  }
}

typedef __attribute__((address_space(3))) unsigned char* lds_bytes;
// The compiler re-associates "lane offset + buffer offset + constant" into one three-operand add per read; hiding
// the sum of the first two behind an empty asm leaves it "register + constant", which becomes the read's
// immediate offset.
__device__ __forceinline__ lds_bytes lds_at(unsigned addr) { return (lds_bytes)(size_t)addr; }
__device__ __forceinline__ lds_bytes lds_opaque(unsigned addr) {
  asm volatile("" : "+v"(addr));
  return lds_at(addr);
}
__device__ __forceinline__ bf16x8 lds_read16(lds_bytes p) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(p);
}
// items k0..k0+3 and k0+8..k0+11 of one value column per lane (see the file header); p addresses row k0
__device__ __forceinline__ bf16x8 lds_read_tr(lds_bytes p) {
  const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 2048));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Instruction J (0..71) of the 16 gates of a lane, in dependency order per half of 8: scale (8), exp2 (8), 1 + (8),
// reciprocal (8), round pairs to bf16 (4). The scores are transformed in place.
template <int J>
__device__ __forceinline__ void gate_step(f32x16& sc, bf16x8& p0, bf16x8& p1, float nsl) {
  constexpr int half = J / 36, r = J % 36, stage = r / 8, e = r % 8, i = half * 8 + e;
  if constexpr (stage == 0) sc[i] *= nsl;
  else if constexpr (stage == 1) sc[i] = __builtin_amdgcn_exp2f(sc[i]);
  else if constexpr (stage == 2) sc[i] += 1.0f;
  else if constexpr (stage == 3) sc[i] = __builtin_amdgcn_rcpf(sc[i]);
  else {
    constexpr int a0 = half * 8 + 2 * e;
    if constexpr (half == 0) { p0[2 * e] = (__bf16)sc[a0]; p0[2 * e + 1] = (__bf16)sc[a0 + 1]; }
    else { p1[2 * e] = (__bf16)sc[a0]; p1[2 * e + 1] = (__bf16)sc[a0 + 1]; }
  }
}
template <int J0>
__device__ __forceinline__ void gate_steps6(f32x16& sc, bf16x8& p0, bf16x8& p1, float nsl) {
  gate_step<J0>(sc, p0, p1, nsl);
  gate_step<J0 + 1>(sc, p0, p1, nsl);
  gate_step<J0 + 2>(sc, p0, p1, nsl);
  gate_step<J0 + 3>(sc, p0, p1, nsl);
  gate_step<J0 + 4>(sc, p0, p1, nsl);
  gate_step<J0 + 5>(sc, p0, p1, nsl);
}

// Barrier without the fence of __syncthreads(): the compiler neither waits for the wave's outstanding LDS reads
// (they are awaited where their registers are used) nor moves memory operations across it.
__device__ __forceinline__ void bare_barrier() { asm volatile("s_barrier" ::: "memory"); }

// NT: H' rows leave with the non-temporal hint (nobody reads them soon) or cacheable (the whole path: the next
// launch streams them back)
template <int NW, bool NTS>
__global__ __launch_bounds__(64 * NW) void sta_mfma_dma_kernel(const unsigned short* __restrict__ q,
                                                               const unsigned short* __restrict__ k,
                                                               const unsigned short* __restrict__ v,
                                                               const int32_t* __restrict__ lens,
                                                           const int32_t* __restrict__ cand_off, int P, int C_all,
                                                           int L, int w,
                                                               int S, int spw, int ctiles, int sruns,
                                                               float neg_scale_log2e,
                                                               unsigned short* __restrict__ seg_out,
                                                               int32_t* __restrict__ seg_cnt) {
  constexpr int DQ = 128, D = 128, KSTEPS = DQ / 16, DB = D / 32;
  static_assert(DB == 4 && KSTEPS == 8, "operand reads below are written out for d_q = d = 128");
  static_assert((16 / NW) % 2 == 0, "wait_vm counts in steps of two");
  constexpr int NT = 64 * NW;
  constexpr int ROWB = 256;          // bytes per K row and per V row
  constexpr int KB = DT_TI * ROWB, VB = DT_TI * ROWB, TB = KB + VB;
  constexpr int OP = OPitch<D>::v, OBYTES = CW * OP;
  constexpr int IPW = 8 / NW;        // 1 KB fetch groups per wave per matrix per tile (a tile has 8 of each)
  constexpr int OPT = 2 * IPW;       // fetch instructions per wave per tile
  __shared__ __attribute__((aligned(1024))) unsigned char smem[DT_NBUF * TB + NW * OBYTES];

  // Workgroups are dealt to the eight XCDs round-robin by index; renumber them so that each XCD gets a contiguous
  // range: the workgroups that share a user's queries then share an L2 as well
  int bid = blockIdx.x;
  if (gridDim.x % 8 == 0) bid = (bid % 8) * (gridDim.x / 8) + bid / 8;
  const int srun = bid % sruns;
  bid /= sruns;
  const int ct = bid % ctiles;
  const int u = bid / ctiles;
  const CandRange crange = cand_range(cand_off, u, C_all, P);
  const int C = crange.count;               // this user's candidates
  const size_t pb = (size_t)crange.first;   // and the index of their first pair
  if (ct * (CW * NW) >= C) {   // a candidate tile past this user's count: nothing to do (the first still writes the counts)
    if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, valid_len(lens, u, L), L, w, S, threadIdx.x, 64 * NW);
    return;
  }

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: fetch addresses and cursors stay scalar
  const int l32 = lane & 31, h = lane >> 5;
  const int cbase = ct * (CW * NW) + wave * CW;
  unsigned char* opatch = smem + DT_NBUF * TB + wave * OBYTES;
  const unsigned lds_base = __builtin_amdgcn_readfirstlane(
      (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem);

  // Queries first, before anything that depends on the valid length: the wave's 32 rows (8 KB, K swizzle) are
  // fetched into its output patch, which is idle until the first segment ends, and read into registers once.
  // Rows past the last candidate repeat it (never stored).
  const int frow = lane >> 4, fpos = lane & 15;
  const unsigned qlds = lds_base + DT_NBUF * TB + wave * OBYTES;
  {
    const unsigned char* qU = reinterpret_cast<const unsigned char*>(q + pb * DQ);
#pragma unroll
    for (int j = 0; j < CW / 4; ++j) {
      const int row = j * 4 + frow;
      const int c = cbase + row < C ? cbase + row : C - 1;
      dma16(qU, (unsigned)c * ROWB + ((fpos ^ (row & 15)) << 4), qlds + j * 1024);
    }
  }
  const unsigned char* kU = reinterpret_cast<const unsigned char*>(k + (size_t)u * L * DQ);
  const unsigned char* vU = reinterpret_cast<const unsigned char*>(v + (size_t)u * L * D);
  const int seg_lo = srun * spw;

  // ---- fetch side: this wave moves rows 4 g .. 4 g + 3 of every tile, g = wave * IPW + j
  unsigned fk[IPW], fv[IPW];   // per-lane byte offsets inside a full tile (row and swizzled chunk)
#pragma unroll
  for (int j = 0; j < IPW; ++j) {
    const int row = (wave * IPW + j) * 4 + frow;
    fk[j] = row * ROWB + ((fpos ^ (row & 15)) << 4);
    fv[j] = row * ROWB + ((fpos ^ (4 * (row & 3))) << 4);
  }
  // The first tile of the run is requested before the valid length is known (the length is one more round trip
  // to memory, and nothing can be computed before this tile has landed): its 32 rows exist whenever they lie
  // inside the history, whatever they hold. If the length then says the tile is not a full one, the request is
  // simply made again the regular way, into the same buffer; it lands after this one (loads retire in order).
  const bool spec = seg_lo < S && w >= DT_TI && seg_lo * w + DT_TI <= L;
  if (spec) {
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
      const int g = wave * IPW + j;
      dma16(kU + (size_t)seg_lo * w * ROWB, fk[j], lds_base + g * 1024);
      dma16(vU + (size_t)seg_lo * w * ROWB, fv[j], lds_base + KB + g * 1024);
    }
  }
  const int n = __builtin_amdgcn_readfirstlane(valid_len(lens, u, L));

  const int seg_hi = (seg_lo + spw) < S ? (seg_lo + spw) : S;
  int seg_ne = seg_lo;
  while (seg_ne < seg_hi && seg_ne * w < n) ++seg_ne;
  const int item_end = n < L ? n : L;   // one past the user's last valid item
  auto seg_end = [&](int i) {
    const int e = i * w + w;
    return e < item_end ? e : item_end;
  };

  auto issue_tile = [&](int t0, int hi, int buf) {   // requires t0 < hi
    const unsigned char* kT = kU + (size_t)t0 * ROWB;
    const unsigned char* vT = vU + (size_t)t0 * ROWB;
    const unsigned dst = lds_base + buf * TB;
    if (hi - t0 >= DT_TI) {
#pragma unroll
      for (int j = 0; j < IPW; ++j) {
        const int g = wave * IPW + j;
        dma16(kT, fk[j], dst + g * 1024);
        dma16(vT, fv[j], dst + KB + g * 1024);
      }
    } else {   // partial tile: rows past the last valid one repeat it
      const int last = hi - t0 - 1;
#pragma unroll
      for (int j = 0; j < IPW; ++j) {
        const int g = wave * IPW + j;
        const int row = g * 4 + frow;
        const int back = row > last ? (row - last) * ROWB : 0;
        dma16(kT, fk[j] - back, dst + g * 1024);
        dma16(vT, fv[j] - back, dst + KB + g * 1024);
      }
    }
  };
  // tile cursor: (segment, first item, end of the segment's valid items); advance() moves to the next tile of the run
  struct Cur { int seg, t0, hi; };
  auto advance = [&](Cur c) {
    Cur o = c;
    o.t0 = c.t0 + DT_TI;
    if (o.t0 >= c.hi) {
      o.seg = c.seg + 1;
      o.t0 = o.seg * w;
      o.hi = o.seg < seg_ne ? seg_end(o.seg) : 0;
    }
    return o;
  };

  // ---- operand side (constant per lane): swizzled byte offsets inside a tile
  unsigned kofs[KSTEPS], vofs[DB];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) kofs[ks] = l32 * ROWB + (((2 * ks + h) ^ (l32 & 15)) << 4);
  {
    const int i16 = lane & 15;
    const int rr = h * 4 + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int c16 = db * 4 + 2 * (l32 >> 4) + ((i16 & 3) >> 1);
      vofs[db] = KB + rr * ROWB + ((c16 ^ (4 * (rr & 3))) << 4) + (i16 & 1) * 8;
    }
  }

  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.0f;

  // ---- output side: the patch is read back 16 bytes per lane, four rows per wave-wide store; the per-lane part
  // of the global address never changes, the rest is a scalar base
  constexpr int LPR = D / 8, RPI = 64 / LPR;
  const unsigned char* opr = opatch + (lane / LPR) * OP + (lane % LPR) * 16;
  const unsigned ooff = (unsigned)(lane / LPR) * (unsigned)S * (D * 2) + (lane % LPR) * 16;
  const unsigned ooff2 = ooff + (unsigned)RPI * (unsigned)S * (D * 2);   // the unit's second row group
  unsigned char* oU = reinterpret_cast<unsigned char*>(seg_out) + (pb + cbase) * S * (D * 2);
  const bool all_rows = cbase + CW <= C;
  // A finished segment leaves in FU units of two row groups (eight rows, 2 KB per wave), a few per step: all
  // waves of a compute unit storing whole patches in the same step saturate its store path for most of a step
  // while it idles in the others.
  constexpr int FU = CW / RPI / 2;
  const size_t unit_stride = (size_t)2 * RPI * S * (D * 2);   // bytes between the first rows of two units in H'
  // where the next unit of the parked segment comes from and goes to (set when a segment is parked, advanced per
  // unit: recomputed from the unit number in every step they cost a dozen scalar instructions)
  unsigned char* fl_dst = oU;
  const unsigned char* fl_src = opr;
  int fl_row = cbase + lane / LPR;
  auto flush_units = [&](int n) {   // the next n units of the parked segment
    // scalar work per unit is kept to two 64-bit additions: a wave issues one instruction every few cycles,
    // whatever its kind, and the other wave of the SIMD is at the same point of the same step
#pragma unroll 1
    for (int b = 0; b < n; ++b) {
      const u32x4 v0 = *reinterpret_cast<const u32x4*>(fl_src);
      const u32x4 v1 = *reinterpret_cast<const u32x4*>(fl_src + RPI * OP);
      // (the s_nop: a store of more than 8 bytes reads its data registers for two more cycles after issue; the
      // compiler pads its own stores against a following register write, but cannot see into this one)
      if (all_rows) {
        if (NTS) {
          asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" ::"v"(ooff), "v"(v0), "s"(fl_dst) : "memory");
          asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" ::"v"(ooff2), "v"(v1), "s"(fl_dst) : "memory");
        } else {
          asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(ooff), "v"(v0), "s"(fl_dst) : "memory");
          asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(ooff2), "v"(v1), "s"(fl_dst) : "memory");
        }
      } else {
        if (fl_row < C) {
          if (NTS) asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" ::"v"(ooff), "v"(v0), "s"(fl_dst) : "memory");
          else asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(ooff), "v"(v0), "s"(fl_dst) : "memory");
        }
        if (fl_row + RPI < C) {
          if (NTS) asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" ::"v"(ooff2), "v"(v1), "s"(fl_dst) : "memory");
          else asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(ooff2), "v"(v1), "s"(fl_dst) : "memory");
        }
      }
      fl_dst += unit_stride;
      fl_src += 2 * RPI * OP;
      fl_row += 2 * RPI;
    }
  };

  const bool any = seg_ne > seg_lo;
  Cur cur{seg_lo, seg_lo * w, any ? seg_end(seg_lo) : 0};   // tile being computed
  Cur fet = cur;                                             // next tile to fetch
  int fetched = 0, done = 0;                                 // tiles requested / tiles finished
  int fbuf = 0, cbuf = 0;                                    // their LDS buffers
  auto issue_next = [&]() {
    if (fet.seg < seg_ne) {
      issue_tile(fet.t0, fet.hi, fbuf);
      fet = advance(fet);
      ++fetched;
      fbuf = fbuf + 1 == DT_NBUF ? 0 : fbuf + 1;
    }
  };
  // Only fetches may be allowed to stay outstanding in a wait: loads retire in order among themselves but not
  // relative to stores, so with H' stores allowed for, the count would no longer say which operations are the
  // outstanding ones. wait_tile(x): this wave's share of tile x has landed (tiles are numbered in request order).
  auto wait_tile = [&](int x) {
    const int beyond = fetched - 1 - x;
    wait_vm(OPT * (beyond > 0 ? beyond : 0));
  };
  if (any) {
    if (spec && fet.hi - fet.t0 >= DT_TI) {   // the early request was the right one: count it
      fet = advance(fet);
      fetched = 1;
      fbuf = 1;
    }
#pragma unroll 1
    for (int a = fetched; a < 2; ++a) issue_next();
  }
  if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, NT);
  wait_tile(1);   // tiles 0 and 1, and the queries, which are older (with nothing requested: everything)
  // the other tiles of the head start are requested only now: in the first microseconds every workgroup of the
  // launch asks for its queries and first tiles at once, and what is asked for later arrives sooner
  if (any) {
#pragma unroll 1
    for (int a = fetched; a < DT_AHEAD; ++a) issue_next();
  }
  __syncthreads();

  bf16x8 qreg[KSTEPS], ka[KSTEPS], va[2][DB];
  auto read_k = [&](int buf) {
    const unsigned tb = lds_base + buf * TB;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) ka[ks] = lds_read16(lds_at(kofs[ks] + tb));
  };
  auto read_v = [&](int buf) {
    const unsigned tb = lds_base + buf * TB;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const lds_bytes a = lds_opaque(vofs[db] + tb);
      va[0][db] = lds_read_tr(a);
      va[1][db] = lds_read_tr(a + 4096);
    }
  };
  if (any) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) qreg[ks] = lds_read16(lds_at(kofs[ks] + qlds));
    read_k(0);
  }
  int out_seg = -1, out_units = 0;   // segment parked in the patch (-1: none) and how much of it has left

  // One step per tile, one barrier per step, software-pipelined inside the wave so that the matrix pipe always
  // has work while the vector ALU evaluates gates:
  //   scores(t+1) [MFMA]  alongside  gates(t) [VALU, on the scores computed one step earlier]
  //   aggregation(t) [MFMA]
  // Operand reads run one step ahead of their use: K(t+2) is requested once scores(t+1) has consumed the K
  // registers, V(t+1) once aggregation(t) has consumed the V registers, and they stay in flight across the
  // barrier (it carries no fence). When a wave reaches the barrier of step t it has consumed, hence received,
  // K(t) and V(t-1): after that barrier the buffer of tile t-1 is idle in all waves and takes the fetch of tile
  // t + NBUF - 1. The same barrier publishes tile t + 2, whose share every wave has awaited just before.
  auto scores = [&]() {
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    f32x16 sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qreg[0], zero, 0, 0, 0);
#pragma unroll
    for (int ks = 1; ks < KSTEPS; ++ks) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qreg[ks], sc, 0, 0, 0);
    return sc;
  };
  f32x16 scA, scB;   // scores of the tile in work and of the next one: the two swap roles every step (no copy)
  u32x4 p0, p1;   // gates of items 0..15 / 16..31 of the current tile, rounded to bf16 pairs: B operands of the
                  // aggregation
  if (any) {
    scA = scores();
    read_k(1);
    // gates of items 0..15 of the first tile, up to the rounding of the last pair (done by the first slot of
    // the loop, as for every later tile)
#pragma unroll
    for (int i = 0; i < 8; ++i) scA[i] = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(scA[i] * neg_scale_log2e));
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const bf16x2 c = {(__bf16)scA[2 * j], (__bf16)scA[2 * j + 1]};
      p0[j] = __builtin_bit_cast(unsigned, c);
    }
  }
  auto step = [&](f32x16& sc_cur, f32x16& sc_nxt) __attribute__((always_inline)) {
    const Cur nxt = advance(cur);
    const bool has_next = nxt.seg < seg_ne;
    const bool has_next2 = has_next && advance(nxt).seg < seg_ne;
    const int nbuf = cbuf + 1 == DT_NBUF ? 0 : cbuf + 1;
    const int nbuf2 = nbuf + 1 == DT_NBUF ? 0 : nbuf + 1;
    // tile done+2 has landed: at this point fetched <= done + 4, so at most one younger tile stays outstanding
    if (fetched - done >= 4) __builtin_amdgcn_s_waitcnt(vmcnt_imm(OPT));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    bare_barrier();
    if (wave < NW / 2) issue_next();

    // One path for every tile, written in issue order. A step issues 16 MFMAs per wave: the eight score MFMAs of
    // the next tile (A0..A7), then the eight aggregation MFMAs of this tile (B0..B7). The 72 gate instructions of
    // a tile (per lane: 16 x scale, exp2, +1, reciprocal; 8 x round a pair to bf16) are spread over 16 MFMAs so
    // that each MFMA hides four or five of them and at most two of the slow exp2/reciprocal ones (measured: a
    // MFMA hides 2 slow + 2..3 plain VALU instructions of the two waves of its SIMD completely, more than that
    // extends the slot): the gates of items 0..15 of tile t+1 ride behind B1..B7 of step t (their scores exist
    // since A7), those of items 16..31 of tile t behind A0..A7 of step t. Consumers sit at least one slot behind
    // an exp2 or reciprocal. Nothing may be moved across the slot borders. After the last tile the score MFMAs run
    // on whatever the K registers hold and their result is dropped; in a partial tile the gates of the rows past
    // the end (copies of the last valid row) are cleared after rounding.
    const int nvt = cur.hi - cur.t0;
    const bool first = cur.t0 == cur.seg * w;
    auto clear_past_end = [&](u32x4& bits, int half) {
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const int i0 = half * 16 + 8 * (e2 >> 1) + 4 * h + 2 * (e2 & 1);
        bits[e2] &= (i0 < nvt ? 0x0000ffffu : 0u) | (i0 + 1 < nvt ? 0xffff0000u : 0u);
      }
    };
    {
      const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
// every gate instruction is followed by an empty asm that takes its result: the compiler otherwise sinks the
// arithmetic towards its use in a later block and undoes the placement
#define LASER_PIN(X) asm volatile("" : "+v"(X));
#define GM(S, I) { float t_ = S[I] * neg_scale_log2e; LASER_PIN(t_) S[I] = t_; }
#define GE(S, I) { float t_ = __builtin_amdgcn_exp2f(S[I]); LASER_PIN(t_) S[I] = t_; }
#define GA(S, I) { float t_ = S[I] + 1.0f; LASER_PIN(t_) S[I] = t_; }
#define GR(S, I) { float t_ = __builtin_amdgcn_rcpf(S[I]); LASER_PIN(t_) S[I] = t_; }
#define GC(P, J, S, I) { bf16x2 c_ = {(__bf16)S[I], (__bf16)S[(I) + 1]}; unsigned t_ = __builtin_bit_cast(unsigned, c_); LASER_PIN(t_) P[J] = t_; }
#define LASER_SLOT(MFMA, OPS)                                                                                        \
  MFMA;                                                                                                              \
  __builtin_amdgcn_sched_barrier(0);                                                                                 \
  OPS                                                                                                                \
  __builtin_amdgcn_sched_barrier(0);
#define LASER_QK(I) sc_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[I], qreg[I], I == 0 ? zero : sc_nxt, 0, 0, 0)
      LASER_SLOT(LASER_QK(0), GC(p0, 3, sc_cur, 6) GM(sc_cur, 8) GM(sc_cur, 9) GM(sc_cur, 10) GM(sc_cur, 11) GE(sc_cur, 8) GE(sc_cur, 9))
      if (nvt < DT_TI) clear_past_end(p0, 0);
      LASER_SLOT(LASER_QK(1), GA(sc_cur, 8) GA(sc_cur, 9) GM(sc_cur, 12) GM(sc_cur, 13) GE(sc_cur, 10) GE(sc_cur, 11))
      // V of this tile, for the second half of this step. (Requested at the end of the previous step these reads
      // were the youngest in flight at the top of the step, and the LDS wait counter, which counts in order and
      // no further than 15, made every score MFMA wait for most of them.)
      read_v(cbuf);
      LASER_SLOT(LASER_QK(2), GA(sc_cur, 10) GA(sc_cur, 11) GR(sc_cur, 8) GR(sc_cur, 9))
      LASER_SLOT(LASER_QK(3), GM(sc_cur, 14) GM(sc_cur, 15) GC(p1, 0, sc_cur, 8) GE(sc_cur, 12) GE(sc_cur, 13))
      LASER_SLOT(LASER_QK(4), GA(sc_cur, 12) GA(sc_cur, 13) GR(sc_cur, 10) GR(sc_cur, 11))
      LASER_SLOT(LASER_QK(5), GC(p1, 1, sc_cur, 10) GE(sc_cur, 14) GE(sc_cur, 15))
      LASER_SLOT(LASER_QK(6), GA(sc_cur, 14) GA(sc_cur, 15) GR(sc_cur, 12) GR(sc_cur, 13))
      LASER_SLOT(LASER_QK(7), GC(p1, 2, sc_cur, 12) GR(sc_cur, 14) GR(sc_cur, 15))
#undef LASER_QK
      // The finished segment's rows leave here rather than right after the barrier: the patch reads and their
      // waits sit behind a branch, and ahead of the score MFMAs they made the compiler wait for every operand
      // read in flight. The stores still have most of a step to complete before the next fetch wait.
      if (out_seg >= 0) {   // an equal share in every step that is left before the patch is needed again
        const int steps_left = (int)((unsigned)(nvt + DT_TI - 1) / DT_TI);
        const int left = FU - out_units;   // n = ceil(left / steps_left), left <= FU = 4, without a division
        static_assert(FU == 4, "the share below is written out for four units");
        const int n = steps_left >= left ? 1 : (steps_left == 1 ? left : 2);
        flush_units(n);
        out_units += n;
        if (out_units == FU) out_seg = -1;
      }
      if (first) {   // first tile of a segment: the sums restart (in a branch of its own: two copies of the slots
                     // below, one starting from an inline zero, made the compiler shuffle registers at the join)
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = zero;
      }
#define LASER_PV0(I) acc[I] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[0][I], __builtin_bit_cast(bf16x8, p0), acc[I], 0, 0, 0)
      LASER_SLOT(LASER_PV0(0), GC(p1, 3, sc_cur, 14))
      LASER_SLOT(LASER_PV0(1), GM(sc_nxt, 0) GM(sc_nxt, 1) GM(sc_nxt, 2) GM(sc_nxt, 3) GE(sc_nxt, 0) GE(sc_nxt, 1))
      LASER_SLOT(LASER_PV0(2), GA(sc_nxt, 0) GA(sc_nxt, 1) GM(sc_nxt, 4) GM(sc_nxt, 5) GE(sc_nxt, 2) GE(sc_nxt, 3))
      LASER_SLOT(LASER_PV0(3), GA(sc_nxt, 2) GA(sc_nxt, 3) GM(sc_nxt, 6) GM(sc_nxt, 7) GR(sc_nxt, 0) GR(sc_nxt, 1))
#undef LASER_PV0
      if (nvt < DT_TI) clear_past_end(p1, 1);
      // Operand reads of later tiles are requested as soon as their registers are free, unconditionally: with no
      // branch around them the compiler counts the outstanding reads exactly and waits only for the ones an
      // instruction needs (with a branch it falls back to waiting for all of them at the top of every step, which
      // exposes the latency of the V reads issued just before). Without such a tile they read stale LDS, unused.
      read_k(nbuf2);
#define LASER_PV1(I) acc[I] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[1][I], __builtin_bit_cast(bf16x8, p1), acc[I], 0, 0, 0)
      // p0 is rewritten for the next tile from here on: its last reader was B3
      LASER_SLOT(LASER_PV1(0), GC(p0, 0, sc_nxt, 0) GE(sc_nxt, 4) GE(sc_nxt, 5) GR(sc_nxt, 2) GR(sc_nxt, 3))
      LASER_SLOT(LASER_PV1(1), GA(sc_nxt, 4) GA(sc_nxt, 5) GC(p0, 1, sc_nxt, 2) GE(sc_nxt, 6) GE(sc_nxt, 7))
      LASER_SLOT(LASER_PV1(2), GA(sc_nxt, 6) GA(sc_nxt, 7) GR(sc_nxt, 4) GR(sc_nxt, 5))
      LASER_SLOT(LASER_PV1(3), GC(p0, 2, sc_nxt, 4) GR(sc_nxt, 6) GR(sc_nxt, 7))
#undef LASER_PV1
#undef LASER_SLOT
#undef LASER_PIN
#undef GM
#undef GE
#undef GA
#undef GR
#undef GC
    }

    if (nxt.seg != cur.seg) {   // segment finished: park H' rows in the patch
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[db][g * 4 + e];
          *reinterpret_cast<u32x2*>(opatch + l32 * OP + (db * 32 + g * 8 + h * 4) * 2) = __builtin_bit_cast(u32x2, o);
        }
      out_seg = cur.seg;
      out_units = 0;
      fl_dst = oU + (size_t)cur.seg * (D * 2);
      fl_src = opr;
      fl_row = cbase + lane / LPR;
    }
    if (wave >= NW / 2) issue_next();
    ++done;
    cbuf = nbuf;
    cur = nxt;
  };
  while (cur.seg < seg_ne) {
    step(scA, scB);
    if (cur.seg >= seg_ne) break;
    step(scB, scA);
  }
  if (out_seg >= 0) flush_units(FU - out_units);

  if (seg_ne < seg_hi) {   // empty segments of the run: exact zeros
    const int ncand = (C - ct * (CW * NW)) < CW * NW ? (C - ct * (CW * NW)) : CW * NW;
    const int per_row = D / 8;
    const int rows = ncand * (seg_hi - seg_ne);
    for (int e = tid; e < rows * per_row; e += NT) {
      const int row = e / per_row, ch = e - row * per_row;
      const int cc = row / (seg_hi - seg_ne), ii = seg_ne + row % (seg_hi - seg_ne);
      *reinterpret_cast<u32x4*>(seg_out + ((pb + ct * (CW * NW) + cc) * S + ii) * D + ch * 8) =
          u32x4{0u, 0u, 0u, 0u};
    }
  }
}

// ------------------------------------------------------------------------------------------ host side
static int pick_nw(int C) {
  const int vv = tuning_int("LASER_STA_NW", 0);   // tuning builds: waves (32 candidates each) per workgroup
  if (vv == 1 || vv == 2 || vv == 4 || vv == 8) return vv;
  return C > 128 ? 8 : (C > 64 ? 4 : (C > 32 ? 2 : 1));
}

bool sta_mfma_supports(const StaArgs& a) {
  if (a.dt != LASER_BF16) return false;
  if (!(a.d_q == 32 || a.d_q == 64 || a.d_q == 128)) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  // several heads: the register-staged form; a head owns whole 16-wide k-steps and whole 32-column blocks
  if (a.heads != 1 && a.heads != 2 && a.heads != 4) return false;
  if (a.heads == 4 && (a.d_q < 64 || a.d != 128)) return false;
  if (a.C < 9) return false;   // fewer candidates than that: the streaming kernel's range
  const int nw = pick_nw(a.C);
  const long long ctiles = (a.C + CW * nw - 1) / (CW * nw);
  return (long long)a.U * ctiles * a.S <= 0x7fffffffLL;
}

template <int DQ, int D, int NW, int NBUF, int HEADS = 1, bool SOFTMAX = false>
static void launch_one(const StaArgs& a, int spw, int ctiles, int sruns, float nsl) {
  const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
  hipLaunchKernelGGL((sta_mfma_kernel<DQ, D, NW, NBUF, HEADS, SOFTMAX>), dim3(blocks), dim3(64 * NW), 0, a.stream,
                     (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens, a.cand_off, a.P, a.C,
                     a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
}

template <int DQ, int D>
static void launch_nw(const StaArgs& a, int nw, int spw, int ctiles, int sruns, float nsl) {
  // eight waves fill a compute unit on their own and prefetch through LDS buffers of their own (direct-to-LDS
  // fetches for d_q = d = 128; a tuning build can select the register-staged form there too, for comparison);
  // smaller workgroups overlap memory and MFMA work across the several workgroups that share a compute unit
  // two heads, the softmax variant: the register-staged form for every workgroup size (two tile buffers with
  // eight waves)
#define LASER_STA_STAGED(H, SM)                                                      \
  do {                                                                               \
    if (nw == 8) launch_one<DQ, D, 8, 2, H, SM>(a, spw, ctiles, sruns, nsl);         \
    else if (nw == 4) launch_one<DQ, D, 4, 1, H, SM>(a, spw, ctiles, sruns, nsl);    \
    else if (nw == 2) launch_one<DQ, D, 2, 1, H, SM>(a, spw, ctiles, sruns, nsl);    \
    else launch_one<DQ, D, 1, 1, H, SM>(a, spw, ctiles, sruns, nsl);                 \
  } while (0)
  if (a.heads == 4) {
    if constexpr ((DQ / 16) % 4 == 0 && (D / 32) % 4 == 0) {
      if (a.softmax) LASER_STA_STAGED(4, true);
      else LASER_STA_STAGED(4, false);
    }
  } else if (a.softmax) {
    if (a.heads == 2) LASER_STA_STAGED(2, true);
    else LASER_STA_STAGED(1, true);
  } else if (a.heads == 2) {
    LASER_STA_STAGED(2, false);
  } else if (nw == 8 && DQ == 128 && D == 128 && tuning_int("LASER_STA_NODMA", 0) == 0) {
    const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
    if (a.reread)
      hipLaunchKernelGGL((sta_mfma_dma_kernel<8, false>), dim3(blocks), dim3(512), 0, a.stream,
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                         a.cand_off, a.P, a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
    else
      hipLaunchKernelGGL((sta_mfma_dma_kernel<8, true>), dim3(blocks), dim3(512), 0, a.stream,
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                         a.cand_off, a.P, a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
  } else if (nw == 8) {
    const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
    hipLaunchKernelGGL((sta_mfma_pipe_kernel<DQ, D, 8>), dim3(blocks), dim3(512), 0, a.stream,
                       (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                       a.cand_off, a.P, a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
  }
  else if (nw == 4 && DQ == 128 && D == 128 && tuning_int("LASER_STA_NODMA", 0) == 0) {
    // 65 to 128 candidates: the same kernel with four waves, one workgroup per compute unit (LDS) and one wave per
    // SIMD; its deep prefetch needs several segments per workgroup to pay (see sta_mfma_launch)
    const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
    if (a.reread)
      hipLaunchKernelGGL((sta_mfma_dma_kernel<4, false>), dim3(blocks), dim3(256), 0, a.stream,
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                         a.cand_off, a.P, a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
    else
      hipLaunchKernelGGL((sta_mfma_dma_kernel<4, true>), dim3(blocks), dim3(256), 0, a.stream,
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                         a.cand_off, a.P, a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, (unsigned short*)a.seg_out, a.seg_cnt);
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
  // (smaller workgroups: more of them fit a compute unit, so more are wanted; 64 users x 64 candidates x 16
  // segments, two waves: 15.1 us with 512 workgroups of two segments, 11.2 us with 1024 of one)
  const long long want = 2048 / nw;
  int spw = 1;
  while (spw < 8 && (long long)a.U * ctiles * ((a.S + 2 * spw - 1) / (2 * spw)) >= want) spw *= 2;
  // the direct-to-LDS kernels take a compute unit's LDS per workgroup: as many segments per workgroup as bring the
  // launch down to one round of 256 workgroups, eight at most (16 users x 128 candidates x 40 segments: 640
  // workgroups of one segment 32.9 us in the register-staged form, 224 of three segments 26.8 us in this one)
  const bool direct = a.heads == 1 && !a.softmax && a.d_q == 128 && a.d == 128 && (nw == 8 || nw == 4) &&
                      tuning_int("LASER_STA_NODMA", 0) == 0;
  if (direct) {
    const long long per_seg = (long long)a.U * ctiles * a.S;
    spw = (int)((per_seg + 255) / 256 < 8 ? (per_seg + 255) / 256 : 8);
    if (spw < 1) spw = 1;
  }
  const int spw_forced = tuning_int("LASER_STA_SPW", 0);   // tuning builds only
  if (spw_forced >= 1 && spw_forced <= 64) spw = spw_forced;
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
