// The whole path without H' in memory: STA (Sec. 3.4.2, global form of Sec. 3.5.1) with one GSTA layer (Sec. 3.4.3)
// applied to every segment vector while it is still in registers, so that only z = t0 + o is written.
//
// For one (user, candidate) pair, with H'_i the STA vector of segment i, the layer is
//   q' = t0 W_q,  r = W_k q'^T / sqrt(d),  e_i = H'_i . r,  a = softmax_i(e_i) over the segments that hold a valid item,
//   p = sum_i a_i H'_i,  z = t0 + p W_v
// (the products with H' re-associated, which is exact). r does not depend on the history, so it is computed first;
// the softmax over segments is then taken online as the segments are produced: a running maximum m, denominator l
// and weighted sum P = sum_i 2^(e_i log2 e - m) H'_i per pair, rescaled when the maximum moves. A workgroup that
// walks only a run of a user's segments (few users: the history must be split to fill the machine) leaves its
// (m, l, P) in a caller-owned work buffer and a second kernel merges the runs of a pair and applies W_v; a workgroup
// that walks the whole history finishes the pair itself and needs no work buffer. The segment vectors enter the
// layer as fp32 sums (they are never rounded to the storage type, unlike the two-launch path).
// One layer only: a second layer needs every H'_i again with another r, i.e. H' in memory.
//
// Two kernels. fused_mfma_kernel (bf16, the matrix-core STA kernel's tile scheme: 32 candidates per wave, the score
// and aggregation products transposed so that the accumulators hold H'^T with lane = candidate); the three small
// products of the layer run on the matrix cores as well, their fp32 operands split into a bf16 head and remainder.
// fused_generic_kernel (fp32 arithmetic, any shape, either storage type): the correctness path.
#include "laser_internal.h"
#include "sta_mfma_tile.h"

namespace laser {

constexpr float FUSED_NEG = -1.0e30f;   // "no segment yet": below any score, and 2^(FUSED_NEG - m) is exactly 0

// ---------------------------------------------------------------------------------------------- matrix cores
// Accumulator layout (the result layout of v_mfma_f32_32x32x16_bf16 with lane = candidate): lane (c = lane % 32,
// h = lane / 32) holds, of candidate c's vector, block b (32 components), register r: component
// 32 b + 8 (r / 4) + 4 h + r % 4. Registers 8 s .. 8 s + 7 of a block are, as they sit, a B operand whose eight
// k-slots are the components 32 b + 16 s + {4h .. 4h+3, 8+4h .. 8+4h+3}: every product below that consumes such a
// vector fetches its A operand with the same slot order.

template <int D>
struct WeightsLds {   // a [D, D] bf16 matrix in LDS, row pitch P bytes
  // A = W^T[e, k-slots] for output block eb and k-step ks (16 input rows): transpose loads from rows stored as given
  // (pitch = 64 mod 256, as for the value tiles)
  static __device__ __forceinline__ bf16x8 transposed(const unsigned char* Wl, int P, int eb, int ks, int lane) {
    const int l32 = lane & 31, h = lane >> 5, i16 = lane & 15;
    const unsigned char* src = Wl + (ks * 16 + h * 4 + (i16 >> 2)) * P + (eb * 32 + (l32 & 16) + 4 * (i16 & 3)) * 2;
    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 8 * P));
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
  }
  // A = W[k, e-slots] for row block kb and the k-step (eb, s): two 8-byte pieces of a row
  static __device__ __forceinline__ bf16x8 rows(const unsigned char* Wl, int P, int kb, int eb, int s, int lane) {
    const int l32 = lane & 31, h = lane >> 5;
    const unsigned char* src = Wl + (kb * 32 + l32) * P + (eb * 32 + 16 * s + 4 * h) * 2;
    const u32x2 a = *reinterpret_cast<const u32x2*>(src);
    const u32x2 b = *reinterpret_cast<const u32x2*>(src + 16);
    const u32x4 both = {a[0], a[1], b[0], b[1]};
    return __builtin_bit_cast(bf16x8, both);
  }
  template <int NT>
  static __device__ __forceinline__ void park(unsigned char* Wl, int P, const unsigned short* W, int tid) {
    constexpr int CH = D / 8;
    for (int e = tid; e < D * CH; e += NT) {
      const int row = e / CH, ch = e % CH;
      *reinterpret_cast<u32x4*>(Wl + row * P + ch * 16) = *reinterpret_cast<const u32x4*>(W + (size_t)row * D + ch * 8);
    }
  }
};

// fp32 registers 8 s .. 8 s + 7 of an accumulator block as two bf16 B operands: the rounded values and what is left
__device__ __forceinline__ void split_operand(const f32x16& x, int s, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float v = x[s * 8 + e];
    const __bf16 hv = (__bf16)v;
    hi[e] = hv;
    lo[e] = (__bf16)(v - (float)hv);
  }
}

// y^T = W^T x^T for the wave's 32 candidates: x and y in accumulator layout, W [D, D] parked with the value pitch.
// (x W in the paper's row-vector notation.)
template <int D>
__device__ __forceinline__ void times_matrix(const f32x16 (&x)[D / 32], const unsigned char* Wl, int P, int lane,
                                             f32x16 (&y)[D / 32]) {
  constexpr int DB = D / 32;
#pragma unroll
  for (int eb = 0; eb < DB; ++eb)
#pragma unroll
    for (int r = 0; r < 16; ++r) y[eb][r] = 0.0f;
#pragma unroll
  for (int kb = 0; kb < DB; ++kb)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      bf16x8 hi, lo;
      split_operand(x[kb], s, hi, lo);
#pragma unroll
      for (int eb = 0; eb < DB; ++eb) {
        const bf16x8 a = WeightsLds<D>::transposed(Wl, P, eb, kb * 2 + s, lane);
        y[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, hi, y[eb], 0, 0, 0);
        y[eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, lo, y[eb], 0, 0, 0);
      }
    }
}

// t0 of the wave's candidates in accumulator layout (fp32), rows past the user's last candidate as zeros
template <int D>
__device__ __forceinline__ void load_targets(const unsigned short* t0, size_t pair0, int cbase, int C, int lane,
                                             f32x16 (&t)[D / 32]) {
  const int l32 = lane & 31, h = lane >> 5;
  const bool live = cbase + l32 < C;
#pragma unroll
  for (int b = 0; b < D / 32; ++b)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      u32x2 raw = {0u, 0u};
      if (live) raw = *reinterpret_cast<const u32x2*>(t0 + (pair0 + cbase + l32) * D + b * 32 + g * 8 + h * 4);
      t[b][g * 4 + 0] = __uint_as_float(raw[0] << 16);
      t[b][g * 4 + 1] = __uint_as_float(raw[0] & 0xffff0000u);
      t[b][g * 4 + 2] = __uint_as_float(raw[1] << 16);
      t[b][g * 4 + 3] = __uint_as_float(raw[1] & 0xffff0000u);
    }
}

// z = t0 + (P / l) W_v for the wave's candidates; Wv parked in LDS with the value pitch
template <int D>
__device__ __forceinline__ void finish_pairs(const f32x16 (&pacc)[D / 32], float l, const unsigned short* t0,
                                             size_t pair0, int cbase, int C, const unsigned char* Wvl, int P, int lane,
                                             float* z) {
  constexpr int DB = D / 32;
  const int l32 = lane & 31, h = lane >> 5;
  const float inv = l > 0.0f ? 1.0f / l : 0.0f;   // no valid segment: z = t0
  f32x16 pn[DB], o[DB], t[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) pn[b][r] = pacc[b][r] * inv;
  times_matrix<D>(pn, Wvl, P, lane, o);
  load_targets<D>(t0, pair0, cbase, C, lane, t);
  if (cbase + l32 < C) {
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 out = {t[b][g * 4] + o[b][g * 4], t[b][g * 4 + 1] + o[b][g * 4 + 1], t[b][g * 4 + 2] + o[b][g * 4 + 2],
                           t[b][g * 4 + 3] + o[b][g * 4 + 3]};
        *reinterpret_cast<f32x4*>(z + (pair0 + cbase + l32) * D + b * 32 + g * 8 + h * 4) = out;
      }
  }
}

// Work buffer: per (tile of 32 candidates, run) the registers of (P, m, l) lane by lane, D / 2 + 2 rows of 64 floats
template <int D> constexpr int part_rows() { return D / 2 + 2; }

template <int DQ, int D, int NW, int NBUF>
__global__ __launch_bounds__(64 * NW) void fused_mfma_kernel(const unsigned short* __restrict__ q,
                                                             const unsigned short* __restrict__ k,
                                                             const unsigned short* __restrict__ v,
                                                             const unsigned short* __restrict__ t0,
                                                             const unsigned short* __restrict__ wq,
                                                             const unsigned short* __restrict__ wk,
                                                             const unsigned short* __restrict__ wv,
                                                             const int32_t* __restrict__ lens, int C, int L, int w,
                                                             int S, int spw, int ctiles, int sruns,
                                                             float neg_scale_log2e, float* __restrict__ z,
                                                             int32_t* __restrict__ seg_cnt, float* __restrict__ part) {
  constexpr int KP = KPitch<DQ>::v, VP = VPitch<D>::v, WKP = KPitch<D>::v;
  constexpr int NT = 64 * NW;
  constexpr int KSTEPS = DQ / 16, DB = D / 32;
  constexpr int KBYTES = TI * KP, VBYTES = TI * VP;
  constexpr int TILES = NBUF * (KBYTES + VBYTES), WEIGHTS = D * VP + D * WKP;
  __shared__ __attribute__((aligned(16))) unsigned char smem[TILES > WEIGHTS ? TILES : WEIGHTS];

  int bid = blockIdx.x;
  const int srun = bid % sruns;
  bid /= sruns;
  const int ct = bid % ctiles;
  const int u = bid / ctiles;
  const size_t pb = (size_t)u * C;   // first pair of this user

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;
  const int cbase = ct * (CW * NW) + wave * CW;     // first candidate of this wave
  const int n = valid_len(lens, u, L);
  if (srun == 0 && ct == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, NT);

  // ---- r = W_k (t0 W_q)^T log2(e) / sqrt(d) for the wave's candidates, in accumulator layout
  f32x16 rr[DB];
  {
    unsigned char* Wql = smem;
    unsigned char* Wkl = smem + D * VP;
    WeightsLds<D>::template park<NT>(Wql, VP, wq, tid);
    WeightsLds<D>::template park<NT>(Wkl, WKP, wk, tid);
    f32x16 t[DB], qp[DB];
    load_targets<D>(t0, pb, cbase, C, lane, t);
    __syncthreads();
    times_matrix<D>(t, Wql, VP, lane, qp);   // q'^T (t0 holds bf16 values: the remainder pass adds zeros)
    const float rscale = 1.4426950408889634f / sqrtf((float)D);
#pragma unroll
    for (int kb = 0; kb < DB; ++kb) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
      for (int eb = 0; eb < DB; ++eb)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          bf16x8 hi, lo;
          split_operand(qp[eb], s, hi, lo);
          const bf16x8 a = WeightsLds<D>::rows(Wkl, WKP, kb, eb, s, lane);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, hi, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, lo, acc, 0, 0, 0);
        }
#pragma unroll
      for (int r = 0; r < 16; ++r) rr[kb][r] = acc[r] * rscale;
    }
    __syncthreads();   // the weights' LDS becomes the tile buffers
  }

  // ---- queries: B operand of the score product
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
  int seg_ne = seg_lo;   // valid items are a prefix of the history: so are the non-empty segments of the run
  while (seg_ne < seg_hi && seg_ne * w < n) ++seg_ne;
  auto seg_end = [&](int i) {
    int e = i * w + w;
    if (e > L) e = L;
    if (e > n) e = n;
    return e;
  };

  f32x16 acc[DB], pacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      acc[db][r] = 0.0f;
      pacc[db][r] = 0.0f;
    }
  float sm_m = FUSED_NEG, sm_l = 0.0f;

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
  // a finished segment's vector enters the layer's online softmax (base 2: rr carries log2 e / sqrt d)
  auto segment_done = [&]() {
    float e2 = 0.0f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) e2 = fmaf(acc[db][r], rr[db][r], e2);
    {   // the other half of the candidate's components sits in lane ^ 32
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(e2), __float_as_uint(e2), false, false);
      e2 = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float m_new = fmaxf(sm_m, e2);
    const float corr = __builtin_amdgcn_exp2f(sm_m - m_new);   // exactly 0 at the first segment
    const float wgt = __builtin_amdgcn_exp2f(e2 - m_new);
    sm_l = fmaf(sm_l, corr, wgt);
    sm_m = m_new;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        pacc[db][r] = fmaf(wgt, acc[db][r], pacc[db][r] * corr);
        acc[db][r] = 0.0f;
      }
  };

  Stage<DQ, D, NT> st;
  int ci = seg_lo, ct0 = seg_lo * w, chi = seg_ne > seg_lo ? seg_end(seg_lo) : 0;   // current tile
  int buf = 0;
  if (seg_ne > seg_lo) {
    st.load(kU, vU, ct0, chi, tid);
    st.store(smem, smem + KBYTES, tid);
  }
  __syncthreads();

  if constexpr (NBUF == 2 && D == 64) {
    // The two 32-item blocks of a tile software-pipelined inside the wave: the score chain of one block runs beside
    // the gates of the other, the aggregation of a block beside the gates of the next. Every tile is computed in
    // full (its padding rows are zeros in LDS). (Measured: 64 users x 64 candidates, d = 64: 29.1 -> 26.9 us for the
    // whole fused path; with d = 128, at 383 registers and one wave per SIMD, the same order is slower, 60 against
    // 51 us for 32 users x 256 candidates, and the plain order below is kept.)
    f32x16 sc0;
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
      st.load(kU, vU, has_next ? nt0 : ct0, has_next ? nhi : chi, tid);   // lands during the products below
      bf16x8 p0[2], p1[2];
      const f32x16 sc1 = score(Ks, 1);
      gates(sc0, p0);
      aggregate(Vs, 0, p0);
      gates(sc1, p1);
      aggregate(Vs, 1, p1);
      if (has_next) st.store(nKs, nKs + KBYTES, tid);
      if (ni != ci) segment_done();
      __syncthreads();
      buf ^= 1;
      if (has_next) sc0 = score(nKs, 0);
      ci = ni;
      ct0 = nt0;
      chi = nhi;
    }
  } else {
    while (ci < seg_ne) {
      int ni = ci, nt0 = ct0 + TI, nhi = chi;
      if (nt0 >= chi) {
        ni = ci + 1;
        nt0 = ni * w;
        nhi = ni < seg_ne ? seg_end(ni) : 0;
      }
      const bool has_next = ni < seg_ne;
      const unsigned char* Ks = smem + buf * (KBYTES + VBYTES);
      // (in flight during the products below; with no next tile the current one is read again, in bounds and unused)
      if (NBUF == 2) st.load(kU, vU, has_next ? nt0 : ct0, has_next ? nhi : chi, tid);
#pragma unroll
      for (int ib = 0; ib < TI / 32; ++ib) {
        if (ct0 + ib * 32 < chi) {   // uniform: otherwise the rest of the tile is padding (zero rows)
          bf16x8 p[2];
          gates(score(Ks, ib), p);
          aggregate(Ks + KBYTES, ib, p);
        }
      }
      if (NBUF == 2 && has_next)
        st.store(smem + (buf ^ 1) * (KBYTES + VBYTES), smem + (buf ^ 1) * (KBYTES + VBYTES) + KBYTES, tid);
      if (ni != ci) segment_done();
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
  }

  if (sruns == 1) {   // the whole history was walked here: finish the pairs (the tile buffers become W_v's)
    __syncthreads();
    WeightsLds<D>::template park<NT>(smem, VP, wv, tid);
    __syncthreads();
    finish_pairs<D>(pacc, sm_l, t0, pb, cbase, C, smem, VP, lane, z);
  } else {            // leave (P, m, l) for the merge
    const size_t tile = ((size_t)u * ctiles + ct) * NW + wave;
    float* dst = part + ((tile * sruns + srun) * part_rows<D>()) * 64 + lane;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[(db * 16 + r) * 64] = pacc[db][r];
    dst[(D / 2) * 64] = sm_m;
    dst[(D / 2 + 1) * 64] = sm_l;
  }
}

// The runs of a pair merged in a fixed order (reproducible), then z = t0 + (P / l) W_v. One workgroup per tile of 32
// candidates (tiles numbered as by the kernel that wrote the partial results: nwf of them per (user, candidate
// tile)); wave v merges runs v, v + NWM, ... in ascending order, the waves' results meet in LDS and wave 0 merges
// them in wave order and finishes the pairs. All waves park W_v meanwhile.
template <int D, int NWM>
__global__ __launch_bounds__(64 * NWM) void fused_merge_kernel(const float* __restrict__ part,
                                                               const unsigned short* __restrict__ t0,
                                                               const unsigned short* __restrict__ wv, int C,
                                                               int ctiles, int nwf, int sruns, float* __restrict__ z) {
  constexpr int VP = VPitch<D>::v, DB = D / 32, ROWS = part_rows<D>();
  __shared__ __attribute__((aligned(16))) unsigned char Wvl[D * VP];
  __shared__ float mix[NWM][ROWS][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  WeightsLds<D>::template park<64 * NWM>(Wvl, VP, wv, tid);
  const long long tile = blockIdx.x;
  const int wv_in = (int)(tile % nwf);
  const long long uc = tile / nwf;
  const int ct = (int)(uc % ctiles);
  const int u = (int)(uc / ctiles);
  const int cbase = ct * (CW * nwf) + wv_in * CW;

  f32x16 pacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) pacc[db][r] = 0.0f;
  float m = FUSED_NEG, l = 0.0f;
  auto absorb = [&](float ms, float ls, auto&& prow) {   // (m, l, P) <- (m, l, P) merged with (ms, ls, prow(.))
    const float m_new = fmaxf(m, ms);
    const float corr = __builtin_amdgcn_exp2f(m - m_new), ws = __builtin_amdgcn_exp2f(ms - m_new);
    l = fmaf(l, corr, ls * ws);
    m = m_new;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) pacc[db][r] = fmaf(prow(db * 16 + r), ws, pacc[db][r] * corr);
  };
  for (int s = wave; s < sruns; s += NWM) {
    const float* src = part + (((size_t)tile * sruns + s) * ROWS) * 64 + lane;
    absorb(src[(D / 2) * 64], src[(D / 2 + 1) * 64], [&](int row) { return src[row * 64]; });
  }
  if (wave > 0) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) mix[wave][db * 16 + r][lane] = pacc[db][r];
    mix[wave][D / 2][lane] = m;
    mix[wave][D / 2 + 1][lane] = l;
  }
  __syncthreads();
  if (wave == 0) {
    for (int o = 1; o < NWM; ++o)
      absorb(mix[o][D / 2][lane], mix[o][D / 2 + 1][lane], [&](int row) { return mix[o][row][lane]; });
    finish_pairs<D>(pacc, l, t0, (size_t)u * C, cbase, C, Wvl, VP, lane, z);
  }
}

// ---------------------------------------------------------------------------------------------- generic kernel
// One workgroup per (user, four candidates), a wave per candidate, walking every non-empty segment of the user in
// chunks of TI items staged in LDS as fp32 (as the generic STA kernel does for one segment). Lane `lane` owns the
// components lane, lane + 64, ... of its candidate's vectors: r, the segment sum, the weighted sum P.
constexpr int FG_WAVES = 4;
constexpr int FG_MAX_COLS = 16;   // d <= 1024

template <typename T>
__global__ __launch_bounds__(256) void fused_generic_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                            const T* __restrict__ v, const T* __restrict__ t0,
                                                            const T* __restrict__ wq, const T* __restrict__ wk,
                                                            const T* __restrict__ wv, const int32_t* __restrict__ lens,
                                                            int C, int L, int dq, int d, int w, int S, int TI,
                                                            float inv_gamma, float* __restrict__ z,
                                                            int32_t* __restrict__ seg_cnt) {
  extern __shared__ float smem[];
  const int kpitch = dq + 1;
  float* Ks = smem;                            // [TI][dq + 1]
  float* Vs = Ks + (size_t)TI * kpitch;        // [TI][d]
  float* qs = Vs + (size_t)TI * d;             // [4][dq]
  float* gs = qs + FG_WAVES * dq;              // [4][TI]
  float* xs = gs + FG_WAVES * TI;              // [4][d] a vector per wave: t0, then q', then P / l

  const int cblocks = (C + FG_WAVES - 1) / FG_WAVES;
  const int cb = blockIdx.x % cblocks, u = blockIdx.x / cblocks;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = cb * FG_WAVES + wave;
  const bool active = c < C;
  const size_t pair = (size_t)u * C + (active ? c : C - 1);   // idle waves repeat the last candidate, and store nothing
  const int n = valid_len(lens, u, L);
  if (cb == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, 256);
  const int nb = (d + 63) >> 6;
  float* xw = xs + wave * d;

  // r = W_k (t0 W_q)^T / sqrt(d), this lane's components
  for (int a = lane; a < d; a += 64) xw[a] = load_as_f32(t0, pair * d + a);
  for (int a = lane; a < dq; a += 64) qs[wave * dq + a] = load_as_f32(q, pair * dq + a);
  __syncthreads();
  float rr[FG_MAX_COLS], qp[FG_MAX_COLS];
#pragma unroll
  for (int b = 0; b < FG_MAX_COLS; ++b) {
    rr[b] = qp[b] = 0.0f;
    if (b >= nb) continue;
    const int col = lane + 64 * b;
    if (col < d)
      for (int a = 0; a < d; ++a) qp[b] = fmaf(xw[a], load_as_f32(wq, (size_t)a * d + col), qp[b]);
  }
  __syncthreads();
#pragma unroll
  for (int b = 0; b < FG_MAX_COLS; ++b)
    if (b < nb && lane + 64 * b < d) xw[lane + 64 * b] = qp[b];
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)d);
#pragma unroll
  for (int b = 0; b < FG_MAX_COLS; ++b) {
    if (b >= nb) continue;
    const int row = lane + 64 * b;
    if (row < d) {
      float s = 0.0f;
      for (int e = 0; e < d; ++e) s = fmaf(load_as_f32(wk, (size_t)row * d + e), xw[e], s);
      rr[b] = s * scale;
    }
  }

  float acc[FG_MAX_COLS], pacc[FG_MAX_COLS];
#pragma unroll
  for (int b = 0; b < FG_MAX_COLS; ++b) acc[b] = pacc[b] = 0.0f;
  float sm_m = -INFINITY, sm_l = 0.0f;

  const T* kU = k + (size_t)u * L * dq;
  const T* vU = v + (size_t)u * L * d;
  const int nseg = (n + w - 1) / w;   // segments that hold a valid item
  for (int i = 0; i < nseg; ++i) {
    const int lo = i * w;
    int hi = lo + w;
    if (hi > L) hi = L;
    if (hi > n) hi = n;
    for (int j0 = lo; j0 < hi; j0 += TI) {
      const int nj = (hi - j0) < TI ? (hi - j0) : TI;
      __syncthreads();
#pragma unroll 8
      for (int e = tid; e < nj * dq; e += 256) {
        const int r = e / dq, a = e - r * dq;
        Ks[r * kpitch + a] = load_as_f32(kU, (size_t)(j0 + r) * dq + a);
      }
#pragma unroll 8
      for (int e = tid; e < nj * d; e += 256) Vs[e] = load_as_f32(vU, (size_t)j0 * d + e);
      __syncthreads();
      if (lane < nj) {
        const float* kr = Ks + lane * kpitch;
        const float* qr = qs + wave * dq;
        float e = 0.0f;
#pragma unroll 8
        for (int a = 0; a < dq; ++a) e = fmaf(qr[a], kr[a], e);
        gs[wave * TI + lane] = 1.0f / (1.0f + expf(-e * inv_gamma));
      }
      __syncthreads();
#pragma unroll 4
      for (int jj = 0; jj < nj; ++jj) {
        const float g = gs[wave * TI + jj];
#pragma unroll
        for (int b = 0; b < FG_MAX_COLS; ++b) {
          if (b >= nb) break;
          const int col = lane + 64 * b;
          if (col < d) acc[b] = fmaf(g, Vs[jj * d + col], acc[b]);
        }
      }
    }
    // segment i is complete: score, online softmax, weighted sum
    float e = 0.0f;
#pragma unroll
    for (int b = 0; b < FG_MAX_COLS; ++b) e = fmaf(acc[b], rr[b], e);
    e = wave_sum(e);
    const float m_new = fmaxf(sm_m, e);
    const float corr = expf(sm_m - m_new);   // 0 at the first segment
    const float wgt = expf(e - m_new);
    sm_l = fmaf(sm_l, corr, wgt);
    sm_m = m_new;
#pragma unroll
    for (int b = 0; b < FG_MAX_COLS; ++b) {
      pacc[b] = fmaf(wgt, acc[b], pacc[b] * corr);
      acc[b] = 0.0f;
    }
  }

  // z = t0 + (P / l) W_v
  __syncthreads();
  const float inv = sm_l > 0.0f ? 1.0f / sm_l : 0.0f;
#pragma unroll
  for (int b = 0; b < FG_MAX_COLS; ++b)
    if (b < nb && lane + 64 * b < d) xw[lane + 64 * b] = pacc[b] * inv;
  __syncthreads();
  if (active) {
#pragma unroll
    for (int b = 0; b < FG_MAX_COLS; ++b) {
      if (b >= nb) continue;
      const int col = lane + 64 * b;
      if (col < d) {
        float o = 0.0f;
        for (int a = 0; a < d; ++a) o = fmaf(xw[a], load_as_f32(wv, (size_t)a * d + col), o);
        z[pair * d + col] = load_as_f32(t0, pair * d + col) + o;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------- host side
static size_t fg_lds_bytes(int TI, int dq, int d) {
  return sizeof(float) * ((size_t)TI * (dq + 1) + (size_t)TI * d + FG_WAVES * dq + (size_t)FG_WAVES * TI + FG_WAVES * d);
}
static int fg_pick_ti(int dq, int d) {
  for (int ti = 64; ti >= 1; ti >>= 1)
    if (fg_lds_bytes(ti, dq, d) <= 60 * 1024) return ti;
  return 0;
}

bool fused_generic_supports(const FusedArgs& a) {
  if (a.d > 64 * FG_MAX_COLS || a.d_q > 1024 || fg_pick_ti(a.d_q, a.d) == 0) return false;
  return (long long)a.U * ((a.C + FG_WAVES - 1) / FG_WAVES) <= 0x7fffffffLL;
}

laser_status fused_generic_launch(const FusedArgs& a) {
  if (!fused_generic_supports(a)) return LASER_ERR_UNSUPPORTED;
  const int TI = fg_pick_ti(a.d_q, a.d);
  const size_t lds = fg_lds_bytes(TI, a.d_q, a.d);
  const unsigned blocks = (unsigned)((long long)a.U * ((a.C + FG_WAVES - 1) / FG_WAVES));
  const float inv_gamma = 1.0f / a.gamma;
  if (a.dt == LASER_F32)
    hipLaunchKernelGGL(fused_generic_kernel<float>, dim3(blocks), dim3(256), lds, a.stream, (const float*)a.q,
                       (const float*)a.k, (const float*)a.v, (const float*)a.t0, (const float*)a.wq, (const float*)a.wk,
                       (const float*)a.wv, a.lens, a.C, a.L, a.d_q, a.d, a.w, a.S, TI, inv_gamma, a.z_out, a.seg_cnt);
  else
    hipLaunchKernelGGL(fused_generic_kernel<unsigned short>, dim3(blocks), dim3(256), lds, a.stream,
                       (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,
                       (const unsigned short*)a.t0, (const unsigned short*)a.wq, (const unsigned short*)a.wk,
                       (const unsigned short*)a.wv, a.lens, a.C, a.L, a.d_q, a.d, a.w, a.S, TI, inv_gamma, a.z_out,
                       a.seg_cnt);
  return launch_status();
}

// Waves (32 candidates each) per workgroup. With d = 128 a wave holds three vectors per candidate in registers
// (segment sum, weighted sum, r: 192 of them) beside the operands: one wave per SIMD, so at most four per workgroup.
static int fused_nw(const FusedArgs& a) {
  const int cap = a.d == 128 ? 4 : 8;
  const int nw = a.C > 128 ? 8 : (a.C > 64 ? 4 : (a.C > 32 ? 2 : 1));
  return nw < cap ? nw : cap;
}

// Runs of segments per user. Without a work buffer a workgroup walks the whole history (one run). With one, the
// history is cut into as many runs as it takes to give every compute unit a workgroup (two for the smaller
// workgroups), but no finer: every run costs a partial result per pair and the set-up of a workgroup.
static void fused_runs(const FusedArgs& a, int nw, int* spw, int* sruns) {
  const int ctiles = (a.C + CW * nw - 1) / (CW * nw);
  const long long groups = (long long)a.U * ctiles;
  const long long want = nw >= 4 ? 256 : 512;
  int runs = 1;
  if (a.work != nullptr && groups < want) {
    runs = (int)((want + groups - 1) / groups);
    if (runs > a.S) runs = a.S;
  }
  *spw = (a.S + runs - 1) / runs;
  *sruns = (a.S + *spw - 1) / *spw;
}

bool fused_mfma_supports(const FusedArgs& a) {
  if (a.dt != LASER_BF16) return false;
  if (!(a.d_q == 32 || a.d_q == 64 || a.d_q == 128)) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  const int nw = fused_nw(a);
  const long long ctiles = (a.C + CW * nw - 1) / (CW * nw);
  return (long long)a.U * ctiles * a.S <= 0x7fffffffLL;
}

size_t fused_work_bytes(const FusedArgs& a) {
  if (!fused_mfma_supports(a)) return 0;
  FusedArgs b = a;
  b.work = reinterpret_cast<float*>(16);   // any non-null value: the run count a work buffer would allow
  const int nw = fused_nw(b);
  int spw, sruns;
  fused_runs(b, nw, &spw, &sruns);
  if (sruns == 1) return 0;
  const size_t ctiles = (a.C + CW * nw - 1) / (CW * nw);
  return (size_t)a.U * ctiles * nw * sruns * (a.d / 2 + 2) * 64 * sizeof(float);
}

template <int DQ, int D, int NW, int NBUF>
static void fused_launch_one(const FusedArgs& a, int spw, int ctiles, int sruns, float nsl) {
  const unsigned blocks = (unsigned)((long long)a.U * ctiles * sruns);
  hipLaunchKernelGGL((fused_mfma_kernel<DQ, D, NW, NBUF>), dim3(blocks), dim3(64 * NW), 0, a.stream,
                     (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,
                     (const unsigned short*)a.t0, (const unsigned short*)a.wq, (const unsigned short*)a.wk,
                     (const unsigned short*)a.wv, a.lens, a.C, a.L, a.w, a.S, spw, ctiles, sruns, nsl, a.z_out, a.seg_cnt,
                     a.work);
}

template <int DQ, int D>
static void fused_launch_nw(const FusedArgs& a, int nw, int spw, int ctiles, int sruns, float nsl) {
  if constexpr (D == 64) {
    if (nw == 8) return fused_launch_one<DQ, D, 8, 2>(a, spw, ctiles, sruns, nsl);
  }
  if (nw >= 4) fused_launch_one<DQ, D, 4, 2>(a, spw, ctiles, sruns, nsl);
  else if (nw == 2) fused_launch_one<DQ, D, 2, 1>(a, spw, ctiles, sruns, nsl);
  else fused_launch_one<DQ, D, 1, 1>(a, spw, ctiles, sruns, nsl);
}

laser_status fused_mfma_launch(const FusedArgs& a) {
  if (!fused_mfma_supports(a)) return LASER_ERR_UNSUPPORTED;
  const int nw = fused_nw(a);
  const int ctiles = (a.C + CW * nw - 1) / (CW * nw);
  int spw, sruns;
  fused_runs(a, nw, &spw, &sruns);
  const float nsl = -1.4426950408889634f / a.gamma;
  switch (a.d_q * 1000 + a.d) {
    case 32064: fused_launch_nw<32, 64>(a, nw, spw, ctiles, sruns, nsl); break;
    case 32128: fused_launch_nw<32, 128>(a, nw, spw, ctiles, sruns, nsl); break;
    case 64064: fused_launch_nw<64, 64>(a, nw, spw, ctiles, sruns, nsl); break;
    case 64128: fused_launch_nw<64, 128>(a, nw, spw, ctiles, sruns, nsl); break;
    case 128064: fused_launch_nw<128, 64>(a, nw, spw, ctiles, sruns, nsl); break;
    case 128128: fused_launch_nw<128, 128>(a, nw, spw, ctiles, sruns, nsl); break;
    default: return LASER_ERR_UNSUPPORTED;
  }
  if (launch_status() != LASER_OK) return LASER_ERR_LAUNCH;
  if (sruns == 1) return LASER_OK;
  const long long tiles = (long long)a.U * ctiles * nw;
  if (tiles > 0x7fffffffLL) return LASER_ERR_SHAPE;
  constexpr int NWM = 4;   // a workgroup per tile: four waves share the runs and the parking of W_v
  if (a.d == 64)
    hipLaunchKernelGGL((fused_merge_kernel<64, NWM>), dim3((unsigned)tiles), dim3(64 * NWM), 0, a.stream, a.work,
                       (const unsigned short*)a.t0, (const unsigned short*)a.wv, a.C, ctiles, nw, sruns, a.z_out);
  else
    hipLaunchKernelGGL((fused_merge_kernel<128, NWM>), dim3((unsigned)tiles), dim3(64 * NWM), 0, a.stream, a.work,
                       (const unsigned short*)a.t0, (const unsigned short*)a.wv, a.C, ctiles, nw, sruns, a.z_out);
  return launch_status();
}

}  // namespace laser
