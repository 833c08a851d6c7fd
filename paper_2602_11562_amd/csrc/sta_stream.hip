// STA for few candidates per user (C <= 8): an HBM streaming kernel on the vector ALUs.
//
// With one or a few candidates the STA equation of Sec. 3.4.2 does about one flop per byte of history read, so
// the matrix cores have nothing to amortise and the only thing that matters is that K and V are read once, in
// full 16-byte lanes, with enough loads in flight. One workgroup owns a user's run of consecutive segments (the
// whole user when there are enough users to fill the machine: a segment is a few tens of KB, too little to pay
// a workgroup launch, a length load and a query load for); it walks them one after the other, its four waves
// taking alternating chunks of the current segment's items. A K row is spread over d_q/8 lanes (16 bytes each), a V row over
// d/8 lanes: the score is an 8-term dot product per lane plus a shuffle tree over the row's lanes, the gate is
// evaluated once per (item, candidate), and each lane accumulates gate * v for its 8 value columns. Segment sums
// are then reduced across the row groups of a wave with shuffles and across the four waves through LDS in a
// fixed order (deterministic). Items at or past the valid length are never read (a partial chunk re-reads the
// segment's last valid row under a zero gate); empty segments are written as zeros.
#include <cstdlib>

#include "laser_internal.h"

namespace laser {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void unpack8(const u32x4& r, float (&x)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    x[2 * e] = __uint_as_float(r[e] << 16);
    x[2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u);
  }
}

// FUSED (the whole path with one GSTA layer and H' never stored; a workgroup then walks a whole user): every finished
// segment vector, still fp32 in the reduction buffer, goes through the online softmax of the layer of Sec. 3.4.3
// instead of to memory: r = W_k (t0 W_q)^T log2(e) / sqrt(d) per candidate first, then per segment the score
// H'_i . r, the running maximum and denominator, and the weighted sum P in LDS; z = t0 + (P / l) W_v at the end. The
// state is C <= 8 vectors per workgroup, and the layer's products are a few thousand multiply-adds per candidate, so
// they run on the vector ALUs from weights read through the caches.
struct StreamFusedTail {
  const unsigned short* t0;   // [P, D]
  const unsigned short* wq;   // [D, D] each
  const unsigned short* wk;
  const unsigned short* wv;
  float* z;                   // [P, D]
};

template <int DQ, int D, int CMAX, int HEADS, bool FUSED = false>
__global__ __launch_bounds__(256) void sta_stream_kernel(const unsigned short* __restrict__ q,
                                                         const unsigned short* __restrict__ k,
                                                         const unsigned short* __restrict__ v,
                                                         const int32_t* __restrict__ lens,
                                                         const int32_t* __restrict__ cand_off, int P, int C_all, int L,
                                                         int w, int S, int spg, int groups, int users, int classes,
                                                         float neg_scale_log2e,
                                                         unsigned short* __restrict__ seg_out,
                                                         int32_t* __restrict__ seg_cnt, StreamFusedTail ft) {
  constexpr int LQ = DQ / 8, LV = D / 8;           // lanes per K row / V row
  constexpr int RQ = 64 / LQ, RV = 64 / LV;        // rows per wave-wide load
  constexpr int IPC = RQ > RV ? RQ : RV;           // items per chunk
  constexpr int NKL = IPC / RQ, NVL = IPC / RV;    // loads per chunk
  constexpr bool SAME = (LQ == LV);
  // Several heads (Sec. 4.1.2): head h owns the h-th run of LQH lanes of a K row and of LVH lanes of a V row; a
  // score is summed over its head's lanes only, and a value lane takes the gate of its own head.
  constexpr int LQH = LQ / HEADS, LVH = LV / HEADS;
  static_assert(LQ % HEADS == 0 && LV % HEADS == 0, "a head's columns must fill whole 16-byte lanes");
  __shared__ float red[4][CMAX][D];
  __shared__ float gs[4][CMAX][HEADS][IPC];
  constexpr int FC = FUSED ? CMAX : 1, FD = FUSED ? D : 1;
  __shared__ float f_r[FC][FD], f_p[FC][FD], f_h[FC][FD];   // r, the weighted sum P, the segment vector just finished
  __shared__ float f_dot[FC][2], f_cw[FC][2], f_ml[FC][2];  // partial scores; (rescale, weight); (maximum, denominator)

  // Longest histories first. Workgroups start in index order and a long history keeps its workgroup busy many times
  // longer than a short one, so the launch would end with a few late starters of long users running alone. With
  // `classes` > 1 the grid holds every (user, run) once per length class, longest class first, and a workgroup
  // leaves at once unless its user's length falls in its class (lengths in (L/2, L], (L/4, L/2], (L/8, L/4], ...,
  // the last class takes the rest): an approximate longest-first order that needs no sorted list and no scratch.
  const int per_class = users * groups;
  const int cls = blockIdx.x / per_class, rest = blockIdx.x - cls * per_class;
  const int u = rest / groups, grp = rest % groups;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = valid_len(lens, u, L);
  if (classes > 1) {
    int mine = 0;
    while (mine < classes - 1 && n <= (L >> (mine + 1))) ++mine;
    if (mine != cls) return;   // (the whole workgroup, before any barrier)
  }
  if (grp == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, 256);
  const CandRange cr = cand_range(cand_off, u, C_all, P);
  const int C = cr.count;               // this user's candidates
  const size_t pb = (size_t)cr.first;   // and the index of their first pair
  if (C == 0) return;                   // (the whole workgroup leaves, before any barrier)
  const int rq = lane / LQ, cq = lane % LQ;
  const int rv = lane / LV, cv = lane % LV;

  float qf[CMAX][8];
#pragma unroll
  for (int c = 0; c < CMAX; ++c) {
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (c < C) raw = *reinterpret_cast<const u32x4*>(q + (pb + c) * DQ + cq * 8);
    unpack8(raw, qf[c]);
  }
  const unsigned short* kU = k + (size_t)u * L * DQ;
  const unsigned short* vU = v + (size_t)u * L * D;
  if constexpr (FUSED) {
    for (int e = tid; e < C * D; e += 256) {   // q' = t0 W_q
      const int c = e / D, col = e - c * D;
      float s = 0.0f;
#pragma unroll 8
      for (int a = 0; a < D; ++a) s = fmaf(bf16_bits_to_f32(ft.t0[(pb + c) * D + a]), bf16_bits_to_f32(ft.wq[a * D + col]), s);
      f_h[c][col] = s;
      f_p[c][col] = 0.0f;
    }
    if (tid < C) {
      f_ml[tid][0] = -1.0e30f;
      f_ml[tid][1] = 0.0f;
    }
    __syncthreads();
    const float rscale = 1.4426950408889634f / sqrtf((float)D);
    for (int e = tid; e < C * D; e += 256) {   // r = W_k q'^T
      const int c = e / D, row = e - c * D;
      float s = 0.0f;
#pragma unroll 8
      for (int a = 0; a < D; ++a) s = fmaf(bf16_bits_to_f32(ft.wk[row * D + a]), f_h[c][a], s);
      f_r[c][row] = s * rscale;
    }
    __syncthreads();
  }

  const int i_beg = grp * spg;
  const int i_end = (grp + 1) * spg < S ? (grp + 1) * spg : S;
  // valid items are a prefix of the history, so the non-empty segments of the run are a prefix of the run
  int i_ne = (n + w - 1) / w;
  if (i_ne > i_end) i_ne = i_end;
  if (i_ne < i_beg) i_ne = i_beg;
  auto seg_hi = [&](int i) {
    int hi = i * w + w;
    if (hi > L) hi = L;
    if (hi > n) hi = n;
    return hi;
  };

  // A step is UNR chunks per wave (4 waves x UNR x IPC items of one segment); all waves take the same steps. The
  // loads of the next step (possibly the next segment's first) are issued before the current step is consumed.
  // Rows at or past the end of the segment are read from its last valid row and get a zero gate: straight-line
  // loads, which the compiler can leave in flight behind the arithmetic.
  constexpr int UNR = 4, STRIDE = 4 * IPC * UNR;
  struct Regs { u32x4 k[UNR][NKL], v[UNR][NVL]; };
  auto load_step = [&](int base, int hi, Regs& r) {
#pragma unroll
    for (int uu = 0; uu < UNR; ++uu) {
      const int j0 = base + wave * IPC + uu * 4 * IPC;
#pragma unroll
      for (int kl = 0; kl < NKL; ++kl) {
        int row = j0 + kl * RQ + rq;
        row = row < hi ? row : hi - 1;
        r.k[uu][kl] = *reinterpret_cast<const u32x4*>(kU + (size_t)row * DQ + cq * 8);
      }
#pragma unroll
      for (int vl = 0; vl < NVL; ++vl) {
        int row = j0 + vl * RV + rv;
        row = row < hi ? row : hi - 1;
        r.v[uu][vl] = *reinterpret_cast<const u32x4*>(vU + (size_t)row * D + cv * 8);
      }
    }
  };
  float acc[CMAX][8];
  auto clear_acc = [&]() {
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[c][e] = 0.0f;
  };
  auto compute_step = [&](int base, int hi, const Regs& r) {
#pragma unroll
    for (int uu = 0; uu < UNR; ++uu) {
      const int j0 = base + wave * IPC + uu * 4 * IPC;
      float vf[NVL][8];
#pragma unroll
      for (int vl = 0; vl < NVL; ++vl) unpack8(r.v[uu][vl], vf[vl]);
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        if (c < C) {
#pragma unroll
          for (int kl = 0; kl < NKL; ++kl) {
            float kf[8];
            unpack8(r.k[uu][kl], kf);
            float s = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(kf[e], qf[c][e], s);
            s = row_sum<LQH>(s);
            const bool ok = (j0 + kl * RQ + rq) < hi;
            const float g = ok ? __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(s * neg_scale_log2e)) : 0.0f;
            if (SAME) {
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[c][e] = fmaf(g, vf[kl][e], acc[c][e]);
            } else if (cq % LQH == 0) {
              gs[wave][c][cq / LQH][kl * RQ + rq] = g;
            }
          }
          if (!SAME) {   // LDS operations of one wave execute in order: the gates written above are visible here
#pragma unroll
            for (int vl = 0; vl < NVL; ++vl) {
              const float g = gs[wave][c][cv / LVH][vl * RV + rv];   // 0 for rows past the end (written as such above)
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[c][e] = fmaf(g, vf[vl][e], acc[c][e]);
            }
          }
        }
      }
    }
  };
  // segment done: sum over the row groups of the wave, then over the four waves (fixed order), and store
  auto finish_segment = [&](int i) {
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      if (c < C) {
#pragma unroll
        for (int off = LV; off < 64; off <<= 1)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[c][e] += __shfl_xor(acc[c][e], off, 64);
        if (rv == 0) {
#pragma unroll
          for (int e = 0; e < 8; ++e) red[wave][c][cv * 8 + e] = acc[c][e];
        }
      }
    }
    __syncthreads();
    if constexpr (FUSED) {
      // the segment vector meets r: 64 consecutive components of one candidate per wave and round
      for (int e = tid; e < C * D; e += 256) {
        const int c = e / D, col = e - c * D;
        const float s = ((red[0][c][col] + red[1][c][col]) + red[2][c][col]) + red[3][c][col];
        f_h[c][col] = s;
        const float part = wave_sum(s * f_r[c][col]);
        if (lane == 0) f_dot[c][col >> 6] = part;
      }
      __syncthreads();
      if (tid < C) {   // online softmax over the segments, base 2
        const float e2 = D > 64 ? f_dot[tid][0] + f_dot[tid][1] : f_dot[tid][0];
        const float m_old = f_ml[tid][0], m_new = fmaxf(m_old, e2);
        const float corr = __builtin_amdgcn_exp2f(m_old - m_new), wgt = __builtin_amdgcn_exp2f(e2 - m_new);
        f_ml[tid][0] = m_new;
        f_ml[tid][1] = fmaf(f_ml[tid][1], corr, wgt);
        f_cw[tid][0] = corr;
        f_cw[tid][1] = wgt;
      }
      __syncthreads();
      for (int e = tid; e < C * D; e += 256) {
        const int c = e / D, col = e - c * D;
        f_p[c][col] = fmaf(f_cw[c][1], f_h[c][col], f_p[c][col] * f_cw[c][0]);
      }
    } else {
      for (int e = tid; e < C * D; e += 256) {
        const int c = e / D, col = e - c * D;
        const float s = ((red[0][c][col] + red[1][c][col]) + red[2][c][col]) + red[3][c][col];
        seg_out[((pb + c) * S + i) * D + col] = f32_to_bf16_bits(s);
      }
    }
    __syncthreads();   // the reduction buffer is reused by the next segment
  };

  if (i_beg < i_ne) {
    int ci = i_beg, cbase = i_beg * w, chi = seg_hi(i_beg);
    Regs cur, nxt;
    load_step(cbase, chi, cur);
    clear_acc();
    bool more = true;
    while (more) {
      int ni = ci, nbase = cbase + STRIDE, nhi = chi;
      if (nbase >= chi) {
        ni = ci + 1;
        nbase = ni * w;
        nhi = ni < i_ne ? seg_hi(ni) : 0;
      }
      more = ni < i_ne;
      if (more) load_step(nbase, nhi, nxt);
      compute_step(cbase, chi, cur);
      if (ni != ci) {
        finish_segment(ci);
        clear_acc();
      }
      cur = nxt;
      ci = ni;
      cbase = nbase;
      chi = nhi;
    }
  }
  if constexpr (FUSED) {   // z = t0 + (P / l) W_v (no valid segment: l = 0 and z = t0)
    __syncthreads();
    for (int e = tid; e < C * D; e += 256) {
      const int c = e / D, col = e - c * D;
      const float l = f_ml[c][1], inv = l > 0.0f ? 1.0f / l : 0.0f;
      float o = 0.0f;
#pragma unroll 8
      for (int a = 0; a < D; ++a) o = fmaf(f_p[c][a], bf16_bits_to_f32(ft.wv[a * D + col]), o);
      ft.z[(pb + c) * D + col] = bf16_bits_to_f32(ft.t0[(pb + c) * D + col]) + o * inv;
    }
    return;
  }
  // empty segments of the run: exact zeros
  for (int e = tid; e < (i_end - i_ne) * C * D; e += 256) {
    const int ii = i_ne + e / (C * D), r2 = e % (C * D);
    const int c = r2 / D, col = r2 - c * D;
    seg_out[((pb + c) * S + ii) * D + col] = 0;
  }
}

// Short segments (w below one step of the kernel above, e.g. the paper's w = 10 with L = 1000, Sec. 4.1.2
// "Implementation Details"): a step of four waves would cover one segment and leave most of its lanes idle, and
// every segment would pay two workgroup barriers. Here each wave owns whole segments (wave v takes segments
// v, v + 4, ... of the run), reduces them inside the wave and stores them itself: no LDS reduction, no barrier.
// Chunks of IPC items are loaded one ahead (the next chunk of the segment or the first of the wave's next one).
// SOFTMAX: the ablation variant of Sec. 4.4.1 (softmax over the valid items of a segment instead of independent
// sigmoid gates). Every value lane keeps a running maximum m and denominator l of its row group's scores (base 2)
// beside its sums, rescaling them when the maximum moves; at the end of a segment the row groups agree on the
// largest maximum, rescale once more, and the reduced sums are divided by the reduced denominator.
template <int DQ, int D, int CMAX, int HEADS, bool SOFTMAX>
__global__ __launch_bounds__(256) void sta_stream_short_kernel(const unsigned short* __restrict__ q,
                                                               const unsigned short* __restrict__ k,
                                                               const unsigned short* __restrict__ v,
                                                               const int32_t* __restrict__ lens,
                                                               const int32_t* __restrict__ cand_off, int P, int C_all,
                                                               int L, int w, int S, int spg, int groups,
                                                               float neg_scale_log2e,
                                                               unsigned short* __restrict__ seg_out,
                                                               int32_t* __restrict__ seg_cnt, int kv_alias) {
  constexpr int LQ = DQ / 8, LV = D / 8;
  constexpr int RQ = 64 / LQ, RV = 64 / LV;
  constexpr int IPC = RQ > RV ? RQ : RV;
  constexpr int NKL = IPC / RQ, NVL = IPC / RV;
  constexpr bool SAME = (LQ == LV);
  // kv_alias: keys and values are the same array (the folded form runs STA over the raw items); with equal widths a
  // lane's value piece is its key piece, and the value loads are left out
  const bool alias = SAME && kv_alias != 0;
  constexpr int LQH = LQ / HEADS, LVH = LV / HEADS;   // lanes per head, as in the kernel above
  static_assert(LQ % HEADS == 0 && LV % HEADS == 0, "a head's columns must fill whole 16-byte lanes");
  __shared__ float gs[4][CMAX][HEADS][IPC];

  const int u = blockIdx.x / groups, grp = blockIdx.x % groups;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = __builtin_amdgcn_readfirstlane(valid_len(lens, u, L));
  if (grp == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, 256);
  const CandRange cr = cand_range(cand_off, u, C_all, P);
  const int C = __builtin_amdgcn_readfirstlane(cr.count);   // this user's candidates
  const size_t pb = (size_t)cr.first;                        // and the index of their first pair
  if (C == 0) return;
  const int rq = lane / LQ, cq = lane % LQ;
  const int rv = lane / LV, cv = lane % LV;

  float qf[CMAX][8];
#pragma unroll
  for (int c = 0; c < CMAX; ++c) {
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (c < C) raw = *reinterpret_cast<const u32x4*>(q + (pb + c) * DQ + cq * 8);
    unpack8(raw, qf[c]);
  }
  const unsigned short* kU = k + (size_t)u * L * DQ;
  const unsigned short* vU = v + (size_t)u * L * D;

  const int i_beg = grp * spg;
  const int i_end = (grp + 1) * spg < S ? (grp + 1) * spg : S;
  int i_ne = (n + w - 1) / w;   // non-empty segments of the run are a prefix of it
  if (i_ne > i_end) i_ne = i_end;
  if (i_ne < i_beg) i_ne = i_beg;
  auto seg_hi = [&](int i) {
    int hi = i * w + w;
    if (hi > L) hi = L;
    if (hi > n) hi = n;
    return hi;
  };

  struct Regs { u32x4 k[NKL], v[NVL]; };
  // rows at or past the end of the segment are read from its last valid row and get a zero gate
  auto load_chunk = [&](int base, int hi, Regs& r) {
#pragma unroll
    for (int kl = 0; kl < NKL; ++kl) {
      int row = base + kl * RQ + rq;
      row = row < hi ? row : hi - 1;
      r.k[kl] = *reinterpret_cast<const u32x4*>(kU + (size_t)row * DQ + cq * 8);
    }
    if (alias) {
#pragma unroll
      for (int vl = 0; vl < NVL; ++vl) r.v[vl] = r.k[vl < NKL ? vl : 0];
      return;
    }
#pragma unroll
    for (int vl = 0; vl < NVL; ++vl) {
      int row = base + vl * RV + rv;
      row = row < hi ? row : hi - 1;
      r.v[vl] = *reinterpret_cast<const u32x4*>(vU + (size_t)row * D + cv * 8);
    }
  };
  float acc[CMAX][8];
  constexpr float NEG = -1.0e30f;      // "no score yet": finite, so that differences of maxima stay finite
  float sm_m[CMAX], sm_l[CMAX];        // softmax state (unused otherwise)
  auto clear_acc = [&]() {
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[c][e] = 0.0f;
      sm_m[c] = NEG;
      sm_l[c] = 0.0f;
    }
  };
  // one row's share of the softmax: t = score * log2(e) / gamma of a valid row, or nothing for a row past the end
  auto softmax_row = [&](int c, float t, bool ok, const float (&vrow)[8]) {
    const float m_new = ok ? fmaxf(sm_m[c], t) : sm_m[c];
    const float sc = __builtin_amdgcn_exp2f(sm_m[c] - m_new);
    const float pr = ok ? __builtin_amdgcn_exp2f(t - m_new) : 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[c][e] = fmaf(pr, vrow[e], acc[c][e] * sc);
    sm_l[c] = fmaf(sm_l[c], sc, pr);
    sm_m[c] = m_new;
  };
  auto compute_chunk = [&](int base, int hi, const Regs& r) {
    float vf[NVL][8];
#pragma unroll
    for (int vl = 0; vl < NVL; ++vl) unpack8(r.v[vl], vf[vl]);
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      if (c < C) {
#pragma unroll
        for (int kl = 0; kl < NKL; ++kl) {
          float kf[8];
          unpack8(r.k[kl], kf);
          float s = 0.0f;
#pragma unroll
          for (int e = 0; e < 8; ++e) s = fmaf(kf[e], qf[c][e], s);
          s = row_sum<LQH>(s);
          const bool ok = (base + kl * RQ + rq) < hi;
          if (SOFTMAX) {
            const float t = -s * neg_scale_log2e;
            if (SAME) softmax_row(c, t, ok, vf[kl]);
            else if (cq % LQH == 0) gs[wave][c][cq / LQH][kl * RQ + rq] = t;
            continue;
          }
          const float g = ok ? __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(s * neg_scale_log2e)) : 0.0f;
          if (SAME) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[c][e] = fmaf(g, vf[kl][e], acc[c][e]);
          } else if (cq % LQH == 0) {
            gs[wave][c][cq / LQH][kl * RQ + rq] = g;
          }
        }
        if (!SAME) {   // LDS operations of one wave execute in order: the gates written above are visible here
#pragma unroll
          for (int vl = 0; vl < NVL; ++vl) {
            const float g = gs[wave][c][cv / LVH][vl * RV + rv];
            if (SOFTMAX) {
              softmax_row(c, g, (base + vl * RV + rv) < hi, vf[vl]);
              continue;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[c][e] = fmaf(g, vf[vl][e], acc[c][e]);
          }
        }
      }
    }
  };
  auto finish_segment = [&](int i) {   // sum over the row groups of the wave, one 16-byte store per value lane
    float inv_l[CMAX];
    if constexpr (SOFTMAX) {
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        inv_l[c] = 0.0f;
        if (c < C) {
          float mx = sm_m[c];
#pragma unroll
          for (int off = LV; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
          const float sc = __builtin_amdgcn_exp2f(sm_m[c] - mx);   // 0 for a row group that saw no valid row
          float lsum = sm_l[c] * sc;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[c][e] *= sc;
#pragma unroll
          for (int off = LV; off < 64; off <<= 1) lsum += __shfl_xor(lsum, off, 64);
          inv_l[c] = 1.0f / lsum;   // a segment that is finished holds at least one valid item
        }
      }
    }
    if constexpr (LV == 16) {
      // Four row groups of 16 lanes: a reduce-scatter with the lane-swap instructions instead of 16 shuffles per
      // candidate. v_permlane32_swap exchanges lanes 32..63 of its first operand with lanes 0..31 of its second,
      // so first + second leaves the first value summed over row groups (g, g + 2) in the lower half and the second
      // value in the upper half; v_permlane16_swap (odd rows of the first with even rows of the second) does the
      // same for neighbouring rows. A lane of row g ends with values 2g and 2g + 1 of its eight, summed over all
      // four groups in a fixed order, and the wave writes the 256-byte row in one 4-byte-per-lane store.
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        if (c < C) {
          float y[4], z[2];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[c][e]), __float_as_uint(acc[c][e + 4]),
                                                            false, false);
            y[e] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
          }
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(y[e]), __float_as_uint(y[e + 2]), false,
                                                            false);
            z[e] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
          }
          if (SOFTMAX) {
            z[0] *= inv_l[c];
            z[1] *= inv_l[c];
          }
          const unsigned o = (unsigned)f32_to_bf16_bits(z[0]) | ((unsigned)f32_to_bf16_bits(z[1]) << 16);
          *reinterpret_cast<unsigned*>(seg_out + ((pb + c) * S + i) * D + cv * 8 + 2 * (lane >> 4)) = o;
        }
      }
      return;
    }
#pragma unroll
    for (int c = 0; c < CMAX; ++c) {
      if (c < C) {
#pragma unroll
        for (int off = LV; off < 64; off <<= 1)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[c][e] += __shfl_xor(acc[c][e], off, 64);
        if (rv == 0) {
          u32x4 o;
          const float mul = SOFTMAX ? inv_l[c] : 1.0f;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            o[e] = (unsigned)f32_to_bf16_bits(acc[c][2 * e] * mul) |
                   ((unsigned)f32_to_bf16_bits(acc[c][2 * e + 1] * mul) << 16);
          *reinterpret_cast<u32x4*>(seg_out + ((pb + c) * S + i) * D + cv * 8) = o;
        }
      }
    }
  };

  int ci = i_beg + wave;
  if (ci < i_ne) {
    int cbase = ci * w, chi = seg_hi(ci);
    Regs cur, nxt;
    load_chunk(cbase, chi, cur);
    clear_acc();
    bool more = true;
    while (more) {
      int ni = ci, nbase = cbase + IPC, nhi = chi;
      if (nbase >= chi) {
        ni = ci + 4;
        nbase = ni * w;
        nhi = ni < i_ne ? seg_hi(ni) : 0;
      }
      more = ni < i_ne;
      if (more) load_chunk(nbase, nhi, nxt);
      compute_chunk(cbase, chi, cur);
      if (ni != ci) {
        finish_segment(ci);
        clear_acc();
      }
      cur = nxt;
      ci = ni;
      cbase = nbase;
      chi = nhi;
    }
  }
  // empty segments of the run: exact zeros
  for (int e = tid; e < (i_end - i_ne) * C * D; e += 256) {
    const int ii = i_ne + e / (C * D), r2 = e % (C * D);
    const int c = r2 / D, col = r2 - c * D;
    seg_out[((pb + c) * S + ii) * D + col] = 0;
  }
}

// ------------------------------------------------------------------------------------------ host side
bool sta_stream_supports(const StaArgs& a) {
  if (a.dt != LASER_BF16) return false;
  if (a.C > 8) return false;
  if (a.heads != 1 && a.heads != 2) return false;
  if (a.softmax) {   // only the short-segment form carries the softmax state
    const int lq = a.d_q / 8, lv = a.d / 8;
    const int ipc = (64 / lq) > (64 / lv) ? (64 / lq) : (64 / lv);
    if (a.w >= 4 * 4 * ipc) return false;
  }
  if (!(a.d_q == 32 || a.d_q == 64 || a.d_q == 128)) return false;
  if (!(a.d == 64 || a.d == 128)) return false;
  return (long long)a.U * a.S <= 0x7fffffffLL;   // an upper bound of the grid size
}

template <int DQ, int D, int HEADS>
static void launch_c(const StaArgs& a, float nsl) {
  // runs of segments per user: the whole user per workgroup once that still gives every compute unit eight
  // workgroups, shorter runs when there are few users
  int groups = (2048 + a.U - 1) / a.U;
  if (groups > a.S) groups = a.S;
  int spg = (a.S + groups - 1) / groups;
  // a step of the long form covers 4 waves x 4 chunks of IPC items; shorter segments go wave by wave
  constexpr int IPC_ = (64 / (DQ / 8)) > (64 / (D / 8)) ? (64 / (DQ / 8)) : (64 / (D / 8));
  const bool short_seg = a.w < 4 * 4 * IPC_;
  // short segments are cheap to start on (a wave owns whole segments, nothing is shared), and histories differ in
  // length: runs of a dozen segments (three per wave) even out the load where whole users do not (measured on
  // 2048 users x 100 segments of 10 items with lengths between 200 and 1000: 110 us -> 86 us)
  if (short_seg && spg > 12) spg = 12;
  const int spg_forced = tuning_int("LASER_STREAM_SPG", 0);   // tuning builds only
  if (spg_forced >= 1 && spg_forced <= a.S) spg = spg_forced;
  groups = (a.S + spg - 1) / spg;
  const unsigned blocks = (unsigned)((long long)a.U * groups);
  // length classes (long form only): worth their empty workgroups once the launch is several rounds of workgroups
  // and the lengths differ at all (4096 users with log-uniform lengths 64..4096: 206 us with one class, 193 with
  // two, 182 with four, 186 with eight)
  int classes = (a.lens != nullptr && blocks >= 4096 && (unsigned long long)blocks * 4 <= 0x7fffffffULL) ? 4 : 1;
  const int cls_forced = tuning_int("LASER_STREAM_CLASSES", 0);   // tuning builds only
  if (cls_forced >= 1 && cls_forced <= 8 && (unsigned long long)blocks * cls_forced <= 0x7fffffffULL) classes = cls_forced;
#define LASER_STREAM_LAUNCH(CM)                                                                                      \
  do {                                                                                                               \
    if (short_seg && a.softmax)                                                                                      \
      hipLaunchKernelGGL((sta_stream_short_kernel<DQ, D, CM, HEADS, true>), dim3(blocks), dim3(256), 0, a.stream,  \
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,       \
                         a.lens, a.cand_off, a.P, a.C, a.L, a.w, a.S, spg, groups, nsl, (unsigned short*)a.seg_out, a.seg_cnt,     \
                         (a.k == a.v && DQ == D) ? 1 : 0);                                                           \
    else if (short_seg)                                                                                              \
      hipLaunchKernelGGL((sta_stream_short_kernel<DQ, D, CM, HEADS, false>), dim3(blocks), dim3(256), 0, a.stream, \
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,       \
                         a.lens, a.cand_off, a.P, a.C, a.L, a.w, a.S, spg, groups, nsl, (unsigned short*)a.seg_out, a.seg_cnt,     \
                         (a.k == a.v && DQ == D) ? 1 : 0);                                                           \
    else                                                                                                             \
      hipLaunchKernelGGL((sta_stream_kernel<DQ, D, CM, HEADS>), dim3(blocks * classes), dim3(256), 0, a.stream,    \
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,       \
                         a.lens, a.cand_off, a.P, a.C, a.L, a.w, a.S, spg, groups, a.U, classes, nsl,               \
                         (unsigned short*)a.seg_out, a.seg_cnt, StreamFusedTail{});                                  \
  } while (0)
  if (a.C <= 1) LASER_STREAM_LAUNCH(1);
  else if (a.C <= 2) LASER_STREAM_LAUNCH(2);
  else if (a.C <= 4) LASER_STREAM_LAUNCH(4);
  else LASER_STREAM_LAUNCH(8);
#undef LASER_STREAM_LAUNCH
}

// The fused form (FusedArgs: the whole path, H' never stored): the long-segment kernel, a whole user per workgroup
bool fused_stream_supports(const FusedArgs& a) {
  if (a.dt != LASER_BF16 || a.C > 8) return false;
  if (!(a.d_q == 32 || a.d_q == 64 || a.d_q == 128) || !(a.d == 64 || a.d == 128)) return false;
  const int lq = a.d_q / 8, lv = a.d / 8;
  const int ipc = (64 / lq) > (64 / lv) ? (64 / lq) : (64 / lv);
  if (a.w < 4 * 4 * ipc) return false;   // short segments go wave by wave (another kernel, not fused)
  return (long long)a.U * 4 <= 0x7fffffffLL;
}

template <int DQ, int D>
static void fused_stream_launch_c(const FusedArgs& a, float nsl) {
  const unsigned blocks = (unsigned)a.U;   // a workgroup walks a whole user: spg = S, one group
  const int classes = (a.lens != nullptr && blocks >= 4096) ? 4 : 1;   // longest histories first, as above
  const StreamFusedTail ft{(const unsigned short*)a.t0, (const unsigned short*)a.wq, (const unsigned short*)a.wk,
                           (const unsigned short*)a.wv, a.z_out};
#define LASER_FUSED_STREAM(CM)                                                                                       \
  hipLaunchKernelGGL((sta_stream_kernel<DQ, D, CM, 1, true>), dim3(blocks * classes), dim3(256), 0, a.stream,        \
                     (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,     \
                     (const int32_t*)nullptr, 0, a.C, a.L, a.w, a.S, a.S, 1, a.U, classes, nsl,                      \
                     (unsigned short*)nullptr, a.seg_cnt, ft)
  if (a.C <= 1) LASER_FUSED_STREAM(1);
  else if (a.C <= 2) LASER_FUSED_STREAM(2);
  else if (a.C <= 4) LASER_FUSED_STREAM(4);
  else LASER_FUSED_STREAM(8);
#undef LASER_FUSED_STREAM
}

laser_status fused_stream_launch(const FusedArgs& a) {
  if (!fused_stream_supports(a)) return LASER_ERR_UNSUPPORTED;
  const float nsl = -1.4426950408889634f / a.gamma;
  switch (a.d_q * 1000 + a.d) {
    case 32064: fused_stream_launch_c<32, 64>(a, nsl); break;
    case 32128: fused_stream_launch_c<32, 128>(a, nsl); break;
    case 64064: fused_stream_launch_c<64, 64>(a, nsl); break;
    case 64128: fused_stream_launch_c<64, 128>(a, nsl); break;
    case 128064: fused_stream_launch_c<128, 64>(a, nsl); break;
    case 128128: fused_stream_launch_c<128, 128>(a, nsl); break;
    default: return LASER_ERR_UNSUPPORTED;
  }
  return launch_status();
}

laser_status sta_stream_launch(const StaArgs& a) {
  if (!sta_stream_supports(a)) return LASER_ERR_UNSUPPORTED;
  const float nsl = -1.4426950408889634f / a.gamma;
  const int key = a.d_q * 1000 + a.d;
#define LASER_STREAM_SHAPE(DQ_, D_)                    \
  if (a.heads == 2) launch_c<DQ_, D_, 2>(a, nsl);      \
  else launch_c<DQ_, D_, 1>(a, nsl);                   \
  break
  switch (key) {
    case 32064: LASER_STREAM_SHAPE(32, 64);
    case 32128: LASER_STREAM_SHAPE(32, 128);
    case 64064: LASER_STREAM_SHAPE(64, 64);
    case 64128: LASER_STREAM_SHAPE(64, 128);
    case 128064: LASER_STREAM_SHAPE(128, 64);
    case 128128: LASER_STREAM_SHAPE(128, 128);
    default: return LASER_ERR_UNSUPPORTED;
  }
#undef LASER_STREAM_SHAPE
  return launch_status();
}

}  // namespace laser
