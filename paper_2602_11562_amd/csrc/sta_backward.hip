// Backward pass of STA for few candidates per user (training batches hold one target per sample; paper Sec. 4.1.2
// trains with batches of 2048 such samples). Derivatives of the forward equations of Sec. 3.4.2,
//   H'[c,i,:] = sum_{j in segment i, j < len} g_cj v_j,   g_cj = sigmoid(q_c . k_j / gamma):
//   dv_j = sum_c g_cj dH'[c,i(j),:]                         dk_j = sum_c ds_cj q_c / gamma
//   ds_cj = (dH'[c,i(j),:] . v_j) g_cj (1 - g_cj)           dq_c = sum_j ds_cj k_j / gamma
// Like the forward pass with few candidates this is HBM streaming work (K and V read once, dk and dv written once),
// so the work is dealt as in the streaming kernels: a workgroup owns a user's run of consecutive segments and its
// four waves take alternating segments. Two kernels share that frame.
// sta_bwd_kernel (any widths up to 256, either storage type, up to eight candidates): a wave holds one item at a
// time, lane l the elements l, l + 64, ... of its key and value rows; the two dot products per (item, candidate) are
// wave-wide sums, after which every lane knows the gate and ds and updates its own elements of dv_j, dk_j (stored once
// per item, fp32) and of dq_c (kept in registers over the run). The queries and the upstream gradient of the current
// segment sit in registers in the same lane layout.
// sta_bwd_wide_kernel (bf16, the usual widths, up to four candidates; further down): the forward kernels' lane layout,
// several items per wave-wide load.
// In both, dq is summed over a workgroup's waves in LDS and over a user's workgroups by a second small kernel, in a
// fixed order (deterministic), and items at or past the valid length get zero gradients.
#include <cstdlib>
#include <type_traits>

#include "laser_internal.h"

namespace laser {

constexpr int SB_CMAX = 8;    // candidates per user
constexpr int SB_TMAX = 4;    // 64-element slices per row: d_q, d <= 256

template <typename T, int TQ, int TV, int CMAX>   // TQ, TV: 64-element slices of a key / value row; CMAX >= C
__global__ __launch_bounds__(256) void sta_bwd_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                      const T* __restrict__ v, const T* __restrict__ dhp,
                                                      const int32_t* __restrict__ lens, int C_all, int c0, int C,
                                                      int accumulate, int L, int dq, int d, int w,
                                                      int S, int spg, int groups, int users, int classes,
                                                      float neg_scale_log2e, float inv_gamma,
                                                      float* __restrict__ dk, float* __restrict__ dv,
                                                      float* __restrict__ dq_part) {
  extern __shared__ float red[];        // [4][C][dq] per-wave dq sums at the end of the run
  // longest histories first (length classes, as in the forward streaming kernel): the grid holds every (user, run)
  // once per class and a workgroup leaves at once unless its user's length falls in its class
  const int per_class = users * groups;
  const int cls = blockIdx.x / per_class, rest = blockIdx.x - cls * per_class;
  const int u = rest / groups, grp = rest % groups;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = __builtin_amdgcn_readfirstlane(valid_len(lens, u, L));
  if (classes > 1) {
    int mine = 0;
    while (mine < classes - 1 && n <= (L >> (mine + 1))) ++mine;
    if (mine != cls) return;   // (the whole workgroup, before any barrier)
  }
  const int i_beg = grp * spg;
  const int i_end = (grp + 1) * spg < S ? (grp + 1) * spg : S;
  const T* kU = k + (size_t)u * L * dq;
  const T* vU = v + (size_t)u * L * d;
  float* dkU = dk + (size_t)u * L * dq;
  float* dvU = dv + (size_t)u * L * d;

  // queries and dq sums: lane l holds elements l, l + 64, ... of every candidate's row
  float qr[CMAX][TQ], dqacc[CMAX][TQ];
#pragma unroll
  for (int c = 0; c < CMAX; ++c)
#pragma unroll
    for (int t = 0; t < TQ; ++t) {
      const int e = lane + 64 * t;
      qr[c][t] = (c < C && e < dq) ? load_as_f32(q, ((size_t)u * C_all + c0 + c) * dq + e) : 0.0f;
      dqacc[c][t] = 0.0f;
    }

  // A wave owns whole segments (wave v takes segments i_beg + v, + 4, ... of the run): the upstream gradient of a
  // segment is read into registers once, and nothing is shared between waves until the run ends.
  for (int i = i_beg + wave; i < i_end; i += 4) {
    const int lo = i * w;
    int hi_all = lo + w;
    if (hi_all > L) hi_all = L;
    const int hi = hi_all < n ? hi_all : n;      // valid items of the segment: [lo, hi)
    if (hi > lo) {
      float dh[CMAX][TV];
#pragma unroll
      for (int c = 0; c < CMAX; ++c)
#pragma unroll
        for (int t = 0; t < TV; ++t) {
          const int e = lane + 64 * t;
          dh[c][t] = (c < C && e < d) ? load_as_f32(dhp, (((size_t)u * C_all + c0 + c) * S + i) * d + e) : 0.0f;
        }
      // the rows of the next item are requested before the current one is worked on (an item is a chain of load, two
      // wave-wide sums, a gate and two stores; only other waves and this prefetch hide the load)
      float kn[TQ], vn[TV];
      auto load_item = [&](int j) {
#pragma unroll
        for (int t = 0; t < TQ; ++t) kn[t] = (lane + 64 * t < dq) ? load_as_f32(kU, (size_t)j * dq + lane + 64 * t) : 0.0f;
#pragma unroll
        for (int t = 0; t < TV; ++t) vn[t] = (lane + 64 * t < d) ? load_as_f32(vU, (size_t)j * d + lane + 64 * t) : 0.0f;
      };
      load_item(lo);
      for (int j = lo; j < hi; ++j) {
        float kr[TQ], vr[TV], dka[TQ], dva[TV];
#pragma unroll
        for (int t = 0; t < TQ; ++t) { kr[t] = kn[t]; dka[t] = 0.0f; }
#pragma unroll
        for (int t = 0; t < TV; ++t) { vr[t] = vn[t]; dva[t] = 0.0f; }
        if (j + 1 < hi) load_item(j + 1);
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
          if (c < C) {
            float s = 0.0f, dot = 0.0f;
#pragma unroll
            for (int t = 0; t < TQ; ++t) s = fmaf(kr[t], qr[c][t], s);
#pragma unroll
            for (int t = 0; t < TV; ++t) dot = fmaf(vr[t], dh[c][t], dot);
            s = wave_sum_rows(s);
            dot = wave_sum_rows(dot);
            const float g = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(s * neg_scale_log2e));
            const float ds = dot * g * (1.0f - g) * inv_gamma;   // d loss / d (q_c . k_j)
#pragma unroll
            for (int t = 0; t < TV; ++t) dva[t] = fmaf(g, dh[c][t], dva[t]);
#pragma unroll
            for (int t = 0; t < TQ; ++t) {
              dka[t] = fmaf(ds, qr[c][t], dka[t]);
              dqacc[c][t] = fmaf(ds, kr[t], dqacc[c][t]);
            }
          }
        }
        // (a later block of candidates adds to what the blocks before it left: the same wave owned the item then)
#pragma unroll
        for (int t = 0; t < TQ; ++t)
          if (lane + 64 * t < dq) {
            float* o = dkU + (size_t)j * dq + lane + 64 * t;
            *o = accumulate ? *o + dka[t] : dka[t];
          }
#pragma unroll
        for (int t = 0; t < TV; ++t)
          if (lane + 64 * t < d) {
            float* o = dvU + (size_t)j * d + lane + 64 * t;
            *o = accumulate ? *o + dva[t] : dva[t];
          }
      }
    }
    // items of the segment at or past the valid length: zero gradients
    // (16 bytes per lane: rows are multiples of eight elements and the outputs 16-byte aligned)
    const int z0 = hi > lo ? hi : lo;
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4* zk = reinterpret_cast<f32x4*>(dkU + (size_t)z0 * dq);
    f32x4* zv = reinterpret_cast<f32x4*>(dvU + (size_t)z0 * d);
    if (!accumulate) {
      for (int e = lane; e < (hi_all - z0) * dq / 4; e += 64) __builtin_nontemporal_store(zero4, zk + e);
      for (int e = lane; e < (hi_all - z0) * d / 4; e += 64) __builtin_nontemporal_store(zero4, zv + e);
    }
  }
  // dq of the run: waves in a fixed order
#pragma unroll
  for (int c = 0; c < CMAX; ++c)
    if (c < C)
#pragma unroll
      for (int t = 0; t < TQ; ++t)
        if (lane + 64 * t < dq) red[(wave * C + c) * dq + lane + 64 * t] = dqacc[c][t];
  __syncthreads();
  for (int e = tid; e < C * dq; e += 256)
    dq_part[(((size_t)u * groups + grp) * C_all + c0) * dq + e] =
        ((red[e] + red[C * dq + e]) + red[2 * C * dq + e]) + red[3 * C * dq + e];
}

// The same computation in the lane layout of the forward streaming kernels, for bf16 storage and the usual widths:
// a key row is spread over d_q / 8 lanes and a value row over d / 8 lanes (16 bytes each), so one wave-wide load
// brings several items, and every instruction below works on 4 to 16 items at once instead of one. The two dot
// products of an (item, candidate) live on different lanes when the widths differ (the score on the key lanes, the
// product dH' . v on the value lanes), and each side needs the other's result (the value lanes the gate, the key
// lanes ds): they change sides through a wave-private LDS patch (LDS operations of a wave execute in order).
typedef unsigned int u32x4b __attribute__((ext_vector_type(4)));
typedef float f32x4b __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void unpack8b(const u32x4b& r, float (&x)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    x[2 * e] = __uint_as_float(r[e] << 16);
    x[2 * e + 1] = __uint_as_float(r[e] & 0xffff0000u);
  }
}

// GB16: dk and dv are written in bf16 (the storage type of k and v: half the bytes of the two largest outputs) instead
// of fp32; the sums are fp32 either way and rounded once.
template <int DQ, int D, int CMAX, bool GB16>
__global__ __launch_bounds__(256) void sta_bwd_wide_kernel(const unsigned short* __restrict__ q,
                                                           const unsigned short* __restrict__ k,
                                                           const unsigned short* __restrict__ v,
                                                           const unsigned short* __restrict__ dhp,
                                                           const int32_t* __restrict__ lens, int C, int L, int w, int S,
                                                           int spg, int groups, int users, int classes,
                                                           float neg_scale_log2e, float inv_gamma,
                                                           void* __restrict__ dk, void* __restrict__ dv,
                                                           float* __restrict__ dq_part) {
  typedef typename std::conditional<GB16, unsigned short, float>::type G;   // element type of dk and dv
  constexpr int LQ = DQ / 8, LV = D / 8;           // lanes per key row / value row
  constexpr int RQ = 64 / LQ, RV = 64 / LV;        // rows per wave-wide load
  constexpr int IPC = RQ > RV ? RQ : RV;           // items per chunk
  constexpr int NKL = IPC / RQ, NVL = IPC / RV;    // loads per chunk
  constexpr bool SAME = (LQ == LV);
  __shared__ float xg[4][CMAX][IPC];               // gate per item, key lanes -> value lanes
  __shared__ float xd[4][CMAX][IPC];               // dH' . v per item, value lanes -> key lanes
  __shared__ float red[4][CMAX][DQ];

  // longest histories first (length classes, as in the forward streaming kernel): the grid holds every (user, run)
  // once per class and a workgroup leaves at once unless its user's length falls in its class
  const int per_class = users * groups;
  const int cls = blockIdx.x / per_class, rest = blockIdx.x - cls * per_class;
  const int u = rest / groups, grp = rest % groups;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = __builtin_amdgcn_readfirstlane(valid_len(lens, u, L));
  if (classes > 1) {
    int mine = 0;
    while (mine < classes - 1 && n <= (L >> (mine + 1))) ++mine;
    if (mine != cls) return;   // (the whole workgroup, before any barrier)
  }
  const int rq = lane / LQ, cq = lane % LQ;
  const int rv = lane / LV, cv = lane % LV;
  const int i_beg = grp * spg;
  const int i_end = (grp + 1) * spg < S ? (grp + 1) * spg : S;
  const unsigned short* kU = k + (size_t)u * L * DQ;
  const unsigned short* vU = v + (size_t)u * L * D;
  G* dkU = static_cast<G*>(dk) + (size_t)u * L * DQ;
  G* dvU = static_cast<G*>(dv) + (size_t)u * L * D;
  auto store8 = [](G* dst, const float (&x)[8]) {   // eight consecutive gradient values: 16 or 32 bytes
    if constexpr (GB16) {
      u32x4b o;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = (unsigned)f32_to_bf16_bits(x[2 * e]) | ((unsigned)f32_to_bf16_bits(x[2 * e + 1]) << 16);
      *reinterpret_cast<u32x4b*>(dst) = o;
    } else {
      f32x4b* d4 = reinterpret_cast<f32x4b*>(dst);
      d4[0] = f32x4b{x[0], x[1], x[2], x[3]};
      d4[1] = f32x4b{x[4], x[5], x[6], x[7]};
    }
  };

  float qf[CMAX][8], dqacc[CMAX][8];
#pragma unroll
  for (int c = 0; c < CMAX; ++c) {
    u32x4b raw = {0u, 0u, 0u, 0u};
    if (c < C) raw = *reinterpret_cast<const u32x4b*>(q + ((size_t)u * C + c) * DQ + cq * 8);
    unpack8b(raw, qf[c]);
#pragma unroll
    for (int e = 0; e < 8; ++e) dqacc[c][e] = 0.0f;
  }

  for (int i = i_beg + wave; i < i_end; i += 4) {   // a wave owns whole segments
    const int lo = i * w;
    int hi_all = lo + w;
    if (hi_all > L) hi_all = L;
    const int hi = hi_all < n ? hi_all : n;          // valid items of the segment: [lo, hi)
    if (hi > lo) {
      float dh[CMAX][8];                             // this lane's piece of the segment's upstream gradient rows
#pragma unroll
      for (int c = 0; c < CMAX; ++c) {
        u32x4b raw = {0u, 0u, 0u, 0u};
        if (c < C) raw = *reinterpret_cast<const u32x4b*>(dhp + (((size_t)u * C + c) * S + i) * D + cv * 8);
        unpack8b(raw, dh[c]);
      }
      u32x4b kn[NKL], vn[NVL];
      // rows at or past the end of the segment are read from its last valid row and take no part (zero gate)
      auto load_chunk = [&](int base) {
#pragma unroll
        for (int kl = 0; kl < NKL; ++kl) {
          int row = base + kl * RQ + rq;
          row = row < hi ? row : hi - 1;
          kn[kl] = *reinterpret_cast<const u32x4b*>(kU + (size_t)row * DQ + cq * 8);
        }
#pragma unroll
        for (int vl = 0; vl < NVL; ++vl) {
          int row = base + vl * RV + rv;
          row = row < hi ? row : hi - 1;
          vn[vl] = *reinterpret_cast<const u32x4b*>(vU + (size_t)row * D + cv * 8);
        }
      };
      load_chunk(lo);
      for (int base = lo; base < hi; base += IPC) {
        float kf[NKL][8], vf[NVL][8], dka[NKL][8], dva[NVL][8];
#pragma unroll
        for (int kl = 0; kl < NKL; ++kl) {
          unpack8b(kn[kl], kf[kl]);
#pragma unroll
          for (int e = 0; e < 8; ++e) dka[kl][e] = 0.0f;
        }
#pragma unroll
        for (int vl = 0; vl < NVL; ++vl) {
          unpack8b(vn[vl], vf[vl]);
#pragma unroll
          for (int e = 0; e < 8; ++e) dva[vl][e] = 0.0f;
        }
        if (base + IPC < hi) load_chunk(base + IPC);   // the next chunk is on its way during the arithmetic
#pragma unroll
        for (int c = 0; c < CMAX; ++c) {
          if (c < C) {
            float dots[NVL];
#pragma unroll
            for (int vl = 0; vl < NVL; ++vl) {         // value lanes: dH' . v of the lane's row
              float t = 0.0f;
#pragma unroll
              for (int e = 0; e < 8; ++e) t = fmaf(vf[vl][e], dh[c][e], t);
              dots[vl] = row_sum<LV>(t);
              if (!SAME && cv == 0) xd[wave][c][vl * RV + rv] = dots[vl];
            }
            float gates[NKL];
#pragma unroll
            for (int kl = 0; kl < NKL; ++kl) {         // key lanes: score, gate, ds; dk and dq
              float sc = 0.0f;
#pragma unroll
              for (int e = 0; e < 8; ++e) sc = fmaf(kf[kl][e], qf[c][e], sc);
              sc = row_sum<LQ>(sc);
              const bool ok = (base + kl * RQ + rq) < hi;
              const float g = ok ? __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(sc * neg_scale_log2e)) : 0.0f;
              gates[kl] = g;
              const float dot = SAME ? dots[kl < NVL ? kl : 0] : xd[wave][c][kl * RQ + rq];
              const float ds = dot * g * (1.0f - g) * inv_gamma;
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                dka[kl][e] = fmaf(ds, qf[c][e], dka[kl][e]);
                dqacc[c][e] = fmaf(ds, kf[kl][e], dqacc[c][e]);
              }
              if (!SAME && cq == 0) xg[wave][c][kl * RQ + rq] = g;
            }
#pragma unroll
            for (int vl = 0; vl < NVL; ++vl) {         // value lanes: dv
              const float g = SAME ? gates[vl < NKL ? vl : 0] : xg[wave][c][vl * RV + rv];
#pragma unroll
              for (int e = 0; e < 8; ++e) dva[vl][e] = fmaf(g, dh[c][e], dva[vl][e]);
            }
          }
        }
#pragma unroll
        for (int kl = 0; kl < NKL; ++kl) {
          const int row = base + kl * RQ + rq;
          if (row < hi) store8(dkU + (size_t)row * DQ + cq * 8, dka[kl]);
        }
#pragma unroll
        for (int vl = 0; vl < NVL; ++vl) {
          const int row = base + vl * RV + rv;
          if (row < hi) store8(dvU + (size_t)row * D + cv * 8, dva[vl]);
        }
      }
    }
    // items of the segment at or past the valid length: zero gradients
    const int z0 = hi > lo ? hi : lo;
    const f32x4b zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    constexpr int PER16 = 16 / (int)sizeof(G);   // gradient elements per 16-byte store
    f32x4b* zk = reinterpret_cast<f32x4b*>(dkU + (size_t)z0 * DQ);
    f32x4b* zv = reinterpret_cast<f32x4b*>(dvU + (size_t)z0 * D);
    for (int e = lane; e < (hi_all - z0) * DQ / PER16; e += 64) __builtin_nontemporal_store(zero4, zk + e);
    for (int e = lane; e < (hi_all - z0) * D / PER16; e += 64) __builtin_nontemporal_store(zero4, zv + e);
  }
  // dq of the run: the row groups of a wave, then the waves, in a fixed order
#pragma unroll
  for (int c = 0; c < CMAX; ++c)
    if (c < C) {
#pragma unroll
      for (int off = LQ; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) dqacc[c][e] += __shfl_xor(dqacc[c][e], off, 64);
      if (rq == 0)
#pragma unroll
        for (int e = 0; e < 8; ++e) red[wave][c][cq * 8 + e] = dqacc[c][e];
    }
  __syncthreads();
  for (int e = tid; e < C * DQ; e += 256) {
    const int c = e / DQ, col = e - c * DQ;
    dq_part[((size_t)u * groups + grp) * C * DQ + e] =
        ((red[0][c][col] + red[1][c][col]) + red[2][c][col]) + red[3][c][col];
  }
}

__global__ __launch_bounds__(256) void sta_bwd_dq_kernel(const float* __restrict__ dq_part, int groups, int row,
                                                         long long total, float* __restrict__ dq_out) {
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;   // element of dq [U, C * dq]
  if (e >= total) return;
  const long long u = e / row, r = e - u * row;
  float s = 0.0f;
  for (int g = 0; g < groups; ++g) s += dq_part[(u * groups + g) * row + r];
  dq_out[e] = s;
}

// runs of segments per user: enough workgroups to fill the machine a few times over, whole users when there are many
static void sta_bwd_shape(int U, int S, int w, int* spg, int* groups) {
  int g = (2048 + U - 1) / U;
  if (g > S) g = S;
  *spg = (S + g - 1) / g;
  // short segments: runs of a dozen even out histories of different lengths (2048 users x 100 segments of 10 items,
  // lengths 200..1000: 677 us with whole users, 588 us with runs of 8 to 12)
  if (w <= 32 && *spg > 12) *spg = 12;
  const int spg_forced = tuning_int("LASER_BWD_SPG", 0);   // tuning builds only
  if (spg_forced >= 1 && spg_forced <= S) *spg = spg_forced;
  *groups = (S + *spg - 1) / *spg;
}

static bool sta_bwd_wide_supports(const StaBwdArgs& a);

// length classes: worth their empty workgroups once the launch is several rounds of workgroups and lengths differ
static int sta_bwd_classes(const StaBwdArgs& a, unsigned blocks) {
  int classes = (a.lens != nullptr && blocks >= 4096 && (unsigned long long)blocks * 4 <= 0x7fffffffULL) ? 4 : 1;
  const int cls_forced = tuning_int("LASER_STREAM_CLASSES", 0);   // tuning builds only, shared with the forward kernel
  if (cls_forced >= 1 && cls_forced <= 8 && (unsigned long long)blocks * cls_forced <= 0x7fffffffULL) classes = cls_forced;
  return classes;
}

bool sta_backward_supports(const StaBwdArgs& a) {
  if (a.grads_bf16) return sta_bwd_wide_supports(a);   // bf16 gradients: the wide kernel only
  return a.d_q <= 64 * SB_TMAX && a.d <= 64 * SB_TMAX;   // any number of candidates, SB_CMAX at a time
}

size_t sta_backward_work_bytes(int U, int C, int L, int d_q, int w) {
  int spg, groups;
  sta_bwd_shape(U, (L + w - 1) / w, w, &spg, &groups);
  return (size_t)U * groups * C * d_q * sizeof(float);
}

template <typename T, int TQ, int TV>
static void sta_bwd_launch_c(const StaBwdArgs& a, unsigned blocks, size_t lds, int spg, int groups) {
  const float inv_gamma = 1.0f / a.gamma;
  const float nsl = -1.4426950408889634f * inv_gamma;
  const int classes = sta_bwd_classes(a, blocks);
  // more than SB_CMAX candidates per user: one launch per block of SB_CMAX, in order on the stream; the first
  // writes dk and dv (and the zeros of the padding rows), the others add to them
#define LASER_BWD_LAUNCH(CM)                                                                                          \
  hipLaunchKernelGGL((sta_bwd_kernel<T, TQ, TV, CM>), dim3(blocks * classes), dim3(256), lds, a.stream,               \
                     (const T*)a.q, (const T*)a.k, (const T*)a.v, (const T*)a.dhp, a.lens, a.C, c0, cn, c0 > 0 ? 1 : 0, \
                     a.L, a.d_q, a.d, a.w, a.S, spg, groups, a.U, classes, nsl, inv_gamma,                             \
                     static_cast<float*>(a.dk), static_cast<float*>(a.dv), a.work)
  for (int c0 = 0; c0 < a.C; c0 += SB_CMAX) {
    const int cn = a.C - c0 < SB_CMAX ? a.C - c0 : SB_CMAX;
    if (cn <= 1) LASER_BWD_LAUNCH(1);
    else if (cn <= 4) LASER_BWD_LAUNCH(4);
    else LASER_BWD_LAUNCH(8);
  }
#undef LASER_BWD_LAUNCH
}

template <typename T, int TQ>
static void sta_bwd_launch_v(const StaBwdArgs& a, unsigned blocks, size_t lds, int spg, int groups) {
  const int tv = (a.d + 63) / 64;
  if (tv <= 1) sta_bwd_launch_c<T, TQ, 1>(a, blocks, lds, spg, groups);
  else if (tv <= 2) sta_bwd_launch_c<T, TQ, 2>(a, blocks, lds, spg, groups);
  else sta_bwd_launch_c<T, TQ, 4>(a, blocks, lds, spg, groups);
}

template <typename T>
static void sta_bwd_launch_q(const StaBwdArgs& a, unsigned blocks, size_t lds, int spg, int groups) {
  const int tq = (a.d_q + 63) / 64;
  if (tq <= 1) sta_bwd_launch_v<T, 1>(a, blocks, lds, spg, groups);
  else if (tq <= 2) sta_bwd_launch_v<T, 2>(a, blocks, lds, spg, groups);
  else sta_bwd_launch_v<T, 4>(a, blocks, lds, spg, groups);
}

static bool sta_bwd_wide_supports(const StaBwdArgs& a) {
  return a.dt == LASER_BF16 && a.C <= 4 && (a.d_q == 32 || a.d_q == 64 || a.d_q == 128) && (a.d == 64 || a.d == 128) &&
         tuning_int("LASER_BWD_NARROW", 0) == 0;   // tuning builds: the one-item-per-wave kernel for every shape
}

template <int DQ, int D>
static void sta_bwd_wide_launch(const StaBwdArgs& a, unsigned blocks, int spg, int groups) {
  const float inv_gamma = 1.0f / a.gamma;
  const float nsl = -1.4426950408889634f * inv_gamma;
  const int classes = sta_bwd_classes(a, blocks);
#define LASER_BWD_WIDE(CM)                                                                                           \
  do {                                                                                                               \
    if (a.grads_bf16)                                                                                                \
      hipLaunchKernelGGL((sta_bwd_wide_kernel<DQ, D, CM, true>), dim3(blocks * classes), dim3(256), 0, a.stream,    \
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,        \
                         (const unsigned short*)a.dhp, a.lens, a.C, a.L, a.w, a.S, spg, groups, a.U, classes, nsl,  \
                         inv_gamma, a.dk, a.dv, a.work);                                                             \
    else                                                                                                             \
      hipLaunchKernelGGL((sta_bwd_wide_kernel<DQ, D, CM, false>), dim3(blocks * classes), dim3(256), 0, a.stream,   \
                         (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,        \
                         (const unsigned short*)a.dhp, a.lens, a.C, a.L, a.w, a.S, spg, groups, a.U, classes, nsl,  \
                         inv_gamma, a.dk, a.dv, a.work);                                                             \
  } while (0)
  if (a.C <= 1) LASER_BWD_WIDE(1);
  else if (a.C <= 2) LASER_BWD_WIDE(2);
  else LASER_BWD_WIDE(4);
#undef LASER_BWD_WIDE
}

laser_status sta_backward_launch(const StaBwdArgs& a) {
  if (!sta_backward_supports(a)) return LASER_ERR_UNSUPPORTED;
  int spg, groups;
  sta_bwd_shape(a.U, a.S, a.w, &spg, &groups);
  const long long blocks = (long long)a.U * groups;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  const size_t lds = sizeof(float) * (size_t)(a.C < SB_CMAX ? a.C : SB_CMAX) * a.d_q * 4;
  if (sta_bwd_wide_supports(a)) {
    const unsigned nb = (unsigned)blocks;
    switch (a.d_q * 1000 + a.d) {
      case 32064: sta_bwd_wide_launch<32, 64>(a, nb, spg, groups); break;
      case 32128: sta_bwd_wide_launch<32, 128>(a, nb, spg, groups); break;
      case 64064: sta_bwd_wide_launch<64, 64>(a, nb, spg, groups); break;
      case 64128: sta_bwd_wide_launch<64, 128>(a, nb, spg, groups); break;
      case 128064: sta_bwd_wide_launch<128, 64>(a, nb, spg, groups); break;
      default: sta_bwd_wide_launch<128, 128>(a, nb, spg, groups); break;
    }
  } else if (a.dt == LASER_BF16) sta_bwd_launch_q<unsigned short>(a, (unsigned)blocks, lds, spg, groups);
  else sta_bwd_launch_q<float>(a, (unsigned)blocks, lds, spg, groups);
  if (launch_status() != LASER_OK) return LASER_ERR_LAUNCH;
  const long long total = (long long)a.U * a.C * a.d_q;
  hipLaunchKernelGGL(sta_bwd_dq_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, a.stream, a.work, groups,
                     a.C * a.d_q, total, a.dq);
  return launch_status();
}

}  // namespace laser
