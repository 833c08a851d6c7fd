// Generic STA kernel: fp32 FMA arithmetic, any shape, fp32 or bf16 storage.
//
// Computes the STA equation of Sec. 3.4.2 in the global form of Sec. 3.5.1:
//   H'[u,c,i,:] = sum_{valid j in segment i} sigmoid(q[u,c,:] . k[u,j,:] / gamma) * v[u,j,:]
// One workgroup owns (user u, segment i, four candidates); each of its four waves owns one
// candidate. The segment is walked in chunks of TI items that the workgroup stages in LDS as
// fp32 (coalesced global reads, shared by the four candidates). Per chunk a wave first gives
// one lane per item the score dot product and the gate, then gives one lane per value column
// the gated sum over the chunk. Sums run over items in ascending order in fp32, so results
// are deterministic. This is the correctness path (fp32 tolerance) and the fallback for shapes
// the MFMA and streaming kernels do not take.
#include "laser_internal.h"

namespace laser {

constexpr int GEN_WAVES = 4;
constexpr int GEN_MAX_COLS = 16;  // d <= 64 * 16

template <typename T>
__global__ __launch_bounds__(256) void sta_generic_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                          const T* __restrict__ v, const int32_t* __restrict__ lens,
                                                          const int32_t* __restrict__ cand_off, int P, int C_all,
                                                          int L, int dq, int d, int w, int S, int TI,
                                                          int heads, int softmax, float inv_gamma,
                                                          T* __restrict__ seg_out,
                                                          int32_t* __restrict__ seg_cnt) {
  extern __shared__ float smem[];
  const int kpitch = dq + 1;                   // +1: lanes read different rows at the same column
  float* Ks = smem;                            // [TI][dq + 1]
  float* Vs = Ks + (size_t)TI * kpitch;        // [TI][d]
  float* qs = Vs + (size_t)TI * d;             // [4][dq]
  float* gs = qs + GEN_WAVES * dq;             // [4][heads][TI]
  // several heads (Sec. 4.1.2): head h owns the h-th run of dq / heads columns of q and k and of d / heads columns of v
  const int dqh = dq / heads, dh = d / heads;

  const int cblocks = (C_all + GEN_WAVES - 1) / GEN_WAVES;
  int bid = blockIdx.x;
  const int i = bid % S;
  bid /= S;
  const int cb = bid % cblocks;
  const int u = bid / cblocks;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const CandRange cr = cand_range(cand_off, u, C_all, P);
  const int C = cr.count;            // this user's candidates
  const size_t pb = (size_t)cr.first;   // and the index of their first pair
  const int c = cb * GEN_WAVES + wave;
  const bool active = c < C;

  const int n = valid_len(lens, u, L);
  if (i == 0 && cb == 0) write_seg_cnt(seg_cnt, u, n, L, w, S, tid, 256);
  if (cb * GEN_WAVES >= C) return;   // a candidate block past this user's count (the whole workgroup leaves)
  const int lo = i * w;
  int hi = lo + w;
  if (hi > L) hi = L;
  if (hi > n) hi = n;

  for (int a = lane; a < dq; a += 64)
    qs[wave * dq + a] = active ? load_as_f32(q, (pb + c) * dq + a) : 0.0f;

  // softmax (ablation of Sec. 4.4.1): gs then holds the scaled scores, and every column keeps a running maximum
  // and denominator of its head's scores, rescaling its sum when the maximum moves (items in ascending order)
  float acc[GEN_MAX_COLS], sm_m[GEN_MAX_COLS], sm_l[GEN_MAX_COLS];
#pragma unroll
  for (int b = 0; b < GEN_MAX_COLS; ++b) {
    acc[b] = 0.0f;
    sm_m[b] = -INFINITY;
    sm_l[b] = 0.0f;
  }

  const T* kU = k + (size_t)u * L * dq;
  const T* vU = v + (size_t)u * L * d;
  const int nb = (d + 63) >> 6;   // blocks of 64 columns in use

  for (int j0 = lo; j0 < hi; j0 += TI) {
    const int nj = (hi - j0) < TI ? (hi - j0) : TI;
    __syncthreads();
#pragma unroll 8
    for (int e = tid; e < nj * dq; e += 256) {   // unrolled so that the loads of several rounds are in flight together
      const int r = e / dq, a = e - r * dq;
      Ks[r * kpitch + a] = load_as_f32(kU, (size_t)(j0 + r) * dq + a);
    }
#pragma unroll 8
    for (int e = tid; e < nj * d; e += 256) Vs[e] = load_as_f32(vU, (size_t)j0 * d + e);
    __syncthreads();
    if (lane < nj) {
      const float* kr = Ks + lane * kpitch;
      const float* qr = qs + wave * dq;
      for (int hh = 0; hh < heads; ++hh) {
        float e = 0.0f;
#pragma unroll 8
        for (int a = hh * dqh; a < (hh + 1) * dqh; ++a) e = fmaf(qr[a], kr[a], e);
        gs[(wave * heads + hh) * TI + lane] =
            softmax ? e * inv_gamma : 1.0f / (1.0f + expf(-e * inv_gamma));   // independent gate per item
      }
    }
    __syncthreads();
#pragma unroll 4
    for (int jj = 0; jj < nj; ++jj) {
#pragma unroll
      for (int b = 0; b < GEN_MAX_COLS; ++b) {
        if (b >= nb) break;   // the same for the whole wave: blocks past d cost nothing
        const int col = lane + 64 * b;
        if (col < d) {
          const float g = gs[(wave * heads + col / dh) * TI + jj];
          if (softmax) {
            const float m_new = fmaxf(sm_m[b], g);
            const float sc = expf(sm_m[b] - m_new);   // 0 the first time (the maximum starts at minus infinity)
            const float pr = expf(g - m_new);
            acc[b] = fmaf(pr, Vs[jj * d + col], acc[b] * sc);
            sm_l[b] = fmaf(sm_l[b], sc, pr);
            sm_m[b] = m_new;
          } else {
            acc[b] = fmaf(g, Vs[jj * d + col], acc[b]);
          }
        }
      }
    }
  }

  if (active) {
    const size_t base = ((pb + c) * S + i) * d;
#pragma unroll
    for (int b = 0; b < GEN_MAX_COLS; ++b) {
      const int col = lane + 64 * b;
      if (col < d) store_from_f32(seg_out, base + col, (softmax && sm_l[b] > 0.0f) ? acc[b] / sm_l[b] : acc[b]);
    }
  }
}

static size_t gen_lds_bytes(int TI, int dq, int d, int heads) {
  return sizeof(float) * ((size_t)TI * (dq + 1) + (size_t)TI * d + GEN_WAVES * dq + (size_t)GEN_WAVES * heads * TI);
}

static int gen_pick_ti(int dq, int d, int heads) {
  for (int ti = 64; ti >= 1; ti >>= 1)
    if (gen_lds_bytes(ti, dq, d, heads) <= 60 * 1024) return ti;
  return 0;
}

bool sta_generic_supports(const StaArgs& a) {
  if (a.d > 64 * GEN_MAX_COLS || a.d_q > 1024) return false;
  if (a.heads < 1 || a.d_q % a.heads != 0 || a.d % a.heads != 0) return false;
  if (gen_pick_ti(a.d_q, a.d, a.heads) == 0) return false;
  const long long blocks = (long long)a.U * ((a.C + GEN_WAVES - 1) / GEN_WAVES) * a.S;
  return blocks <= 0x7fffffffLL;
}

laser_status sta_generic_launch(const StaArgs& a) {
  if (!sta_generic_supports(a)) return LASER_ERR_UNSUPPORTED;
  const int TI = gen_pick_ti(a.d_q, a.d, a.heads);
  const size_t lds = gen_lds_bytes(TI, a.d_q, a.d, a.heads);
  const unsigned blocks = (unsigned)((long long)a.U * ((a.C + GEN_WAVES - 1) / GEN_WAVES) * a.S);
  const float inv_gamma = 1.0f / a.gamma;
  if (a.dt == LASER_F32) {
    hipLaunchKernelGGL(sta_generic_kernel<float>, dim3(blocks), dim3(256), lds, a.stream, (const float*)a.q,
                       (const float*)a.k, (const float*)a.v, a.lens, a.cand_off, a.P, a.C, a.L, a.d_q, a.d, a.w, a.S, TI, a.heads,
                       a.softmax ? 1 : 0, inv_gamma, (float*)a.seg_out, a.seg_cnt);
  } else {
    hipLaunchKernelGGL(sta_generic_kernel<unsigned short>, dim3(blocks), dim3(256), lds, a.stream,
                       (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v, a.lens,
                       a.cand_off, a.P, a.C, a.L, a.d_q, a.d, a.w, a.S, TI, a.heads, a.softmax ? 1 : 0, inv_gamma,
                       (unsigned short*)a.seg_out, a.seg_cnt);
  }
  return launch_status();
}

}  // namespace laser
