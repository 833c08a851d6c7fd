// Backward pass of STA for few candidates per user (training batches hold one target per sample; paper Sec. 4.1.2
// trains with batches of 2048 such samples). Derivatives of the forward equations of Sec. 3.4.2,
//   H'[c,i,:] = sum_{j in segment i, j < len} g_cj v_j,   g_cj = sigmoid(q_c . k_j / gamma):
//   dv_j = sum_c g_cj dH'[c,i(j),:]                         dk_j = sum_c ds_cj q_c / gamma
//   ds_cj = (dH'[c,i(j),:] . v_j) g_cj (1 - g_cj)           dq_c = sum_j ds_cj k_j / gamma
// Like the forward pass with few candidates this is HBM streaming work (K and V read once, dk and dv written once),
// so the layout is the streaming kernel's: a workgroup owns a user's run of consecutive segments and its four waves
// take alternating items. A wave holds one item at a time, lane l the elements l, l + 64, ... of its key and value
// rows; the two dot products per (item, candidate) are wave-wide sums, after which every lane knows the gate and ds
// and updates its own elements of dv_j, dk_j (stored once per item, fp32) and of dq_c (kept in registers over the
// run). The upstream gradients of the current segment and the queries sit in LDS as fp32. dq is summed over a
// workgroup's waves in LDS and over a user's workgroups by a second small kernel, both in a fixed order
// (deterministic). Items at or past the valid length get zero gradients.
#include "laser_internal.h"

namespace laser {

constexpr int SB_CMAX = 8;    // candidates per user
constexpr int SB_TMAX = 4;    // 64-element slices per row: d_q, d <= 256

template <typename T>
__global__ __launch_bounds__(256) void sta_bwd_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                      const T* __restrict__ v, const T* __restrict__ dhp,
                                                      const int32_t* __restrict__ lens, int C, int L, int dq, int d, int w,
                                                      int S, int spg, int groups, float inv_gamma,
                                                      float* __restrict__ dk, float* __restrict__ dv,
                                                      float* __restrict__ dq_part) {
  extern __shared__ float sm[];
  float* qs = sm;                       // [C][dq]
  float* dhs = qs + C * dq;             // [C][d]   upstream gradient of the current segment
  float* red = dhs + C * d;             // [4][C][dq] per-wave dq sums at the end of the run
  const int u = blockIdx.x / groups, grp = blockIdx.x % groups;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = valid_len(lens, u, L);
  const int TQ = (dq + 63) / 64, TV = (d + 63) / 64;

  for (int e = tid; e < C * dq; e += 256) qs[e] = load_as_f32(q, (size_t)u * C * dq + e);
  const int i_beg = grp * spg;
  const int i_end = (grp + 1) * spg < S ? (grp + 1) * spg : S;
  const T* kU = k + (size_t)u * L * dq;
  const T* vU = v + (size_t)u * L * d;
  float* dkU = dk + (size_t)u * L * dq;
  float* dvU = dv + (size_t)u * L * d;

  float dqacc[SB_CMAX][SB_TMAX];
#pragma unroll
  for (int c = 0; c < SB_CMAX; ++c)
#pragma unroll
    for (int t = 0; t < SB_TMAX; ++t) dqacc[c][t] = 0.0f;

  for (int i = i_beg; i < i_end; ++i) {
    const int lo = i * w;
    int hi_all = lo + w;
    if (hi_all > L) hi_all = L;
    const int hi = hi_all < n ? hi_all : n;      // valid items of the segment: [lo, hi)
    __syncthreads();                              // the previous segment's gradients are no longer read
    if (hi > lo)
      for (int e = tid; e < C * d; e += 256) {
        const int c = e / d, col = e - c * d;
        dhs[e] = load_as_f32(dhp, (((size_t)u * C + c) * S + i) * d + col);
      }
    __syncthreads();
    for (int j = lo + wave; j < hi; j += 4) {
      float kr[SB_TMAX], vr[SB_TMAX], dka[SB_TMAX], dva[SB_TMAX];
#pragma unroll
      for (int t = 0; t < SB_TMAX; ++t) {
        const int eq = lane + 64 * t;
        kr[t] = (t < TQ && eq < dq) ? load_as_f32(kU, (size_t)j * dq + eq) : 0.0f;
        vr[t] = (t < TV && eq < d) ? load_as_f32(vU, (size_t)j * d + eq) : 0.0f;
        dka[t] = 0.0f;
        dva[t] = 0.0f;
      }
#pragma unroll
      for (int c = 0; c < SB_CMAX; ++c) {
        if (c < C) {
          float s = 0.0f, dot = 0.0f;
#pragma unroll
          for (int t = 0; t < SB_TMAX; ++t) {
            const int e = lane + 64 * t;
            if (t < TQ && e < dq) s = fmaf(kr[t], qs[c * dq + e], s);
            if (t < TV && e < d) dot = fmaf(vr[t], dhs[c * d + e], dot);
          }
          s = wave_sum(s);
          dot = wave_sum(dot);
          const float g = 1.0f / (1.0f + expf(-s * inv_gamma));
          const float ds = dot * g * (1.0f - g) * inv_gamma;   // d loss / d (q_c . k_j)
#pragma unroll
          for (int t = 0; t < SB_TMAX; ++t) {
            const int e = lane + 64 * t;
            if (t < TV && e < d) dva[t] = fmaf(g, dhs[c * d + e], dva[t]);
            if (t < TQ && e < dq) {
              dka[t] = fmaf(ds, qs[c * dq + e], dka[t]);
              dqacc[c][t] = fmaf(ds, kr[t], dqacc[c][t]);
            }
          }
        }
      }
#pragma unroll
      for (int t = 0; t < SB_TMAX; ++t) {
        const int e = lane + 64 * t;
        if (t < TQ && e < dq) dkU[(size_t)j * dq + e] = dka[t];
        if (t < TV && e < d) dvU[(size_t)j * d + e] = dva[t];
      }
    }
    // items of the segment at or past the valid length: zero gradients
    const int z0 = hi > lo ? hi : lo;
    for (int e = tid; e < (hi_all - z0) * dq; e += 256) dkU[(size_t)z0 * dq + e] = 0.0f;
    for (int e = tid; e < (hi_all - z0) * d; e += 256) dvU[(size_t)z0 * d + e] = 0.0f;
  }
  // dq of the run: waves in a fixed order
#pragma unroll
  for (int c = 0; c < SB_CMAX; ++c)
    if (c < C)
#pragma unroll
      for (int t = 0; t < SB_TMAX; ++t) {
        const int e = lane + 64 * t;
        if (t < TQ && e < dq) red[(wave * C + c) * dq + e] = dqacc[c][t];
      }
  __syncthreads();
  for (int e = tid; e < C * dq; e += 256)
    dq_part[((size_t)u * groups + grp) * C * dq + e] =
        ((red[e] + red[C * dq + e]) + red[2 * C * dq + e]) + red[3 * C * dq + e];
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
static void sta_bwd_shape(int U, int S, int* spg, int* groups) {
  int g = (2048 + U - 1) / U;
  if (g > S) g = S;
  *spg = (S + g - 1) / g;
  *groups = (S + *spg - 1) / *spg;
}

bool sta_backward_supports(const StaBwdArgs& a) {
  return a.C <= SB_CMAX && a.d_q <= 64 * SB_TMAX && a.d <= 64 * SB_TMAX;
}

size_t sta_backward_work_bytes(int U, int C, int L, int d_q, int w) {
  int spg, groups;
  sta_bwd_shape(U, (L + w - 1) / w, &spg, &groups);
  return (size_t)U * groups * C * d_q * sizeof(float);
}

laser_status sta_backward_launch(const StaBwdArgs& a) {
  if (!sta_backward_supports(a)) return LASER_ERR_UNSUPPORTED;
  int spg, groups;
  sta_bwd_shape(a.U, a.S, &spg, &groups);
  const long long blocks = (long long)a.U * groups;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  const size_t lds = sizeof(float) * ((size_t)a.C * a.d_q * 5 + (size_t)a.C * a.d);
  const float inv_gamma = 1.0f / a.gamma;
  if (a.dt == LASER_BF16)
    hipLaunchKernelGGL(sta_bwd_kernel<unsigned short>, dim3((unsigned)blocks), dim3(256), lds, a.stream,
                       (const unsigned short*)a.q, (const unsigned short*)a.k, (const unsigned short*)a.v,
                       (const unsigned short*)a.dhp, a.lens, a.C, a.L, a.d_q, a.d, a.w, a.S, spg, groups, inv_gamma,
                       a.dk, a.dv, a.work);
  else
    hipLaunchKernelGGL(sta_bwd_kernel<float>, dim3((unsigned)blocks), dim3(256), lds, a.stream, (const float*)a.q,
                       (const float*)a.k, (const float*)a.v, (const float*)a.dhp, a.lens, a.C, a.L, a.d_q, a.d, a.w,
                       a.S, spg, groups, inv_gamma, a.dk, a.dv, a.work);
  if (launch_status() != LASER_OK) return LASER_ERR_LAUNCH;
  const long long total = (long long)a.U * a.C * a.d_q;
  hipLaunchKernelGGL(sta_bwd_dq_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, a.stream, a.work, groups,
                     a.C * a.d_q, total, a.dq);
  return launch_status();
}

}  // namespace laser
