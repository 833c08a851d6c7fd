// Generic GSTA kernel: fp32 FMA arithmetic, one workgroup per (user, candidate), any shape.
//
// Per layer l (Sec. 3.4.3): a_l = softmax((t W_q)(H' W_k)^T / sqrt(d)), o_l = a_l (H' W_v), t += o_l.
// The two products with H' are re-associated, which is exact up to rounding:
//   (t W_q)(H' W_k)^T = H' (W_k (t W_q)^T)   and   a (H' W_v) = (a H') W_v,
// so a pair costs three d x d matrix-vector products and two passes over its S x d block of H'
// per layer instead of two S x d x d products. Only the first ceil(len/w) segments (those that
// hold a valid item) enter the softmax. Every sum has a fixed order: results are deterministic.
#include "laser_internal.h"

namespace laser {

template <typename T>
__global__ __launch_bounds__(256) void gsta_generic_kernel(const T* __restrict__ seg, const T* __restrict__ t0,
                                                           const T* __restrict__ wq, const T* __restrict__ wk,
                                                           const T* __restrict__ wv, const int32_t* __restrict__ lens,
                                                           const int32_t* __restrict__ cand_off, int U, int C, int L,
                                                           int d, int w, int S, int M, float* __restrict__ z) {
  extern __shared__ float smem[];
  float* ts = smem;        // [d] running target vector t_l
  float* qp = ts + d;      // [d] t W_q
  float* rr = qp + d;      // [d] W_k (t W_q)^T
  float* pp = rr + d;      // [d] a H'
  float* es = pp + d;      // [S] scores, then softmax weights
  __shared__ float red[2];

  const int pair = blockIdx.x;
  const int u = pair_user(cand_off, U, C, pair);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = valid_len(lens, u, L);
  const int nv = (n + w - 1) / w;          // valid segments are a prefix
  const float scale = 1.0f / sqrtf((float)d);
  const T* H = seg + (size_t)pair * S * d;

  for (int b = tid; b < d; b += 256) ts[b] = load_as_f32(t0, (size_t)pair * d + b);

  for (int l = 0; l < M && nv > 0; ++l) {
    const T* Wq = wq + (size_t)l * d * d;
    const T* Wk = wk + (size_t)l * d * d;
    const T* Wv = wv + (size_t)l * d * d;
    __syncthreads();
    for (int b = tid; b < d; b += 256) {
      float s = 0.0f;
#pragma unroll 8
      for (int a = 0; a < d; ++a) s = fmaf(ts[a], load_as_f32(Wq, (size_t)a * d + b), s);
      qp[b] = s;
    }
    __syncthreads();
    for (int a = wave; a < d; a += 4) {
      float s = 0.0f;
      for (int b = lane; b < d; b += 64) s = fmaf(load_as_f32(Wk, (size_t)a * d + b), qp[b], s);
      s = wave_sum(s);
      if (lane == 0) rr[a] = s;
    }
    __syncthreads();
    for (int i = wave; i < nv; i += 4) {
      float s = 0.0f;
      for (int b = lane; b < d; b += 64) s = fmaf(load_as_f32(H, (size_t)i * d + b), rr[b], s);
      s = wave_sum(s);
      if (lane == 0) es[i] = s * scale;
    }
    __syncthreads();
    if (wave == 0) {
      float mx = -INFINITY;
      for (int i = lane; i < nv; i += 64) mx = fmaxf(mx, es[i]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      float den = 0.0f;
      for (int i = lane; i < nv; i += 64) den += expf(es[i] - mx);
      den = wave_sum(den);
      if (lane == 0) { red[0] = mx; red[1] = den; }
    }
    __syncthreads();
    {
      const float mx = red[0], inv = 1.0f / red[1];
      for (int i = tid; i < nv; i += 256) es[i] = expf(es[i] - mx) * inv;
    }
    __syncthreads();
    for (int b = tid; b < d; b += 256) {
      float s = 0.0f;
#pragma unroll 8
      for (int i = 0; i < nv; ++i) s = fmaf(es[i], load_as_f32(H, (size_t)i * d + b), s);
      pp[b] = s;
    }
    __syncthreads();
    for (int b = tid; b < d; b += 256) {
      float s = 0.0f;
#pragma unroll 8
      for (int a = 0; a < d; ++a) s = fmaf(pp[a], load_as_f32(Wv, (size_t)a * d + b), s);
      ts[b] += s;                           // residual update of the target
    }
  }
  __syncthreads();
  for (int b = tid; b < d; b += 256) z[(size_t)pair * d + b] = ts[b];
}

bool gsta_generic_supports(const GstaArgs& a) {
  return a.d <= 1024 && a.S <= 4096 && (long long)a.U * a.C <= 0x7fffffffLL;
}

laser_status gsta_generic_launch(const GstaArgs& a) {
  if (!gsta_generic_supports(a)) return LASER_ERR_UNSUPPORTED;
  const size_t lds = sizeof(float) * (4 * (size_t)a.d + a.S);
  const unsigned blocks = (unsigned)gsta_pairs(a);
  if (blocks == 0) return LASER_OK;
  if (a.dt == LASER_F32) {
    hipLaunchKernelGGL(gsta_generic_kernel<float>, dim3(blocks), dim3(256), lds, a.stream, (const float*)a.seg,
                       (const float*)a.t0, (const float*)a.wq, (const float*)a.wk, (const float*)a.wv, a.lens, a.cand_off, a.U, a.C,
                       a.L, a.d, a.w, a.S, a.M, a.z_out);
  } else {
    hipLaunchKernelGGL(gsta_generic_kernel<unsigned short>, dim3(blocks), dim3(256), lds, a.stream,
                       (const unsigned short*)a.seg, (const unsigned short*)a.t0, (const unsigned short*)a.wq,
                       (const unsigned short*)a.wk, (const unsigned short*)a.wv, a.lens, a.cand_off, a.U, a.C, a.L, a.d, a.w, a.S,
                       a.M, a.z_out);
  }
  return launch_status();
}

}  // namespace laser
