// s_i <- LN(FFN(s_i) + s_i) on every segment vector of H' (paper Sec. 3.4.2, the equation that follows the STA
// paragraph), FFN(s) = relu(s W1 + b1) W2 + b2, LN over the d components with gain, bias and epsilon.
// Segments without a valid item are written as zeros.
//
// Two kernels. segment_ffn_generic_kernel: fp32 arithmetic, any d and d_ff, either storage type; a workgroup takes
// eight rows so that the weights, which it reads from L2, are used eight times.
#include "laser_internal.h"

namespace laser {

constexpr int FG_ROWS = 8, FG_THREADS = 256;

template <typename T>
__global__ __launch_bounds__(FG_THREADS) void segment_ffn_generic_kernel(
    const T* seg, const int32_t* __restrict__ lens, const T* __restrict__ w1, const float* __restrict__ b1,
    const T* __restrict__ w2, const float* __restrict__ b2, const float* __restrict__ ln_g,
    const float* __restrict__ ln_b, long long rows, int C, int L, int d, int d_ff, int w, int S, float eps,
    T* out) {   // out may be seg: a workgroup has read its rows before it writes them
  extern __shared__ float sm[];            // x [FG_ROWS][d], hidden [FG_ROWS][d_ff], y [FG_ROWS][d], stats [FG_ROWS][2]
  float* x = sm;
  float* hid = x + FG_ROWS * d;
  float* y = hid + FG_ROWS * d_ff;
  float* stats = y + FG_ROWS * d;
  __shared__ int valid[FG_ROWS];
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * FG_ROWS;
  if (tid < FG_ROWS) {
    const long long r = row0 + tid;
    int ok = 0;
    if (r < rows) {
      const int i = (int)(r % S);
      const int u = (int)(r / ((long long)C * S));
      ok = (long long)i * w < valid_len(lens, u, L);
    }
    valid[tid] = ok;
  }
  for (int e = tid; e < FG_ROWS * d; e += FG_THREADS) {
    const int rr = e / d, c = e - rr * d;
    const long long r = row0 + rr;
    x[e] = r < rows ? load_as_f32(seg, (size_t)r * d + c) : 0.0f;
  }
  __syncthreads();
  for (int j = tid; j < d_ff; j += FG_THREADS) {   // hidden unit j of the eight rows
    float acc[FG_ROWS];
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = b1[j];
    for (int e = 0; e < d; ++e) {
      const float wv = load_as_f32(w1, (size_t)e * d_ff + j);
#pragma unroll
      for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = fmaf(x[rr * d + e], wv, acc[rr]);
    }
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) hid[rr * d_ff + j] = fmaxf(acc[rr], 0.0f);
  }
  __syncthreads();
  for (int e = tid; e < d; e += FG_THREADS) {      // output component e of the eight rows, residual included
    float acc[FG_ROWS];
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = b2[e] + x[rr * d + e];
    for (int j = 0; j < d_ff; ++j) {
      const float wv = load_as_f32(w2, (size_t)j * d + e);
#pragma unroll
      for (int rr = 0; rr < FG_ROWS; ++rr) acc[rr] = fmaf(hid[rr * d_ff + j], wv, acc[rr]);
    }
#pragma unroll
    for (int rr = 0; rr < FG_ROWS; ++rr) y[rr * d + e] = acc[rr];
  }
  __syncthreads();
  // mean and variance of each row: one wave per two rows, fixed order
  {
    const int wave = tid >> 6, lane = tid & 63;
    for (int rr = wave; rr < FG_ROWS; rr += FG_THREADS / 64) {
      float s = 0.0f;
      for (int e = lane; e < d; e += 64) s += y[rr * d + e];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
      const float mean = s / (float)d;
      float q = 0.0f;
      for (int e = lane; e < d; e += 64) {
        const float t = y[rr * d + e] - mean;
        q = fmaf(t, t, q);
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off, 64);
      if (lane == 0) {
        stats[rr * 2] = mean;
        stats[rr * 2 + 1] = 1.0f / sqrtf(q / (float)d + eps);
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < FG_ROWS * d; e += FG_THREADS) {
    const int rr = e / d, c = e - rr * d;
    const long long r = row0 + rr;
    if (r < rows) {
      const float o = valid[rr] ? (y[e] - stats[rr * 2]) * stats[rr * 2 + 1] * ln_g[c] + ln_b[c] : 0.0f;
      store_from_f32(out, (size_t)r * d + c, o);
    }
  }
}

bool segment_ffn_generic_supports(const FfnArgs& a) {
  const size_t lds = (size_t)FG_ROWS * (2 * a.d + a.d_ff + 2) * sizeof(float);
  return lds <= 150 * 1024;
}

laser_status segment_ffn_generic_launch(const FfnArgs& a) {
  if (!segment_ffn_generic_supports(a)) return LASER_ERR_UNSUPPORTED;
  const long long rows = (long long)a.U * a.C * a.S;
  const long long blocks = (rows + FG_ROWS - 1) / FG_ROWS;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  const size_t lds = (size_t)FG_ROWS * (2 * a.d + a.d_ff + 2) * sizeof(float);
  if (a.dt == LASER_BF16) {
    auto kern = segment_ffn_generic_kernel<unsigned short>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(FG_THREADS), lds, a.stream, (const unsigned short*)a.seg,
                       a.lens, (const unsigned short*)a.w1, a.b1, (const unsigned short*)a.w2, a.b2, a.ln_g, a.ln_b,
                       rows, a.C, a.L, a.d, a.d_ff, a.w, a.S, a.eps, (unsigned short*)a.seg_out);
  } else {
    auto kern = segment_ffn_generic_kernel<float>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(FG_THREADS), lds, a.stream, (const float*)a.seg, a.lens,
                       (const float*)a.w1, a.b1, (const float*)a.w2, a.b2, a.ln_g, a.ln_b, rows, a.C, a.L, a.d,
                       a.d_ff, a.w, a.S, a.eps, (float*)a.seg_out);
  }
  return launch_status();
}

}  // namespace laser

namespace laser {
// placeholder until the matrix-core form exists
bool segment_ffn_mfma_supports(const FfnArgs&) { return false; }
laser_status segment_ffn_mfma_launch(const FfnArgs&) { return LASER_ERR_UNSUPPORTED; }
}  // namespace laser
