// Backward pass of GSTA (derivatives of the forward equations of paper Sec. 3.4.3), generic form: fp32 arithmetic,
// either storage type, one workgroup per (user, candidate) pair with the pair's valid rows of H' and their
// gradients in LDS. Per layer, in the re-associated form the forward kernels use (exact re-association):
//   q' = t W_q,  r = W_k q',  e_i = H'_i . r / sqrt(d),  a = softmax(e),  p = sum_i a_i H'_i,  o = p W_v,  t += o.
// The layers' inputs t_l are kept from a first forward sweep; the backward sweep replays a layer's q', r, a, p and
// applies the chain rule. All three weight gradients of a pair and layer are outer products of d-vectors,
//   dW_v = p (x) do,   dW_k = dr (x) q',   dW_q = t_l (x) dq',
// so the pair kernel only writes those six vectors to the caller's scratch, and two small kernels sum the outer
// products over all pairs in a fixed order (deterministic).
#include "laser_internal.h"

namespace laser {

constexpr int GB_THREADS = 256, GB_MAXM = 8, GB_MAXD = 256;

// eight consecutive elements (16-byte aligned for bf16, 32-byte for fp32) as fp32
__device__ __forceinline__ void load8_as_f32(const unsigned short* p, float (&out)[8]) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 raw = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    out[2 * e] = __uint_as_float(raw[e] << 16);
    out[2 * e + 1] = __uint_as_float(raw[e] & 0xffff0000u);
  }
}
__device__ __forceinline__ void load8_as_f32(const float* p, float (&out)[8]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    out[e] = a[e];
    out[4 + e] = b[e];
  }
}

template <typename T>
__global__ __launch_bounds__(GB_THREADS) void gsta_bwd_kernel(const T* __restrict__ seg, const T* __restrict__ t0,
                                                              const T* __restrict__ wq, const T* __restrict__ wk,
                                                              const T* __restrict__ wv, const int32_t* __restrict__ lens,
                                                              const float* __restrict__ dz, int C, int L, int d, int w,
                                                              int S, int M, T* __restrict__ dseg,
                                                              float* __restrict__ dt0, float* __restrict__ pv) {
  extern __shared__ float sm[];
  const int pair = blockIdx.x, u = pair / C;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nv = (valid_len(lens, u, L) + w - 1) / w;     // valid segments are a prefix
  // With one layer the gradient of H' is written straight from the layer's vectors at the end, and its block is
  // not kept: less LDS, more workgroups per compute unit.
  const bool keep = M > 1;
  // H' stays in LDS in its storage type (half the space for bf16: more workgroups per compute unit, and the pair
  // kernel is a chain of short phases that only other workgroups can overlap)
  float* dHs = sm;                                // [nv][d] (several layers only)
  float* ts = dHs + (keep ? (size_t)nv * d : 0);  // [M][d]  t_0 .. t_{M-1}
  float* qp = ts + M * d;            // the seven vectors below: [d] each
  float* rv = qp + d;
  float* pvv = rv + d;
  float* g = pvv + d;
  float* dp = g + d;
  float* drv = dp + d;
  float* dqp = drv + d;
  float* av = dqp + d;               // [S] softmax weights
  float* da = av + S;                // [S]
  T* Hs = reinterpret_cast<T*>(da + S + ((2 * S) & 3));   // [nv][d]; the two [S] arrays are padded to 16 bytes
  __shared__ float red[4];
  __shared__ float halves[GB_THREADS / 2];
  const float scale = 1.0f / sqrtf((float)d);
  const T* H = seg + (size_t)pair * S * d;
  T* dH = dseg + (size_t)pair * S * d;
  float* pvp = pv + (size_t)pair * M * 6 * d;

  for (int e = tid * 8; e < nv * d; e += GB_THREADS * 8) {   // d is a multiple of eight
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      Hs[e + j] = H[e + j];
      if (keep) dHs[e + j] = 0.0f;
    }
  }
  for (int e = tid; e < d; e += GB_THREADS) {
    ts[e] = load_as_f32(t0, (size_t)pair * d + e);
    g[e] = dz[(size_t)pair * d + e];
  }
  __syncthreads();
  if (nv == 0) {   // z = t0: the gradient passes straight through, nothing else gets any
    for (int e = tid; e < d; e += GB_THREADS) dt0[(size_t)pair * d + e] = g[e];
    for (int e = tid; e < S * d; e += GB_THREADS) store_from_f32(dH, (size_t)e, 0.0f);
    for (int e = tid; e < M * 6 * d; e += GB_THREADS) pvp[e] = 0.0f;
    return;
  }

  // out[y] = sum_x in[x] W[x][y]: one thread per column, coalesced over y
  // (with d <= 128 the two halves of the workgroup take the two halves of x and meet in LDS)
  auto col_matvec = [&](float* out, const float* in, const T* W) {
    if (d <= GB_THREADS / 2) {
      const int half = tid / (GB_THREADS / 2), y = tid % (GB_THREADS / 2);
      const int x0 = half * (d / 2), x1 = half ? d : d / 2;
      float acc = 0.0f;
      if (y < d)
        for (int x = x0; x < x1; ++x) acc = fmaf(in[x], load_as_f32(W, (size_t)x * d + y), acc);
      if (half == 1 && y < d) halves[y] = acc;
      __syncthreads();
      if (half == 0 && y < d) out[y] = acc + halves[y];
      return;
    }
    for (int y = tid; y < d; y += GB_THREADS) {
      float acc = 0.0f;
      for (int x = 0; x < d; ++x) acc = fmaf(in[x], load_as_f32(W, (size_t)x * d + y), acc);
      out[y] = acc;
    }
  };
  // out[x] (+)= sum_y W[x][y] in[y]: one thread per row, the row read in 16-byte pieces (a wave's 64 rows stay in
  // the first-level cache from one piece to the next; a wave per row would be a chain of load, wave-wide sum and
  // store per row, with nothing to overlap it)
  auto row_matvec = [&](float* out, const float* in, const T* W, bool add) {
    for (int x = tid; x < d; x += GB_THREADS) {
      float acc = 0.0f;
      for (int y = 0; y < d; y += 8) {
        float wrow[8];
        load8_as_f32(W + (size_t)x * d + y, wrow);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(wrow[e], in[y + e], acc);
      }
      out[x] = add ? out[x] + acc : acc;
    }
  };
  // q', r, a, p of layer l from its input t_l (the forward pass up to the value projection)
  auto replay = [&](int l) {
    col_matvec(qp, ts + l * d, wq + (size_t)l * d * d);
    __syncthreads();
    row_matvec(rv, qp, wk + (size_t)l * d * d, false);
    __syncthreads();
    for (int i = wave; i < nv; i += GB_THREADS / 64) {
      float acc = 0.0f;
      for (int x = lane; x < d; x += 64) acc = fmaf(load_as_f32(Hs, (size_t)(i * d + x)), rv[x], acc);
      acc = wave_sum_rows(acc);
      if (lane == 0) av[i] = acc * scale;
    }
    __syncthreads();
    if (wave == 0) {   // softmax over the valid segments
      float m = -INFINITY;
      for (int i = lane; i < nv; i += 64) m = fmaxf(m, av[i]);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
      float ssum = 0.0f;
      for (int i = lane; i < nv; i += 64) {
        const float ex = expf(av[i] - m);
        av[i] = ex;
        ssum += ex;
      }
      ssum = wave_sum_rows(ssum);
      if (lane == 0) red[0] = 1.0f / ssum;
    }
    __syncthreads();
    for (int i = tid; i < nv; i += GB_THREADS) av[i] *= red[0];
    __syncthreads();
    for (int x = tid; x < d; x += GB_THREADS) {
      float acc = 0.0f;
      for (int i = 0; i < nv; ++i) acc = fmaf(av[i], load_as_f32(Hs, (size_t)(i * d + x)), acc);
      pvv[x] = acc;
    }
    __syncthreads();
  };

  // forward sweep: the inputs of layers 1 .. M-1
  for (int l = 0; l + 1 < M; ++l) {
    replay(l);
    col_matvec(dp, pvv, wv + (size_t)l * d * d);   // o = p W_v (dp is free here)
    __syncthreads();
    for (int e = tid; e < d; e += GB_THREADS) ts[(l + 1) * d + e] = ts[l * d + e] + dp[e];
    __syncthreads();
  }
  // backward sweep
  for (int l = M - 1; l >= 0; --l) {
    replay(l);
    float* out6 = pvp + (size_t)l * 6 * d;
    row_matvec(dp, g, wv + (size_t)l * d * d, false);             // dp = do W_v^T, do = g
    for (int e = tid; e < d; e += GB_THREADS) {
      out6[e] = pvv[e];                                           // dW_v = p (x) do
      out6[d + e] = g[e];
    }
    __syncthreads();
    for (int i = wave; i < nv; i += GB_THREADS / 64) {            // da_i = dp . H'_i
      float acc = 0.0f;
      for (int x = lane; x < d; x += 64) acc = fmaf(load_as_f32(Hs, (size_t)(i * d + x)), dp[x], acc);
      acc = wave_sum_rows(acc);
      if (lane == 0) da[i] = acc;
    }
    __syncthreads();
    if (wave == 0) {                                              // sum_k a_k da_k
      float acc = 0.0f;
      for (int i = lane; i < nv; i += 64) acc = fmaf(av[i], da[i], acc);
      acc = wave_sum_rows(acc);
      if (lane == 0) red[1] = acc;
    }
    __syncthreads();
    for (int e = tid; e < nv * d; e += GB_THREADS) {              // dH'_i += a_i dp + de_i r / sqrt(d)
      const int i = e / d, x = e - i * d;
      const float de = av[i] * (da[i] - red[1]);
      const float val = av[i] * dp[x] + de * rv[x] * scale;
      if (keep) dHs[e] += val;
      else store_from_f32(dH, (size_t)e, val);
    }
    for (int x = tid; x < d; x += GB_THREADS) {                   // dr = sum_i de_i H'_i / sqrt(d)
      float acc = 0.0f;
      for (int i = 0; i < nv; ++i) acc = fmaf(av[i] * (da[i] - red[1]), load_as_f32(Hs, (size_t)(i * d + x)), acc);
      drv[x] = acc * scale;
    }
    __syncthreads();
    col_matvec(dqp, drv, wk + (size_t)l * d * d);                 // dq' = dr W_k
    __syncthreads();
    for (int e = tid; e < d; e += GB_THREADS) {
      out6[2 * d + e] = drv[e];                                   // dW_k = dr (x) q'
      out6[3 * d + e] = qp[e];
      out6[4 * d + e] = ts[l * d + e];                            // dW_q = t_l (x) dq'
      out6[5 * d + e] = dqp[e];
    }
    row_matvec(g, dqp, wq + (size_t)l * d * d, true);             // g += dq' W_q^T (the residual path keeps g)
    __syncthreads();
  }
  for (int e = tid; e < d; e += GB_THREADS) dt0[(size_t)pair * d + e] = g[e];
  if (keep)
    for (int e = tid; e < nv * d; e += GB_THREADS) store_from_f32(dH, (size_t)e, dHs[e]);
  for (int e = nv * d + tid; e < S * d; e += GB_THREADS) store_from_f32(dH, (size_t)e, 0.0f);
}

// dW[l][x][y] = sum over pairs of A[pair][l][x] * B[pair][l][y]. Two steps, both in a fixed order: the pairs are cut
// into chunks, a workgroup sums one chunk for a 32 x 32 tile of one matrix (pairs ascending), and a second kernel adds
// the chunks' partial matrices in ascending order.
__global__ __launch_bounds__(256) void gsta_bwd_w_partial_kernel(const float* __restrict__ pv, int P, int M, int d,
                                                                 int chunks, float* __restrict__ part) {
  // a 32 x 32 tile of one matrix per workgroup, 2 x 2 entries per thread; the two vectors of 64 pairs at a time are
  // staged in LDS (32 consecutive floats of each), so every global load is a 32-byte piece and is used 32 times
  constexpr int TP = 64, TW = 32;
  __shared__ float As[TP][TW + 1], Bs[TP][TW + 1];
  const int tiles = (d + TW - 1) / TW;
  int bid = blockIdx.x;
  const int ty = bid % tiles;
  bid /= tiles;
  const int tx = bid % tiles;
  bid /= tiles;
  const int which = bid % 3;     // 0: dW_v (p, do), 1: dW_k (dr, q'), 2: dW_q (t_l, dq')
  bid /= 3;
  const int l = bid % M, chunk = bid / M;
  const int tid = threadIdx.x, r = tid / 16, c = tid % 16;
  const int per = (P + chunks - 1) / chunks;
  const int p0 = chunk * per, p1 = (p0 + per) < P ? (p0 + per) : P;
  const float* a = pv + ((size_t)l * 6 + 2 * which) * d + tx * TW;
  const float* b = pv + ((size_t)l * 6 + 2 * which + 1) * d + ty * TW;
  const size_t stride = (size_t)M * 6 * d;
  const int spr = tid / 4, sc = (tid % 4) * 8;   // staging: pair row and first of this thread's eight columns
  float acc[2][2] = {{0.0f, 0.0f}, {0.0f, 0.0f}};
  for (int pb = p0; pb < p1; pb += TP) {
    const int pr = pb + spr;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const bool oka = pr < p1 && tx * TW + sc + e < d, okb = pr < p1 && ty * TW + sc + e < d;
      As[spr][sc + e] = oka ? a[(size_t)pr * stride + sc + e] : 0.0f;
      Bs[spr][sc + e] = okb ? b[(size_t)pr * stride + sc + e] : 0.0f;
    }
    __syncthreads();
#pragma unroll 8
    for (int pp = 0; pp < TP; ++pp) {   // pairs in ascending order (rows past the chunk hold zeros)
      const float a0 = As[pp][2 * r], a1 = As[pp][2 * r + 1], b0 = Bs[pp][2 * c], b1 = Bs[pp][2 * c + 1];
      acc[0][0] = fmaf(a0, b0, acc[0][0]);
      acc[0][1] = fmaf(a0, b1, acc[0][1]);
      acc[1][0] = fmaf(a1, b0, acc[1][0]);
      acc[1][1] = fmaf(a1, b1, acc[1][1]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jx = 0; jx < 2; ++jx) {
      const int x = tx * TW + 2 * r + i, y = ty * TW + 2 * c + jx;
      if (x < d && y < d) part[((((size_t)chunk * M + l) * 3 + which) * d + x) * d + y] = acc[i][jx];
    }
}

__global__ __launch_bounds__(256) void gsta_bwd_w_reduce_kernel(const float* __restrict__ part, int M, int d, int chunks,
                                                                float* __restrict__ dwq, float* __restrict__ dwk,
                                                                float* __restrict__ dwv) {
  const long long per_l = (long long)3 * d * d, total = (long long)M * per_l;
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;     // (l, which, x, y)
  if (e >= total) return;
  float acc = 0.0f;
  for (int c = 0; c < chunks; ++c) acc += part[(size_t)c * total + e];
  const int l = (int)(e / per_l);
  const long long r = e - (long long)l * per_l;
  const int which = (int)(r / ((long long)d * d));
  const long long xy = r - (long long)which * d * d;
  float* out = which == 0 ? dwv : (which == 1 ? dwk : dwq);
  out[(size_t)l * d * d + xy] = acc;
}

static int gsta_bwd_chunks(int P) {
  int c = (P + 63) / 64;
  return c < 1 ? 1 : (c > 32 ? 32 : c);
}

static size_t gsta_bwd_lds(const GstaBwdArgs& a) {
  const size_t esz = a.dt == LASER_BF16 ? 2 : 4;
  // H' in its storage type, its gradient in fp32 when several layers add to it, the vectors, alignment slack
  return (size_t)a.S * a.d * esz + sizeof(float) * ((a.M > 1 ? (size_t)a.S * a.d : 0) + (size_t)(a.M + 7) * a.d +
                                                    2 * (size_t)a.S + 4);
}

bool gsta_backward_supports(const GstaBwdArgs& a) {
  return a.d <= GB_MAXD && a.M <= GB_MAXM && gsta_bwd_lds(a) <= 150 * 1024;
}

// per-pair vectors [P][M][6][d], then the chunks' partial weight gradients [chunks][M][3][d][d]
size_t gsta_backward_work_bytes(int U, int C, int d, int M) {
  const size_t P = (size_t)U * C;
  return (P * M * 6 * d + (size_t)gsta_bwd_chunks((int)P) * M * 3 * d * d) * sizeof(float);
}

laser_status gsta_backward_launch(const GstaBwdArgs& a) {
  if (!gsta_backward_supports(a)) return LASER_ERR_UNSUPPORTED;
  const int P = a.U * a.C;
  const size_t lds = gsta_bwd_lds(a);
  if (a.dt == LASER_BF16) {
    auto kern = gsta_bwd_kernel<unsigned short>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)P), dim3(GB_THREADS), lds, a.stream, (const unsigned short*)a.seg,
                       (const unsigned short*)a.t0, (const unsigned short*)a.wq, (const unsigned short*)a.wk,
                       (const unsigned short*)a.wv, a.lens, a.dz, a.C, a.L, a.d, a.w, a.S, a.M,
                       (unsigned short*)a.dseg, a.dt0, a.work);
  } else {
    auto kern = gsta_bwd_kernel<float>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)P), dim3(GB_THREADS), lds, a.stream, (const float*)a.seg,
                       (const float*)a.t0, (const float*)a.wq, (const float*)a.wk, (const float*)a.wv, a.lens, a.dz, a.C,
                       a.L, a.d, a.w, a.S, a.M, (float*)a.dseg, a.dt0, a.work);
  }
  if (launch_status() != LASER_OK) return LASER_ERR_LAUNCH;
  const int tiles = (a.d + 31) / 32, chunks = gsta_bwd_chunks(P);
  float* part = a.work + (size_t)P * a.M * 6 * a.d;
  hipLaunchKernelGGL(gsta_bwd_w_partial_kernel, dim3((unsigned)(chunks * a.M * 3 * tiles * tiles)), dim3(256), 0,
                     a.stream, a.work, P, a.M, a.d, chunks, part);
  if (launch_status() != LASER_OK) return LASER_ERR_LAUNCH;
  const long long total = (long long)a.M * 3 * a.d * a.d;
  hipLaunchKernelGGL(gsta_bwd_w_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, a.stream, part, a.M,
                     a.d, chunks, a.dwq, a.dwk, a.dwv);
  return launch_status();
}

}  // namespace laser
