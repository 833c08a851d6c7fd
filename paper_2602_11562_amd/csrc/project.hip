// The linear maps ahead of STA (paper Sec. 3.5.1, first two equations): Q = t W_q for the targets, K = H W_k and
// V = H W_v for every item of the raw history. One pass over the rows of X produces up to two outputs
// (Y_a = X W_a, Y_b = X W_b), so that H is read once for K and V.
//
// Two kernels. project_generic_kernel: fp32 arithmetic, any sizes, either storage type; a workgroup takes eight
// rows so that the weights, which it reads from L2, are used eight times. project_mfma_kernel: bf16 storage,
// d_in = 128, output widths multiples of 32 with at most 256 columns together, the product on the matrix cores
// with both weight matrices resident in LDS.
#include <cstdlib>

#include "laser_internal.h"

namespace laser {

constexpr int PG_ROWS = 8, PG_THREADS = 256;

template <typename T>
__global__ __launch_bounds__(PG_THREADS) void project_generic_kernel(const T* __restrict__ x, const T* __restrict__ wa,
                                                                     const T* __restrict__ wb, long long rows, int d_in,
                                                                     int na, int nb, int wpa, int wpb, int ypa, int ypb,
                                                                     T* __restrict__ ya, T* __restrict__ yb) {
  extern __shared__ float xs[];            // [PG_ROWS][d_in]
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * PG_ROWS;
  for (int e = tid; e < PG_ROWS * d_in; e += PG_THREADS) {
    const int rr = e / d_in, c = e - rr * d_in;
    const long long r = row0 + rr;
    xs[e] = r < rows ? load_as_f32(x, (size_t)r * d_in + c) : 0.0f;
  }
  __syncthreads();
  for (int j = tid; j < na + nb; j += PG_THREADS) {   // output column j of the eight rows
    const bool second = j >= na;
    const T* w = second ? wb : wa;
    const int col = second ? j - na : j, wp = second ? wpb : wpa, yp = second ? ypb : ypa;
    float acc[PG_ROWS];
#pragma unroll
    for (int rr = 0; rr < PG_ROWS; ++rr) acc[rr] = 0.0f;
    for (int e = 0; e < d_in; ++e) {
      const float wv = load_as_f32(w, (size_t)e * wp + col);
#pragma unroll
      for (int rr = 0; rr < PG_ROWS; ++rr) acc[rr] = fmaf(xs[rr * d_in + e], wv, acc[rr]);
    }
    T* y = second ? yb : ya;
#pragma unroll
    for (int rr = 0; rr < PG_ROWS; ++rr)
      if (row0 + rr < rows) store_from_f32(y, (size_t)(row0 + rr) * yp + col, acc[rr]);
  }
}

laser_status project_generic_launch(const ProjArgs& a) {
  const size_t lds = (size_t)PG_ROWS * a.d_in * sizeof(float);
  if (lds > 150 * 1024) return LASER_ERR_UNSUPPORTED;
  const long long blocks = (a.rows + PG_ROWS - 1) / PG_ROWS;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  if (blocks == 0) return LASER_OK;
  if (a.dt == LASER_BF16) {
    auto kern = project_generic_kernel<unsigned short>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(PG_THREADS), lds, a.stream, (const unsigned short*)a.x,
                       (const unsigned short*)a.w[0], (const unsigned short*)a.w[1], a.rows, a.d_in, a.n[0], a.n[1],
                       a.wpitch[0], a.wpitch[1], a.ypitch[0], a.ypitch[1], (unsigned short*)a.y[0],
                       (unsigned short*)a.y[1]);
  } else {
    auto kern = project_generic_kernel<float>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(PG_THREADS), lds, a.stream, (const float*)a.x,
                       (const float*)a.w[0], (const float*)a.w[1], a.rows, a.d_in, a.n[0], a.n[1], a.wpitch[0],
                       a.wpitch[1], a.ypitch[0], a.ypitch[1], (float*)a.y[0], (float*)a.y[1]);
  }
  return launch_status();
}

// ------------------------------------------------------------------------------------------ matrix-core form
// The operand scheme of the first layer of the segment FFN kernel (segment_ffn.hip): a wave owns 32 rows of X at a
// time (the B operand, read once into registers) and walks the output columns in tiles of 32:
//   Y^T tile [32 columns x 32 rows] = W^T tile . X^T      (v_mfma_f32_32x32x16_bf16, A from LDS 16 bytes per lane)
// In the accumulator layout a lane holds, for one row, four runs of four consecutive columns; they are rounded to
// bf16 and written into a wave-private LDS patch, and when the tiles of one output are done its rows leave as whole
// rows in 16-byte pieces. Both weight matrices are parked once per workgroup, transposed on the way in (row =
// output column, the d_in values of a column next to each other, padded pitch); workgroups walk the row tiles with
// a grid stride.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int PM_WAVES = 8, PM_THREADS = 64 * PM_WAVES, PM_ROWS = 32, PM_D = 128, PM_NMAX = 256, PM_OMAX = 128;

template <bool PF, bool NTS>   // PF: rows of the next tile requested one tile ahead; NTS: non-temporal output stores
__global__ __launch_bounds__(PM_THREADS) void project_mfma_kernel(const unsigned short* __restrict__ x,
                                                                  const unsigned short* __restrict__ wa,
                                                                  const unsigned short* __restrict__ wb, long long rows,
                                                                  int na, int nb, int wpa, int wpb, int ypa, int ypb,
                                                                  unsigned short* __restrict__ ya,
                                                                  unsigned short* __restrict__ yb) {
  constexpr int D = PM_D, KSTEPS = D / 16;
  constexpr int WP = D * 2 + 16;             // W^T row pitch: 16-byte reads of 32 consecutive rows hit all banks
  constexpr int OP = PM_OMAX * 2 + 16;       // output patch row pitch
  __shared__ __attribute__((aligned(16))) unsigned char WT[PM_NMAX * WP];
  __shared__ __attribute__((aligned(16))) unsigned char patch[PM_WAVES * PM_ROWS * OP];

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // The wave's first rows are requested before the weights are parked, and each later tile's rows while the
  // current tile is multiplied: the row loads are the only traffic that waits on HBM.
  const long long ntiles = (rows + PM_ROWS - 1) / PM_ROWS;
  const long long tstride = (long long)gridDim.x * PM_WAVES;
  long long t = (long long)blockIdx.x * PM_WAVES + wave;
  bf16x8 xreg[KSTEPS], xnext[KSTEPS];
  auto load_rows = [&](long long tile, bf16x8 (&dst)[KSTEPS]) {   // rows past the end repeat the last one; never stored
    long long r = tile * PM_ROWS + l32;
    r = r < rows ? r : rows - 1;
    const unsigned short* xr = x + (size_t)r * D + h * 8;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) dst[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xr + ks * 16));
  };
  load_rows(t < ntiles ? t : 0, xnext);

  // ---- park the weights: 16 bytes = 8 output columns of one k; consecutive threads take consecutive k, so that
  // their 2-byte writes into the transposed rows fall next to each other
  for (int which = 0; which < 2; ++which) {
    const unsigned short* wsrc = which ? wb : wa;
    const int n = which ? nb : na, base = which ? na : 0, wp = which ? wpb : wpa;
    for (int e = tid; e < D * n / 8; e += PM_THREADS) {
      const int kk = e % D, n0 = (e / D) * 8;
      const u32x4 raw = *reinterpret_cast<const u32x4*>(wsrc + (size_t)kk * wp + n0);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned short val = (unsigned short)((raw[j >> 1] >> ((j & 1) * 16)) & 0xffffu);
        *reinterpret_cast<unsigned short*>(WT + (base + n0 + j) * WP + kk * 2) = val;
      }
    }
  }
  __syncthreads();

  const unsigned char* wlane = WT + l32 * WP + h * 16;            // + tile * 32 * WP + ks * 32
  unsigned char* opatch = patch + wave * PM_ROWS * OP;
  const int nta = na / 32, ntiles_out = (na + nb) / 32;

  for (; t < ntiles; t += tstride) {
    const long long r0 = t * PM_ROWS;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) xreg[ks] = xnext[ks];   // the wave's rows as the B operand
    if (PF) load_rows(t + tstride < ntiles ? t + tstride : t, xnext);
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    bf16x8 wr[KSTEPS];
    auto read_w = [&](int j) {
      const unsigned char* a1 = wlane + j * 32 * WP;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) wr[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(a1 + ks * 32));
    };
    read_w(0);
#pragma unroll 1
    for (int j = 0; j < ntiles_out; ++j) {
      __builtin_amdgcn_sched_barrier(0);
      f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[0], xreg[0], zero, 0, 0, 0);
#pragma unroll
      for (int ks = 1; ks < KSTEPS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[ks], xreg[ks], acc, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      read_w(j + 1 < ntiles_out ? j + 1 : j);   // the next tile's weights are on their way during the rounding
      __builtin_amdgcn_sched_barrier(0);
      // column of element r inside the tile: 8 (r >> 2) + 4 h + (r & 3)
      const int jj = j < nta ? j : j - nta;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bf16x4 o = {(__bf16)acc[4 * g], (__bf16)acc[4 * g + 1], (__bf16)acc[4 * g + 2], (__bf16)acc[4 * g + 3]};
        *reinterpret_cast<u32x2*>(opatch + l32 * OP + (jj * 32 + g * 8 + h * 4) * 2) = __builtin_bit_cast(u32x2, o);
      }
      // last tile of an output: its rows leave as whole rows (LDS operations of a wave execute in order, so the
      // reads below see the writes above, and the next output's writes come after these reads: no barrier)
      if (j == nta - 1 || j == ntiles_out - 1) {
        const bool second = j >= nta;
        const int n = second ? nb : na, yp = second ? ypb : ypa;
        unsigned short* y = second ? yb : ya;
        const int lpr = n / 8;                     // 16-byte pieces per row
        for (int idx = lane; idx < PM_ROWS * lpr; idx += 64) {
          const int rr = idx / lpr, c = idx - rr * lpr;
          const u32x4 val = *reinterpret_cast<const u32x4*>(opatch + rr * OP + c * 16);
          if (r0 + rr < rows) {
            u32x4* dst = reinterpret_cast<u32x4*>(y + (size_t)(r0 + rr) * yp + c * 8);
            if (NTS) __builtin_nontemporal_store(val, dst);
            else *dst = val;
          }
        }
      }
    }
    if (!PF && t + tstride < ntiles) load_rows(t + tstride, xnext);
  }
}

// ------------------------------------------------------------------------------------------ folded form
// With few candidates per user it is cheaper not to form K and V at all (Sec. 3.5.1: the matrices do not depend on
// the position, so the products can be re-associated): the score of head h is (t A_h) . h_j with
// A_h = W_q,h W_k,h^T, the gated sums run over the raw items, and W_v is applied to the S segment sums instead of
// the L items. fold_weights_kernel forms A = [A_1 | ... | A_heads] once per model; the STA kernels then run with one
// pseudo-candidate per (candidate, head) and the raw history as keys and values; project_heads_* apply head h's
// columns of W_v to that head's sums and lay the results side by side:
//   y[p, i, h b + e] = sum_k x[p, h, i, k] W_v[k, h b + e],   b = d / heads,   x [P, heads, S, d_in], y [P, S, d].
template <typename T>
__global__ __launch_bounds__(256) void fold_weights_kernel(const T* __restrict__ wq, const T* __restrict__ wk, int d_in,
                                                           int d_q, int heads, T* __restrict__ a_out) {
  const long long total = (long long)d_in * heads * d_in;
  const int a = d_q / heads;
  for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
    const int r = (int)(e / ((long long)heads * d_in));
    const int c = (int)(e % ((long long)heads * d_in));
    const int h = c / d_in, kk = c % d_in;
    float acc = 0.0f;
    for (int x = 0; x < a; ++x)
      acc = fmaf(load_as_f32(wq, (size_t)r * d_q + h * a + x), load_as_f32(wk, (size_t)kk * d_q + h * a + x), acc);
    store_from_f32(a_out, (size_t)e, acc);
  }
}

laser_status fold_weights_launch(const void* wq, const void* wk, int d_in, int d_q, int heads, laser_dtype dt,
                                 void* a_out, hipStream_t stream) {
  const long long total = (long long)d_in * heads * d_in;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
  if (dt == LASER_BF16)
    hipLaunchKernelGGL(fold_weights_kernel<unsigned short>, dim3(blocks), dim3(256), 0, stream,
                       (const unsigned short*)wq, (const unsigned short*)wk, d_in, d_q, heads, (unsigned short*)a_out);
  else
    hipLaunchKernelGGL(fold_weights_kernel<float>, dim3(blocks), dim3(256), 0, stream, (const float*)wq,
                       (const float*)wk, d_in, d_q, heads, (float*)a_out);
  return launch_status();
}

template <typename T>
__global__ __launch_bounds__(PG_THREADS) void project_heads_generic_kernel(const T* __restrict__ x,
                                                                           const T* __restrict__ wv, long long rows,
                                                                           int S, int d_in, int d, int heads,
                                                                           T* __restrict__ y) {
  extern __shared__ float xs[];            // [PG_ROWS][heads][d_in]
  const int tid = threadIdx.x;
  const long long row0 = (long long)blockIdx.x * PG_ROWS;
  const int per_row = heads * d_in;
  for (int e = tid; e < PG_ROWS * per_row; e += PG_THREADS) {
    const int rr = e / per_row, rem = e - rr * per_row;
    const int h = rem / d_in, c = rem - h * d_in;
    const long long r = row0 + rr;
    float val = 0.0f;
    if (r < rows) {
      const long long p = r / S;
      const int i = (int)(r - p * S);
      val = load_as_f32(x, (size_t)(((p * heads + h) * S + i) * d_in + c));
    }
    xs[e] = val;
  }
  __syncthreads();
  const int b = d / heads;
  for (int j = tid; j < d; j += PG_THREADS) {
    const int h = j / b;
    float acc[PG_ROWS];
#pragma unroll
    for (int rr = 0; rr < PG_ROWS; ++rr) acc[rr] = 0.0f;
    for (int e = 0; e < d_in; ++e) {
      const float w = load_as_f32(wv, (size_t)e * d + j);
#pragma unroll
      for (int rr = 0; rr < PG_ROWS; ++rr) acc[rr] = fmaf(xs[(rr * heads + h) * d_in + e], w, acc[rr]);
    }
#pragma unroll
    for (int rr = 0; rr < PG_ROWS; ++rr)
      if (row0 + rr < rows) store_from_f32(y, (size_t)(row0 + rr) * d + j, acc[rr]);
  }
}

laser_status project_heads_generic_launch(const ProjHeadsArgs& a) {
  const size_t lds = (size_t)PG_ROWS * a.heads * a.d_in * sizeof(float);
  if (lds > 150 * 1024) return LASER_ERR_UNSUPPORTED;
  const long long rows = a.P * a.S;
  const long long blocks = (rows + PG_ROWS - 1) / PG_ROWS;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  if (blocks == 0) return LASER_OK;
  if (a.dt == LASER_BF16) {
    auto kern = project_heads_generic_kernel<unsigned short>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(PG_THREADS), lds, a.stream, (const unsigned short*)a.x,
                       (const unsigned short*)a.wv, rows, a.S, a.d_in, a.d, a.heads, (unsigned short*)a.y);
  } else {
    auto kern = project_heads_generic_kernel<float>;
    if (lds > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return LASER_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(PG_THREADS), lds, a.stream, (const float*)a.x,
                       (const float*)a.wv, rows, a.S, a.d_in, a.d, a.heads, (float*)a.y);
  }
  return launch_status();
}

// Matrix-core form of the same: project_mfma_kernel with one output, whose 32 rows are re-read per head from that
// head's block of x (row r = p S + i of head h lies at ((p heads + h) S + i) d_in) before the head's column tiles.
__global__ __launch_bounds__(PM_THREADS) void project_heads_mfma_kernel(const unsigned short* __restrict__ x,
                                                                        const unsigned short* __restrict__ wv,
                                                                        long long rows, int S, int d, int heads,
                                                                        unsigned short* __restrict__ y) {
  constexpr int D = PM_D, KSTEPS = D / 16;
  constexpr int WP = D * 2 + 16, OP = PM_OMAX * 2 + 16;
  __shared__ __attribute__((aligned(16))) unsigned char WT[PM_OMAX * WP];
  __shared__ __attribute__((aligned(16))) unsigned char patch[PM_WAVES * PM_ROWS * OP];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int e = tid; e < D * d / 8; e += PM_THREADS) {   // W_v transposed, as in project_mfma_kernel
    const int kk = e % D, n0 = (e / D) * 8;
    const u32x4 raw = *reinterpret_cast<const u32x4*>(wv + (size_t)kk * d + n0);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned short val = (unsigned short)((raw[j >> 1] >> ((j & 1) * 16)) & 0xffffu);
      *reinterpret_cast<unsigned short*>(WT + (n0 + j) * WP + kk * 2) = val;
    }
  }
  __syncthreads();
  const unsigned char* wlane = WT + l32 * WP + h * 16;
  unsigned char* opatch = patch + wave * PM_ROWS * OP;
  const int tiles_per_head = d / heads / 32;
  const int lpr = d / 8;
  const long long ntiles = (rows + PM_ROWS - 1) / PM_ROWS;
  for (long long t = (long long)blockIdx.x * PM_WAVES + wave; t < ntiles; t += (long long)gridDim.x * PM_WAVES) {
    const long long r0 = t * PM_ROWS;
    long long r = r0 + l32;
    r = r < rows ? r : rows - 1;           // rows past the end repeat the last one; never stored
    const long long p = r / S;
    const int i = (int)(r - p * S);
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 1
    for (int hd = 0; hd < heads; ++hd) {
      bf16x8 xreg[KSTEPS];
      const unsigned short* xr = x + (size_t)(((p * heads + hd) * S + i) * D) + h * 8;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) xreg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xr + ks * 16));
#pragma unroll 1
      for (int jt = 0; jt < tiles_per_head; ++jt) {
        const int j = hd * tiles_per_head + jt;
        const unsigned char* a1 = wlane + j * 32 * WP;
        bf16x8 wr[KSTEPS];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) wr[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(a1 + ks * 32));
        f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[0], xreg[0], zero, 0, 0, 0);
#pragma unroll
        for (int ks = 1; ks < KSTEPS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[ks], xreg[ks], acc, 0, 0, 0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 o = {(__bf16)acc[4 * g], (__bf16)acc[4 * g + 1], (__bf16)acc[4 * g + 2], (__bf16)acc[4 * g + 3]};
          *reinterpret_cast<u32x2*>(opatch + l32 * OP + (j * 32 + g * 8 + h * 4) * 2) = __builtin_bit_cast(u32x2, o);
        }
      }
    }
    for (int idx = lane; idx < PM_ROWS * lpr; idx += 64) {   // LDS operations of a wave execute in order: no barrier
      const int rr = idx / lpr, c = idx - rr * lpr;
      const u32x4 val = *reinterpret_cast<const u32x4*>(opatch + rr * OP + c * 16);
      if (r0 + rr < rows) *reinterpret_cast<u32x4*>(y + (size_t)(r0 + rr) * d + c * 8) = val;
    }
  }
}

bool project_heads_mfma_supports(const ProjHeadsArgs& a) {
  if (a.dt != LASER_BF16 || a.d_in != PM_D || a.d > PM_OMAX || a.heads < 1) return false;
  return a.d % a.heads == 0 && (a.d / a.heads) % 32 == 0;
}

laser_status project_heads_mfma_launch(const ProjHeadsArgs& a) {
  if (!project_heads_mfma_supports(a)) return LASER_ERR_UNSUPPORTED;
  const long long rows = a.P * a.S;
  if (rows == 0) return LASER_OK;
  const long long ntiles = (rows + PM_ROWS - 1) / PM_ROWS;
  long long blocks = (ntiles + PM_WAVES - 1) / PM_WAVES;
  if (blocks > 256) blocks = 256;
  hipLaunchKernelGGL(project_heads_mfma_kernel, dim3((unsigned)blocks), dim3(PM_THREADS), 0, a.stream,
                     (const unsigned short*)a.x, (const unsigned short*)a.wv, rows, a.S, a.d, a.heads,
                     (unsigned short*)a.y);
  return launch_status();
}

bool project_mfma_supports(const ProjArgs& a) {
  if (a.dt != LASER_BF16 || a.d_in != PM_D) return false;
  for (int o = 0; o < 2; ++o)
    if (a.n[o] % 32 != 0 || a.n[o] > PM_OMAX || a.wpitch[o] % 8 != 0 || a.ypitch[o] % 8 != 0) return false;
  return a.n[0] >= 32 && a.n[0] + a.n[1] <= PM_NMAX;
}

laser_status project_mfma_launch(const ProjArgs& a) {
  if (!project_mfma_supports(a)) return LASER_ERR_UNSUPPORTED;
  if (a.rows == 0) return LASER_OK;
  const long long ntiles = (a.rows + PM_ROWS - 1) / PM_ROWS;
  long long blocks = (ntiles + PM_WAVES - 1) / PM_WAVES;
  if (blocks > 256) blocks = 256;   // one workgroup per compute unit (LDS), each walking several tiles per wave
  // Non-temporal stores are worth 10-15 % up to about a gigabyte of traffic and cost a few per cent beyond it;
  // requesting rows a tile ahead gains nothing measurable (two waves per SIMD already cover the latency).
  const double bytes = (double)a.rows * (a.d_in + a.n[0] + a.n[1]) * 2.0;
  int mode = bytes <= 2.0e9 ? 2 : 0;
  mode = tuning_int("LASER_PROJECT_MODE", mode) & 3;   // tuning builds only: 1 = PF, 2 = NTS
#define LASER_PROJECT_LAUNCH(PF, NTS)                                                                              \
  hipLaunchKernelGGL((project_mfma_kernel<PF, NTS>), dim3((unsigned)blocks), dim3(PM_THREADS), 0, a.stream,        \
                     (const unsigned short*)a.x, (const unsigned short*)a.w[0], (const unsigned short*)a.w[1],     \
                     a.rows, a.n[0], a.n[1], a.wpitch[0], a.wpitch[1], a.ypitch[0], a.ypitch[1],                  \
                     (unsigned short*)a.y[0], (unsigned short*)a.y[1])
  if (mode == 0) LASER_PROJECT_LAUNCH(false, false);
  else if (mode == 1) LASER_PROJECT_LAUNCH(true, false);
  else if (mode == 2) LASER_PROJECT_LAUNCH(false, true);
  else LASER_PROJECT_LAUNCH(true, true);
#undef LASER_PROJECT_LAUNCH
  return launch_status();
}

}  // namespace laser
