// The two other views of the multi-resolution fusion (paper Sec. 3.4.4), from a stored H' [U, C, S, d]:
//   pool   [U, C, d]    = component-wise maximum over the segment vectors that hold at least one valid item
//                         (0 when there is none), in the storage type: a maximum of stored values is a stored value,
//                         so the result is exact;
//   recent [U, C, r, d] = the r most recent segments, rows 0 .. r-1 of H' (a copy).
// HBM streaming, nothing to contract: one thread owns one 16-byte piece of a pair's row (8 bf16 or 4 fp32 values)
// and walks the pair's valid segments, so that the threads of a wave read whole consecutive rows. Only valid segments
// are read; `recent` rows past them are copied as stored (STA stores zeros there).
#include "laser_internal.h"

namespace laser {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// larger of two packed bf16 pairs, component by component (values compared as floats, bits passed through)
__device__ __forceinline__ unsigned int max_bf16x2(unsigned int a, unsigned int b) {
  const float alo = __uint_as_float(a << 16), blo = __uint_as_float(b << 16);
  const float ahi = __uint_as_float(a & 0xffff0000u), bhi = __uint_as_float(b & 0xffff0000u);
  const unsigned int lo = blo > alo ? (b & 0xffffu) : (a & 0xffffu);
  const unsigned int hi = bhi > ahi ? (b & 0xffff0000u) : (a & 0xffff0000u);
  return lo | hi;
}

template <bool BF16>
__device__ __forceinline__ u32x4 max_piece(const u32x4& a, const u32x4& b) {
  u32x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (BF16) o[e] = max_bf16x2(a[e], b[e]);
    else o[e] = __uint_as_float(b[e]) > __uint_as_float(a[e]) ? b[e] : a[e];
  }
  return o;
}

// pieces = 16-byte pieces per row; one thread per (pair, piece)
template <bool BF16>
__global__ __launch_bounds__(256) void multires_kernel(const u32x4* __restrict__ seg, const int32_t* __restrict__ lens,
                                                       const int32_t* __restrict__ cand_off, int U,
                                                       long long total, int pieces, int C, int L, int w, int S, int r,
                                                       u32x4* __restrict__ pool, u32x4* __restrict__ recent) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= total) return;
  const long long pair = t / pieces;
  const int piece = (int)(t - pair * pieces);
  const int u = pair_user(cand_off, U, C, (int)pair);
  const int nv = (valid_len(lens, u, L) + w - 1) / w;   // segments with a valid item: a prefix
  const u32x4* H = seg + (size_t)pair * S * pieces + piece;
  if (recent != nullptr) {
    u32x4* R = recent + (size_t)pair * r * pieces + piece;
    for (int i = 0; i < r; ++i) R[(size_t)i * pieces] = H[(size_t)i * pieces];
  }
  if (pool != nullptr) {
    u32x4 m = {0u, 0u, 0u, 0u};
    if (nv > 0) {
      m = H[0];
      int i = 1;
      for (; i + 4 <= nv; i += 4) {   // four independent loads in flight
        const u32x4 a = H[(size_t)i * pieces], b = H[(size_t)(i + 1) * pieces];
        const u32x4 c = H[(size_t)(i + 2) * pieces], d = H[(size_t)(i + 3) * pieces];
        m = max_piece<BF16>(m, max_piece<BF16>(max_piece<BF16>(a, b), max_piece<BF16>(c, d)));
      }
      for (; i < nv; ++i) m = max_piece<BF16>(m, H[(size_t)i * pieces]);
    }
    pool[(size_t)pair * pieces + piece] = m;
  }
}

laser_status multires_launch(const MultiresArgs& a) {
  const int esize = a.dt == LASER_BF16 ? 2 : 4;
  const int pieces = a.d * esize / 16;
  const long long total = (long long)(a.cand_off ? a.P : a.U * a.C) * pieces;
  const long long blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffLL) return LASER_ERR_SHAPE;
  if (a.dt == LASER_BF16)
    hipLaunchKernelGGL((multires_kernel<true>), dim3((unsigned)blocks), dim3(256), 0, a.stream, (const u32x4*)a.seg,
                       a.lens, a.cand_off, a.U, total, pieces, a.C, a.L, a.w, a.S, a.r, (u32x4*)a.pool_out, (u32x4*)a.recent_out);
  else
    hipLaunchKernelGGL((multires_kernel<false>), dim3((unsigned)blocks), dim3(256), 0, a.stream, (const u32x4*)a.seg,
                       a.lens, a.cand_off, a.U, total, pieces, a.C, a.L, a.w, a.S, a.r, (u32x4*)a.pool_out, (u32x4*)a.recent_out);
  return launch_status();
}

}  // namespace laser
