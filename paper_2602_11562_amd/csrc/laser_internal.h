// Internal declarations shared by the host entry points and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "laser.h"

namespace laser {

// Problem sizes after validation. S = ceil(L / w).
struct StaArgs {
  const void* q;
  const void* k;
  const void* v;
  const int32_t* lens;
  int U, C, L, d_q, d, w, S;
  float gamma;
  laser_dtype dt;
  void* seg_out;
  int32_t* seg_cnt;   // may be nullptr
  hipStream_t stream;
  bool reread;        // H' is read again right after this launch (the whole path): store it cacheable
  // ragged candidate counts: user u owns pairs cand_off[u] .. cand_off[u+1]-1 of q and seg_out (at most C of
  // them), P pairs in all; nullptr = every user has exactly C (pair index u * C + c)
  const int32_t* cand_off = nullptr;
  int P = 0;
  int heads = 1;      // attention heads: head h owns the h-th run of d_q / heads and d / heads columns
  bool softmax = false;   // softmax over a segment's valid items instead of sigmoid gates (ablation of Sec. 4.4.1)
};

struct GstaArgs {
  const void* seg;
  const void* t0;
  const void* wq;
  const void* wk;
  const void* wv;
  const int32_t* lens;
  int U, C, L, d, w, S, M;
  laser_dtype dt;
  float* z_out;
  hipStream_t stream;
  // optional: the views of laser_multires_forward from the same pass over H' (one-kernel form only)
  void* pool_out = nullptr;
  void* recent_out = nullptr;
  int r = 0;
  // ragged candidate counts, as in StaArgs (seg, t0 and z_out hold P pairs)
  const int32_t* cand_off = nullptr;
  int P = 0;
};

struct MultiresArgs {
  const void* seg;
  const int32_t* lens;
  int U, C, L, d, w, S, r;
  laser_dtype dt;
  void* pool_out;     // may be nullptr
  void* recent_out;   // may be nullptr (r == 0)
  hipStream_t stream;
  const int32_t* cand_off = nullptr;   // ragged candidate counts, as in StaArgs (seg and the outputs hold P pairs)
  int P = 0;
};
laser_status multires_launch(const MultiresArgs& a);
inline int gsta_pairs(const GstaArgs& a) { return a.cand_off ? a.P : a.U * a.C; }   // pairs in seg, t0 and z_out

struct FfnArgs {
  const void* seg;
  const int32_t* lens;
  const void* w1;
  const float* b1;
  const void* w2;
  const float* b2;
  const float* ln_g;
  const float* ln_b;
  int U, C, L, d, d_ff, w, S;
  float eps;
  laser_dtype dt;
  void* seg_out;
  hipStream_t stream;
  const int32_t* cand_off = nullptr;   // ragged candidate counts, as in StaArgs (seg and seg_out hold P pairs)
  int P = 0;
};
bool segment_ffn_generic_supports(const FfnArgs& a);
laser_status segment_ffn_generic_launch(const FfnArgs& a);
bool segment_ffn_mfma_supports(const FfnArgs& a);
laser_status segment_ffn_mfma_launch(const FfnArgs& a);

struct ProjArgs {          // Y_a = X W_a and, when n[1] > 0, Y_b = X W_b from the same pass over X
  const void* x;           // [rows, d_in]
  long long rows;
  int d_in;
  const void* w[2];        // [d_in, n[o]]
  int n[2];
  void* y[2];              // [rows, n[o]]
  laser_dtype dt;
  hipStream_t stream;
  int wpitch[2];           // elements between rows of w[o] and of y[o]: n[o] unless the matrices are column blocks of
  int ypitch[2];           // wider ones (the folded queries: two halves of one [d_in, 2 d_in] matrix and of its output)
};
laser_status project_generic_launch(const ProjArgs& a);
bool project_mfma_supports(const ProjArgs& a);
laser_status project_mfma_launch(const ProjArgs& a);

struct ProjHeadsArgs {     // y[p, i, h b + e] = sum_k x[p, h, i, k] wv[k, h b + e], b = d / heads
  const void* x;           // [P, heads, S, d_in]
  const void* wv;          // [d_in, d]
  long long P;
  int S, d_in, d, heads;
  laser_dtype dt;
  void* y;                 // [P, S, d]
  hipStream_t stream;
};
laser_status project_heads_generic_launch(const ProjHeadsArgs& a);
bool project_heads_mfma_supports(const ProjHeadsArgs& a);
laser_status project_heads_mfma_launch(const ProjHeadsArgs& a);
laser_status fold_weights_launch(const void* wq, const void* wk, int d_in, int d_q, int heads, laser_dtype dt,
                                 void* a_out, hipStream_t stream);

struct StaBwdArgs {        // gradients of STA: dq [U,C,d_q], dk [U,L,d_q], dv [U,L,d] (fp32) from dhp = dH' [U,C,S,d]
  const void* q;
  const void* k;
  const void* v;
  const void* dhp;
  const int32_t* lens;
  int U, C, L, d_q, d, w, S;
  float gamma;
  laser_dtype dt;
  float* dq;
  void* dk;                // fp32, or bf16 when grads_bf16
  void* dv;
  float* work;             // [U, groups, C, d_q] partial dq sums, sta_backward_work_bytes() bytes
  hipStream_t stream;
  bool grads_bf16 = false; // dk and dv in bf16 (the storage type of k and v)
};
bool sta_backward_supports(const StaBwdArgs& a);
size_t sta_backward_work_bytes(int U, int C, int L, int d_q, int w);
laser_status sta_backward_launch(const StaBwdArgs& a);

struct GstaBwdArgs {       // gradients of GSTA from dz = d loss / d z [U,C,d] (fp32)
  const void* seg;         // H' [U,C,S,d]
  const void* t0;
  const void* wq;
  const void* wk;
  const void* wv;
  const int32_t* lens;
  const float* dz;
  int U, C, L, d, w, S, M;
  laser_dtype dt;
  void* dseg;              // [U,C,S,d] dt
  float* dt0;              // [U,C,d]
  float* dwq;              // [M,d,d] each, summed over all pairs
  float* dwk;
  float* dwv;
  float* work;             // [U*C, M, 6, d] per-pair vectors, gsta_backward_work_bytes() bytes
  hipStream_t stream;
};
bool gsta_backward_supports(const GstaBwdArgs& a);
size_t gsta_backward_work_bytes(int U, int C, int d, int M);
laser_status gsta_backward_launch(const GstaBwdArgs& a);

struct FusedArgs {         // the whole path with one GSTA layer and H' never stored: z [U,C,d] fp32 from q, k, v, t0, weights
  const void* q;
  const void* k;
  const void* v;
  const void* t0;
  const void* wq;
  const void* wk;
  const void* wv;
  const int32_t* lens;
  int U, C, L, d_q, d, w, S;
  float gamma;
  laser_dtype dt;
  int32_t* seg_cnt;        // may be nullptr
  float* z_out;
  float* work;             // partial results of the runs of a user's history; nullptr = one run per user
  hipStream_t stream;
};
bool fused_generic_supports(const FusedArgs& a);
laser_status fused_generic_launch(const FusedArgs& a);
bool fused_mfma_supports(const FusedArgs& a);
size_t fused_work_bytes(const FusedArgs& a);   // what fused_mfma_launch wants in a.work to cut histories into runs (0: nothing)
laser_status fused_mfma_launch(const FusedArgs& a);
bool fused_stream_supports(const FusedArgs& a);   // few candidates per user: the streaming kernel with the layer as its epilogue
laser_status fused_stream_launch(const FusedArgs& a);

// Each launcher returns LASER_ERR_UNSUPPORTED (launching nothing) when the shape is outside its range.
bool sta_generic_supports(const StaArgs& a);
laser_status sta_generic_launch(const StaArgs& a);
bool sta_mfma_supports(const StaArgs& a);
laser_status sta_mfma_launch(const StaArgs& a);
bool sta_stream_supports(const StaArgs& a);
laser_status sta_stream_launch(const StaArgs& a);

bool gsta_generic_supports(const GstaArgs& a);
laser_status gsta_generic_launch(const GstaArgs& a);
bool gsta_tiled_supports(const GstaArgs& a);
laser_status gsta_tiled_launch(const GstaArgs& a);
bool gsta_split_supports(const GstaArgs& a);
laser_status gsta_split_launch(const GstaArgs& a);
laser_status gsta_r_launch(const GstaArgs& a);     // first launch of the split form alone: r into the z rows
laser_status gsta_out_launch(const GstaArgs& a);   // its last launch alone: z = t0 + p W_v from the z rows
// FFN + LayerNorm feeding one GSTA layer from a single pass over H' (ffn_gsta.hip); f.seg_out may be null
bool ffn_gsta_fused_supports(const FfnArgs& f, const GstaArgs& g);
laser_status ffn_gsta_fused_launch(const FfnArgs& f, const GstaArgs& g);
bool gsta_one_supports(const GstaArgs& a);
laser_status gsta_one_launch(const GstaArgs& a);
int gsta_one_max_recent(int d);   // largest r whose recent_out the one-kernel form writes itself

// Tuning overrides (workgroup shapes, kernel forms) exist only in builds made with -DLASER_TUNING, which are for
// parameter sweeps: the library as shipped never reads the environment, so it has one behaviour. Returns the
// variable's integer value, or `unset` when the variable is absent or the build is the shipped one.
inline int tuning_int(const char* name, int unset) {
#ifdef LASER_TUNING
  if (const char* e = getenv(name)) return atoi(e);
#endif
  (void)name;
  return unset;
}

inline laser_status launch_status() { return hipGetLastError() == hipSuccess ? LASER_OK : LASER_ERR_LAUNCH; }

// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b) { return __uint_as_float(((unsigned int)b) << 16); }

// Round-to-nearest-even float -> bfloat16 bits (hardware conversion on gfx950).
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float x) {
  __bf16 h = (__bf16)x;
  return __builtin_bit_cast(unsigned short, h);
}

template <typename T>
__device__ __forceinline__ float load_as_f32(const T* p, size_t i);
template <>
__device__ __forceinline__ float load_as_f32<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float load_as_f32<unsigned short>(const unsigned short* p, size_t i) {
  return bf16_bits_to_f32(p[i]);
}

template <typename T>
__device__ __forceinline__ void store_from_f32(T* p, size_t i, float x);
template <>
__device__ __forceinline__ void store_from_f32<float>(float* p, size_t i, float x) { p[i] = x; }
template <>
__device__ __forceinline__ void store_from_f32<unsigned short>(unsigned short* p, size_t i, float x) {
  p[i] = f32_to_bf16_bits(x);
}

// Valid length of user u, clamped to [0, L]; lens == nullptr means full length.
__device__ __forceinline__ int valid_len(const int32_t* lens, int u, int L) {
  if (lens == nullptr) return L;
  int n = lens[u];
  return n < 0 ? 0 : (n > L ? L : n);
}

// Pairs of user u: first pair index and how many. Dense layout (cand_off == nullptr): u * C and C. Ragged layout:
// cand_off[u] and cand_off[u+1] - cand_off[u], clamped to [0, P] and [0, min(C, P - first)], so that whatever the
// offsets hold, no index leaves the P pairs the buffers have.
struct CandRange { int first, count; };
__device__ __forceinline__ CandRange cand_range(const int32_t* cand_off, int u, int C, int P) {
  if (cand_off == nullptr) return CandRange{u * C, C};
  int b = cand_off[u], n = cand_off[u + 1] - b;
  b = b < 0 ? 0 : (b > P ? P : b);
  const int room = (P - b) < C ? (P - b) : C;
  n = n < 0 ? 0 : (n > room ? room : n);
  return CandRange{b, n};
}

// User of pair pr: pr / C in the dense layout, else the last u with cand_off[u] <= pr (users without candidates
// share their offset with the next user and are passed over).
__device__ __forceinline__ int pair_user(const int32_t* cand_off, int U, int C, int pr) {
  if (cand_off == nullptr) return pr / C;
  int lo = 0, hi = U;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cand_off[mid] <= pr) lo = mid;
    else hi = mid;
  }
  return lo;
}

// seg_cnt[u, i] = number of valid items of user u inside segment i (integer, exact). Called by one workgroup per
// user inside the STA kernels, so the counts cost no launch of their own.
__device__ __forceinline__ void write_seg_cnt(int32_t* seg_cnt, int u, int n, int L, int w, int S, int tid, int nt) {
  if (seg_cnt == nullptr) return;
  for (int i = tid; i < S; i += nt) {
    const int lo = i * w;
    int hi = lo + w;
    if (hi > L) hi = L;
    if (hi > n) hi = n;
    seg_cnt[(size_t)u * S + i] = hi > lo ? hi - lo : 0;
  }
}

// Sum over aligned groups of LANES consecutive lanes (2, 4, 8 or 16), the result in every lane of the group. The
// adds read their second operand through the data-parallel-primitive lane permutations of a 16-lane row (swap in
// pairs, swap pairs in quads, mirror the half row, mirror the row: after each step the lanes that were combined
// hold equal values, so a mirror reaches the other half's sum). A generic shuffle is an LDS round trip per step.
#define LASER_DPP_ADD(v, ctrl) \
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, 0xf, 0xf, false))
template <int LANES>
__device__ __forceinline__ float row_sum(float v) {
  static_assert(LANES == 1 || LANES == 2 || LANES == 4 || LANES == 8 || LANES == 16, "one 16-lane row at most");
  if (LANES >= 2) LASER_DPP_ADD(v, 0xB1);    // quad_perm [1,0,3,2]
  if (LANES >= 4) LASER_DPP_ADD(v, 0x4E);    // quad_perm [2,3,0,1]
  if (LANES >= 8) LASER_DPP_ADD(v, 0x141);   // row_half_mirror
  if (LANES >= 16) LASER_DPP_ADD(v, 0x140);  // row_mirror
  return v;
}
#undef LASER_DPP_ADD

// Sum over the 64 lanes, the same value in every lane: inside each row of 16 lanes with the lane-permute adds, then the
// four row sums are read into scalar registers and added (six generic shuffles would be six LDS round trips in the
// middle of every item's dependency chain).
__device__ __forceinline__ float wave_sum_rows(float x) {
  x = row_sum<16>(x);
  const int b = __float_as_int(x);
  return ((__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
          __int_as_float(__builtin_amdgcn_readlane(b, 32))) + __int_as_float(__builtin_amdgcn_readlane(b, 48));
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

}  // namespace laser
