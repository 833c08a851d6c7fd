// Host side of the C ABI: argument validation (GPU-free), kernel selection, launches.
#include <initializer_list>
#include <mutex>

#include "laser_internal.h"

namespace laser {

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// a * b * c * d <= lim for non-negative factors, without overflow: the product is cut off as soon as it passes lim
static bool product_fits(long long lim, long long a, long long b = 1, long long c = 1, long long d = 1) {
  long long p = 1;
  for (long long f : {a, b, c, d}) {
    if (f < 0) return false;
    if (f != 0 && p > lim / f) return false;
    p *= f;
  }
  return p <= lim;
}

static laser_status check_dims(int U, int C, int L, int d_q, int d, int w) {
  if (U <= 0 || C <= 0 || L <= 0 || d_q <= 0 || d <= 0 || w <= 0) return LASER_ERR_SHAPE;
  if (d_q > 1024 || d > 1024 || (d_q % 8) != 0 || (d % 8) != 0) return LASER_ERR_SHAPE;
  const long long S = ((long long)L + w - 1) / w;
  const long long lim = 0x7fffffffLL;
  if (!product_fits(lim, U, C, d_q) || !product_fits(lim, U, L, d_q) || !product_fits(lim, U, L, d) ||
      !product_fits(lim, U, C, S, d) || !product_fits(lim, U, S))
    return LASER_ERR_SHAPE;
  return LASER_OK;
}

// S = ceil(L / w) for sizes that passed check_dims (L + w may pass the range of int)
static int segments(int L, int w) { return (int)(((long long)L + w - 1) / w); }

static laser_status validate_sta(const void* q, const void* k, const void* v, const int32_t* lens, int U, int C,
                                 int L, int d_q, int d, int w, float gamma, laser_dtype dt, void* seg_out,
                                 int32_t* seg_cnt, void* stream, StaArgs* out, bool seg_required = true) {
  if (!q || !k || !v || (seg_required && !seg_out)) return LASER_ERR_NULL;
  if (dt != LASER_F32 && dt != LASER_BF16) return LASER_ERR_DTYPE;
  laser_status s = check_dims(U, C, L, d_q, d, w);
  if (s != LASER_OK) return s;
  if (!(gamma > 0.0f) || !(gamma < INFINITY)) return LASER_ERR_SHAPE;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(seg_out)) return LASER_ERR_ALIGN;
  if ((lens && (reinterpret_cast<uintptr_t>(lens) & 3u)) || (seg_cnt && (reinterpret_cast<uintptr_t>(seg_cnt) & 3u)))
    return LASER_ERR_ALIGN;
  *out = StaArgs{q, k, v, lens, U, C, L, d_q, d, w, segments(L, w), gamma, dt, seg_out, seg_cnt,
                 static_cast<hipStream_t>(stream)};
  return LASER_OK;
}

static laser_status validate_gsta(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                  const int32_t* lens, int U, int C, int L, int d, int w, int M, laser_dtype dt,
                                  float* z_out, void* stream, GstaArgs* out) {
  if (!seg || !t0 || !wq || !wk || !wv || !z_out) return LASER_ERR_NULL;
  if (dt != LASER_F32 && dt != LASER_BF16) return LASER_ERR_DTYPE;
  laser_status s = check_dims(U, C, L, d, d, w);
  if (s != LASER_OK) return s;
  const int S = segments(L, w);
  if (M <= 0 || M > 64 || S > 4096) return LASER_ERR_SHAPE;
  if (!aligned16(seg) || !aligned16(t0) || !aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(z_out))
    return LASER_ERR_ALIGN;
  if (lens && (reinterpret_cast<uintptr_t>(lens) & 3u)) return LASER_ERR_ALIGN;
  *out = GstaArgs{seg, t0, wq, wk, wv, lens, U, C, L, d, w, S, M, dt, z_out, static_cast<hipStream_t>(stream)};
  return LASER_OK;
}

static laser_status validate_multires(const void* seg, const int32_t* lens, int U, int C, int L, int d, int w, int r,
                                      laser_dtype dt, void* pool_out, void* recent_out, void* stream,
                                      MultiresArgs* out) {
  if (!seg || (!pool_out && !recent_out)) return LASER_ERR_NULL;
  if (dt != LASER_F32 && dt != LASER_BF16) return LASER_ERR_DTYPE;
  laser_status s = check_dims(U, C, L, d, d, w);
  if (s != LASER_OK) return s;
  const int S = segments(L, w);
  if (r < 0 || r > S || (r > 0) != (recent_out != nullptr)) return LASER_ERR_SHAPE;
  if (!product_fits(0x7fffffffLL, U, C, r > 0 ? r : 1, d)) return LASER_ERR_SHAPE;
  if (!aligned16(seg) || !aligned16(pool_out) || !aligned16(recent_out)) return LASER_ERR_ALIGN;
  if (lens && (reinterpret_cast<uintptr_t>(lens) & 3u)) return LASER_ERR_ALIGN;
  *out = MultiresArgs{seg, lens, U, C, L, d, w, S, r, dt, pool_out, recent_out, static_cast<hipStream_t>(stream)};
  return LASER_OK;
}

static laser_status validate_ffn(const void* seg, const int32_t* lens, const void* w1, const float* b1, const void* w2,
                                 const float* b2, const float* ln_g, const float* ln_b, int U, int C, int L, int d,
                                 int d_ff, int w, float eps, laser_dtype dt, void* seg_out, void* stream, FfnArgs* out,
                                 bool seg_out_required = true) {
  if (!seg || !w1 || !b1 || !w2 || !b2 || !ln_g || !ln_b || (seg_out_required && !seg_out)) return LASER_ERR_NULL;
  if (dt != LASER_F32 && dt != LASER_BF16) return LASER_ERR_DTYPE;
  laser_status s = check_dims(U, C, L, d, d, w);
  if (s != LASER_OK) return s;
  if (d_ff <= 0 || d_ff > 4096 || (d_ff % 8) != 0) return LASER_ERR_SHAPE;
  if (!(eps >= 0.0f) || !(eps < INFINITY)) return LASER_ERR_SHAPE;
  if (!aligned16(seg) || !aligned16(w1) || !aligned16(w2) || !aligned16(seg_out)) return LASER_ERR_ALIGN;
  for (const void* p : {(const void*)b1, (const void*)b2, (const void*)ln_g, (const void*)ln_b, (const void*)lens})
    if (reinterpret_cast<uintptr_t>(p) & 3u) return LASER_ERR_ALIGN;
  *out = FfnArgs{seg, lens, w1, b1, w2, b2, ln_g, ln_b, U, C, L, d, d_ff, w, segments(L, w), eps, dt, seg_out,
                 static_cast<hipStream_t>(stream)};
  return LASER_OK;
}

static laser_sta_variant pick_sta(const StaArgs& a) {
  if (sta_stream_supports(a)) return LASER_STA_STREAM;
  if (sta_mfma_supports(a)) return LASER_STA_MFMA;
  return LASER_STA_GENERIC;
}

static laser_gsta_variant pick_gsta(const GstaArgs& a) {
  if (gsta_one_supports(a)) return LASER_GSTA_ONE;
  if (gsta_split_supports(a)) return LASER_GSTA_SPLIT;
  return gsta_tiled_supports(a) ? LASER_GSTA_TILED : LASER_GSTA_GENERIC;
}

static laser_status run_sta(const StaArgs& a, laser_sta_variant variant) {
  if (variant == LASER_STA_AUTO) variant = pick_sta(a);
  laser_status s;
  switch (variant) {
    case LASER_STA_GENERIC: s = sta_generic_launch(a); break;
    case LASER_STA_MFMA: s = sta_mfma_launch(a); break;
    case LASER_STA_MFMA_CACHED: {
      StaArgs b = a;
      b.reread = true;
      s = sta_mfma_launch(b);
      break;
    }
    case LASER_STA_STREAM: s = sta_stream_launch(a); break;
    default: return LASER_ERR_UNSUPPORTED;
  }
  return s;   // every STA kernel also writes seg_cnt when it is requested
}

static laser_status run_gsta(const GstaArgs& a, laser_gsta_variant variant) {
  if (variant == LASER_GSTA_AUTO) variant = pick_gsta(a);
  switch (variant) {
    case LASER_GSTA_GENERIC: return gsta_generic_launch(a);
    case LASER_GSTA_TILED: return gsta_tiled_launch(a);
    case LASER_GSTA_SPLIT: return gsta_split_launch(a);
    case LASER_GSTA_ONE: return gsta_one_launch(a);
    default: return LASER_ERR_UNSUPPORTED;
  }
}

// GSTA and the two other views of Sec. 3.4.4 from one pass over H' where the GSTA kernel writes them itself (the
// one-kernel form, up to the number of recent rows it can stage, and the split form's streaming kernel); a second
// launch over H' otherwise
static laser_status run_gsta_views(GstaArgs& ga, MultiresArgs& ma) {
  const laser_gsta_variant variant = pick_gsta(ga);
  if (variant == LASER_GSTA_ONE) {
    ga.pool_out = ma.pool_out;
    if (ma.r <= gsta_one_max_recent(ga.d)) {
      ga.recent_out = ma.recent_out;
      ga.r = ma.r;
      return run_gsta(ga, LASER_GSTA_ONE);
    }
    const laser_status s = run_gsta(ga, LASER_GSTA_ONE);   // more recent segments than the kernel can stage: a copy launch for those
    if (s != LASER_OK) return s;
    ma.pool_out = nullptr;
    return multires_launch(ma);
  }
  if (variant == LASER_GSTA_SPLIT) {
    ga.pool_out = ma.pool_out;
    ga.recent_out = ma.recent_out;
    ga.r = ma.r;
    return run_gsta(ga, LASER_GSTA_SPLIT);
  }
  const laser_status s = run_gsta(ga, variant);
  if (s != LASER_OK) return s;
  return multires_launch(ma);
}

// The whole path without H' in memory (one GSTA layer): checks, then the fused kernels' arguments
static laser_status validate_fused(const void* q, const void* k, const void* v, const void* t0, const void* wq,
                                   const void* wk, const void* wv, const int32_t* lens, int U, int C, int L, int d_q,
                                   int d, int w, float gamma, laser_dtype dt, int32_t* seg_cnt, float* z_out,
                                   void* stream, FusedArgs* out) {
  StaArgs sa;
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, nullptr, seg_cnt, stream, &sa, false);
  if (s != LASER_OK) return s;
  if (!t0 || !wq || !wk || !wv || !z_out) return LASER_ERR_NULL;
  if (sa.S > 4096) return LASER_ERR_SHAPE;   // as for laser_gsta_forward
  if (!aligned16(t0) || !aligned16(wq) || !aligned16(wk) || !aligned16(wv) || !aligned16(z_out)) return LASER_ERR_ALIGN;
  *out = FusedArgs{q, k, v, t0, wq, wk, wv, lens, U, C, L, d_q, d, w, sa.S, gamma, dt, seg_cnt, z_out, nullptr,
                   static_cast<hipStream_t>(stream)};
  return LASER_OK;
}

// Scratch the fused kernels want in a.work to cut histories into runs (0: whole histories per workgroup)
static size_t fused_need_bytes(const FusedArgs& a) { return fused_stream_supports(a) ? 0 : fused_work_bytes(a); }

static laser_status run_fused(const FusedArgs& a) {
  if (fused_stream_supports(a)) return fused_stream_launch(a);
  return fused_mfma_supports(a) ? fused_mfma_launch(a) : fused_generic_launch(a);
}

}  // namespace laser

using namespace laser;

extern "C" {

laser_status laser_sta_forward_variant(const void* q, const void* k, const void* v, const int32_t* lens, int U,
                                       int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt,
                                       void* seg_out, int32_t* seg_cnt, void* stream, laser_sta_variant variant) {
  StaArgs a;
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &a);
  if (s != LASER_OK) return s;
  if (variant < LASER_STA_AUTO || variant > LASER_STA_MFMA_CACHED) return LASER_ERR_UNSUPPORTED;
  return run_sta(a, variant);
}

laser_status laser_sta_forward_heads(const void* q, const void* k, const void* v, const int32_t* lens, int U, int C,
                                     int L, int d_q, int d, int w, float gamma, int heads, laser_dtype dt,
                                     void* seg_out, int32_t* seg_cnt, void* stream, laser_sta_variant variant) {
  StaArgs a;
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &a);
  if (s != LASER_OK) return s;
  if (heads < 1 || heads > 64 || d_q % heads != 0 || d % heads != 0) return LASER_ERR_SHAPE;
  if (variant < LASER_STA_AUTO || variant > LASER_STA_MFMA_CACHED) return LASER_ERR_UNSUPPORTED;
  a.heads = heads;
  return run_sta(a, variant);
}

laser_status laser_sta_forward_softmax(const void* q, const void* k, const void* v, const int32_t* lens, int U, int C,
                                       int L, int d_q, int d, int w, float gamma, int heads, laser_dtype dt,
                                       void* seg_out, int32_t* seg_cnt, void* stream, laser_sta_variant variant) {
  StaArgs a;
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &a);
  if (s != LASER_OK) return s;
  if (heads < 1 || heads > 64 || d_q % heads != 0 || d % heads != 0) return LASER_ERR_SHAPE;
  if (variant < LASER_STA_AUTO || variant > LASER_STA_MFMA_CACHED) return LASER_ERR_UNSUPPORTED;
  a.heads = heads;
  a.softmax = true;
  return run_sta(a, variant);
}

// Ragged candidate counts: the pair tensors hold P rows, user u's candidates are rows cand_off[u] .. cand_off[u+1]-1
static laser_status validate_ragged(const int32_t* cand_off, int U, int C_max, int P, int L, int d_q, int d, int w) {
  if (!cand_off) return LASER_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(cand_off) & 3u) return LASER_ERR_ALIGN;
  if (P <= 0 || (long long)P > (long long)U * C_max) return LASER_ERR_SHAPE;
  const long long S = ((long long)L + w - 1) / w;
  if (!product_fits(0x7fffffffLL, P, S, d) || !product_fits(0x7fffffffLL, P, d_q)) return LASER_ERR_SHAPE;
  return LASER_OK;
}

laser_status laser_sta_forward_ragged(const void* q, const void* k, const void* v, const int32_t* lens,
                                      const int32_t* cand_off, int U, int C_max, int P, int L, int d_q, int d, int w,
                                      float gamma, laser_dtype dt, void* seg_out, int32_t* seg_cnt, void* stream) {
  StaArgs a;
  laser_status s = validate_sta(q, k, v, lens, U, C_max, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &a);
  if (s != LASER_OK) return s;
  s = validate_ragged(cand_off, U, C_max, P, L, d_q, d, w);
  if (s != LASER_OK) return s;
  a.cand_off = cand_off;
  a.P = P;
  return run_sta(a, LASER_STA_AUTO);
}

laser_status laser_gsta_forward_ragged(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                       const int32_t* lens, const int32_t* cand_off, int U, int C_max, int P, int L,
                                       int d, int w, int M, laser_dtype dt, float* z_out, void* stream) {
  GstaArgs a;
  laser_status s = validate_gsta(seg, t0, wq, wk, wv, lens, U, C_max, L, d, w, M, dt, z_out, stream, &a);
  if (s != LASER_OK) return s;
  s = validate_ragged(cand_off, U, C_max, P, L, d, d, w);
  if (s != LASER_OK) return s;
  a.cand_off = cand_off;
  a.P = P;
  return run_gsta(a, LASER_GSTA_AUTO);
}

laser_status laser_forward_ragged(const void* q, const void* k, const void* v, const void* t0, const void* wq,
                                  const void* wk, const void* wv, const int32_t* lens, const int32_t* cand_off, int U,
                                  int C_max, int P, int L, int d_q, int d, int w, float gamma, int M, laser_dtype dt,
                                  void* seg_out, int32_t* seg_cnt, float* z_out, void* stream) {
  StaArgs sa;
  GstaArgs ga;
  laser_status s = validate_sta(q, k, v, lens, U, C_max, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &sa);
  if (s != LASER_OK) return s;
  s = validate_gsta(seg_out, t0, wq, wk, wv, lens, U, C_max, L, d, w, M, dt, z_out, stream, &ga);
  if (s != LASER_OK) return s;
  s = validate_ragged(cand_off, U, C_max, P, L, d_q, d, w);
  if (s != LASER_OK) return s;   // everything validated before the first launch
  sa.cand_off = ga.cand_off = cand_off;
  sa.P = ga.P = P;
  sa.reread = true;
  s = run_sta(sa, LASER_STA_AUTO);
  if (s != LASER_OK) return s;
  return run_gsta(ga, LASER_GSTA_AUTO);
}

laser_status laser_sta_forward(const void* q, const void* k, const void* v, const int32_t* lens, int U, int C,
                               int L, int d_q, int d, int w, float gamma, laser_dtype dt, void* seg_out,
                               int32_t* seg_cnt, void* stream) {
  return laser_sta_forward_variant(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream,
                                   LASER_STA_AUTO);
}

laser_status laser_gsta_forward_variant(const void* seg, const void* t0, const void* wq, const void* wk,
                                        const void* wv, const int32_t* lens, int U, int C, int L, int d, int w,
                                        int M, laser_dtype dt, float* z_out, void* stream,
                                        laser_gsta_variant variant) {
  GstaArgs a;
  laser_status s = validate_gsta(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream, &a);
  if (s != LASER_OK) return s;
  if (variant < LASER_GSTA_AUTO || variant > LASER_GSTA_ONE) return LASER_ERR_UNSUPPORTED;
  return run_gsta(a, variant);
}

laser_status laser_gsta_forward(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                const int32_t* lens, int U, int C, int L, int d, int w, int M, laser_dtype dt,
                                float* z_out, void* stream) {
  return laser_gsta_forward_variant(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream,
                                    LASER_GSTA_AUTO);
}

laser_status laser_forward(const void* q, const void* k, const void* v, const void* t0, const void* wq,
                           const void* wk, const void* wv, const int32_t* lens, int U, int C, int L, int d_q, int d,
                           int w, float gamma, int M, laser_dtype dt, void* seg_out, int32_t* seg_cnt, float* z_out,
                           void* stream) {
  if (seg_out == nullptr) {   // H' not wanted: the fused kernels, every workgroup walking a whole history
    FusedArgs fa;
    const laser_status fs = validate_fused(q, k, v, t0, wq, wk, wv, lens, U, C, L, d_q, d, w, gamma, dt, seg_cnt, z_out,
                                           stream, &fa);
    if (fs != LASER_OK) return fs;
    if (M <= 0 || M > 64) return LASER_ERR_SHAPE;
    if (M != 1) return LASER_ERR_UNSUPPORTED;   // a second layer reads every segment vector again
    return run_fused(fa);
  }
  StaArgs sa;
  GstaArgs ga;
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &sa);
  if (s != LASER_OK) return s;
  s = validate_gsta(seg_out, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream, &ga);
  if (s != LASER_OK) return s;   // both validated before the first launch
  sa.reread = true;   // GSTA streams H' next: leave it where the last-level cache can keep it
  s = run_sta(sa, LASER_STA_AUTO);
  if (s != LASER_OK) return s;
  return run_gsta(ga, LASER_GSTA_AUTO);
}

size_t laser_forward_fused_work_bytes(int U, int C, int L, int d_q, int d, int w, laser_dtype dt) {
  if (check_dims(U, C, L, d_q, d, w) != LASER_OK || (dt != LASER_F32 && dt != LASER_BF16)) return 0;
  FusedArgs a{};
  a.U = U; a.C = C; a.L = L; a.d_q = d_q; a.d = d; a.w = w; a.S = segments(L, w); a.gamma = 1.0f; a.dt = dt;
  return fused_need_bytes(a);
}

laser_status laser_forward_fused(const void* q, const void* k, const void* v, const void* t0, const void* wq,
                                 const void* wk, const void* wv, const int32_t* lens, int U, int C, int L, int d_q,
                                 int d, int w, float gamma, laser_dtype dt, int32_t* seg_cnt, float* z_out, void* work,
                                 size_t work_bytes, void* stream) {
  FusedArgs fa;
  const laser_status s = validate_fused(q, k, v, t0, wq, wk, wv, lens, U, C, L, d_q, d, w, gamma, dt, seg_cnt, z_out,
                                        stream, &fa);
  if (s != LASER_OK) return s;
  if (work != nullptr) {
    if (!aligned16(work)) return LASER_ERR_ALIGN;
    if (work_bytes < fused_need_bytes(fa)) return LASER_ERR_SHAPE;
    fa.work = static_cast<float*>(work);
  }
  return run_fused(fa);
}

laser_status laser_multires_forward(const void* seg, const int32_t* lens, int U, int C, int L, int d, int w, int r,
                                    laser_dtype dt, void* pool_out, void* recent_out, void* stream) {
  MultiresArgs a;
  laser_status s = validate_multires(seg, lens, U, C, L, d, w, r, dt, pool_out, recent_out, stream, &a);
  if (s != LASER_OK) return s;
  return multires_launch(a);
}

laser_status laser_multires_forward_ragged(const void* seg, const int32_t* lens, const int32_t* cand_off, int U,
                                           int C_max, int P, int L, int d, int w, int r, laser_dtype dt, void* pool_out,
                                           void* recent_out, void* stream) {
  MultiresArgs a;
  laser_status s = validate_multires(seg, lens, U, C_max, L, d, w, r, dt, pool_out, recent_out, stream, &a);
  if (s != LASER_OK) return s;
  s = validate_ragged(cand_off, U, C_max, P, L, d, d, w);
  if (s != LASER_OK) return s;
  a.cand_off = cand_off;
  a.P = P;
  return multires_launch(a);
}

laser_status laser_segment_ffn_forward_ragged(const void* seg, const int32_t* lens, const int32_t* cand_off,
                                              const void* w1, const float* b1, const void* w2, const float* b2,
                                              const float* ln_g, const float* ln_b, int U, int C_max, int P, int L,
                                              int d, int d_ff, int w, float eps, laser_dtype dt, void* seg_out,
                                              void* stream) {
  FfnArgs a;
  laser_status s = validate_ffn(seg, lens, w1, b1, w2, b2, ln_g, ln_b, U, C_max, L, d, d_ff, w, eps, dt, seg_out, stream,
                                &a);
  if (s != LASER_OK) return s;
  s = validate_ragged(cand_off, U, C_max, P, L, d, d, w);
  if (s != LASER_OK) return s;
  a.cand_off = cand_off;
  a.P = P;
  return segment_ffn_mfma_supports(a) ? segment_ffn_mfma_launch(a) : segment_ffn_generic_launch(a);
}

laser_status laser_forward_multires(const void* q, const void* k, const void* v, const void* t0, const void* wq,
                                    const void* wk, const void* wv, const int32_t* lens, int U, int C, int L,
                                    int d_q, int d, int w, float gamma, int M, laser_dtype dt, void* seg_out,
                                    int32_t* seg_cnt, float* z_out, int r, void* pool_out, void* recent_out,
                                    void* stream) {
  StaArgs sa;
  GstaArgs ga;
  MultiresArgs ma;
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, seg_out, seg_cnt, stream, &sa);
  if (s != LASER_OK) return s;
  s = validate_gsta(seg_out, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream, &ga);
  if (s != LASER_OK) return s;
  s = validate_multires(seg_out, lens, U, C, L, d, w, r, dt, pool_out, recent_out, stream, &ma);
  if (s != LASER_OK) return s;   // everything validated before the first launch
  sa.reread = true;
  s = run_sta(sa, LASER_STA_AUTO);
  if (s != LASER_OK) return s;
  return run_gsta_views(ga, ma);
}

laser_status laser_gsta_forward_multires(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                         const int32_t* lens, int U, int C, int L, int d, int w, int M, laser_dtype dt,
                                         float* z_out, int r, void* pool_out, void* recent_out, void* stream) {
  GstaArgs ga;
  MultiresArgs ma;
  laser_status s = validate_gsta(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream, &ga);
  if (s != LASER_OK) return s;
  s = validate_multires(seg, lens, U, C, L, d, w, r, dt, pool_out, recent_out, stream, &ma);
  if (s != LASER_OK) return s;
  return run_gsta_views(ga, ma);
}

laser_status laser_segment_ffn_forward_variant(const void* seg, const int32_t* lens, const void* w1, const float* b1,
                                               const void* w2, const float* b2, const float* ln_g, const float* ln_b,
                                               int U, int C, int L, int d, int d_ff, int w, float eps, laser_dtype dt,
                                               void* seg_out, void* stream, laser_ffn_variant variant) {
  FfnArgs a;
  const laser_status s = validate_ffn(seg, lens, w1, b1, w2, b2, ln_g, ln_b, U, C, L, d, d_ff, w, eps, dt, seg_out,
                                      stream, &a);
  if (s != LASER_OK) return s;
  if (variant < LASER_FFN_AUTO || variant > LASER_FFN_MFMA) return LASER_ERR_UNSUPPORTED;
  if (variant == LASER_FFN_AUTO) variant = segment_ffn_mfma_supports(a) ? LASER_FFN_MFMA : LASER_FFN_GENERIC;
  return variant == LASER_FFN_MFMA ? segment_ffn_mfma_launch(a) : segment_ffn_generic_launch(a);
}

laser_status laser_ffn_gsta_forward(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                    const int32_t* lens, const void* w1, const float* b1, const void* w2,
                                    const float* b2, const float* ln_g, const float* ln_b, int U, int C, int L, int d,
                                    int d_ff, int w, int M, float eps, laser_dtype dt, void* seg_out, float* z_out,
                                    void* stream) {
  FfnArgs fa;
  GstaArgs ga;
  laser_status s = validate_ffn(seg, lens, w1, b1, w2, b2, ln_g, ln_b, U, C, L, d, d_ff, w, eps, dt, seg_out, stream,
                                &fa, false);
  if (s != LASER_OK) return s;
  s = validate_gsta(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream, &ga);
  if (s != LASER_OK) return s;
  if (ffn_gsta_fused_supports(fa, ga)) return ffn_gsta_fused_launch(fa, ga);
  // no kernel takes both steps for this shape: the two launches, through the transformed H'
  if (!seg_out) return LASER_ERR_UNSUPPORTED;
  s = segment_ffn_mfma_supports(fa) ? segment_ffn_mfma_launch(fa) : segment_ffn_generic_launch(fa);
  if (s != LASER_OK) return s;
  ga.seg = seg_out;
  return run_gsta(ga, LASER_GSTA_AUTO);
}

laser_status laser_ffn_gsta_forward_multires(const void* seg, const void* t0, const void* wq, const void* wk,
                                             const void* wv, const int32_t* lens, const void* w1, const float* b1,
                                             const void* w2, const float* b2, const float* ln_g, const float* ln_b,
                                             int U, int C, int L, int d, int d_ff, int w, int M, float eps,
                                             laser_dtype dt, void* seg_out, float* z_out, int r, void* pool_out,
                                             void* recent_out, void* stream) {
  FfnArgs fa;
  GstaArgs ga;
  MultiresArgs ma;
  laser_status s = validate_ffn(seg, lens, w1, b1, w2, b2, ln_g, ln_b, U, C, L, d, d_ff, w, eps, dt, seg_out, stream,
                                &fa, false);
  if (s != LASER_OK) return s;
  s = validate_gsta(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z_out, stream, &ga);
  if (s != LASER_OK) return s;
  s = validate_multires(seg, lens, U, C, L, d, w, r, dt, pool_out, recent_out, stream, &ma);
  if (s != LASER_OK) return s;
  if (ffn_gsta_fused_supports(fa, ga)) {
    ga.pool_out = pool_out;
    ga.recent_out = recent_out;
    ga.r = r;
    return ffn_gsta_fused_launch(fa, ga);
  }
  if (!seg_out) return LASER_ERR_UNSUPPORTED;
  s = segment_ffn_mfma_supports(fa) ? segment_ffn_mfma_launch(fa) : segment_ffn_generic_launch(fa);
  if (s != LASER_OK) return s;
  ga.seg = seg_out;
  ma.seg = seg_out;
  return run_gsta_views(ga, ma);
}

laser_status laser_segment_ffn_forward(const void* seg, const int32_t* lens, const void* w1, const float* b1,
                                       const void* w2, const float* b2, const float* ln_g, const float* ln_b, int U,
                                       int C, int L, int d, int d_ff, int w, float eps, laser_dtype dt, void* seg_out,
                                       void* stream) {
  return laser_segment_ffn_forward_variant(seg, lens, w1, b1, w2, b2, ln_g, ln_b, U, C, L, d, d_ff, w, eps, dt, seg_out,
                                           stream, LASER_FFN_AUTO);
}

static laser_status run_project(ProjArgs& a, laser_project_variant variant) {
  if (a.dt != LASER_F32 && a.dt != LASER_BF16) return LASER_ERR_DTYPE;
  if (a.rows < 0 || a.rows > (1LL << 40) || a.d_in <= 0 || a.d_in > 4096) return LASER_ERR_SHAPE;
  for (int o = 0; o < 2; ++o) {
    if (a.n[o] < 0 || a.n[o] > 4096 || (o == 0 && a.n[o] == 0)) return LASER_ERR_SHAPE;
    if (a.n[o] > 0 && (!a.w[o] || !a.y[o])) return LASER_ERR_NULL;
    if (!aligned16(a.w[o]) || !aligned16(a.y[o])) return LASER_ERR_ALIGN;
  }
  if (!a.x) return LASER_ERR_NULL;
  if (!aligned16(a.x)) return LASER_ERR_ALIGN;
  if (variant < LASER_PROJECT_AUTO || variant > LASER_PROJECT_MFMA) return LASER_ERR_UNSUPPORTED;
  if (variant == LASER_PROJECT_AUTO) variant = project_mfma_supports(a) ? LASER_PROJECT_MFMA : LASER_PROJECT_GENERIC;
  return variant == LASER_PROJECT_MFMA ? project_mfma_launch(a) : project_generic_launch(a);
}

laser_status laser_project_q_forward_variant(const void* t, const void* w_q, int U, int C, int d_in, int d_q,
                                             laser_dtype dt, void* q_out, void* stream,
                                             laser_project_variant variant) {
  if (U <= 0 || C <= 0) return LASER_ERR_SHAPE;
  ProjArgs a{t, (long long)U * C, d_in, {w_q, nullptr}, {d_q, 0}, {q_out, nullptr}, dt, static_cast<hipStream_t>(stream),
             {d_q, 0}, {d_q, 0}};
  return run_project(a, variant);
}

laser_status laser_project_q_forward(const void* t, const void* w_q, int U, int C, int d_in, int d_q, laser_dtype dt,
                                     void* q_out, void* stream) {
  return laser_project_q_forward_variant(t, w_q, U, C, d_in, d_q, dt, q_out, stream, LASER_PROJECT_AUTO);
}

laser_status laser_project_kv_forward_variant(const void* h, const void* w_k, const void* w_v, int U, int L, int d_in,
                                              int d_q, int d, laser_dtype dt, void* k_out, void* v_out, void* stream,
                                              laser_project_variant variant) {
  if (U <= 0 || L <= 0 || d <= 0) return LASER_ERR_SHAPE;
  ProjArgs a{h, (long long)U * L, d_in, {w_k, w_v}, {d_q, d}, {k_out, v_out}, dt, static_cast<hipStream_t>(stream),
             {d_q, d}, {d_q, d}};
  return run_project(a, variant);
}

laser_status laser_project_kv_forward(const void* h, const void* w_k, const void* w_v, int U, int L, int d_in, int d_q,
                                      int d, laser_dtype dt, void* k_out, void* v_out, void* stream) {
  return laser_project_kv_forward_variant(h, w_k, w_v, U, L, d_in, d_q, d, dt, k_out, v_out, stream, LASER_PROJECT_AUTO);
}

laser_status laser_fold_query_weights(const void* w_q, const void* w_k, int d_in, int d_q, int heads, laser_dtype dt,
                                      void* a_out, void* stream) {
  if (!w_q || !w_k || !a_out) return LASER_ERR_NULL;
  if (dt != LASER_F32 && dt != LASER_BF16) return LASER_ERR_DTYPE;
  if (d_in <= 0 || d_in > 4096 || d_q <= 0 || d_q > 4096 || heads < 1 || heads > 64 || d_q % heads != 0)
    return LASER_ERR_SHAPE;
  if (!aligned16(w_q) || !aligned16(w_k) || !aligned16(a_out)) return LASER_ERR_ALIGN;
  return fold_weights_launch(w_q, w_k, d_in, d_q, heads, dt, a_out, static_cast<hipStream_t>(stream));
}

static laser_status validate_project_heads(const void* x, const void* w_v, int P, int S, int d_in, int d, int heads,
                                           laser_dtype dt, void* y, void* stream, ProjHeadsArgs* out) {
  if (!x || !w_v || !y) return LASER_ERR_NULL;
  if (dt != LASER_F32 && dt != LASER_BF16) return LASER_ERR_DTYPE;
  if (P <= 0 || S <= 0 || d_in <= 0 || d_in > 4096 || d <= 0 || d > 4096 || heads < 1 || heads > 64 || d % heads != 0)
    return LASER_ERR_SHAPE;
  if ((d_in % 8) != 0 || (d % 8) != 0) return LASER_ERR_SHAPE;
  if (!product_fits(0x7fffffffLL, P, heads, S, d_in) || !product_fits(0x7fffffffLL, P, S, d)) return LASER_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(w_v) || !aligned16(y)) return LASER_ERR_ALIGN;
  *out = ProjHeadsArgs{x, w_v, (long long)P, S, d_in, d, heads, dt, y, static_cast<hipStream_t>(stream)};
  return LASER_OK;
}

static laser_status run_project_heads(const ProjHeadsArgs& a, laser_project_variant variant) {
  if (variant == LASER_PROJECT_AUTO)
    variant = project_heads_mfma_supports(a) ? LASER_PROJECT_MFMA : LASER_PROJECT_GENERIC;
  return variant == LASER_PROJECT_MFMA ? project_heads_mfma_launch(a) : project_heads_generic_launch(a);
}

laser_status laser_project_heads_forward(const void* x, const void* w_v, int P, int S, int d_in, int d, int heads,
                                         laser_dtype dt, void* y, void* stream, laser_project_variant variant) {
  ProjHeadsArgs a;
  laser_status s = validate_project_heads(x, w_v, P, S, d_in, d, heads, dt, y, stream, &a);
  if (s != LASER_OK) return s;
  if (variant < LASER_PROJECT_AUTO || variant > LASER_PROJECT_MFMA) return LASER_ERR_UNSUPPORTED;
  return run_project_heads(a, variant);
}

laser_status laser_sta_folded_forward(const void* t, const void* h, const void* a_fold, const void* w_v,
                                      const int32_t* lens, int U, int C, int L, int d_in, int d, int w, float gamma,
                                      int heads, laser_dtype dt, void* qf_work, void* g_work, void* seg_out,
                                      int32_t* seg_cnt, void* stream) {
  if (!t || !a_fold || !qf_work) return LASER_ERR_NULL;
  if (heads < 1 || heads > 64 || C <= 0 || (long long)C * heads > 0x7fffffffLL) return LASER_ERR_SHAPE;
  if (!aligned16(t) || !aligned16(a_fold)) return LASER_ERR_ALIGN;
  StaArgs sa;
  ProjHeadsArgs pa;
  // STA over the raw history: one pseudo-candidate per (candidate, head), the raw items as keys and values
  laser_status s = validate_sta(qf_work, h, h, lens, U, C * heads, L, d_in, d_in, w, gamma, dt, g_work, seg_cnt, stream,
                                &sa);
  if (s != LASER_OK) return s;
  if ((long long)U * C > 0x7fffffffLL) return LASER_ERR_SHAPE;
  s = validate_project_heads(g_work, w_v, U * C, sa.S, d_in, d, heads, dt, seg_out, stream, &pa);
  if (s != LASER_OK) return s;   // everything validated before the first launch
  const int nq = heads * d_in;
  if (nq > 4096) return LASER_ERR_SHAPE;
  ProjArgs qa{t, (long long)U * C, d_in, {a_fold, nullptr}, {nq, 0}, {qf_work, nullptr}, dt,
              static_cast<hipStream_t>(stream), {nq, 0}, {nq, 0}};
  if (heads == 2 && dt == LASER_BF16) {   // two heads: the halves of A and of the output as the kernel's two outputs
    const size_t half = (size_t)d_in * 2;   // bytes
    qa.w[1] = static_cast<const char*>(a_fold) + half;
    qa.y[1] = static_cast<char*>(qf_work) + half;
    qa.n[0] = qa.n[1] = d_in;
    qa.wpitch[1] = qa.ypitch[1] = nq;
  }
  s = run_project(qa, LASER_PROJECT_AUTO);
  if (s != LASER_OK) return s;
  sa.reread = true;
  s = run_sta(sa, LASER_STA_AUTO);
  if (s != LASER_OK) return s;
  return run_project_heads(pa, LASER_PROJECT_AUTO);
}

size_t laser_sta_backward_work_bytes(int U, int C, int L, int d_q, int w) {
  if (check_dims(U, C, L, d_q, 8, w) != LASER_OK) return 0;   // (8: any valid value width; it does not enter the size)
  return sta_backward_work_bytes(U, C, L, d_q, w);
}

// Everything about a backward call of STA except its scratch: checks, then the launcher's arguments (work unset)
static laser_status sta_backward_validate(const void* q, const void* k, const void* v, const int32_t* lens,
                                          const void* dseg, int U, int C, int L, int d_q, int d, int w, float gamma,
                                          laser_dtype dt, float* dq_out, void* dk_out, void* dv_out, bool grads_bf16,
                                          void* stream, StaBwdArgs* out) {
  if (!dseg || !dq_out || !dk_out || !dv_out) return LASER_ERR_NULL;
  StaArgs fa;   // the forward pass's checks of the shared arguments (dseg stands in for seg_out: same shape and type)
  laser_status s = validate_sta(q, k, v, lens, U, C, L, d_q, d, w, gamma, dt, const_cast<void*>(dseg), nullptr, stream,
                                &fa);
  if (s != LASER_OK) return s;
  if (!aligned16(dq_out) || !aligned16(dk_out) || !aligned16(dv_out)) return LASER_ERR_ALIGN;
  *out = StaBwdArgs{q, k, v, dseg, lens, U, C, L, d_q, d, w, fa.S, gamma, dt, dq_out, dk_out, dv_out, nullptr,
                    static_cast<hipStream_t>(stream)};
  out->grads_bf16 = grads_bf16;
  return LASER_OK;
}

static laser_status sta_backward_any(const void* q, const void* k, const void* v, const int32_t* lens, const void* dseg,
                                     int U, int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt,
                                     float* dq_out, void* dk_out, void* dv_out, bool grads_bf16, void* work,
                                     size_t work_bytes, void* stream) {
  if (!work) return LASER_ERR_NULL;
  StaBwdArgs a;
  const laser_status s = sta_backward_validate(q, k, v, lens, dseg, U, C, L, d_q, d, w, gamma, dt, dq_out, dk_out,
                                               dv_out, grads_bf16, stream, &a);
  if (s != LASER_OK) return s;
  if (!aligned16(work)) return LASER_ERR_ALIGN;
  if (work_bytes < sta_backward_work_bytes(U, C, L, d_q, w)) return LASER_ERR_SHAPE;
  a.work = static_cast<float*>(work);
  return sta_backward_launch(a);
}

laser_status laser_sta_backward(const void* q, const void* k, const void* v, const int32_t* lens, const void* dseg, int U,
                                int C, int L, int d_q, int d, int w, float gamma, laser_dtype dt, float* dq_out,
                                float* dk_out, float* dv_out, void* work, size_t work_bytes, void* stream) {
  return sta_backward_any(q, k, v, lens, dseg, U, C, L, d_q, d, w, gamma, dt, dq_out, dk_out, dv_out, false, work,
                          work_bytes, stream);
}

laser_status laser_sta_backward_bf16(const void* q, const void* k, const void* v, const int32_t* lens, const void* dseg,
                                     int U, int C, int L, int d_q, int d, int w, float gamma, float* dq_out,
                                     void* dk_out, void* dv_out, void* work, size_t work_bytes, void* stream) {
  return sta_backward_any(q, k, v, lens, dseg, U, C, L, d_q, d, w, gamma, LASER_BF16, dq_out, dk_out, dv_out, true, work,
                          work_bytes, stream);
}

// Scratch of laser_sta_backward_static: device memory that belongs to this code object, so no call ever allocates.
// In host code the array's name is only a handle for the symbol lookup below, not a device address: everything that
// needs the memory (kernel arguments) takes the looked-up pointer. Every GPU holds its own copy at its own address.
static __device__ __align__(256) unsigned char scratch[LASER_STATIC_SCRATCH_BYTES];

// Address of `scratch` on the current device: looked up on the first call per device, kept until the process ends.
static laser_status static_scratch(void** out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void* ptr[MAX_DEVICES] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return LASER_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return LASER_ERR_LAUNCH;
    }
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return LASER_OK;
}

laser_status laser_sta_backward_static(const void* q, const void* k, const void* v, const int32_t* lens,
                                       const void* dseg, int U, int C, int L, int d_q, int d, int w, float gamma,
                                       laser_dtype dt, float* dq_out, float* dk_out, float* dv_out, void* stream) {
  StaBwdArgs a;
  laser_status s = sta_backward_validate(q, k, v, lens, dseg, U, C, L, d_q, d, w, gamma, dt, dq_out, dk_out, dv_out,
                                         false, stream, &a);
  if (s != LASER_OK) return s;
  // the sizes are known to be sane here; what the kernels need must fit the array
  if (sta_backward_work_bytes(U, C, L, d_q, w) > (size_t)LASER_STATIC_SCRATCH_BYTES) return LASER_ERR_SHAPE;
  if (!sta_backward_supports(a)) return LASER_ERR_UNSUPPORTED;   // before the device is touched
  void* work = nullptr;
  s = static_scratch(&work);
  if (s != LASER_OK) return s;
  a.work = static_cast<float*>(work);
  return sta_backward_launch(a);
}

size_t laser_gsta_backward_work_bytes(int U, int C, int d, int M) {
  if (U <= 0 || C <= 0 || d <= 0 || M <= 0 || d > 1024 || M > 64 || !product_fits(0x7fffffffLL, U, C, d)) return 0;
  return gsta_backward_work_bytes(U, C, d, M);
}

laser_status laser_gsta_backward(const void* seg, const void* t0, const void* wq, const void* wk, const void* wv,
                                 const int32_t* lens, const float* dz, int U, int C, int L, int d, int w, int M,
                                 laser_dtype dt, void* dseg_out, float* dt0_out, float* dwq_out, float* dwk_out,
                                 float* dwv_out, void* work, size_t work_bytes, void* stream) {
  if (!dz || !dseg_out || !dt0_out || !dwq_out || !dwk_out || !dwv_out || !work) return LASER_ERR_NULL;
  GstaArgs fa;   // the forward pass's checks of the shared arguments (dt0_out stands in for z_out: same shape and type)
  laser_status s = validate_gsta(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, dt0_out, stream, &fa);
  if (s != LASER_OK) return s;
  for (const void* p : {(const void*)dz, (const void*)dseg_out, (const void*)dwq_out, (const void*)dwk_out,
                        (const void*)dwv_out, (const void*)work})
    if (!aligned16(p)) return LASER_ERR_ALIGN;
  if (work_bytes < gsta_backward_work_bytes(U, C, d, M)) return LASER_ERR_SHAPE;
  const GstaBwdArgs a{seg, t0, wq, wk, wv, lens, dz, U, C, L, d, w, fa.S, M, dt, dseg_out, dt0_out, dwq_out, dwk_out,
                      dwv_out, static_cast<float*>(work), static_cast<hipStream_t>(stream)};
  return gsta_backward_launch(a);
}

const char* laser_sta_kernel_name(int C, int d_q, int d, int w, laser_dtype dt) {
  StaArgs a{};
  a.U = 1; a.C = C; a.L = w > 0 ? w : 1; a.d_q = d_q; a.d = d; a.w = w; a.S = 1; a.gamma = 1.0f; a.dt = dt;
  if (C <= 0 || d_q <= 0 || d <= 0 || w <= 0 || (dt != LASER_F32 && dt != LASER_BF16)) return "invalid";
  switch (pick_sta(a)) {
    case LASER_STA_MFMA: return "sta_mfma_bf16";
    case LASER_STA_STREAM: return "sta_stream_bf16";
    default: return "sta_generic";
  }
}

const char* laser_gsta_kernel_name(int C, int S, int d, laser_dtype dt) {
  return laser_gsta_kernel_name_layers(C, S, d, 1, dt);
}

const char* laser_gsta_kernel_name_layers(int C, int S, int d, int M, laser_dtype dt) {
  GstaArgs a{};
  a.U = 1; a.C = C; a.L = S; a.w = 1; a.S = S; a.d = d; a.M = M; a.dt = dt;
  if (C <= 0 || S <= 0 || d <= 0 || M <= 0 || (dt != LASER_F32 && dt != LASER_BF16)) return "invalid";
  switch (pick_gsta(a)) {
    case LASER_GSTA_SPLIT: return "gsta_split_bf16";
    case LASER_GSTA_ONE: return "gsta_one_bf16";
    case LASER_GSTA_TILED: return "gsta_tiled_bf16";
    default: return "gsta_generic";
  }
}

const char* laser_status_string(laser_status s) {
  switch (s) {
    case LASER_OK: return "ok";
    case LASER_ERR_NULL: return "required pointer is NULL";
    case LASER_ERR_SHAPE: return "invalid or inconsistent size";
    case LASER_ERR_DTYPE: return "unknown dtype";
    case LASER_ERR_UNSUPPORTED: return "shape not supported by the requested kernel";
    case LASER_ERR_LAUNCH: return "HIP launch failed";
    case LASER_ERR_ALIGN: return "pointer not sufficiently aligned";
    default: break;
  }
  return "unknown status";
}

int laser_version(void) { return 100; }

}  // extern "C"
