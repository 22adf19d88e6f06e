// C ABI of spa2: argument validation, workspace layout, kernel sequencing.
// No device memory is allocated here and nothing is kept between calls.
#include <math.h>

#include "spa2_internal.h"

using namespace spa2;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

int check_shape(const spa2_shape* s) {
  if (!s) return SPA2_ERR_NULL;
  if (s->B <= 0 || s->H <= 0 || s->N <= 0 || s->d <= 0) return SPA2_ERR_SHAPE;
  if (s->bq != SPA2_BQ || s->bkv != SPA2_BKV) return SPA2_ERR_UNSUPPORTED;
  if (s->d != 64 && s->d != 128) return SPA2_ERR_UNSUPPORTED;
  if (s->sb <= 0 || s->sh <= 0 || s->sn < s->d) return SPA2_ERR_SHAPE;
  if ((s->sb % 8) || (s->sh % 8) || (s->sn % 8)) return SPA2_ERR_ALIGN;
  if ((int64_t)s->B * s->H > (int64_t)1 << 24) return SPA2_ERR_SHAPE;
  return SPA2_OK;
}

struct MaskWs { size_t qbar, kbar, total; };
MaskWs mask_ws(const Dims& m) {
  MaskWs w;
  const size_t bh = (size_t)m.B * m.H;
  w.qbar = 0;
  w.kbar = round256(bh * m.Tm * m.d * sizeof(float));
  w.total = w.kbar + round256(bh * m.Tn * m.d * sizeof(float));
  return w;
}

}  // namespace

extern "C" {

int spa2_version(void) { return 100; }

const char* spa2_strerror(int code) {
  switch (code) {
    case SPA2_OK: return "ok";
    case SPA2_ERR_NULL: return "a required pointer is NULL";
    case SPA2_ERR_SHAPE: return "invalid shape or strides";
    case SPA2_ERR_UNSUPPORTED: return "unsupported head dimension or block size (d must be 64 or 128, blocks 128x64)";
    case SPA2_ERR_ALIGN: return "pointer not 16-byte aligned or stride not a multiple of 8 elements";
    case SPA2_ERR_RANGE: return "parameter out of range (topk_blocks in [0,T_n], top_p in [0,1], not both zero, scale > 0)";
    case SPA2_ERR_WORKSPACE: return "workspace missing or too small";
    case SPA2_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown spa2 error code";
  }
}

int32_t spa2_topk_blocks(double k_frac, int32_t Tn) {
  if (Tn <= 0 || !(k_frac > 0.0)) return 0;
  double c = ceil(k_frac * (double)Tn - 1e-9);
  if (c < 1.0) c = 1.0;
  if (c > (double)Tn) c = (double)Tn;
  return (int32_t)c;
}

size_t spa2_mask_workspace_bytes(const spa2_shape* shape) {
  if (check_shape(shape) != SPA2_OK) return 0;
  return mask_ws(make_dims(*shape)).total;
}

size_t spa2_bwd_workspace_bytes(const spa2_shape* shape) {
  if (check_shape(shape) != SPA2_OK) return 0;
  const Dims m = make_dims(*shape);
  return round256((size_t)m.B * m.H * m.N * sizeof(float));
}

int spa2_mask(const void* q, const void* k, const spa2_shape* shape, int32_t topk_blocks, float top_p,
              float scale, spa2_pattern* out, float* pbar_out, void* workspace, size_t workspace_bytes,
              void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !out || !out->mask || !out->row_cnt || !out->row_idx) return SPA2_ERR_NULL;
  if ((out->col_cnt == nullptr) != (out->col_idx == nullptr)) return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k)) return SPA2_ERR_ALIGN;
  const Dims m = make_dims(*shape);
  if (m.Tn > SPA2_MAX_TN) return SPA2_ERR_SHAPE;
  if (topk_blocks < 0 || topk_blocks > m.Tn) return SPA2_ERR_RANGE;
  if (!(top_p >= 0.f) || !(top_p <= 1.f)) return SPA2_ERR_RANGE;
  if (topk_blocks == 0 && top_p == 0.f) return SPA2_ERR_RANGE;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const MaskWs w = mask_ws(m);
  if (!workspace || workspace_bytes < w.total) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  float* qbar = (float*)((char*)workspace + w.qbar);
  float* kbar = (float*)((char*)workspace + w.kbar);
  if (launch_pool(q, k, m, qbar, kbar, st) != hipSuccess) return SPA2_ERR_LAUNCH;
  if (launch_select(qbar, kbar, m, topk_blocks, top_p, scale, out->mask, out->row_cnt, out->row_idx, pbar_out,
                    st) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  if (out->col_cnt &&
      launch_columns(out->mask, m, out->col_cnt, out->col_idx, st) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  return SPA2_OK;
}

int spa2_pattern_full(const spa2_shape* shape, spa2_pattern* out, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!out || !out->mask || !out->row_cnt || !out->row_idx) return SPA2_ERR_NULL;
  if ((out->col_cnt == nullptr) != (out->col_idx == nullptr)) return SPA2_ERR_NULL;
  const Dims m = make_dims(*shape);
  if (launch_pattern_full(m, out->mask, out->row_cnt, out->row_idx, out->col_cnt, out->col_idx,
                          (hipStream_t)stream) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  return SPA2_OK;
}

int spa2_fwd(const void* q, const void* k, const void* v, const spa2_shape* shape, const spa2_pattern* pattern,
             float scale, void* o, float* lse, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !v || !o || !lse || !pattern || !pattern->row_cnt || !pattern->row_idx) return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return SPA2_ERR_ALIGN;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const Dims m = make_dims(*shape);
  if (launch_fwd(q, k, v, m, pattern->row_cnt, pattern->row_idx, scale, o, lse, (hipStream_t)stream) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  return SPA2_OK;
}

int spa2_bwd(const void* q, const void* k, const void* v, const void* o, const void* d_o, const float* lse,
             const spa2_shape* shape, const spa2_pattern* pattern, float scale, void* dq, void* dk, void* dv,
             void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !pattern) return SPA2_ERR_NULL;
  if (!pattern->row_cnt || !pattern->row_idx || !pattern->col_cnt || !pattern->col_idx) return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv))
    return SPA2_ERR_ALIGN;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const Dims m = make_dims(*shape);
  const size_t need = round256((size_t)m.B * m.H * m.N * sizeof(float));
  if (!workspace || workspace_bytes < need) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  float* delta = (float*)workspace;
  if (launch_bwd_delta(o, d_o, m, delta, st) != hipSuccess) return SPA2_ERR_LAUNCH;
  if (launch_bwd_dkdv(q, k, v, d_o, lse, delta, m, pattern->col_cnt, pattern->col_idx, scale, dk, dv, st) !=
      hipSuccess)
    return SPA2_ERR_LAUNCH;
  if (launch_bwd_dq(q, k, v, d_o, lse, delta, m, pattern->row_cnt, pattern->row_idx, scale, dq, st) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  return SPA2_OK;
}

}  // extern "C"
