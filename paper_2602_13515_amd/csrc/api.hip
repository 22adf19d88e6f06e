// C ABI of spa2: argument validation, workspace layout, kernel sequencing.
// No device memory is allocated here.  Nothing is kept between calls except the per-device address of the
// fixed scratch array that spa2_bwd_static uses (looked up once per device).
#include <math.h>

#include <mutex>

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
  // the kernels address a tile as a 64-bit base plus a 32-bit byte offset of up to 128 token rows
  if (s->sn > SPA2_MAX_TOKEN_STRIDE) return SPA2_ERR_SHAPE;
  if ((int64_t)s->B * s->H > (int64_t)1 << 24) return SPA2_ERR_SHAPE;
  // one-dimensional grids of up to B*H*(T_m + T_n + 16) workgroups, 32-bit workgroup arithmetic in the kernels
  const int64_t tm = ((int64_t)s->N + SPA2_BQ - 1) / SPA2_BQ, tn = ((int64_t)s->N + SPA2_BKV - 1) / SPA2_BKV;
  if ((int64_t)s->B * s->H * (tm + tn + 16) > (int64_t)0x7fffffff) return SPA2_ERR_SHAPE;
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

// Backward workspace: D (fp32, one value per token row), then the split plans and partial-result pools of the dQ
// and the dK/dV kernel.  Only D is mandatory: with less than the full size the kernels walk every list whole.
struct BwdWs { size_t d_bytes, dq_off, dq_bytes, dkdv_off, dkdv_bytes, total; };
BwdWs bwd_ws(const Dims& m) {
  BwdWs w;
  w.d_bytes = round256((size_t)m.B * m.H * m.N * sizeof(float));
  w.dq_off = w.d_bytes;
  w.dq_bytes = round256(split_ws_bytes((int64_t)m.B * m.H * m.Tm, dq_slot_bytes(m)));
  w.dkdv_off = w.dq_off + w.dq_bytes;
  w.dkdv_bytes = round256(split_ws_bytes((int64_t)m.B * m.H * m.Tn, dkdv_slot_bytes(m)));
  w.total = w.dkdv_off + w.dkdv_bytes;
  return w;
}
size_t bwd_ws_min_bytes(const Dims& m) { return bwd_ws(m).d_bytes; }

// the part of a workspace section that the caller's buffer really covers
SplitPlan section_plan(void* ws, size_t ws_bytes, size_t off, size_t bytes, int64_t units, size_t slot_bytes) {
  if (!ws || ws_bytes <= off) return split_layout(nullptr, 0, units, slot_bytes);
  const size_t have = ws_bytes - off < bytes ? ws_bytes - off : bytes;
  return split_layout((char*)ws + off, have, units, slot_bytes);
}

}  // namespace

extern "C" {

int spa2_version(void) { return 100; }

const char* spa2_strerror(int code) {
  switch (code) {
    case SPA2_OK: return "ok";
    case SPA2_ERR_NULL: return "a required pointer is NULL";
    case SPA2_ERR_SHAPE: return "invalid shape or strides";
    case SPA2_ERR_UNSUPPORTED: return "unsupported head dimension, block size or element type (d must be 64 or 128, blocks 128x64)";
    case SPA2_ERR_ALIGN: return "pointer not 16-byte aligned or stride not a multiple of 8 elements";
    case SPA2_ERR_RANGE: return "parameter out of range (topk_blocks in [0,T_n], top_p in [0,1], not both zero, scale > 0, weight > 0)";
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
  return bwd_ws(make_dims(*shape)).total;
}

size_t spa2_bwd_workspace_min_bytes(const spa2_shape* shape) {
  if (check_shape(shape) != SPA2_OK) return 0;
  return bwd_ws_min_bytes(make_dims(*shape));
}

size_t spa2_fwd_workspace_bytes(const spa2_shape* shape) {
  if (check_shape(shape) != SPA2_OK) return 0;
  const Dims m = make_dims(*shape);
  return round256(split_ws_bytes((int64_t)m.B * m.H * m.Tm, fwd_slot_bytes(m)));
}

int spa2_mask_pool(const void* q, const void* k, const spa2_shape* shape, void* workspace,
                   size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k) return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k)) return SPA2_ERR_ALIGN;
  const Dims m = make_dims(*shape);
  const MaskWs w = mask_ws(m);
  if (!workspace || workspace_bytes < w.total) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  float* qbar = (float*)((char*)workspace + w.qbar);
  float* kbar = (float*)((char*)workspace + w.kbar);
  return launch_pool(q, k, m, qbar, kbar, (hipStream_t)stream) == hipSuccess ? SPA2_OK : SPA2_ERR_LAUNCH;
}

int spa2_mask_select(const spa2_shape* shape, int32_t topk_blocks, float top_p, float scale, spa2_pattern* out,
                     float* pbar_out, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!out || !out->mask || !out->row_cnt || !out->row_idx) return SPA2_ERR_NULL;
  const Dims m = make_dims(*shape);
  if (m.Tn > SPA2_MAX_TN) return SPA2_ERR_SHAPE;
  if (topk_blocks < 0 || topk_blocks > m.Tn) return SPA2_ERR_RANGE;
  if (!(top_p >= 0.f) || !(top_p <= 1.f)) return SPA2_ERR_RANGE;
  if (topk_blocks == 0 && top_p == 0.f) return SPA2_ERR_RANGE;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const MaskWs w = mask_ws(m);
  if (!workspace || workspace_bytes < w.total) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  const float* qbar = (const float*)((char*)workspace + w.qbar);
  const float* kbar = (const float*)((char*)workspace + w.kbar);
  return launch_select(qbar, kbar, m, topk_blocks, top_p, scale, out->mask, out->row_cnt, out->row_idx, pbar_out,
                       (hipStream_t)stream) == hipSuccess ? SPA2_OK : SPA2_ERR_LAUNCH;
}

int spa2_mask_columns(const spa2_shape* shape, spa2_pattern* out, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!out || !out->mask || !out->col_cnt || !out->col_idx) return SPA2_ERR_NULL;
  const Dims m = make_dims(*shape);
  if (m.Tn > SPA2_MAX_TN) return SPA2_ERR_SHAPE;     // the column sort holds one head's T_n keys in LDS
  return launch_columns(out->mask, m, out->col_cnt, out->col_idx, out->col_order, (hipStream_t)stream) == hipSuccess
             ? SPA2_OK : SPA2_ERR_LAUNCH;
}

int spa2_mask(const void* q, const void* k, const spa2_shape* shape, int32_t topk_blocks, float top_p,
              float scale, spa2_pattern* out, float* pbar_out, void* workspace, size_t workspace_bytes,
              void* stream) {
  // validate everything first, so that a rejected call has launched nothing
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
  if (!workspace || workspace_bytes < mask_ws(m).total) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  rc = spa2_mask_pool(q, k, shape, workspace, workspace_bytes, stream);
  if (rc != SPA2_OK) return rc;
  rc = spa2_mask_select(shape, topk_blocks, top_p, scale, out, pbar_out, workspace, workspace_bytes, stream);
  if (rc != SPA2_OK) return rc;
  if (out->col_cnt) rc = spa2_mask_columns(shape, out, stream);
  return rc;
}

int spa2_pattern_full(const spa2_shape* shape, spa2_pattern* out, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!out || !out->mask || !out->row_cnt || !out->row_idx) return SPA2_ERR_NULL;
  if ((out->col_cnt == nullptr) != (out->col_idx == nullptr)) return SPA2_ERR_NULL;
  const Dims m = make_dims(*shape);
  if (launch_pattern_full(m, out->mask, out->row_cnt, out->row_idx, out->col_cnt, out->col_idx,
                          out->col_cnt ? out->col_order : nullptr, (hipStream_t)stream) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  return SPA2_OK;
}

int spa2_fwd(const void* q, const void* k, const void* v, const spa2_shape* shape, const spa2_pattern* pattern,
             float scale, void* o, void* o_res, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !v || !o || !lse || !pattern || !pattern->row_cnt || !pattern->row_idx) return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(o_res)) return SPA2_ERR_ALIGN;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  if (workspace && !aligned16(workspace)) return SPA2_ERR_ALIGN;
  const Dims m = make_dims(*shape);
  const SplitPlan plan = section_plan(workspace, workspace_bytes, 0, spa2_fwd_workspace_bytes(shape),
                                      (int64_t)m.B * m.H * m.Tm, fwd_slot_bytes(m));
  if (launch_fwd(q, k, v, m, pattern->row_cnt, pattern->row_idx, pattern->row_order, scale, o, o_res, lse, plan,
                 (hipStream_t)stream) != hipSuccess)
    return SPA2_ERR_LAUNCH;
  return SPA2_OK;
}

int spa2_bwd_delta(const void* o, const void* o_res, const void* d_o, const spa2_shape* shape, void* workspace,
                   size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!o || !d_o) return SPA2_ERR_NULL;
  if (!aligned16(o) || !aligned16(d_o) || !aligned16(o_res)) return SPA2_ERR_ALIGN;
  const Dims m = make_dims(*shape);
  if (!workspace || workspace_bytes < bwd_ws_min_bytes(m)) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  return launch_bwd_delta(o, o_res, d_o, m, (float*)workspace, (hipStream_t)stream) == hipSuccess ? SPA2_OK
                                                                                           : SPA2_ERR_LAUNCH;
}

int spa2_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                  const spa2_shape* shape, const spa2_pattern* pattern, float scale, void* dk, void* dv,
                  void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !v || !d_o || !lse || !dk || !dv || !pattern || !pattern->col_cnt || !pattern->col_idx)
    return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dk) || !aligned16(dv))
    return SPA2_ERR_ALIGN;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const Dims m = make_dims(*shape);
  if (!workspace || workspace_bytes < bwd_ws_min_bytes(m)) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  const BwdWs w = bwd_ws(m);
  const SplitPlan plan = section_plan(workspace, workspace_bytes, w.dkdv_off, w.dkdv_bytes, (int64_t)m.B * m.H * m.Tn,
                                      dkdv_slot_bytes(m));
  return launch_bwd_dkdv(q, k, v, d_o, lse, (const float*)workspace, m, pattern->col_cnt, pattern->col_idx,
                         pattern->col_order, scale, dk, dv, plan, (hipStream_t)stream) == hipSuccess ? SPA2_OK : SPA2_ERR_LAUNCH;
}

int spa2_bwd_dq(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                const spa2_shape* shape, const spa2_pattern* pattern, float scale, void* dq,
                void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !v || !d_o || !lse || !dq || !pattern || !pattern->row_cnt || !pattern->row_idx)
    return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq)) return SPA2_ERR_ALIGN;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const Dims m = make_dims(*shape);
  if (!workspace || workspace_bytes < bwd_ws_min_bytes(m)) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  const BwdWs w = bwd_ws(m);
  const SplitPlan plan = section_plan(workspace, workspace_bytes, w.dq_off, w.dq_bytes, (int64_t)m.B * m.H * m.Tm,
                                      dq_slot_bytes(m));
  return launch_bwd_dq(q, k, v, d_o, lse, (const float*)workspace, m, pattern->row_cnt, pattern->row_idx,
                       pattern->row_order, scale, dq, plan, (hipStream_t)stream) == hipSuccess ? SPA2_OK : SPA2_ERR_LAUNCH;
}

int spa2_bwd(const void* q, const void* k, const void* v, const void* o, const void* o_res, const void* d_o,
             const float* lse, const spa2_shape* shape, const spa2_pattern* pattern, float scale, void* dq,
             void* dk, void* dv, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !pattern) return SPA2_ERR_NULL;
  if (!pattern->row_cnt || !pattern->row_idx || !pattern->col_cnt || !pattern->col_idx) return SPA2_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv) || !aligned16(o_res))
    return SPA2_ERR_ALIGN;
  if (!(scale > 0.f) || !isfinite(scale)) return SPA2_ERR_RANGE;
  const Dims m = make_dims(*shape);
  if (!workspace || workspace_bytes < bwd_ws_min_bytes(m)) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  rc = spa2_bwd_delta(o, o_res, d_o, shape, workspace, workspace_bytes, stream);
  if (rc != SPA2_OK) return rc;
  rc = spa2_bwd_dkdv(q, k, v, d_o, lse, shape, pattern, scale, dk, dv, workspace, workspace_bytes, stream);
  if (rc != SPA2_OK) return rc;
  return spa2_bwd_dq(q, k, v, d_o, lse, shape, pattern, scale, dq, workspace, workspace_bytes, stream);
}


size_t spa2_error_workspace_bytes(const spa2_shape* shape) {
  if (check_shape(shape) != SPA2_OK) return 0;
  return round256(error_ws_bytes(make_dims(*shape)));
}

int spa2_error_terms(const void* o_sparse, const void* o_dense, const float* lse_sparse, const float* lse_dense,
                     const spa2_shape* shape, double* out, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if (!o_sparse || !o_dense || !lse_sparse || !lse_dense || !out) return SPA2_ERR_NULL;
  if (!aligned16(o_sparse) || !aligned16(o_dense) || !aligned16(workspace)) return SPA2_ERR_ALIGN;
  const Dims m = make_dims(*shape);
  if (!workspace || workspace_bytes < error_ws_bytes(m)) return SPA2_ERR_WORKSPACE;
  return launch_error_terms(o_sparse, o_dense, lse_sparse, lse_dense, m, out, workspace, (hipStream_t)stream) == hipSuccess
             ? SPA2_OK : SPA2_ERR_LAUNCH;
}

size_t spa2_vd_loss_workspace_bytes(void) { return round256(vd_ws_bytes()); }

static int check_vd(const void* u_sparse, const void* u_full, int64_t n, int32_t dtype, double weight) {
  if (!u_sparse || !u_full) return SPA2_ERR_NULL;
  if (n <= 0) return SPA2_ERR_SHAPE;
  if (dtype != SPA2_DTYPE_BF16 && dtype != SPA2_DTYPE_F32) return SPA2_ERR_UNSUPPORTED;
  if (!aligned16(u_sparse) || !aligned16(u_full)) return SPA2_ERR_ALIGN;
  if (!(weight > 0.0) || !isfinite(weight)) return SPA2_ERR_RANGE;
  return SPA2_OK;
}

int spa2_vd_loss(const void* u_sparse, const void* u_full, int64_t n, int32_t dtype, double weight, double* loss,
                 void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_vd(u_sparse, u_full, n, dtype, weight);
  if (rc != SPA2_OK) return rc;
  if (!loss) return SPA2_ERR_NULL;
  if (!workspace || workspace_bytes < vd_ws_bytes()) return SPA2_ERR_WORKSPACE;
  if (!aligned16(workspace)) return SPA2_ERR_ALIGN;
  return launch_vd_loss(u_sparse, u_full, n, dtype == SPA2_DTYPE_BF16, weight, loss, workspace, (hipStream_t)stream) ==
                 hipSuccess ? SPA2_OK : SPA2_ERR_LAUNCH;
}

int spa2_vd_loss_grad(const void* u_sparse, const void* u_full, int64_t n, int32_t dtype, double weight,
                      const double* upstream, void* grad, void* stream) {
  int rc = check_vd(u_sparse, u_full, n, dtype, weight);
  if (rc != SPA2_OK) return rc;
  if (!grad) return SPA2_ERR_NULL;
  if (!aligned16(grad)) return SPA2_ERR_ALIGN;
  return launch_vd_grad(u_sparse, u_full, n, dtype == SPA2_DTYPE_BF16, weight, upstream, grad, (hipStream_t)stream) ==
                 hipSuccess ? SPA2_OK : SPA2_ERR_LAUNCH;
}
}  // extern "C"

// ---------------------------------------------------------------- spa2_bwd without a workspace argument
// D = rowsum(dO * O) (fp32, one value per token row) lives in a fixed array in device memory instead of a
// caller's workspace.  The array's name is only a host-side handle: its device address differs per GPU and is
// looked up once per device with that device current; kernels and every other use take that address.
namespace {

__device__ __align__(256) float scratch[SPA2_STATIC_MAX_ROWS];

constexpr int MAX_DEVICES = 64;
float* scratch_ptr[MAX_DEVICES];     // per device, nullptr until looked up
std::mutex scratch_mutex;

int scratch_for_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return SPA2_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SPA2_ERR_LAUNCH;
    scratch_ptr[dev] = (float*)p;
  }
  *out = scratch_ptr[dev];
  return SPA2_OK;
}

}  // namespace

extern "C" int spa2_bwd_static(const void* q, const void* k, const void* v, const void* o, const void* o_res,
                               const void* d_o, const float* lse, const spa2_shape* shape,
                               const spa2_pattern* pattern, float scale, void* dq, void* dk, void* dv,
                               void* stream) {
  int rc = check_shape(shape);
  if (rc != SPA2_OK) return rc;
  if ((int64_t)shape->B * shape->H * shape->N > (int64_t)SPA2_STATIC_MAX_ROWS) return SPA2_ERR_WORKSPACE;
  float* ws = nullptr;
  rc = scratch_for_current_device(&ws);
  if (rc != SPA2_OK) return rc;
  // every row of D that the kernels read is written by the delta pass of this same call: nothing to clear
  // exactly the mandatory part of the workspace: long rows and columns are not split on this path
  return spa2_bwd(q, k, v, o, o_res, d_o, lse, shape, pattern, scale, dq, dk, dv, ws,
                  spa2_bwd_workspace_min_bytes(shape), stream);
}
