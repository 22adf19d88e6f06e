// Host-side declarations shared by the spa2 translation units (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "spa2.h"

namespace spa2 {

struct Dims {
  int B, H, N, d, Tm, Tn;
  int64_t sb, sh, sn;
};

inline Dims make_dims(const spa2_shape& s) {
  Dims m;
  m.B = s.B; m.H = s.H; m.N = s.N; m.d = s.d;
  m.Tm = (s.N + SPA2_BQ - 1) / SPA2_BQ;
  m.Tn = (s.N + SPA2_BKV - 1) / SPA2_BKV;
  m.sb = s.sb; m.sh = s.sh; m.sn = s.sn;
  return m;
}

// Splitting of long rows / columns over several workgroups (split.hip).  All pointers lie in the caller's
// workspace; pool_slots == 0 means "no splitting" and every other member is then null.
constexpr int SPLIT_POOL_MAX = 2048;         // partial-result slots of one launch at most
constexpr int SPLIT_MIN_PART = 16;           // a part has at least this many list entries
struct SplitPlan {
  const int32_t* header;       // [0] number of extra parts, [1] S = list entries per part, [2] number of split units
  const int32_t* unit_slot;    // [units] first pool slot of a split unit (its part p uses slot + p), -1 if not split
  const int32_t* part_table;   // [pool_slots][2] (unit, part >= 1) of extra part g
  const int32_t* merge_table;  // [pool_slots] unit of split unit m
  float* pool;                 // [pool_slots][slot_floats] fp32 partial results
  int pool_slots;
  int slot_floats;
};
size_t split_ws_bytes(int64_t units, size_t slot_bytes);
SplitPlan split_layout(void* ws, size_t ws_bytes, int64_t units, size_t slot_bytes);
hipError_t launch_split_plan(const int32_t* cnt, int64_t units, int cnt_max, int min_part, const SplitPlan& p,
                             hipStream_t stream);

// Each launcher enqueues its kernels on `stream` and returns hipGetLastError().
hipError_t launch_pool(const void* q, const void* k, const Dims& m, float* qbar, float* kbar, hipStream_t stream);
hipError_t launch_select(const float* qbar, const float* kbar, const Dims& m, int topk_blocks, float top_p,
                         float scale, uint8_t* mask, int32_t* row_cnt, int32_t* row_idx, float* pbar_out,
                         hipStream_t stream);
hipError_t launch_columns(const uint8_t* mask, const Dims& m, int32_t* col_cnt, int32_t* col_idx,
                          int32_t* col_order, hipStream_t stream);
hipError_t launch_pattern_full(const Dims& m, uint8_t* mask, int32_t* row_cnt, int32_t* row_idx,
                               int32_t* col_cnt, int32_t* col_idx, int32_t* col_order, hipStream_t stream);
size_t fwd_slot_bytes(const Dims& m);
hipError_t launch_fwd(const void* q, const void* k, const void* v, const Dims& m, const int32_t* row_cnt,
                      const int32_t* row_idx, const int32_t* row_order, float scale, void* o, void* o_res,
                      float* lse, const SplitPlan& plan, hipStream_t stream);
hipError_t launch_bwd_delta(const void* o, const void* o_res, const void* d_o, const Dims& m, float* delta,
                            hipStream_t stream);
size_t dq_slot_bytes(const Dims& m);
size_t dkdv_slot_bytes(const Dims& m);
hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                         const float* delta, const Dims& m, const int32_t* row_cnt, const int32_t* row_idx,
                         const int32_t* row_order, float scale, void* dq, const SplitPlan& plan, hipStream_t stream);
hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                           const float* delta, const Dims& m, const int32_t* col_cnt, const int32_t* col_idx,
                           const int32_t* col_order, float scale, void* dk, void* dv, const SplitPlan& plan,
                           hipStream_t stream);

size_t error_ws_bytes(const Dims& m);
hipError_t launch_error_terms(const void* o_sparse, const void* o_dense, const float* lse_sparse,
                              const float* lse_dense, const Dims& m, double* out, void* ws, hipStream_t stream);

size_t vd_ws_bytes();
hipError_t launch_vd_loss(const void* u_sparse, const void* u_full, int64_t n, bool bf16, double weight, double* loss,
                          void* ws, hipStream_t stream);
hipError_t launch_vd_grad(const void* u_sparse, const void* u_full, int64_t n, bool bf16, double weight,
                          const double* upstream, void* grad, hipStream_t stream);

}  // namespace spa2
