// Block-sparse attention backward for gfx950 (gradients of Alg. 1's O w.r.t. Q, K, V with
// the block mask held constant; Sec. 4.3 only states that a backward pass exists, the
// formulas are the usual softmax-attention calculus):
//   P = exp(S - LSE) on selected tiles,  dV = P^T dO,  dP = dO V^T,  D = rowsum(dO * O),
//   dS = P * (dP - D),  dQ = dS K * scale,  dK = dS^T Q * scale.
//
//   delta_kernel  D, one pass over O and dO.
//   dq_kernel     one workgroup per query block, walking its row of the mask (same shape
//                 as the forward kernel: a lane owns one query row).
//   dkdv_kernel   one workgroup per key block, walking the query blocks that selected it.
// dQ is produced by a second, row-oriented pass instead of atomics: results are
// deterministic and there is no fp32 dQ scratch tensor.
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

// ------------------------------------------------------------------ D = rowsum(dO * O)
struct DeltaArgs {
  const uint16_t* o; const uint16_t* d_o; float* delta;
  int H, N; int64_t sb, sh, sn;
};

template <int D>
__global__ __launch_bounds__(256) void delta_kernel(DeltaArgs a) {
  constexpr int LPR = D / 8, RP = 256 / LPR;
  const int bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x;
  const int col = (tid % LPR) * 8;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int row = (blockIdx.x * 4 + it) * RP + tid / LPR;
    float s = 0.f;
    if (row < a.N) {
      const u32x4 x = *(const u32x4*)(a.o + base + (int64_t)row * a.sn + col);
      const u32x4 y = *(const u32x4*)(a.d_o + base + (int64_t)row * a.sn + col);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s = fmaf(__builtin_bit_cast(float, x[e] << 16), __builtin_bit_cast(float, y[e] << 16), s);
        s = fmaf(__builtin_bit_cast(float, x[e] & 0xffff0000u), __builtin_bit_cast(float, y[e] & 0xffff0000u), s);
      }
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row < a.N && (tid % LPR) == 0) a.delta[(int64_t)bh * a.N + row] = s;
  }
}

hipError_t launch_bwd_delta(const void* o, const void* d_o, const Dims& m, float* delta, hipStream_t stream) {
  DeltaArgs a;
  a.o = (const uint16_t*)o; a.d_o = (const uint16_t*)d_o; a.delta = delta;
  a.H = m.H; a.N = m.N; a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  const int rows_per_wg = 4 * 256 / (m.d / 8);
  const dim3 grid((unsigned)((m.N + rows_per_wg - 1) / rows_per_wg), (unsigned)(m.B * m.H)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(delta_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(delta_kernel<64>, grid, block, 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------ dQ
struct DqArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v; const uint16_t* d_o;
  const float* lse; const float* delta; uint16_t* dq;
  const int32_t* row_cnt; const int32_t* row_idx;
  int H, N, Tm, Tn, chunk;
  int64_t sb, sh, sn;
  float scale, scale_log2;
};

template <int D>
struct DqCfg {
  static constexpr int KP = D + 8;     // K tile pitch (row reads for S^T, transposing reads for dQ^T)
  static constexpr int VP = D + 8;     // V tile pitch (row reads for dP^T)
  static constexpr int K_ELEMS = BKV * KP;
  static constexpr int V_ELEMS = BKV * VP;
  static constexpr int CH = BKV * D / 8 / 256;
};

// Transposed formulation, a lane owns one query row (see fwd.hip):
//   S^T  = K_j Q_i^T        P^T  = exp(S^T - LSE)
//   dP^T = V_j dO_i^T       dS^T = P^T * (dP^T - D)
//   dQ^T += K_j^T dS^T      (K^T through transposing LDS reads)
template <int D>
__global__ __launch_bounds__(256, 2) void dq_kernel(DqArgs a) {
  using C = DqCfg<D>;
  __shared__ __align__(16) uint16_t Ks[2 * C::K_ELEMS];
  __shared__ __align__(16) uint16_t Vs[2 * C::V_ELEMS];

  const HeadBlock hb = xcd_map(blockIdx.x, a.Tm, a.chunk);
  if (!hb.valid) return;
  const int bh = hb.bh, i = hb.blk;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r32 = lane & 31, hf = lane >> 5;
  const int N = a.N;
  const int cnt = min(max(a.row_cnt[(int64_t)bh * a.Tm + i], 0), a.Tn);   // clamped: see fwd.hip
  const int32_t* idx = a.row_idx + ((int64_t)bh * a.Tm + i) * a.Tn;

  const int qrow = i * BQ + w * 32 + r32;
  const int qrow_ld = qrow < N ? qrow : N - 1;
  bf16x8 qf[D / 16], dof[D / 16];
  {
    const int64_t off = base + (int64_t)qrow_ld * a.sn + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      qf[kk] = *(const bf16x8*)(a.q + off + 16 * kk);
      dof[kk] = *(const bf16x8*)(a.d_o + off + 16 * kk);
    }
  }
  const float lse2 = a.lse[(int64_t)bh * N + qrow_ld] * LOG2E;
  const float dlt = a.delta[(int64_t)bh * N + qrow_ld];

  u32x4 kreg[C::CH], vreg[C::CH];
  auto load_tile = [&](int j) {
    j = min(max(j, 0), a.Tn - 1);
#pragma unroll
    for (int r = 0; r < C::CH; ++r) {
      const int c = tid + 256 * r;
      const int row = c / (D / 8), col = (c % (D / 8)) * 8;
      const int tok = j * BKV + row;
      if (tok < N) {
        const int64_t off = base + (int64_t)tok * a.sn + col;
        kreg[r] = *(const u32x4*)(a.k + off);
        vreg[r] = *(const u32x4*)(a.v + off);
      } else {
        kreg[r] = u32x4{0, 0, 0, 0};
        vreg[r] = u32x4{0, 0, 0, 0};
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int r = 0; r < C::CH; ++r) {
      const int c = tid + 256 * r;
      const int row = c / (D / 8), col = (c % (D / 8)) * 8;
      *(u32x4*)(Ks + buf * C::K_ELEMS + row * C::KP + col) = kreg[r];
      *(u32x4*)(Vs + buf * C::V_ELEMS + row * C::VP + col) = vreg[r];
    }
  };

  f32x16 acc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;

  const int k_off = r32 * C::KP + 8 * hf;
  const int v_off = r32 * C::VP + 8 * hf;
  const int s16 = lane & 15, blk16 = lane >> 4;
  const int kt_off = (4 * hf + (s16 >> 2)) * C::KP + 16 * (blk16 & 1) + 4 * (s16 & 3);

  if (cnt > 0) {
    load_tile(idx[0]);
    store_tile(0);
  }
  __syncthreads();

  for (int t = 0; t < cnt; ++t) {
    const int j = min(max(idx[t], 0), a.Tn - 1);
    const bool more = t + 1 < cnt;
    if (more) load_tile(idx[t + 1]);
    const uint16_t* Kb = Ks + (t & 1) * C::K_ELEMS;
    const uint16_t* Vb = Vs + (t & 1) * C::V_ELEMS;

    f32x16 s[2], dp[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[kb][v] = 0.f; dp[kb][v] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 ka = *(const bf16x8*)(Kb + k_off + kb * 32 * C::KP + 16 * kk);
        s[kb] = mfma32(ka, qf[kk], s[kb]);
      }
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 va = *(const bf16x8*)(Vb + v_off + kb * 32 * C::VP + 16 * kk);
        dp[kb] = mfma32(va, dof[kk], dp[kb]);
      }
    }
    const bool tail = (j + 1) * BKV > N;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float p = fast_exp2(fmaf(s[kb][v], a.scale_log2, -lse2));
        if (tail) {
          const int key = j * BKV + kb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
          if (key >= N) p = 0.f;
        }
        s[kb][v] = p * (dp[kb][v] - dlt);     // dS^T
      }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const bf16x8 dsb = make_bf16x8(s[kb][8 * cc + 0], s[kb][8 * cc + 1], s[kb][8 * cc + 2], s[kb][8 * cc + 3],
                                       s[kb][8 * cc + 4], s[kb][8 * cc + 5], s[kb][8 * cc + 6], s[kb][8 * cc + 7]);
        const uint16_t* krow = Kb + kt_off + (32 * kb + 16 * cc) * C::KP;
#pragma unroll
        for (int mb = 0; mb < D / 32; ++mb) {
          const bf16x8 kta = join_tr(lds_read_tr4(krow + 32 * mb), lds_read_tr4(krow + 8 * C::KP + 32 * mb));
          acc[mb] = mfma32(kta, dsb, acc[mb]);
        }
      }
    if (more) store_tile((t + 1) & 1);
    __syncthreads();
  }

  if (qrow < N) {
    uint16_t* op = a.dq + base + (int64_t)qrow * a.sn + 4 * hf;
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk = {pack_bf16(acc[mb][4 * g + 0] * a.scale, acc[mb][4 * g + 1] * a.scale),
                    pack_bf16(acc[mb][4 * g + 2] * a.scale, acc[mb][4 * g + 3] * a.scale)};
        *(u32x2*)(op + 32 * mb + 8 * g) = pk;
      }
  }
}

hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                         const float* delta, const Dims& m, const int32_t* row_cnt, const int32_t* row_idx,
                         float scale, void* dq, hipStream_t stream) {
  DqArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.lse = lse; a.delta = delta; a.dq = (uint16_t*)dq;
  a.row_cnt = row_cnt; a.row_idx = row_idx;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn; a.chunk = (m.Tm + 7) / 8;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  a.scale = scale; a.scale_log2 = scale * LOG2E;
  const dim3 grid((unsigned)(m.B * m.H * 8 * a.chunk)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(dq_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(dq_kernel<64>, grid, block, 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------ dK, dV
struct DkvArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v; const uint16_t* d_o;
  const float* lse; const float* delta; uint16_t* dk; uint16_t* dv;
  const int32_t* col_cnt; const int32_t* col_idx;
  int H, N, Tm, Tn, chunk;
  int64_t sb, sh, sn;
  float scale, scale_log2;
};

template <int D>
struct DkvCfg {
  static constexpr int QP = D + 8;                // Q / dO tile pitch
  static constexpr int T_ELEMS = BQ * QP;
  static constexpr int CH = BQ * D / 8 / 256;     // 16-byte chunks per thread per 128-row tile
};

// One workgroup per key block j (64 keys); wave w owns keys 16w..16w+15 and keeps its
// K and V rows in registers.  For every query block i that selected j (128 queries,
// staged in LDS together with dO, LSE and D):
//   S  (q x keys) = Q_i K_j^T        16x16x32 MFMA, A = Q rows from LDS, B = K^T in registers
//   dP (q x keys) = dO_i V_j^T       same with dO and V
//   P = exp(S - LSE), dS = P * (dP - D)     accumulator layout: lane = key, registers = queries
//   dV^T (d x keys) += dO_i^T P      A = dO^T via transposing LDS reads, B = P from registers
//   dK^T (d x keys) += Q_i^T dS      A = Q^T  via transposing LDS reads, B = dS from registers
template <int D>
__global__ __launch_bounds__(256, 2) void dkdv_kernel(DkvArgs a) {
  using C = DkvCfg<D>;
  __shared__ __align__(16) uint16_t Qs[C::T_ELEMS];
  __shared__ __align__(16) uint16_t Os[C::T_ELEMS];
  __shared__ __align__(16) float lse_s[BQ];
  __shared__ __align__(16) float dlt_s[BQ];

  const HeadBlock hb = xcd_map(blockIdx.x, a.Tn, a.chunk);
  if (!hb.valid) return;
  const int bh = hb.bh, j = hb.blk;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r16 = lane & 15, G = lane >> 4;
  const int N = a.N;
  const int cnt = min(max(a.col_cnt[(int64_t)bh * a.Tn + j], 0), a.Tm);   // clamped: see fwd.hip
  const int32_t* idx = a.col_idx + ((int64_t)bh * a.Tn + j) * a.Tm;

  // K^T / V^T fragments (B operands): lane = key, 8 consecutive channels per 32-wide k step
  const int key = j * BKV + w * 16 + r16;
  const bool key_ok = key < N;
  bf16x8 kf[D / 32], vf[D / 32];
  {
    const int64_t off = base + (int64_t)(key_ok ? key : N - 1) * a.sn + 8 * G;
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      kf[kk] = *(const bf16x8*)(a.k + off + 32 * kk);
      vf[kk] = *(const bf16x8*)(a.v + off + 32 * kk);
    }
  }

  f32x4 dk_acc[D / 16], dv_acc[D / 16];
#pragma unroll
  for (int nb = 0; nb < D / 16; ++nb) {
    dk_acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    dv_acc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int a_off = r16 * C::QP + 8 * G;                                        // row reads (A operand)
  const int t_off = (4 * G + (r16 >> 2)) * C::QP + 4 * (r16 & 3);               // transposing reads

  for (int t = 0; t < cnt; ++t) {
    const int i = min(max(idx[t], 0), a.Tm - 1);
    __syncthreads();                       // previous tile fully consumed
#pragma unroll
    for (int r = 0; r < C::CH; ++r) {
      const int c = tid + 256 * r;
      const int row = c / (D / 8), col = (c % (D / 8)) * 8;
      const int tok = i * BQ + row;
      u32x4 qv = u32x4{0, 0, 0, 0}, ov = u32x4{0, 0, 0, 0};
      if (tok < N) {
        const int64_t off = base + (int64_t)tok * a.sn + col;
        qv = *(const u32x4*)(a.q + off);
        ov = *(const u32x4*)(a.d_o + off);
      }
      *(u32x4*)(Qs + row * C::QP + col) = qv;
      *(u32x4*)(Os + row * C::QP + col) = ov;
    }
    if (tid < BQ) {
      const int tok = i * BQ + tid;
      // rows past N get LSE = +inf, so their P is exactly zero
      lse_s[tid] = tok < N ? a.lse[(int64_t)bh * N + tok] * LOG2E : INFINITY;
      dlt_s[tid] = tok < N ? a.delta[(int64_t)bh * N + tok] : 0.f;
    }
    __syncthreads();

#pragma unroll
    for (int qc = 0; qc < 4; ++qc) {        // 32 queries at a time
      f32x4 s[2], dp[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int qb = 2 * qc + u;
        s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        dp[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
          const bf16x8 qa = *(const bf16x8*)(Qs + a_off + qb * 16 * C::QP + 32 * kk);
          s[u] = mfma16(qa, kf[kk], s[u]);
          const bf16x8 oa = *(const bf16x8*)(Os + a_off + qb * 16 * C::QP + 32 * kk);
          dp[u] = mfma16(oa, vf[kk], dp[u]);
        }
        const f32x4 l4 = *(const f32x4*)(lse_s + qb * 16 + 4 * G);
        const f32x4 d4 = *(const f32x4*)(dlt_s + qb * 16 + 4 * G);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          float p = fast_exp2(fmaf(s[u][v], a.scale_log2, -l4[v]));
          if (!key_ok) p = 0.f;
          s[u][v] = p;
          dp[u][v] = p * (dp[u][v] - d4[v]);
        }
      }
      // this lane's 8 query slots: 32qc + 4G + {0..3} and 32qc + 16 + 4G + {0..3}
      const bf16x8 pb = make_bf16x8(s[0][0], s[0][1], s[0][2], s[0][3], s[1][0], s[1][1], s[1][2], s[1][3]);
      const bf16x8 dsb = make_bf16x8(dp[0][0], dp[0][1], dp[0][2], dp[0][3], dp[1][0], dp[1][1], dp[1][2], dp[1][3]);
      const uint16_t* orow = Os + t_off + 32 * qc * C::QP;
      const uint16_t* qrow = Qs + t_off + 32 * qc * C::QP;
#pragma unroll
      for (int nb = 0; nb < D / 16; ++nb) {
        const bf16x8 ot = join_tr(lds_read_tr4(orow + 16 * nb), lds_read_tr4(orow + 16 * C::QP + 16 * nb));
        dv_acc[nb] = mfma16(ot, pb, dv_acc[nb]);
        const bf16x8 qt = join_tr(lds_read_tr4(qrow + 16 * nb), lds_read_tr4(qrow + 16 * C::QP + 16 * nb));
        dk_acc[nb] = mfma16(qt, dsb, dk_acc[nb]);
      }
    }
  }

  // accumulators hold dK^T / dV^T: lane = key, registers = 4 consecutive channels 16nb + 4G ..
  if (key_ok) {
    const int64_t off = base + (int64_t)key * a.sn + 4 * G;
#pragma unroll
    for (int nb = 0; nb < D / 16; ++nb) {
      u32x2 pk = {pack_bf16(dk_acc[nb][0] * a.scale, dk_acc[nb][1] * a.scale),
                  pack_bf16(dk_acc[nb][2] * a.scale, dk_acc[nb][3] * a.scale)};
      *(u32x2*)(a.dk + off + 16 * nb) = pk;
      u32x2 pv = {pack_bf16(dv_acc[nb][0], dv_acc[nb][1]), pack_bf16(dv_acc[nb][2], dv_acc[nb][3])};
      *(u32x2*)(a.dv + off + 16 * nb) = pv;
    }
  }
}

hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                           const float* delta, const Dims& m, const int32_t* col_cnt, const int32_t* col_idx,
                           float scale, void* dk, void* dv, hipStream_t stream) {
  DkvArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.lse = lse; a.delta = delta; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv;
  a.col_cnt = col_cnt; a.col_idx = col_idx;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn; a.chunk = (m.Tn + 7) / 8;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  a.scale = scale; a.scale_log2 = scale * LOG2E;
  const dim3 grid((unsigned)(m.B * m.H * 8 * a.chunk)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(dkdv_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(dkdv_kernel<64>, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace spa2
