// Block-sparse attention forward (Alg. 1 steps 7-21; Sec. 2.1) for gfx950.
//
// One workgroup (4 waves) per query block of 128 rows; wave w owns rows
// 32w..32w+31.  The workgroup walks the selected key blocks of its row of the
// block mask; each K/V tile (64 x d) is staged through LDS once and shared by
// the four waves.
//
// Everything is computed transposed so that a lane owns ONE query row:
//   S^T (keys x queries) = K_j Q_i^T      A = K rows from LDS, B = Q^T held in registers
//   O^T (d x queries)   += V_j^T P^T      A = V^T via transposing LDS reads, B = P^T
// The accumulator layout of S^T (lane = query, registers = keys) is exactly the
// B-operand layout the second product wants, so P never leaves registers, and
// the running maximum / sum of Alg. 1 (m_ij, l_ij) are per-lane scalars that
// need one exchange between the two halves of the wave per tile.
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

struct FwdArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v;
  uint16_t* o; float* lse;
  const int32_t* row_cnt; const int32_t* row_idx;
  int H, N, Tm, Tn, chunk;
  int64_t sb, sh, sn;
  float scale_log2;     // scale * log2(e): softmax is evaluated with exp2
};

template <int D>
struct FwdCfg {
  static constexpr int KP = D + 8;      // K tile row pitch (elements): row-wise 16-byte reads, conflict-free
  static constexpr int VP = D + 32;     // V tile row pitch: transposing 8-byte reads, conflict-free
  static constexpr int K_ELEMS = BKV * KP;
  static constexpr int V_ELEMS = BKV * VP;
  static constexpr int CH = BKV * D / 8 / 256;   // 16-byte chunks per thread per tile
};

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_kernel(FwdArgs a) {
  using C = FwdCfg<D>;
  __shared__ __align__(16) uint16_t Ks[2 * C::K_ELEMS];
  __shared__ __align__(16) uint16_t Vs[2 * C::V_ELEMS];

  const HeadBlock hb = xcd_map(blockIdx.x, a.Tm, a.chunk);
  if (!hb.valid) return;
  const int bh = hb.bh, i = hb.blk;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r32 = lane & 31, hf = lane >> 5;
  const int N = a.N;
  // counts and indices come from the caller's pattern: clamp them so that a corrupt list cannot
  // address memory outside the tensors
  const int cnt = min(max(a.row_cnt[(int64_t)bh * a.Tm + i], 0), a.Tn);
  const int32_t* idx = a.row_idx + ((int64_t)bh * a.Tm + i) * a.Tn;

  // Q^T fragments (B operand): lane = query row, 8 consecutive channels per 16-wide k step.
  const int qrow = i * BQ + w * 32 + r32;
  const int qrow_ld = qrow < N ? qrow : N - 1;
  bf16x8 qf[D / 16];
  {
    const uint16_t* qp = a.q + base + (int64_t)qrow_ld * a.sn + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) qf[kk] = *(const bf16x8*)(qp + 16 * kk);
  }

  // global -> register staging of one K/V tile (rows past N read as zeros)
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

  f32x16 oacc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[mb][v] = 0.f;
  float m_run = -INFINITY;   // running maximum, in log2 units (already multiplied by scale_log2)
  float l_run = 0.f;         // running sum over THIS lane's keys; the two halves are added at the end

  // per-lane offsets inside a tile
  const int k_off = r32 * C::KP + 8 * hf;                                   // K row read (A operand of S^T)
  const int s16 = lane & 15, blk16 = lane >> 4;
  const int v_off = (4 * hf + (s16 >> 2)) * C::VP + 16 * (blk16 & 1) + 4 * (s16 & 3);  // V transposing read

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

    // S^T = K_j Q_i^T : two 32-key blocks
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        const bf16x8 ka = *(const bf16x8*)(Kb + k_off + kb * 32 * C::KP + 16 * kk);
        s[kb] = mfma32(ka, qf[kk], s[kb]);
      }
    }
    // keys past N (short last block) do not take part in the softmax
    if ((j + 1) * BKV > N) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j * BKV + kb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
          if (key >= N) s[kb][v] = -INFINITY;
        }
    }
    // running maximum (Alg. 1 step 11)
    float mx = s[0][0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[0][v]);
#pragma unroll
    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[1][v]);
    mx = fmaxf(mx, other_half(mx));
    const float m_new = fmaxf(m_run, mx * a.scale_log2);
    const float alpha = fast_exp2(m_run - m_new);
    // P^T = exp(S^T - m) (step 12), partial row sum (step 13)
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = fast_exp2(fmaf(s[kb][v], a.scale_log2, -m_new));
        s[kb][v] = p;
        rs += p;
      }
    l_run = fmaf(l_run, alpha, rs);
    m_run = m_new;
    // O^T = diag(alpha) O^T + V^T P^T (step 14)
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[mb][v] *= alpha;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        // key slots of this lane: 32kb + 16cc + 4hf + {0..3} and +8: the order the accumulator holds them in
        const bf16x8 pb = make_bf16x8(s[kb][8 * cc + 0], s[kb][8 * cc + 1], s[kb][8 * cc + 2], s[kb][8 * cc + 3],
                                      s[kb][8 * cc + 4], s[kb][8 * cc + 5], s[kb][8 * cc + 6], s[kb][8 * cc + 7]);
        const uint16_t* vrow = Vb + v_off + (32 * kb + 16 * cc) * C::VP;
#pragma unroll
        for (int mb = 0; mb < D / 32; ++mb) {
          const bf16x8 va = join_tr(lds_read_tr4(vrow + 32 * mb), lds_read_tr4(vrow + 8 * C::VP + 32 * mb));
          oacc[mb] = mfma32(va, pb, oacc[mb]);
        }
      }
    if (more) store_tile((t + 1) & 1);
    __syncthreads();
  }

  // O_i = diag(l)^-1 O (step 18) and the log-sum-exp the backward pass needs
  const float l_tot = l_run + other_half(l_run);
  const float inv = cnt > 0 ? 1.f / l_tot : 0.f;
  if (qrow < N) {
    uint16_t* op = a.o + base + (int64_t)qrow * a.sn + 4 * hf;
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk = {pack_bf16(oacc[mb][4 * g + 0] * inv, oacc[mb][4 * g + 1] * inv),
                    pack_bf16(oacc[mb][4 * g + 2] * inv, oacc[mb][4 * g + 3] * inv)};
        *(u32x2*)(op + 32 * mb + 8 * g) = pk;
      }
    if (hf == 0) a.lse[(int64_t)bh * N + qrow] = cnt > 0 ? m_run * LN2 + __logf(l_tot) : -INFINITY;
  }
}

hipError_t launch_fwd(const void* q, const void* k, const void* v, const Dims& m, const int32_t* row_cnt,
                      const int32_t* row_idx, float scale, void* o, float* lse, hipStream_t stream) {
  FwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.o = (uint16_t*)o; a.lse = lse;
  a.row_cnt = row_cnt; a.row_idx = row_idx;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn;
  a.chunk = (m.Tm + 7) / 8;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  a.scale_log2 = scale * LOG2E;
  const dim3 grid((unsigned)(m.B * m.H * 8 * a.chunk)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(fwd_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(fwd_kernel<64>, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace spa2
