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
  uint16_t* o; uint16_t* o_res; float* lse;
  const int32_t* row_cnt; const int32_t* row_idx; const int32_t* row_order;
  int H, N, Tm, Tn, chunk;
  int64_t sb, sh, sn;
  float scale_log2;     // scale * log2(e): softmax is evaluated with exp2
  SplitPlan sp;         // long rows cut into parts (split.hip); sp.pool_slots == 0: every row is walked whole
};

// Partial result of one part of a split row, per thread of the workgroup: the unnormalised accumulator, then
// the running maximum (log2 units) and the row sum, both already combined over the two halves of the wave.
template <int D> constexpr int fwd_slot_floats() { return 256 * (D / 2) + 512; }
size_t fwd_slot_bytes(const Dims& m) { return (size_t)(m.d == 128 ? fwd_slot_floats<128>() : fwd_slot_floats<64>()) * 4; }

// O_i = diag(l)^-1 O (Alg. 1 step 18) -> bf16 (+ optional residual), LSE = m ln 2 + log l.
template <int D>
__device__ __forceinline__ void fwd_store_rows(const FwdArgs& a, int bh, int64_t base, int qrow, int hf,
                                               const f32x16 (&oacc)[D / 32], float m_run, float l_tot) {
  const float inv = 1.f / l_tot;
  if (qrow < a.N) {
    uint16_t* op = a.o + base + (int64_t)qrow * a.sn + 4 * hf;
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = oacc[mb][4 * g + e] * inv;
        const u32x2 pk2 = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
        *(u32x2*)(op + 32 * mb + 8 * g) = pk2;
        if (a.o_res) {      // what the rounding to bf16 dropped, itself rounded to bf16
          const float r0 = x[0] - __builtin_bit_cast(float, pk2[0] << 16);
          const float r1 = x[1] - __builtin_bit_cast(float, pk2[0] & 0xffff0000u);
          const float r2 = x[2] - __builtin_bit_cast(float, pk2[1] << 16);
          const float r3 = x[3] - __builtin_bit_cast(float, pk2[1] & 0xffff0000u);
          const u32x2 pr = {pack_bf16(r0, r1), pack_bf16(r2, r3)};
          *(u32x2*)(a.o_res + (op - a.o) + 32 * mb + 8 * g) = pr;
        }
      }
    if (hf == 0) a.lse[(int64_t)bh * a.N + qrow] = m_run * LN2 + __logf(l_tot);
  }
}

template <int D>
struct FwdCfg {
  static constexpr int KP = D + 8;      // K tile row pitch (elements): row-wise 16-byte reads, conflict-free
  static constexpr int VP = D + 32;     // V tile row pitch: transposing 8-byte reads, conflict-free
  static constexpr int K_ELEMS = BKV * KP;
  static constexpr int V_ELEMS = BKV * VP;
  static constexpr int CH = BKV * D / 8 / 256;   // 16-byte chunks per thread per tile
};
constexpr int PD = 4;   // how many MFMAs ahead an LDS operand is requested

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_kernel(FwdArgs a) {
  using C = FwdCfg<D>;
  __shared__ __align__(16) uint16_t Ks[2 * C::K_ELEMS];
  __shared__ __align__(16) uint16_t Vs[2 * C::V_ELEMS];

  // Which row, and which part of its list.  The first sp.pool_slots workgroups of the launch are the extra parts of
  // split rows (part >= 1); the others take one row each: the whole list, or part 0 if the row is split.
  int bh, i, part = 0, slot = -1;
  if ((int)blockIdx.x < a.sp.pool_slots) {
    if ((int)blockIdx.x >= a.sp.header[0]) return;
    const int unit = a.sp.part_table[2 * blockIdx.x];
    part = a.sp.part_table[2 * blockIdx.x + 1];
    bh = unit / a.Tm; i = unit % a.Tm;
    slot = a.sp.unit_slot[unit] + part;
  } else {
    const HeadBlock hb = xcd_map(blockIdx.x - a.sp.pool_slots, a.Tm, a.chunk);
    if (!hb.valid) return;
    bh = hb.bh;
    // optional launch order: position hb.blk of this head's schedule -> query block (clamped: caller data)
    i = a.row_order ? min(max(a.row_order[(int64_t)bh * a.Tm + hb.blk], 0), a.Tm - 1) : hb.blk;
    if (a.sp.pool_slots) slot = a.sp.unit_slot[(int64_t)bh * a.Tm + i];
  }
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r32 = lane & 31, hf = lane >> 5;
  const int N = a.N;
  // counts and indices come from the caller's pattern: clamp them so that a corrupt list cannot
  // address memory outside the tensors
  int cnt = min(max(a.row_cnt[(int64_t)bh * a.Tm + i], 0), a.Tn);
  const int32_t* idx = a.row_idx + ((int64_t)bh * a.Tm + i) * a.Tn;
  if (slot >= 0) {            // entries [part * S, (part + 1) * S) of the list (never empty: part < ceil(cnt / S))
    const int S = a.sp.header[1];
    idx += part * S;
    cnt = min(cnt - part * S, S);
  }
  const int qrow = i * BQ + w * 32 + r32;

  if (cnt == 0) {   // a row without any selected block (never produced by the masker): O = 0, LSE = -inf
    if (qrow < N) {
      uint16_t* op = a.o + base + (int64_t)qrow * a.sn + (D / 2) * hf;
#pragma unroll
      for (int c = 0; c < D / 16; ++c) *(u32x4*)(op + 8 * c) = u32x4{0, 0, 0, 0};
      if (a.o_res) {
        uint16_t* rp = a.o_res + (op - a.o);
#pragma unroll
        for (int c = 0; c < D / 16; ++c) *(u32x4*)(rp + 8 * c) = u32x4{0, 0, 0, 0};
      }
      if (hf == 0) a.lse[(int64_t)bh * N + qrow] = -INFINITY;
    }
    return;
  }

  // Q^T fragments (B operand): lane = query row, 8 consecutive channels per 16-wide k step.
  const int qrow_ld = qrow < N ? qrow : N - 1;
  bf16x8 qf[D / 16];
  {
    const uint16_t* qp = a.q + base + (int64_t)qrow_ld * a.sn + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) qf[kk] = *(const bf16x8*)(qp + 16 * kk);
  }

  // global -> register staging of one K/V tile.  Thread t moves 16-byte chunk (row, col) with
  // row = t / (D/8) + r * 256 / (D/8).  Rows past N (short last block) are clamped to the last
  // token: their keys are masked out of the softmax below and their P is exactly zero, so the
  // duplicated K/V rows never contribute.
  constexpr int RSTEP = 256 / (D / 8);
  const int ld_row = tid / (D / 8), ld_col = (tid % (D / 8)) * 8;
  uint32_t goff[C::CH];          // byte offset of this thread's chunks inside a full tile
#pragma unroll
  for (int r = 0; r < C::CH; ++r) goff[r] = (uint32_t)(((ld_row + RSTEP * r) * a.sn + ld_col) * 2);
  const int lds_k = ld_row * C::KP + ld_col, lds_v = ld_row * C::VP + ld_col;
  // Two staging sets: a tile is requested two iterations before it is needed, so that a request has
  // two tiles' worth of compute to come back from L2 / HBM (one is not enough under load).
  struct Stage { u32x4 k[C::CH], v[C::CH]; };
  Stage stA, stB;
  auto load_tile = [&](Stage& st, int j) {
    j = min(max(j, 0), a.Tn - 1);
    const int64_t tile = (base + (int64_t)j * BKV * a.sn) * 2;       // uniform
    const char* kp = (const char*)a.k + tile;
    const char* vp = (const char*)a.v + tile;
    if ((j + 1) * BKV <= N) {
#pragma unroll
      for (int r = 0; r < C::CH; ++r) {
        st.k[r] = *(const u32x4*)(kp + goff[r]);
        st.v[r] = *(const u32x4*)(vp + goff[r]);
      }
    } else {
      const int last = N - 1 - j * BKV;
#pragma unroll
      for (int r = 0; r < C::CH; ++r) {
        const uint32_t o2 = (uint32_t)((min(ld_row + RSTEP * r, last) * a.sn + ld_col) * 2);
        st.k[r] = *(const u32x4*)(kp + o2);
        st.v[r] = *(const u32x4*)(vp + o2);
      }
    }
  };
  auto store_tile = [&](const Stage& st, int buf) {
#pragma unroll
    for (int r = 0; r < C::CH; ++r) {
      *(u32x4*)(Ks + buf * C::K_ELEMS + lds_k + RSTEP * r * C::KP) = st.k[r];
      *(u32x4*)(Vs + buf * C::V_ELEMS + lds_v + RSTEP * r * C::VP) = st.v[r];
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

  // Pipeline: tile T is requested during iteration T-3 into the staging set of its parity, written to
  // LDS buffer T&1 during iteration T-1 (that buffer held tile T-2, fully consumed before the barrier that
  // ended iteration T-2), and consumed in iteration T.  Two tiles are in flight at any time and one
  // barrier per tile is enough.
  // The list of selected key blocks is read with scalar loads, one entry per iteration and one iteration
  // ahead of its use: jw[m] is the (clamped) block of tile t+m, jpre the entry that becomes jw[3] next.
  // Where in its list a row starts is a free choice (the online softmax does not depend on the order of the
  // tiles, up to rounding), and it is used to keep the rows that run on one XCD at the same time close
  // together in key space: query block i starts at the first selected block at or after (i mod 64) / 64 of
  // the key range and wraps around.  An XCD takes consecutive query blocks, and its workgroups start as slots
  // free up, one row-duration spread over its 64 slots; so a row that starts 1/64 of a row-duration later
  // also starts 1/64 of the key range further on: all of them sweep the keys together and share K/V tiles
  // through the XCD's L2.  The start depends on the row alone, so results do not depend on the launch order.
  int t0 = 0;
  {
    const int start_blk = (int)(((int64_t)(i & 63) * a.Tn) >> 6);
    for (int c = 0; c < cnt; c += 64) {
      const int e = c + lane;
      const bool below = e < cnt && idx[min(e, cnt - 1)] < start_blk;
      t0 += __builtin_popcountll(__builtin_amdgcn_ballot_w64(below));
    }
    t0 = __builtin_amdgcn_readfirstlane(t0);
    if (t0 >= cnt) t0 = 0;
  }
  auto rot = [&](int t) -> int { const int p = min(t, cnt - 1) + t0; return p >= cnt ? p - cnt : p; };
  auto list_at = [&](int t) -> int { return min(max(idx[rot(t)], 0), a.Tn - 1); };
  int jw[4] = {list_at(0), list_at(1), list_at(2), list_at(3)};
  int jpre = idx[rot(4)];      // raw: clamped when it is used, so that nothing waits for it here
  // One piece of the staging work of an iteration: chunk r of K (p even) or V (p odd) of `next` goes to LDS
  // buffer `buf` (tile t+1, requested two iterations ago), then the same registers request tile t+3.  The
  // pieces are handed out between the MFMAs of the S^T loop: issued back to back, the eight requests would
  // keep the wave at the issue stage until the texture unit has taken the last one.
  // Both halves are unconditional (past the end of the list the last tile is requested again and the store
  // goes to a buffer nobody reads): a branch around a memory operation inside the loop would make the
  // compiler wait for every outstanding request at each store.
  auto stage_piece = [&](Stage& st, int p, int buf, const char* kp, const char* vp, int last) {
    const int r = p >> 1;
    const uint32_t off = (uint32_t)((min(ld_row + RSTEP * r, last) * a.sn + ld_col) * 2);
    if (p & 1) {
      *(u32x4*)(Vs + buf * C::V_ELEMS + lds_v + RSTEP * r * C::VP) = st.v[r];
      st.v[r] = *(const u32x4*)(vp + off);
    } else {
      *(u32x4*)(Ks + buf * C::K_ELEMS + lds_k + RSTEP * r * C::KP) = st.k[r];
      st.k[r] = *(const u32x4*)(kp + off);
    }
  };
  load_tile(stA, jw[0]);
  store_tile(stA, 0);
  load_tile(stB, jw[1]);
  load_tile(stA, jw[2]);
  __syncthreads();

  auto iteration = [&](int t, Stage& next, Stage& /*unused*/) {
    const int j = jw[0], j3 = jw[3];
    const int64_t tile3 = (base + (int64_t)j3 * BKV * a.sn) * 2;       // uniform
    const char* kp3 = (const char*)a.k + tile3;
    const char* vp3 = (const char*)a.v + tile3;
    const int last3 = min(BKV - 1, N - 1 - j3 * BKV);
    jw[0] = jw[1]; jw[1] = jw[2]; jw[2] = jw[3]; jw[3] = min(max(jpre, 0), a.Tn - 1);
    jpre = idx[rot(t + 5)];
    const uint16_t* Kb = Ks + (t & 1) * C::K_ELEMS;
    const uint16_t* Vb = Vs + (t & 1) * C::V_ELEMS;

    // S^T = K_j Q_i^T : two 32-key blocks.  LDS operand reads run PD MFMAs ahead of their use.
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
    {
      constexpr int NQK = 2 * (D / 16);
      bf16x8 kfr[PD];
#pragma unroll
      for (int x = 0; x < PD; ++x)
        kfr[x] = *(const bf16x8*)(Kb + k_off + (x / (D / 16)) * 32 * C::KP + 16 * (x % (D / 16)));
#pragma unroll
      for (int x = 0; x < NQK; ++x) {
        const int kb = x / (D / 16), kk = x % (D / 16);
        s[kb] = mfma32(kfr[x % PD], qf[kk], s[kb]);
        if (x + PD < NQK) {
          const int y = x + PD;
          kfr[x % PD] = *(const bf16x8*)(Kb + k_off + (y / (D / 16)) * 32 * C::KP + 16 * (y % (D / 16)));
        }
        if (x % 2 == 0) stage_piece(next, x / 2, (t + 1) & 1, kp3, vp3, last3);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // first V^T operands of the second product are requested now, so that they arrive during the softmax
    constexpr int NPV = 4 * (D / 32);
    bf16x8 vfr[PD];
    auto v_frag = [&](int y) {
      const int kb = y / (2 * (D / 32)), cc = (y / (D / 32)) % 2, mb = y % (D / 32);
      const uint16_t* vrow = Vb + v_off + (32 * kb + 16 * cc) * C::VP + 32 * mb;
      return join_tr(lds_read_tr4(vrow), lds_read_tr4(vrow + 8 * C::VP));
    };
#pragma unroll
    for (int x = 0; x < PD; ++x) vfr[x] = v_frag(x);
    __builtin_amdgcn_sched_barrier(0);
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
    mx = max_halves(mx);
    const float m_new = fmaxf(m_run, mx * a.scale_log2);
    // rescale the accumulators (steps 13-14) only when some row's maximum moved: after the first
    // few tiles it rarely does, and the branch is uniform over the wave
    if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
      const float alpha = fast_exp2(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[mb][v] *= alpha;
      m_run = m_new;
    }
    // P^T = exp(S^T - m) (step 12), rounded to bf16 for the second product; the row sum (step 13)
    // is taken over the rounded values, so numerator and denominator use the same weights
    uint32_t pk[2][8];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float p0 = fast_exp2(fmaf(s[kb][2 * u], a.scale_log2, -m_run));
        const float p1 = fast_exp2(fmaf(s[kb][2 * u + 1], a.scale_log2, -m_run));
        pk[kb][u] = pack_bf16(p0, p1);
        l_run = dot2_ones(pk[kb][u], l_run);
      }
    // O^T += V^T P^T (step 14).  MFMA x uses key slots 32kb + 16cc + 4hf + {0..3} and + 8 (the order the
    // accumulator of S^T holds them in) of output block mb.
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int x = 0; x < NPV; ++x) {
      const int kb = x / (2 * (D / 32)), cc = (x / (D / 32)) % 2, mb = x % (D / 32);
      const u32x4 pu = {pk[kb][4 * cc], pk[kb][4 * cc + 1], pk[kb][4 * cc + 2], pk[kb][4 * cc + 3]};
      oacc[mb] = mfma32(vfr[x % PD], __builtin_bit_cast(bf16x8, pu), oacc[mb]);
      if (x + PD < NPV) vfr[x % PD] = v_frag(x + PD);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  };
  for (int t = 0; t < cnt; t += 2) {
    iteration(t, stB, stA);                       // tile t+1 (odd) lives in set B
    if (t + 1 < cnt) iteration(t + 1, stA, stB);  // tile t+2 (even) lives in set A
  }

  const float l_tot = sum_halves(l_run);
  if (slot >= 0) {            // one part of a split row: leave the partial result to the merge kernel
    float* ps = a.sp.pool + (int64_t)slot * a.sp.slot_floats;
    f32x4* pa = (f32x4*)(ps + tid * (D / 2));
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        pa[mb * 4 + g] = f32x4{oacc[mb][4 * g], oacc[mb][4 * g + 1], oacc[mb][4 * g + 2], oacc[mb][4 * g + 3]};
    ps[256 * (D / 2) + tid] = m_run;
    ps[256 * (D / 2) + 256 + tid] = l_tot;
    return;
  }
  // O_i = diag(l)^-1 O (step 18) and the log-sum-exp the backward pass needs
  fwd_store_rows<D>(a, bh, base, qrow, hf, oacc, m_run, l_tot);
}

// Combines the parts of every split row, in part order (so the result does not depend on which part finished
// first): m = max m_p, l = sum l_p 2^(m_p - m), O = sum O_p 2^(m_p - m) / l.  Same thread -> (row, channel) mapping
// as fwd_kernel.  Workgroup x takes split row x of the plan; there are at most pool_slots / 2 of them.
template <int D>
__device__ __forceinline__ void fwd_merge_kernel_one(const FwdArgs& a, int m_idx) {
  const int unit = a.sp.merge_table[m_idx];
  const int bh = unit / a.Tm, i = unit % a.Tm;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r32 = lane & 31, hf = lane >> 5;
  const int cnt = min(max(a.row_cnt[unit], 0), a.Tn);
  const int S = a.sp.header[1];
  const int parts = (cnt + S - 1) / S;
  const float* p0 = a.sp.pool + (int64_t)a.sp.unit_slot[unit] * a.sp.slot_floats;
  float m = -INFINITY;
  for (int p = 0; p < parts; p += 4) {       // four loads in flight per step
    float mp[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) mp[x] = p0[(int64_t)min(p + x, parts - 1) * a.sp.slot_floats + 256 * (D / 2) + tid];
    m = fmaxf(fmaxf(m, fmaxf(mp[0], mp[1])), fmaxf(mp[2], mp[3]));
  }
  f32x16 oacc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[mb][v] = 0.f;
  float l = 0.f;
  // two parts per step: the loads of both are in flight together (the chain of parts is what takes the time)
  for (int p = 0; p < parts; p += 2) {
    const bool two = p + 1 < parts;
    const float* ps0 = p0 + (int64_t)p * a.sp.slot_floats;
    const float* ps1 = p0 + (int64_t)(two ? p + 1 : p) * a.sp.slot_floats;
    const float sc0 = fast_exp2(ps0[256 * (D / 2) + tid] - m);
    const float sc1 = two ? fast_exp2(ps1[256 * (D / 2) + tid] - m) : 0.f;
    l = fmaf(ps0[256 * (D / 2) + 256 + tid], sc0, l);
    l = fmaf(ps1[256 * (D / 2) + 256 + tid], sc1, l);
    const f32x4* pa0 = (const f32x4*)(ps0 + tid * (D / 2));
    const f32x4* pa1 = (const f32x4*)(ps1 + tid * (D / 2));
    f32x4 x0[D / 8], x1[D / 8];
#pragma unroll
    for (int c = 0; c < D / 8; ++c) { x0[c] = pa0[c]; x1[c] = pa1[c]; }
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          oacc[mb][4 * g + e] = fmaf(x1[mb * 4 + g][e], sc1, fmaf(x0[mb * 4 + g][e], sc0, oacc[mb][4 * g + e]));
  }
  fwd_store_rows<D>(a, bh, base, i * BQ + w * 32 + r32, hf, oacc, m, l);
}

// (one workgroup per split list as a rule; the loop covers a launch with fewer workgroups than lists)
template <int D>
__global__ __launch_bounds__(256) void fwd_merge_kernel(FwdArgs a) {
  const int n = a.sp.header[2];
  for (int m_idx = blockIdx.x; m_idx < n; m_idx += gridDim.x) fwd_merge_kernel_one<D>(a, m_idx);
}

hipError_t launch_fwd(const void* q, const void* k, const void* v, const Dims& m, const int32_t* row_cnt,
                      const int32_t* row_idx, const int32_t* row_order, float scale, void* o, void* o_res,
                      float* lse, const SplitPlan& plan, hipStream_t stream) {
  FwdArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.o = (uint16_t*)o; a.o_res = (uint16_t*)o_res; a.lse = lse;
  a.row_cnt = row_cnt; a.row_idx = row_idx; a.row_order = row_order;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn;
  a.chunk = (m.Tm + 7) / 8;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  a.scale_log2 = scale * LOG2E;
  a.sp = plan;
  if (plan.pool_slots) {
    const hipError_t e = launch_split_plan(row_cnt, (int64_t)m.B * m.H * m.Tm, m.Tn, SPLIT_MIN_PART, plan, stream);
    if (e != hipSuccess) return e;
  }
  const dim3 grid((unsigned)(plan.pool_slots + m.B * m.H * 8 * a.chunk)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(fwd_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(fwd_kernel<64>, grid, block, 0, stream, a);
  if (plan.pool_slots) {
    const dim3 mg((unsigned)(plan.pool_slots / 2));
    if (m.d == 128) hipLaunchKernelGGL(fwd_merge_kernel<128>, mg, block, 0, stream, a);
    else            hipLaunchKernelGGL(fwd_merge_kernel<64>, mg, block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace spa2
