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
  const uint16_t* o; const uint16_t* o_res; const uint16_t* d_o; float* delta;
  int H, N; int64_t sb, sh, sn;
};

template <int D>
__global__ __launch_bounds__(256) void delta_kernel(DeltaArgs a) {
  constexpr int LPR = D / 8, RP = 256 / LPR;
  constexpr int NIT = 4;              // row groups per workgroup; all their loads are issued before the first use
  const int bh = blockIdx.y;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x;
  const int col = (tid % LPR) * 8;
  u32x4 x[NIT], y[NIT], z[NIT];
  int row[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    row[it] = (blockIdx.x * NIT + it) * RP + tid / LPR;
    const int64_t off = base + (int64_t)min(row[it], a.N - 1) * a.sn + col;   // rows past the end: clamped, not stored
    x[it] = *(const u32x4*)(a.o + off);
    y[it] = *(const u32x4*)(a.d_o + off);
    z[it] = u32x4{0, 0, 0, 0};
  }
  if (a.o_res) {
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      z[it] = *(const u32x4*)(a.o_res + base + (int64_t)min(row[it], a.N - 1) * a.sn + col);
  }
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float o0 = __builtin_bit_cast(float, x[it][e] << 16) + __builtin_bit_cast(float, z[it][e] << 16);
      const float o1 = __builtin_bit_cast(float, x[it][e] & 0xffff0000u) + __builtin_bit_cast(float, z[it][e] & 0xffff0000u);
      s = fmaf(o0, __builtin_bit_cast(float, y[it][e] << 16), s);
      s = fmaf(o1, __builtin_bit_cast(float, y[it][e] & 0xffff0000u), s);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (row[it] < a.N && (tid % LPR) == 0) a.delta[(int64_t)bh * a.N + row[it]] = s;
  }
}

hipError_t launch_bwd_delta(const void* o, const void* o_res, const void* d_o, const Dims& m, float* delta,
                            hipStream_t stream) {
  DeltaArgs a;
  a.o = (const uint16_t*)o; a.o_res = (const uint16_t*)o_res; a.d_o = (const uint16_t*)d_o; a.delta = delta;
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
  const int32_t* row_cnt; const int32_t* row_idx; const int32_t* row_order;
  int H, N, Tm, Tn, chunk;
  int64_t sb, sh, sn;
  float scale, scale_log2;
  SplitPlan sp;         // long rows cut into parts (split.hip); sp.pool_slots == 0: every row is walked whole
};

// Partial result of one part of a split row: the fp32 accumulator of every thread of the workgroup.
template <int D> constexpr int dq_slot_floats() { return 256 * (D / 2); }
size_t dq_slot_bytes(const Dims& m) { return (size_t)(m.d == 128 ? dq_slot_floats<128>() : dq_slot_floats<64>()) * 4; }

// dQ = acc * scale -> bf16; a lane owns one query row, accumulator register v of block mb is channel
// 32 mb + 8 (v / 4) + 4 hf + v % 4.
template <int D>
__device__ __forceinline__ void dq_store_rows(const DqArgs& a, int64_t base, int qrow, int hf, const f32x16 (&acc)[D / 32]) {
  if (qrow < a.N) {
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

template <int D>
struct DqCfg {
  // K and V tiles, XOR-swizzled and unpadded (the layout a direct global -> LDS copy can write): K is read
  // along rows (S^T) and transposed (dQ^T), V along rows (dP^T)
  static constexpr int K_ELEMS = BKV * D;
  static constexpr int V_ELEMS = BKV * D;
  static constexpr int CH = BKV * D / 8 / 256;
};

// Transposed formulation, a lane owns one query row (see fwd.hip):
//   S^T  = K_j Q_i^T        P^T  = exp(S^T - LSE)
//   dP^T = V_j dO_i^T       dS^T = P^T * (dP^T - D)
//   dQ^T += K_j^T dS^T      (K^T through transposing LDS reads)
template <int D>
__global__ __launch_bounds__(256, 2) void dq_kernel(DqArgs a) {
  using C = DqCfg<D>;
  __shared__ __align__(16) uint16_t smem[2 * (C::K_ELEMS + C::V_ELEMS)];   // stage s: K tile, then V tile
  constexpr int STAGE = C::K_ELEMS + C::V_ELEMS;

  // Which row, and which part of its list (see fwd.hip: the first sp.pool_slots workgroups are the extra parts)
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
    i = a.row_order ? min(max(a.row_order[(int64_t)bh * a.Tm + hb.blk], 0), a.Tm - 1) : hb.blk;
    if (a.sp.pool_slots) slot = a.sp.unit_slot[(int64_t)bh * a.Tm + i];
  }
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r32 = lane & 31, hf = lane >> 5;
  const int N = a.N;
  int cnt = min(max(a.row_cnt[(int64_t)bh * a.Tm + i], 0), a.Tn);   // clamped: see fwd.hip
  const int32_t* idx = a.row_idx + ((int64_t)bh * a.Tm + i) * a.Tn;
  if (slot >= 0) {            // entries [part * S, (part + 1) * S) of the list
    const int S = a.sp.header[1];
    idx += part * S;
    cnt = min(cnt - part * S, S);
  }
  const int qrow = i * BQ + w * 32 + r32;

  if (cnt == 0) {
    if (qrow < N) {
      uint16_t* op = a.dq + base + (int64_t)qrow * a.sn + (D / 2) * hf;
#pragma unroll
      for (int c = 0; c < D / 16; ++c) *(u32x4*)(op + 8 * c) = u32x4{0, 0, 0, 0};
    }
    return;
  }

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

  // K/V tiles are copied global -> LDS directly (no staging registers).  The destination of a wave-wide
  // 16-byte-per-lane copy is linear (wave base + 16 * lane), so the swizzle is applied on the source side: the
  // lane that fills chunk position pc of a row fetches logical chunk pc ^ swz(row).  Thread t fills chunk
  // position t % CPR of rows t / CPR + r * RSTEP; RSTEP is a multiple of 16 rows, so the swizzle term is the
  // same for every r.  Rows past N (short last block) are clamped to the last token: their P is zero.
  constexpr int CPR = D / 8, RSTEP = 256 / CPR;
  const int ld_row = tid / CPR;
  int ld_c8 = ((tid % CPR) ^ swz<D>(ld_row)) * 8;
  auto copy_piece = [&](int p, int buf, const char* kp, const char* vp, int last) {   // p in [0, 2 CH)
    const int r = p >> 1;
    const uint32_t off = (uint32_t)((min(ld_row + RSTEP * r, last) * a.sn + ld_c8) * 2);
    const uint16_t* dst = smem + buf * STAGE + (p & 1) * C::K_ELEMS + (r * 256 + w * 64) * 8;   // wave-uniform
    raw_copy16_to_lds((p & 1) ? vp : kp, off, dst);
  };
  constexpr int NPIECE = 2 * C::CH;

  f32x16 acc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;

  // per-lane LDS element offsets.  K row reads: row 32kb + r32, logical chunk 2kk + hf; the part of the
  // chunk index that depends on kk is XORed in as (kk << 4).
  int ka_base = swz_idx<D>(r32, 8 * hf);       // the V row reads use the same offsets
  // K transposing reads: rows (16-row group) + 8*which + 4hf + (s16>>2), columns 32mb + 16hb + 4(s16&3);
  // the part that depends on mb is XORed in as (mb << 5)
  const int s16 = lane & 15, hb16 = (lane >> 4) & 1;
  int kt_base0 = swz_idx<D>(4 * hf + (s16 >> 2), 16 * hb16 + 4 * (s16 & 3));
  int kt_base1 = swz_idx<D>(8 + 4 * hf + (s16 >> 2), 16 * hb16 + 4 * (s16 & 3));

  // The copies of tile t+1 are handed out between the MFMAs of the S^T / dP^T products of iteration t: issued
  // back to back they keep the wave at the issue stage until the texture unit has taken the last one.  They are
  // unconditional (past the end of the list the last tile is requested again, into the buffer nobody reads).
  // the index list, 64 entries at a time in one register (lane l holds entry 64c + l): reading an entry is
  // a lane read, not a memory access whose result the loop would have to wait for
  int idx_v = idx[min(lane, cnt - 1)];
  auto list_entry = [&](int t) -> int {      // t uniform, inside the chunk that idx_v holds
    return min(max(__builtin_amdgcn_readlane(idx_v, t & 63), 0), a.Tn - 1);
  };
  int j_cur = list_entry(0);
  {
    const int64_t tile0 = (base + (int64_t)j_cur * BKV * a.sn) * 2;
    const int last0 = min(BKV - 1, N - 1 - j_cur * BKV);
#pragma unroll
    for (int p = 0; p < NPIECE; ++p) copy_piece(p, 0, (const char*)a.k + tile0, (const char*)a.v + tile0, last0);
  }
  raw_copies_done();
  __syncthreads();

  for (int t = 0; t < cnt; ++t) {
    const int j = j_cur;
    if (((t + 1) & 63) == 0 && t + 1 < cnt) idx_v = idx[min(t + 1 + lane, cnt - 1)];     // next 64 entries
    const int j_nxt = list_entry(min(t + 1, cnt - 1));
    const int64_t tile_n = (base + (int64_t)j_nxt * BKV * a.sn) * 2;      // uniform
    const char* kpn = (const char*)a.k + tile_n;
    const char* vpn = (const char*)a.v + tile_n;
    const int last_n = min(BKV - 1, N - 1 - j_nxt * BKV);
    j_cur = j_nxt;
    const uint16_t* Kb = smem + (t & 1) * STAGE;
    const uint16_t* Vb = Kb + C::K_ELEMS;

    // keep the XORed operand addresses out of loop-invariant hoisting (one VALU op per read instead of
    // a dozen live registers)
    asm volatile("" : "+v"(ka_base), "+v"(kt_base0), "+v"(kt_base1), "+v"(ld_c8));

    // ---- S^T and dP^T: for each 32-key block D/16 MFMAs of K Q^T, then D/16 of V dO^T.  LDS operands run
    // PDQ MFMAs ahead of their use; request piece p of tile t+1 goes out after MFMA p * NM1 / NPIECE.
    constexpr int NM1 = 4 * (D / 16), PDQ = 4;
    auto frag1 = [&](int y) -> bf16x8 {
      const int kb = y / (2 * (D / 16)), rem = y % (2 * (D / 16)), kk = rem % (D / 16);
      return *(const bf16x8*)((rem < D / 16 ? Kb : Vb) + (ka_base ^ (kk << 4)) + kb * 32 * D);
    };
    f32x16 s[2], dp[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[kb][v] = 0.f; dp[kb][v] = 0.f; }
    {
      bf16x8 fr[PDQ];
#pragma unroll
      for (int x = 0; x < PDQ; ++x) fr[x] = frag1(x);
#pragma unroll
      for (int y = 0; y < NM1; ++y) {
        const int kb = y / (2 * (D / 16)), rem = y % (2 * (D / 16)), kk = rem % (D / 16);
        if (rem < D / 16) s[kb] = mfma32(fr[y % PDQ], qf[kk], s[kb]);
        else              dp[kb] = mfma32(fr[y % PDQ], dof[kk], dp[kb]);
        if (y + PDQ < NM1) fr[y % PDQ] = frag1(y + PDQ);
        if (y % (NM1 / NPIECE) == 0) copy_piece(y / (NM1 / NPIECE), (t + 1) & 1, kpn, vpn, last_n);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // first K^T operands of the dQ^T product are requested now, so that they arrive during the dS arithmetic
    constexpr int NM2 = 4 * (D / 32);
    auto frag2 = [&](int y) -> bf16x8 {
      const int kb = y / (2 * (D / 32)), cc = (y / (D / 32)) % 2, mb = y % (D / 32);
      const uint16_t* krow = Kb + (32 * kb + 16 * cc) * D;
      return join_tr(lds_read_tr4(krow + (kt_base0 ^ (mb << 5))), lds_read_tr4(krow + (kt_base1 ^ (mb << 5))));
    };
    bf16x8 f2[PDQ];
#pragma unroll
    for (int x = 0; x < PDQ; ++x) f2[x] = frag2(x);
    __builtin_amdgcn_sched_barrier(0);
    const bool tail = (j + 1) * BKV > N;
    uint32_t dsk[2][8];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        float ds2[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int v = 2 * u + e;
          float p = fast_exp2(fmaf(s[kb][v], a.scale_log2, -lse2));
          if (tail) {
            const int key = j * BKV + kb * 32 + 8 * (v >> 2) + 4 * hf + (v & 3);
            if (key >= N) p = 0.f;
          }
          ds2[e] = p * (dp[kb][v] - dlt);     // dS^T
        }
        dsk[kb][u] = pack_bf16(ds2[0], ds2[1]);
      }
    __builtin_amdgcn_sched_barrier(0);
    // ---- dQ^T += K^T dS^T
#pragma unroll
    for (int y = 0; y < NM2; ++y) {
      const int kb = y / (2 * (D / 32)), cc = (y / (D / 32)) % 2, mb = y % (D / 32);
      const u32x4 du = {dsk[kb][4 * cc], dsk[kb][4 * cc + 1], dsk[kb][4 * cc + 2], dsk[kb][4 * cc + 3]};
      acc[mb] = mfma32(f2[y % PDQ], __builtin_bit_cast(bf16x8, du), acc[mb]);
      if (y + PDQ < NM2) f2[y % PDQ] = frag2(y + PDQ);
      __builtin_amdgcn_sched_barrier(0);
    }
    raw_copies_done();    // the copies requested in this iteration have landed
    __syncthreads();
  }

  if (slot >= 0) {            // one part of a split row: leave the partial sum to the merge kernel
    f32x4* pa = (f32x4*)(a.sp.pool + (int64_t)slot * a.sp.slot_floats + tid * (D / 2));
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        pa[mb * 4 + g] = f32x4{acc[mb][4 * g], acc[mb][4 * g + 1], acc[mb][4 * g + 2], acc[mb][4 * g + 3]};
    return;
  }
  dq_store_rows<D>(a, base, qrow, hf, acc);
}

// Adds the parts of every split row in part order (fixed order: deterministic).  Same thread -> (row, channel)
// mapping as dq_kernel; workgroup x takes split row x of the plan.
template <int D>
__device__ __forceinline__ void dq_merge_kernel_one(const DqArgs& a, int m_idx) {
  const int unit = a.sp.merge_table[m_idx];
  const int bh = unit / a.Tm, i = unit % a.Tm;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int cnt = min(max(a.row_cnt[unit], 0), a.Tn);
  const int S = a.sp.header[1];
  const int parts = (cnt + S - 1) / S;
  const float* p0 = a.sp.pool + (int64_t)a.sp.unit_slot[unit] * a.sp.slot_floats + tid * (D / 2);
  f32x16 acc[D / 32];
#pragma unroll
  for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;
  // two parts per step: the loads of both are in flight together; the order of addition stays part 0, 1, 2, ...
  for (int p = 0; p < parts; p += 2) {
    const bool two = p + 1 < parts;
    const f32x4* pa0 = (const f32x4*)(p0 + (int64_t)p * a.sp.slot_floats);
    const f32x4* pa1 = (const f32x4*)(p0 + (int64_t)(two ? p + 1 : p) * a.sp.slot_floats);
    f32x4 x0[D / 8], x1[D / 8];
#pragma unroll
    for (int c = 0; c < D / 8; ++c) { x0[c] = pa0[c]; x1[c] = pa1[c]; }
#pragma unroll
    for (int mb = 0; mb < D / 32; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc[mb][4 * g + e] += x0[mb * 4 + g][e];
          if (two) acc[mb][4 * g + e] += x1[mb * 4 + g][e];
        }
  }
  dq_store_rows<D>(a, base, i * BQ + w * 32 + (lane & 31), lane >> 5, acc);
}

// (one workgroup per split list as a rule; the loop covers a launch with fewer workgroups than lists)
template <int D>
__global__ __launch_bounds__(256) void dq_merge_kernel(DqArgs a) {
  const int n = a.sp.header[2];
  for (int m_idx = blockIdx.x; m_idx < n; m_idx += gridDim.x) dq_merge_kernel_one<D>(a, m_idx);
}

hipError_t launch_bwd_dq(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                         const float* delta, const Dims& m, const int32_t* row_cnt, const int32_t* row_idx,
                         const int32_t* row_order, float scale, void* dq, const SplitPlan& plan, hipStream_t stream) {
  DqArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.lse = lse; a.delta = delta; a.dq = (uint16_t*)dq;
  a.row_cnt = row_cnt; a.row_idx = row_idx; a.row_order = row_order;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn; a.chunk = (m.Tm + 7) / 8;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  a.scale = scale; a.scale_log2 = scale * LOG2E;
  a.sp = plan;
  if (plan.pool_slots) {
    const hipError_t e = launch_split_plan(row_cnt, (int64_t)m.B * m.H * m.Tm, m.Tn, SPLIT_MIN_PART, plan, stream);
    if (e != hipSuccess) return e;
  }
  const dim3 grid((unsigned)(plan.pool_slots + m.B * m.H * 8 * a.chunk)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(dq_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(dq_kernel<64>, grid, block, 0, stream, a);
  if (plan.pool_slots) {
    const dim3 mg((unsigned)(plan.pool_slots / 2));
    if (m.d == 128) hipLaunchKernelGGL(dq_merge_kernel<128>, mg, block, 0, stream, a);
    else            hipLaunchKernelGGL(dq_merge_kernel<64>, mg, block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace spa2
