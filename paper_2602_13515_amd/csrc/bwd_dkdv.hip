// Block-sparse attention backward, key-block side: dK and dV (see bwd.hip for the formulas and the other two
// kernels).  This file is compiled with -mllvm -amdgpu-mfma-vgpr-form: the S / dP products then leave their
// results in ordinary vector registers, where the exp / dS arithmetic reads them directly, while the dK / dV
// accumulators are pinned to the accumulation registers through mfma32_acc below.
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

// C += A B with C held in accumulation registers (the compiler allocates them there and never moves them).
// The compiler does not know that this is a matrix instruction and adds no wait states around it, so they are
// written here: an operand register that a vector ALU instruction has just written must not be read by the very
// next instruction (measured: one wait state is enough; two are kept).
__device__ __forceinline__ void mfma32_acc(bf16x8 a, bf16x8 b, f32x16& c) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
#endif
}

// ------------------------------------------------------------------ dK, dV
struct DkvArgs {
  const uint16_t* q; const uint16_t* k; const uint16_t* v; const uint16_t* d_o;
  const float* lse; const float* delta; uint16_t* dk; uint16_t* dv;
  const int32_t* col_cnt; const int32_t* col_idx; const int32_t* col_order;
  int H, N, Tm, Tn, chunk;
  int64_t sb, sh, sn;
  float scale, scale_log2;
  SplitPlan sp;         // long columns cut into parts (split.hip); sp.pool_slots == 0: every column is walked whole
};

// Partial result of one part of a split column: the fp32 sums of the two waves, dK^T then dV^T, in the order
// [tensor][finishing wave][output block][group of four registers][lane][register in the group].
template <int D> constexpr int dkdv_slot_floats() { return 2 * 2 * (D / 32) * 16 * 64; }
size_t dkdv_slot_bytes(const Dims& m) { return (size_t)(m.d == 128 ? dkdv_slot_floats<128>() : dkdv_slot_floats<64>()) * 4; }

// One workgroup of two waves per key block j (64 keys); one wave per SIMD (512 registers), four waves per CU.
// The query blocks that selected j are taken in halves of 64 rows; wave w owns the 32 queries 32w.. of the half
// and ALL 64 keys of the block.  It keeps K_j^T, V_j^T (B operands) and its dK^T, dV^T accumulators (d x 64
// keys each) in registers for the whole column, so every operand fragment that comes from LDS feeds two MFMAs
// (one per 32-key half), and a wave only ever reads its own 32 rows of Q and dO:
//   S  (q x keys) = Q_i K_j^T        A = Q rows from LDS,  B = K^T fragments (registers)
//   dP (q x keys) = dO_i V_j^T       A = dO rows from LDS, B = V^T fragments (registers)
//   P = exp(S - LSE), dS = P * (dP - D)      accumulator layout: lane = key, registers = queries
//   dV^T (d x keys) += dO_i^T P      A = dO^T through transposing LDS reads, B = P  (registers)
//   dK^T (d x keys) += Q_i^T dS      A = Q^T  through transposing LDS reads, B = dS (registers)
// Because no wave reads another wave's rows, each wave stages its own rows (global -> LDS directly, XOR-swizzled,
// double-buffered one step ahead) and waits only for its own copies: there is no workgroup barrier in the loop.
// With a single wave per SIMD the vector arithmetic has to hide behind that wave's own MFMAs: the order is
// S products, then dP products with exp(S - LSE) between them, dS of the first 16 queries, then the dV / dK
// products of those 16 queries with the dS arithmetic of the other 16 between them.
// The two waves add their partial sums through LDS at the end of the column.
template <int D>
__global__ __attribute__((amdgpu_flat_work_group_size(128, 128), amdgpu_waves_per_eu(1, 1)))
void dkdv_kernel(DkvArgs a) {
  constexpr int QW = 32;                             // query rows per wave and step
  constexpr int HQ = 64;                             // query rows per workgroup and step
  constexpr int NK = D / 16;                         // 16-wide contraction steps over the head dimension
  constexpr int NMB = D / 32;                        // 32-channel output blocks
  constexpr int CPR = D / 8;                         // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;                      // rows that one wave-wide copy instruction covers
  constexpr int NCP = QW / RPI;                      // copy instructions per tensor and step
  constexpr int NOFF = 16 / RPI;                     // the swizzle repeats every 16 rows: distinct lane offsets
  constexpr int TILE_B = QW * D * 2;                 // bytes of one wave's 32-row tile
  constexpr int STAGE_B = 2 * TILE_B;                // Q rows, then dO rows
  constexpr int STAT_B = 512;                        // LSE of the 32 rows at +0, D at +256
  __shared__ __align__(1024) unsigned char smem[2 * 2 * STAGE_B];   // (aligned: compile-time parts are XORed into addresses)   // wave w, stage s at (2w + s) * STAGE_B
  __shared__ __align__(1024) unsigned char stat_s[2 * 2 * STAT_B];  // wave w, stage s
  // The registers hold 512 values per lane: 256 accumulators, 128 for K^T / V^T, 64 for S / dP, and what is left
  // does not quite hold the operand rings, the packed P / dS and the addresses.  The last VL fragments of V^T
  // (key half 1) therefore live in LDS in fragment order (lane l's 16 bytes at 16 l: conflict-free) and are read
  // just before their product, like the Q / dO fragments.
#ifndef DKDV_VL
#define DKDV_VL 0
#endif
  constexpr int VL = D == 128 ? DKDV_VL : 0;    // fragment f = kh * NK + kk of V^T is in LDS when f >= 2 NK - VL
  __shared__ __align__(1024) unsigned char vfrag_s[(VL ? VL : 1) * 1024];

  // Which key block, and which part of its list (the first sp.pool_slots workgroups of the launch are the extra
  // parts of split columns, part >= 1; the others take one key block each: the whole list, or part 0)
  int bh, j, part = 0, slot = -1;
  if ((int)blockIdx.x < a.sp.pool_slots) {
    if ((int)blockIdx.x >= a.sp.header[0]) return;
    const int unit = a.sp.part_table[2 * blockIdx.x];
    part = a.sp.part_table[2 * blockIdx.x + 1];
    bh = unit / a.Tn; j = unit % a.Tn;
    slot = a.sp.unit_slot[unit] + part;
  } else {
    const HeadBlock hbk = xcd_map(blockIdx.x - a.sp.pool_slots, a.Tn, a.chunk);
    if (!hbk.valid) return;
    bh = hbk.bh;
    j = a.col_order ? min(max(a.col_order[(int64_t)bh * a.Tn + hbk.blk], 0), a.Tn - 1) : hbk.blk;
    if (a.sp.pool_slots) slot = a.sp.unit_slot[(int64_t)bh * a.Tn + j];
  }
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform, in a scalar register
  const int r32 = lane & 31, hf = lane >> 5;
  const int N = a.N;
  int cnt = min(max(a.col_cnt[(int64_t)bh * a.Tn + j], 0), a.Tm);   // clamped: see fwd.hip
  const int32_t* idx = a.col_idx + ((int64_t)bh * a.Tn + j) * a.Tm;
  if (slot >= 0) {            // entries [part * S, (part + 1) * S) of the list
    const int S = a.sp.header[1];
    idx += part * S;
    cnt = min(cnt - part * S, S);
  }

  const int key0 = j * BKV + r32;                    // this lane's key of half 0; half 1 is 32 further
  const bool keys_short = (j + 1) * BKV > N;         // uniform: the block reaches past the last token

  if (cnt == 0) {   // no query block selected this key block: zero gradients (wave w writes key half w)
    const int key = key0 + 32 * w;
    if (key < N) {
      const int64_t out_off = base + (int64_t)key * a.sn + 4 * hf;
#pragma unroll
      for (int c = 0; c < D / 8; ++c) {
        *(u32x2*)(a.dk + out_off + 8 * c) = u32x2{0, 0};
        *(u32x2*)(a.dv + out_off + 8 * c) = u32x2{0, 0};
      }
    }
    return;
  }

  const uint32_t vfrag_addr = lds_addr_of(vfrag_s) + 16 * lane;
  // K^T / V^T fragments (B operands): lane = key, 8 consecutive channels per 16-wide k step
  bf16x8 kf[2][NK], vf[2][NK];
#pragma unroll
  for (int kh = 0; kh < 2; ++kh) {
    const int key = min(key0 + 32 * kh, N - 1);
    const int64_t off = base + (int64_t)key * a.sn + 8 * hf;
#pragma unroll
    for (int kk = 0; kk < NK; ++kk) {
      kf[kh][kk] = *(const bf16x8*)(a.k + off + 16 * kk);
      if (kh * NK + kk < 2 * NK - VL) vf[kh][kk] = *(const bf16x8*)(a.v + off + 16 * kk);
      else if (w == 0) *(bf16x8*)(vfrag_s + (kh * NK + kk - (2 * NK - VL)) * 1024 + 16 * lane) = *(const bf16x8*)(a.v + off + 16 * kk);
    }
  }
  if (VL) __syncthreads();

  f32x16 dk_acc[2][NMB], dv_acc[2][NMB];
#pragma unroll
  for (int kh = 0; kh < 2; ++kh)
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
      for (int v = 0; v < 16; ++v) { dk_acc[kh][mb][v] = 0.f; dv_acc[kh][mb][v] = 0.f; }

  // global -> LDS copies of this wave's 32 rows.  A wave-wide 16-byte-per-lane copy lands linearly (wave base +
  // 16 * lane), i.e. lane l fills chunk position l % CPR of row RPI * r + l / CPR for copy instruction r; the
  // swizzle is applied on the source side (the lane fetches logical chunk position ^ swz(row)).  swz repeats every
  // 16 rows, so NOFF lane offsets cover all instructions; everything else of a request is wave-uniform: four
  // 64-bit bases per step (Q and dO, rows 0.. and 16..) and compile-time LDS offsets.
  uint32_t loff[NOFF];
#pragma unroll
  for (int b = 0; b < NOFF; ++b) {
    const int row_l = RPI * b + lane / CPR;
    loff[b] = (uint32_t)((row_l * a.sn + (((lane % CPR) ^ swz<D>(row_l)) * 8)) * 2);
  }
  const uint32_t soff = (uint32_t)(r32 * 4);
  const char* q_head = (const char*)(a.q + base);
  const char* o_head = (const char*)(a.d_o + base);
  const char* lse_head = (const char*)(a.lse + (int64_t)bh * N);
  const char* dlt_head = (const char*)(a.delta + (int64_t)bh * N);
  const uint64_t row_bytes = (uint64_t)a.sn * 2;
  const uint32_t wsm = lds_addr_of(smem) + 2 * w * STAGE_B;       // uniform LDS byte addresses
  const uint32_t wstat = lds_addr_of(stat_s) + 2 * w * STAT_B;

  // the same for 32 rows that reach past N: rows are clamped to the last token (their P is zeroed below)
  auto request_ragged = [&](int row0, uint32_t stage_addr, uint32_t stat_addr) {
#pragma unroll
    for (int r = 0; r < NCP; ++r) {
      const int first = min(row0 + RPI * r, N - 1);                       // uniform
      const int row_l = lane / CPR;
      const int sw_row = RPI * r + row_l;                                 // the row of the LDS tile being filled
      const uint32_t off = (uint32_t)((min(row_l, N - 1 - first) * a.sn + (((lane % CPR) ^ swz<D>(sw_row)) * 8)) * 2);
      raw_copy16_to_lds_at<0>(q_head + (uint64_t)first * row_bytes, off, stage_addr + r * 1024);
      raw_copy16_to_lds_at<0>(o_head + (uint64_t)first * row_bytes, off, stage_addr + TILE_B + r * 1024);
    }
    const int first = min(row0, N - 1);
    const uint32_t so = (uint32_t)(min(r32, N - 1 - first) * 4);
    raw_copy4_to_lds_at<0>(lse_head + (uint64_t)first * 4, so, stat_addr);
    raw_copy4_to_lds_at<256>(dlt_head + (uint64_t)first * 4, so, stat_addr);
  };

  // the index list, 64 entries at a time in one register (lane l holds entry 64c + l): reading entry t is a
  // lane read, not a memory access
  int idx_v = idx[min(lane, cnt - 1)];
  auto list_entry = [&](int t) -> int {      // t uniform, inside the chunk that idx_v holds
    return min(max(__builtin_amdgcn_readlane(idx_v, t & 63), 0), a.Tm - 1);
  };

  // per-lane LDS byte offsets inside a 32-row tile.  Row reads: row r32, logical chunk 2kk + hf (the part that
  // depends on kk is XORed in as kk << 5).  Transposing reads: row 16c + 8*which + 4hf + (s16>>2), columns
  // 32mb + 16hb + 4(s16&3) (the part that depends on mb is XORed in as mb << 6).
  const int s16 = lane & 15, hb16 = (lane >> 4) & 1;
  const uint32_t a_off = 2 * swz_idx<D>(r32, 8 * hf);
  const uint32_t t_off0 = 2 * swz_idx<D>(4 * hf + (s16 >> 2), 16 * hb16 + 4 * (s16 & 3));
  const uint32_t t_off1 = 2 * swz_idx<D>(8 + 4 * hf + (s16 >> 2), 16 * hb16 + 4 * (s16 & 3));

  const int steps = 2 * cnt;                 // step u: half u & 1 of list entry u >> 1
  {
    const int row0 = list_entry(0) * BQ + QW * w;
    request_ragged(row0, wsm, wstat);        // (the general form; the loop uses the cheaper one for full tiles)
  }
  raw_copies_done();

  constexpr int PD = 4;                      // how many operand fragments ahead an LDS read is issued
  for (int u = 0; u < steps; ++u) {
    const int st = u & 1;
    const int row_cur = list_entry(u >> 1) * BQ + (u & 1) * HQ + QW * w;
    const int un = min(u + 1, steps - 1);    // past the end the last step is requested again (nobody reads it)
    if (((u + 1) & 127) == 0 && u + 1 < steps) idx_v = idx[min(((u + 1) >> 1) + lane, cnt - 1)];   // next 64 entries
    const int row_nx = list_entry(un >> 1) * BQ + (un & 1) * HQ + QW * w;
    const bool piecewise = row_nx + QW <= N;
    const uint32_t nx_stage = wsm + (st ^ 1) * STAGE_B, nx_stat = wstat + (st ^ 1) * STAT_B;
    // uniform bases of the next step's request
    const char* qn0 = q_head + (uint64_t)row_nx * row_bytes;
    const char* on0 = o_head + (uint64_t)row_nx * row_bytes;
    const char* qn1 = qn0 + 16 * row_bytes;
    const char* on1 = on0 + 16 * row_bytes;
    if (!piecewise) {
      request_ragged(row_nx, nx_stage, nx_stat);
    } else {
      raw_copy4_to_lds_at<0>(lse_head + (uint64_t)row_nx * 4, soff, nx_stat);
      raw_copy4_to_lds_at<256>(dlt_head + (uint64_t)row_nx * 4, soff, nx_stat);
    }
    // piece P of the request for 32 full rows: Q chunk rows, dO chunk rows alternately
    auto request_piece = [&](auto P) {
      constexpr int p = decltype(P)::v, r = p >> 1, aa = r / NOFF, b = r % NOFF;
      const char* src = (p & 1) ? (aa ? on1 : on0) : (aa ? qn1 : qn0);
      raw_copy16_to_lds_at<(p & 1) * TILE_B + r * 1024>(src, loff[b], nx_stage);
    };
    // this step's operand addresses (one add per step; the XOR of the compile-time part is one more op per read)
    const uint32_t q_rd = wsm + st * STAGE_B + a_off, q_t0 = wsm + st * STAGE_B + t_off0, q_t1 = wsm + st * STAGE_B + t_off1;
    const uint32_t lb = wstat + st * STAT_B + 16 * hf;

    // ---- S = Q K^T, then dP = dO V^T; fragment y of the sequence is Q chunk y (y < NK) or dO chunk y - NK
    auto row_frag = [&](int y) -> bf16x8 { return lds_ld16((q_rd ^ ((y % NK) << 5)) + (y < NK ? 0 : TILE_B)); };
    f32x16 s[2], dp[2];
    bf16x8 fr[PD];
#pragma unroll
    for (int x = 0; x < PD; ++x) fr[x] = row_frag(x);
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    static_for<0, NK>([&](auto Y) {
      constexpr int y = decltype(Y)::v;
      s[0] = mfma32(fr[y % PD], kf[0][y], y == 0 ? zero : s[0]);
      s[1] = mfma32(fr[y % PD], kf[1][y], y == 0 ? zero : s[1]);
      fr[y % PD] = row_frag(y + PD);
      if (piecewise) {
        constexpr int PER = (2 * NCP) / NK;
        static_for<0, PER>([&](auto C) { request_piece(Int<y * PER + decltype(C)::v>{}); });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // exp(S - LSE) in groups of four queries (accumulator registers 4g .. 4g+3), between the dP products
    constexpr int GPS = 8 / NK;                // (key half, query group) pairs handled per dP step
    f32x4 l4;
    auto v_frag = [&](int kh, int kk) -> bf16x8 {     // from registers or, for the last VL fragments, from LDS
      const int f = kh * NK + kk;
      return f < 2 * NK - VL ? vf[kh][kk] : lds_ld16(vfrag_addr + (f - (2 * NK - VL)) * 1024);
    };
    static_for<NK, 2 * NK>([&](auto Y) {
      constexpr int y = decltype(Y)::v, kk = y - NK;
      dp[0] = mfma32(fr[y % PD], v_frag(0, kk), kk == 0 ? zero : dp[0]);
      dp[1] = mfma32(fr[y % PD], v_frag(1, kk), kk == 0 ? zero : dp[1]);
      if constexpr (y + PD < 2 * NK) fr[y % PD] = row_frag(y + PD);
#pragma unroll
      for (int x = 0; x < GPS; ++x) {
        const int pair = kk * GPS + x, g = pair >> 1, kh = pair & 1;
        if (kh == 0) l4 = lds_ldf4(lb + 32 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          s[kh][4 * g + e] = fast_exp2(fmaf(s[kh][4 * g + e], a.scale_log2, -LOG2E * l4[e]));
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // keys past N (short last key block) and query rows past N (short last query block): P = 0
    if (keys_short) {
#pragma unroll
      for (int kh = 0; kh < 2; ++kh)
        if (key0 + 32 * kh >= N) {
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kh][v] = 0.f;
        }
    }
    if (row_cur + QW > N) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (row_cur + 8 * (v >> 2) + 4 * hf + (v & 3) >= N) { s[0][v] = 0.f; s[1][v] = 0.f; }
    }
    // ---- dS = P * (dP - D), P and dS packed to bf16: pk[kh][2g], pk[kh][2g+1] hold the four queries of group g
    uint32_t pk[2][8], dsk[2][8];
    auto finish_group = [&](int g, int kh) {
      const f32x4 d4 = lds_ldf4(lb + 256 + 32 * g);
      float ds[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) ds[e] = s[kh][4 * g + e] * (dp[kh][4 * g + e] - d4[e]);
      pk[kh][2 * g] = pack_bf16(s[kh][4 * g], s[kh][4 * g + 1]);
      pk[kh][2 * g + 1] = pack_bf16(s[kh][4 * g + 2], s[kh][4 * g + 3]);
      dsk[kh][2 * g] = pack_bf16(ds[0], ds[1]);
      dsk[kh][2 * g + 1] = pack_bf16(ds[2], ds[3]);
    };
    auto tr_frag = [&](int tile, int x) -> bf16x8 {     // tile 0 = Q, 1 = dO; x = c * NMB + mb
      const int c = x / NMB, mb = x % NMB;
      const uint32_t o = tile * TILE_B + 32 * c * D;
      return join_tr(lds_tr4_at((q_t0 ^ (mb << 6)) + o), lds_tr4_at((q_t1 ^ (mb << 6)) + o));
    };
    constexpr int NX = 2 * NMB, PDT = 2;
    bf16x8 fo[PDT], fq[PDT];
    finish_group(0, 0); finish_group(0, 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int x = 0; x < PDT; ++x) { fo[x] = tr_frag(1, x); fq[x] = tr_frag(0, x); }
    finish_group(1, 0); finish_group(1, 1);
    __builtin_amdgcn_sched_barrier(0);
    // ---- dV^T += dO^T P and dK^T += Q^T dS.  Step x = (c, mb): the 16 queries 16c.. (accumulator registers
    // 8c .. 8c+7), output block mb; each transposed fragment feeds both key halves.  The dS arithmetic of the
    // second 16 queries runs between the products of the first 16.
#pragma unroll
    for (int x = 0; x < NX; ++x) {
      const int c = x / NMB, mb = x % NMB;
      const u32x4 p0 = {pk[0][4 * c], pk[0][4 * c + 1], pk[0][4 * c + 2], pk[0][4 * c + 3]};
      const u32x4 p1 = {pk[1][4 * c], pk[1][4 * c + 1], pk[1][4 * c + 2], pk[1][4 * c + 3]};
      const u32x4 d0 = {dsk[0][4 * c], dsk[0][4 * c + 1], dsk[0][4 * c + 2], dsk[0][4 * c + 3]};
      const u32x4 d1 = {dsk[1][4 * c], dsk[1][4 * c + 1], dsk[1][4 * c + 2], dsk[1][4 * c + 3]};
      mfma32_acc(fo[x % PDT], __builtin_bit_cast(bf16x8, p0), dv_acc[0][mb]);
      mfma32_acc(fo[x % PDT], __builtin_bit_cast(bf16x8, p1), dv_acc[1][mb]);
      if (x + PDT < NX) fo[x % PDT] = tr_frag(1, x + PDT);
      mfma32_acc(fq[x % PDT], __builtin_bit_cast(bf16x8, d0), dk_acc[0][mb]);
      mfma32_acc(fq[x % PDT], __builtin_bit_cast(bf16x8, d1), dk_acc[1][mb]);
      if (x + PDT < NX) fq[x % PDT] = tr_frag(0, x + PDT);
      if (c == 0) {                             // groups 2, 3 of both key halves, spread over the NMB steps
        constexpr int PER = 4 / NMB;
#pragma unroll
        for (int t = 0; t < PER; ++t) finish_group(2 + ((mb * PER + t) >> 1), (mb * PER + t) & 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    raw_copies_done();      // the copies requested in this step have landed in the other stage
  }

  // the accumulators are read by ordinary vector instructions from here on: let the last products finish first
  // (the compiler does not know that mfma32_acc is a matrix instruction and inserts no wait states for it)
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#endif
  // sum the partial results of the two waves: first pass dK, second pass dV.  Wave w writes its partial
  // into its own staging area and then finishes key half w.
  float* scratch = (float*)smem;
  constexpr int REGION = 2 * NMB * 16 * 64;           // floats per wave
  static_assert(REGION * 4 == 2 * STAGE_B, "a wave's partial sums fill exactly its two stages");
  const int key = key0 + 32 * w;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    float* mine = scratch + w * REGION + lane;
#pragma unroll
    for (int kh = 0; kh < 2; ++kh)
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          mine[((kh * NMB + mb) * 16 + v) * 64] = round == 0 ? dk_acc[kh][mb][v] : dv_acc[kh][mb][v];
    __syncthreads();
    if (key < N || slot >= 0) {     // (a part writes its whole slot, so that the merge never reads stale sums)
      const int64_t out_off = base + (int64_t)key * a.sn + 4 * hf;
      const float sc = round == 0 ? a.scale : 1.f;
#pragma unroll
      for (int mb = 0; mb < NMB; ++mb) {
        uint16_t* out = (round == 0 ? a.dk : a.dv) + out_off + 32 * mb;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int at = ((w * NMB + mb) * 16 + 4 * g + e) * 64 + lane;
            x[e] = scratch[at] + scratch[REGION + at];
          }
          if (slot >= 0) {      // one part of a split column: leave the sums to the merge kernel
            float* ps = a.sp.pool + (int64_t)slot * a.sp.slot_floats + ((((round * 2 + w) * NMB + mb) * 4 + g) * 64 + lane) * 4;
            *(f32x4*)ps = f32x4{x[0], x[1], x[2], x[3]};
            continue;
          }
          u32x2 pk2 = {pack_bf16(x[0] * sc, x[1] * sc), pack_bf16(x[2] * sc, x[3] * sc)};
          *(u32x2*)(out + 8 * g) = pk2;
        }
      }
    }
    __syncthreads();
  }
}

// Adds the parts of every split column in part order (fixed order: deterministic) and stores dK, dV.  Same thread
// -> (key, channel) mapping as the end of dkdv_kernel; workgroup x takes split column x of the plan.
template <int D>
__device__ __forceinline__ void dkdv_merge_kernel_one(const DkvArgs& a, int m_idx) {
  constexpr int NMB = D / 32;
  const int unit = a.sp.merge_table[m_idx];
  const int bh = unit / a.Tn, j = unit % a.Tn;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, r32 = lane & 31, hf = lane >> 5;
  const int cnt = min(max(a.col_cnt[unit], 0), a.Tm);
  const int S = a.sp.header[1];
  const int parts = (cnt + S - 1) / S;
  const float* p0 = a.sp.pool + (int64_t)a.sp.unit_slot[unit] * a.sp.slot_floats;
  const int key = j * BKV + r32 + 32 * w;
  if (key >= a.N) return;
  const int64_t out_off = base + (int64_t)key * a.sn + 4 * hf;
  // all sums of this thread at once, part after part (the 16-byte loads of one part are in flight together)
  f32x4 x[2 * NMB * 4];
#pragma unroll
  for (int c = 0; c < 2 * NMB * 4; ++c) x[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < parts; ++p) {
    const f32x4* ps = (const f32x4*)(p0 + (int64_t)p * a.sp.slot_floats) + lane;
#pragma unroll
    for (int round = 0; round < 2; ++round)
#pragma unroll
      for (int c = 0; c < NMB * 4; ++c)
        x[round * NMB * 4 + c] += ps[((round * 2 + w) * NMB * 4 + c) * 64];
  }
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const float sc = round == 0 ? a.scale : 1.f;
#pragma unroll
    for (int mb = 0; mb < NMB; ++mb) {
      uint16_t* out = (round == 0 ? a.dk : a.dv) + out_off + 32 * mb;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 y = x[round * NMB * 4 + mb * 4 + g];
        u32x2 pk2 = {pack_bf16(y[0] * sc, y[1] * sc), pack_bf16(y[2] * sc, y[3] * sc)};
        *(u32x2*)(out + 8 * g) = pk2;
      }
    }
  }
}

// (one workgroup per split list as a rule; the loop covers a launch with fewer workgroups than lists)
template <int D>
__global__ __launch_bounds__(128) void dkdv_merge_kernel(DkvArgs a) {
  const int n = a.sp.header[2];
  for (int m_idx = blockIdx.x; m_idx < n; m_idx += gridDim.x) dkdv_merge_kernel_one<D>(a, m_idx);
}

hipError_t launch_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                           const float* delta, const Dims& m, const int32_t* col_cnt, const int32_t* col_idx,
                           const int32_t* col_order, float scale, void* dk, void* dv, const SplitPlan& plan,
                           hipStream_t stream) {
  DkvArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.d_o = (const uint16_t*)d_o;
  a.lse = lse; a.delta = delta; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv;
  a.col_cnt = col_cnt; a.col_idx = col_idx; a.col_order = col_order;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn; a.chunk = (m.Tn + 7) / 8;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  a.scale = scale; a.scale_log2 = scale * LOG2E;
  a.sp = plan;
  if (plan.pool_slots) {
    const hipError_t e = launch_split_plan(col_cnt, (int64_t)m.B * m.H * m.Tn, m.Tm, SPLIT_MIN_PART / 2, plan, stream);
    if (e != hipSuccess) return e;
  }
  const dim3 grid((unsigned)(plan.pool_slots + m.B * m.H * 8 * a.chunk)), block(128);
  if (m.d == 128) hipLaunchKernelGGL(dkdv_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(dkdv_kernel<64>, grid, block, 0, stream, a);
  if (plan.pool_slots) {
    const dim3 mg((unsigned)(plan.pool_slots / 2));
    if (m.d == 128) hipLaunchKernelGGL(dkdv_merge_kernel<128>, mg, block, 0, stream, a);
    else            hipLaunchKernelGGL(dkdv_merge_kernel<64>, mg, block, 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace spa2
