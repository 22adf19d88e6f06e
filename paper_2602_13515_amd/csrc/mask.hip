// Hybrid Top-k + Top-p block masker (Alg. 1 steps 2-6; Sec. 2.2, Sec. 4.1) for gfx950.
//
//   pool_kernel     mean of each 128-token query block and 64-token key block
//                   (Sec. 2.2 "pooled within each block"); the one pass over Q
//                   and K in HBM, everything after it works on the pooled data.
//   select_kernel   for a few rows of the pooled map at a time: scores
//                   Sbar = Qbar Kbar^T * scale, row softmax Pbar, ordering by
//                   (Pbar descending, block index ascending), cumulative sum in
//                   that order, n = max(1, k_cnt, n_p), mask row + ascending
//                   index list.  The row never leaves LDS/registers.
//   select16_kernel the same for rows of up to 1536 blocks, sixteen rows per workgroup, with the
//                   score product on the fp64 matrix cores.
//   columns_kernel  the same pattern listed per key block (for dK/dV).
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

// Which of the two selection kernels a shape gets (the pooled keys are laid out for it by the pooling pass):
// sixteen rows per workgroup with the scores on the fp64 matrix cores where a row has at most 1536 blocks (the scores
// of sixteen rows fit the registers) and the launch still has four workgroups per compute unit, else four rows per
// workgroup on the vector ALU.
static bool select16_applies(const Dims& m) {
  return m.Tn <= 1536 && (int64_t)m.B * m.H * ((m.Tm + 15) / 16) >= 1024;
}

// ------------------------------------------------------------------ pooling
struct PoolArgs {
  const uint16_t* q; const uint16_t* k;
  float* qbar;      // [BH][Tm][d]
  float* kbar_t;    // [BH][d][TnP]   (transposed: select_kernel's score loop reads it along the block index),
                    // or [BH][Tn][d] for select16_kernel (k_rows)
  int H, N, Tm, Tn, TnP, k_rows;
  int64_t sb, sh, sn;
};

// Sum of the valid token rows of one block, as 8 channels per thread.  All loads of the block are issued before
// the first add (rows past the end are clamped to the last valid row and not added), so a wave keeps LEN / RP
// 16-byte requests in flight instead of one.
template <int D, int LEN>
__device__ __forceinline__ void pool_rows(const uint16_t* x, int64_t sn, int tok0, int valid, int rsub, int col,
                                          float (&acc)[8]) {
  constexpr int RP = 256 / (D / 8);   // token rows per pass
  constexpr int NP = LEN / RP;
  u32x4 raw[NP];
#pragma unroll
  for (int p = 0; p < NP; ++p) raw[p] = *(const u32x4*)(x + (int64_t)(tok0 + min(rsub + p * RP, valid - 1)) * sn + col);
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const bool live = rsub + p * RP < valid;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __builtin_bit_cast(float, raw[p][e] << 16);
      const float hi = __builtin_bit_cast(float, raw[p][e] & 0xffff0000u);
      acc[2 * e] += live ? lo : 0.f;
      acc[2 * e + 1] += live ? hi : 0.f;
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void pool_kernel(PoolArgs a) {
  constexpr int LPR = D / 8;          // lanes per token row (16 bytes each)
  constexpr int RP = 256 / LPR;       // token rows per pass
  __shared__ float red[RP][D];
  const int per_head = a.Tm + a.Tn;
  const int bh = blockIdx.x / per_head;
  const int rem = blockIdx.x % per_head;
  const bool is_q = rem < a.Tm;
  const int blk = is_q ? rem : rem - a.Tm;
  const int len = is_q ? BQ : BKV;
  const uint16_t* x = (is_q ? a.q : a.k) + (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int tid = threadIdx.x;
  const int rsub = tid / LPR, col = (tid % LPR) * 8;
  const int tok0 = blk * len;
  const int valid = min(len, a.N - tok0);

  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  if (is_q) pool_rows<D, BQ>(x, a.sn, tok0, valid, rsub, col, acc);
  else      pool_rows<D, BKV>(x, a.sn, tok0, valid, rsub, col, acc);
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rsub][col + e] = acc[e];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RP; ++r) s += red[r][tid];
    s /= (float)valid;
    if (is_q) a.qbar[((int64_t)bh * a.Tm + blk) * D + tid] = s;
    else if (a.k_rows) a.kbar_t[((int64_t)bh * a.Tn + blk) * D + tid] = s;
    else      a.kbar_t[((int64_t)bh * D + tid) * a.TnP + blk] = s;
  }
}

hipError_t launch_pool(const void* q, const void* k, const Dims& m, float* qbar, float* kbar, hipStream_t stream) {
  PoolArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.qbar = qbar; a.kbar_t = kbar;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn; a.TnP = m.Tn; a.k_rows = select16_applies(m) ? 1 : 0;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  const dim3 grid((unsigned)((int64_t)m.B * m.H * (m.Tm + m.Tn))), block(256);
  if (m.d == 128) hipLaunchKernelGGL(pool_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(pool_kernel<64>, grid, block, 0, stream, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------ selection
struct SelArgs {
  const float* qbar; const float* kbar_t;
  uint8_t* mask; int32_t* row_cnt; int32_t* row_idx; float* pbar_out;
  int d, Tm, Tn, TnP, groups;   // groups = ceil(Tm / R) row groups per head
  int k_cnt; float top_p; float scale;
};

// exclusive scan of x over the threads of a segment (seg_threads = 64, 128 or 256 consecutive
// threads of the 256-thread workgroup), fixed association order; also returns the segment total
template <typename T>
__device__ __forceinline__ T segment_scan(T x, int tid, int seg_threads, T* sm4, T& seg_total) {
  const int lane = tid & 63, w = tid >> 6;
  T inc = x;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const T y = __shfl_up(inc, off, 64);
    if (lane >= off) inc += y;
  }
  T excl = __shfl_up(inc, 1, 64);
  if (lane == 0) excl = (T)0;
  if (lane == 63) sm4[w] = inc;
  __syncthreads();
  const int wps = seg_threads >> 6;
  const int w0 = (w / wps) * wps;
  T pre = (T)0, tot = (T)0;
  for (int ww = w0; ww < w0 + wps; ++ww) {
    if (ww < w) pre += sm4[ww];
    tot += sm4[ww];
  }
  __syncthreads();
  seg_total = tot;
  return pre + excl;
}

// Pbar in [0, 2) as a 62-bit fixed-point integer (truncated below 2^-62): sums of these are exact and do
// not depend on the order of addition, which makes the Top-p comparison deterministic under LDS atomics.
__device__ __forceinline__ uint64_t fixed62(uint32_t fbits) {
  const int e = (int)(fbits >> 23);                 // the sign bit is clear
  if (e == 0) return 0;                             // zero or denormal
  const uint64_t m = (uint64_t)((fbits & 0x7fffffu) | 0x800000u);
  const int sh = e - 88;                            // value = m * 2^(e-150); times 2^62
  return sh >= 0 ? (m << sh) : (sh > -24 ? (m >> (-sh)) : 0);
}

// Inclusive sum over the 64 lanes of a wave with data-parallel-primitive moves (no LDS traffic, unlike shuffles):
// three shifts by 1, 2, 3 lanes inside each row of 16 lanes, shifts by 4 and 8 for the upper lanes of a row, then the
// last lane of row 0 / 2 added to row 1 / 3 and the last lane of row 1 added to rows 2 and 3.  Lanes without a source
// add 0.
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t x) {
  uint32_t r = x;
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x113, 0xf, 0xf, false);   // row_shr:3
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)r, 0x114, 0xf, 0xe, false);   // row_shr:4, lanes 4..15 of a row
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)r, 0x118, 0xf, 0xc, false);   // row_shr:8, lanes 8..15 of a row
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)r, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  r += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)r, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return r;
}

// One pass of the radix descent, after the histograms of the pass have been accumulated: the calling wave walks the
// bins of row r from the top (lane l owns bins 255-4l .. 252-4l), picks the lowest bin whose top entry is still selected,
// extends the key prefix of the row by it and clears the bins for the next pass.
__device__ __forceinline__ void sel_scan_pass(int pass, int sh, int lane, int r, uint32_t (*h_cnt)[256],
                                              uint64_t (*h_mass)[256], uint64_t* st_key, uint32_t* st_cnt,
                                              uint64_t* st_mass, uint32_t kc, uint64_t p_fx, uint32_t* st_done = nullptr) {
  uint32_t c4[4]; uint64_t m4[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int bin = 255 - 4 * lane - e;
    c4[e] = h_cnt[r][bin]; m4[e] = h_mass[r][bin];
    h_cnt[r][bin] = 0; h_mass[r][bin] = 0;         // ready for the next pass
  }
  uint32_t ct = c4[0] + c4[1] + c4[2] + c4[3];
  uint64_t mt = m4[0] + m4[1] + m4[2] + m4[3];
  // inclusive scans over the lanes (lane 0 = highest bins), on the vector ALU; the 62-bit mass goes as three limbs of
  // 21 bits, whose sums over 64 lanes stay below 2^27, and is put together again exactly
  const uint32_t ci = wave_scan_add(ct);
  const uint64_t mi = (uint64_t)wave_scan_add((uint32_t)(mt & 0x1fffffu)) +
                      ((uint64_t)wave_scan_add((uint32_t)((mt >> 21) & 0x1fffffu)) << 21) +
                      ((uint64_t)wave_scan_add((uint32_t)(mt >> 42)) << 42);
  uint32_t c_above = st_cnt[r] + (ci - ct);          // entries above this lane's first bin
  uint64_t m_above = st_mass[r] + (mi - mt);
  int sel_bin = -1; uint32_t sel_c = 0, sel_n = 0; uint64_t sel_m = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    if (c4[e] != 0 && (c_above < kc || m_above < p_fx)) { sel_bin = 255 - 4 * lane - e; sel_c = c_above; sel_m = m_above; sel_n = c4[e]; }
    c_above += c4[e]; m_above += m4[e];
  }
  const uint64_t bal = __builtin_amdgcn_ballot_w64(sel_bin >= 0);
  // the predicate is monotone, so the selected bins are a prefix of the walk; the last one is the boundary.
  // (bal is never zero: the top non-empty bin always qualifies because cnt_gt of its top entry is below kc
  // on the first pass and the boundary bin's top entry qualifies on later passes.)
  const int src = bal ? 63 - __builtin_clzll(bal) : 0;          // (uniform: a lane read, not a shuffle)
  const int b_bin = __builtin_amdgcn_readlane(sel_bin, src);
  const uint32_t b_c = (uint32_t)__builtin_amdgcn_readlane((int)sel_c, src);
  const uint64_t b_m = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(sel_m >> 32), src) << 32) |
                       (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)sel_m, src);
  const uint32_t b_n = (uint32_t)__builtin_amdgcn_readlane((int)sel_n, src);      // entries in the boundary bin
  if (lane == 0) {
    uint64_t key = st_key[r] | ((uint64_t)(uint32_t)max(b_bin, 0) << sh);
    if (pass == 3) key |= 0xffff0000ull;             // bits 31..16 of every key are ones (block index < 65536)
    st_key[r] = key; st_cnt[r] = b_c; st_mass[r] = b_m;
    // A boundary bin with a single entry needs no further passes: that entry is selected (it is the bin's top entry),
    // so the lower end of the bin, which is what the key prefix with zeros below it says, already is a threshold.
    if (st_done) st_done[r] = b_n == 1u ? 1u : 0u;
  }
}

// Mask rows and ascending index lists of up to R rows from their flags (R * NP bytes in LDS): thread t compacts E
// consecutive block indices of row t / (256 / R).
template <int NP, int R>
__device__ __forceinline__ void sel_compact(const SelArgs& a, int bh, int i0, int nrows, int tid, const uint8_t* flag,
                                            int* sm4i) {
  constexpr int E = R * NP / 256;         // consecutive block indices per thread
  constexpr int SEG_T = 256 / R;          // threads per row
  const int Tn = a.Tn;
  const int seg = tid / SEG_T;                    // which row this thread compacts
  const int pos0 = (tid % SEG_T) * E;             // first block index handled by this thread
  int cntl = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) cntl += flag[seg * NP + pos0 + e];
  int seg_tot_i;
  int wr = segment_scan<int>(cntl, tid, SEG_T, sm4i, seg_tot_i);
  if (seg < nrows) {
    const int64_t row = (int64_t)bh * a.Tm + i0 + seg;
    uint8_t* mrow = a.mask + row * Tn;
    int32_t* irow = a.row_idx + row * Tn;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int j = pos0 + e;
      if (j < Tn) {
        const uint8_t f = flag[seg * NP + j];
        mrow[j] = f;
        if (f) irow[wr++] = j;
      }
    }
    if ((tid % SEG_T) == 0) a.row_cnt[row] = seg_tot_i;
  }
}

// NP: padded row length (a multiple of 256 >= T_n; the closer, the fewer score columns are computed for
// nothing).  R = 4 rows of one head per workgroup.
//
// Selection without sorting.  Entries are ordered by the 64-bit key (bits(Pbar) << 32) | ~j (larger Pbar
// first, equal Pbar: lower block index first).  With cnt_gt(e) / mass_gt(e) the number / total Pbar of
// the entries whose key is greater than e's, the rule "first max(1, k_cnt, n_p) entries of the order,
// n_p = shortest prefix with sum >= p" is the same as
//        e selected  <=>  cnt_gt(e) < max(1, k_cnt)  or  mass_gt(e) < p,
// a predicate that is monotone in the key, so the selected set is {key >= T}.  T is found by a radix
// descent over the key, 8 bits per pass (6 passes: four over the bits of Pbar, two over the index bits
// that break ties): per pass a 256-bin histogram of count and mass of the entries that match the prefix
// found so far, then one wave per row walks the bins from the top and picks the lowest bin whose top
// entry is still selected.
constexpr int score_group(int jj) {
  for (int g = 8; g > 1; --g)
    if (jj % g == 0) return g;
  return 1;
}

template <int NP, int R>
__global__ __launch_bounds__(256) void select_kernel(SelArgs a) {
  static_assert(R == 4, "one wave scans the histogram of one row");
  constexpr int JJ = NP / 256;            // score columns per thread per row
  constexpr int G = score_group(JJ);      // columns per thread processed together in the score loop (divides JJ)
  constexpr int CB = G <= 4 ? 8 : 4;      // channels whose loads are in flight together (CB * G requests per lane)
  constexpr int E = R * NP / 256;         // consecutive block indices per thread in the compaction pass
  constexpr int SEG_T = 256 / R;          // threads per row in the compaction pass
  __shared__ uint32_t h_cnt[R][256];
  __shared__ uint64_t h_mass[R][256];
  __shared__ __align__(16) double qd[128][R];
  __shared__ uint8_t flag[R * NP];
  __shared__ float redf[R][4];
  __shared__ int sm4i[4];
  __shared__ uint64_t st_key[R];          // key prefix found so far (lower bits zero)
  __shared__ uint32_t st_cnt[R];          // number of entries above the prefix range
  __shared__ uint64_t st_mass[R];         // their mass

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int bh = blockIdx.x / a.groups;
  const int i0 = (blockIdx.x % a.groups) * R;
  const int nrows = min(R, a.Tm - i0);
  const int d = a.d, Tn = a.Tn;

  for (int x = tid; x < R * d; x += 256) {
    const int r = x / d, c = x % d;
    qd[c][r] = r < nrows ? (double)a.qbar[((int64_t)bh * a.Tm + i0 + r) * d + c] : 0.0;
  }
  for (int x = tid; x < R * NP; x += 256) flag[x] = 0;
  for (int x = tid; x < R * 256; x += 256) { h_cnt[x >> 8][x & 255] = 0; h_mass[x >> 8][x & 255] = 0; }
  if (tid < R) { st_key[tid] = 0; st_cnt[tid] = 0; st_mass[tid] = 0; }
  __syncthreads();

  // ---- Sbar = Qbar Kbar^T * scale: fp32 pooled values, fp64 accumulation, rounded once to fp32
  float s[R][JJ];
  const float* kt = a.kbar_t + (int64_t)bh * d * a.TnP;
#pragma unroll
  for (int jg = 0; jg < JJ; jg += G) {
    double acc[R][G];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int u = 0; u < G; ++u) acc[r][u] = 0.0;
    if (tid + 256 * jg < Tn) {       // whole groups past the end of the row are skipped
      int jc[G];                     // this thread's columns of the group, clamped to the row
#pragma unroll
      for (int u = 0; u < G; ++u) jc[u] = min(tid + 256 * (jg + u), Tn - 1);
      // CB channels at a time: their CB * G loads are issued together, then the products are added channel by
      // channel, so every accumulator still sums c = 0, 1, 2, ... in order (d is a multiple of 64)
      for (int c0 = 0; c0 < d; c0 += CB) {
        float kraw[CB][G];
#pragma unroll
        for (int cc = 0; cc < CB; ++cc)
#pragma unroll
          for (int u = 0; u < G; ++u) kraw[cc][u] = kt[(int64_t)(c0 + cc) * a.TnP + jc[u]];
#pragma unroll
        for (int cc = 0; cc < CB; ++cc) {
          double q4[R];
#pragma unroll
          for (int r = 0; r < R; ++r) q4[r] = qd[c0 + cc][r];
#pragma unroll
          for (int u = 0; u < G; ++u) {
            const double kv = (double)kraw[cc][u];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r][u] = fma(q4[r], kv, acc[r][u]);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int u = 0; u < G; ++u)
        s[r][jg + u] = (tid + 256 * (jg + u)) < Tn ? (float)(acc[r][u] * (double)a.scale) : -INFINITY;
  }

  // ---- Pbar = softmax(Sbar) per row, fp32
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float mx = s[r][0];
#pragma unroll
    for (int jj = 1; jj < JJ; ++jj) mx = fmaxf(mx, s[r][jj]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) redf[r][w] = mx;
  }
  __syncthreads();
  float rowmax[R];
#pragma unroll
  for (int r = 0; r < R; ++r) rowmax[r] = fmaxf(fmaxf(redf[r][0], redf[r][1]), fmaxf(redf[r][2], redf[r][3]));
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float sum = 0.f;
#pragma unroll
    for (int jj = 0; jj < JJ; ++jj) {
      const float e = (tid + 256 * jj) < Tn ? expf(s[r][jj] - rowmax[r]) : 0.f;
      s[r][jj] = e;
      sum += e;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) redf[r][w] = sum;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const float tot = (redf[r][0] + redf[r][1]) + (redf[r][2] + redf[r][3]);
#pragma unroll
    for (int jj = 0; jj < JJ; ++jj) {
      const int j = tid + 256 * jj;
      if (j < Tn) {
        const float p = s[r][jj] / tot;
        s[r][jj] = p;                      // from here on s holds Pbar
        if (a.pbar_out && r < nrows) a.pbar_out[((int64_t)bh * a.Tm + i0 + r) * Tn + j] = p;
      }
    }
  }

  // ---- radix descent for the threshold key of each row
  const uint32_t kc = (uint32_t)max(1, a.k_cnt);
  uint64_t p_fx = fixed62(__builtin_bit_cast(uint32_t, a.top_p));
  if (a.top_p > 0.f && p_fx == 0) p_fx = 1;
#pragma unroll 1
  for (int pass = 0; pass < 6; ++pass) {
    const int sh = pass < 4 ? 56 - 8 * pass : (pass == 4 ? 8 : 0);
    // accumulate: entries that match the prefix found so far
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const uint64_t pre = st_key[r];
#pragma unroll
      for (int jj = 0; jj < JJ; ++jj) {
        const int j = tid + 256 * jj;
        if (j < Tn) {
          const uint32_t fb = __builtin_bit_cast(uint32_t, s[r][jj]);
          const uint64_t key = ((uint64_t)fb << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
          const bool match = pass == 0 ? true : (((key ^ pre) >> (sh + 8)) == 0);
          if (match) {
            const int dig = (int)((key >> sh) & 255u);
            atomicAdd(&h_cnt[r][dig], 1u);
            atomicAdd((unsigned long long*)&h_mass[r][dig], (unsigned long long)fixed62(fb));
          }
        }
      }
    }
    __syncthreads();
    sel_scan_pass(pass, sh, lane, w, h_cnt, h_mass, st_key, st_cnt, st_mass, kc, p_fx);
    __syncthreads();
  }

  // ---- flags: key >= threshold
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const uint64_t thr = st_key[r];
#pragma unroll
    for (int jj = 0; jj < JJ; ++jj) {
      const int j = tid + 256 * jj;
      if (j < Tn) {
        const uint64_t key = ((uint64_t)__builtin_bit_cast(uint32_t, s[r][jj]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
        if (key >= thr) flag[r * NP + j] = 1;
      }
    }
  }
  __syncthreads();

  sel_compact<NP, R>(a, bh, i0, nrows, tid, flag, sm4i);
}

// The same selection with the score product on the fp64 matrix cores, for rows of up to 1536 blocks.  A workgroup
// takes 16 rows of the pooled map: Sbar (16 x NP) = Qbar (16 x d) Kbar^T in tiles of 16 x 16 by
// v_mfma_f64_16x16x4_f64 (A[m][k]: lane l holds m = l % 16, k = l / 16; B[k][n]: k = l / 16, n = l % 16;
// C[m][n]: n = l % 16, m = l / 16 + 4 v for accumulator element v), so a pooled key value that is loaded and widened
// serves 16 rows instead of 4 and the products no longer run on the vector ALU.  Wave w takes the column tiles
// w, w + 4, ...; its accumulators then hold, for each of the four row batches v = 0..3 (rows 4v .. 4v + 3 of the
// workgroup), the scores of ONE row per lane (row l / 16 of the batch) at the columns 16 (w + 4 t) + l % 16.  The
// sixteen rows are selected together exactly as in select_kernel (same keys, histograms, threshold rule and
// compaction), with that row / column assignment in place of (all four rows, columns tid + 256 jj).
// fp64 sums of the same products in a different order than select_kernel's chain of FMAs: the scores of the two
// kernels may differ in the last bit of their fp32 rounding.
typedef __attribute__((ext_vector_type(4))) double f64x4;
template <int NP, int D>
__global__ __launch_bounds__(256) void select16_kernel(SelArgs a) {
  constexpr int R = 4, RW = 16;
  constexpr int NT = NP / 64;             // column tiles per wave
  constexpr int KS = D / 4;               // contraction steps of 4 channels
  __shared__ uint32_t h_cnt[RW][256];
  __shared__ uint64_t h_mass[RW][256];
  __shared__ uint8_t flag[RW * NP];
  __shared__ float redf[RW][4];
  __shared__ float redm[RW][4];
  __shared__ int sm4i[4];
  __shared__ uint64_t st_key[RW];
  __shared__ uint32_t st_cnt[RW];
  __shared__ uint64_t st_mass[RW];
  __shared__ uint32_t st_done[RW];        // the row's threshold is final (see sel_scan_pass)

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int lg = lane >> 4, ln = lane & 15;
  const int bh = blockIdx.x / a.groups;
  const int iw = (blockIdx.x % a.groups) * RW;        // first row of the workgroup
  const int nrows_w = min(RW, a.Tm - iw);
  const int Tn = a.Tn;

  for (int x = tid; x < RW * 256; x += 256) { h_cnt[x >> 8][x & 255] = 0; h_mass[x >> 8][x & 255] = 0; }
  for (int x = tid; x < RW * NP; x += 256) flag[x] = 0;
  if (tid < RW) { st_key[tid] = 0; st_cnt[tid] = 0; st_mass[tid] = 0; st_done[tid] = 0; }

  // ---- Sbar = Qbar Kbar^T * scale: fp32 pooled values widened to fp64, fp64 products and sums, rounded once to fp32
  // Contraction step c = 4g + e takes the four channels 16g + 4k + e, k = 0..3 (which channels make up a step is free
  // as long as both operands agree): lane (k = lg) then needs the channels 16g + 4lg + 0..3 for the steps 4g .. 4g+3,
  // one 16-byte load from the row-major pooled keys.
  double af[KS];                          // A operand: row iw + ln
  {
    const float* qrow = a.qbar + ((int64_t)bh * a.Tm + iw + min(ln, nrows_w - 1)) * D + 4 * lg;
#pragma unroll
    for (int g = 0; g < KS / 4; ++g) {
      const f32x4 q4 = *(const f32x4*)(qrow + 16 * g);
#pragma unroll
      for (int e = 0; e < 4; ++e) af[4 * g + e] = ln < nrows_w ? (double)q4[e] : 0.0;
    }
  }
  float sv[4][NT];                        // [row batch][tile]: this lane's row of the batch, column 16 (w + 4t) + ln
  const float* kb = a.kbar_t + (int64_t)bh * Tn * D + 4 * lg;
  auto load_tile = [&](int t, f32x4 (&kr)[KS / 4]) {      // B operand of tile t (columns past the row: clamped)
    const float* kc = kb + (int64_t)min(16 * (w + 4 * t) + ln, Tn - 1) * D;
#pragma unroll
    for (int g = 0; g < KS / 4; ++g) kr[g] = *(const f32x4*)(kc + 16 * g);
  };
  f32x4 krA[KS / 4], krB[KS / 4];         // the loads of tile t+1 are in flight during the products of tile t
  load_tile(0, krA);
  auto tile = [&](auto T, f32x4 (&kr)[KS / 4], f32x4 (&kn)[KS / 4]) {
    constexpr int t = decltype(T)::v;
    if constexpr (t + 1 < NT) load_tile(t + 1, kn);
    const int col = 16 * (w + 4 * t) + ln;
    f64x4 acc = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};      // two chains: even and odd contraction steps
    if (16 * (w + 4 * t) < Tn) {          // (uniform per wave: tiles past the end of the row are skipped)
#pragma unroll
      for (int c = 0; c < KS; c += 2) {
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(af[c], (double)kr[c / 4][c % 4], acc, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(af[c + 1], (double)kr[(c + 1) / 4][(c + 1) % 4], acc1, 0, 0, 0);
      }
      acc += acc1;
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) sv[v][t] = col < Tn ? (float)(acc[v] * (double)a.scale) : -INFINITY;
  };
  static_for<0, NT>([&](auto T) {
    if constexpr ((decltype(T)::v & 1) == 0) tile(T, krA, krB); else tile(T, krB, krA);
  });
  __syncthreads();

  const uint32_t kc = (uint32_t)max(1, a.k_cnt);
  uint64_t p_fx = fixed62(__builtin_bit_cast(uint32_t, a.top_p));
  if (a.top_p > 0.f && p_fx == 0) p_fx = 1;

  // ---- selection of all sixteen rows together; of batch v (rows 4v .. 4v+3) this lane holds row 4v + lg
  // Pbar = softmax(Sbar) per row, fp32: maximum and sum over the 16 lanes of the row in this wave, then over the four
  // waves through LDS
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    float mx = sv[v][0];
#pragma unroll
    for (int t = 1; t < NT; ++t) mx = fmaxf(mx, sv[v][t]);
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (ln == 0) redf[4 * v + lg][w] = mx;
  }
  __syncthreads();
  float rowmax[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int r = 4 * v + lg;
    rowmax[v] = fmaxf(fmaxf(redf[r][0], redf[r][1]), fmaxf(redf[r][2], redf[r][3]));
  }
  __syncthreads();
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    float sum = 0.f, emin = INFINITY;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bool in_row = (16 * (w + 4 * t) + ln) < Tn;
      const float e = in_row ? expf(sv[v][t] - rowmax[v]) : 0.f;
      sv[v][t] = e;
      sum += e;
      emin = in_row ? fminf(emin, e) : emin;
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) {
      sum += __shfl_xor(sum, off, 64);
      emin = fminf(emin, __shfl_xor(emin, off, 64));
    }
    if (ln == 0) { redf[4 * v + lg][w] = sum; redm[4 * v + lg][w] = emin; }
  }
  __syncthreads();
  // The selection below only uses the order of the probabilities, so their bit patterns are first mapped, row by
  // row, onto the whole 32-bit range: b -> (b - b_min) << (leading zeros of b_max - b_min), with b_min / b_max the
  // patterns of the row's smallest / largest probability (non-negative floats order like their patterns; the map is
  // increasing and keeps ties).  The top eight bits of a probability are its sign and seven exponent bits, the same
  // three or four values for almost every entry of a row: unmapped, the first pass of the descent would tell almost
  // nothing apart; mapped, a pass spreads a row over all 256 bins, the boundary bin holds a single entry after two
  // passes for most rows, and the row's descent stops there (see sel_scan_pass).
  uint32_t bmin[4]; int bsh[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int r = 4 * v + lg;
    const float tot = (redf[r][0] + redf[r][1]) + (redf[r][2] + redf[r][3]);
    const float emin = fminf(fminf(redm[r][0], redm[r][1]), fminf(redm[r][2], redm[r][3]));
    // (the smallest / largest e over the same sum; the largest e is exp(0) = 1.  Two patterns of margin on either
    // side, so that the map stays inside 32 bits whatever the last bit of these two divisions is.)
    const uint32_t lo = __builtin_bit_cast(uint32_t, emin / tot), hi = __builtin_bit_cast(uint32_t, 1.0f / tot);
    bmin[v] = lo >= 2u ? lo - 2u : 0u;
    bsh[v] = __builtin_clz((max(hi, lo) + 2u - bmin[v]) | 1u);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int j = 16 * (w + 4 * t) + ln;
      if (j < Tn) {
        const float p = sv[v][t] / tot;
        sv[v][t] = p;                                  // from here on sv holds Pbar
        if (a.pbar_out && r < nrows_w) a.pbar_out[((int64_t)bh * a.Tm + iw + r) * Tn + j] = p;
      }
    }
  }

  // radix descent for the threshold key of each row (see select_kernel); wave w scans the histograms of rows 4w .. 4w+3
#pragma unroll 1
  for (int pass = 0; pass < 6; ++pass) {
    const int sh = pass < 4 ? 56 - 8 * pass : (pass == 4 ? 8 : 0);
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = 4 * v + lg;
      const uint64_t pre = st_key[r];
      const bool open = st_done[r] == 0;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int j = 16 * (w + 4 * t) + ln;
        if (j < Tn && open) {
          uint32_t fb = __builtin_bit_cast(uint32_t, sv[v][t]);
#if defined(__HIP_DEVICE_COMPILE__)
          asm volatile("" : "+v"(fb));     // (keeps the keys and fixed-point masses of all 80 entries from being
                                           // computed once and held in registers across the passes)
#endif
          const uint64_t key = ((uint64_t)((fb - bmin[v]) << bsh[v]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
          const bool match = pass == 0 ? true : (((key ^ pre) >> (sh + 8)) == 0);
          if (match) {
            const int dig = (int)((key >> sh) & 255u);
            atomicAdd(&h_cnt[r][dig], 1u);
            atomicAdd((unsigned long long*)&h_mass[r][dig], (unsigned long long)fixed62(fb));
          }
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4; ++x)
      if (st_done[4 * w + x] == 0) sel_scan_pass(pass, sh, lane, 4 * w + x, h_cnt, h_mass, st_key, st_cnt, st_mass, kc, p_fx, st_done);
    if (__syncthreads_and(st_done[tid & (RW - 1)] != 0)) break;       // every row of the workgroup has its threshold
  }

  // flags: key >= threshold
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int r = 4 * v + lg;
    const uint64_t thr = st_key[r];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int j = 16 * (w + 4 * t) + ln;
      if (j < Tn) {
        const uint64_t key = ((uint64_t)((__builtin_bit_cast(uint32_t, sv[v][t]) - bmin[v]) << bsh[v]) << 32) |
                             (uint64_t)(0xffffffffu - (uint32_t)j);
        if (key >= thr) flag[r * NP + j] = 1;
      }
    }
  }
  __syncthreads();
  // mask rows and index lists, four rows at a time
  for (int v = 0; v < 4 && 4 * v < nrows_w; ++v) {
    sel_compact<NP, R>(a, bh, iw + 4 * v, min(R, nrows_w - 4 * v), tid, flag + 4 * v * NP, sm4i);
    __syncthreads();                                   // (the scan scratch is reused)
  }
}

template <int NP, int R>
static void launch_select_t(const SelArgs& a0, int BH, hipStream_t stream) {
  SelArgs a = a0;
  a.groups = (a.Tm + R - 1) / R;
  hipLaunchKernelGGL((select_kernel<NP, R>), dim3((unsigned)(BH * a.groups)), dim3(256), 0, stream, a);
}

template <int NP>
static void launch_select16_t(const SelArgs& a0, int BH, hipStream_t stream) {
  SelArgs a = a0;
  a.groups = (a.Tm + 15) / 16;
  if (a.d == 128) hipLaunchKernelGGL((select16_kernel<NP, 128>), dim3((unsigned)(BH * a.groups)), dim3(256), 0, stream, a);
  else            hipLaunchKernelGGL((select16_kernel<NP, 64>), dim3((unsigned)(BH * a.groups)), dim3(256), 0, stream, a);
}

hipError_t launch_select(const float* qbar, const float* kbar, const Dims& m, int topk_blocks, float top_p,
                         float scale, uint8_t* mask, int32_t* row_cnt, int32_t* row_idx, float* pbar_out,
                         hipStream_t stream) {
  SelArgs a;
  a.qbar = qbar; a.kbar_t = kbar; a.mask = mask; a.row_cnt = row_cnt; a.row_idx = row_idx; a.pbar_out = pbar_out;
  a.d = m.d; a.Tm = m.Tm; a.Tn = m.Tn; a.TnP = m.Tn; a.groups = 0;
  a.k_cnt = topk_blocks; a.top_p = top_p; a.scale = scale;
  const int BH = m.B * m.H;
  // the smallest instantiated width that holds the row: steps of 256 up to 2048, then of 512, then of 1024
  if (select16_applies(m)) {        // (the pooling pass has laid out the pooled keys for this kernel)
#define SPA2_SELECT16_CASE(np) if (m.Tn <= np) { launch_select16_t<np>(a, BH, stream); return hipGetLastError(); }
    SPA2_SELECT16_CASE(256)  SPA2_SELECT16_CASE(512)  SPA2_SELECT16_CASE(768)  SPA2_SELECT16_CASE(1024)
    SPA2_SELECT16_CASE(1280) SPA2_SELECT16_CASE(1536)
#undef SPA2_SELECT16_CASE
  }
#define SPA2_SELECT_CASE(np) if (m.Tn <= np) { launch_select_t<np, 4>(a, BH, stream); return hipGetLastError(); }
  SPA2_SELECT_CASE(256)  SPA2_SELECT_CASE(512)  SPA2_SELECT_CASE(768)  SPA2_SELECT_CASE(1024)
  SPA2_SELECT_CASE(1280) SPA2_SELECT_CASE(1536) SPA2_SELECT_CASE(1792) SPA2_SELECT_CASE(2048) SPA2_SELECT_CASE(2560) SPA2_SELECT_CASE(3072) SPA2_SELECT_CASE(3584) SPA2_SELECT_CASE(4096)
  SPA2_SELECT_CASE(5120) SPA2_SELECT_CASE(6144) SPA2_SELECT_CASE(7168)
#undef SPA2_SELECT_CASE
  launch_select_t<8192, 4>(a, BH, stream);
  return hipGetLastError();
}

// ------------------------------------------------------------------ column lists
// One workgroup lists 64 key blocks of one head: thread (seg, c) walks one of COL_SEGS runs of query blocks of
// column c twice, first counting, then (after the counts of the column's runs have been exchanged through LDS)
// writing its ascending piece of the list at the right offset.
constexpr int COL_SEGS = 16;
__global__ __launch_bounds__(64 * COL_SEGS) void columns_kernel(const uint8_t* mask, int Tm, int Tn, int32_t* col_cnt,
                                                                int32_t* col_idx) {
  __shared__ int seg_cnt[COL_SEGS][64];
  const int bh = blockIdx.y;
  const int c = threadIdx.x & 63, seg = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + c;
  const int per = (Tm + COL_SEGS - 1) / COL_SEGS;
  const int i0 = min(Tm, seg * per), i1 = min(Tm, i0 + per);
  const bool live = j < Tn;
  const uint8_t* mp = mask + (int64_t)bh * Tm * Tn + (live ? j : 0);
  int n = 0;
  if (live)
    for (int i = i0; i < i1; ++i) n += mp[(int64_t)i * Tn] != 0;
  seg_cnt[seg][c] = n;
  __syncthreads();
  if (!live) return;
  int at = 0;
  for (int s2 = 0; s2 < seg; ++s2) at += seg_cnt[s2][c];
  int32_t* out = col_idx + ((int64_t)bh * Tn + j) * Tm;
  for (int i = i0; i < i1; ++i)
    if (mp[(int64_t)i * Tn]) out[at++] = i;
  if (seg == COL_SEGS - 1) col_cnt[(int64_t)bh * Tn + j] = at;
}

// Launch order of the key blocks of one head for the dK/dV kernel: longest column first, dealt round-robin
// to the eight XCD chunks of the schedule (position x*chunk + s belongs to XCD x), so that every XCD gets the
// same mix of long and short columns and the long ones start early.  One workgroup per head.
template <int NP>
__global__ __launch_bounds__(NP / 2 < 1024 ? NP / 2 : 1024) void col_order_kernel(const int32_t* col_cnt, int Tn, int32_t* col_order) {
  __shared__ uint32_t keys[NP];
  constexpr int BT = NP / 2 < 1024 ? NP / 2 : 1024;     // one compare-exchange per thread and step where that fits
  const int bh = blockIdx.x, tid = threadIdx.x;
  for (int j = tid; j < NP; j += BT)
    keys[j] = j < Tn ? ((uint32_t)min(col_cnt[(int64_t)bh * Tn + j], 0xffff) << 16) | (uint32_t)(0xffff - j) : 0u;
  __syncthreads();
  for (int k = 2; k <= NP; k <<= 1)
    for (int st = k >> 1; st > 0; st >>= 1) {
      for (int pr = tid; pr < NP / 2; pr += BT) {
        const int lo = 2 * st * (pr / st) + (pr % st), hi = lo + st;
        const bool desc = (lo & k) == 0;
        const uint32_t x = keys[lo], y = keys[hi];
        if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
      }
      __syncthreads();
    }
  const int chunk = (Tn + 7) / 8;
  for (int pos = tid; pos < Tn; pos += BT) {
    const int x = pos / chunk, sidx = pos % chunk;
    int rank = 0;                                  // how many schedule positions are dealt before this one
    for (int xx = 0; xx < 8; ++xx) {
      const int len = min(max(Tn - xx * chunk, 0), chunk);
      rank += min(len, sidx) + ((xx < x && sidx < len) ? 1 : 0);
    }
    col_order[(int64_t)bh * Tn + pos] = 0xffff - (int)(keys[rank] & 0xffffu);
  }
}

hipError_t launch_columns(const uint8_t* mask, const Dims& m, int32_t* col_cnt, int32_t* col_idx,
                          int32_t* col_order, hipStream_t stream) {
  const dim3 grid((unsigned)((m.Tn + 63) / 64), (unsigned)(m.B * m.H)), block(256);
  hipLaunchKernelGGL(columns_kernel, grid, dim3(64 * COL_SEGS), 0, stream, mask, m.Tm, m.Tn, col_cnt, col_idx);
  if (col_order) {
    const dim3 g2((unsigned)(m.B * m.H));
    if (m.Tn <= 512)       hipLaunchKernelGGL(col_order_kernel<512>, g2, dim3(256), 0, stream, col_cnt, m.Tn, col_order);
    else if (m.Tn <= 2048) hipLaunchKernelGGL(col_order_kernel<2048>, g2, dim3(1024), 0, stream, col_cnt, m.Tn, col_order);
    else                   hipLaunchKernelGGL(col_order_kernel<8192>, g2, dim3(1024), 0, stream, col_cnt, m.Tn, col_order);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------ all-ones pattern
__global__ __launch_bounds__(256) void full_rows_kernel(int Tm, int Tn, uint8_t* mask, int32_t* row_cnt,
                                                        int32_t* row_idx) {
  const int64_t row = blockIdx.x;   // bh * Tm + i
  for (int j = threadIdx.x; j < Tn; j += 256) {
    mask[row * Tn + j] = 1;
    row_idx[row * Tn + j] = j;
  }
  if (threadIdx.x == 0) row_cnt[row] = Tn;
}
__global__ __launch_bounds__(256) void full_cols_kernel(int Tm, int Tn, int32_t* col_cnt, int32_t* col_idx,
                                                        int32_t* col_order) {
  const int64_t colr = blockIdx.x;  // bh * Tn + j
  for (int i = threadIdx.x; i < Tm; i += 256) col_idx[colr * Tm + i] = i;
  if (threadIdx.x == 0) {
    col_cnt[colr] = Tm;
    if (col_order) col_order[colr] = (int32_t)(colr % Tn);
  }
}

hipError_t launch_pattern_full(const Dims& m, uint8_t* mask, int32_t* row_cnt, int32_t* row_idx,
                               int32_t* col_cnt, int32_t* col_idx, int32_t* col_order, hipStream_t stream) {
  const int BH = m.B * m.H;
  hipLaunchKernelGGL(full_rows_kernel, dim3((unsigned)(BH * m.Tm)), dim3(256), 0, stream, m.Tm, m.Tn, mask,
                     row_cnt, row_idx);
  if (col_cnt)
    hipLaunchKernelGGL(full_cols_kernel, dim3((unsigned)(BH * m.Tn)), dim3(256), 0, stream, m.Tm, m.Tn, col_cnt,
                       col_idx, col_order);
  return hipGetLastError();
}

}  // namespace spa2
