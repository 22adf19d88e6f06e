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
//   columns_kernel  the same pattern listed per key block (for dK/dV).
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

// ------------------------------------------------------------------ pooling
struct PoolArgs {
  const uint16_t* q; const uint16_t* k;
  float* qbar;      // [BH][Tm][d]
  float* kbar_t;    // [BH][d][TnP]   (transposed: the score loop reads it along the block index)
  int H, N, Tm, Tn, TnP;
  int64_t sb, sh, sn;
};

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
#pragma unroll 4
  for (int r = rsub; r < len; r += RP) {
    if (r < valid) {
      const u32x4 raw = *(const u32x4*)(x + (int64_t)(tok0 + r) * a.sn + col);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += __builtin_bit_cast(float, raw[e] << 16);
        acc[2 * e + 1] += __builtin_bit_cast(float, raw[e] & 0xffff0000u);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rsub][col + e] = acc[e];
  __syncthreads();
  if (tid < D) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < RP; ++r) s += red[r][tid];
    s /= (float)valid;
    if (is_q) a.qbar[((int64_t)bh * a.Tm + blk) * D + tid] = s;
    else      a.kbar_t[((int64_t)bh * D + tid) * a.TnP + blk] = s;
  }
}

hipError_t launch_pool(const void* q, const void* k, const Dims& m, float* qbar, float* kbar, hipStream_t stream) {
  PoolArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.qbar = qbar; a.kbar_t = kbar;
  a.H = m.H; a.N = m.N; a.Tm = m.Tm; a.Tn = m.Tn; a.TnP = m.Tn;
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

// NP: padded row length (power of two >= T_n, >= 256).  R rows of one head per workgroup.
template <int NP, int R>
__global__ __launch_bounds__(256) void select_kernel(SelArgs a) {
  constexpr int JJ = NP / 256;            // score columns per thread per row
  constexpr int E = R * NP / 256;         // consecutive sorted / index-ordered elements per thread
  constexpr int SEG_T = 256 / R;          // threads per row in the scans
  __shared__ uint64_t keys[R * NP];
  __shared__ double qd[R][128];
  __shared__ uint8_t flag[R * NP];
  __shared__ float redf[R][4];
  __shared__ double sm4d[4];
  __shared__ int sm4i[4];
  __shared__ int n_sel[R];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int bh = blockIdx.x / a.groups;
  const int i0 = (blockIdx.x % a.groups) * R;
  const int nrows = min(R, a.Tm - i0);
  const int d = a.d, Tn = a.Tn;

  for (int x = tid; x < R * d; x += 256) {
    const int r = x / d, c = x % d;
    qd[r][c] = r < nrows ? (double)a.qbar[((int64_t)bh * a.Tm + i0 + r) * d + c] : 0.0;
  }
  for (int x = tid; x < R * NP; x += 256) flag[x] = 0;
  __syncthreads();

  // ---- Sbar = Qbar Kbar^T * scale: fp32 pooled values, fp64 accumulation, rounded once to fp32
  float s[R][JJ];
  const float* kt = a.kbar_t + (int64_t)bh * d * a.TnP;
#pragma unroll
  for (int jj = 0; jj < JJ; ++jj) {
    const int j = tid + 256 * jj;
    double acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.0;
    if (j < Tn) {
      for (int c = 0; c < d; ++c) {
        const double kv = (double)kt[(int64_t)c * a.TnP + j];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = fma(qd[r][c], kv, acc[r]);
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) s[r][jj] = j < Tn ? (float)(acc[r] * (double)a.scale) : -INFINITY;
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
      uint64_t key = 0;                                   // padding sorts last
      if (j < Tn) {
        const float p = s[r][jj] / tot;
        if (a.pbar_out && r < nrows) a.pbar_out[((int64_t)bh * a.Tm + i0 + r) * Tn + j] = p;
        // larger Pbar first; equal Pbar: lower block index first
        key = ((uint64_t)__builtin_bit_cast(uint32_t, p) << 32) | (uint64_t)(0xffffffffu - (uint32_t)j);
      }
      keys[r * NP + j] = key;
    }
  }
  __syncthreads();

  // ---- bitonic sort of each row, descending
  for (int k = 2; k <= NP; k <<= 1) {
    for (int st = k >> 1; st > 0; st >>= 1) {
#pragma unroll
      for (int e = 0; e < E / 2; ++e) {
        const int pr = tid + 256 * e;
        const int lo = 2 * st * (pr / st) + (pr % st);
        const int hi = lo + st;
        const bool desc = ((lo & (NP - 1)) & k) == 0;
        const uint64_t x = keys[lo], y = keys[hi];
        if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
      }
      __syncthreads();
    }
  }

  // ---- cumulative probability in sorted order (fp64), n_p, n
  const int seg = tid / SEG_T;                    // which row this thread scans
  const int pos0 = (tid % SEG_T) * E;             // first sorted position (within the row) of this thread
  double excl[E];
  double run = 0.0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    excl[e] = run;
    run += (double)__builtin_bit_cast(float, (uint32_t)(keys[seg * NP + pos0 + e] >> 32));
  }
  double seg_tot_d;
  const double pre = segment_scan<double>(run, tid, SEG_T, sm4d, seg_tot_d);
  int below = 0;   // positions r (0-based) whose preceding sum c_r is still < top_p
  const double pth = (double)a.top_p;
#pragma unroll
  for (int e = 0; e < E; ++e)
    if (pos0 + e < Tn && (pre + excl[e]) < pth) ++below;
  int n_p;
  segment_scan<int>(below, tid, SEG_T, sm4i, n_p);
  if ((tid % SEG_T) == 0) {
    int n = max(max(1, a.k_cnt), n_p);
    n_sel[seg] = min(n, Tn);
  }
  __syncthreads();
  {
    const int n = n_sel[seg];
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (pos0 + e < n) {
        const uint32_t j = 0xffffffffu - (uint32_t)(keys[seg * NP + pos0 + e] & 0xffffffffu);
        flag[seg * NP + j] = 1;
      }
  }
  __syncthreads();

  // ---- mask row and ascending index list
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
    if ((tid % SEG_T) == 0) a.row_cnt[row] = n_sel[seg];
  }
}

template <int NP, int R>
static void launch_select_t(const SelArgs& a0, int BH, hipStream_t stream) {
  SelArgs a = a0;
  a.groups = (a.Tm + R - 1) / R;
  hipLaunchKernelGGL((select_kernel<NP, R>), dim3((unsigned)(BH * a.groups)), dim3(256), 0, stream, a);
}

hipError_t launch_select(const float* qbar, const float* kbar, const Dims& m, int topk_blocks, float top_p,
                         float scale, uint8_t* mask, int32_t* row_cnt, int32_t* row_idx, float* pbar_out,
                         hipStream_t stream) {
  SelArgs a;
  a.qbar = qbar; a.kbar_t = kbar; a.mask = mask; a.row_cnt = row_cnt; a.row_idx = row_idx; a.pbar_out = pbar_out;
  a.d = m.d; a.Tm = m.Tm; a.Tn = m.Tn; a.TnP = m.Tn; a.groups = 0;
  a.k_cnt = topk_blocks; a.top_p = top_p; a.scale = scale;
  const int BH = m.B * m.H;
  if (m.Tn <= 256)       launch_select_t<256, 4>(a, BH, stream);
  else if (m.Tn <= 512)  launch_select_t<512, 4>(a, BH, stream);
  else if (m.Tn <= 1024) launch_select_t<1024, 4>(a, BH, stream);
  else if (m.Tn <= 2048) launch_select_t<2048, 4>(a, BH, stream);
  else if (m.Tn <= 4096) launch_select_t<4096, 2>(a, BH, stream);
  else                   launch_select_t<8192, 1>(a, BH, stream);
  return hipGetLastError();
}

// ------------------------------------------------------------------ column lists
__global__ __launch_bounds__(256) void columns_kernel(const uint8_t* mask, int Tm, int Tn, int32_t* col_cnt,
                                                      int32_t* col_idx) {
  const int bh = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= Tn) return;
  const uint8_t* mp = mask + (int64_t)bh * Tm * Tn + j;
  int32_t* out = col_idx + ((int64_t)bh * Tn + j) * Tm;
  int c = 0;
  for (int i = 0; i < Tm; ++i)
    if (mp[(int64_t)i * Tn]) out[c++] = i;
  col_cnt[(int64_t)bh * Tn + j] = c;
}

hipError_t launch_columns(const uint8_t* mask, const Dims& m, int32_t* col_cnt, int32_t* col_idx,
                          hipStream_t stream) {
  const dim3 grid((unsigned)((m.Tn + 255) / 256), (unsigned)(m.B * m.H)), block(256);
  hipLaunchKernelGGL(columns_kernel, grid, block, 0, stream, mask, m.Tm, m.Tn, col_cnt, col_idx);
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
__global__ __launch_bounds__(256) void full_cols_kernel(int Tm, int Tn, int32_t* col_cnt, int32_t* col_idx) {
  const int64_t colr = blockIdx.x;  // bh * Tn + j
  for (int i = threadIdx.x; i < Tm; i += 256) col_idx[colr * Tm + i] = i;
  if (threadIdx.x == 0) col_cnt[colr] = Tm;
}

hipError_t launch_pattern_full(const Dims& m, uint8_t* mask, int32_t* row_cnt, int32_t* row_idx,
                               int32_t* col_cnt, int32_t* col_idx, hipStream_t stream) {
  const int BH = m.B * m.H;
  hipLaunchKernelGGL(full_rows_kernel, dim3((unsigned)(BH * m.Tm)), dim3(256), 0, stream, m.Tm, m.Tn, mask,
                     row_cnt, row_idx);
  if (col_cnt)
    hipLaunchKernelGGL(full_cols_kernel, dim3((unsigned)(BH * m.Tn)), dim3(256), 0, stream, m.Tm, m.Tn, col_cnt,
                       col_idx);
  return hipGetLastError();
}

}  // namespace spa2
