// Error of sparse attention against full attention, split into its two parts (Sec. 3.1).
//
// For one query row with full weights p, mask m, retained mass tau = sum_j p_j m_j, full output o = pV and
// sparse output o_s = (p.m / tau) V the paper writes  o - o_s = (p.(1-m)) V + (1 - 1/tau)(p.m) V, i.e.
//   dropped error         = o - tau o_s
//   renormalisation error = (tau - 1) o_s
// and tau is available from the two log-sum-exps: tau = exp(LSE_sparse - LSE_full).  The kernel below reads
// both outputs and both LSE vectors once (HBM-bound) and returns per (batch, head) the L1 norms of the total
// error, of o, of the two parts, and the sum of tau over the rows.  The reduction order is fixed
// (per-workgroup partial sums, then one thread per result walks them in order), so results are deterministic.
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

constexpr int DIAG_ROWS = 256;      // query rows per workgroup
constexpr int DIAG_TERMS = 5;

struct DiagArgs {
  const uint16_t* o_s; const uint16_t* o_f; const float* lse_s; const float* lse_f;
  double* part;          // [B*H, chunks, 5]
  int H, N, chunks;
  int64_t sb, sh, sn;
};

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

template <int D>
__global__ __launch_bounds__(256) void error_terms_kernel(DiagArgs a) {
  constexpr int CPR = D / 8;                  // 16-byte chunks per row
  constexpr int RPP = 256 / CPR;              // rows per pass of the workgroup
  __shared__ double red[4][DIAG_TERMS];
  const int bh = blockIdx.y, chunk = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
  const int row0 = chunk * DIAG_ROWS;
  double acc[DIAG_TERMS] = {0.0, 0.0, 0.0, 0.0, 0.0};
  for (int r = tid / CPR; r < DIAG_ROWS; r += RPP) {
    const int row = row0 + r;
    if (row >= a.N) break;
    const int64_t off = base + (int64_t)row * a.sn + (tid % CPR) * 8;
    const u32x4 us = *(const u32x4*)(a.o_s + off);
    const u32x4 uf = *(const u32x4*)(a.o_f + off);
    const float tau = __expf(a.lse_s[(int64_t)bh * a.N + row] - a.lse_f[(int64_t)bh * a.N + row]);
    float e_tot = 0.f, e_ref = 0.f, e_drop = 0.f, e_ren = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const float os = h ? bf16_hi(us[c]) : bf16_lo(us[c]);
        const float of = h ? bf16_hi(uf[c]) : bf16_lo(uf[c]);
        e_tot += fabsf(of - os);
        e_ref += fabsf(of);
        e_drop += fabsf(of - tau * os);
        e_ren += fabsf((tau - 1.f) * os);
      }
    }
    acc[0] += (double)e_tot; acc[1] += (double)e_ref; acc[2] += (double)e_drop; acc[3] += (double)e_ren;
    if (tid % CPR == 0) acc[4] += (double)tau;
  }
  // wave reduction (fixed butterfly order), then the four waves in order
#pragma unroll
  for (int k = 0; k < DIAG_TERMS; ++k) {
    double v = acc[k];
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
    if (lane == 0) red[w][k] = v;
  }
  __syncthreads();
  if (tid < DIAG_TERMS)
    a.part[((int64_t)bh * a.chunks + chunk) * DIAG_TERMS + tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
}

__global__ void error_terms_finish(const double* part, int chunks, double* out) {
  const int bh = blockIdx.x, k = threadIdx.x;
  if (k >= DIAG_TERMS) return;
  double s = 0.0;
  for (int c = 0; c < chunks; ++c) s += part[((int64_t)bh * chunks + c) * DIAG_TERMS + k];
  out[(int64_t)bh * DIAG_TERMS + k] = s;
}

size_t error_ws_bytes(const Dims& m) {
  const size_t chunks = (size_t)(m.N + DIAG_ROWS - 1) / DIAG_ROWS;
  return (size_t)m.B * m.H * chunks * DIAG_TERMS * sizeof(double);
}

hipError_t launch_error_terms(const void* o_sparse, const void* o_dense, const float* lse_sparse,
                              const float* lse_dense, const Dims& m, double* out, void* ws, hipStream_t stream) {
  DiagArgs a;
  a.o_s = (const uint16_t*)o_sparse; a.o_f = (const uint16_t*)o_dense; a.lse_s = lse_sparse; a.lse_f = lse_dense;
  a.part = (double*)ws;
  a.H = m.H; a.N = m.N; a.chunks = (m.N + DIAG_ROWS - 1) / DIAG_ROWS;
  a.sb = m.sb; a.sh = m.sh; a.sn = m.sn;
  const dim3 grid((unsigned)a.chunks, (unsigned)(m.B * m.H)), block(256);
  if (m.d == 128) hipLaunchKernelGGL(error_terms_kernel<128>, grid, block, 0, stream, a);
  else            hipLaunchKernelGGL(error_terms_kernel<64>, grid, block, 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(error_terms_finish, dim3((unsigned)(m.B * m.H)), dim3(64), 0, stream, (const double*)ws, a.chunks, out);
  return hipGetLastError();
}

}  // namespace spa2
