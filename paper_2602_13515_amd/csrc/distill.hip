// Velocity distillation loss (Sec. 4.2; loss step of Alg. 2):  L_VD = weight * sum (u_sparse - u_full)^2  and its
// gradient with respect to the student's prediction,  upstream * 2 * weight * (u_sparse - u_full).
//
// Both kernels are one pass over the two predictions (HBM-bound: 2 reads per element for the loss, 2 reads and
// 1 write for the gradient), 16 bytes per lane and request.  The difference is taken in fp32, squared and summed
// in fp64; partial sums go workgroup by workgroup to the workspace and are added in a fixed order, so the loss is
// deterministic.
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

constexpr int VD_MAX_WGS = 2048;      // workgroups of the loss pass = partial sums kept in the workspace

__device__ __forceinline__ float vd_bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float vd_bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
// by value on purpose: a bit cast applied directly to an element of a vector type reads element 0
__device__ __forceinline__ float vd_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t vd_to_bf16(float x) {            // round to nearest even; NaN stays NaN
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// element e of a tensor of the given type, as fp32
template <bool BF16>
__device__ __forceinline__ float vd_scalar(const void* p, int64_t e) {
  if (BF16) return __builtin_bit_cast(float, (uint32_t)((const uint16_t*)p)[e] << 16);
  return ((const float*)p)[e];
}

// the differences of the 16-byte vector v of both tensors: 8 (bf16) or 4 (fp32) values
template <bool BF16>
__device__ __forceinline__ void vd_diffs(const void* us, const void* uf, int64_t v, float (&d)[8]) {
  const u32x4 a = ((const u32x4*)us)[v], b = ((const u32x4*)uf)[v];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (BF16) {
      d[2 * c] = vd_bf16_lo(a[c]) - vd_bf16_lo(b[c]);
      d[2 * c + 1] = vd_bf16_hi(a[c]) - vd_bf16_hi(b[c]);
    } else {
      d[c] = vd_f32(a[c]) - vd_f32(b[c]);
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void vd_loss_kernel(const void* us, const void* uf, int64_t n, double* part) {
  constexpr int VEC = BF16 ? 8 : 4;
  __shared__ double red[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t nvec = n / VEC;
  double acc = 0.0;
  for (int64_t v = (int64_t)blockIdx.x * 256 + tid; v < nvec; v += (int64_t)gridDim.x * 256) {
    float d[8];
    vd_diffs<BF16>(us, uf, v, d);
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc = fma((double)d[c], (double)d[c], acc);
  }
  if (blockIdx.x == 0 && nvec * VEC + tid < n) {                      // fewer than VEC elements are left over
    const float d = vd_scalar<BF16>(us, nvec * VEC + tid) - vd_scalar<BF16>(uf, nvec * VEC + tid);
    acc = fma((double)d, (double)d, acc);
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s, 64);
  if (lane == 0) red[w] = acc;
  __syncthreads();
  if (tid == 0) part[blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
}

__global__ __launch_bounds__(64) void vd_loss_finish(const double* part, int count, double weight, double* loss) {
  double s = 0.0;
  for (int c = threadIdx.x; c < count; c += 64) s += part[c];
#pragma unroll
  for (int k = 32; k >= 1; k >>= 1) s += __shfl_xor(s, k, 64);
  if (threadIdx.x == 0) *loss = weight * s;
}

template <bool BF16>
__global__ __launch_bounds__(256) void vd_grad_kernel(const void* us, const void* uf, int64_t n, double coef,
                                                      const double* upstream, void* grad) {
  constexpr int VEC = BF16 ? 8 : 4;
  const int tid = threadIdx.x;
  const int64_t nvec = n / VEC;
  const float g = (float)(upstream ? coef * *upstream : coef);
  for (int64_t v = (int64_t)blockIdx.x * 256 + tid; v < nvec; v += (int64_t)gridDim.x * 256) {
    float d[8];
    vd_diffs<BF16>(us, uf, v, d);
    u32x4 out;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (BF16) out[c] = vd_to_bf16(g * d[2 * c]) | (vd_to_bf16(g * d[2 * c + 1]) << 16);
      else      out[c] = __builtin_bit_cast(uint32_t, g * d[c]);
    }
    ((u32x4*)grad)[v] = out;
  }
  if (blockIdx.x == 0 && nvec * VEC + tid < n) {
    const int64_t e = nvec * VEC + tid;
    const float x = g * (vd_scalar<BF16>(us, e) - vd_scalar<BF16>(uf, e));
    if (BF16) ((uint16_t*)grad)[e] = (uint16_t)vd_to_bf16(x);
    else      ((float*)grad)[e] = x;
  }
}

static unsigned vd_grid(int64_t n, bool bf16) {
  const int64_t nvec = n / (bf16 ? 8 : 4);
  const int64_t wgs = (nvec + 255) / 256;
  return (unsigned)(wgs < 1 ? 1 : (wgs > VD_MAX_WGS ? VD_MAX_WGS : wgs));
}

size_t vd_ws_bytes() { return (size_t)VD_MAX_WGS * sizeof(double); }

hipError_t launch_vd_loss(const void* us, const void* uf, int64_t n, bool bf16, double weight, double* loss, void* ws,
                          hipStream_t stream) {
  const unsigned grid = vd_grid(n, bf16);
  if (bf16) hipLaunchKernelGGL(vd_loss_kernel<true>, dim3(grid), dim3(256), 0, stream, us, uf, n, (double*)ws);
  else      hipLaunchKernelGGL(vd_loss_kernel<false>, dim3(grid), dim3(256), 0, stream, us, uf, n, (double*)ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(vd_loss_finish, dim3(1), dim3(64), 0, stream, (const double*)ws, (int)grid, weight, loss);
  return hipGetLastError();
}

hipError_t launch_vd_grad(const void* us, const void* uf, int64_t n, bool bf16, double weight, const double* upstream,
                          void* grad, hipStream_t stream) {
  const unsigned grid = vd_grid(n, bf16);
  if (bf16) hipLaunchKernelGGL(vd_grad_kernel<true>, dim3(grid), dim3(256), 0, stream, us, uf, n, 2.0 * weight, upstream, grad);
  else      hipLaunchKernelGGL(vd_grad_kernel<false>, dim3(grid), dim3(256), 0, stream, us, uf, n, 2.0 * weight, upstream, grad);
  return hipGetLastError();
}

}  // namespace spa2
