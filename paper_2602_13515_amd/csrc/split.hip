// Splitting of long rows (columns) of the block pattern over several workgroups.
//
// One workgroup walks one row of the pattern in the forward and dQ kernels (one column in the dK/dV kernel), so a
// launch cannot finish before its longest row has.  On a layer with few rows per workgroup slot the longest rows
// (Top-p-bound rows are ten times the Top-k length) then set the time.  This plan cuts every list longer than S
// entries into parts of S entries.  Part 0 stays with the row's own workgroup, parts >= 1 are given to extra
// workgroups at the front of the same launch; every part leaves an fp32 partial result in a pool slot and a small
// merge kernel combines the parts of a row in part order, so results do not depend on the order of execution.
//
// The plan is computed on the device from the list lengths (the host never reads the pattern):
//   T = total number of list entries of the launch,  S = max(min_part, ceil(T / 2048)),
// i.e. a part is at most a quarter of the mean work of one of the 512 workgroup slots; on large launches S exceeds
// every list and nothing is split.  Split units are taken in unit order for as long as pool slots last.
#include "spa2_device.h"
#include "spa2_internal.h"

namespace spa2 {

namespace {
inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
}

// Pool sizes are powers of two from 8 to SPLIT_POOL_MAX (a multiple of 8 keeps the workgroup -> XCD phase of the
// launch that the extra parts are put in front of).
static int64_t pool_wanted(int64_t units) {
  int64_t pool = 8;
  while (pool < SPLIT_POOL_MAX && pool < 4 * units) pool *= 2;
  return pool;
}

int split_pool_slots(int64_t units, size_t slot_bytes, size_t ws_bytes) {
  // shrink the pool if the caller gave less than the full workspace
  for (int64_t pool = pool_wanted(units); pool >= 8; pool /= 2) {
    const size_t need = 256 + up256((size_t)units * 4) + up256((size_t)pool * 8) + up256((size_t)pool * 4) +
                        (size_t)pool * slot_bytes;
    if (need <= ws_bytes) return (int)pool;
  }
  return 0;
}

size_t split_ws_bytes(int64_t units, size_t slot_bytes) {
  const int64_t pool = pool_wanted(units);
  return 256 + up256((size_t)units * 4) + up256((size_t)pool * 8) + up256((size_t)pool * 4) + (size_t)pool * slot_bytes;
}

SplitPlan split_layout(void* ws, size_t ws_bytes, int64_t units, size_t slot_bytes) {
  SplitPlan p;
  p.pool_slots = ws ? split_pool_slots(units, slot_bytes, ws_bytes) : 0;
  if (p.pool_slots == 0) { p.header = nullptr; p.unit_slot = nullptr; p.part_table = nullptr; p.merge_table = nullptr; p.pool = nullptr; p.slot_floats = 0; return p; }
  char* c = (char*)ws;
  p.header = (int32_t*)c;                 c += 256;
  p.unit_slot = (int32_t*)c;              c += up256((size_t)units * 4);
  p.part_table = (int32_t*)c;             c += up256((size_t)p.pool_slots * 8);
  p.merge_table = (int32_t*)c;            c += up256((size_t)p.pool_slots * 4);
  p.pool = (float*)c;
  p.slot_floats = (int)(slot_bytes / 4);
  return p;
}

// One workgroup of 1024 threads walks the units 1024 at a time (coalesced loads): first the total T, then, tile by
// tile, an exclusive prefix sum over the units of (pool slots, extra parts, split units), carried from tile to tile.
__device__ __forceinline__ int wave_incl_scan(int x, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  return x;
}

__global__ __launch_bounds__(1024) void split_plan_kernel(const int32_t* cnt, int units, int cnt_max, int pool,
                                                          int min_part, int32_t* header, int32_t* unit_slot,
                                                          int32_t* part_table, int32_t* merge_table) {
  constexpr int UPT = 8;                                   // consecutive units per thread and tile (two 16-byte loads)
  __shared__ unsigned long long tot_s[16];
  __shared__ int wsum[3][16];
  __shared__ int n_extra_s, n_split_s;
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  if (t == 0) { n_extra_s = 0; n_split_s = 0; }
  const bool vec_ok = ((uintptr_t)cnt & 15) == 0;
  auto load4 = [&](int u, int (&c)[UPT]) {                 // lengths of units u .. u+UPT-1 (0 past the end), clamped
    if (vec_ok && u + UPT <= units) {
      typedef __attribute__((ext_vector_type(4))) int i32x4;
      const i32x4 a = *(const i32x4*)(cnt + u), b = *(const i32x4*)(cnt + u + 4);
#pragma unroll
      for (int x = 0; x < 4; ++x) { c[x] = min(max(a[x], 0), cnt_max); c[4 + x] = min(max(b[x], 0), cnt_max); }
    } else {
#pragma unroll
      for (int x = 0; x < UPT; ++x) c[x] = u + x < units ? min(max(cnt[u + x], 0), cnt_max) : 0;
    }
  };
  unsigned long long mine = 0;
  for (int u = UPT * t; u < units; u += UPT * 1024) {
    int c[UPT]; load4(u, c);
#pragma unroll
    for (int x = 0; x < UPT; ++x) mine += (unsigned long long)c[x];
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mine += __shfl_xor(mine, off, 64);
  if (lane == 0) tot_s[wv] = mine;
  __syncthreads();
  long long T = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) T += (long long)tot_s[i];
  const int S = (int)max((long long)min_part, (T + 2047) / 2048);

  int base_slot = 0, base_extra = 0, base_split = 0;     // running totals of the tiles before this one
  for (int u0 = 0; u0 < units; u0 += UPT * 1024) {
    const int u = u0 + UPT * t;
    int c[UPT], parts[UPT]; load4(u, c);
    int v0 = 0, v1 = 0, v2 = 0;
#pragma unroll
    for (int x = 0; x < UPT; ++x) {
      parts[x] = c[x] > S ? (c[x] + S - 1) / S : 0;
      v0 += parts[x]; v1 += parts[x] ? parts[x] - 1 : 0; v2 += parts[x] ? 1 : 0;
    }
    const int i0 = wave_incl_scan(v0, lane), i1 = wave_incl_scan(v1, lane), i2 = wave_incl_scan(v2, lane);
    __syncthreads();                                     // (the sums of the previous tile have been read)
    if (lane == 63) { wsum[0][wv] = i0; wsum[1][wv] = i1; wsum[2][wv] = i2; }
    __syncthreads();
    int p0 = 0, p1 = 0, p2 = 0, t0 = 0, t1 = 0, t2 = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (i < wv) { p0 += wsum[0][i]; p1 += wsum[1][i]; p2 += wsum[2][i]; }
      t0 += wsum[0][i]; t1 += wsum[1][i]; t2 += wsum[2][i];
    }
    int slot = base_slot + p0 + i0 - v0, ex = base_extra + p1 + i1 - v1, ns = base_split + p2 + i2 - v2;
#pragma unroll
    for (int x = 0; x < UPT; ++x) {
      if (u + x >= units) break;
      int s = -1;
      if (parts[x]) {
        if (slot + parts[x] <= pool) {   // (slot only grows: the accepted units are a prefix of the split ones)
          s = slot;
          for (int p = 1; p < parts[x]; ++p) { part_table[2 * (ex + p - 1)] = u + x; part_table[2 * (ex + p - 1) + 1] = p; }
          merge_table[ns] = u + x;
          // the last accepted unit fixes the counts: every accepted unit reports, the largest values win
          atomicMax(&n_extra_s, ex + parts[x] - 1);
          atomicMax(&n_split_s, ns + 1);
        }
        slot += parts[x]; ex += parts[x] - 1; ++ns;
      }
      unit_slot[u + x] = s;
    }
    base_slot += t0; base_extra += t1; base_split += t2;
  }
  __syncthreads();
  if (t == 0) { header[0] = n_extra_s; header[1] = S; header[2] = n_split_s; }
}

hipError_t launch_split_plan(const int32_t* cnt, int64_t units, int cnt_max, int min_part, const SplitPlan& p,
                             hipStream_t stream) {
  if (p.pool_slots == 0) return hipSuccess;
  hipLaunchKernelGGL(split_plan_kernel, dim3(1), dim3(1024), 0, stream, cnt, (int)units, cnt_max, p.pool_slots,
                     min_part, (int32_t*)p.header, (int32_t*)p.unit_slot, (int32_t*)p.part_table,
                     (int32_t*)p.merge_table);
  return hipGetLastError();
}

}  // namespace spa2
