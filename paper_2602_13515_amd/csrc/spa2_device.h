// Device-side helpers shared by the spa2 kernels (gfx950 / CDNA4, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spa2 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// address-space qualified pointers of the direct global -> LDS copy builtin
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

constexpr int BQ = 128;
constexpr int BKV = 64;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Operand layout of the bf16 MFMA shape used here (lane l of a wave64):
//   32x32x16:  A[m][k]: m = l%32, k = 8*(l/32)+s (s=0..7)   B[k][n]: n = l%32, same k
//              C[m][n]: n = l%32, m = 8*(v/4) + 4*(l/32) + v%4 for accumulator register v = 0..15
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// compile-time loop: f(Int<B>{}), ..., f(Int<E-1>{})
template <int I> struct Int { static constexpr int v = I; };
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) { f(Int<B>{}); static_for<B + 1, E>(f); }
}

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes,
// lane s supplies the address of four consecutive 16-bit elements; lane i of
// the group receives element (i%4) of the data addressed by lanes i/4, 4+i/4,
// 8+i/4, 12+i/4.  If lane s points at row (s/4), columns 4*(s%4).. of a
// row-major tile, lane i ends up with column i of rows 0..3: a 4x16 patch read
// column-wise, which is what an MFMA operand needs when the contraction index
// is the row of the tile in memory.
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
__device__ __forceinline__ u32x2 lds_read_tr4(const uint16_t* lds_ptr) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lds_ptr));
  return __builtin_bit_cast(u32x2, v);
}
__device__ __forceinline__ bf16x8 join_tr(u32x2 lo, u32x2 hi) {
  u32x4 u = {lo[0], lo[1], hi[0], hi[1]};
  return __builtin_bit_cast(bf16x8, u);
}

// Exchange between the two 32-lane halves of a wave on the vector ALU (v_permlane32_swap), without a trip
// through LDS: max / sum of the values that lanes l and l^32 hold, in both lanes.
__device__ __forceinline__ void both_halves(float x, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = __builtin_bit_cast(float, (uint32_t)r[0]);
  hi = __builtin_bit_cast(float, (uint32_t)r[1]);
}
__device__ __forceinline__ float max_halves(float x) { float lo, hi; both_halves(x, lo, hi); return fmaxf(lo, hi); }
__device__ __forceinline__ float sum_halves(float x) { float lo, hi; both_halves(x, lo, hi); return lo + hi; }

// acc + lo(p) + hi(p) for a packed bf16 pair p, accumulated in fp32 (v_dot2c_f32_bf16 with a pair of ones)
__device__ __forceinline__ float dot2_ones(uint32_t p, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, p), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc,
                                         false);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Direct global -> LDS copy, 16 bytes per lane: lane l's bytes land at lds_dst + 16 l (lds_dst wave-uniform);
// the source is a wave-uniform base plus a 32-bit byte offset per lane.  Issued as an assembly statement so
// that the compiler's wait-count insertion does not see it: through the builtin, LDS reads that follow a copy
// are made to wait for it (the two cannot be told apart by address).  The caller therefore owns the
// ordering: raw_copies_done() before the barrier that publishes the tile.  In-order completion of vector
// memory operations keeps the compiler's own counted waits safe (they can only wait for more, never less).
// m0 carries the LDS address and is declared clobbered; a kernel that uses this helper must not also rely on
// the compiler keeping a value of its own in m0 across it (the builtin form of the same copy would).
__device__ __forceinline__ void raw_copy16_to_lds(const void* src_base, uint32_t src_off, const uint16_t* lds_dst) {
#if defined(__HIP_DEVICE_COMPILE__)      // (the host pass of hipcc parses device functions too and knows no m0)
  // (wave-uniform by contract; the lane read makes that visible to the register allocator)
  const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lptr_t*)lds_dst);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(src_off), "s"(src_base) : "memory", "m0");
#endif
}
__device__ __forceinline__ void raw_copies_done() {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
}

// LDS accesses by 32-bit byte address.  A generic pointer into LDS is turned into its LDS address once
// (lds_addr_of); from then on addresses are plain integers, so that address arithmetic stays 32-bit and constant
// parts can be folded into the instructions' offset fields, and no generic-pointer null checks are generated.
typedef __attribute__((address_space(3))) const bf16x8 lds_cbf16x8;
typedef __attribute__((address_space(3))) const f32x4 lds_cf32x4;
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) { return (uint32_t)(size_t)(lptr_t*)p; }
#if defined(__HIP_DEVICE_COMPILE__)      // (LDS pointers are 32 bits wide only in the device pass)
__device__ __forceinline__ bf16x8 lds_ld16(uint32_t addr) { return *(lds_cbf16x8*)addr; }
__device__ __forceinline__ f32x4 lds_ldf4(uint32_t addr) { return *(lds_cf32x4*)addr; }
__device__ __forceinline__ u32x2 lds_tr4_at(uint32_t addr) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)addr);
  return __builtin_bit_cast(u32x2, v);
}
#else
__device__ bf16x8 lds_ld16(uint32_t addr);
__device__ f32x4 lds_ldf4(uint32_t addr);
__device__ u32x2 lds_tr4_at(uint32_t addr);
#endif
// Direct global -> LDS copies as above, with the (wave-uniform) LDS byte address given as an integer.
// LDS_CONST is a compile-time part of the destination that is added while m0 is written.
template <int LDS_CONST>
__device__ __forceinline__ void raw_copy16_to_lds_at(const void* src_base, uint32_t src_off, uint32_t lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_addr), "v"(src_off), "s"(src_base), "n"(LDS_CONST) : "memory", "m0", "scc");
#endif
}
template <int LDS_CONST>
__device__ __forceinline__ void raw_copy4_to_lds_at(const void* src_base, uint32_t src_off, uint32_t lds_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :: "s"(lds_addr), "v"(src_off), "s"(src_base), "n"(LDS_CONST) : "memory", "m0", "scc");
#endif
}

// XOR-swizzled LDS tile: rows of D bf16, unpadded; the 16-byte chunk c of row r lives at chunk position
// c ^ swz<D>(r).  The function is chosen so that BOTH access patterns the kernels use are free of bank
// conflicts (64 banks x 4 bytes): 16 lanes reading the same chunk of 16 consecutive rows (MFMA operand read
// along rows), and 32 lanes reading 64 contiguous bytes of each of 4 consecutive rows (transposing read).
template <int D> __device__ __forceinline__ int swz(int r);
template <> __device__ __forceinline__ int swz<128>(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
template <> __device__ __forceinline__ int swz<64>(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }
// element index of logical (row, col) in a swizzled tile
template <int D> __device__ __forceinline__ int swz_idx(int row, int col) {
  return row * D + ((((col >> 3) ^ swz<D>(row))) << 3) + (col & 7);
}

// Workgroup id -> (head, block) mapping that keeps one head's blocks resident
// on all eight XCDs at once: consecutive workgroup ids go round-robin to the
// XCDs, so XCD x receives ids x, x+8, ...; those are given a contiguous chunk
// of the head's blocks, which share K/V tiles through that XCD's L2.
struct HeadBlock { int bh; int blk; bool valid; };
__device__ __forceinline__ HeadBlock xcd_map(int wg, int blocks_per_head, int chunk) {
  const int xcd = wg & 7;
  const int slot = wg >> 3;
  HeadBlock r;
  r.bh = slot / chunk;
  r.blk = xcd * chunk + slot % chunk;
  r.valid = r.blk < blocks_per_head;
  return r;
}

}  // namespace spa2
