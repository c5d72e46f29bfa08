// Device-side pieces shared by the attention kernels: vector types, tile geometry in LDS, the
// direct global -> LDS copy and the exchange between the two halves of a wave.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mc_types.h"

namespace mc {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#define MC_LDS __attribute__((address_space(3)))

constexpr int kWaves = 8;              // waves of a workgroup: two per SIMD, 32 stacked rows each
static_assert(kWaves * 32 == kAttnTileRows, "the host cuts the work list into tiles of kAttnTileRows rows");
constexpr int kTileKeys = kAttnTileKeys;   // keys per LDS tile = 4 pages of 16
constexpr int kPageTokens = 16;
constexpr int kRowBytes = 256;         // one K or V row: 128 bf16 or 64 f32
constexpr int kPageHeadBytes = kPageTokens * kRowBytes;   // 4 KiB, contiguous in the pool
constexpr int kKTileBytes = kTileKeys * kRowBytes;        // 16 KiB; rows dense, granules swizzled
constexpr int kVTileBytes = kTileKeys * kRowBytes;
constexpr int kBuffers = 3;
// LDS: the K tiles of the three buffers, then the V tiles.  Every tile starts at a multiple of
// 16 KiB, so the XOR constants of the swizzle (< 256) never reach a tile base, and the offset of
// any fragment from its lane's base register stays below the 64 KiB a ds_read immediate can hold.
constexpr int kVBase = kBuffers * kKTileBytes;
constexpr float kRescaleSlack = 8.0f;  // log2 units the running max may lag behind
// stands in for a reference of -inf when probabilities are formed: masked scores (-inf) then give
// exp2(-inf) = 0 instead of exp2(-inf + inf) = NaN; a row with a finite score has a finite reference
constexpr float kNoKeyYet = -1e30f;

// Combine a value with the one held by lane ^ 32.  v_permlane32_swap exchanges the upper
// half of its first register with the lower half of its second, so after it every lane
// holds its own value in one register and its partner's in the other; max and sum do not
// care which is which.  Written as asm with two distinct read-write registers (the builtin
// called with one value for both operands gets its two results merged by the optimiser);
// the s_nop covers the VALU-write -> permlane read hazard the compiler cannot see.
__device__ __forceinline__ void swap_halves(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float max_with_other_half(float x) {
  float a = x, b = x;
  swap_halves(a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  float a = x, b = x;
  swap_halves(a, b);
  return a + b;
}

// Direct global -> LDS copy of 16 bytes per lane: lane i's bytes land at lds_base + 16*i
// (lds_base wave-uniform, it travels in M0).  Written as asm so that the compiler does not
// know LDS is being written behind its back: it would otherwise make the first LDS read
// after the copy wait for the copy (vmcnt), which is exactly what the tile pipeline avoids.
// Ordering is the kernel's own business: s_waitcnt vmcnt(0) + barrier before a tile is read.
// (M0 is a register the compiler reserves for itself; it sets it right before each of its own
// uses and has none in this kernel, so naming it as clobbered is all that is needed - the
// diagnostic about reserved registers in a clobber list is expected here.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const char* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
               :: "s"(sbase), "v"(voff), "s"(lds_base) : "m0", "memory");
}
__device__ __forceinline__ void dma16(const char* vaddr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(vaddr), "s"(lds_base) : "m0", "memory");
}
#pragma clang diagnostic pop

}  // namespace
}  // namespace mc
