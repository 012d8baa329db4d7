// Device helpers shared by the pipelined attention kernels (attn_pipe.hip, attn_duo.hip): vector
// types, the geometry of a 32-key sub-tile in LDS, compile-time loops, the lane-half exchange,
// pool -> LDS requests, and the two LDS operand reads.
#pragma once
#include "calvo_internal.h"

namespace calvo {
namespace attn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) unsigned char lds_u8;

constexpr int kD = 128;
constexpr int kSK = 32;                        // keys per sub-tile / ring slot
constexpr int kRow = 256;                      // bytes per token row of one head
constexpr int kSlot = kSK * kRow;              // 8192
template <int V>
struct Tag { static constexpr int value = V; };
// f(Tag<B>{}), f(Tag<B+1>{}), ... f(Tag<E-1>{}): a loop whose index is a compile-time constant
template <int B, int E, typename F>
__device__ inline void static_for(F&& f) {
  if constexpr (B < E) {
    f(Tag<B>{});
    static_for<B + 1, E>(f);
  }
}
constexpr int kPD = 4;   // LDS operand reads run this many MFMAs ahead

// lanes [32,64) of a <-> lanes [0,32) of b (the compiler builtin for this instruction returns
// its first result twice, hence inline asm)
__device__ inline void half_swap(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ inline float half_swap_max(float v) {
  float a = v, b = v;
  half_swap(a, b);
  return fmaxf(a, b);
}
__device__ inline float half_swap_sum(float v) {
  float a = v, b = v;
  half_swap(a, b);
  return a + b;
}

// maximum / sum over the four lanes c, c+16, c+32, c+48 (the lanes that share a query): every lane
// of the wave must call these
__device__ inline float quad_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return half_swap_max(v);
}
__device__ inline float quad_sum(float v) {
  v += __shfl_xor(v, 16, 64);
  return half_swap_sum(v);
}

// 64 lanes x 16 bytes from global memory (uniform base + per-lane byte offset) to 1 KiB of LDS
// starting at lds_addr (uniform).  Completion is tracked by vmcnt.  No "memory" clobber on
// purpose: every read of the deposited data sits behind wait_vm + a workgroup barrier, and a
// clobber would stop the compiler from keeping the block-table loads on the scalar unit.
__device__ inline void dma_1k(const unsigned char* sbase, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(sbase), "s"(lds_addr));
}
// compiler-level fence for one value: it is 'rewritten' here, so its producers stay above this
// point and its consumers below it; emits no instruction
template <typename T>
__device__ inline void pin(T& x) {
  asm volatile("" : "+v"(x));
}
template <int N>
__device__ inline void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N));
}

__device__ inline bf16x8 read_k(const lds_u8* a) { return *(const __attribute__((address_space(3))) bf16x8*)a; }
// V^T operand of a 16x16x32 MFMA: four keys for the lane's d from the rows the 16-lane group points
// at, and four more from 16 rows further on
__device__ inline bf16x8 read_vt(const lds_u8* a) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a + 16 * kRow));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

}  // namespace attn
}  // namespace calvo
