// Helpers shared by the tiled (matrix-core) verify-attention kernels: operand types, the
// hand-placed synchronisation primitives of the direct-to-LDS tile ring, bf16 packing.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "seer_device.h"

namespace seer {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define SEER_AS1 __attribute__((address_space(1)))
#define SEER_AS3 __attribute__((address_space(3)))

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 v = {lo, hi};
    bf16x2 r = __builtin_convertvector(v, bf16x2);   // round-to-nearest-even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(uint32_t, r);
}

// acc + lo + hi of a packed pair of bf16 values, in fp32 (v_dot2_f32_bf16 against the pair (1, 1)): the sum of
// the probabilities exactly as the P.V matrix product will see them, in one instruction per pair.
__device__ __forceinline__ float add_bf16_pair(uint32_t pair, float acc) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
}

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at "do not wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
// Workgroup barrier WITHOUT the memory fences of __syncthreads(): a fence (even one scoped to
// LDS) makes the compiler drain every outstanding load, including the direct-to-LDS loads of
// the tiles still in flight, which is exactly what the ring of stages exists to avoid.  The
// kernel orders its LDS traffic by hand instead: wait_vmcnt for the tile about to be read, then
// this barrier; LDS reads of a stage are complete (their results consumed by MFMAs) before the
// wave reaches the barrier after which that stage is overwritten.
__device__ __forceinline__ void bare_barrier() { __builtin_amdgcn_s_barrier(); }
// A workgroup-uniform 32-bit value read from global memory, moved to a scalar register.  The
// hand-placed fences keep the compiler from proving such loads invariant, so it issues them as
// vector loads; without this the control flow that depends on them would be treated as divergent.
__device__ __forceinline__ int uniform_load(const int32_t* p) { return __builtin_amdgcn_readfirstlane(*p); }

}  // namespace seer
