// Small device-side helpers shared by the HIP kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace heatkv {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

// 2^x on the transcendental unit; 2^-inf = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Value of lane (l ^ 32): the partner in the other half of the wavefront.
__device__ __forceinline__ float swap_halves(float v) { return __shfl_xor(v, 32, 64); }

// Reductions over the two halves of a wavefront (lane l with lane l ^ 32) with one v_permlane32_swap.
// The instruction exchanges the upper half of its first register with the lower half of its second, in
// place; fed two copies of v it leaves {lower-half values on all lanes, upper-half values on all lanes}.
// It is issued through inline assembly with two read-write operands: the compiler builtin of this
// toolchain folds its two results into one register.  The leading s_nop covers the wait states the
// instruction needs after a vector-ALU write of its operands.
__device__ __forceinline__ void split_halves(float v, float& lower, float& upper) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  lower = a;
  upper = b;
}
__device__ __forceinline__ float max_halves(float v) {
  float a, b;
  split_halves(v, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_halves(float v) {
  float a, b;
  split_halves(v, a, b);
  return a + b;
}

// s_waitcnt on the vector-memory counter alone (at most N loads outstanding), as an instruction the compiler
// sees.  The tile copies of the bf16 kernels are issued as text the compiler does not look into, so it does not
// count them, but the hardware counter does: a wait the compiler adds for one of ITS loads (the query rows, say)
// then also waits for every tile copy issued before that point.  Where such a load may still be outstanding on
// some path into a loop, the compiler repeats those waits in every iteration, i.e. in the middle of the math
// right after the next tiles' copies went out.  A visible full wait at a point where the kernel waits anyway
// tells it that nothing of its own is outstanding any more.
// Encoding (gfx9 family): vmcnt[3:0] in bits 3:0 and vmcnt[5:4] in bits 15:14; expcnt (bits 6:4) and lgkmcnt
// (bits 11:8) stay at their maxima, which means no wait on them.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

__device__ __forceinline__ uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// A 64-bit LDS read that transposes 16-bit elements inside each group of 16
// lanes: the 16 lanes address a 4 x 16 block (lane i points at row i/4, columns
// 4*(i%4)..+3) and lane i receives column i, rows 0..3.
__device__ __forceinline__ s16x4 lds_read_tr16(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(reinterpret_cast<const short*>(p)));
}

}  // namespace heatkv
