// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define STS_WAVE 64

__device__ __forceinline__ float bf2f(bf16 x) { return (float)x; }
__device__ __forceinline__ bf16 f2bf(float x) { return (bf16)x; }   // round to nearest even

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wave writes at
// lds_dst + 16 * l (lds_dst must be wave-uniform); completion is counted by vmcnt. Buffers filled
// this way are kept 1 KB above LDS address 0.
__device__ __forceinline__ void load_to_lds16(const void* gsrc, void* lds_dst) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_dst, 16, 0, 0);
#endif
}
// The same with the non-temporal hint: for bytes that are read once.
__device__ __forceinline__ void load_to_lds16_nt(const void* gsrc, void* lds_dst) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_dst, 16, 0, 2);
#endif
}
// The same transfer with the address given as a wave-uniform base plus a 32-bit byte offset per lane
// (the scalar-base form of the instruction: 4 address bytes per lane travel to the memory pipeline
// instead of 8, and advancing along K is scalar arithmetic). lds_dst must be wave-uniform. The
// compiler does not see this load: the caller orders it against LDS reads with wait_vmem and a
// barrier, as for load_to_lds16.
__device__ __forceinline__ void lds_dma16(const void* base, unsigned lane_off, void* lds_dst) {
#if defined(__HIP_DEVICE_COMPILE__)
  const unsigned m = (unsigned)(size_t)(__attribute__((address_space(3))) void*)lds_dst;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(m) : "memory");
#endif
}
// Wait until at most N of this wave's vector-memory loads are outstanding (they complete in
// order); the other counters are left alone.
template <int N>
__device__ __forceinline__ void wait_vmem() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
#endif
}

// Workgroup id -> work item so that the workgroups resident on one XCD (hardware hands
// consecutive ids to the 8 XCDs in turn) get a contiguous range of items and share its L2.
__device__ __forceinline__ int xcd_contiguous(int bid, int per_xcd) { return (bid & 7) * per_xcd + (bid >> 3); }
