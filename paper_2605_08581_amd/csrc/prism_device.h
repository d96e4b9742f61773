// Device-side helpers shared by the attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>

#include "prism_internal.h"

namespace prism {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int D>
__device__ __forceinline__ int swz(int key) {
  if (D == 128) return ((key & 3) << 2) | ((key >> 2) & 3);
  return (((key >> 1) & 1) << 2) | ((key >> 2) & 3);
}

template <int D>
__device__ __forceinline__ int lds_off(int key, int chunk) {   // byte offset of a 16-byte chunk
  return key * (D * 2) + ((chunk ^ swz<D>(key)) << 4);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max over the two 32-lane halves of a wave, result in every lane
__device__ __forceinline__ float max_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16 bytes per lane from global memory straight into LDS: lane l's data lands
// at lds_base + 16*l (lds_base is wave-uniform and travels in M0).  The source
// is a buffer resource (wave-uniform base of one (page, head) block, in scalar
// registers) plus a per-lane byte offset, which keeps all address arithmetic
// off the vector ALU and makes a stray offset read zeros instead of faulting.
// Inline assembly, so that the compiler does not make later LDS reads of
// *other* slots wait for these copies; the kernel waits for them itself
// (s_waitcnt vmcnt(0), then a workgroup barrier) before a slot is read.
typedef __attribute__((ext_vector_type(4))) int32_t i32x4;
__device__ __forceinline__ i32x4 block_resource(const void *base, uint32_t bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)base;
  i32x4 r;
  r[0] = (int32_t)(uint32_t)a;
  r[1] = (int32_t)(uint32_t)((a >> 32) & 0xFFFFu);   // stride 0: a raw byte buffer
  r[2] = (int32_t)bytes;                             // offsets at or past this read as zero
  r[3] = 0x00020000;                                 // 32-bit untyped data
  return r;
}
__device__ __forceinline__ void copy16_to_lds(i32x4 rsrc, uint32_t lane_off, uint32_t lds_base) {
  // wave-uniform by construction; say so, in case the value was computed on the vector ALU
#pragma unroll
  for (int i = 0; i < 4; ++i) rsrc[i] = __builtin_amdgcn_readfirstlane(rsrc[i]);
  lds_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_base);
  // M0 (the LDS destination) is written and consumed inside this one statement.
  // The compiler rejects M0 in a clobber list (a reserved register), so the
  // kernels that copy this way use nothing for which the compiler would set
  // M0 itself (no LDS-DMA builtins, no indexed register moves, no messages);
  // tests/test_kernel_assembly.py checks the generated code for that.
  __asm__ volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %0, 0 offen lds"
                   :
                   : "s"(rsrc), "v"(lane_off), "s"(lds_base)
                   : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

constexpr float kRescaleThreshold = 8.0f;   // log2 units

// O^T += V^T P^T.  With 64 rows per wave the O^T accumulators (128 registers at
// d = 128) live in accumulation registers for the whole kernel while the score
// tiles, which the vector ALU works on, stay in ordinary registers; the
// compiler picks one register kind for every MFMA of a function, so this one
// is written out.  Only MFMAs and the (fenced) rescale and epilogue touch the
// accumulators.
template <bool ACC>
__device__ __forceinline__ void pv_mfma(f32x16 &o, bf16x8 a, bf16x8 b) {
  if constexpr (ACC) {
    __asm__ volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(a), "v"(b));
  } else {
    o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o, 0, 0, 0);
  }
}
// Wait until every MFMA issued so far has written its result (the longest one
// here takes 8 passes of 4 cycles): needed before accumulators written by
// pv_mfma<true> are read by anything but another MFMA.
__device__ __forceinline__ void mfma_drain() {
  __builtin_amdgcn_sched_barrier(0);
  __asm__ volatile("s_nop 15\n\ts_nop 3");
  __builtin_amdgcn_sched_barrier(0);
}


// f(integral_constant<int, B>) ... f(integral_constant<int, E-1>), expanded at
// compile time: the body sees its index as a constant expression.
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

// Launch with the launch's own status as the return value: reading the
// runtime's last-error slot instead would also return, and clear, an error
// that an earlier call of the caller's left there.
template <class... Params, class... Args>
inline int launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                         Args... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "argument count");
  std::tuple<Params...> values{static_cast<Params>(args)...};
  void *ptrs[sizeof...(Params)];
  int i = 0;
  std::apply([&](auto &...v) { ((ptrs[i++] = (void *)&v), ...); }, values);
  return (int)hipLaunchKernel((const void *)kernel, grid, block, ptrs, lds_bytes, stream);
}

}  // namespace prism
