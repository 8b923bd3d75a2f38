// Shared device/host helpers of the MoE hot-path library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "moe_hotpath.h"

#define MOE_WAVE 64

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// fp32 -> bf16 bits, round to nearest even (hardware conversion on gfx950).
__device__ __forceinline__ uint16_t f32_to_bf16(float v) {
  __bf16 b = static_cast<__bf16>(v);
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// two packed bf16 (low half = element 0) <-> two floats
__device__ __forceinline__ float bf16lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16hi(uint32_t p) { return __uint_as_float(p & 0xFFFF0000u); }
// one v_cvt_pk_bf16_f32 (round to nearest even, as the scalar conversion)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

static inline bool moe_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- launch bookkeeping (prof.hip) ----------------------------------------
// When profiling is on, brackets the launch with two events on `stream`.
struct MoeLaunchScope {
  MoeLaunchScope(const char* name, hipStream_t stream);
  ~MoeLaunchScope();
  int slot;
  hipStream_t stream;
};
int moe_check_launch();  // MOE_OK or MOE_ERR_LAUNCH from hipGetLastError()

#define MOE_LAUNCH(name, kernel, grid, block, shmem, stream, ...)              \
  do {                                                                         \
    MoeLaunchScope _scope(name, stream);                                       \
    hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);       \
  } while (0)
