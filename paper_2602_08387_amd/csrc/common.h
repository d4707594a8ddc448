// Shared device/host helpers for the gfx950 decoder-layer kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T) __attribute__((address_space(3))) T*

constexpr int kWave = 64;

// Sum / max across the 64 lanes of a wavefront; every lane receives the result.
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

// Logistic function from v_exp_f32 and v_rcp_f32 (about 1 ulp each; every use rounds the result to
// bf16 afterwards).  Written as a division it compiles to the correctly rounded sequence of some ten
// instructions per element, which the SwiGLU epilogues of the GEMMs (64 or 128 elements per lane and
// tile, the matrix pipe idle meanwhile) pay for in full.  Every SwiGLU kernel uses this one function,
// so the fused and the stand-alone paths give the same bits.
__device__ __forceinline__ float logistic(float z) { return __builtin_amdgcn_rcpf(1.0f + __expf(-z)); }

__device__ __forceinline__ void unpack8(const bf16x8& v, float (&f)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) f[i] = (float)v[i];
}
__device__ __forceinline__ bf16x8 pack8(const float (&f)[8]) {
  bf16x8 v;
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (bf16_t)f[i];
  return v;
}

// Host-side status plumbing (definitions in api.hip).
namespace dl {
int fail(int code, const char* fmt, ...);
int check_launch(const char* what);
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Raises a kernel's dynamic LDS limit, once per device: the attribute belongs to the device the call is
// made on, so a process that launches on a second GPU must set it there too.  `done` is the caller's
// (per kernel) bit mask of devices already served; threads may race to set the attribute (setting it
// twice is harmless), never on the mask.
template <typename K>
inline int reserve_lds(K kern, size_t bytes, std::atomic<unsigned long long>& done, const char* what) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return fail(-3, "%s: no current device", what);
  if ((done.load(std::memory_order_acquire) >> dev) & 1ull) return 0;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return fail(-3, "%s: cannot reserve %zu B of LDS: %s", what, bytes, hipGetErrorString(e));
  done.fetch_or(1ull << dev, std::memory_order_release);
  return 0;
}
}  // namespace dl
