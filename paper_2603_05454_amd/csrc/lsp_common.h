// Internal helpers of liblsp (HIP side only).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <stdint.h>
#include <stdio.h>

#include "lsp.h"

namespace lsp {

// Text of the calling thread's last failure (returned by lsp_last_error()).
void set_error(const char *fmt, ...);

inline int32_t hip_fail(hipError_t e, const char *what) {
  set_error("%s: %s", what, hipGetErrorString(e));
  return LSP_ERR_HIP;
}

#define LSP_CHECK_ARG(cond, ...)        \
  do {                                  \
    if (!(cond)) {                      \
      lsp::set_error(__VA_ARGS__);      \
      return LSP_ERR_INVALID_ARG;       \
    }                                   \
  } while (0)

#define LSP_CHECK_LAUNCH(what)                          \
  do {                                                  \
    hipError_t e__ = hipGetLastError();                 \
    if (e__ != hipSuccess) return lsp::hip_fail(e__, what); \
  } while (0)

// Raise a kernel's dynamic LDS limit.  The attribute belongs to (kernel, device),
// so `done` keeps one bit per device ordinal (one atomic per kernel instantiation):
// the first launch on each GPU sets it, from whichever host thread gets there
// (two threads racing both set the same value, which is harmless).
inline int32_t ensure_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done, const char *what) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, what);
  const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t(1) << dev : 0;  // ordinals beyond 63: set every time
  if (bit != 0 && (done.load(std::memory_order_acquire) & bit)) return LSP_OK;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes));
  if (e != hipSuccess) return hip_fail(e, what);
  done.fetch_or(bit, std::memory_order_release);
  return LSP_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(int32_t dtype) { return dtype == LSP_F32 ? 4 : 2; }

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(uint32_t(h) << 16); }

// Round-to-nearest-even fp32 -> bf16 (finite inputs; NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

}  // namespace lsp
