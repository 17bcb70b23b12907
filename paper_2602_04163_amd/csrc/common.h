// Shared host/device helpers of the BPDQ library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/bpdq.h"

#define BPDQ_HIP_TRY(expr)                      \
  do {                                          \
    if ((expr) != hipSuccess) {                 \
      (void)hipGetLastError();                  \
      return BPDQ_ERR_LAUNCH;                   \
    }                                           \
  } while (0)

#define BPDQ_LAUNCH_CHECK()                     \
  do {                                          \
    if (hipGetLastError() != hipSuccess) return BPDQ_ERR_LAUNCH; \
  } while (0)

// Raises a kernel's dynamic-LDS limit once per process and kernel.  `bpdq_lds_limit<&kernel>(n)`
// holds one function-local static per kernel (initialised under the language's own lock, so
// concurrent first calls from several host threads are safe) and returns the HIP status of that
// one-off call.
template <auto KERNEL>
static inline hipError_t bpdq_lds_limit(size_t bytes) {
  static const hipError_t status = hipFuncSetAttribute(
      reinterpret_cast<const void*>(KERNEL), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  return status;
}

static inline size_t bpdq_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
__host__ __device__ static inline int bpdq_ceil_div(int a, int b) { return (a + b - 1) / b; }

// bump allocator over the caller's workspace
struct BpdqArena {
  char* base;
  size_t off;
  explicit BpdqArena(void* p) : base(static_cast<char*>(p)), off(0) {}
  template <typename T>
  T* take(size_t n) {
    T* r = reinterpret_cast<T*>(base + off);
    off += bpdq_align_up(n * sizeof(T), 256);
    return r;
  }
};
