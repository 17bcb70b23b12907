// Measured ceilings of the chip the library runs on: register-only loops of the matrix-core
// instructions the pass uses, and a streaming copy.  They are what a roofline fraction of the
// Hessian / block-update / prepare kernels is quoted against besides the published peaks: the
// rate the instruction itself sustains on this GPU, on operand values like the real ones (the
// sustained clock under matrix load depends on how many operand bits toggle).
//
// One work-group per compute unit; every wavefront keeps a grid of accumulator tiles (2 x 4 of
// 32 x 32, or 4 x 4 of 16 x 16 in fp64: at most 128 registers, so that two wavefronts fit a SIMD)
// and walks it with as many A and B operand registers, as a tiled GEMM does: consecutive
// instructions are independent and their operands differ.
#include "common.h"

namespace bpdq {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ unsigned probe_hash(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// data 0: zero, 1: one, 2: standard normal (Box-Muller on hashed uniforms)
__device__ __forceinline__ float probe_value(int data, unsigned seed) {
  if (data == 0) return 0.f;
  if (data == 1) return 1.f;
  const float u1 = (float)((probe_hash(seed) >> 8) + 1u) * (1.0f / 16777217.0f);
  const float u2 = (float)(probe_hash(seed ^ 0x9e3779b9u) >> 8) * (1.0f / 16777216.0f);
  return sqrtf(-2.0f * __logf(u1)) * __cosf(6.2831853f * u2);
}

enum : int { kProbeF32 = 0, kProbeBF16 = 1, kProbeF16 = 2, kProbeF64 = 3, kProbeI8 = 4 };
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

template <int KIND>
__global__ __launch_bounds__(512) void probe_mfma_kernel(int iters, int data, float* __restrict__ out) {
  const unsigned tid = blockIdx.x * blockDim.x + threadIdx.x;
  float sum = 0.f;
  if constexpr (KIND == kProbeF32) {
    float a[2], b[4];
    f32x16 c[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i < 2) a[i] = probe_value(data, tid * 16 + i);
      b[i] = probe_value(data, tid * 16 + 8 + i);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          c[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], c[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += c[i][j][r];
  } else if constexpr (KIND == kProbeBF16 || KIND == kProbeF16) {
    using V = std::conditional_t<KIND == kProbeBF16, bf16x8, f16x8>;
    using S = std::conditional_t<KIND == kProbeBF16, __bf16, _Float16>;
    V a[2], b[4];
    f32x16 c[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (i < 2) a[i][e] = (S)probe_value(data, tid * 64 + i * 8 + e);
        b[i][e] = (S)probe_value(data, tid * 64 + 32 + i * 8 + e);
      }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if constexpr (KIND == kProbeBF16)
            c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], c[i][j], 0, 0, 0);
          else
            c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], c[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += c[i][j][r];
  } else if constexpr (KIND == kProbeI8) {
    // v_mfma_i32_32x32x32_i8: 16 signed bytes per lane and operand; "normal" = round(32 z) clamped
    i32x4 a[2], b[4];
    i32x16 c[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        unsigned pa = 0, pb = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float va = probe_value(data, tid * 128 + i * 16 + w * 4 + e) * (data == 2 ? 32.f : 1.f);
          const float vb = probe_value(data, tid * 128 + 64 + i * 16 + w * 4 + e) * (data == 2 ? 32.f : 1.f);
          pa |= ((unsigned)(int)fminf(fmaxf(rintf(va), -127.f), 127.f) & 0xffu) << (8 * e);
          pb |= ((unsigned)(int)fminf(fmaxf(rintf(vb), -127.f), 127.f) & 0xffu) << (8 * e);
        }
        if (i < 2) a[i][w] = (int)pa;
        b[i][w] = (int)pb;
      }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) c[i][j][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], c[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += (float)c[i][j][r];
  } else {
    double a[4], b[4];
    f64x4 c[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = (double)probe_value(data, tid * 16 + i);
      b[i] = (double)probe_value(data, tid * 16 + 8 + i);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) c[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          c[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], c[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) sum += (float)c[i][j][r];
  }
  out[tid] = sum;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const float4* __restrict__ src,
                                                         float4* __restrict__ dst, long n_vec) {
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n_vec; e += (long)gridDim.x * 256)
    dst[e] = src[e];
}

}  // namespace bpdq

using namespace bpdq;

// flops of one instruction: 2 * M * N * K
static double probe_flops_per_mfma(int kind) {
  switch (kind) {
    case kProbeF32: return 2.0 * 32 * 32 * 2;
    case kProbeBF16:
    case kProbeF16: return 2.0 * 32 * 32 * 16;
    case kProbeI8: return 2.0 * 32 * 32 * 32;
    default: return 2.0 * 16 * 16 * 4;
  }
}

extern "C" int bpdq_probe_mfma(int kind, int data, int waves_per_simd, int groups, int iters,
                               float* out, double* flops, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (kind < 0 || kind > 4) return -1;
  if (data < 0 || data > 2) return -2;
  if (waves_per_simd != 1 && waves_per_simd != 2) return -3;
  if (groups < 1 || groups > 65536) return -4;
  if (iters < 1) return -5;
  if (!out) return -6;
  const int threads = 256 * waves_per_simd;
  switch (kind) {
    case kProbeF32:
      hipLaunchKernelGGL(probe_mfma_kernel<kProbeF32>, dim3(groups), dim3(threads), 0, stream, iters, data, out);
      break;
    case kProbeBF16:
      hipLaunchKernelGGL(probe_mfma_kernel<kProbeBF16>, dim3(groups), dim3(threads), 0, stream, iters, data, out);
      break;
    case kProbeF16:
      hipLaunchKernelGGL(probe_mfma_kernel<kProbeF16>, dim3(groups), dim3(threads), 0, stream, iters, data, out);
      break;
    case kProbeI8:
      hipLaunchKernelGGL(probe_mfma_kernel<kProbeI8>, dim3(groups), dim3(threads), 0, stream, iters, data, out);
      break;
    default:
      hipLaunchKernelGGL(probe_mfma_kernel<kProbeF64>, dim3(groups), dim3(threads), 0, stream, iters, data, out);
      break;
  }
  BPDQ_LAUNCH_CHECK();
  const double per_iter = (kind == kProbeF64) ? 16.0 : 8.0;      // instructions per loop iteration
  if (flops) *flops = probe_flops_per_mfma(kind) * per_iter * iters * (threads / 64) * (double)groups;
  return 0;
}

extern "C" int bpdq_probe_copy(const float* src, float* dst, long n_floats, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!src || (reinterpret_cast<uintptr_t>(src) & 15)) return -1;
  if (!dst || (reinterpret_cast<uintptr_t>(dst) & 15)) return -2;
  if (n_floats <= 0 || n_floats % 4) return -3;
  hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 16), dim3(256), 0, stream,
                     reinterpret_cast<const float4*>(src), reinterpret_cast<float4*>(dst), n_floats / 4);
  BPDQ_LAUNCH_CHECK();
  return 0;
}
