// Channel ordering around the pass (paper Sec. 4.1: GPTQ sorts the channels in descending order
// of the Hessian diagonal; BPDQ's experiments use a group-preserving reordering).  The pass
// itself always runs left to right; these helpers build a permutation and move W / H / W_hat in
// and out of the permuted order.
#include <mutex>

#include "common.h"

namespace bpdq {

// Scratch of bpdq_channel_order_noalloc: the sort keys, one double per block of channels.  A
// device-resident array of the library itself, so that the call needs no workspace and no
// allocation; every GPU the library runs on holds its own copy (256 KB) until the process ends.
constexpr int kOrderNoAllocMaxKeys = 32768;
static __device__ __align__(256) double scratch[kOrderNoAllocMaxKeys];

// key[b] = sum of H_jj over block b of `gs` consecutive channels, fp64, index order
__global__ __launch_bounds__(256) void order_key_kernel(const float* __restrict__ H, int d, int gs,
                                                        double* __restrict__ key) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= d / gs) return;
  double s = 0.0;
  for (int m = 0; m < gs; ++m) {
    const long j = (long)b * gs + m;
    s += (double)H[j * d + j];
  }
  key[b] = s;
}

// Sorting by counting: block b goes to position #{c : key_c > key_b, or key_c == key_b and
// c < b}.  One thread per block, the keys stream through LDS; deterministic and stable, and
// n^2 comparisons are nothing for n <= 32768.
__global__ __launch_bounds__(256) void order_rank_kernel(const double* __restrict__ key, int n, int gs,
                                                         int* __restrict__ perm) {
  __shared__ double sk[1024];
  const int b = blockIdx.x * 256 + threadIdx.x;
  const double kb = (b < n) ? key[b] : 0.0;
  int rank = 0;
  for (int c0 = 0; c0 < n; c0 += 1024) {
    __syncthreads();
    for (int e = threadIdx.x; e < 1024; e += 256) sk[e] = (c0 + e < n) ? key[c0 + e] : 0.0;
    __syncthreads();
    const int lim = (n - c0 < 1024) ? n - c0 : 1024;
    for (int e = 0; e < lim; ++e) {
      const double kc = sk[e];
      rank += (kc > kb || (kc == kb && c0 + e < b)) ? 1 : 0;
    }
  }
  if (b < n)
    for (int m = 0; m < gs; ++m) perm[rank * gs + m] = b * gs + m;
}

// dst[r][i] = src[r][perm[i]] (GATHER) or dst[r][perm[i]] = src[r][i]
template <bool GATHER>
__global__ __launch_bounds__(256) void permute_columns_kernel(const float* __restrict__ src, int d_out,
                                                              int d_in, const int* __restrict__ perm,
                                                              float* __restrict__ dst) {
  const long n = (long)d_out * d_in;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const long r = e / d_in;
    const int i = (int)(e % d_in);
    const int p = perm[i];
    if (GATHER) dst[e] = src[r * d_in + p];
    else dst[r * d_in + p] = src[e];
  }
}

__global__ __launch_bounds__(256) void gather_symmetric_kernel(const float* __restrict__ H, int d,
                                                               const int* __restrict__ perm,
                                                               float* __restrict__ Hp) {
  const long n = (long)d * d;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const int i = (int)(e / d), j = (int)(e % d);
    Hp[e] = H[(long)perm[i] * d + perm[j]];
  }
}

static inline int grid_for(long n) {
  const long g = (n + 255) / 256;
  return (int)(g < 65536 ? (g > 0 ? g : 1) : 65536);
}

}  // namespace bpdq

using namespace bpdq;

extern "C" size_t bpdq_channel_order_workspace_bytes(int d_in) {
  return d_in > 0 ? bpdq_align_up((size_t)d_in * sizeof(double), 256) : 0;
}

extern "C" int bpdq_channel_order(const float* H, int d_in, int group_size, int* perm, void* ws,
                                  size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!H) return -1;
  if (d_in <= 0) return -2;
  if (group_size < 1 || d_in % group_size) return -3;
  if (!perm) return -4;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 7)) return -5;
  if (ws_bytes < bpdq_channel_order_workspace_bytes(d_in)) return -6;
  double* key = static_cast<double*>(ws);
  const int n = d_in / group_size;
  hipLaunchKernelGGL(order_key_kernel, dim3(bpdq_ceil_div(n, 256)), dim3(256), 0, stream, H, d_in,
                     group_size, key);
  BPDQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(order_rank_kernel, dim3(bpdq_ceil_div(n, 256)), dim3(256), 0, stream, key, n,
                     group_size, perm);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

// Device address of `scratch` on the current GPU.  In host code the array's name is only a handle
// for the runtime; the address is looked up once per device (with that device current) and kept.
static int order_scratch(double** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex lock;
  static double* ptr[kMaxDevices] = {};
  int dev = -1;
  BPDQ_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return BPDQ_ERR_LAUNCH;
  std::lock_guard<std::mutex> guard(lock);
  if (!ptr[dev]) {
    double* p = nullptr;
    BPDQ_HIP_TRY(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    if (!p) return BPDQ_ERR_LAUNCH;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return 0;
}

extern "C" int bpdq_channel_order_noalloc(const float* H, int d_in, int group_size, int* perm,
                                          void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!H) return -1;
  if (d_in <= 0) return -2;
  if (group_size < 1 || d_in % group_size) return -3;
  if (d_in / group_size > kOrderNoAllocMaxKeys) return -2;      // beyond the built-in scratch
  if (!perm) return -4;
  double* key = nullptr;
  const int rc = order_scratch(&key);
  if (rc) return rc;
  // every key the second kernel reads is written by the first: nothing of the previous call's
  // contents survives into the result
  const int n = d_in / group_size;
  hipLaunchKernelGGL(order_key_kernel, dim3(bpdq_ceil_div(n, 256)), dim3(256), 0, stream, H, d_in,
                     group_size, key);
  BPDQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(order_rank_kernel, dim3(bpdq_ceil_div(n, 256)), dim3(256), 0, stream, key, n,
                     group_size, perm);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

static int permute_columns(const float* src, int d_out, int d_in, const int* perm, float* dst,
                           bool gather, hipStream_t stream) {
  if (!src) return -1;
  if (d_out <= 0) return -2;
  if (d_in <= 0) return -3;
  if (!perm) return -4;
  if (!dst || dst == src) return -5;
  const long n = (long)d_out * d_in;
  if (gather) {
    hipLaunchKernelGGL(permute_columns_kernel<true>, dim3(grid_for(n)), dim3(256), 0, stream, src,
                       d_out, d_in, perm, dst);
  } else {
    hipLaunchKernelGGL(permute_columns_kernel<false>, dim3(grid_for(n)), dim3(256), 0, stream, src,
                       d_out, d_in, perm, dst);
  }
  BPDQ_LAUNCH_CHECK();
  return 0;
}

extern "C" int bpdq_gather_columns(const float* W, int d_out, int d_in, const int* perm, float* Wp,
                                   void* stream) {
  return permute_columns(W, d_out, d_in, perm, Wp, true, static_cast<hipStream_t>(stream));
}

extern "C" int bpdq_scatter_columns(const float* Wp, int d_out, int d_in, const int* perm, float* W,
                                    void* stream) {
  return permute_columns(Wp, d_out, d_in, perm, W, false, static_cast<hipStream_t>(stream));
}

extern "C" int bpdq_gather_symmetric(const float* H, int d_in, const int* perm, float* Hp,
                                     void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!H) return -1;
  if (d_in <= 0) return -2;
  if (!perm) return -3;
  if (!Hp || Hp == H) return -4;
  hipLaunchKernelGGL(gather_symmetric_kernel, dim3(grid_for((long)d_in * d_in)), dim3(256), 0, stream,
                     H, d_in, perm, Hp);
  BPDQ_LAUNCH_CHECK();
  return 0;
}
