// Steps 3-4 of the pass, host side: the loop over blocks and groups (paper Sec. 3.2, 3.3), the
// lazy block-update GEMM (Eq. 4 applied to whole blocks; App. B.3 tail form) and the storage
// helpers.  The per-group kernels live in group_sweep.h.
#include "group_sweep.h"

namespace bpdq {

// W'[:, c_begin:c_end] -= Et^T * U[k0:k0+Kd, c_begin:c_end]   (Eq. 4 applied to a whole block:
// the lazy update of the columns not yet quantized; also the rest-of-block update when g < B)
__global__ __launch_bounds__(TailGemm::kThreads) void tail_update_kernel(
    const float* __restrict__ Et, int lde, int Kd, const float* __restrict__ U, int ldu, int k0,
    float* __restrict__ Wp, int ldw, int d_out, int c_begin, int c_end, int tiles_n) {
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  TailGemm::Acc acc;
  TailGemm::zero(acc);
  TailGemm::run<0>(Et, lde, tm * TailGemm::kTileM, lde, U + (long)k0 * ldu, ldu,
                       c_begin + tn * TailGemm::kTileN, c_end, 0, Kd, acc);
  const int r0 = tm * TailGemm::kTileM, c0 = c_begin + tn * TailGemm::kTileN;
  TailGemm::for_each(acc, [&](int row, int col, float v) {
    const int r = r0 + row, c = c0 + col;
    if (r < d_out && c < c_end) Wp[(long)r * ldw + c] -= v;
  });
}

// working copy of W with dead input channels zeroed
__global__ __launch_bounds__(256) void copy_in_kernel(const float* __restrict__ W, long n, int d_in,
                                                      const unsigned char* __restrict__ dead,
                                                      float* __restrict__ Wp) {
  for (long e = ((long)blockIdx.x * 256 + threadIdx.x) * 4; e < n; e += (long)gridDim.x * 1024) {
    float4 v = *reinterpret_cast<const float4*>(W + e);
    if (dead) {
      const int c = (int)(e % d_in);
      if (dead[c]) v.x = 0.f;
      if (dead[c + 1]) v.y = 0.f;
      if (dead[c + 2]) v.z = 0.f;
      if (dead[c + 3]) v.w = 0.f;
    }
    *reinterpret_cast<float4*>(Wp + e) = v;
  }
}

// ------------------------------------------------------------------ storage helpers --------
__global__ __launch_bounds__(256) void pack_planes_kernel(const unsigned char* __restrict__ codes,
                                                          int d_out, int d_in, int bits,
                                                          uint32_t* __restrict__ planes) {
  const int n_word = d_in / 32;
  const long n = (long)d_out * n_word;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const unsigned char* cp = codes + e * 32;
    uint32_t word[4] = {0u, 0u, 0u, 0u};
    for (int j = 0; j < 32; ++j) {
      const int code = cp[j];
#pragma unroll
      for (int i = 0; i < 4; ++i) word[i] |= (uint32_t)((code >> i) & 1) << j;
    }
    for (int i = 0; i < bits; ++i) planes[(long)i * n + e] = word[i];
  }
}

__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t* __restrict__ planes,
                                                      const float* __restrict__ coefs, int d_out,
                                                      int d_in, int bits, int group,
                                                      float* __restrict__ W_hat) {
  const int n_word = d_in / 32, n_grp = d_in / group;
  const long n = (long)d_out * d_in;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const int r = (int)(e / d_in), c = (int)(e % d_in);
    const int gi = c / group;
    float v = coefs[(long)r * n_grp + gi];
    for (int i = 0; i < bits; ++i) {
      const uint32_t w = planes[((long)i * d_out + r) * n_word + c / 32];
      if ((w >> (c & 31)) & 1u) v = v + coefs[((long)(i + 1) * d_out + r) * n_grp + gi];
    }
    W_hat[e] = v;
  }
}

// ------------------------------------------------------------------ host side --------------
static int check_params(int d_out, int d_in, const bpdq_params* p) {
  if (!p) return 1;
  if (p->bits < 1 || p->bits > 4) return 1;
  if (p->group != 32 && p->group != 64 && p->group != 128 && p->group != 256) return 1;
  if (d_in % p->group || d_in % 32) return 1;
  const int B = p->block > p->group ? p->block : p->group;
  if (p->block < 1 || B % p->group) return 1;
  if (p->refine_iters < 0 || p->refine_iters > 63) return 1;
  if (!(p->alpha >= 0.f)) return 1;
  if (p->grid != BPDQ_GRID_VARIABLE && p->grid != BPDQ_GRID_UNIFORM) return 1;
  if (d_out <= 0 || d_in <= 0) return 1;
  return 0;
}

static GroupLauncher pick_group(int k, int g) {
  if (g == 256) {
    switch (k) {
      case 1: return group256_k1();
      case 2: return group256_k2();
      case 3: return group256_k3();
      case 4: return group256_k4();
    }
    return nullptr;
  }
  switch (k) {
    case 1: return pick_group_k1(g);
    case 2: return pick_group_k2(g);
    case 3: return pick_group_k3(g);
    case 4: return pick_group_k4(g);
  }
  return nullptr;
}

static int launch_tail_update(hipStream_t stream, const float* Et, int lde, int Kd, const float* U,
                              int d_in, int k0, float* Wp, int d_out, int c_begin, int c_end) {
  if (c_end <= c_begin) return 0;
  static bool attr_set = false;
  if (!attr_set) {
    BPDQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(tail_update_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)TailGemm::kLdsBytes));
    attr_set = true;
  }
  const int tiles_m = bpdq_ceil_div(lde, TailGemm::kTileM);
  const int tiles_n = bpdq_ceil_div(c_end - c_begin, TailGemm::kTileN);
  hipLaunchKernelGGL(tail_update_kernel, dim3(tiles_m * tiles_n), dim3(TailGemm::kThreads),
                     TailGemm::kLdsBytes, stream, Et, lde, Kd, U, d_in, k0, Wp, d_in, d_out, c_begin, c_end, tiles_n);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

}  // namespace bpdq

using namespace bpdq;

extern "C" int bpdq_version(void) { return 100; }

extern "C" size_t bpdq_quantize_workspace_bytes(int d_out, int d_in, const bpdq_params* p) {
  if (check_params(d_out, d_in, p)) return 0;
  return quant_layout(d_out, d_in, *p).total;
}

extern "C" int bpdq_quantize_layer(const float* W, int d_out, int d_in, const float* U,
                                   const unsigned char* dead, const bpdq_params* p,
                                   uint32_t* planes, float* coefs, float* W_hat, double* grp_err,
                                   int* grp_iter, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!W || (reinterpret_cast<uintptr_t>(W) & 15)) return -1;
  if (d_out <= 0) return -2;
  if (d_in <= 0 || d_in % 32) return -3;
  if (!U || (reinterpret_cast<uintptr_t>(U) & 15)) return -4;
  if (check_params(d_out, d_in, p)) return -6;
  if (!planes) return -7;
  if (!coefs) return -8;
  if (!grp_err) return -10;
  if (!grp_iter) return -11;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return -12;
  const QuantLayout L = quant_layout(d_out, d_in, *p);
  if (ws_bytes < L.total) return -13;
  char* base = static_cast<char*>(ws);
  float* Wp = reinterpret_cast<float*>(base + L.wp_off);
  float* Eblk = reinterpret_cast<float*>(base + L.eblk_off);
  GroupLauncher group = pick_group(p->bits, p->group);
  if (!group) return -6;

  const long n = (long)d_out * d_in;
  const int grid = (int)((n / 4 + 255) / 256 < 65536 ? (n / 4 + 255) / 256 : 65536);
  hipLaunchKernelGGL(copy_in_kernel, dim3(grid), dim3(256), 0, stream, W, n, d_in, dead, Wp);
  BPDQ_LAUNCH_CHECK();

  const int g = p->group, B = L.B;
  for (int b0 = 0; b0 < d_in; b0 += B) {
    const int b1 = b0 + B < d_in ? b0 + B : d_in;
    for (int s0 = b0; s0 < b1; s0 += g) {
      int rc = group(stream, Wp, d_out, d_in, U, s0, b0, *p, L, base, planes, coefs, W_hat,
                     grp_err, grp_iter);
      if (rc) return rc;
      // rest of this block (only when g < B): W'[:, s0+g:b1] -= E* U[s0:s0+g, s0+g:b1]
      rc = launch_tail_update(stream, Eblk + (long)(s0 - b0) * L.lde, L.lde, g, U, d_in, s0, Wp,
                              d_out, s0 + g, b1);
      if (rc) return rc;
    }
    // lazy block update of every later column
    const int rc = launch_tail_update(stream, Eblk, L.lde, b1 - b0, U, d_in, b0, Wp, d_out, b1, d_in);
    if (rc) return rc;
  }
  return 0;
}

extern "C" int bpdq_pack_planes(const unsigned char* codes, int d_out, int d_in, int bits,
                                uint32_t* planes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!codes) return -1;
  if (d_out <= 0) return -2;
  if (d_in <= 0 || d_in % 32) return -3;
  if (bits < 1 || bits > 4) return -4;
  if (!planes) return -5;
  const long n = (long)d_out * (d_in / 32);
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(pack_planes_kernel, dim3(grid), dim3(256), 0, stream, codes, d_out, d_in, bits, planes);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

extern "C" int bpdq_dequant(const uint32_t* planes, const float* coefs, int d_out, int d_in,
                            int bits, int group, float* W_hat, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!planes) return -1;
  if (!coefs) return -2;
  if (d_out <= 0) return -3;
  if (d_in <= 0 || d_in % 32) return -4;
  if (bits < 1 || bits > 4) return -5;
  if (group <= 0 || d_in % group) return -6;
  if (!W_hat) return -7;
  const long n = (long)d_out * d_in;
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(dequant_kernel, dim3(grid), dim3(256), 0, stream, planes, coefs, d_out, d_in,
                     bits, group, W_hat);
  BPDQ_LAUNCH_CHECK();
  return 0;
}
