// Serving side: y = What x for one token from the stored bit-plane format (paper Eq. 1; Sec. 5
// discusses the inference kernel).  Regrouped per (row, group G):
//   y_r = sum_G ( C_0[r,G] S(G) + sum_i C_i[r,G] sum_{c in G} B_i[r,c] x_c ),   S(G) = sum_{c in G} x_c.
// A weight costs one masked add per plane and no multiply; a row reads bits/8 bytes per weight.
//
// One wavefront per pair of rows (pairs strided over the grid); lane l takes the 32-column words
// l, l + 64, ...
// x is staged once per work-group in LDS, transposed (xT[j][w] = x[32 w + j]) so that the lanes
// of a wavefront, which hold consecutive words, read consecutive addresses for every bit j.
#include "common.h"

namespace bpdq {

constexpr int kGemvMaxDin = 36864;
constexpr int kGemvThreads = 1024;   // 16 wavefronts share one staged copy of x and hide each other's loads
constexpr int kGemvWaves = kGemvThreads / 64;

template <int K>
__global__ __launch_bounds__(kGemvThreads) void gemv_planes_kernel(const uint32_t* __restrict__ planes,
                                                          const _Float16* __restrict__ coefs,
                                                          int d_out, int d_in, int group,
                                                          const float* __restrict__ x,
                                                          float* __restrict__ y) {
  extern __shared__ float lds[];
  const int nw = d_in / 32, n_grp = d_in / group, wpg = group / 32;
  float* xT = lds;                    // [32][nw]
  float* gs = lds + 32 * nw;          // S(G)
  const int tid = threadIdx.x;
  for (int e = tid; e < d_in; e += kGemvThreads) xT[(e & 31) * nw + (e >> 5)] = x[e];
  __syncthreads();
  for (int G = tid; G < n_grp; G += kGemvThreads) {
    float s = 0.f;
    for (int wq = 0; wq < wpg; ++wq)
      for (int j = 0; j < 32; ++j) s += xT[j * nw + G * wpg + wq];
    gs[G] = s;
  }
  __syncthreads();
  const int lane = tid & 63, wave = tid >> 6;
  // two rows per wavefront and pass: their plane words are requested together
  for (int r0 = (blockIdx.x * kGemvWaves + wave) * 2; r0 < d_out; r0 += gridDim.x * kGemvWaves * 2) {
    const bool two = r0 + 1 < d_out;
    const int r1 = two ? r0 + 1 : r0;
    float acc0 = 0.f, acc1 = 0.f;
    for (int w = lane; w < nw; w += 64) {
      uint32_t wa[K], wb[K];
#pragma unroll
      for (int i = 0; i < K; ++i) {
        wa[i] = planes[((long)i * d_out + r0) * nw + w];
        wb[i] = planes[((long)i * d_out + r1) * nw + w];
      }
      float ma[K], mb[K];
#pragma unroll
      for (int i = 0; i < K; ++i) ma[i] = mb[i] = 0.f;
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        const int xv = __builtin_bit_cast(int, xT[j * nw + w]);
#pragma unroll
        for (int i = 0; i < K; ++i) {
          // all-ones where the bit is set: the masked add needs no compare
          ma[i] += __builtin_bit_cast(float, xv & __builtin_amdgcn_sbfe(static_cast<int>(wa[i]), j, 1));
          mb[i] += __builtin_bit_cast(float, xv & __builtin_amdgcn_sbfe(static_cast<int>(wb[i]), j, 1));
        }
      }
      const int G = w / wpg;
#pragma unroll
      for (int i = 0; i < K; ++i) {
        acc0 = fmaf((float)coefs[((long)(i + 1) * d_out + r0) * n_grp + G], ma[i], acc0);
        acc1 = fmaf((float)coefs[((long)(i + 1) * d_out + r1) * n_grp + G], mb[i], acc1);
      }
    }
    for (int G = lane; G < n_grp; G += 64) {
      acc0 = fmaf((float)coefs[(long)r0 * n_grp + G], gs[G], acc0);
      acc1 = fmaf((float)coefs[(long)r1 * n_grp + G], gs[G], acc1);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      acc0 += __shfl_xor(acc0, o, 64);
      acc1 += __shfl_xor(acc1, o, 64);
    }
    if (lane == 0) {
      y[r0] = acc0;
      if (two) y[r1] = acc1;
    }
  }
}

}  // namespace bpdq

using namespace bpdq;

extern "C" int bpdq_gemv(const uint32_t* planes, const uint16_t* coefs_h, int d_out, int d_in,
                         int bits, int group, const float* x, float* y, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!planes) return -1;
  if (!coefs_h || (reinterpret_cast<uintptr_t>(coefs_h) & 1)) return -2;
  if (d_out <= 0) return -3;
  if (d_in <= 0 || d_in % 32 || d_in > kGemvMaxDin) return -4;
  if (bits < 1 || bits > 4) return -5;
  if (group < 32 || group % 32 || d_in % group) return -6;
  if (!x) return -7;
  if (!y) return -8;
  const size_t lds = (size_t)(d_in + d_in / group) * sizeof(float);
  const _Float16* ch = reinterpret_cast<const _Float16*>(coefs_h);
  int grid = bpdq_ceil_div(d_out, kGemvWaves * 2);   // 2 rows per wavefront and pass
  if (grid > 256) grid = 256;                        // one work-group per CU; each stages x once
  auto launch = [&](auto kern) -> int {
    static bool attr_set = false;
    if (!attr_set) {
      BPDQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)((kGemvMaxDin + kGemvMaxDin / 32) * sizeof(float))));
      attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kGemvThreads), lds, stream, planes, ch, d_out, d_in, group, x, y);
    BPDQ_LAUNCH_CHECK();
    return 0;
  };
  switch (bits) {
    case 1: return launch(gemv_planes_kernel<1>);
    case 2: return launch(gemv_planes_kernel<2>);
    case 3: return launch(gemv_planes_kernel<3>);
    default: return launch(gemv_planes_kernel<4>);
  }
}
