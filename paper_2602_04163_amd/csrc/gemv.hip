// Serving side: y = What x for one token from the stored bit-plane format (paper Eq. 1; Sec. 5
// discusses the inference kernel).  Regrouped per (row, group G):
//   y_r = sum_G ( C_0[r,G] S(G) + sum_i C_i[r,G] sum_{c in G} B_i[r,c] x_c ),   S(G) = sum_{c in G} x_c.
// A weight costs one masked add per plane and no multiply; a row reads bits/8 bytes per weight.
//
// A look-up table replaces the per-bit work: for every segment of 4 columns the 16 partial sums
// of its x values, T[seg][nibble]; a plane word then costs 8 (extract, look up, add) triples
// instead of 32 masked adds.  The table of a chunk of up to 8192 columns (136 KB of LDS with
// its padding) is built once per work-group and chunk -- 15 adds per segment -- and used by all
// its rows.  One wavefront owns a pair of rows for the whole call (16 wavefronts per work-group,
// one work-group per CU); lane l takes the 32-column words l, l + 64, ... of the chunk.  The table
// is laid out T[q][nibble][w] (q = nibble position inside a word, w = word, fastest): the 64 lanes
// of a wavefront hold consecutive words, so whatever their nibbles are they fall into consecutive
// banks -- two lanes per bank, the minimum for 64 lanes.
#include "common.h"

namespace bpdq {

constexpr int kGemvThreads = 1024;
constexpr int kGemvWaves = kGemvThreads / 64;
constexpr int kGemvChunk = 8192;                  // columns per table
constexpr int kChunkWords = kGemvChunk / 32;      // 256: the word stride of the table, also for a short last chunk
constexpr size_t kGemvLdsBytes = (size_t)(8 * 16 * kChunkWords + kChunkWords) * sizeof(float);

template <int K>
__global__ __launch_bounds__(kGemvThreads) void gemv_planes_kernel(const uint32_t* __restrict__ planes,
                                                                   const _Float16* __restrict__ coefs,
                                                                   int d_out, int d_in, int group,
                                                                   const float* __restrict__ x,
                                                                   float* __restrict__ y) {
  extern __shared__ float lds[];
  float* T = lds;                                        // [8][16][kChunkWords]
  float* Sw = lds + 8 * 16 * kChunkWords;                // sum of x over each word of the chunk
  const int nw = d_in / 32, n_grp = d_in / group, wpg = group / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rows_per_pass = gridDim.x * kGemvWaves * 2;
  for (int c0 = 0; c0 < d_in; c0 += kGemvChunk) {
    const int cols = (d_in - c0 < kGemvChunk) ? d_in - c0 : kGemvChunk;
    const int n_word = cols / 32;
    __syncthreads();                                     // the previous chunk's table is no longer read
    for (int sgm = tid; sgm < 8 * n_word; sgm += kGemvThreads) {
      const int q = sgm / n_word, w = sgm % n_word;      // consecutive threads: consecutive words
      const float4 v = *reinterpret_cast<const float4*>(x + c0 + 32 * w + 4 * q);
      float* t = T + q * 16 * kChunkWords + w;
      const float s01 = v.x + v.y, s23 = v.z + v.w;
      const float e[16] = {0.f,  v.x,       v.y,       s01,       v.z, v.x + v.z, v.y + v.z, s01 + v.z,
                           v.w,  v.x + v.w, v.y + v.w, s01 + v.w, s23, v.x + s23, v.y + s23, s01 + s23};
#pragma unroll
      for (int n = 0; n < 16; ++n) t[n * kChunkWords] = e[n];
    }
    __syncthreads();
    for (int w = tid; w < n_word; w += kGemvThreads) {
      float sw = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) sw += T[(q * 16 + 15) * kChunkWords + w];
      Sw[w] = sw;
    }
    __syncthreads();
    const int w0 = c0 / 32;                              // first word of the chunk in a row
    for (int r0 = (blockIdx.x * kGemvWaves + wave) * 2; r0 < d_out; r0 += rows_per_pass) {
      const bool two = r0 + 1 < d_out;
      const int r1 = two ? r0 + 1 : r0;
      float acc0 = 0.f, acc1 = 0.f;
      for (int w = lane; w < n_word; w += 64) {
        uint32_t wa[K], wb[K];
#pragma unroll
        for (int i = 0; i < K; ++i) {
          wa[i] = planes[((long)i * d_out + r0) * nw + w0 + w];
          wb[i] = planes[((long)i * d_out + r1) * nw + w0 + w];
        }
        const int G = (w0 + w) / wpg;
        const float sw = Sw[w];
        acc0 = fmaf((float)coefs[(long)r0 * n_grp + G], sw, acc0);
        acc1 = fmaf((float)coefs[(long)r1 * n_grp + G], sw, acc1);
        const float* tw = T + w;
#pragma unroll
        for (int i = 0; i < K; ++i) {
          float ma = 0.f, mb = 0.f;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            ma += tw[(q * 16 + ((wa[i] >> (4 * q)) & 15u)) * kChunkWords];
            mb += tw[(q * 16 + ((wb[i] >> (4 * q)) & 15u)) * kChunkWords];
          }
          acc0 = fmaf((float)coefs[((long)(i + 1) * d_out + r0) * n_grp + G], ma, acc0);
          acc1 = fmaf((float)coefs[((long)(i + 1) * d_out + r1) * n_grp + G], mb, acc1);
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        acc0 += __shfl_xor(acc0, o, 64);
        acc1 += __shfl_xor(acc1, o, 64);
      }
      if (lane == 0) {                                   // this wavefront owns these rows: no race
        y[r0] = (c0 == 0 ? 0.f : y[r0]) + acc0;
        if (two) y[r1] = (c0 == 0 ? 0.f : y[r1]) + acc1;
      }
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
  if (d_in <= 0 || d_in % 32) return -4;
  if (bits < 1 || bits > 4) return -5;
  if (group < 32 || group % 32 || d_in % group) return -6;
  if (!x || (reinterpret_cast<uintptr_t>(x) & 15)) return -7;
  if (!y) return -8;
  const size_t lds = kGemvLdsBytes;
  const _Float16* ch = reinterpret_cast<const _Float16*>(coefs_h);
  int grid = bpdq_ceil_div(d_out, kGemvWaves * 2);   // 2 rows per wavefront and pass
  if (grid > 256) grid = 256;                        // one work-group per CU; each builds the table once
  auto launch = [&](auto kern, hipError_t limit) -> int {
    BPDQ_HIP_TRY(limit);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kGemvThreads), lds, stream, planes, ch, d_out, d_in, group, x, y);
    BPDQ_LAUNCH_CHECK();
    return 0;
  };
  switch (bits) {
    case 1: return launch(gemv_planes_kernel<1>, bpdq_lds_limit<&gemv_planes_kernel<1>>(lds));
    case 2: return launch(gemv_planes_kernel<2>, bpdq_lds_limit<&gemv_planes_kernel<2>>(lds));
    case 3: return launch(gemv_planes_kernel<3>, bpdq_lds_limit<&gemv_planes_kernel<3>>(lds));
    default: return launch(gemv_planes_kernel<4>, bpdq_lds_limit<&gemv_planes_kernel<4>>(lds));
  }
}
