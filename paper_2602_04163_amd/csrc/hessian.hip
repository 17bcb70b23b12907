// Step 1 of the pass: calibration Hessian H += scale * Xc^T Xc (paper Sec. 3.1, H = X X^T).
//
// A symmetric rank-k update on the fp32 matrix cores.  Only the upper triangle of 256 x 256
// tiles is computed.  The token axis is cut into S deterministic slices so that
// (tiles x S) work-groups fill the 256 compute units; slice partials go to the workspace and
// are summed in a fixed order (no float atomics => bit-reproducible H).
#include "mfma_kmajor.h"

namespace bpdq {

constexpr int kNumCU = 256;   // MI355X

struct HessPlan {
  int nb;        // tile rows/cols
  int n_tiles;   // upper-triangular tiles
  int S;         // token slices
  int k_per;     // tokens per slice (multiple of kStageK)
};

static HessPlan plan_hessian(int n_tok, int d_in) {
  HessPlan p;
  p.nb = bpdq_ceil_div(d_in, HessGemm::kTileM);
  p.n_tiles = p.nb * (p.nb + 1) / 2;
  p.S = 1;
  p.k_per = (int)bpdq_align_up((size_t)(n_tok > 0 ? n_tok : 1), kStageK);
  if (n_tok <= 0 || p.n_tiles >= 4 * kNumCU) return p;
  // estimated time (us) = rounds * (slice MFMA time + fixed cost) + reduction traffic
  const double us_per_tok = 0.28, us_fixed = 8.0, us_per_partial = 0.131;
  double best = 1e300;
  const int s_max = n_tok / 256 < 64 ? (n_tok / 256 < 1 ? 1 : n_tok / 256) : 64;
  for (int S = 1; S <= s_max; ++S) {
    const int k_per = (int)bpdq_align_up((size_t)bpdq_ceil_div(n_tok, S), kStageK);
    const int rounds = bpdq_ceil_div(p.n_tiles * S, kNumCU);
    double t = rounds * (k_per * us_per_tok + us_fixed);
    if (S > 1) t += (double)p.n_tiles * S * us_per_partial;
    if (t < best * 0.995) {
      best = t;
      p.S = S;
      p.k_per = k_per;
    }
  }
  return p;
}

__device__ __forceinline__ void decode_upper_tile(int tile, int nb, int& bi, int& bj) {
  bi = 0;
  while (tile >= nb - bi) {
    tile -= nb - bi;
    ++bi;
  }
  bj = bi + tile;
}

__global__ __launch_bounds__(HessGemm::kThreads) void hess_syrk_f32_kernel(
    const float* __restrict__ X, int n_tok, int d, long ldx, float scale, float* __restrict__ H,
    float* __restrict__ partial, int nb, int n_tiles, int S, int k_per) {
  const int item = blockIdx.x;
  const int split = item / n_tiles;
  int bi, bj;
  decode_upper_tile(item % n_tiles, nb, bi, bj);
  const int k_begin = split * k_per;
  const int k_end = min(n_tok, k_begin + k_per);
  HessGemm::Acc acc;
  HessGemm::zero(acc);
  if (bi == bj) {
    HessGemm::run<true>(X, ldx, bi * HessGemm::kTileM, d, X, ldx, bj * HessGemm::kTileN, d, k_begin, k_end, acc);
  } else {
    HessGemm::run<false>(X, ldx, bi * HessGemm::kTileM, d, X, ldx, bj * HessGemm::kTileN, d, k_begin, k_end, acc);
  }
  if (S == 1) {
    const int r0 = bi * HessGemm::kTileM, c0 = bj * HessGemm::kTileN;
    HessGemm::for_each(acc, [&](int row, int col, float v) {
      const int r = r0 + row, c = c0 + col;
      if (r < d && c < d) H[(long)r * d + c] += scale * v;
    });
  } else {
    float* out = partial + (long)item * (HessGemm::kTileM * HessGemm::kTileN);
    HessGemm::for_each(acc, [&](int row, int col, float v) { out[row * HessGemm::kTileN + col] = v; });
  }
}

// H[tile] += scale * sum_s partial[s][tile], slices added in index order.
__global__ __launch_bounds__(256) void hess_reduce_kernel(const float* __restrict__ partial,
                                                          int n_tiles, int S, int nb, int d,
                                                          float scale, float* __restrict__ H) {
  const int tile = blockIdx.x >> 6;
  const int e = ((blockIdx.x & 63) * 256 + threadIdx.x) * 4;
  int bi, bj;
  decode_upper_tile(tile, nb, bi, bj);
  const int r = bi * HessGemm::kTileM + e / HessGemm::kTileN;
  const int c = bj * HessGemm::kTileN + e % HessGemm::kTileN;
  if (r >= d || c >= d) return;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp = 0; sp < S; ++sp) {
    const float4 v = *reinterpret_cast<const float4*>(
        partial + ((long)sp * n_tiles + tile) * (HessGemm::kTileM * HessGemm::kTileN) + e);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  float4* h = reinterpret_cast<float4*>(H + (long)r * d + c);
  float4 o = *h;
  o.x += scale * s.x; o.y += scale * s.y; o.z += scale * s.z; o.w += scale * s.w;
  *h = o;
}

// lower triangle <- transpose of the upper triangle, 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void symmetrize_kernel(float* __restrict__ H, int d) {
  __shared__ float t[32][33];
  const int bi = blockIdx.y, bj = blockIdx.x;      // tile (bi, bj) with bj >= bi is the source
  if (bj < bi) return;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int y = ty; y < 32; y += 8) {
    const int r = bi * 32 + y, c = bj * 32 + tx;
    t[y][tx] = (r < d && c < d) ? H[(long)r * d + c] : 0.f;
  }
  __syncthreads();
  for (int y = ty; y < 32; y += 8) {
    const int r = bj * 32 + y, c = bi * 32 + tx;     // destination (r, c) = source (c, r)
    if (r < d && c < d && r > c) H[(long)r * d + c] = t[tx][y];
  }
}

}  // namespace bpdq

using namespace bpdq;

extern "C" size_t bpdq_hessian_workspace_bytes(int n_tok, int d_in) {
  if (n_tok <= 0 || d_in <= 0) return 0;
  const HessPlan p = plan_hessian(n_tok, d_in);
  if (p.S == 1) return 0;
  return (size_t)p.S * p.n_tiles * HessGemm::kTileM * HessGemm::kTileN * sizeof(float);
}

extern "C" int bpdq_hessian_accumulate(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                                       float* H, int symmetrize, void* ws, size_t ws_bytes,
                                       void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (n_tok < 0) return -2;
  if (d_in <= 0 || d_in % 4) return -3;
  if (ldx < d_in || ldx % 4) return -4;
  if (n_tok > 0 && (!Xc || (reinterpret_cast<uintptr_t>(Xc) & 15))) return -1;
  if (!H || (reinterpret_cast<uintptr_t>(H) & 15)) return -6;
  if (n_tok > 0) {
    const HessPlan p = plan_hessian(n_tok, d_in);
    const size_t need = p.S == 1 ? 0 : (size_t)p.S * p.n_tiles * HessGemm::kTileM * HessGemm::kTileN * sizeof(float);
    if (need > 0 && (!ws || (reinterpret_cast<uintptr_t>(ws) & 15))) return -8;
    if (ws_bytes < need) return -9;
    static bool attr_set = false;
    if (!attr_set) {
      BPDQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(hess_syrk_f32_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)HessGemm::kLdsBytes));
      attr_set = true;
    }
    hipLaunchKernelGGL(hess_syrk_f32_kernel, dim3(p.n_tiles * p.S), dim3(HessGemm::kThreads),
                       HessGemm::kLdsBytes, stream, Xc, n_tok, d_in, (long)ldx, scale, H,
                       static_cast<float*>(ws), p.nb, p.n_tiles, p.S, p.k_per);
    BPDQ_LAUNCH_CHECK();
    if (p.S > 1) {
      hipLaunchKernelGGL(hess_reduce_kernel, dim3(p.n_tiles * 64), dim3(256), 0, stream,
                         static_cast<const float*>(ws), p.n_tiles, p.S, p.nb, d_in, scale, H);
      BPDQ_LAUNCH_CHECK();
    }
  }
  if (symmetrize) {
    const int nt = bpdq_ceil_div(d_in, 32);
    hipLaunchKernelGGL(symmetrize_kernel, dim3(nt, nt), dim3(256), 0, stream, H, d_in);
    BPDQ_LAUNCH_CHECK();
  }
  return 0;
}
