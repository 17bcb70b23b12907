// fp32 MFMA tile product for operands stored "K-major":
//   C[m][n] = sum_k A[k][m] * B[k][n],   A row k holds all m contiguously, likewise B.
// Both dense contractions of the pass have this shape:
//   Hessian      H[i][j]  += sum_t X[t][i] X[t][j]            (A = B = token-major X)
//   block update W'[r][c] -= sum_l Et[l][r] U[l][c]            (A = E transposed, B = rows of U)
//
// Work-group: 512 threads = 8 wavefronts arranged 4 (M) x 2 (N); block tile 256 x 256; each
// wavefront owns 64 x 128 = 2 x 4 tiles of v_mfma_f32_32x32x2_f32 (128 accumulator registers).
// K is consumed in stages of 16 rows, double-buffered through LDS (2 x 32 KB): the next
// stage's global loads are issued before the current stage's 64 MFMAs and parked in
// registers, so HBM/L2 latency hides behind 4096 MFMA cycles.
//
// Operand register layout of v_mfma_f32_32x32x2_f32 (64 lanes):
//   A: lane l holds A[m = l % 32][k = l / 32];  B: lane l holds B[k = l / 32][n = l % 32];
//   D: register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l % 32].
// With K-major tiles in LDS both operand reads are 32 consecutive floats per half-wave:
// conflict-free ds_read_b32.
#pragma once
#include "common.h"

namespace bpdq {

constexpr int kTileM = 256;
constexpr int kTileN = 256;
constexpr int kStageK = 16;
constexpr int kGemmThreads = 512;
constexpr int kStageFloats = kStageK * kTileM;          // one operand, one stage
constexpr size_t kGemmLdsBytes = 4u * kStageFloats * sizeof(float);   // A,B x 2 buffers = 64 KB

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct TileAcc {
  f32x16 c[2][4];
};

struct StageRegs {
  float4 a[2];
  float4 b[2];
};

// Loads rows [k0, k0+16) x columns [col0, col0+256) of a K-major operand; out-of-range rows
// (>= k_end) and columns (>= col_lim) read as zero.  Thread t covers float4 column t%64 of
// rows t/64 and t/64+8.
__device__ __forceinline__ void load_stage_operand(const float* __restrict__ P, long ld, int k0,
                                                   int k_end, int col0, int col_lim,
                                                   float4 (&r)[2]) {
  const int c = col0 + (threadIdx.x & 63) * 4;
  const int kr = k0 + (threadIdx.x >> 6);
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int k = kr + 8 * p;
    if (k < k_end && c < col_lim) {
      r[p] = *reinterpret_cast<const float4*>(P + (long)k * ld + c);
    } else {
      r[p] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}

__device__ __forceinline__ void store_stage_operand(float* s, const float4 (&r)[2]) {
  const int c = (threadIdx.x & 63) * 4;
  const int kr = threadIdx.x >> 6;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    *reinterpret_cast<float4*>(s + (kr + 8 * p) * kTileM + c) = r[p];
  }
}

// acc += A[k_begin:k_end, m0:m0+256]^T * B[k_begin:k_end, n0:n0+256].
// SAME_TILE: A and B are the same tile (diagonal block of a symmetric product), B is not
// loaded.  All 512 threads of the work-group must call this with identical arguments.
template <bool SAME_TILE>
__device__ __forceinline__ void mfma_kmajor_tile(const float* __restrict__ A, long lda, int m0,
                                                 int m_lim, const float* __restrict__ B, long ldb,
                                                 int n0, int n_lim, int k_begin, int k_end,
                                                 TileAcc& acc) {
  // dynamic LDS of the kernel: [buffer][operand][16][256]; addressed by integer offsets so the
  // compiler keeps the LDS address space (ds_read/ds_write, not flat accesses)
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1;   // 0..3
  const int wn = wave & 1;    // 0..1
  constexpr int kBufFloats = 2 * kStageFloats;
  constexpr int kBOff = SAME_TILE ? 0 : kStageFloats;

  const int n_stage = (k_end - k_begin + kStageK - 1) / kStageK;
  if (n_stage <= 0) return;
  StageRegs g;
  load_stage_operand(A, lda, k_begin, k_end, m0, m_lim, g.a);
  if (!SAME_TILE) load_stage_operand(B, ldb, k_begin, k_end, n0, n_lim, g.b);
  store_stage_operand(smem, g.a);
  if (!SAME_TILE) store_stage_operand(smem + kStageFloats, g.b);
  __syncthreads();

  const int a_off = (lane >> 5) * kTileM + wm * 64 + (lane & 31);
  const int b_off = (lane >> 5) * kTileM + wn * 128 + (lane & 31);
  for (int s = 0; s < n_stage; ++s) {
    const int cur = s & 1;
    const bool more = (s + 1 < n_stage);
    if (more) {
      const int k0 = k_begin + (s + 1) * kStageK;
      load_stage_operand(A, lda, k0, k_end, m0, m_lim, g.a);
      if (!SAME_TILE) load_stage_operand(B, ldb, k0, k_end, n0, n_lim, g.b);
    }
    const int pa = cur * kBufFloats + a_off;
    const int pb = cur * kBufFloats + kBOff + b_off;
#pragma unroll
    for (int kk = 0; kk < kStageK; kk += 2) {
      float a[2], b[4];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = smem[pa + kk * kTileM + i * 32];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = smem[pb + kk * kTileM + j * 32];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc.c[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc.c[i][j], 0, 0, 0);
    }
    if (more) {
      store_stage_operand(smem + (cur ^ 1) * kBufFloats, g.a);
      if (!SAME_TILE) store_stage_operand(smem + (cur ^ 1) * kBufFloats + kStageFloats, g.b);
    }
    __syncthreads();
  }
}

__device__ __forceinline__ void zero_acc(TileAcc& acc) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;
}

// Calls f(row_in_tile, col_in_tile, value) for the 128 accumulator values of this lane.
template <typename F>
__device__ __forceinline__ void for_each_acc(const TileAcc& acc, F f) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int col = wn * 128 + j * 32 + (lane & 31);
        f(row, col, acc.c[i][j][r]);
      }
}

}  // namespace bpdq
