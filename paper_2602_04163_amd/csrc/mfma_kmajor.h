// fp32 MFMA tile product for operands stored "K-major":
//   C[m][n] = sum_k A[k][m] * B[k][n],   A row k holds all m contiguously, likewise B.
// Both dense contractions of the pass have this shape:
//   Hessian      H[i][j]  += sum_t X[t][i] X[t][j]            (A = B = token-major X)
//   block update W'[r][c] -= sum_l Et[l][r] U[l][c]            (A = E transposed, B = rows of U)
//
// KMajorGemm<WM, WN, TI, TJ>: WM x WN wavefronts per work-group, each owning TI x TJ tiles of
// v_mfma_f32_32x32x2_f32 (16 accumulator registers per tile).  K is consumed in stages of
// 16 rows, double-buffered through LDS: the next stage's global loads are issued before the
// current stage's MFMAs and parked in registers, so HBM/L2 latency hides behind the MFMAs.
//   Hessian:      <4, 2, 2, 4>  512 threads, 256 x 256 tile, 64 KB LDS  (long K, maximal reuse)
//   block update: <2, 2, 2, 2>  256 threads, 128 x 128 tile, 32 KB LDS  (K = 128: many small
//                 work-groups, so that every launch spreads over all compute units)
//
// Operand register layout of v_mfma_f32_32x32x2_f32 (64 lanes):
//   A: lane l holds A[m = l % 32][k = l / 32];  B: lane l holds B[k = l / 32][n = l % 32];
//   D: register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l % 32].
// With K-major tiles in LDS both operand reads are 32 consecutive floats per half-wave:
// conflict-free LDS reads, and no transpose anywhere.
#pragma once
#include "common.h"

namespace bpdq {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kStageK = 16;

template <int WM, int WN, int TI, int TJ>
struct KMajorGemm {
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int kTileM = 32 * TI * WM;
  static constexpr int kTileN = 32 * TJ * WN;
  static constexpr int kStageA = kStageK * kTileM;            // floats per stage, operand A
  static constexpr int kStageB = kStageK * kTileN;
  static constexpr int kBufFloats = kStageA + kStageB;
  static constexpr size_t kLdsBytes = 2u * kBufFloats * sizeof(float);
  static constexpr int kVecA = kStageA / 4 / kThreads;         // float4 loads per thread per stage
  static constexpr int kVecB = kStageB / 4 / kThreads;
  static_assert(kStageA % (4 * kThreads) == 0 && kStageB % (4 * kThreads) == 0, "tile/threads");

  struct Acc {
    f32x16 c[TI][TJ];
  };

  __device__ static __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;
  }

  // Rows [k0, k0+16) x columns [col0, col0+TILE) of a K-major operand; rows >= k_end and
  // columns >= col_lim read as zero (col_lim and col0 are multiples of 4).
  template <int TILE, int NV>
  __device__ static __forceinline__ void load_stage(const float* __restrict__ P, long ld, int k0,
                                                    int k_end, int col0, int col_lim,
                                                    float4 (&r)[NV]) {
    constexpr int kVecPerRow = TILE / 4;
#pragma unroll
    for (int p = 0; p < NV; ++p) {
      const int v = threadIdx.x + p * kThreads;
      const int k = k0 + v / kVecPerRow;
      const int c = col0 + (v % kVecPerRow) * 4;
      if (k < k_end && c < col_lim) {
        r[p] = *reinterpret_cast<const float4*>(P + (long)k * ld + c);
      } else {
        r[p] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  }

  template <int NV>
  __device__ static __forceinline__ void store_stage(float* s, const float4 (&r)[NV]) {
#pragma unroll
    for (int p = 0; p < NV; ++p) {
      const int v = threadIdx.x + p * kThreads;
      *reinterpret_cast<float4*>(s + v * 4) = r[p];
    }
  }

  // acc += A[k_begin:k_end, m0:m0+TileM]^T * B[k_begin:k_end, n0:n0+TileN].
  // SAME_TILE: A and B are the same tile (diagonal block of a symmetric product; needs
  // TileM == TileN), B is not loaded.  All threads of the work-group must call this with
  // identical arguments.  Uses the kernel's dynamic LDS (kLdsBytes).
  template <bool SAME_TILE>
  __device__ static __forceinline__ void run(const float* __restrict__ A, long lda, int m0,
                                             int m_lim, const float* __restrict__ B, long ldb,
                                             int n0, int n_lim, int k_begin, int k_end, Acc& acc) {
    // [buffer][A stage | B stage]; addressed by integer offsets so the compiler keeps the LDS
    // address space (ds_read / ds_write instead of flat accesses)
    extern __shared__ float smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / WN;
    const int wn = wave % WN;
    constexpr int kBOff = SAME_TILE ? 0 : kStageA;

    const int n_stage = (k_end - k_begin + kStageK - 1) / kStageK;
    if (n_stage <= 0) return;
    float4 ga[kVecA], gb[kVecB];
    load_stage<kTileM, kVecA>(A, lda, k_begin, k_end, m0, m_lim, ga);
    if (!SAME_TILE) load_stage<kTileN, kVecB>(B, ldb, k_begin, k_end, n0, n_lim, gb);
    store_stage<kVecA>(smem, ga);
    if (!SAME_TILE) store_stage<kVecB>(smem + kStageA, gb);
    __syncthreads();

    const int a_off = (lane >> 5) * kTileM + wm * (32 * TI) + (lane & 31);
    const int b_off = (lane >> 5) * (SAME_TILE ? kTileM : kTileN) + wn * (32 * TJ) + (lane & 31);
    for (int s = 0; s < n_stage; ++s) {
      const int cur = s & 1;
      const bool more = (s + 1 < n_stage);
      if (more) {
        const int k0 = k_begin + (s + 1) * kStageK;
        load_stage<kTileM, kVecA>(A, lda, k0, k_end, m0, m_lim, ga);
        if (!SAME_TILE) load_stage<kTileN, kVecB>(B, ldb, k0, k_end, n0, n_lim, gb);
      }
      const int pa = cur * kBufFloats + a_off;
      const int pb = cur * kBufFloats + kBOff + b_off;
#pragma unroll
      for (int kk = 0; kk < kStageK; kk += 2) {
        float a[TI], b[TJ];
#pragma unroll
        for (int i = 0; i < TI; ++i) a[i] = smem[pa + kk * kTileM + i * 32];
#pragma unroll
        for (int j = 0; j < TJ; ++j) b[j] = smem[pb + kk * (SAME_TILE ? kTileM : kTileN) + j * 32];
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j)
            acc.c[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc.c[i][j], 0, 0, 0);
      }
      if (more) {
        store_stage<kVecA>(smem + (cur ^ 1) * kBufFloats, ga);
        if (!SAME_TILE) store_stage<kVecB>(smem + (cur ^ 1) * kBufFloats + kStageA, gb);
      }
      __syncthreads();
    }
  }

  // Calls f(row_in_tile, col_in_tile, value) for the accumulator values of this lane.
  template <typename F>
  __device__ static __forceinline__ void for_each(const Acc& acc, F f) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / WN, wn = wave % WN;
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = wm * (32 * TI) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const int col = wn * (32 * TJ) + j * 32 + (lane & 31);
          f(row, col, acc.c[i][j][r]);
        }
  }
};

using HessGemm = KMajorGemm<4, 2, 2, 4>;   // 256 x 256, 512 threads
using TailGemm = KMajorGemm<2, 2, 2, 2>;   // 128 x 128, 256 threads

}  // namespace bpdq
