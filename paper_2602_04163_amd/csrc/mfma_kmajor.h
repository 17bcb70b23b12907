// fp32 MFMA tile product for operands stored "K-major":
//   C[m][n] = sum_k A[k][m] * B[k][n],   A row k holds all m contiguously, likewise B.
// Both dense contractions of the pass have this shape:
//   Hessian      H[i][j]  += sum_t X[t][i] X[t][j]            (A = B = token-major X)
//   block update W'[r][c] -= sum_l Et[l][r] U[l][c]            (A = E transposed, B = rows of U)
//
// KMajorGemm<WM, WN, TI, TJ, SK>: WM x WN wavefronts per work-group, each owning TI x TJ tiles
// of v_mfma_f32_32x32x2_f32 (16 accumulator registers per tile).  K is consumed in stages of
// SK rows, double-buffered through LDS: the next stage's global loads are issued early in the
// current stage and parked in registers, and written to the other LDS buffer late in it, both
// in the shadow of MFMAs.  The two wavefronts that share a SIMD do this at different k-steps:
// a barrier puts them in phase, and a non-MFMA section run by both at once would idle the pipe.
//   Hessian:      <4, 2, 2, 4, 32>  512 threads, 256 x 256 tile  (long K, maximal reuse)
//   block update: <2, 2, 2, 2, 16>  256 threads, 128 x 128 tile  (K = 128: many small
//                 work-groups so that every launch spreads over all compute units and several
//                 work-groups share a compute unit, hiding one another's load latency)
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

template <int WM, int WN, int TI, int TJ, int SK>
struct KMajorGemm {
  static constexpr int kStageK = SK;                          // K rows per LDS stage
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
  static constexpr int kAccPerLane = TI * TJ * 16;             // accumulator values per lane

  __device__ static __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;
  }

  // Rows [k0, k0+SK) x columns [col0, col0+TILE) of a K-major operand; rows >= k_end and
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

  // Same rows and columns without any bounds test: p points at this thread's first vector of
  // the stage (row threadIdx / (TILE/4)); vector q lies q * (threads / (TILE/4)) rows below.
  template <int TILE, int NV>
  __device__ static __forceinline__ void load_stage_fast(const float* __restrict__ p, long ld,
                                                         float4 (&r)[NV]) {
    constexpr int kRowStep = kThreads / (TILE / 4);
#pragma unroll
    for (int q = 0; q < NV; ++q) r[q] = *reinterpret_cast<const float4*>(p + (long)q * kRowStep * ld);
  }

  template <int NV>
  __device__ static __forceinline__ void store_stage(float* s, const float4 (&r)[NV]) {
#pragma unroll
    for (int p = 0; p < NV; ++p) {
      const int v = threadIdx.x + p * kThreads;
      *reinterpret_cast<float4*>(s + v * 4) = r[p];
    }
  }

  // Upper-triangular schedule of a diagonal (symmetric) 256 x 256 tile, <4, 2, 2, 4> only: the
  // 36 blocks of 32 x 32 on or above the diagonal are dealt to the 8 wavefronts, at most 5
  // each (a full tile costs 8 per wavefront), as (block row, block column) pairs.
  static constexpr int kDiagN[8] = {5, 5, 5, 5, 5, 5, 5, 1};
  static constexpr int kDiagRow[8][5] = {{0, 0, 0, 0, 0}, {0, 0, 0, 6, 6}, {1, 1, 1, 1, 1}, {1, 1, 5, 5, 5},
                                         {2, 2, 2, 2, 2}, {2, 4, 4, 4, 4}, {3, 3, 3, 3, 3}, {7, 7, 7, 7, 7}};
  static constexpr int kDiagCol[8][5] = {{0, 1, 2, 3, 4}, {5, 6, 7, 6, 7}, {1, 2, 3, 4, 5}, {6, 7, 5, 6, 7},
                                         {2, 3, 4, 5, 6}, {7, 4, 5, 6, 7}, {3, 4, 5, 6, 7}, {7, 7, 7, 7, 7}};

  template <int W>
  __device__ static __forceinline__ void diag_stage(const float* smem, int base, Acc& acc) {
#pragma unroll
    for (int kk = 0; kk < kStageK; kk += 2) {
      float a[5], b[5];
#pragma unroll
      for (int q = 0; q < kDiagN[W]; ++q) {
        a[q] = smem[base + kk * kTileM + 32 * kDiagRow[W][q]];
        b[q] = smem[base + kk * kTileM + 32 * kDiagCol[W][q]];
      }
#pragma unroll
      for (int q = 0; q < kDiagN[W]; ++q)
        acc.c[q / TJ][q % TJ] =
            __builtin_amdgcn_mfma_f32_32x32x2f32(a[q], b[q], acc.c[q / TJ][q % TJ], 0, 0, 0);
    }
  }

  // f(row_in_tile, col_in_tile, value) for a tile accumulated with the upper-triangular schedule
  template <typename F>
  __device__ static __forceinline__ void for_each_diag(const Acc& acc, F f) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < 5; ++q) {
      if (q >= kDiagN[wave]) break;
      const int rb = kDiagRow[wave][q], cb = kDiagCol[wave][q];
#pragma unroll
      for (int r = 0; r < 16; ++r)
        f(32 * rb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), 32 * cb + (lane & 31),
          acc.c[q / TJ][q % TJ][r]);
    }
  }

  // acc += A[k_begin:k_end, m0:m0+TileM]^T * B[k_begin:k_end, n0:n0+TileN].
  // MODE 0: two different operand tiles.  MODE 1: A and B are the same tile (diagonal block of
  // a symmetric product; needs TileM == TileN), B is not loaded.  MODE 2: same tile, and only the
  // blocks on or above the diagonal are accumulated (read the result with for_each_diag).
  // All threads of the work-group must call this with identical arguments.  Uses the kernel's
  // dynamic LDS (kLdsBytes).
  template <int MODE>
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
    constexpr bool SAME_TILE = (MODE != 0);
    constexpr int kBOff = SAME_TILE ? 0 : kStageA;

    const int n_stage = (k_end - k_begin + kStageK - 1) / kStageK;
    if (n_stage <= 0) return;
    float4 ga[kVecA], gb[kVecB];
    load_stage<kTileM, kVecA>(A, lda, k_begin, k_end, m0, m_lim, ga);
    if (!SAME_TILE) load_stage<kTileN, kVecB>(B, ldb, k_begin, k_end, n0, n_lim, gb);
    store_stage<kVecA>(smem, ga);
    if (!SAME_TILE) store_stage<kVecB>(smem + kStageA, gb);
    __syncthreads();

    // per-thread source of the unchecked loads, and whether the tile needs column checks
    const float* srcA = A + (long)(k_begin + threadIdx.x / (kTileM / 4)) * lda + m0 + (threadIdx.x % (kTileM / 4)) * 4;
    const float* srcB = B + (long)(k_begin + threadIdx.x / (kTileN / 4)) * ldb + n0 + (threadIdx.x % (kTileN / 4)) * 4;
    const bool full_cols = (m0 + kTileM <= m_lim) && (SAME_TILE || n0 + kTileN <= n_lim);
    // the two wavefronts that share a SIMD run their load / store sections at different k-steps,
    // so that one of them always keeps the matrix pipe fed
    const bool late_half = wave >= (WM * WN) / 2;
    const int a_off = (lane >> 5) * kTileM + wm * (32 * TI) + (lane & 31);
    const int b_off = (lane >> 5) * (SAME_TILE ? kTileM : kTileN) + wn * (32 * TJ) + (lane & 31);
    for (int s = 0; s < n_stage; ++s) {
      const int cur = s & 1;
      const bool more = (s + 1 < n_stage);
      const int k0n = k_begin + (s + 1) * kStageK;
      if constexpr (MODE == 2) {
        static_assert(MODE != 2 || (WM == 4 && WN == 2 && TI == 2 && TJ == 4), "diag schedule");
        if (more) load_stage<kTileM, kVecA>(A, lda, k0n, k_end, m0, m_lim, ga);
        const int base = cur * kBufFloats + (lane >> 5) * kTileM + (lane & 31);
        switch (wave) {
          case 0: diag_stage<0>(smem, base, acc); break;
          case 1: diag_stage<1>(smem, base, acc); break;
          case 2: diag_stage<2>(smem, base, acc); break;
          case 3: diag_stage<3>(smem, base, acc); break;
          case 4: diag_stage<4>(smem, base, acc); break;
          case 5: diag_stage<5>(smem, base, acc); break;
          case 6: diag_stage<6>(smem, base, acc); break;
          default: diag_stage<7>(smem, base, acc); break;
        }
        if (more) store_stage<kVecA>(smem + (cur ^ 1) * kBufFloats, ga);
      } else {
        const int pa = cur * kBufFloats + a_off;
        const int pb = cur * kBufFloats + kBOff + b_off;
        constexpr int kPitchB = SAME_TILE ? kTileM : kTileN;
        constexpr int kSteps = kStageK / 2;
        // operand fragments are fetched one k-step ahead of the MFMAs that consume them
        float fa[2][TI], fb[2][TJ];
#pragma unroll
        for (int i = 0; i < TI; ++i) fa[0][i] = smem[pa + i * 32];
#pragma unroll
        for (int j = 0; j < TJ; ++j) fb[0][j] = smem[pb + j * 32];
        // k-steps after / before which the next stage is loaded from memory / written to LDS,
        // for the first and the second half of the wavefronts
        constexpr int kLoadEarly = 0, kLoadLate = kSteps / 2 - 1;
        constexpr int kStoreEarly = kSteps / 2, kStoreLate = kSteps - 1;
        static_assert(kSteps >= 4, "stage too short for the staggered schedule");
        const bool fast = full_cols && (k0n + kStageK <= k_end);
#pragma unroll
        for (int ks = 0; ks < kSteps; ++ks) {
          const int kk = 2 * ks;
          const int c = ks & 1, n = c ^ 1;
          if ((ks == kStoreEarly || ks == kStoreLate) && more && (late_half == (ks == kStoreLate))) {
            // next stage: registers -> the other LDS buffer, hidden behind the MFMAs in flight
            store_stage<kVecA>(smem + (cur ^ 1) * kBufFloats, ga);
            if (!SAME_TILE) store_stage<kVecB>(smem + (cur ^ 1) * kBufFloats + kStageA, gb);
          }
          if (ks + 1 < kSteps) {
#pragma unroll
            for (int i = 0; i < TI; ++i) fa[n][i] = smem[pa + (kk + 2) * kTileM + i * 32];
#pragma unroll
            for (int j = 0; j < TJ; ++j) fb[n][j] = smem[pb + (kk + 2) * kPitchB + j * 32];
          }
          __builtin_amdgcn_sched_barrier(0);      // keep the prefetch ahead of this step's MFMAs
#pragma unroll
          for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int j = 0; j < TJ; ++j)
              acc.c[i][j] =
                  __builtin_amdgcn_mfma_f32_32x32x2f32(fa[c][i], fb[c][j], acc.c[i][j], 0, 0, 0);
          if ((ks == kLoadEarly || ks == kLoadLate) && more && (late_half == (ks == kLoadLate))) {
            // global loads of the next stage go out while MFMAs occupy the pipe
            __builtin_amdgcn_sched_barrier(0);
            if (fast) {
              load_stage_fast<kTileM, kVecA>(srcA + (long)(s + 1) * kStageK * lda, lda, ga);
              if (!SAME_TILE) load_stage_fast<kTileN, kVecB>(srcB + (long)(s + 1) * kStageK * ldb, ldb, gb);
            } else {
              load_stage<kTileM, kVecA>(A, lda, k0n, k_end, m0, m_lim, ga);
              if (!SAME_TILE) load_stage<kTileN, kVecB>(B, ldb, k0n, k_end, n0, n_lim, gb);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
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

using HessGemm = KMajorGemm<4, 2, 2, 4, 32>;   // 256 x 256, 512 threads, 128 KB LDS
using TailGemm = KMajorGemm<2, 2, 2, 2, 16>;   // 128 x 128, 256 threads, 32 KB LDS

}  // namespace bpdq
