// Symmetric tile product on the fp16 matrix cores from pre-split operands (split-precision SYRK):
//   C[m][n] = sum_k X[k][m0 + m] * X[k][n0 + n]
// where every value, scaled per channel by a power of two so that the channel's largest magnitude
// lies in [2^13, 2^14), has been cut into two halves  x s = h + l,  h = fp16(x s),
// l = fp16(x s - h)  (the difference is exact in fp32; 22 significant bits survive, and a value
// far below its channel's maximum keeps an absolute error of 2^-25 in the scaled units).  A product
// keeps the three terms of weight >= 2^-11,
//   x y = h h' + (h l' + l h')  +  O(2^-22 |x y|),
// each an exact fp16 x fp16 product accumulated in fp32 by v_mfma_f32_32x32x16_f16: three 8-pass
// instructions per 16 tokens where the fp32 matrix cores need eight 16-pass instructions.
//
// The split is done once per call by a streaming pre-pass (hessian.hip) that also lays the halves
// out in the operand order of the instruction: plane[piece][token / 8][channel] is a 16-byte
// vector of 8 consecutive tokens of one channel -- exactly one lane's A or B operand (lane l: row
// or column l % 32, tokens 8 (l / 32) .. + 7).  A stage of 16 tokens of a 256-channel operand is
// four runs of 4 KB, which go from global memory straight into LDS (global_load_lds_dwordx4: no
// registers, no conversion, no LDS-store instructions in the main loop) and from there to the
// lanes with conflict-free ds_read_b128.
//
// Work-group: 256 threads = 2 x 2 wavefronts, one per SIMD, each owning 128 x 128 = 4 x 4 blocks
// of 32 x 32 (256 accumulator registers): 16 fragment reads feed 48 MFMAs per stage.  LDS holds a
// ring of kStages stages (32 KB each); a stage is requested kStages - 1 iterations before its
// MFMAs and read into registers one iteration before them, so neither memory nor LDS latency is
// on the matrix pipe's path.  The compiler does not see the LDS-DMA loads (inline assembly), so
// the vmcnt waits that order them against the LDS reads are written by hand.
#pragma once
#include "common.h"

namespace bpdq {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

struct SplitF16 {
  static constexpr int kTile = 256;                        // channels per operand tile
  static constexpr int kThreads = 256;
  static constexpr int kStageK = 16;                       // tokens per stage = k of one MFMA
  static constexpr int kVecRun = kTile;                    // one (piece, k-group) run: 256 vectors = 4 KB
  static constexpr int kVecOperand = 4 * kVecRun;          // [piece 2][k-group 2][channel 256]
  static constexpr int kVecStage = 2 * kVecOperand;        // operands A, B: 32 KB
#ifndef BPDQ_F16_STAGES
#define BPDQ_F16_STAGES 4
#endif
  static constexpr int kStages = BPDQ_F16_STAGES;
  static constexpr size_t kLdsBytes = (size_t)kStages * kVecStage * 16u;
  static constexpr int kDiagBlocks = 9;                    // blocks per wavefront of a diagonal tile

  struct Acc {
    f32x16_t c[4][4];        // off-diagonal: block (i, j) of the wavefront's 4 x 4; diagonal: q = 4 i + j < 9
  };
  __device__ static __forceinline__ void zero(Acc& acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc.c[i][j][r] = 0.f;
  }

  // Upper-triangular schedule of a diagonal tile: its 36 blocks on or above the diagonal dealt to
  // the four wavefronts, nine each, as (block row, block column).
  static constexpr int kDiagRow[4][9] = {{0, 0, 0, 0, 0, 0, 0, 0, 7}, {1, 1, 1, 1, 1, 1, 1, 6, 6},
                                         {2, 2, 2, 2, 2, 2, 5, 5, 5}, {3, 3, 3, 3, 3, 4, 4, 4, 4}};
  static constexpr int kDiagCol[4][9] = {{0, 1, 2, 3, 4, 5, 6, 7, 7}, {1, 2, 3, 4, 5, 6, 7, 6, 7},
                                         {2, 3, 4, 5, 6, 7, 5, 6, 7}, {3, 4, 5, 6, 7, 4, 5, 6, 7}};

  // One LDS-DMA load: 64 lanes x 16 bytes from `base + voff` (per lane) to the 1 KB of LDS that
  // starts at byte address lds_addr (wave-uniform, handed over in M0; the kernel uses M0 for
  // nothing else).  Counts as one outstanding vector-memory operation of the wavefront.
  __device__ static __forceinline__ void dma_1k(const uint4* base, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
  }
  template <int N>
  __device__ static __forceinline__ void wait_vm() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    // vmcnt is split over bits 3:0 and 15:14 of the immediate; expcnt / lgkmcnt fields stay at
    // their maxima (no wait)
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0070 | 0x0f00);
  }

  struct Frag {
    f16x8 h, l;
  };
  __device__ static __forceinline__ Frag read_frag(const uint4* smem, int idx) {
    Frag f;
    f.h = __builtin_bit_cast(f16x8, smem[idx]);
    f.l = __builtin_bit_cast(f16x8, smem[idx + 2 * kVecRun]);
    return f;
  }
  // the three products of a block, smallest first
  template <int T>
  __device__ static __forceinline__ void piece_mfma(const Frag& a, const Frag& b, f32x16_t& c) {
    if constexpr (T == 0) c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.l, b.h, c, 0, 0, 0);
    if constexpr (T == 1) c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.l, c, 0, 0, 0);
    if constexpr (T == 2) c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.h, b.h, c, 0, 0, 0);
  }

  // Fragment t (0..7) of a stage for this wavefront.  Off-diagonal: 0..3 the four row blocks of A,
  // 4..7 the four column blocks of B.  Diagonal: block t of the one operand.
  template <bool DIAG, int T>
  __device__ static __forceinline__ Frag read_one(const uint4* smem, int buf, int a_idx, int b_idx) {
    const int base = buf * kVecStage;
    if constexpr (DIAG) return read_frag(smem, base + a_idx + 32 * T);
    else if constexpr (T < 4) return read_frag(smem, base + a_idx + 32 * T);
    else return read_frag(smem, base + kVecOperand + b_idx + 32 * (T - 4));
  }

  // The MFMAs of a stage in issue order: three passes (products l h', h l', h h': smallest first)
  // over the wavefront's blocks, so that consecutive instructions write different accumulators.
  // Off-diagonal: 16 blocks (i, j); diagonal: the 9 blocks of wavefront W's schedule.
  template <bool DIAG, int W>
  static constexpr int kMfmaPerStage = 3 * (DIAG ? kDiagBlocks : 16);
  template <bool DIAG, int W, int N>
  __device__ static __forceinline__ void mfma_n(const Frag (&f)[8], Acc& acc) {
    constexpr int nb = DIAG ? kDiagBlocks : 16;
    constexpr int t = N / nb, q = N % nb;
    if constexpr (DIAG) piece_mfma<t>(f[kDiagRow[W][q]], f[kDiagCol[W][q]], acc.c[q / 4][q % 4]);
    else piece_mfma<t>(f[q / 4], f[4 + q % 4], acc.c[q / 4][q % 4]);
  }
  template <bool DIAG, int W, int N0, int N1>
  __device__ static __forceinline__ void mfma_range(const Frag (&f)[8], Acc& acc) {
    if constexpr (N0 < N1) {
      mfma_n<DIAG, W, N0>(f, acc);
      mfma_range<DIAG, W, N0 + 1, N1>(f, acc);
    }
  }

  // acc += sum over k-groups [kg_begin, kg_begin + 2 n_stage) of the tile product of the channel
  // tiles at m0 and n0 (multiples of 256, below d_pad).  planes: [piece][n_kg][d_pad] vectors.
  // n_stage must be even (the pre-pass pads the token axis with zeros to a multiple of 32): the
  // loop below handles two stages per iteration without a branch inside.
  // DIAG: m0 == n0, only the blocks of the upper-triangular schedule are accumulated.
  // All threads of the work-group call this with identical arguments; uses kLdsBytes of dynamic LDS.
  template <bool DIAG>
  __device__ static __forceinline__ void run(const uint4* __restrict__ planes, long n_kg, int d_pad,
                                             int m0, int n0, long kg_begin, int n_stage, Acc& acc) {
    if constexpr (DIAG) {
      // the wavefront's block schedule is a compile-time table: one copy of the loop per wavefront
      switch (threadIdx.x >> 6) {
        case 0: run_wave<true, 0>(planes, n_kg, d_pad, m0, n0, kg_begin, n_stage, acc); break;
        case 1: run_wave<true, 1>(planes, n_kg, d_pad, m0, n0, kg_begin, n_stage, acc); break;
        case 2: run_wave<true, 2>(planes, n_kg, d_pad, m0, n0, kg_begin, n_stage, acc); break;
        default: run_wave<true, 3>(planes, n_kg, d_pad, m0, n0, kg_begin, n_stage, acc); break;
      }
    } else {
      run_wave<false, 0>(planes, n_kg, d_pad, m0, n0, kg_begin, n_stage, acc);
    }
  }

  template <bool DIAG, int W>
  __device__ static __forceinline__ void run_wave(const uint4* __restrict__ planes, long n_kg, int d_pad,
                                                  int m0, int n0, long kg_begin, int n_stage, Acc& acc) {
    extern __shared__ uint4 smem_f16[];
    if (n_stage <= 0) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: addresses below are scalar
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int kRuns = DIAG ? 4 : 8;                    // 4 KB runs per stage; a quarter each per wavefront
    // run r = 4 * operand + 2 * piece + k-group: global vector of its first channel in stage 0
    const uint4* src[kRuns];
#pragma unroll
    for (int r = 0; r < kRuns; ++r) {
      const int opnd = r >> 2, piece = (r >> 1) & 1, half = r & 1;
      src[r] = planes + ((long)piece * n_kg + kg_begin + half) * d_pad + (opnd ? n0 : m0) + wave * 64;
    }
    const long stage_stride = 2L * d_pad;                  // vectors between consecutive stages
    const unsigned voff = lane * 16u;
    typedef __attribute__((address_space(3))) uint4 lds_vec;
    const unsigned lds0 = (unsigned)(size_t)(lds_vec*)smem_f16 + wave * 1024u;   // LDS byte address
    auto request = [&](int s, int ring) {                  // stage s of the operands -> ring slot `ring` % kStages
      const unsigned slot = lds0 + (unsigned)(ring % kStages) * (kVecStage * 16u);
#pragma unroll
      for (int r = 0; r < kRuns; ++r)
        dma_1k(src[r] + (long)s * stage_stride, voff, slot + (unsigned)r * (kVecRun * 16u));
    };
    // the last stages are requested again instead of nothing, into slots nobody reads any more, so
    // that the number of outstanding loads -- what the vmcnt waits count -- is the same in every
    // iteration
    const int last = n_stage - 1;
    constexpr int kAhead = kStages - 1;                    // stages requested ahead of the current one
#pragma unroll
    for (int s = 0; s < kAhead; ++s) request(s < last ? s : last, s);
    wait_vm<kRuns*(kAhead - 1)>();                         // stage 0 of this wavefront has landed
    __syncthreads();                                       // ... and of the others

    const int a_idx = (lane >> 5) * kVecRun + (DIAG ? 0 : wm * 128) + (lane & 31);
    const int b_idx = (lane >> 5) * kVecRun + wn * 128 + (lane & 31);
    Frag f0[8], f1[8];
    f0[0] = read_one<DIAG, 0>(smem_f16, 0, a_idx, b_idx); f0[1] = read_one<DIAG, 1>(smem_f16, 0, a_idx, b_idx);
    f0[2] = read_one<DIAG, 2>(smem_f16, 0, a_idx, b_idx); f0[3] = read_one<DIAG, 3>(smem_f16, 0, a_idx, b_idx);
    f0[4] = read_one<DIAG, 4>(smem_f16, 0, a_idx, b_idx); f0[5] = read_one<DIAG, 5>(smem_f16, 0, a_idx, b_idx);
    f0[6] = read_one<DIAG, 6>(smem_f16, 0, a_idx, b_idx); f0[7] = read_one<DIAG, 7>(smem_f16, 0, a_idx, b_idx);

    // One stage = eight steps; step t requests run t of the stage kAhead ahead (runs 0..3 only on a
    // diagonal tile), reads fragment t of the next stage and issues an eighth of this stage's
    // MFMAs.  A wavefront is alone on its SIMD, so whatever it issues between two MFMAs must fit
    // under the 32 cycles the matrix pipe spends on one: spread like this, the loads and LDS
    // reads cost the pipe nothing, bunched at the head of the stage they would stall it.
    constexpr int kM = kMfmaPerStage<DIAG, W>;
    auto stage = [&](int s, Frag (&cur)[8], Frag (&nxt)[8]) {
      // stage s + 1 must be complete in LDS before its fragments are read below; the barrier also
      // tells that every wavefront has consumed stage s - 1, whose slot the requests overwrite
      // (a bare barrier: the LDS reads still in flight belong to this stage's own slot, which no
      // request touches, so they need not be waited for here; the empty statement keeps the
      // compiler from moving an LDS access across the barrier)
      wait_vm<kRuns*(kAhead - 2)>();
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      const int sr = s + kAhead;
      const int sc = sr < last ? sr : last;
      const unsigned slot = lds0 + (unsigned)(sr % kStages) * (kVecStage * 16u);
      const int nb = (s + 1) % kStages;          // (after the last stage: a slot nobody uses)
#define BPDQ_F16_STEP(T)                                                                         \
      if constexpr (T < kRuns)                                                                     \
        dma_1k(src[T < kRuns ? T : 0] + (long)sc * stage_stride, voff, slot + (unsigned)(T) * (kVecRun * 16u)); \
      nxt[T] = read_one<DIAG, T>(smem_f16, nb, a_idx, b_idx);                                      \
      mfma_range<DIAG, W, (T) * kM / 8, ((T) + 1) * kM / 8>(cur, acc);                             \
      __builtin_amdgcn_sched_barrier(0);
      BPDQ_F16_STEP(0) BPDQ_F16_STEP(1) BPDQ_F16_STEP(2) BPDQ_F16_STEP(3)
      BPDQ_F16_STEP(4) BPDQ_F16_STEP(5) BPDQ_F16_STEP(6) BPDQ_F16_STEP(7)
#undef BPDQ_F16_STEP
    };
    for (int s = 0; s < n_stage; s += 2) {
      stage(s, f0, f1);
      stage(s + 1, f1, f0);
    }
    wait_vm<0>();            // no load may still be writing LDS when the work-group moves on
    __syncthreads();
  }

  // f(row_in_tile, col_in_tile, value) over this lane's results of an off-diagonal tile
  template <typename F>
  __device__ static __forceinline__ void for_each(const Acc& acc, F f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          f(wm * 128 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), wn * 128 + j * 32 + (lane & 31),
            acc.c[i][j][r]);
  }
  // ... of a diagonal tile (upper-triangular schedule)
  template <typename F>
  __device__ static __forceinline__ void for_each_diag(const Acc& acc, F f) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int q = 0; q < kDiagBlocks; ++q) {
      const int rb = kDiagRow[wave][q], cb = kDiagCol[wave][q];
#pragma unroll
      for (int r = 0; r < 16; ++r)
        f(32 * rb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), 32 * cb + (lane & 31), acc.c[q / 4][q % 4][r]);
    }
  }
};

}  // namespace bpdq
