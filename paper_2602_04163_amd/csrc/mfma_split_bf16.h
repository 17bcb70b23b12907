// fp32-accurate symmetric tile product on the bf16 matrix cores (split-precision SYRK):
//   C[m][n] = sum_k X[k][m0 + m] * X[k][n0 + n],   X token-major (row k holds all channels).
//
// Every fp32 value is cut into three bf16 pieces, x = h + m + l exactly up to 2^-25 |x|
// (h = bf16(x), m = bf16(x - h), l = bf16(x - h - m); both differences are exact in fp32), and
// the product keeps the six piece products of weight >= 2^-16:
//   x y = h h' + (h m' + m h') + (m m' + h l' + l h')  +  O(2^-24 |x y|),
// each an exact bf16 x bf16 product accumulated in fp32 by v_mfma_f32_32x32x16_bf16.  The dropped
// terms are below the rounding of an fp32 product, so the result is as accurate as the fp32
// matrix-core path.  Six bf16 instructions of 8 passes cover 16 tokens where the fp32 path needs
// eight instructions of 16 passes: 2.67 times the fp32 rate at equal pipe utilisation.
//
// Work-group: 512 threads = 4 x 2 wavefronts, each 2 x 4 blocks of 32 x 32 (the accumulator
// layout of HessGemm, whose for_each / for_each_diag read the result).  K is consumed in stages
// of 16 tokens, double-buffered in LDS.  A thread stages one channel of one operand: 16 dword
// loads (64 lanes = 256 contiguous bytes per token row), split in registers, written as three
// pairs of 16-byte vectors "channel-major": LDS vector [piece][k-group of 8][channel] holds the
// 8 tokens of that k-group, which is exactly one lane's operand of the 32x32x16 MFMA
// (lane l: row/column l % 32, k = 8 * (l / 32) .. + 7).  Reads and writes of consecutive lanes
// are consecutive 16-byte vectors: no bank conflicts, no transpose pass.
// Loads for stage s + 3 are issued in stage s, right after their registers were drained into LDS
// for stage s + 1 (two register sets take turns), so they have two stages of MFMAs to land.
#pragma once
#include "mfma_kmajor.h"

namespace bpdq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

struct SplitSyrk {
  using Shape = HessGemm;                                   // tile and accumulator geometry
  static constexpr int kStageK = 16;                        // tokens per stage = k of one MFMA
  static constexpr int kTile = Shape::kTileM;               // 256 channels per operand
  static constexpr int kThreads = Shape::kThreads;          // 512
  static constexpr int kVecPiece = 2 * kTile;               // [k-group 2][channel 256] 16-byte vectors
  static constexpr int kVecOperand = 3 * kVecPiece;         // pieces h, m, l
  static constexpr int kVecBuf = 2 * kVecOperand;           // operands A, B
  static constexpr size_t kLdsBytes = 2u * kVecBuf * 16u;   // two buffers: 96 KB
  static_assert(kTile == 256 && kThreads == 512 && Shape::kTileN == 256, "one channel per thread");

  // 16 tokens of one channel, straight into the staging registers.  Nothing is selected or zeroed
  // here: an instruction that touched the loaded values would make the wavefront wait for memory
  // in the middle of its MFMAs.  Rows are clamped to the last token (store_group zeroes the tokens
  // past the end when it drains the registers) and ch is a valid channel (a channel past d_in
  // duplicates the last one; its rows and columns of the product are never stored).
  __device__ static __forceinline__ void load_tokens(const float* __restrict__ X, long ldx, int k0,
                                                     int k_end, int ch, bool fast,
                                                     float (&g)[kStageK]) {
    if (fast) {
      const float* p = X + (long)k0 * ldx + ch;
#pragma unroll
      for (int i = 0; i < kStageK; ++i) g[i] = p[(long)i * ldx];
    } else {
      const int k_last = k_end - 1;
#pragma unroll
      for (int i = 0; i < kStageK; ++i) g[i] = X[(long)min(k0 + i, k_last) * ldx + ch];
    }
  }

  // two values -> their (h, m, l) pieces, each pair packed low | high
  __device__ static __forceinline__ void split2(float x0, float x1, unsigned& h, unsigned& m,
                                                unsigned& l) {
    f32x2 v = {x0, x1};
    h = __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
    v[0] = x0 - __builtin_bit_cast(float, h << 16);
    v[1] = x1 - __builtin_bit_cast(float, h & 0xffff0000u);
    m = __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
    v[0] -= __builtin_bit_cast(float, m << 16);
    v[1] -= __builtin_bit_cast(float, m & 0xffff0000u);
    l = __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
  }

  // k-group kg (tokens 8 kg .. 8 kg + 7) of the staged registers -> LDS vectors at dst + kg * kTile;
  // only the first n_valid of the 16 staged tokens exist, the others count as zero
  template <int KG>
  __device__ static __forceinline__ void store_group(uint4* smem, int dst, const float (&g)[kStageK],
                                                     int n_valid) {
    unsigned h[4], m[4], l[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int i = 8 * KG + 2 * p;
      split2(i < n_valid ? g[i] : 0.f, i + 1 < n_valid ? g[i + 1] : 0.f, h[p], m[p], l[p]);
    }
    smem[dst + KG * kTile] = make_uint4(h[0], h[1], h[2], h[3]);
    smem[dst + KG * kTile + kVecPiece] = make_uint4(m[0], m[1], m[2], m[3]);
    smem[dst + KG * kTile + 2 * kVecPiece] = make_uint4(l[0], l[1], l[2], l[3]);
  }

  struct Frag {
    bf16x8 p[3];   // h, m, l
  };
  __device__ static __forceinline__ Frag read_frag(const uint4* smem, int idx) {
    Frag f;
#pragma unroll
    for (int s = 0; s < 3; ++s) f.p[s] = __builtin_bit_cast(bf16x8, smem[idx + s * kVecPiece]);
    return f;
  }

  // the six piece products, smallest first
  template <int T>
  __device__ static __forceinline__ void piece_mfma(const Frag& a, const Frag& b, f32x16& c) {
    constexpr int pa[6] = {2, 0, 1, 1, 0, 0};
    constexpr int pb[6] = {0, 2, 1, 0, 1, 0};
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.p[pa[T]], b.p[pb[T]], c, 0, 0, 0);
  }
  template <int NA>
  __device__ static __forceinline__ void product(const Frag (&a)[NA], const Frag& b, f32x16* c0,
                                                 f32x16* c1) {
    // accumulators alternate so that consecutive MFMAs are independent
    static_assert(NA == 2, "two row blocks per wavefront");
    piece_mfma<0>(a[0], b, *c0); piece_mfma<0>(a[1], b, *c1);
    piece_mfma<1>(a[0], b, *c0); piece_mfma<1>(a[1], b, *c1);
    piece_mfma<2>(a[0], b, *c0); piece_mfma<2>(a[1], b, *c1);
    piece_mfma<3>(a[0], b, *c0); piece_mfma<3>(a[1], b, *c1);
    piece_mfma<4>(a[0], b, *c0); piece_mfma<4>(a[1], b, *c1);
    piece_mfma<5>(a[0], b, *c0); piece_mfma<5>(a[1], b, *c1);
  }

  // blocks q0, q0 + 1 (if present) of wavefront W's upper-triangular schedule of a diagonal tile
  template <int W, int Q0>
  __device__ static __forceinline__ void diag_pair(const uint4* smem, int base, Shape::Acc& acc) {
    constexpr int TJ = 4;
    constexpr bool two = (Q0 + 1 < Shape::kDiagN[W]);
    constexpr int Q1 = two ? Q0 + 1 : Q0;
    const Frag a0 = read_frag(smem, base + 32 * Shape::kDiagRow[W][Q0]);
    const Frag b0 = read_frag(smem, base + 32 * Shape::kDiagCol[W][Q0]);
    Frag a1 = a0, b1 = b0;
    if constexpr (two) {
      a1 = read_frag(smem, base + 32 * Shape::kDiagRow[W][Q1]);
      b1 = read_frag(smem, base + 32 * Shape::kDiagCol[W][Q1]);
    }
    f32x16& c0 = acc.c[Q0 / TJ][Q0 % TJ];
    f32x16& c1 = acc.c[Q1 / TJ][Q1 % TJ];
    piece_mfma<0>(a0, b0, c0); if constexpr (two) piece_mfma<0>(a1, b1, c1);
    piece_mfma<1>(a0, b0, c0); if constexpr (two) piece_mfma<1>(a1, b1, c1);
    piece_mfma<2>(a0, b0, c0); if constexpr (two) piece_mfma<2>(a1, b1, c1);
    piece_mfma<3>(a0, b0, c0); if constexpr (two) piece_mfma<3>(a1, b1, c1);
    piece_mfma<4>(a0, b0, c0); if constexpr (two) piece_mfma<4>(a1, b1, c1);
    piece_mfma<5>(a0, b0, c0); if constexpr (two) piece_mfma<5>(a1, b1, c1);
  }
  template <int W>
  __device__ static __forceinline__ void diag_stage(const uint4* smem, int base, Shape::Acc& acc) {
    diag_pair<W, 0>(smem, base, acc);
    if constexpr (Shape::kDiagN[W] > 2) diag_pair<W, 2>(smem, base, acc);
    if constexpr (Shape::kDiagN[W] > 4) diag_pair<W, 4>(smem, base, acc);
  }

  // acc += X[k_begin:k_end, m0:m0+256]^T X[k_begin:k_end, n0:n0+256]; channels >= d read as zero.
  // DIAG: m0 == n0 and only the 32 x 32 blocks on or above the diagonal are accumulated (read
  // with Shape::for_each_diag), else all of them (Shape::for_each).  All threads of the
  // work-group call this with identical arguments; uses the kernel's dynamic LDS (kLdsBytes).
  template <bool DIAG>
  __device__ static __forceinline__ void run(const float* __restrict__ X, long ldx, int m0, int n0,
                                             int d, int k_begin, int k_end, Shape::Acc& acc) {
    extern __shared__ uint4 smem_v[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave / 2, wn = wave % 2;
    const int n_stage = (k_end - k_begin + kStageK - 1) / kStageK;
    if (n_stage <= 0) return;

    // staging role: threads 0..255 operand A, 256..511 operand B (idle on a diagonal tile)
    const int opnd = threadIdx.x >> 8;
    const int chl = threadIdx.x & 255;
    const int ch_raw = (opnd ? n0 : m0) + chl;
    const bool loader = !(DIAG && opnd);
    const int ch = min(ch_raw, d - 1);
    const int dst0 = opnd * kVecOperand + chl;

    // two staging register sets: the set drained in stage s (tokens of stage s + 1) is refilled
    // with stage s + 3, so a load has two stages of MFMAs to land
    float g[kStageK], g2[kStageK];
#pragma unroll
    for (int i = 0; i < kStageK; ++i) g[i] = g2[i] = 0.f;
    const int k_last_stage = k_begin + (n_stage - 1) * kStageK;
    if (loader) {
      load_tokens(X, ldx, k_begin, k_end, ch, false, g);
      store_group<0>(smem_v, dst0, g, k_end - k_begin);
      store_group<1>(smem_v, dst0, g, k_end - k_begin);
      load_tokens(X, ldx, min(k_begin + kStageK, k_last_stage), k_end, ch, false, g);
      load_tokens(X, ldx, min(k_begin + 2 * kStageK, k_last_stage), k_end, ch, false, g2);
    }
    __syncthreads();

    const int a_idx = (lane >> 5) * kTile + wm * 64 + (lane & 31);
    const int b_idx = kVecOperand + (lane >> 5) * kTile + wn * 128 + (lane & 31);
    const int d_idx = (lane >> 5) * kTile + (lane & 31);
    // The staging runs in every stage, without branches, so that it can be interleaved with the
    // MFMAs: in the last stage it rewrites the buffer nobody reads any more, and the loads of the
    // last stages fetch the last stage again.
    if constexpr (DIAG) {
      auto stage = [&](int s, float (&gs)[kStageK]) {
        const int cur = (s & 1) * kVecBuf;
        const int nxt = kVecBuf - cur;
        const int k3 = min(k_begin + (s + 3) * kStageK, k_last_stage);
        const bool fast = k3 + kStageK <= k_end;
        const int n_valid = k_end - (k_begin + (s + 1) * kStageK);   // of the tokens being drained
        store_group<0>(smem_v, nxt + dst0, gs, n_valid);
        store_group<1>(smem_v, nxt + dst0, gs, n_valid);
        if (loader) load_tokens(X, ldx, k3, k_end, ch, fast, gs);
        switch (wave) {
          case 0: diag_stage<0>(smem_v, cur + d_idx, acc); break;
          case 1: diag_stage<1>(smem_v, cur + d_idx, acc); break;
          case 2: diag_stage<2>(smem_v, cur + d_idx, acc); break;
          case 3: diag_stage<3>(smem_v, cur + d_idx, acc); break;
          case 4: diag_stage<4>(smem_v, cur + d_idx, acc); break;
          case 5: diag_stage<5>(smem_v, cur + d_idx, acc); break;
          case 6: diag_stage<6>(smem_v, cur + d_idx, acc); break;
          default: diag_stage<7>(smem_v, cur + d_idx, acc); break;
        }
        __syncthreads();
      };
      for (int s = 0; s < n_stage; s += 2) {
        stage(s, g);
        if (s + 1 < n_stage) stage(s + 1, g2);
      }
    } else {
      // One barrier per stage, in its middle.  Before it a wavefront writes the next stage's
      // pieces and issues its last reads of the current buffer; after it the next stage is
      // complete in LDS, so its first operands are fetched under the second half of this
      // stage's MFMAs and no stage starts with the matrix pipe waiting for LDS.  A buffer is
      // rewritten only in the stage after the next, i.e. behind the barrier that follows the
      // last read of it.
      Frag a[2], b[4];
      a[0] = read_frag(smem_v, a_idx);
      a[1] = read_frag(smem_v, a_idx + 32);
      b[0] = read_frag(smem_v, b_idx);
      b[1] = read_frag(smem_v, b_idx + 32);
      auto stage = [&](int s, float (&gs)[kStageK]) {
        const int cur = (s & 1) * kVecBuf;
        const int nxt = kVecBuf - cur;
        const int k3 = min(k_begin + (s + 3) * kStageK, k_last_stage);
        const bool fast = k3 + kStageK <= k_end;
        const int n_valid = k_end - (k_begin + (s + 1) * kStageK);   // of the tokens being drained
        b[2] = read_frag(smem_v, cur + b_idx + 64);
        b[3] = read_frag(smem_v, cur + b_idx + 96);
        product<2>(a, b[0], &acc.c[0][0], &acc.c[1][0]);
        store_group<0>(smem_v, nxt + dst0, gs, n_valid);
        product<2>(a, b[1], &acc.c[0][1], &acc.c[1][1]);
        store_group<1>(smem_v, nxt + dst0, gs, n_valid);
        load_tokens(X, ldx, k3, k_end, ch, fast, gs);
        __syncthreads();
        b[0] = read_frag(smem_v, nxt + b_idx);
        b[1] = read_frag(smem_v, nxt + b_idx + 32);
        product<2>(a, b[2], &acc.c[0][2], &acc.c[1][2]);
        Frag an[2];
        an[0] = read_frag(smem_v, nxt + a_idx);
        an[1] = read_frag(smem_v, nxt + a_idx + 32);
        product<2>(a, b[3], &acc.c[0][3], &acc.c[1][3]);
        a[0] = an[0];
        a[1] = an[1];
      };
      for (int s = 0; s < n_stage; s += 2) {
        stage(s, g);
        if (s + 1 < n_stage) stage(s + 1, g2);
      }
    }
  }
};

}  // namespace bpdq
