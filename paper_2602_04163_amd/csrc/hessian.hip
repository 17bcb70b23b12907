// Step 1 of the pass: calibration Hessian H += scale * Xc^T Xc (paper Sec. 3.1, H = X X^T).
//
// A symmetric rank-k update on the matrix cores, in three kernels that share everything but the
// tile product: fp32 MFMAs (bpdq_hessian_accumulate_f32), bf16 MFMAs on three exact bf16 pieces
// of every value (bpdq_hessian_accumulate_bf16x3; mfma_split_bf16.h), or fp16 MFMAs on two fp16
// halves of every value, split and laid out in operand order by a streaming pre-pass
// (bpdq_hessian_accumulate; mfma_split_f16.h).  Only the upper triangle
// of 256 x 256 tiles is computed, and of a diagonal tile only the 32 x 32 blocks on or above the diagonal.
// The token axis is cut into deterministic slices so that the work-groups fill the 256 compute
// units in whole rounds: off-diagonal tiles into S_off slices, diagonal tiles (5/8 of the work
// per token) into fewer, longer slices S_diag, so that every work-group costs about the same.
// Slice partials go to the workspace and are summed in a fixed order (no float atomics, so H is
// bit-reproducible).
#include "mfma_kmajor.h"
#include "mfma_split_bf16.h"
#include "mfma_split_f16.h"

namespace bpdq {

constexpr int kNumCU = 256;   // MI355X: 8 XCDs x 32 compute units
constexpr int kNumXCD = 8;
constexpr int kTileFloats = HessGemm::kTileM * HessGemm::kTileN;

struct HessPlan {
  int nb;               // tile rows / cols
  int n_off, n_diag;    // off-diagonal and diagonal tiles of the upper triangle
  int S_off, S_diag;    // token slices per off-diagonal / diagonal tile
  int k_off, k_diag;    // tokens per slice (multiples of the stage depth)
  bool direct;          // one slice each: accumulate into H without partials
  int items() const { return n_off * S_off + n_diag * S_diag; }
  size_t ws_bytes() const { return direct ? 0 : (size_t)items() * kTileFloats * sizeof(float); }
};

// Makespan (us) of the busiest XCD: work-groups go round-robin to the XCDs and, inside one, to
// the first free of its 32 compute units; all off-diagonal slices are dispatched first.
static double hess_makespan(int n_full, double c_full, int n_short, double c_short) {
  const int per = kNumCU / kNumXCD;
  const int nf = bpdq_ceil_div(n_full, kNumXCD), ns = bpdq_ceil_div(n_short, kNumXCD);
  double free_at[kNumCU / kNumXCD];
  const int q = nf / per, r = nf % per;
  for (int i = 0; i < per; ++i) free_at[i] = (q + (i < r ? 1 : 0)) * c_full;
  for (int j = 0; j < ns; ++j) {
    int m = 0;
    for (int i = 1; i < per; ++i)
      if (free_at[i] < free_at[m]) m = i;
    free_at[m] += c_short;
  }
  double t = 0.0;
  for (int i = 0; i < per; ++i) t = free_at[i] > t ? free_at[i] : t;
  return t;
}

// Measured: a sum of squares (the diagonal of H) accumulated by chained MFMAs comes out low, the
// more so the longer the chain, as if the products of an instruction were truncated when aligned
// to the running sum: about -1.3e-6 relative after 11 k tokens on the fp32 path, -4.5e-6 after
// 52 k tokens and -2.5e-6 after 8 k tokens on the split path.  Both paths therefore end every
// chain after kChainTokens[kind] tokens; the partial sums are added by ordinary round-to-nearest
// fp32 additions, which do not drift.
constexpr int kChainTokens[3] = {16384, 8192, 8192};
constexpr int kMaxSlices = 64;

// kind 0: fp32 MFMA kernel; kind 1: split-bf16 kernel (about 1.8 times the rate per token);
// kind 2: pre-split fp16 kernel (about twice the rate of kind 1)
enum : int { kKindF32 = 0, kKindBf16x3 = 1, kKindF16x2 = 2, kNumKinds = 3 };

static HessPlan plan_hessian(int n_tok, int d_in, int kind) {
  // the last plan of each kind, per host thread (the search below costs a fraction of a millisecond,
  // which a stream of short calls would otherwise pay every time)
  thread_local HessPlan cache[kNumKinds];
  thread_local int cache_n[kNumKinds] = {-1, -1, -1}, cache_d[kNumKinds] = {-1, -1, -1};
  if (n_tok == cache_n[kind] && d_in == cache_d[kind]) return cache[kind];
  HessPlan p;
  p.nb = bpdq_ceil_div(d_in, HessGemm::kTileM);
  p.n_diag = p.nb;
  p.n_off = p.nb * (p.nb - 1) / 2;
  p.S_off = p.S_diag = 1;
  p.k_off = p.k_diag = (int)bpdq_align_up((size_t)(n_tok > 0 ? n_tok : 1), HessGemm::kStageK);
  p.direct = true;
  if (n_tok > 0 && p.n_off + p.n_diag < 4 * kNumCU) {
    // per-token MFMA time of one 256 x 256 tile, fixed cost per work-group, cost per partial tile
    constexpr double kUsPerTok[kNumKinds] = {0.26, 0.14, 0.055};
    constexpr double kDiagFrac[kNumKinds] = {0.64, 0.64, 0.60};
    const double us_per_tok = kUsPerTok[kind], us_fixed = 8.0, us_per_partial = 0.131;
    const double diag_frac = kDiagFrac[kind];
    const int s_max = n_tok / 256 < kMaxSlices ? (n_tok / 256 < 1 ? 1 : n_tok / 256) : kMaxSlices;
    // every accumulation chain stays short (see kChainTokens)
    int s_min = bpdq_ceil_div(n_tok, kChainTokens[kind]);
    if (s_min > s_max) s_min = s_max;
    double best = 1e300;
    for (int So = s_min; So <= s_max; ++So) {
      for (int dd = -1; dd <= 1; ++dd) {
        int Sd = (int)(So * 0.625 + 0.5) + dd;
        if (Sd < s_min) Sd = s_min;
        if (Sd > s_max) Sd = s_max;
        const int ko = (int)bpdq_align_up((size_t)bpdq_ceil_div(n_tok, So), HessGemm::kStageK);
        const int kd = (int)bpdq_align_up((size_t)bpdq_ceil_div(n_tok, Sd), HessGemm::kStageK);
        double t = hess_makespan(p.n_off * So, ko * us_per_tok + us_fixed, p.n_diag * Sd,
                                 kd * us_per_tok * diag_frac + us_fixed);
        if (So > 1 || Sd > 1) t += (double)(p.n_off * So + p.n_diag * Sd) * us_per_partial;
        if (t < best * 0.998) {
          best = t;
          p.S_off = So; p.S_diag = Sd; p.k_off = ko; p.k_diag = kd;
        }
      }
    }
    p.direct = (p.S_off == 1 && p.S_diag == 1);
  }
  cache[kind] = p; cache_n[kind] = n_tok; cache_d[kind] = d_in;
  return p;
}

// Tile orders.  The 32 tiles an XCD has in flight stream their 256-channel panels through its L2,
// so an order is as good as the number of different panels a run of 32 consecutive tiles meets.
// The triangle is cut into blocks of kTileBlock panels: the blocks on the diagonal are cliques
// (every pair of kTileBlock panels: 28 tiles on 8 panels), the others kTileBlock x kTileBlock
// squares (64 tiles on 16 panels); blocks are taken column by column, tiles row-major inside.
// On 74 x 74 tiles a run of 32 meets 13 panels on average, in plain row-major order 32.  Measured
// against row-major in one process: 6.5 % less time at 116 x 116 tiles, 2-3 % at 74 and 32, none at 14.
constexpr int kTileBlock = 8;

// seq-th tile of that order -> (bi, bj).  DIAG: the diagonal tiles are part of the sequence
// (bi <= bj), else only bi < bj.  seq must be below the number of such tiles.
template <bool DIAG>
__device__ __forceinline__ void block_order_tile(int seq, int nb, int& bi, int& bj) {
  const int n_blk = bpdq_ceil_div(nb, kTileBlock);
  bi = bj = 0;
  for (int bc = 0; bc < n_blk; ++bc) {
    const int c0 = bc * kTileBlock, mc = (c0 + kTileBlock < nb ? kTileBlock : nb - c0);
    // the column of blocks above the diagonal one: bc full squares of kTileBlock x mc tiles
    const int above = bc * kTileBlock * mc;
    if (seq < above) {
      const int br = seq / (kTileBlock * mc), t = seq % (kTileBlock * mc);
      bi = br * kTileBlock + t / mc;
      bj = c0 + t % mc;
      return;
    }
    seq -= above;
    const int clique = DIAG ? mc * (mc + 1) / 2 : mc * (mc - 1) / 2;
    if (seq < clique) {
      for (int r = 0; r < mc; ++r) {
        const int cnt = DIAG ? mc - r : mc - 1 - r;
        if (seq < cnt) {
          bi = c0 + r;
          bj = c0 + r + (DIAG ? 0 : 1) + seq;
          return;
        }
        seq -= cnt;
      }
    }
    seq -= clique;
  }
}

// off-diagonal tile index -> (bi, bj), bi < bj
__device__ __forceinline__ void decode_off_tile(int tile, int nb, int& bi, int& bj) {
  block_order_tile<false>(tile, nb, bi, bj);
}

// Work-group -> work item.  Work-groups are handed to the 8 XCDs round-robin (work-group w runs
// on XCD w % 8), each XCD has its own L2, and items are numbered slice-major (item = slice *
// tiles + tile).  Taken in that order every XCD would work on all token slices at once and each
// L2 would stream the whole of X: 8 x the traffic.  Instead XCD x takes the slices congruent to
// x modulo 8, tile after tile: the work-groups running on an XCD at one time walk the same
// tokens in step, its L2 serves every 256-channel block of a stage to all of them from one
// fetch, and each token is fetched by one XCD only.  Slices beyond the last multiple of 8 keep
// the plain order.  The map is a bijection on the items, so partials and reduction are unchanged.
__device__ __forceinline__ int xcd_item(int w, int n_off_items, const HessPlan& p) {
  int base = 0, tiles = p.n_off, slices = p.S_off;
  if (w >= n_off_items) {
    base = n_off_items;
    tiles = p.n_diag;
    slices = p.S_diag;
  }
  const int j = w - base;
  const int grouped = tiles * (slices / kNumXCD) * kNumXCD;   // items of the slices that are remapped
  if (j >= grouped) return w;
  // j % 8 names the XCD up to a fixed rotation (base need not be a multiple of 8)
  const int y = j % kNumXCD, q = j / kNumXCD;
  return base + ((q / tiles) * kNumXCD + y) * tiles + q % tiles;
}

// Tile order of a launch without token slices (wide layers: more tiles than the chip runs at
// once): the block order above over the whole upper triangle, diagonal tiles included, and XCD x
// takes the runs of 32 numbered x, x + 8, ... of that sequence (work-group w runs on XCD w % 8).
// Work-group w -> tile; false beyond the last tile.
__host__ __device__ inline int direct_grid(int nb) {
  const int tiles = nb * (nb + 1) / 2;
  return bpdq_ceil_div(tiles, kNumCU) * kNumCU;
}
__device__ __forceinline__ bool direct_tile(int w, int nb, int& bi, int& bj) {
  const int per = kNumCU / kNumXCD;                       // 32
  const int x = w % kNumXCD, n = w / kNumXCD;
  const int seq = ((n / per) * kNumXCD + x) * per + n % per;
  if (seq >= nb * (nb + 1) / 2) return false;
  block_order_tile<true>(seq, nb, bi, bj);
  return true;
}

// SPLIT false: fp32 matrix cores (v_mfma_f32_32x32x2_f32); true: three bf16 pieces per value and
// six bf16 products per fp32 product (v_mfma_f32_32x32x16_bf16), same accumulator layout.
template <bool SPLIT>
__device__ __forceinline__ void hess_syrk_body(const float* __restrict__ X, int n_tok, int d,
                                               long ldx, float scale, float* __restrict__ H,
                                               float* __restrict__ partial, const HessPlan& p) {
  const int n_off_items = p.n_off * p.S_off;
  const int item = xcd_item(blockIdx.x, n_off_items, p);
  int bi, bj, k_begin, k_end;
  if (item < n_off_items) {
    decode_off_tile(item % p.n_off, p.nb, bi, bj);
    k_begin = (item / p.n_off) * p.k_off;
    k_end = min(n_tok, k_begin + p.k_off);
  } else {
    const int j = item - n_off_items;
    bi = bj = j % p.n_diag;
    k_begin = (j / p.n_diag) * p.k_diag;
    k_end = min(n_tok, k_begin + p.k_diag);
  }
  HessGemm::Acc acc;
  HessGemm::zero(acc);
  const int r0 = bi * HessGemm::kTileM, c0 = bj * HessGemm::kTileN;
  // diagonal tile: only the 32 x 32 blocks on or above the diagonal are computed
  if (bi == bj) {
    if constexpr (SPLIT) SplitSyrk::run<true>(X, ldx, r0, c0, d, k_begin, k_end, acc);
    else HessGemm::run<2>(X, ldx, r0, d, X, ldx, c0, d, k_begin, k_end, acc);
  } else {
    if constexpr (SPLIT) SplitSyrk::run<false>(X, ldx, r0, c0, d, k_begin, k_end, acc);
    else HessGemm::run<0>(X, ldx, r0, d, X, ldx, c0, d, k_begin, k_end, acc);
  }
  if (p.direct) {
    auto emit = [&](int row, int col, float v) {
      const int r = r0 + row, c = c0 + col;
      if (r < d && c < d) H[(long)r * d + c] += scale * v;
    };
    if (bi == bj) HessGemm::for_each_diag(acc, emit);
    else HessGemm::for_each(acc, emit);
  } else {
    float* out = partial + (long)item * kTileFloats;
    auto emit = [&](int row, int col, float v) { out[row * HessGemm::kTileN + col] = v; };
    if (bi == bj) HessGemm::for_each_diag(acc, emit);
    else HessGemm::for_each(acc, emit);
  }
}

__global__ __launch_bounds__(HessGemm::kThreads) void hess_syrk_f32_kernel(
    const float* __restrict__ X, int n_tok, int d, long ldx, float scale, float* __restrict__ H,
    float* __restrict__ partial, HessPlan p) {
  hess_syrk_body<false>(X, n_tok, d, ldx, scale, H, partial, p);
}

__global__ __launch_bounds__(SplitSyrk::kThreads) void hess_syrk_bf16x3_kernel(
    const float* __restrict__ X, int n_tok, int d, long ldx, float scale, float* __restrict__ H,
    float* __restrict__ partial, HessPlan p) {
  hess_syrk_body<true>(X, n_tok, d, ldx, scale, H, partial, p);
}

// ---- pre-pass of the fp16 path ---------------------------------------------------------------
// (1) per-channel largest magnitude of the call's tokens, as partial maxima over token ranges;
// (2) per channel the power of two that brings that maximum into [2^13, 2^14) (so every half is
//     far from the ends of the fp16 range whatever the activations' units), and its inverse;
// (3) the split itself: X -> planes[piece][token / 8][channel] (see mfma_split_f16.h), zeros for
//     the tokens up to the next multiple of 32 and the channels up to the next multiple of 256.
constexpr int kColmaxRows = 1024;      // tokens per partial maximum
constexpr int kSplitKgPerWG = 16;      // k-groups (8 tokens each) per work-group of the split

__global__ __launch_bounds__(256) void hess_colmax_kernel(const float* __restrict__ X, int n_tok, int d,
                                                          long ldx, float* __restrict__ pmax, int d_pad) {
  __shared__ float4 red[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 256 + lane * 4;
  const int t0 = blockIdx.y * kColmaxRows;
  const int t1 = min(n_tok, t0 + kColmaxRows);
  float4 m = make_float4(0.f, 0.f, 0.f, 0.f);
  if (c < d) {                                    // d % 4 == 0: the float4 is inside the row
    const float* p = X + c;
    for (int t = t0 + wave; t < t1; t += 32) {    // 8 rows of this wavefront in flight
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int tt = min(t + 4 * u, t1 - 1);    // past the end: the last row again
        v[u] = *reinterpret_cast<const float4*>(p + (long)tt * ldx);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        m.x = fmaxf(m.x, fabsf(v[u].x)); m.y = fmaxf(m.y, fabsf(v[u].y));
        m.z = fmaxf(m.z, fabsf(v[u].z)); m.w = fmaxf(m.w, fabsf(v[u].w));
      }
    }
  }
  red[wave][lane] = m;
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const float4 o = red[w][lane];
      m.x = fmaxf(m.x, o.x); m.y = fmaxf(m.y, o.y); m.z = fmaxf(m.z, o.z); m.w = fmaxf(m.w, o.w);
    }
    *reinterpret_cast<float4*>(pmax + (long)blockIdx.y * d_pad + c) = m;     // c < d_pad always
  }
}

__global__ __launch_bounds__(256) void hess_scale_kernel(const float* __restrict__ pmax, int n_split,
                                                         int d_pad, float* __restrict__ mul,
                                                         float* __restrict__ inv) {
  // 64 channels per work-group, the partial maxima of a channel dealt to four threads
  __shared__ float red[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), q = threadIdx.x >> 6;
  float m = 0.f;
  for (int s = q; s < n_split; s += 4) m = fmaxf(m, pmax[(long)s * d_pad + c]);
  red[q][threadIdx.x & 63] = m;
  __syncthreads();
  if (q) return;
  m = fmaxf(fmaxf(red[0][threadIdx.x], red[1][threadIdx.x]), fmaxf(red[2][threadIdx.x], red[3][threadIdx.x]));
  int e = 0;
  if (m > 0.f && m < 3.0e38f) {
    int ex;
    (void)frexpf(m, &ex);           // m = f * 2^ex, f in [0.5, 1)
    e = 14 - ex;                    // m * 2^e in [2^13, 2^14)
    e = e > 100 ? 100 : (e < -100 ? -100 : e);
  }
  mul[c] = ldexpf(1.0f, e);
  inv[c] = ldexpf(1.0f, -e);
}

__device__ __forceinline__ unsigned pack_halves(_Float16 a, _Float16 b) {
  return (unsigned)__builtin_bit_cast(unsigned short, a) | ((unsigned)__builtin_bit_cast(unsigned short, b) << 16);
}

__global__ __launch_bounds__(256) void hess_split_f16_kernel(const float* __restrict__ X, int n_tok, int d,
                                                             long ldx, const float* __restrict__ mul,
                                                             uint4* __restrict__ planes, long n_kg,
                                                             int d_pad) {
  const int ch = blockIdx.x * 256 + threadIdx.x;
  const bool live = ch < d;
  const int chc = live ? ch : d - 1;
  const float s = mul[chc];
  const float* p = X + chc;
  const long kg0 = (long)blockIdx.y * kSplitKgPerWG;
  const int t_last = n_tok - 1;
  for (int g = 0; g < kSplitKgPerWG; g += 2) {
    const long kg = kg0 + g;
    if (kg >= n_kg) break;
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const long t = 8 * kg + i;
      x[i] = p[(t < t_last ? t : (long)t_last) * ldx];
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      if (kg + half >= n_kg) break;
      unsigned hw[4], lw[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        _Float16 h[2], l[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int i = 8 * half + 2 * q + e;
          const bool in = live && (8 * kg + i) < n_tok;
          const float xs = in ? x[i] * s : 0.f;
          h[e] = (_Float16)xs;                       // round to nearest even
          l[e] = (_Float16)(xs - (float)h[e]);       // exact difference, then rounded
        }
        hw[q] = pack_halves(h[0], h[1]);
        lw[q] = pack_halves(l[0], l[1]);
      }
      planes[(kg + half) * d_pad + ch] = make_uint4(hw[0], hw[1], hw[2], hw[3]);
      planes[(n_kg + kg + half) * d_pad + ch] = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    }
  }
}

// The tile product of the fp16 path and its epilogue: every result is brought back to the
// activations' own units by the two channel factors (powers of two: exact).
__global__ __launch_bounds__(SplitF16::kThreads, 1) void hess_syrk_f16x2_kernel(
    const uint4* __restrict__ planes, long n_kg, int d_pad, const float* __restrict__ inv, int n_tok,
    int d, float scale, float* __restrict__ H, float* __restrict__ partial, HessPlan p) {
  const int n_off_items = p.n_off * p.S_off;
  int item = 0, bi, bj, k_begin, k_end;
  if (p.direct) {
    if (!direct_tile(blockIdx.x, p.nb, bi, bj)) return;
    k_begin = 0;
    k_end = n_tok;
  } else {
    item = xcd_item(blockIdx.x, n_off_items, p);
    if (item < n_off_items) {
      decode_off_tile(item % p.n_off, p.nb, bi, bj);
      k_begin = (item / p.n_off) * p.k_off;
      k_end = min(n_tok, k_begin + p.k_off);
    } else {
      const int j = item - n_off_items;
      bi = bj = j % p.n_diag;
      k_begin = (j / p.n_diag) * p.k_diag;
      k_end = min(n_tok, k_begin + p.k_diag);
    }
  }
  // two stages of 16 tokens per loop iteration; the planes are zero beyond n_tok
  const int n_stage = k_end > k_begin ? 2 * ((k_end - k_begin + 2 * SplitF16::kStageK - 1) / (2 * SplitF16::kStageK)) : 0;
  SplitF16::Acc acc;
  SplitF16::zero(acc);
  const int r0 = bi * SplitF16::kTile, c0 = bj * SplitF16::kTile;
  if (bi == bj) SplitF16::run<true>(planes, n_kg, d_pad, r0, c0, k_begin / 8, n_stage, acc);
  else SplitF16::run<false>(planes, n_kg, d_pad, r0, c0, k_begin / 8, n_stage, acc);
  // the LDS ring is free now: the channel factors of this tile's rows and columns
  extern __shared__ uint4 smem_f16[];
  float* sInv = reinterpret_cast<float*>(smem_f16);
  sInv[threadIdx.x] = inv[r0 + threadIdx.x];
  sInv[256 + threadIdx.x] = inv[c0 + threadIdx.x];
  __syncthreads();
  if (p.direct) {
    auto emit = [&](int row, int col, float v) {
      const int r = r0 + row, c = c0 + col;
      if (r < d && c < d) H[(long)r * d + c] += scale * (v * sInv[row] * sInv[256 + col]);
    };
    if (bi == bj) SplitF16::for_each_diag(acc, emit);
    else SplitF16::for_each(acc, emit);
  } else {
    float* out = partial + (long)item * kTileFloats;
    auto emit = [&](int row, int col, float v) {
      out[row * SplitF16::kTile + col] = v * sInv[row] * sInv[256 + col];
    };
    if (bi == bj) SplitF16::for_each_diag(acc, emit);
    else SplitF16::for_each(acc, emit);
  }
}

// H[tile] += scale * sum_s partial[s][tile], slices added in index order.  64 work-groups per
// tile; tiles 0 .. n_off-1 are off-diagonal, the rest diagonal.
__global__ __launch_bounds__(256) void hess_reduce_kernel(const float* __restrict__ partial,
                                                          HessPlan p, int d, float scale,
                                                          float* __restrict__ H) {
  const int tile = blockIdx.x >> 6;
  const int e = ((blockIdx.x & 63) * 256 + threadIdx.x) * 4;
  int bi, bj, S;
  long first, stride;
  if (tile < p.n_off) {
    decode_off_tile(tile, p.nb, bi, bj);
    S = p.S_off;
    first = tile;
    stride = p.n_off;
  } else {
    bi = bj = tile - p.n_off;
    S = p.S_diag;
    first = (long)p.n_off * p.S_off + bi;
    stride = p.n_diag;
    // blocks of 32 x 32 below the diagonal of a diagonal tile are never computed
    if ((e % HessGemm::kTileN) / 32 < (e / HessGemm::kTileN) / 32) return;
  }
  const int r = bi * HessGemm::kTileM + e / HessGemm::kTileN;
  const int c = bj * HessGemm::kTileN + e % HessGemm::kTileN;
  if (r >= d || c >= d) return;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int sp = 0; sp < S; ++sp) {
    const float4 v = *reinterpret_cast<const float4*>(partial + (first + sp * stride) * kTileFloats + e);
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

// Tokens of the next launch: the chain length is bounded (kChainTokens).  A launch that adds
// straight into H (no slices) takes one chain's worth of tokens, a sliced one as many as its
// slices can cover; successive launches on one stream accumulate in order.
static int hessian_launch_tokens(int kind, int n_left, int d_in) {
  const int chain = kChainTokens[kind];
  const long cover = (long)chain * kMaxSlices;
  int n = n_left > cover ? (int)cover : n_left;
  if (n > chain && plan_hessian(n, d_in, kind).direct) n = chain;
  return n;
}

// Workspace of one launch of n_part tokens: split-K partial tiles, then (fp16 path) the split
// planes, the partial channel maxima and the two channel factors.
struct HessWs {
  size_t partial_off, planes_off, pmax_off, mul_off, inv_off, total;
  long n_kg;
  int d_pad, n_split;
};

static HessWs hessian_ws_layout(int kind, int n_part, int d_in) {
  HessWs L{};
  size_t off = 0;
  L.partial_off = off;
  off += bpdq_align_up(plan_hessian(n_part, d_in, kind).ws_bytes(), 256);
  if (kind == kKindF16x2) {
    L.d_pad = (int)bpdq_align_up((size_t)d_in, SplitF16::kTile);
    L.n_kg = (long)bpdq_align_up((size_t)n_part, 2 * SplitF16::kStageK) / 8;
    L.n_split = bpdq_ceil_div(n_part, kColmaxRows);
    L.planes_off = off; off += bpdq_align_up((size_t)2 * L.n_kg * L.d_pad * sizeof(uint4), 256);
    L.pmax_off = off;   off += bpdq_align_up((size_t)L.n_split * L.d_pad * sizeof(float), 256);
    L.mul_off = off;    off += bpdq_align_up((size_t)L.d_pad * sizeof(float), 256);
    L.inv_off = off;    off += bpdq_align_up((size_t)L.d_pad * sizeof(float), 256);
  }
  L.total = off;
  return L;
}

// the first launch of a call is its largest
static size_t hessian_ws_bytes(int kind, int n_tok, int d_in) {
  return hessian_ws_layout(kind, hessian_launch_tokens(kind, n_tok, d_in), d_in).total;
}

static int hessian_accumulate(int kind, const float* Xc, int n_tok, int d_in, int ldx, float scale,
                              float* H, int symmetrize, void* ws, size_t ws_bytes, void* stream_,
                              void* ev_begin = nullptr, void* ev_end = nullptr) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (kind < 0 || kind >= kNumKinds) return -11;
  if (n_tok < 0) return -2;
  if (d_in <= 0 || d_in % 4) return -3;
  if (ldx < d_in || ldx % 4) return -4;
  if (n_tok > 0 && (!Xc || (reinterpret_cast<uintptr_t>(Xc) & 15))) return -1;
  if (!H || (reinterpret_cast<uintptr_t>(H) & 15)) return -6;
  const size_t need = n_tok > 0 ? hessian_ws_bytes(kind, n_tok, d_in) : 0;
  if (need > 0 && (!ws || (reinterpret_cast<uintptr_t>(ws) & 255))) return -8;
  if (ws_bytes < need) return -9;
  char* base = static_cast<char*>(ws);
  for (int done = 0; done < n_tok;) {
    const int n_part = hessian_launch_tokens(kind, n_tok - done, d_in);
    const HessPlan p = plan_hessian(n_part, d_in, kind);
    const HessWs L = hessian_ws_layout(kind, n_part, d_in);
    float* partial = reinterpret_cast<float*>(base + L.partial_off);
    const float* Xpart = Xc + (long)done * ldx;
    const bool first = (done == 0);
    done += n_part;
    // (the pre-pass of the fp16 path precedes the first event; later launches' pre-passes fall
    // between the two events)
    auto mark_begin = [&]() -> int {
      if (first && ev_begin) BPDQ_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(ev_begin), stream));
      return 0;
    };
    if (kind == kKindF32) {
      if (mark_begin()) return BPDQ_ERR_LAUNCH;
      BPDQ_HIP_TRY(bpdq_lds_limit<&hess_syrk_f32_kernel>(HessGemm::kLdsBytes));
      hipLaunchKernelGGL(hess_syrk_f32_kernel, dim3(p.items()), dim3(HessGemm::kThreads),
                         HessGemm::kLdsBytes, stream, Xpart, n_part, d_in, (long)ldx, scale, H,
                         partial, p);
    } else if (kind == kKindBf16x3) {
      if (mark_begin()) return BPDQ_ERR_LAUNCH;
      BPDQ_HIP_TRY(bpdq_lds_limit<&hess_syrk_bf16x3_kernel>(SplitSyrk::kLdsBytes));
      hipLaunchKernelGGL(hess_syrk_bf16x3_kernel, dim3(p.items()), dim3(SplitSyrk::kThreads),
                         SplitSyrk::kLdsBytes, stream, Xpart, n_part, d_in, (long)ldx, scale, H,
                         partial, p);
    } else {
      BPDQ_HIP_TRY(bpdq_lds_limit<&hess_syrk_f16x2_kernel>(SplitF16::kLdsBytes));
      uint4* planes = reinterpret_cast<uint4*>(base + L.planes_off);
      float* pmax = reinterpret_cast<float*>(base + L.pmax_off);
      float* mul = reinterpret_cast<float*>(base + L.mul_off);
      float* inv = reinterpret_cast<float*>(base + L.inv_off);
      const int cb = L.d_pad / SplitF16::kTile;
      hipLaunchKernelGGL(hess_colmax_kernel, dim3(cb, L.n_split), dim3(256), 0, stream, Xpart, n_part,
                         d_in, (long)ldx, pmax, L.d_pad);
      BPDQ_LAUNCH_CHECK();
      hipLaunchKernelGGL(hess_scale_kernel, dim3(L.d_pad / 64), dim3(256), 0, stream, pmax, L.n_split,
                         L.d_pad, mul, inv);
      BPDQ_LAUNCH_CHECK();
      hipLaunchKernelGGL(hess_split_f16_kernel, dim3(cb, (unsigned)bpdq_ceil_div((int)L.n_kg, kSplitKgPerWG)),
                         dim3(256), 0, stream, Xpart, n_part, d_in, (long)ldx, mul, planes, L.n_kg, L.d_pad);
      BPDQ_LAUNCH_CHECK();
      if (mark_begin()) return BPDQ_ERR_LAUNCH;
      hipLaunchKernelGGL(hess_syrk_f16x2_kernel, dim3(p.direct ? direct_grid(p.nb) : p.items()),
                         dim3(SplitF16::kThreads),
                         SplitF16::kLdsBytes, stream, planes, L.n_kg, L.d_pad, inv, n_part, d_in, scale,
                         H, partial, p);
    }
    BPDQ_LAUNCH_CHECK();
    if (done >= n_tok && ev_end) BPDQ_HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(ev_end), stream));
    if (!p.direct) {
      hipLaunchKernelGGL(hess_reduce_kernel, dim3((p.n_off + p.n_diag) * 64), dim3(256), 0, stream,
                         partial, p, d_in, scale, H);
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

extern "C" size_t bpdq_hessian_workspace_bytes(int n_tok, int d_in) {
  if (n_tok <= 0 || d_in <= 0) return 0;
  // one workspace serves any of the kernels
  size_t need = 0;
  for (int kind = 0; kind < kNumKinds; ++kind) {
    const size_t b = hessian_ws_bytes(kind, n_tok, d_in);
    need = b > need ? b : need;
  }
  return need;
}

extern "C" int bpdq_hessian_accumulate_f32(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                                           float* H, int symmetrize, void* ws, size_t ws_bytes,
                                           void* stream) {
  return hessian_accumulate(kKindF32, Xc, n_tok, d_in, ldx, scale, H, symmetrize, ws, ws_bytes, stream);
}

extern "C" int bpdq_hessian_accumulate_bf16x3(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                                              float* H, int symmetrize, void* ws, size_t ws_bytes,
                                              void* stream) {
  return hessian_accumulate(kKindBf16x3, Xc, n_tok, d_in, ldx, scale, H, symmetrize, ws, ws_bytes, stream);
}

extern "C" int bpdq_hessian_accumulate_timed(int kernel, const float* Xc, int n_tok, int d_in, int ldx,
                                             float scale, float* H, int symmetrize, void* ws,
                                             size_t ws_bytes, void* stream, void* ev_begin, void* ev_end) {
  const int kind = kernel == BPDQ_HESSIAN_F16X2 ? kKindF16x2
                   : kernel == BPDQ_HESSIAN_BF16X3 ? kKindBf16x3
                   : kernel == BPDQ_HESSIAN_F32 ? kKindF32 : -1;
  if (kind < 0) return -1;
  const int rc = hessian_accumulate(kind, Xc, n_tok, d_in, ldx, scale, H, symmetrize, ws, ws_bytes, stream,
                                    ev_begin, ev_end);
  return rc < 0 && rc > -11 ? rc - 1 : rc;      // the arguments are shifted by one
}

// the default entry: two fp16 halves per scaled value
extern "C" int bpdq_hessian_accumulate(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                                       float* H, int symmetrize, void* ws, size_t ws_bytes,
                                       void* stream) {
  return hessian_accumulate(kKindF16x2, Xc, n_tok, d_in, ldx, scale, H, symmetrize, ws, ws_bytes, stream);
}
