// Steps 3-4 of the pass: the group / column sweep of BPDQ with lazy block updates
// (paper Sec. 3.2, 3.3; Eq. 3-9; App. B).
//
// Mapping.  Every formula of the method is row-wise; the only sequential axis is the column
// index inside a group.  One row of a group lives in 16 lanes (one DPP row): column j sits in
// lane j % 16, register slot j / 16, so the live columns stay spread over all 16 lanes while
// the sweep advances.  A wavefront carries 4 rows, a work-group 16.  The local factor
// U_loc (g x g) is staged once per work-group in LDS, permuted so that a lane's slots are
// contiguous, with the diagonal and lower part zeroed (no masks in the inner loop).
//
// What is computed.  For a row with group-start working weights t and bit rows b_i, all the
// quantities the method needs are right-solves with U_loc:
//     tau = t U_loc^-1,   P_0 = 1 U_loc^-1,   P_i = b_i U_loc^-1.
// They are produced by the same forward recurrence as the error propagation of Eq. 3-4
// (x_l = v_l / U_ll;  v_{l+1:} -= x_l U_{l,l+1:}), so the bit-plane update of a column, its
// error coordinate and the k plane solves advance together, one column per step.  Then
//   * the fit of Eq. 6 is the (k+1) x (k+1) system G c = r with G_ab = P_a.P_b, r_a = P_a.tau
//     (since U_loc^-T B_r = [P_0 .. P_k]^T), accumulated and solved in fp64;
//   * the corrected propagation coordinates of Eq. 9 are E' = tau - sum_a c_a P_a
//     (App. B.3: E' U_loc = T - What_new), so What_old / Delta E are never materialised;
//   * the score of an iterate is ||E'||^2.
// Decisions (8-bit RTN code, nearest level) are taken in fp32 in a fixed operation order.
#pragma once
#include <utility>

#include "mfma_kmajor.h"

namespace bpdq {

constexpr int kRowsPerWG = 16;
constexpr int kSweepThreads = 256;
// Two work-groups per CU (a sweeping one and one in the tail role) need the kernel within 256
// registers per lane; the state of a g = 256 group does not fit that.
template <int G>
constexpr int kSweepWavesPerSimd = (G <= 128) ? 2 : 1;
// The lazy block update rides along with the sweep (extra work-groups of the group launch) only
// where a sweeping and an updating work-group fit on one CU; at g = 256 it is a launch of its own.
template <int G>
constexpr bool kTailInSweep = (G <= 128);

// ------------------------------------------------------------------ lane helpers -----------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  // every lane reads a valid lane of its own row, so the "old" operand is never used: passing x
  // itself spares the compiler a zero-initialisation per DPP move
  const int xi = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(xi, xi, CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ double dpp_d(double x) {
  const long long b = __builtin_bit_cast(long long, x);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffLL), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, false);
  return __builtin_bit_cast(double, ((long long)hi << 32) | (unsigned int)lo);
}
// value of lane O of this 16-lane row, in every lane of the row
template <int O>
__device__ __forceinline__ float bcast16(float x) { return dpp_f<0x150 + O>(x); }

// Butterfly over the 16 lanes of a row: xor 1, xor 2 (quad permutes), then half-row mirror and
// row mirror, which act as xor 4 / xor 8 once quads are uniform.  Every lane ends with the same
// bits (each stage adds the same two operands in both partners).
template <typename OP>
__device__ __forceinline__ float row_reduce_f(float v, OP op) {
  v = op(v, dpp_f<0xB1>(v));
  v = op(v, dpp_f<0x4E>(v));
  v = op(v, dpp_f<0x141>(v));
  v = op(v, dpp_f<0x140>(v));
  return v;
}
__device__ __forceinline__ double row_sum_d(double v) {
  v += dpp_d<0xB1>(v);
  v += dpp_d<0x4E>(v);
  v += dpp_d<0x141>(v);
  v += dpp_d<0x140>(v);
  return v;
}

// ------------------------------------------------------------------ per-row state ----------
template <int K, int G>
struct RowState {
  static constexpr int CPL = G / 16;
  float t[CPL];       // group-start working weights (frozen for the group)
  float tau[CPL];     // t U_loc^-1
  float p0[CPL];      // 1 U_loc^-1
  float wg[CPL];      // working copy during a sweep
  float P[K][CPL];    // running right-hand sides, then P_i = b_i U_loc^-1
  int code[CPL];      // plane bits of my columns, bit (i-1) = B_i
};

// LDS layout of the local factor.  Row l only ever meets columns j > l, and column j lives in
// slot j / 16 of lane j % 16, so row l keeps just the S = CPL - l / 16 slots m >= M = l / 16 of
// every lane: 16 S floats, no padding.  The slots are cut into chunks of 4, then 2, then 1
// (S = 7 -> 4 + 2 + 1); a chunk of width w that starts at slot M + o holds
//   sU[row_offset(l) + 16 o + lane * w + e] = U[l][16 (M + o + e) + lane]     (0 where j <= l)
// so one ds_read_b128 / b64 / b32 of the 16 lanes of a row covers 16 w contiguous floats (no bank
// conflicts) at an immediate offset, no register is loaded that the step does not use, and the
// lower part reads as zero (no masks in the inner loop).  36 KB at g = 128, 136 KB at g = 256.
template <int G>
struct SuLayout {
  static constexpr int CPL = G / 16;
  static constexpr int live(int M) { return CPL - M; }
  static constexpr int row_offset(int l) {
    int off = 0;
    for (int M = 0; M < l / 16; ++M) off += 256 * live(M);
    return off + 16 * (l % 16) * live(l / 16);
  }
  static constexpr int floats() { return row_offset(G); }
  // widest chunk: 4 floats (ds_read_b128); 2 at g = 256, where the wider reads push the
  // fully unrolled sweep over the register file
  static constexpr int kMaxVec = (G >= 256) ? 2 : 4;
  // width of the chunk that holds live slot o (0-based among the live slots) of a row with S
  // live slots, and the live slot that chunk starts at
  static constexpr int chunk_width(int S, int o) {
    const int g0 = o / kMaxVec * kMaxVec, r = S - g0, i = o - g0;
    if (r >= kMaxVec) return kMaxVec;     // a full chunk
    return (r >= 2 && i < 2) ? 2 : 1;     // r = 3: 2 + 1;  r = 2: 2;  r = 1: 1
  }
  static constexpr int chunk_start(int S, int o) {
    const int g0 = o / kMaxVec * kMaxVec, r = S - g0, i = o - g0;
    if (r >= kMaxVec) return g0;
    return (r >= 2 && i < 2) ? g0 : g0 + i;
  }
  // float index (relative to the row) of live slot o for lane `lane`
  static constexpr int slot_index(int S, int o, int lane) {
    const int w = chunk_width(S, o), c0 = chunk_start(S, o);
    return 16 * c0 + lane * w + (o - c0);
  }
};

// the live slots [M, CPL) of one row for this lane; p = sU + row_offset(l)
template <int G, int M>
__device__ __forceinline__ void load_u_row(const float* __restrict__ p, int lane16,
                                           float (&u)[G / 16]) {
  using Lay = SuLayout<G>;
  constexpr int CPL = G / 16, S = CPL - M;
  typedef float vec4 __attribute__((ext_vector_type(4)));
  typedef float vec2 __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int o = 0; o < S; ++o) {
    if (Lay::chunk_start(S, o) != o) continue;
    const int w = Lay::chunk_width(S, o);
    if (w == 4) {
      const vec4 v = *reinterpret_cast<const vec4*>(p + 16 * o + lane16 * 4);
      u[M + o] = v[0]; u[M + o + 1] = v[1]; u[M + o + 2] = v[2]; u[M + o + 3] = v[3];
    } else if (w == 2) {
      const vec2 v = *reinterpret_cast<const vec2*>(p + 16 * o + lane16 * 2);
      u[M + o] = v[0]; u[M + o + 1] = v[1];
    } else {
      u[M + o] = p[16 * o + lane16];
    }
  }
}

enum : int { kStepInit = 0, kStepSweep = 1, kStepUniform = 2 };

// One column of the forward recurrence.
//   kStepInit:    initial pass (codes known): builds tau, P_0 and the plane solves P_i.
//   kStepSweep:   bit-plane update of column L (Eq. 7-8), its error coordinate (Eq. 3),
//                 compensation of the later columns (Eq. 4), and the plane solves.
//   kStepUniform: the same column update with frozen coefficients and nothing else: the error
//                 coordinates themselves are kept in st.tau (fixed-grid GPTQ comparator).
// Row L of the local factor (`u`, `inv` = 1 / U_LL) arrives in registers; the step first issues
// the LDS reads of row L + 1 and hands them over at its end, so that their latency overlaps this
// column's arithmetic (one wave per SIMD: nothing else would hide it).
template <int K, int G, int L, int MODE>
__device__ __forceinline__ void column_step(RowState<K, G>& st, const float* __restrict__ sU,
                                            const float* __restrict__ sInv,
                                            const float (&lv)[1 << K], int lane16,
                                            float (&u)[G / 16], float& inv) {
  constexpr int CPL = G / 16, M = L / 16, O = L % 16;
  const bool owner = (lane16 == O);
  constexpr bool kPinState = true;
  constexpr bool kPrefetch = true;
  float un[CPL];
  float invn = 0.f;
  if constexpr (!kPrefetch) {
    load_u_row<G, M>(sU + SuLayout<G>::row_offset(L), lane16, u);
    inv = sInv[L];
  } else if constexpr (L + 1 < G) {
    load_u_row<G, (L + 1) / 16>(sU + SuLayout<G>::row_offset(L + 1), lane16, un);
    invn = sInv[L + 1];
    __builtin_amdgcn_sched_barrier(0);   // keep the reads ahead of the arithmetic below
  }
  float x[K], xb[K];
  if constexpr (MODE != kStepInit) {
    const float w = st.wg[M];
    float diff = w - lv[0];
    float bd = diff * diff;
    float bq = lv[0];
    int bc = 0;
#pragma unroll
    for (int c = 1; c < (1 << K); ++c) {
      diff = w - lv[c];
      const float dist = diff * diff;
      const bool lt = dist < bd;      // strict: the lowest code wins ties
      bd = lt ? dist : bd;
      bq = lt ? lv[c] : bq;
      bc = lt ? c : bc;
    }
    const float e = (w - bq) * inv;
    if (owner) st.code[M] = bc;
    if constexpr (MODE == kStepUniform) {
      if (owner) st.tau[M] = e;
    } else {
#pragma unroll
      for (int i = 0; i < K; ++i) x[i] = ((float)((bc >> i) & 1) + st.P[i][M]) * inv;
    }
    const float eb = bcast16<O>(e);
#pragma unroll
    for (int m = M; m < CPL; ++m) st.wg[m] = fmaf(-eb, u[m], st.wg[m]);
  } else {
    const float xt = st.tau[M] * inv;
    const float x0 = st.p0[M] * inv;
#pragma unroll
    for (int i = 0; i < K; ++i) x[i] = ((float)((st.code[M] >> i) & 1) + st.P[i][M]) * inv;
    if (owner) {
      st.tau[M] = xt;
      st.p0[M] = x0;
    }
    const float tb = bcast16<O>(xt);
    const float ob = bcast16<O>(x0);
#pragma unroll
    for (int m = M; m < CPL; ++m) {
      st.tau[m] = fmaf(-tb, u[m], st.tau[m]);
      st.p0[m] = fmaf(-ob, u[m], st.p0[m]);
    }
  }
  if constexpr (MODE != kStepUniform) {
#pragma unroll
    for (int i = 0; i < K; ++i) {
      if (owner) st.P[i][M] = x[i];
      xb[i] = bcast16<O>(x[i]);
#pragma unroll
      for (int m = M; m < CPL; ++m) st.P[i][m] = fmaf(-xb[i], u[m], st.P[i][m]);
    }
  }
  // The updates of far slots are not consumed for many steps; left alone, instruction selection
  // lets them drift there, together with the factor rows they need (hundreds of live registers).
  // Empty asm statements with the values as in/out operands pin them to this step.
  if constexpr (kPinState) {
#pragma unroll
    for (int m = M; m < CPL; ++m) {
      if constexpr (MODE != kStepInit) asm volatile("" : "+v"(st.wg[m]));
      if constexpr (MODE == kStepInit) asm volatile("" : "+v"(st.tau[m]), "+v"(st.p0[m]));
      if constexpr (MODE != kStepUniform) {
#pragma unroll
        for (int i = 0; i < K; ++i) asm volatile("" : "+v"(st.P[i][m]));
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);     // later steps' reads stay behind this step
  if constexpr (kPrefetch && L + 1 < G) {
#pragma unroll
    for (int m = (L + 1) / 16; m < CPL; ++m) u[m] = un[m];
    inv = invn;
  }
}

template <int K, int G, int MODE, int... Ls>
__device__ __forceinline__ void run_columns(RowState<K, G>& st, const float* sU, const float* sInv,
                                            const float (&lv)[1 << K], int lane16,
                                            std::integer_sequence<int, Ls...>) {
  float u[G / 16];
  load_u_row<G, 0>(sU, lane16, u);
  float inv = sInv[0];
  (column_step<K, G, Ls, MODE>(st, sU, sInv, lv, lane16, u, inv), ...);
}

// Stage the local factor U[s0:s0+G, s0:s0+G] in LDS (layout above) and 1 / U_ll in sInv.
// The G x G block is fetched as float4 with up to 16 loads of a thread in flight at once (a rolled
// element loop would wait for memory once per element); the part on or below the diagonal of a
// kept slot is stored as zero.
template <int G>
__device__ __forceinline__ void stage_local_factor(const float* __restrict__ U, int ldu, int s0,
                                                   float* sU, float* sInv) {
  using Lay = SuLayout<G>;
  constexpr int CPL = G / 16;
  if constexpr (G >= 256) {
    // the g = 256 kernels are at the limit of what the compiler handles in reasonable time:
    // they keep the plain element loop
    for (int e = threadIdx.x; e < G * G; e += kSweepThreads) {
      const int l = e / G, j = e % G;
      const int M = l >> 4, m = j >> 4;
      if (m >= M) {
        const float v = U[(long)(s0 + l) * ldu + s0 + j];
        const int off = 256 * (M * CPL - M * (M - 1) / 2) + 16 * (l & 15) * Lay::live(M);
        sU[off + Lay::slot_index(Lay::live(M), m - M, j & 15)] = (j > l) ? v : 0.f;
        if (j == l) sInv[l] = 1.0f / v;
      }
    }
    return;
  }
  constexpr int kPer = G * G / 4 / kSweepThreads;        // float4 loads per thread: 1, 4, 16
  constexpr int kBatch = kPer < 16 ? kPer : 16;
  for (int b = 0; b < kPer; b += kBatch) {
    float4 v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int q = threadIdx.x + (b + u) * kSweepThreads;
      const int l = q / (G / 4), j4 = (q % (G / 4)) * 4;
      v[u] = *reinterpret_cast<const float4*>(U + (long)(s0 + l) * ldu + s0 + j4);
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int q = threadIdx.x + (b + u) * kSweepThreads;
      const int l = q / (G / 4), j4 = (q % (G / 4)) * 4;
      const int M = l >> 4, m = j4 >> 4;                  // the four columns share one slot
      if (m >= M) {
        const int off = 256 * (M * CPL - M * (M - 1) / 2) + 16 * (l & 15) * Lay::live(M);
        const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int j = j4 + c;
          sU[off + Lay::slot_index(Lay::live(M), m - M, j & 15)] = (j > l) ? e[c] : 0.f;
          if (j == l) sInv[l] = 1.0f / e[c];
        }
      }
    }
  }
}

// Storage precision of a coefficient: IEEE half (nearest even) when the layer is stored with
// 16-bit coefficients (Table 1), so that everything computed from it belongs to the stored value.
__device__ __forceinline__ float store_precision(float c, int coef_fp16) {
  return coef_fp16 ? (float)(_Float16)c : c;
}

// Coefficient fit (Eq. 6) from the solved vectors; returns c (fp32) and the row's ||E'||^2.
template <int K, int G>
__device__ __forceinline__ double fit_and_score(const RowState<K, G>& st, double alpha, int coef_fp16,
                                                float (&c32)[K + 1], float (&Ep)[G / 16]) {
  constexpr int CPL = G / 16, N = K + 1;
  double Gm[N][N], r[N];
#pragma unroll
  for (int a = 0; a < N; ++a) {
#pragma unroll
    for (int b = a; b < N; ++b) {
      double s = 0.0;
#pragma unroll
      for (int m = 0; m < CPL; ++m) {
        const float va = (a == 0) ? st.p0[m] : st.P[a - 1 < 0 ? 0 : a - 1][m];
        const float vb = (b == 0) ? st.p0[m] : st.P[b - 1 < 0 ? 0 : b - 1][m];
        s += (double)va * (double)vb;
      }
      Gm[a][b] = row_sum_d(s);
    }
    double s = 0.0;
#pragma unroll
    for (int m = 0; m < CPL; ++m) {
      const float va = (a == 0) ? st.p0[m] : st.P[a - 1 < 0 ? 0 : a - 1][m];
      s += (double)va * (double)st.tau[m];
    }
    r[a] = row_sum_d(s);
  }
  double tr = 0.0;
#pragma unroll
  for (int a = 0; a < N; ++a) tr += Gm[a][a];
  const double mu = alpha * tr / (double)N;
#pragma unroll
  for (int a = 0; a < N; ++a) {
    Gm[a][a] += mu;
#pragma unroll
    for (int b = 0; b < a; ++b) Gm[a][b] = Gm[b][a];
  }
  // Gaussian elimination without pivoting (G is symmetric positive definite after the ridge)
#pragma unroll
  for (int p = 0; p < N; ++p) {
    const double ip = 1.0 / Gm[p][p];
#pragma unroll
    for (int a = p + 1; a < N; ++a) {
      const double f = Gm[a][p] * ip;
#pragma unroll
      for (int b = p + 1; b < N; ++b) Gm[a][b] -= f * Gm[p][b];
      r[a] -= f * r[p];
    }
  }
  double c[N];
#pragma unroll
  for (int a = N - 1; a >= 0; --a) {
    double s = r[a];
#pragma unroll
    for (int b = a + 1; b < N; ++b) s -= Gm[a][b] * c[b];
    c[a] = s / Gm[a][a];
  }
#pragma unroll
  for (int a = 0; a < N; ++a) c32[a] = store_precision((float)c[a], coef_fp16);
  double sc = 0.0;
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    float e = fmaf(-c32[0], st.p0[m], st.tau[m]);
#pragma unroll
    for (int i = 0; i < K; ++i) e = fmaf(-c32[i + 1], st.P[i][m], e);
    Ep[m] = e;
    sc += (double)e * (double)e;
  }
  return row_sum_d(sc);
}

// v(code) = ((c0 + b1 c1) + b2 c2) + ...  in fp32 (Eq. 7)
template <int K>
__device__ __forceinline__ void level_table(const float (&c)[K + 1], float (&lv)[1 << K]) {
#pragma unroll
  for (int code = 0; code < (1 << K); ++code) {
    float v = c[0];
#pragma unroll
    for (int i = 0; i < K; ++i)
      if ((code >> i) & 1) v = v + c[i + 1];
    lv[code] = v;
  }
}

// ------------------------------------------------------------------ pending updates --------
// Error compensation of the columns not yet quantized (Eq. 4) is applied lazily, block by block
// (App. B.3, tail form), and never on the critical path between two groups:
//   * every committed E* is kept K-major in Eall[column][row] (leading dimension lde);
//   * the group that starts at column s0 reads its target left-looking:
//       t = W'[rows, s0:s0+g] - Eall[kp0:s0, rows]^T U[kp0:s0, s0:s0+g]
//     where kp0 is the start of the previous block: W' itself holds the updates of all blocks
//     before that one;
//   * the update of block q-1 to the columns beyond block q is a GEMM that extra work-groups of
//     the first group launch of block q perform (the "tail role"): it only needs E* committed
//     before the launch and touches no column the launch's sweep reads, so it overlaps the
//     latency-bound sweep instead of waiting between two of them;
//   * two levels: that per-block update (depth B) only reaches to the end of the NEXT super-block
//     (about 1024 columns per super-block); the columns beyond receive one deep update per finished
//     super-block (depth ~1024: an eighth of the traffic on W' per flop, and long enough to
//     amortise a tile's prologue), dealt in column chunks to the group launches of the following
//     super-block.  The two updates of one launch never touch the same columns (see the host loop).
//     Only the order of summation differs from one update per block.
struct TailTask {
  const float* Et;     // Eall + k0 * lde
  int Kd;              // depth of the update (finished columns)
  int k0;              // first finished column (row of U)
  int c_begin, c_end;  // columns [c_begin, c_end) of W' to update
  int tiles_n;         // column tiles; 0 = nothing to do
};
struct TailArgs {
  TailTask far, near;  // deep update of a finished super-block / update of the previous block
  float* Wp;           // working copy W'
  int first_wg;        // work-groups below this index sweep
  int far_wgs;         // tail work-groups [first_wg, first_wg + far_wgs) take `far`, the rest `near`
};

// Layers that share one input share U and go through the sweep stacked by rows; the best
// iterate of a group is chosen per layer (segment).  Boundaries in work-groups of 16 rows.
constexpr int kMaxSegments = 8;
struct SegArgs {
  int n_seg;
  int wg_end[kMaxSegments];   // ascending; wg_end[n_seg - 1] = number of sweeping work-groups
};

// W'[:, c_begin:c_end] -= Et^T U[k0:k0+Kd, c_begin:c_end], one 128 x 128 tile per work-group
__device__ __forceinline__ void tail_role(const TailArgs& ta, const float* __restrict__ U, int ldu,
                                          int lde, int ldw, int d_out) {
  int t = blockIdx.x - ta.first_wg;
  const bool is_far = t < ta.far_wgs;          // uniform over the work-group
  if (!is_far) t -= ta.far_wgs;
  const TailTask& task = is_far ? ta.far : ta.near;
  const int tm = t / task.tiles_n, tn = t % task.tiles_n;
  TailGemm::Acc acc;
  TailGemm::zero(acc);
  TailGemm::run<0>(task.Et, lde, tm * TailGemm::kTileM, lde, U + (long)task.k0 * ldu, ldu,
                   task.c_begin + tn * TailGemm::kTileN, task.c_end, 0, task.Kd, acc);
  const int r0 = tm * TailGemm::kTileM, c0 = task.c_begin + tn * TailGemm::kTileN;
  float* Wp = ta.Wp;
  const int c_end = task.c_end;
  // in-place read-modify-write of this lane's 64 results: all loads first (masked elements read
  // a valid address and are not stored), then the stores
  float old[TailGemm::kAccPerLane];
  int n = 0;
  TailGemm::for_each(acc, [&](int row, int col, float) {
    const int r = r0 + row, c = c0 + col;
    old[n++] = Wp[(r < d_out && c < c_end) ? (long)r * ldw + c : 0L];
  });
  n = 0;
  TailGemm::for_each(acc, [&](int row, int col, float v) {
    const int r = r0 + row, c = c0 + col;
    if (r < d_out && c < c_end) Wp[(long)r * ldw + c] = old[n] - v;
    ++n;
  });
}

// sT[r][c] = sum_{k < Kp} Eall[kp0 + k][row0 + r] * U[kp0 + k][s0 + c]   (16 rows x G columns)
// with v_mfma_f32_16x16x4_f32: the column blocks of 16 are dealt to the four wavefronts; operands
// go straight from global memory to registers (lane l: A[l % 16][l / 16], B[l / 16][l % 16]),
// the result (register r of lane l = D[4 (l / 16) + r][l % 16]) to LDS.  Kp % 32 == 0.
template <int G>
struct PendingTile {
  static constexpr int kStride = G + 4;
  static constexpr int kFloats = kRowsPerWG * kStride;
};
template <int G>
__device__ __forceinline__ void pending_update_tile(const float* __restrict__ Eall, int lde,
                                                    const float* __restrict__ U, int ldu, int kp0,
                                                    int Kp, int row0, int s0, float* sT) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  constexpr int NB = G / 16, BPW = (NB + 3) / 4;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = lane & 15, kq = lane >> 4;
  f4 acc[BPW];
#pragma unroll
  for (int b = 0; b < BPW; ++b) acc[b] = f4{0.f, 0.f, 0.f, 0.f};
  const float* ap = Eall + (long)(kp0 + kq) * lde + row0 + i;
  const float* bp = U + (long)(kp0 + kq) * ldu + s0 + 16 * wave * BPW + i;
  const bool active = wave * BPW < NB;          // g = 32: two blocks, wavefronts 2 and 3 idle
  if (active) {
    // kChunk MFMA steps (4 columns of E* each) per round trip to memory: all their operands are
    // requested before the first one is used.  Kp % 32 == 0 (g >= 32 divides it).
    constexpr int kChunk = (BPW <= 2) ? 16 : 8;
    for (int k = 0; k < Kp; k += 4 * kChunk) {
      float a[kChunk], bv[kChunk][BPW];
#pragma unroll
      for (int u = 0; u < kChunk; ++u) {
        // steps past Kp re-read step k (a valid address) and contribute nothing
        const bool in = k + 4 * u < Kp;
        const long kk = in ? k + 4 * u : k;
        const float av = ap[kk * lde];
        a[u] = in ? av : 0.f;
#pragma unroll
        for (int b = 0; b < BPW; ++b) bv[u][b] = bp[kk * ldu + 16 * b];
      }
#pragma unroll
      for (int u = 0; u < kChunk; ++u)
#pragma unroll
        for (int b = 0; b < BPW; ++b)
          acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u], bv[u][b], acc[b], 0, 0, 0);
    }
#pragma unroll
    for (int b = 0; b < BPW; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        sT[(4 * kq + r) * PendingTile<G>::kStride + 16 * (wave * BPW + b) + i] = acc[b][r];
  }
}

// Group-start working weights of this lane's columns: W' minus the pending updates.
template <int K, int G>
__device__ __forceinline__ void load_group_target(RowState<K, G>& st, const float* __restrict__ Wp,
                                                  int ldw, int rr, int s0, int lane16,
                                                  const float* __restrict__ Eall, int lde,
                                                  const float* __restrict__ U, int ldu, int kp0,
                                                  float* sT) {
  constexpr int CPL = G / 16;
  const float* wrow = Wp + (long)rr * ldw + s0;
#pragma unroll
  for (int m = 0; m < CPL; ++m) st.t[m] = wrow[16 * m + lane16];
  if (kp0 < s0) {                                   // uniform over the launch
    pending_update_tile<G>(Eall, lde, U, ldu, kp0, s0 - kp0, blockIdx.x * kRowsPerWG, s0, sT);
    __syncthreads();
    const float* trow = sT + (threadIdx.x >> 4) * PendingTile<G>::kStride;
#pragma unroll
    for (int m = 0; m < CPL; ++m) st.t[m] -= trow[16 * m + lane16];
  }
}

template <int K, int G>
struct Candidates {          // per-iterate scratch in the workspace
  unsigned char* codes;      // [T+1][d_out][G]
  float* coef;               // [T+1][d_out][K+1]
  float* E;                  // [T+1][d_out][G]
  double* score;             // [T+1][n_wg]
};

template <int K, int G>
__device__ __forceinline__ void store_candidate(const RowState<K, G>& st, const float (&c32)[K + 1],
                                                const float (&Ep)[G / 16], double rowscore, int it,
                                                int row, bool valid, int d_out, int n_wg,
                                                unsigned char* codes, float* coef, float* E,
                                                double* score, double* sScore, int lane16) {
  constexpr int CPL = G / 16;
  if (valid) {
    const long base = ((long)it * d_out + row) * G;
#pragma unroll
    for (int m = 0; m < CPL; ++m) {
      codes[base + 16 * m + lane16] = (unsigned char)st.code[m];
      E[base + 16 * m + lane16] = Ep[m];
    }
    if (lane16 <= K) {
      float v = c32[0];
#pragma unroll
      for (int i = 1; i <= K; ++i) v = (lane16 == i) ? c32[i] : v;
      coef[((long)it * d_out + row) * (K + 1) + lane16] = v;
    }
  }
  __syncthreads();
  if (lane16 == 0) sScore[threadIdx.x >> 4] = valid ? rowscore : 0.0;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int q = 0; q < kRowsPerWG; ++q) s += sScore[q];
    score[(long)it * n_wg + blockIdx.x] = s;
  }
}

// One group of g columns for 16 rows per work-group: initialisation, fit, T refinement
// iterations; every iterate's (codes, coefficients, E', score) is kept for the selection.
template <int K, int G>
__global__ __launch_bounds__(kSweepThreads, kSweepWavesPerSimd<G>) void bpdq_group_kernel(
    const float* __restrict__ Wp, int ldw, int d_out, const float* __restrict__ U, int ldu, int s0,
    int T, float alpha, int coef_fp16, unsigned char* __restrict__ cand_codes,
    float* __restrict__ cand_coef,
    float* __restrict__ cand_E, double* __restrict__ cand_score, int n_wg,
    const float* __restrict__ Eall, int lde, int kp0, TailArgs ta) {
  if constexpr (kTailInSweep<G>) {
    if ((int)blockIdx.x >= ta.first_wg) {
      tail_role(ta, U, ldu, lde, ldw, d_out);
      return;
    }
  }
  // the sweep is the critical path of the launch: where a sweeping and an updating wavefront share
  // a SIMD, the sweeping one issues first
  __builtin_amdgcn_s_setprio(3);
  constexpr int CPL = G / 16;
  extern __shared__ float lds[];
  float* sU = lds;                            // packed local factor, see SuLayout
  float* sInv = lds + SuLayout<G>::floats();          // 1 / U_ll
  double* sScore = reinterpret_cast<double*>(lds + SuLayout<G>::floats() + G);
  float* sT = lds + SuLayout<G>::floats() + G + 2 * kRowsPerWG;   // pending-update tile
  const int tid = threadIdx.x;
  const int lane16 = tid & 15;
  stage_local_factor<G>(U, ldu, s0, sU, sInv);

  const int row = blockIdx.x * kRowsPerWG + (tid >> 4);
  const bool valid = row < d_out;
  const int rr = valid ? row : d_out - 1;
  RowState<K, G> st;
  load_group_target<K, G>(st, Wp, ldw, rr, s0, lane16, Eall, lde, U, ldu, kp0, sT);
  __syncthreads();

  // ---- bit-plane initialisation (Sec. 3.2, Eq. 5): 8-bit affine RTN, keep the k MSB planes
  float lo = st.t[0], hi = st.t[0];
#pragma unroll
  for (int m = 1; m < CPL; ++m) {
    lo = fminf(lo, st.t[m]);
    hi = fmaxf(hi, st.t[m]);
  }
  lo = row_reduce_f(lo, [](float a, float b) { return fminf(a, b); });
  hi = row_reduce_f(hi, [](float a, float b) { return fmaxf(a, b); });
  const float sc = (hi - lo) / 255.0f;
  const bool flat = (hi == lo);
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    const float q = (st.t[m] - lo) / (flat ? 1.0f : sc);
    float z = rintf(q);                       // round half to even
    z = fminf(fmaxf(z, 0.f), 255.f);
    st.code[m] = flat ? 0 : ((int)z >> (8 - K));
    st.tau[m] = st.t[m];
    st.p0[m] = 1.0f;
#pragma unroll
    for (int i = 0; i < K; ++i) st.P[i][m] = 0.f;
  }
  float lv[1 << K];
#pragma unroll
  for (int c = 0; c < (1 << K); ++c) lv[c] = 0.f;
  using Seq = std::make_integer_sequence<int, G>;
  run_columns<K, G, kStepInit>(st, sU, sInv, lv, lane16, Seq{});

  float c32[K + 1], Ep[CPL];
  double rs = fit_and_score<K, G>(st, (double)alpha, coef_fp16, c32, Ep);
  store_candidate<K, G>(st, c32, Ep, rs, 0, row, valid, d_out, n_wg, cand_codes, cand_coef,
                        cand_E, cand_score, sScore, lane16);

  // ---- refinement iterations (Sec. 3.3)
  for (int it = 1; it <= T; ++it) {
    level_table<K>(c32, lv);
#pragma unroll
    for (int m = 0; m < CPL; ++m) {
      st.wg[m] = st.t[m];
#pragma unroll
      for (int i = 0; i < K; ++i) st.P[i][m] = 0.f;
    }
    run_columns<K, G, kStepSweep>(st, sU, sInv, lv, lane16, Seq{});
    rs = fit_and_score<K, G>(st, (double)alpha, coef_fp16, c32, Ep);
    store_candidate<K, G>(st, c32, Ep, rs, it, row, valid, d_out, n_wg, cand_codes, cand_coef,
                          cand_E, cand_score, sScore, lane16);
  }
}

// Fixed-uniform-grid comparator (App. A, "Fixed Grid"): the same column sweep with the levels
// frozen to lo + s * {0 .. 2^k - 1}, s = (hi - lo) / (2^k - 1), written as bit-plane coefficients
// (lo, s, 2s, 4s, ...) -- the special case of Prop. 1.  One pass, no fit, no iteration: this is
// GPTQ on the asymmetric min/max grid.  The result is stored as iterate 0.
template <int K, int G>
__global__ __launch_bounds__(kSweepThreads, kSweepWavesPerSimd<G>) void uniform_group_kernel(
    const float* __restrict__ Wp, int ldw, int d_out, const float* __restrict__ U, int ldu, int s0,
    int coef_fp16, unsigned char* __restrict__ cand_codes, float* __restrict__ cand_coef,
    float* __restrict__ cand_E, double* __restrict__ cand_score, int n_wg,
    const float* __restrict__ Eall, int lde, int kp0, TailArgs ta) {
  if constexpr (kTailInSweep<G>) {
    if ((int)blockIdx.x >= ta.first_wg) {
      tail_role(ta, U, ldu, lde, ldw, d_out);
      return;
    }
  }
  // the sweep is the critical path of the launch: where a sweeping and an updating wavefront share
  // a SIMD, the sweeping one issues first
  __builtin_amdgcn_s_setprio(3);
  constexpr int CPL = G / 16;
  extern __shared__ float lds[];
  float* sU = lds;
  float* sInv = lds + SuLayout<G>::floats();
  double* sScore = reinterpret_cast<double*>(lds + SuLayout<G>::floats() + G);
  float* sT = lds + SuLayout<G>::floats() + G + 2 * kRowsPerWG;
  const int tid = threadIdx.x;
  const int lane16 = tid & 15;
  stage_local_factor<G>(U, ldu, s0, sU, sInv);

  const int row = blockIdx.x * kRowsPerWG + (tid >> 4);
  const bool valid = row < d_out;
  const int rr = valid ? row : d_out - 1;
  RowState<K, G> st;
  load_group_target<K, G>(st, Wp, ldw, rr, s0, lane16, Eall, lde, U, ldu, kp0, sT);
  __syncthreads();
  float lo = st.t[0], hi = st.t[0];
#pragma unroll
  for (int m = 1; m < CPL; ++m) {
    lo = fminf(lo, st.t[m]);
    hi = fmaxf(hi, st.t[m]);
  }
  lo = row_reduce_f(lo, [](float a, float b) { return fminf(a, b); });
  hi = row_reduce_f(hi, [](float a, float b) { return fmaxf(a, b); });
  float step = (hi - lo) / (float)((1 << K) - 1);
  if (step == 0.f) step = 1.0f;                 // flat row: every weight takes code 0
  float c32[K + 1], lv[1 << K], Ep[CPL];
  c32[0] = store_precision(lo, coef_fp16);
#pragma unroll
  for (int i = 0; i < K; ++i) c32[i + 1] = store_precision(step * (float)(1 << i), coef_fp16);
  level_table<K>(c32, lv);
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    st.wg[m] = st.t[m];
    st.tau[m] = 0.f;
    st.code[m] = 0;
  }
  using Seq = std::make_integer_sequence<int, G>;
  run_columns<K, G, kStepUniform>(st, sU, sInv, lv, lane16, Seq{});
  double sc = 0.0;
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    Ep[m] = st.tau[m];
    sc += (double)Ep[m] * (double)Ep[m];
  }
  sc = row_sum_d(sc);
  store_candidate<K, G>(st, c32, Ep, sc, 0, row, valid, d_out, n_wg, cand_codes, cand_coef,
                        cand_E, cand_score, sScore, lane16);
}

// Selection + commit of one group, 16 rows per work-group (same lane mapping as the sweep).
// Every work-group first sums the row-block scores of each iterate over its own layer (segment)
// in one fixed order and takes the earliest minimum (Sec. 3.3: keep the iterate with the smallest
// ||E_group||_F^2), so all work-groups of a layer agree bit for bit; the first work-group of a
// segment publishes grp_iter / grp_err (arrays of n_grp entries per segment).  Then the kept
// iterate is written out: packed planes (wave ballots), coefficients, What, and E* transposed
// into the K-major error buffer Eblk[(s0 - b0) + j][row] (leading dimension lde).
template <int K, int G>
__global__ __launch_bounds__(256) void commit_group_kernel(
    const unsigned char* __restrict__ cand_codes, const float* __restrict__ cand_coef,
    const float* __restrict__ cand_E, const double* __restrict__ cand_score, int n_wg, int T,
    SegArgs seg, double* __restrict__ grp_err, int* __restrict__ grp_iter, int d_out, int d_in,
    int s0, int b0,
    uint32_t* __restrict__ planes, float* __restrict__ coefs, float* __restrict__ W_hat,
    float* __restrict__ Eblk, int lde) {
  constexpr int CPL = G / 16;
  __shared__ double tot[64];
  __shared__ float sE[G][17];
  const int tid = threadIdx.x, lane16 = tid & 15;
  // my segment (work-groups past the last row belong to the last one; they write nothing)
  int wg_lo = 0, wg_hi = seg.wg_end[0], si = 0;
#pragma unroll
  for (int q = 1; q < kMaxSegments; ++q)
    if (q < seg.n_seg && (int)blockIdx.x >= seg.wg_end[q - 1]) {
      wg_lo = seg.wg_end[q - 1];
      wg_hi = seg.wg_end[q];
      si = q;
    }
  // iterate q is summed by wavefront q % 4: strided partial sums per lane, then a fixed
  // xor butterfly over the 64 lanes
  for (int q = tid >> 6; q <= T; q += 4) {
    double s = 0.0;
    for (int w = wg_lo + (tid & 63); w < wg_hi; w += 64) s += cand_score[(long)q * n_wg + w];
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) s += __shfl_xor(s, m, 64);
    if ((tid & 63) == 0) tot[q] = s;
  }
  __syncthreads();
  int it = 0;
  for (int q = 1; q <= T; ++q)
    if (tot[q] < tot[it]) it = q;
  if ((int)blockIdx.x == wg_lo && tid == 0) {
    grp_iter[(long)si * (d_in / G)] = it;
    grp_err[(long)si * (d_in / G)] = tot[it];
  }

  const int row0 = blockIdx.x * kRowsPerWG;
  const int rloc = tid >> 4;
  const int row = row0 + rloc;
  const bool valid = row < d_out;
  const int rr = valid ? row : d_out - 1;
  const int n_grp = d_in / G, gi = s0 / G, n_word = d_in / 32;
  const long cbase = ((long)it * d_out + rr) * G;
  float c[K + 1], lv[1 << K];
#pragma unroll
  for (int i = 0; i <= K; ++i) c[i] = cand_coef[((long)it * d_out + rr) * (K + 1) + i];
  level_table<K>(c, lv);
  int code[CPL];
#pragma unroll
  for (int m = 0; m < CPL; ++m) {
    code[m] = cand_codes[cbase + 16 * m + lane16];
    sE[16 * m + lane16][rloc] = valid ? cand_E[cbase + 16 * m + lane16] : 0.f;
  }
  // planes: a wave ballot holds bit (16 q + lane16) for row q of the wave
  const int shift = 16 * ((tid & 63) >> 4);
#pragma unroll
  for (int i = 0; i < K; ++i) {
#pragma unroll
    for (int w = 0; w < G / 32; ++w) {
      const unsigned long long lo = __ballot((code[2 * w] >> i) & 1);
      const unsigned long long hi = __ballot((code[2 * w + 1] >> i) & 1);
      const uint32_t word = (uint32_t)((lo >> shift) & 0xffffu) | ((uint32_t)((hi >> shift) & 0xffffu) << 16);
      if (valid && lane16 == 0) planes[((long)i * d_out + row) * n_word + s0 / 32 + w] = word;
    }
  }
  if (valid) {
    if (W_hat) {
#pragma unroll
      for (int m = 0; m < CPL; ++m) {
        float v = lv[0];
#pragma unroll
        for (int q = 1; q < (1 << K); ++q) v = (code[m] == q) ? lv[q] : v;
        W_hat[(long)row * d_in + s0 + 16 * m + lane16] = v;
      }
    }
    if (lane16 <= K) {
      float v = c[0];
#pragma unroll
      for (int i = 1; i <= K; ++i) v = (lane16 == i) ? c[i] : v;
      coefs[((long)lane16 * d_out + row) * n_grp + gi] = v;
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * kRowsPerWG; idx += 256) {
    const int j = idx >> 4, r = idx & 15;
    Eblk[(long)(s0 - b0 + j) * lde + row0 + r] = sE[j][r];
  }
}

// ------------------------------------------------------------------ host side --------------
struct QuantLayout {
  size_t wp_off, eall_off, codes_off, coef_off, e_off, score_off, total;
  int B, lde, n_wg;
};

static inline QuantLayout quant_layout(int d_out, int d_in, const bpdq_params& p) {
  QuantLayout L;
  const int g = p.group, T = p.refine_iters, K = p.bits;
  L.B = p.block > g ? p.block : g;
  L.lde = (int)bpdq_align_up((size_t)d_out, 64);
  L.n_wg = bpdq_ceil_div(d_out, kRowsPerWG);
  size_t off = 0;
  L.wp_off = off;    off += bpdq_align_up((size_t)d_out * d_in * sizeof(float), 256);
  L.eall_off = off;  off += bpdq_align_up((size_t)d_in * L.lde * sizeof(float), 256);
  L.codes_off = off; off += bpdq_align_up((size_t)(T + 1) * d_out * g, 256);
  L.coef_off = off;  off += bpdq_align_up((size_t)(T + 1) * d_out * (K + 1) * sizeof(float), 256);
  L.e_off = off;     off += bpdq_align_up((size_t)(T + 1) * d_out * g * sizeof(float), 256);
  L.score_off = off; off += bpdq_align_up((size_t)(T + 1) * L.n_wg * sizeof(double), 256);
  L.total = off;
  return L;
}

// the tail role as a kernel of its own (defined with the host loop)
int launch_tail_update(hipStream_t stream, TailArgs ta, const float* U, int ldu, int lde, int ldw,
                       int d_out, int n_tiles);

template <int G>
constexpr size_t sweep_lds_bytes() {
  const size_t a = (size_t)(SuLayout<G>::floats() + G + 2 * kRowsPerWG + PendingTile<G>::kFloats) * sizeof(float);
  return a < TailGemm::kLdsBytes ? TailGemm::kLdsBytes : a;
}

// launch of the fixed-grid comparator's sweep kernel
struct UniformSweepArgs {
  hipStream_t stream;
  int grid;
  const float* Wp;
  int d_in, d_out;
  const float* U;
  int s0, coef_fp16;
  unsigned char* c_codes;
  float* c_coef;
  float* c_E;
  double* c_score;
  int n_wg;
  const float* Eall;
  int lde, kp0;
  TailArgs ta;
};

template <int K, int G>
static inline int launch_uniform_sweep(const UniformSweepArgs& a) {
  const size_t lds = sweep_lds_bytes<G>();
  BPDQ_HIP_TRY((bpdq_lds_limit<&uniform_group_kernel<K, G>>(lds)));
  hipLaunchKernelGGL((uniform_group_kernel<K, G>), dim3(a.grid), dim3(kSweepThreads), lds, a.stream,
                     a.Wp, a.d_in, a.d_out, a.U, a.d_in, a.s0, a.coef_fp16, a.c_codes, a.c_coef, a.c_E,
                     a.c_score, a.n_wg, a.Eall, a.lde, a.kp0, a.ta);
  BPDQ_LAUNCH_CHECK();
  return 0;
}
// group size 256: defined in group_sweep_k{K}_g256u.hip (the two g = 256 kernels of a plane count
// are the longest compilations of the build; apart they run in parallel)
template <int K>
int launch_uniform_sweep_256(const UniformSweepArgs& a);

// One group: the sweep kernel (with the pending updates read left-looking from column kp0 on, and
// the tail role `ta` for the previous block, see above), then selection + commit.
template <int K, int G>
static inline int launch_group(hipStream_t stream, const float* Wp, int d_out, int d_in, const float* U,
                        int s0, int kp0, TailArgs ta, const SegArgs& seg, const bpdq_params& p,
                        const QuantLayout& L, char* base, uint32_t* planes, float* coefs,
                        float* W_hat, double* grp_err, int* grp_iter) {
  unsigned char* c_codes = reinterpret_cast<unsigned char*>(base + L.codes_off);
  float* c_coef = reinterpret_cast<float*>(base + L.coef_off);
  float* c_E = reinterpret_cast<float*>(base + L.e_off);
  double* c_score = reinterpret_cast<double*>(base + L.score_off);
  float* Eall = reinterpret_cast<float*>(base + L.eall_off);
  const size_t lds = sweep_lds_bytes<G>();
  const int gi = s0 / G;
  const bool uniform = (p.grid == BPDQ_GRID_UNIFORM);
  const int T = uniform ? 0 : p.refine_iters;
  ta.first_wg = L.n_wg;
  const int row_tiles = bpdq_ceil_div(L.lde, TailGemm::kTileM);
  ta.far_wgs = row_tiles * ta.far.tiles_n;
  int n_tail = row_tiles * (ta.far.tiles_n + ta.near.tiles_n);
  if (!kTailInSweep<G> && n_tail > 0) {
    const int rc = launch_tail_update(stream, ta, U, d_in, L.lde, d_in, d_out, n_tail);
    if (rc) return rc;
    n_tail = 0;
  }
  const int grid = L.n_wg + n_tail;
  if (uniform) {
    const UniformSweepArgs a{stream, grid, Wp, d_in, d_out, U, s0, p.coef_fp16, c_codes, c_coef, c_E,
                             c_score, L.n_wg, Eall, L.lde, kp0, ta};
    int rc;
    if constexpr (G >= 256) rc = launch_uniform_sweep_256<K>(a);   // a translation unit of its own
    else rc = launch_uniform_sweep<K, G>(a);
    if (rc) return rc;
  } else {
    BPDQ_HIP_TRY((bpdq_lds_limit<&bpdq_group_kernel<K, G>>(lds)));
    hipLaunchKernelGGL((bpdq_group_kernel<K, G>), dim3(grid), dim3(kSweepThreads), lds, stream,
                       Wp, d_in, d_out, U, d_in, s0, T, p.alpha, p.coef_fp16, c_codes, c_coef, c_E, c_score,
                       L.n_wg, Eall, L.lde, kp0, ta);
  }
  BPDQ_LAUNCH_CHECK();
  hipLaunchKernelGGL((commit_group_kernel<K, G>), dim3(L.lde / kRowsPerWG), dim3(256), 0, stream,
                     c_codes, c_coef, c_E, c_score, L.n_wg, T, seg, grp_err + gi, grp_iter + gi, d_out,
                     d_in, s0, 0, planes, coefs, W_hat, Eall, L.lde);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

typedef int (*GroupLauncher)(hipStream_t, const float*, int, int, const float*, int, int, TailArgs,
                             const SegArgs&, const bpdq_params&, const QuantLayout&, char*, uint32_t*,
                             float*, float*, double*, int*);

// The group kernels are large, fully unrolled kernels: one translation unit per plane count
// instantiates group sizes 32 / 64 / 128, and two more per plane count (1..3) group size 256
// (variable grid, fixed grid), which keeps the build parallel.  Four planes at g = 256 -- a
// combination the paper does not use -- would by itself double the build time and is left out.
GroupLauncher pick_group_k1(int g);
GroupLauncher pick_group_k2(int g);
GroupLauncher pick_group_k3(int g);
GroupLauncher pick_group_k4(int g);
GroupLauncher group256_k1();
GroupLauncher group256_k2();
GroupLauncher group256_k3();

template <int K>
static inline GroupLauncher pick_group_g(int g) {
  switch (g) {
    case 32: return launch_group<K, 32>;
    case 64: return launch_group<K, 64>;
    case 128: return launch_group<K, 128>;
  }
  return nullptr;
}
}  // namespace bpdq
