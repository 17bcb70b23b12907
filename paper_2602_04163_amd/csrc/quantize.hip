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
#include <utility>

#include "mfma_kmajor.h"

namespace bpdq {

constexpr int kRowsPerWG = 16;
constexpr int kSweepThreads = 256;

// ------------------------------------------------------------------ lane helpers -----------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
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

// One column of the forward recurrence.  SWEEP = false: initial pass (codes known, also
// builds tau and P_0).  SWEEP = true: bit-plane update of column L (Eq. 7-8), its error
// coordinate (Eq. 3) and compensation of the later columns (Eq. 4), plus the plane solves.
template <int K, int G, int L, bool SWEEP>
__device__ __forceinline__ void column_step(RowState<K, G>& st, const float* __restrict__ sU,
                                            const float* __restrict__ sInv,
                                            const float (&lv)[1 << K], int lane16) {
  constexpr int CPL = G / 16, M = L / 16, O = L % 16;
  const float inv = sInv[L];
  const bool owner = (lane16 == O);
  float u[CPL];
#pragma unroll
  for (int m = M; m < CPL; ++m) u[m] = sU[L * G + lane16 * CPL + m];

  float x[K], xb[K];
  if constexpr (SWEEP) {
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
#pragma unroll
    for (int i = 0; i < K; ++i) x[i] = ((float)((bc >> i) & 1) + st.P[i][M]) * inv;
    if (owner) st.code[M] = bc;
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
#pragma unroll
  for (int i = 0; i < K; ++i) {
    if (owner) st.P[i][M] = x[i];
    xb[i] = bcast16<O>(x[i]);
#pragma unroll
    for (int m = M; m < CPL; ++m) st.P[i][m] = fmaf(-xb[i], u[m], st.P[i][m]);
  }
}

template <int K, int G, bool SWEEP, int... Ls>
__device__ __forceinline__ void run_columns(RowState<K, G>& st, const float* sU, const float* sInv,
                                            const float (&lv)[1 << K], int lane16,
                                            std::integer_sequence<int, Ls...>) {
  (column_step<K, G, Ls, SWEEP>(st, sU, sInv, lv, lane16), ...);
}

// Coefficient fit (Eq. 6) from the solved vectors; returns c (fp32) and the row's ||E'||^2.
template <int K, int G>
__device__ __forceinline__ double fit_and_score(const RowState<K, G>& st, double alpha,
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
  for (int a = 0; a < N; ++a) c32[a] = (float)c[a];
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
__global__ __launch_bounds__(kSweepThreads) void bpdq_group_kernel(
    const float* __restrict__ Wp, int ldw, int d_out, const float* __restrict__ U, int ldu, int s0,
    int T, float alpha, unsigned char* __restrict__ cand_codes, float* __restrict__ cand_coef,
    float* __restrict__ cand_E, double* __restrict__ cand_score) {
  constexpr int CPL = G / 16;
  extern __shared__ float lds[];
  float* sU = lds;                 // [G][16][CPL], zero on and below the diagonal
  float* sInv = lds + G * G;       // 1 / U_ll
  double* sScore = reinterpret_cast<double*>(lds + G * G + G);
  const int tid = threadIdx.x;
  const int lane16 = tid & 15;
  for (int e = tid; e < G * G; e += kSweepThreads) {
    const int l = e / G, j = e % G;
    const float v = U[(long)(s0 + l) * ldu + s0 + j];
    sU[l * G + (j & 15) * CPL + (j >> 4)] = (j > l) ? v : 0.f;
    if (j == l) sInv[l] = 1.0f / v;
  }
  __syncthreads();

  const int row = blockIdx.x * kRowsPerWG + (tid >> 4);
  const bool valid = row < d_out;
  const int rr = valid ? row : d_out - 1;
  RowState<K, G> st;
  const float* wrow = Wp + (long)rr * ldw + s0;
#pragma unroll
  for (int m = 0; m < CPL; ++m) st.t[m] = wrow[16 * m + lane16];

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
  run_columns<K, G, false>(st, sU, sInv, lv, lane16, Seq{});

  const int n_wg = gridDim.x;
  float c32[K + 1], Ep[CPL];
  double rs = fit_and_score<K, G>(st, (double)alpha, c32, Ep);
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
    run_columns<K, G, true>(st, sU, sInv, lv, lane16, Seq{});
    rs = fit_and_score<K, G>(st, (double)alpha, c32, Ep);
    store_candidate<K, G>(st, c32, Ep, rs, it, row, valid, d_out, n_wg, cand_codes, cand_coef,
                          cand_E, cand_score, sScore, lane16);
  }
}

// Sum the row-block scores of every iterate in a fixed order and keep the earliest minimum.
__global__ __launch_bounds__(256) void select_iterate_kernel(const double* __restrict__ score,
                                                             int n_wg, int T, double* grp_err,
                                                             int* grp_iter) {
  __shared__ double red[256];
  __shared__ double tot[64];
  for (int it = 0; it <= T; ++it) {
    double s = 0.0;
    for (int q = threadIdx.x; q < n_wg; q += 256) s += score[(long)it * n_wg + q];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) tot[it] = red[0];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    int best = 0;
    for (int it = 1; it <= T; ++it)
      if (tot[it] < tot[best]) best = it;
    *grp_iter = best;
    *grp_err = tot[best];
  }
}

// Write the kept iterate: packed planes, coefficients, What, and E* transposed into the
// block's K-major error buffer Eblk[(s0 - b0) + j][row] (leading dimension lde).
template <int K, int G>
__global__ __launch_bounds__(256) void commit_group_kernel(
    const unsigned char* __restrict__ cand_codes, const float* __restrict__ cand_coef,
    const float* __restrict__ cand_E, const int* __restrict__ grp_iter, int d_out, int d_in,
    int s0, int b0, uint32_t* __restrict__ planes, float* __restrict__ coefs,
    float* __restrict__ W_hat, float* __restrict__ Eblk, int lde) {
  __shared__ float sE[G][65];
  const int it = *grp_iter;
  const int row0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
  const int n_grp = d_in / G, gi = s0 / G, n_word = d_in / 32;
  constexpr int WPG = G / 32;
  for (int idx = tid; idx < 64 * WPG; idx += 256) {
    const int r = row0 + idx / WPG, w = idx % WPG;
    if (r >= d_out) continue;
    const unsigned char* cp = cand_codes + ((long)it * d_out + r) * G + 32 * w;
    const float* cf = cand_coef + ((long)it * d_out + r) * (K + 1);
    float c[K + 1], lv[1 << K];
#pragma unroll
    for (int i = 0; i <= K; ++i) c[i] = cf[i];
    level_table<K>(c, lv);
    uint32_t word[K];
#pragma unroll
    for (int i = 0; i < K; ++i) word[i] = 0u;
    for (int j = 0; j < 32; ++j) {
      const int code = cp[j];
#pragma unroll
      for (int i = 0; i < K; ++i) word[i] |= (uint32_t)((code >> i) & 1) << j;
      if (W_hat) {
        float v = lv[0];
#pragma unroll
        for (int q = 1; q < (1 << K); ++q) v = (code == q) ? lv[q] : v;
        W_hat[(long)r * d_in + s0 + 32 * w + j] = v;
      }
    }
#pragma unroll
    for (int i = 0; i < K; ++i) planes[((long)i * d_out + r) * n_word + s0 / 32 + w] = word[i];
  }
  for (int idx = tid; idx < 64 * (K + 1); idx += 256) {
    const int r = row0 + idx / (K + 1), i = idx % (K + 1);
    if (r < d_out) coefs[((long)i * d_out + r) * n_grp + gi] = cand_coef[((long)it * d_out + r) * (K + 1) + i];
  }
  for (int idx = tid; idx < 64 * G; idx += 256) {
    const int r = idx / G, j = idx % G;
    sE[j][r] = (row0 + r < d_out) ? cand_E[((long)it * d_out + row0 + r) * G + j] : 0.f;
  }
  __syncthreads();
  for (int idx = tid; idx < 64 * G; idx += 256) {
    const int j = idx / 64, r = idx % 64;
    Eblk[(long)(s0 - b0 + j) * lde + row0 + r] = sE[j][r];
  }
}

// W'[:, c_begin:c_end] -= Et^T * U[k0:k0+Kd, c_begin:c_end]   (Eq. 4 applied to a whole block:
// the lazy update of the columns not yet quantized; also the rest-of-block update when g < B)
__global__ __launch_bounds__(TailGemm::kThreads) void tail_update_kernel(
    const float* __restrict__ Et, int lde, int Kd, const float* __restrict__ U, int ldu, int k0,
    float* __restrict__ Wp, int ldw, int d_out, int c_begin, int c_end, int tiles_n) {
  const int tm = blockIdx.x / tiles_n, tn = blockIdx.x % tiles_n;
  TailGemm::Acc acc;
  TailGemm::zero(acc);
  TailGemm::run<false>(Et, lde, tm * TailGemm::kTileM, lde, U + (long)k0 * ldu, ldu,
                       c_begin + tn * TailGemm::kTileN, c_end, 0, Kd, acc);
  const int r0 = tm * TailGemm::kTileM, c0 = c_begin + tn * TailGemm::kTileN;
  TailGemm::for_each(acc, [&](int row, int col, float v) {
    const int r = r0 + row, c = c0 + col;
    if (r < d_out && c < c_end) Wp[(long)r * ldw + c] -= v;
  });
}

// working copy of W with dead input channels zeroed
__global__ __launch_bounds__(256) void copy_in_kernel(const float* __restrict__ W, long n, int d_in,
                                                      const unsigned char* __restrict__ dead,
                                                      float* __restrict__ Wp) {
  for (long e = ((long)blockIdx.x * 256 + threadIdx.x) * 4; e < n; e += (long)gridDim.x * 1024) {
    float4 v = *reinterpret_cast<const float4*>(W + e);
    if (dead) {
      const int c = (int)(e % d_in);
      if (dead[c]) v.x = 0.f;
      if (dead[c + 1]) v.y = 0.f;
      if (dead[c + 2]) v.z = 0.f;
      if (dead[c + 3]) v.w = 0.f;
    }
    *reinterpret_cast<float4*>(Wp + e) = v;
  }
}

// ------------------------------------------------------------------ storage helpers --------
__global__ __launch_bounds__(256) void pack_planes_kernel(const unsigned char* __restrict__ codes,
                                                          int d_out, int d_in, int bits,
                                                          uint32_t* __restrict__ planes) {
  const int n_word = d_in / 32;
  const long n = (long)d_out * n_word;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const unsigned char* cp = codes + e * 32;
    uint32_t word[4] = {0u, 0u, 0u, 0u};
    for (int j = 0; j < 32; ++j) {
      const int code = cp[j];
#pragma unroll
      for (int i = 0; i < 4; ++i) word[i] |= (uint32_t)((code >> i) & 1) << j;
    }
    for (int i = 0; i < bits; ++i) planes[(long)i * n + e] = word[i];
  }
}

__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t* __restrict__ planes,
                                                      const float* __restrict__ coefs, int d_out,
                                                      int d_in, int bits, int group,
                                                      float* __restrict__ W_hat) {
  const int n_word = d_in / 32, n_grp = d_in / group;
  const long n = (long)d_out * d_in;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const int r = (int)(e / d_in), c = (int)(e % d_in);
    const int gi = c / group;
    float v = coefs[(long)r * n_grp + gi];
    for (int i = 0; i < bits; ++i) {
      const uint32_t w = planes[((long)i * d_out + r) * n_word + c / 32];
      if ((w >> (c & 31)) & 1u) v = v + coefs[((long)(i + 1) * d_out + r) * n_grp + gi];
    }
    W_hat[e] = v;
  }
}

// ------------------------------------------------------------------ host side --------------
struct QuantLayout {
  size_t wp_off, eblk_off, codes_off, coef_off, e_off, score_off, total;
  int B, lde, n_wg;
};

static QuantLayout quant_layout(int d_out, int d_in, const bpdq_params& p) {
  QuantLayout L;
  const int g = p.group, T = p.refine_iters, K = p.bits;
  L.B = p.block > g ? p.block : g;
  L.lde = (int)bpdq_align_up((size_t)d_out, 64);
  L.n_wg = bpdq_ceil_div(d_out, kRowsPerWG);
  size_t off = 0;
  L.wp_off = off;    off += bpdq_align_up((size_t)d_out * d_in * sizeof(float), 256);
  L.eblk_off = off;  off += bpdq_align_up((size_t)L.B * L.lde * sizeof(float), 256);
  L.codes_off = off; off += bpdq_align_up((size_t)(T + 1) * d_out * g, 256);
  L.coef_off = off;  off += bpdq_align_up((size_t)(T + 1) * d_out * (K + 1) * sizeof(float), 256);
  L.e_off = off;     off += bpdq_align_up((size_t)(T + 1) * d_out * g * sizeof(float), 256);
  L.score_off = off; off += bpdq_align_up((size_t)(T + 1) * L.n_wg * sizeof(double), 256);
  L.total = off;
  return L;
}

static int check_params(int d_out, int d_in, const bpdq_params* p) {
  if (!p) return 1;
  if (p->bits < 1 || p->bits > 4) return 1;
  if (p->group != 32 && p->group != 64 && p->group != 128) return 1;
  if (d_in % p->group || d_in % 32) return 1;
  const int B = p->block > p->group ? p->block : p->group;
  if (p->block < 1 || B % p->group) return 1;
  if (p->refine_iters < 0 || p->refine_iters > 63) return 1;
  if (!(p->alpha >= 0.f)) return 1;
  if (p->select_per_row != 0) return 1;
  if (d_out <= 0 || d_in <= 0) return 1;
  return 0;
}

template <int K, int G>
static int launch_group(hipStream_t stream, const float* Wp, int d_out, int d_in, const float* U,
                        int s0, int b0, const bpdq_params& p, const QuantLayout& L, char* base,
                        uint32_t* planes, float* coefs, float* W_hat, double* grp_err,
                        int* grp_iter) {
  unsigned char* c_codes = reinterpret_cast<unsigned char*>(base + L.codes_off);
  float* c_coef = reinterpret_cast<float*>(base + L.coef_off);
  float* c_E = reinterpret_cast<float*>(base + L.e_off);
  double* c_score = reinterpret_cast<double*>(base + L.score_off);
  float* Eblk = reinterpret_cast<float*>(base + L.eblk_off);
  const size_t lds = (size_t)(G * G + G) * sizeof(float) + kRowsPerWG * sizeof(double);
  static bool attr_set = false;
  if (!attr_set) {
    BPDQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(bpdq_group_kernel<K, G>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  const int gi = s0 / G;
  hipLaunchKernelGGL((bpdq_group_kernel<K, G>), dim3(L.n_wg), dim3(kSweepThreads), lds, stream, Wp,
                     d_in, d_out, U, d_in, s0, p.refine_iters, p.alpha, c_codes, c_coef, c_E, c_score);
  BPDQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(select_iterate_kernel, dim3(1), dim3(256), 0, stream, c_score, L.n_wg,
                     p.refine_iters, grp_err + gi, grp_iter + gi);
  BPDQ_LAUNCH_CHECK();
  hipLaunchKernelGGL((commit_group_kernel<K, G>), dim3(L.lde / 64), dim3(256), 0, stream, c_codes,
                     c_coef, c_E, grp_iter + gi, d_out, d_in, s0, b0, planes, coefs, W_hat, Eblk,
                     L.lde);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

typedef int (*GroupLauncher)(hipStream_t, const float*, int, int, const float*, int, int,
                             const bpdq_params&, const QuantLayout&, char*, uint32_t*, float*,
                             float*, double*, int*);

template <int K>
static GroupLauncher pick_group_g(int g) {
  switch (g) {
    case 32: return launch_group<K, 32>;
    case 64: return launch_group<K, 64>;
    case 128: return launch_group<K, 128>;
  }
  return nullptr;
}
static GroupLauncher pick_group(int k, int g) {
  switch (k) {
    case 1: return pick_group_g<1>(g);
    case 2: return pick_group_g<2>(g);
    case 3: return pick_group_g<3>(g);
    case 4: return pick_group_g<4>(g);
  }
  return nullptr;
}

static int launch_tail_update(hipStream_t stream, const float* Et, int lde, int Kd, const float* U,
                              int d_in, int k0, float* Wp, int d_out, int c_begin, int c_end) {
  if (c_end <= c_begin) return 0;
  static bool attr_set = false;
  if (!attr_set) {
    BPDQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(tail_update_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)TailGemm::kLdsBytes));
    attr_set = true;
  }
  const int tiles_m = bpdq_ceil_div(lde, TailGemm::kTileM);
  const int tiles_n = bpdq_ceil_div(c_end - c_begin, TailGemm::kTileN);
  hipLaunchKernelGGL(tail_update_kernel, dim3(tiles_m * tiles_n), dim3(TailGemm::kThreads),
                     TailGemm::kLdsBytes, stream, Et, lde, Kd, U, d_in, k0, Wp, d_in, d_out, c_begin, c_end, tiles_n);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

}  // namespace bpdq

using namespace bpdq;

extern "C" int bpdq_version(void) { return 100; }

extern "C" size_t bpdq_quantize_workspace_bytes(int d_out, int d_in, const bpdq_params* p) {
  if (check_params(d_out, d_in, p)) return 0;
  return quant_layout(d_out, d_in, *p).total;
}

extern "C" int bpdq_quantize_layer(const float* W, int d_out, int d_in, const float* U,
                                   const unsigned char* dead, const bpdq_params* p,
                                   uint32_t* planes, float* coefs, float* W_hat, double* grp_err,
                                   int* grp_iter, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!W || (reinterpret_cast<uintptr_t>(W) & 15)) return -1;
  if (d_out <= 0) return -2;
  if (d_in <= 0 || d_in % 32) return -3;
  if (!U || (reinterpret_cast<uintptr_t>(U) & 15)) return -4;
  if (check_params(d_out, d_in, p)) return -6;
  if (!planes) return -7;
  if (!coefs) return -8;
  if (!grp_err) return -10;
  if (!grp_iter) return -11;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return -12;
  const QuantLayout L = quant_layout(d_out, d_in, *p);
  if (ws_bytes < L.total) return -13;
  char* base = static_cast<char*>(ws);
  float* Wp = reinterpret_cast<float*>(base + L.wp_off);
  float* Eblk = reinterpret_cast<float*>(base + L.eblk_off);
  GroupLauncher group = pick_group(p->bits, p->group);
  if (!group) return -6;

  const long n = (long)d_out * d_in;
  const int grid = (int)((n / 4 + 255) / 256 < 65536 ? (n / 4 + 255) / 256 : 65536);
  hipLaunchKernelGGL(copy_in_kernel, dim3(grid), dim3(256), 0, stream, W, n, d_in, dead, Wp);
  BPDQ_LAUNCH_CHECK();

  const int g = p->group, B = L.B;
  for (int b0 = 0; b0 < d_in; b0 += B) {
    const int b1 = b0 + B < d_in ? b0 + B : d_in;
    for (int s0 = b0; s0 < b1; s0 += g) {
      int rc = group(stream, Wp, d_out, d_in, U, s0, b0, *p, L, base, planes, coefs, W_hat,
                     grp_err, grp_iter);
      if (rc) return rc;
      // rest of this block (only when g < B): W'[:, s0+g:b1] -= E* U[s0:s0+g, s0+g:b1]
      rc = launch_tail_update(stream, Eblk + (long)(s0 - b0) * L.lde, L.lde, g, U, d_in, s0, Wp,
                              d_out, s0 + g, b1);
      if (rc) return rc;
    }
    // lazy block update of every later column
    const int rc = launch_tail_update(stream, Eblk, L.lde, b1 - b0, U, d_in, b0, Wp, d_out, b1, d_in);
    if (rc) return rc;
  }
  return 0;
}

extern "C" int bpdq_pack_planes(const unsigned char* codes, int d_out, int d_in, int bits,
                                uint32_t* planes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!codes) return -1;
  if (d_out <= 0) return -2;
  if (d_in <= 0 || d_in % 32) return -3;
  if (bits < 1 || bits > 4) return -4;
  if (!planes) return -5;
  const long n = (long)d_out * (d_in / 32);
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(pack_planes_kernel, dim3(grid), dim3(256), 0, stream, codes, d_out, d_in, bits, planes);
  BPDQ_LAUNCH_CHECK();
  return 0;
}

extern "C" int bpdq_dequant(const uint32_t* planes, const float* coefs, int d_out, int d_in,
                            int bits, int group, float* W_hat, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!planes) return -1;
  if (!coefs) return -2;
  if (d_out <= 0) return -3;
  if (d_in <= 0 || d_in % 32) return -4;
  if (bits < 1 || bits > 4) return -5;
  if (group <= 0 || d_in % group) return -6;
  if (!W_hat) return -7;
  const long n = (long)d_out * d_in;
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(dequant_kernel, dim3(grid), dim3(256), 0, stream, planes, coefs, d_out, d_in,
                     bits, group, W_hat);
  BPDQ_LAUNCH_CHECK();
  return 0;
}
