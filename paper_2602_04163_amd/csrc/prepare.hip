// Step 2 of the pass: damping and U = chol(H^-1), H^-1 = U^T U with U upper triangular
// (paper Sec. 3.1, "Quantization Error Compensation").
//
// Route: with Ht = H + lambda I, factor Ht = R R^T with R UPPER triangular (a Cholesky
// factorisation that runs from the last column to the first).  Then
// Ht^-1 = R^-T R^-1 = (R^-1)^T (R^-1), so U = R^-1: one factorisation plus one triangular
// inverse (2/3 d^3 flops) and Ht^-1 is never formed.  Everything runs in fp64 inside the
// workspace; the result is rounded to fp32 once, on output.
//
//   factor : right-looking over 64-column panels from the right, two panels per launch: every
//            panel work-group factors the two diagonal blocks for itself (in LDS, by panels of
//            16 columns) and solves its 64 rows of R12 R22^T = A12.  The trailing update
//            A11 -= R12 R12^T (fp64 MFMA) is two-level: after each panel pair only inside the
//            current 512-column outer block (64 x 64 tiles), and once per outer block, with
//            K = 512, on everything to its left (128 x 128 tiles fed by LDS-DMA from 4096
//            columns on).
//   invert : divide and conquer over block ranges, [R11 R12; 0 R22]^-1 =
//            [U11, -U11 R12 U22; 0, U22]; every tree level is two launches (128 x 128 tiles
//            where a level has enough of them, 64 x 64 otherwise).
#include "common.h"

namespace bpdq {

constexpr int NB = 64;    // panel / tile size (fp64)

// ---------------------------------------------------------------- damping ------------------
// One work-group: dead flags, mean of the (fixed) diagonal, lambda.  scal[0] = lambda.
__global__ __launch_bounds__(1024) void prep_diag_kernel(const float* __restrict__ H, int d,
                                                         float damp, unsigned char* __restrict__ dead,
                                                         double* __restrict__ scal, int* info) {
  __shared__ double red[1024];
  double s = 0.0;
  for (int i = threadIdx.x; i < d; i += 1024) {
    float h = H[(long)i * d + i];
    const bool dd = (h == 0.f);
    if (dead) dead[i] = dd ? 1 : 0;
    s += dd ? 1.0 : (double)h;
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    scal[0] = (double)damp * (red[0] / (double)d);
    *info = 0;
  }
}

// A (fp64, d x d) <- upper triangle of H with the diagonal fixed and damped; lower part 0.
__global__ __launch_bounds__(256) void prep_load_kernel(const float* __restrict__ H, int d,
                                                        const double* __restrict__ scal,
                                                        double* __restrict__ A) {
  const long n = (long)d * d;
  const double lam = scal[0];
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const int i = (int)(e / d), j = (int)(e % d);
    double v = 0.0;
    if (j >= i) {
      const float h = H[e];
      v = (double)h;
      if (i == j) v = (h == 0.f ? 1.0 : v) + lam;
    }
    A[e] = v;
  }
}

// ---------------------------------------------------------------- factor -------------------
// 1 / x in fp64: hardware estimate (about 2^-27 relative) + one Newton step (about 2^-52): the
// pivot reciprocal sits on the critical path of every column step, where every dependent fp64
// operation costs tens of cycles; an error of an ulp or two in it is far below the fp32 rounding
// of H and of the result.
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = fma(fma(-x, r, 1.0), r, r);
  return r;
}

// A 64 x 64 tile of doubles moves between global memory and LDS through registers, 16 elements
// per thread of 256 (element e = tid + 256 t -> row e / 64, column e % 64).  All 16 loads of a
// thread are issued before the first is used: a rolled loop would wait for memory 16 times.
// ok(i, j): is the element read (else 0);  idx(i, j): its offset from `base`, which must itself
// be a valid address (masked elements read base[0] and discard it).
template <typename OK, typename IDX>
__device__ __forceinline__ void fetch_tile64(const double* __restrict__ base, OK ok, IDX idx,
                                             double (&v)[16]) {
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const int e = threadIdx.x + 256 * t;
    const int i = e >> 6, j = e & 63;
    const bool in = ok(i, j);
    const double x = base[in ? idx(i, j) : 0L];
    v[t] = in ? x : 0.0;
  }
}
template <typename ROW>
__device__ __forceinline__ void put_tile64(ROW* s, const double (&v)[16]) {
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const int e = threadIdx.x + 256 * t;
    s[e >> 6][e & 63] = v[t];
  }
}

typedef double f64x4 __attribute__((ext_vector_type(4)));

// Reversed Cholesky of one 64 x 64 block held in LDS: D = R R^T, R upper, columns taken from the
// last to the first, in panels of 16 columns.
//   in : sD, the full symmetric block (both triangles; identity padding where the block is ragged)
//   out: sD = R (zero below the diagonal), sInvD[j] = 1 / R_jj
// A panel is factored by ONE wavefront, lane r holding row r of its 16 columns in registers: a
// column step writes the pivot column to LDS and reads the pivot and the (at most 15) entries it
// needs back as broadcasts -- LDS serves one wavefront in order, so no barrier is involved -- then
// updates only the panel's columns left of the pivot.  The other columns of the block receive the
// panel's rank-16 update afterwards on the fp64 matrix cores (all four wavefronts).  Against a
// column step that updates the whole block (16 multiply-adds per thread of 256 behind a barrier)
// the dependent chain per column is a third as long.  Square roots are taken once, at the end.
// A non-positive pivot is reported as column p0 + j + 1 (by the work-group with `report`) and
// replaced by 1.  All 256 threads call this; sCol and sPiv are 64 doubles each.
template <int JL>
__device__ __forceinline__ void factor_panel_step(double (&pa)[16], double* sCol, double* sPiv, int c0,
                                                  int lane, int* info, int p0, bool report) {
  sCol[lane] = pa[JL];
  const double piv_raw = sCol[c0 + JL];
  double cc[JL > 0 ? JL : 1];
#pragma unroll
  for (int e = 0; e < JL; ++e) cc[e] = sCol[c0 + e];
  const bool bad = !(piv_raw > 0.0);
  const double piv = bad ? 1.0 : piv_raw;
  const double t = pa[JL] * fast_rcp(piv);
#pragma unroll
  for (int e = 0; e < JL; ++e) pa[e] = fma(-t, cc[e], pa[e]);
  if (lane == 0) {
    sPiv[c0 + JL] = piv;
    if (bad && report) atomicCAS(info, 0, p0 + c0 + JL + 1);
  }
  if constexpr (JL > 0) factor_panel_step<JL - 1>(pa, sCol, sPiv, c0, lane, info, p0, report);
}

__device__ __forceinline__ void factor64_blocked(double (*sD)[NB + 1], double* sCol, double* sPiv,
                                                 double* sInvD, int* info, int p0, bool report) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
#pragma unroll 1
  for (int J = NB / 16 - 1; J >= 0; --J) {
    const int c0 = 16 * J;
    __syncthreads();                        // the block, with every earlier panel's update, is in LDS
    if (w == 0) {
      double pa[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) pa[e] = sD[lane][c0 + e];
      factor_panel_step<15>(pa, sCol, sPiv, c0, lane, info, p0, report);
#pragma unroll
      for (int e = 0; e < 16; ++e) sD[lane][c0 + e] = (lane <= c0 + e) ? pa[e] : 0.0;   // unscaled columns of R
    }
    __syncthreads();
    // leading block [0, c0) x [0, c0), upper 16 x 16 tiles:  -= Rp diag(1 / pivot) Rp^T
    const int m = lane & 15, kq = lane >> 4;
    int t = 0;
    for (int tk = 0; tk < J; ++tk)
      for (int ti = 0; ti <= tk; ++ti, ++t) {
        if ((t & 3) != w) continue;
        f64x4 acc = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int kk = c0 + 4 * ks + kq;
          const double a = sD[16 * ti + m][kk] * fast_rcp(sPiv[kk]);
          const double b = sD[16 * tk + m][kk];
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) sD[16 * ti + 4 * r + kq][16 * tk + m] -= acc[r];
      }
  }
  __syncthreads();
  if (tid < NB) sInvD[tid] = 1.0 / sqrt(sPiv[tid]);
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    sD[i][j] = (i <= j) ? sD[i][j] * sInvD[j] : 0.0;          // R[:, j] = column_j / sqrt(pivot_j)
  }
  __syncthreads();
}


// Inverses of the four 16 x 16 diagonal blocks of R (upper triangular, sInvD[j] = 1 / R_jj):
// sRinv[J][i][c] = (R_JJ^-1)[i][c], zero below the diagonal.  Wavefront J takes block J, lane
// c < 16 column c by back substitution from row 15 up (rows below c are zero, row c is 1 / R_cc).
// All 256 threads call this; it ends with a barrier.
typedef double Inv16[16][16];
__device__ __forceinline__ void invert_diag16(const double (*sR)[NB + 1], const double* sInvD, Inv16* sRinv) {
  const int lane = threadIdx.x & 63, J = threadIdx.x >> 6;
  if (lane < 16) {
    const int c = lane, o = 16 * J;
    double x[16];
#pragma unroll
    for (int i = 15; i >= 0; --i) {
      double acc = 0.0;
#pragma unroll
      for (int m = 15; m > i; --m) acc = fma(sR[o + i][o + m], x[m], acc);   // (x[m] = 0 for m > c) the newest x last:
                                                                             // only that term waits for the row before
      const double v = (i == c) ? 1.0 : -acc;
      x[i] = (i <= c) ? v * sInvD[o + i] : 0.0;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) sRinv[J][i][c] = x[i];
  }
  __syncthreads();
}

// X R^T = A for one or two 64 x 64 tiles at once, in place, by blocks of 16 columns from the
// right (R upper, sRinv = inverses of its 16 x 16 diagonal blocks), all on the fp64 matrix cores
// (v_mfma_f64_16x16x4_f64):
//   (1) X_J = A_J R_JJ^-T;
//   (2) the blocks to its left receive  A_J' -= X_J R[J', J]^T.
// Wavefront w takes rows 16 w .. 16 w + 15 of both tiles through all four blocks; a row block
// never meets another one's data, so there is no barrier inside and no dependent substitution
// chain: against a column-by-column substitution inside each block (one lane per row, 120 LDS
// broadcasts per block) a solve takes 2 us instead of 7.
// All 256 threads call this; it ends with a barrier.
// One block step for TILES tiles at once (their chains of dependent matrix instructions
// interleave): X_J = A_J R_JJ^-T, then A_J' -= X_J R[J', J]^T for every J' < J.
template <int J, int TILES>
__device__ __forceinline__ void trsm_block_step(double (*const (&sX)[2])[NB + 1], const double (*sR)[NB + 1],
                                                const Inv16* sRinv) {
  const int lane = threadIdx.x & 63, i0 = 16 * (threadIdx.x >> 6);
  const int lm = lane & 15, lq = lane >> 4;
  double a[TILES][4], b[4];
  f64x4 acc[TILES];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    b[ks] = sRinv[J][lm][4 * ks + lq];                                             // B[k][n] = Rinv[n][k]
#pragma unroll
    for (int t = 0; t < TILES; ++t) a[t][ks] = sX[t][i0 + lm][16 * J + 4 * ks + lq];   // A[m][k] = A_J
  }
#pragma unroll
  for (int t = 0; t < TILES; ++t) acc[t] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int t = 0; t < TILES; ++t) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[t][ks], b[ks], acc[t], 0, 0, 0);
#pragma unroll
  for (int t = 0; t < TILES; ++t)
#pragma unroll
    for (int r = 0; r < 4; ++r) sX[t][i0 + 4 * r + lq][16 * J + lm] = acc[t][r];   // D[4r + l/16][l%16]
  if constexpr (J > 0) {
    // X_J back in operand layout (this wavefront's own rows: LDS serves a wavefront in order)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int t = 0; t < TILES; ++t) a[t][ks] = sX[t][i0 + lm][16 * J + 4 * ks + lq];
    f64x4 upd[J][TILES];
#pragma unroll
    for (int Jp = 0; Jp < J; ++Jp) {
      double br[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) br[ks] = sR[16 * Jp + lm][16 * J + 4 * ks + lq];   // B[k][n] = R[J'n][Jk]
#pragma unroll
      for (int t = 0; t < TILES; ++t) upd[Jp][t] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int t = 0; t < TILES; ++t)
          upd[Jp][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[t][ks], br[ks], upd[Jp][t], 0, 0, 0);
    }
#pragma unroll
    for (int Jp = 0; Jp < J; ++Jp)
#pragma unroll
      for (int t = 0; t < TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) sX[t][i0 + 4 * r + lq][16 * Jp + lm] -= upd[Jp][t][r];
    trsm_block_step<J - 1, TILES>(sX, sR, sRinv);
  }
}

__device__ __forceinline__ void trsm64_blocked(double (*sXa)[NB + 1], double (*sXb)[NB + 1], bool two,
                                               const double (*sR)[NB + 1], const Inv16* sRinv) {
  double (*const tiles[2])[NB + 1] = {sXa, sXb};
  if (two) trsm_block_step<NB / 16 - 1, 2>(tiles, sR, sRinv);
  else trsm_block_step<NB / 16 - 1, 1>(tiles, sR, sRinv);
  __syncthreads();
}

// The symmetric 64 x 64 block at (p0, p0), both triangles (only the upper triangle of A is valid),
// identity padding beyond nb: 16 elements per thread in the order of fetch_tile64 / put_tile64.
__device__ __forceinline__ void fetch_diag_block(const double* __restrict__ A, int d, int p0, int nb,
                                                 double (&v)[16]) {
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const int e = threadIdx.x + 256 * t;
    const int i = e >> 6, j = e & 63;
    const bool in = i < nb && j < nb;
    const int lo = i < j ? i : j, hi = i < j ? j : i;
    const double x = A[in ? (long)(p0 + lo) * d + p0 + hi : 0L];
    v[t] = in ? x : ((i == j) ? 1.0 : 0.0);
  }
}

// Panel step of the reversed Cholesky for ONE 64-column panel, one work-group (256 threads) per
// 64 rows of the panel.
//   (1) every work-group factors the 64 x 64 diagonal block for itself (factor64);
//   (2) rows [64 b, 64 b + 64) of the panel above the block: X R^T = A12, one thread per row.
// Work-group 0 also writes R of the diagonal block to Rdiag (NB x NB, row-major, zero below the
// diagonal, identity-padded), clears the block's pair flag and reports a non-positive pivot.
// Launch with max(p, 1) work-groups, p = number of 64-row blocks above the diagonal block.
__global__ __launch_bounds__(256) void panel_factor_kernel(double* __restrict__ A, int d, int p0,
                                                           int nb, int n_above,
                                                           double* __restrict__ Rdiag,
                                                           int* __restrict__ pair_flag, int* info) {
  __shared__ double sR[NB][NB + 1];     // R (upper) of the diagonal block
  __shared__ double sA[NB][NB + 1];     // panel tile of this work-group
  __shared__ double col[2][NB];
  __shared__ double sInvD[NB];
  __shared__ Inv16 sRinv[NB / 16];
  const int tid = threadIdx.x;

  {
    double v[16];
    fetch_diag_block(A, d, p0, nb, v);
    put_tile64(sR, v);
  }
  // panel tile (coalesced), used after the factorisation
  const int r0 = blockIdx.x * NB;
  if (n_above > 0) {
    double v[16];
    fetch_tile64(A, [&](int i, int j) { return r0 + i < p0 && j < nb; },
                 [&](int i, int j) { return (long)(r0 + i) * d + p0 + j; }, v);
    put_tile64(sA, v);
  }
  factor64_blocked(sR, col[0], col[1], sInvD, info, p0, blockIdx.x == 0);
  // R of the diagonal block goes to its own buffer: the block itself must stay untouched, because
  // work-groups of this launch that start later still have to read it
  if (blockIdx.x == 0) {
    for (int e = tid; e < NB * NB; e += 256) Rdiag[e] = sR[e / NB][e % NB];
    if (tid == 0) *pair_flag = 0;
  }
  if (n_above == 0) return;
  invert_diag16(sR, sInvD, sRinv);
  trsm64_blocked(sA, sA, false, sR, sRinv);
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    if (r0 + i < p0 && j < nb) A[(long)(r0 + i) * d + p0 + j] = sA[i][j];
  }
}

// Inverses of all diagonal blocks of R at once (one work-group per block, thread c < 64 solves
// R x = e_c by back substitution); the inverse replaces the diagonal block of A (upper part,
// zeros below), which until now still held the unfactored block.  A block that was the second of
// a panel pair also brings its R12 (rows of the block before it) from the side buffer into A.
__global__ __launch_bounds__(256) void diag_inverse_kernel(const double* __restrict__ Rdiag,
                                                           const double* __restrict__ R12buf,
                                                           const int* __restrict__ pair_flag,
                                                           double* __restrict__ A, int d) {
  __shared__ double s[NB][NB + 1];
  __shared__ double x[NB][NB + 1];
  const int p0 = blockIdx.x * NB;
  const int nb = (d - p0 < NB) ? d - p0 : NB;
  const int tid = threadIdx.x;
  const double* src = Rdiag + (long)blockIdx.x * NB * NB;
  const bool pair = pair_flag[blockIdx.x] != 0;
  {
    double v[16], r12[16];
    fetch_tile64(src, [](int, int) { return true; }, [](int i, int j) { return (long)i * NB + j; }, v);
    if (pair)
      fetch_tile64(R12buf + (long)blockIdx.x * NB * NB, [](int, int) { return true; },
                   [](int i, int j) { return (long)i * NB + j; }, r12);
    put_tile64(s, v);
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const int e = tid + 256 * t;
      const int i = e >> 6, j = e & 63;
      x[i][j] = 0.0;
      if (pair && j < nb) A[(long)(p0 - NB + i) * d + p0 + j] = r12[t];
    }
  }
  __syncthreads();
  if (tid < NB) {
    const int c = tid;
    x[c][c] = 1.0 / s[c][c];
    for (int i = c - 1; i >= 0; --i) {
      double acc = 0.0;
      for (int m = i + 1; m <= c; ++m) acc += s[i][m] * x[m][c];
      x[i][c] = -acc / s[i][i];
    }
  }
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    if (i < nb && j < nb) A[(long)(p0 + i) * d + p0 + j] = (j >= i) ? x[i][j] : 0.0;
    // the block to the left of the diagonal one: the 128-tile products of the inversion read it as
    // part of a triangular operand, where it stands for zeros
    if (p0 > 0 && i < nb) A[(long)(p0 + i) * d + p0 - NB + j] = 0.0;
  }
}

// 64 x 64 x 64 fp64 product on the matrix cores for a 256-thread work-group: wavefront w owns
// the 32 x 32 quadrant (w / 2, w % 2) as 2 x 2 tiles of v_mfma_f64_16x16x4_f64.
//   A operand: lane l holds A[m = l % 16][k = l / 16];  B operand: B[k = l / 16][n = l % 16];
//   D: register r of lane l is D[4 * r + l / 16][l % 16].
// sa is [m][k]; sb is [k][n], or [n][k] when B_T (second operand given by rows, as in a SYRK).
// With the 65-double row pitch every 16-lane group reads 16 distinct bank pairs.
struct Quad64 {
  f64x4 c[2][2];
};

__device__ __forceinline__ void quad_zero(Quad64& q) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) q.c[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};
}

template <bool B_T>
__device__ __forceinline__ void quad_mfma_64(const double (*sa)[NB + 1], const double (*sb)[NB + 1],
                                             Quad64& q) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int m0 = (w >> 1) * 32 + (lane & 15), n0 = (w & 1) * 32 + (lane & 15);
  const int kq = lane >> 4;
#pragma unroll 4
  for (int k0 = 0; k0 < NB; k0 += 4) {
    const int k = k0 + kq;
    double a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = sa[m0 + 16 * i][k];
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = B_T ? sb[n0 + 16 * j][k] : sb[k][n0 + 16 * j];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        q.c[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], q.c[i][j], 0, 0, 0);
  }
}

// f(row, col, value) over this lane's 16 results, row / col inside the 64 x 64 tile
template <typename F>
__device__ __forceinline__ void quad_for_each(const Quad64& q, F f) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        f((w >> 1) * 32 + 16 * i + 4 * r + (lane >> 4), (w & 1) * 32 + 16 * j + (lane & 15),
          q.c[i][j][r]);
}

// Two adjacent 64-column panels -- block b1 (columns p1 ..) and block b2 = b1 + 1 -- in one
// launch, one work-group per 64 rows above them.  With the diagonal 128 x 128 block
// [D11 D12; D12^T D22] every work-group computes for itself
//     D22 = R22 R22^T,   R12 = D12 R22^-T,   D11 - R12 R12^T = R11 R11^T
// and for its own rows [A1 A2] of the two panels
//     X2 = A2 R22^-T,    X1 = (A1 - X2 R12^T) R11^-T.
// The two small products run on the fp64 matrix cores.  This halves the number of dependent
// launches of the panel chain (each is short and latency-bound).  Work-group 0 writes R11, R22
// to Rdiag and R12 to R12buf (never into A, whose blocks later-scheduled work-groups still
// read) and sets the pair flag of b2, so that the inverse step puts R12 in place.
constexpr size_t kPairLdsBytes = (size_t)(4 * NB * (NB + 1) + 3 * NB + NB * 16) * sizeof(double);

__global__ __launch_bounds__(256) void panel_pair_kernel(double* __restrict__ A, int d, int p1,
                                                         int nb2, int n_above,
                                                         double* __restrict__ Rdiag1,
                                                         double* __restrict__ Rdiag2,
                                                         double* __restrict__ R12buf,
                                                         int* __restrict__ pair_flag1,
                                                         int* __restrict__ pair_flag2, int* info) {
  extern __shared__ double dyn[];
  typedef double Row[NB + 1];
  Row* sR = reinterpret_cast<Row*>(dyn);            // R22, then R12 R12^T, then R11
  Row* sR12 = sR + NB;                              // D12 -> R12
  Row* sA1 = sR12 + NB;                             // own rows, columns of b1
  Row* sA2 = sA1 + NB;                              // own rows, columns of b2
  double (*col)[NB] = reinterpret_cast<double (*)[NB]>(dyn + 4 * NB * (NB + 1));
  double* sInvD = dyn + 4 * NB * (NB + 1) + 2 * NB;
  Inv16* sRinv = reinterpret_cast<Inv16*>(dyn + 4 * NB * (NB + 1) + 3 * NB);
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int p2 = p1 + NB;
  const int r0 = blockIdx.x * NB;
  const bool first = blockIdx.x == 0;

  double d11[16];                                   // D11, needed after the first factorisation
  fetch_diag_block(A, d, p1, NB, d11);
  {
    double v22[16], v12[16], v1[16], v2[16];
    fetch_diag_block(A, d, p2, nb2, v22);           // D22
    put_tile64(sR, v22);
    fetch_tile64(A, [&](int, int j) { return j < nb2; },
                 [&](int i, int j) { return (long)(p1 + i) * d + p2 + j; }, v12);
    if (n_above > 0) {
      fetch_tile64(A, [&](int i, int) { return r0 + i < p1; },
                   [&](int i, int j) { return (long)(r0 + i) * d + p1 + j; }, v1);
      fetch_tile64(A, [&](int i, int j) { return r0 + i < p1 && j < nb2; },
                   [&](int i, int j) { return (long)(r0 + i) * d + p2 + j; }, v2);
      put_tile64(sA1, v1);
      put_tile64(sA2, v2);
    }
    put_tile64(sR12, v12);
  }
  factor64_blocked(sR, col[0], col[1], sInvD, info, p2, first);
  if (first)
    for (int e = tid; e < NB * NB; e += 256) Rdiag2[e] = sR[e / NB][e % NB];
  // R12 = D12 R22^-T and X2 = A2 R22^-T
  invert_diag16(sR, sInvD, sRinv);                  // (its barrier: Rdiag2 has been read out of sR)
  trsm64_blocked(sR12, sA2, n_above > 0, sR, sRinv);
  {
    Quad64 q;
    quad_zero(q);
    quad_mfma_64<true>(sR12, sR12, q);              // R12 R12^T
    quad_for_each(q, [&](int r, int c, double v) { sR[r][c] = -v; });     // (R22 is no longer needed)
    if (n_above > 0) {
      quad_zero(q);
      quad_mfma_64<true>(sA2, sR12, q);             // X2 R12^T
      quad_for_each(q, [&](int r, int c, double v) { sA1[r][c] -= v; });
    }
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < 16; ++t) {                    // sR = D11 - R12 R12^T
    const int e = tid + 256 * t;
    sR[e >> 6][e & 63] += d11[t];
  }
  factor64_blocked(sR, col[0], col[1], sInvD, info, p1, first);
  if (first) {
    for (int e = tid; e < NB * NB; e += 256) {
      Rdiag1[e] = sR[e / NB][e % NB];
      R12buf[e] = sR12[e / NB][e % NB];
    }
    if (tid == 0) {
      *pair_flag1 = 0;
      *pair_flag2 = 1;
    }
  }
  if (n_above == 0) return;
  invert_diag16(sR, sInvD, sRinv);
  trsm64_blocked(sA1, sA1, false, sR, sRinv);
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    if (r0 + i < p1) {
      A[(long)(r0 + i) * d + p1 + j] = sA1[i][j];
      if (j < nb2) A[(long)(r0 + i) * d + p2 + j] = sA2[i][j];
    }
  }
}

// Trailing update with the panel columns [k0, k0 + Kd):  A[i][j] -= sum_k A[i][k] A[j][k]  on the
// upper 64 x 64 tiles (bi <= bj) whose block column bj lies in [cb0, cb1).  Used twice:
//   inner: after each 64-column panel, only for the block columns of the same outer panel that
//          are still to be factored (Kd = 64);
//   outer: once per outer panel, for everything to its left (Kd = outer width, up to 512), so
//          the big trailing matrix is read and written 8 times less often.
__global__ __launch_bounds__(256) void syrk_trailing_kernel(double* __restrict__ A, int d, int k0,
                                                            int Kd, int cb0, int cb1) {
  __shared__ double si[NB][NB + 1];
  __shared__ double sj[NB][NB + 1];
  int tile = blockIdx.x, bj = cb0;
  while (tile >= bj + 1) {
    tile -= bj + 1;
    ++bj;
  }
  const int bi = tile;
  const int tid = threadIdx.x;
  const int k_end = (k0 + Kd < d) ? k0 + Kd : d;
  Quad64 q;
  quad_zero(q);
  double vi[16], vj[16];
  auto fetch = [&](int kc) {
    fetch_tile64(A, [&](int, int k) { return kc + k < k_end; },
                 [&](int i, int k) { return (long)(bi * NB + i) * d + kc + k; }, vi);
    fetch_tile64(A, [&](int, int k) { return kc + k < k_end; },
                 [&](int i, int k) { return (long)(bj * NB + i) * d + kc + k; }, vj);
  };
  fetch(k0);
  for (int kc = k0; kc < k_end; kc += NB) {
    put_tile64(si, vi);
    put_tile64(sj, vj);
    __syncthreads();
    if (kc + NB < k_end) fetch(kc + NB);          // in flight during the products below
    quad_mfma_64<true>(si, sj, q);
    __syncthreads();
  }
  // read-modify-write of the 16 results of this lane, all loads first
  double old[16];
  int n = 0;
  quad_for_each(q, [&](int r, int c, double) {
    const int i = bi * NB + r, j = bj * NB + c;
    old[n++] = A[(j >= i) ? (long)i * d + j : 0L];
  });
  n = 0;
  quad_for_each(q, [&](int r, int c, double v) {
    const int i = bi * NB + r, j = bj * NB + c;
    if (j >= i) A[(long)i * d + j] = old[n] - v;
    ++n;
  });
}

// ---- fp64 products on 128 x 128 tiles, operands streamed to LDS by the DMA path -------------
// For the wide layers.  A 64 x 64 tile moves 2 x 64 operand rows per 64 x 64 results, which at
// the fp64 matrix rate is more than the caches deliver, and its loads pass through registers,
// whose address arithmetic and LDS writes sit between the matrix instructions.  Here 256 threads
// own 128 x 128 results, wavefront w the 64 x 64 quadrant (w / 2, w % 2) as 4 x 4 tiles of
// v_mfma_f64_16x16x4_f64, and both operands reach LDS in slices of 16 along K through the LDS-DMA
// path (global_load_lds_dwordx4: 64 lanes x 16 bytes land in 1 KB of LDS, no registers involved),
// double-buffered: the requests for slice s + 1 go out right behind the first operand reads of
// slice s.  64 KB of LDS and fewer than 256 registers: two work-groups per compute unit.
//
// LDS image of a slice of an operand given by rows ([row][k], k contiguous in memory): row r
// (128 bytes = 8 pairs of doubles) keeps pair p at position p ^ ((r / 2) % 8).  The DMA writes
// lane-linear, so the lane that fills position q of row r fetches pair q ^ ((r / 2) % 8).  An
// operand read (16 rows x one column per quarter wave) then touches 16 distinct bank pairs;
// unswizzled, rows 128 bytes apart would share two.
// LDS image of a slice of an operand given as [k][n] (n contiguous): k-row k (1 KB = 64 pairs)
// keeps pair c at position c ^ (8 (k % 2)), so that the two k-rows a half wave reads lie in
// different halves of the banks.
//
// Requirements (the launchers fall back to the 64-tile kernels otherwise): even leading
// dimensions and 16-byte aligned slices; K ranges that are multiples of 32.  Rows (columns) past
// an operand's limit are clamped to a valid one: their products land in results never stored.
constexpr int kGemmTile = 128;
constexpr int kGemmK = 16;
constexpr unsigned kGemmOpBytes = kGemmTile * kGemmK * sizeof(double);       // one operand slice
constexpr unsigned kGemmStageBytes = 2 * kGemmOpBytes;
constexpr size_t kGemmLdsBytes = 2 * kGemmStageBytes;

struct Acc128 {
  f64x4 c[4][4];
};

// 64 lanes x 16 bytes from gptr (per lane) to the 1 KB of LDS at byte address lds_addr (uniform,
// passed in M0, which these kernels use for nothing else).  One outstanding vector-memory operation.
__device__ __forceinline__ void dma_1k_f64(const double* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(gptr) : "memory");
}
__device__ __forceinline__ void wait_all_vm() {
  __builtin_amdgcn_s_waitcnt(0x0070 | 0x0f00);      // vmcnt 0; expcnt / lgkmcnt at their maxima
}

// DMA sources of wavefront w for slice 0 of an operand given by rows: rows [32 w, 32 w + 32) of the
// tile that starts at row0, 8 rows per request.
__device__ __forceinline__ void gemm128_row_sources(const double* base, long ld, int row0, int row_limit,
                                                    int k_begin, int w, int lane, const double* (&src)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = 32 * w + 8 * j + (lane >> 3);
    const int pair = (lane & 7) ^ ((r >> 1) & 7);
    const int g = (row0 + r < row_limit) ? row0 + r : row_limit - 1;
    src[j] = base + (long)g * ld + k_begin + 2 * pair;
  }
}
// ... of an operand given as [k][n]: k-rows [4 w, 4 w + 4) of the slice, columns [col0, col0 + 128)
__device__ __forceinline__ void gemm128_col_sources(const double* base, long ld, int k_begin, int col0,
                                                    int col_limit, int w, int lane, const double* (&src)[4]) {
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int pair = lane ^ ((j & 1) << 3);                    // (4 w + j) % 2 == j % 2
    const int col = (col0 + 2 * pair < col_limit) ? col0 + 2 * pair : col0;
    src[j] = base + (long)(k_begin + 4 * w + j) * ld + col;
  }
}

// q += A B over n_stage (even) slices.  B_ROWS: B is given by rows like A (C = A B^T, the SYRK
// form), else as [k][n].  step_a / step_b: elements between consecutive slices of a source.
template <bool B_ROWS>
__device__ __forceinline__ void gemm128_accumulate(const double* const (&src_a)[4], const double* const (&src_b)[4],
                                                   long step_a, long step_b, int n_stage, Acc128& q) {
  extern __shared__ __align__(16) double gemm128_lds[];
  typedef __attribute__((address_space(3))) double lds_f64;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned lds0 = (unsigned)(size_t)(lds_f64*)gemm128_lds;
  auto request = [&](int s) {
    const unsigned slot = lds0 + (unsigned)(s & 1) * kGemmStageBytes + (unsigned)w * 4096u;
#pragma unroll
    for (int j = 0; j < 4; ++j) dma_1k_f64(src_a[j] + s * step_a, slot + j * 1024u);
#pragma unroll
    for (int j = 0; j < 4; ++j) dma_1k_f64(src_b[j] + s * step_b, slot + kGemmOpBytes + j * 1024u);
  };
  // operand reads: lane (m = lane % 16, kq = lane / 16) takes column 4 t + kq of rows m + 16 i
  const int l15 = lane & 15, kq = lane >> 4;
  const unsigned sw = (unsigned)((((kq >> 1) ^ (l15 >> 1)) << 4) | ((kq & 1) << 3));
  unsigned a_off[4], b_off[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    a_off[t] = ((unsigned)(((w >> 1) * 64 + l15) * 128) + sw) ^ (unsigned)(32 * t);
    b_off[t] = kGemmOpBytes + (((unsigned)(((w & 1) * 64 + l15) * 128) + sw) ^ (unsigned)(32 * t));
  }
  // [k][n] form: byte = 1024 k + 16 (pair ^ 8 (k % 2)) + 8 (n % 2) with k = 4 t + kq, n = 64 (w % 2) + 16 j + m
  const unsigned b_base = kGemmOpBytes + (unsigned)(kq * 1024 + (w & 1) * 512 + l15 * 8);
  const unsigned b_even = b_base + (unsigned)((kq & 1) * 128), b_odd = b_base + (unsigned)(((kq & 1) ^ 1) * 128);
  const char* const lds_bytes = reinterpret_cast<const char*>(gemm128_lds);
  auto compute = [&](unsigned stage_off, int next) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      double a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = *reinterpret_cast<const double*>(lds_bytes + stage_off + a_off[t] + i * 2048);
        if constexpr (B_ROWS)
          b[i] = *reinterpret_cast<const double*>(lds_bytes + stage_off + b_off[t] + i * 2048);
        else
          b[i] = *reinterpret_cast<const double*>(lds_bytes + stage_off + ((i & 1) ? b_odd : b_even) + t * 4096 +
                                                  (i >> 1) * 256);
      }
      if (t == 0 && next >= 0) request(next);      // behind the first reads, ahead of the products
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          q.c[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], q.c[i][j], 0, 0, 0);
    }
  };
  if (n_stage <= 0) return;
  request(0);
  for (int s = 0; s < n_stage; s += 2) {
    wait_all_vm();                                 // this wavefront's part of slice s has landed
    __builtin_amdgcn_s_barrier();                  // ... everyone's has, and slice s - 1 is read out
    asm volatile("" ::: "memory");
    compute(0u, s + 1);
    wait_all_vm();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    compute(kGemmStageBytes, (s + 2 < n_stage) ? s + 2 : -1);
  }
}

// f(i, j, r, row, col): result register r of tile (i, j) of this lane and where it sits in the 128 x 128 tile
template <typename F>
__device__ __forceinline__ void acc128_for_each_in_row(int i, F f) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r)
      f(j, r, (w >> 1) * 64 + 16 * i + 4 * r + (lane >> 4), (w & 1) * 64 + 16 * j + (lane & 15));
}

// The trailing update on this engine.  Tile order: the hardware deals work-groups to the 8 dies in
// turn (work-group b runs on die b % 8, each die with an L2 of its own).  Die x takes the row tiles
// I = x, x + 8, ... of every band of 4 column tiles, four consecutive work-groups sharing one row
// strip; a band's four column strips (2 MB at depth 512) stay in that die's L2 while its row tiles
// stream past.  Needs d even, Kd a multiple of 32, k0 + Kd <= d.
constexpr int kTrailBand = 4;

// Row tiles of band `band` that die x works on: I = x + 8 n, n < the value returned.  The band's
// last column is min(cbeg + 128 (4 band + 4), cend) - 1; row tiles beyond it lie below the diagonal.
__host__ __device__ inline int trail_band_rows(int band, int x, int cbeg, int cend) {
  long last = (long)cbeg + (long)kGemmTile * kTrailBand * (band + 1);
  if (last > cend) last = cend;
  const int i_last = (int)((last - 1) / kGemmTile);
  return (i_last >= x) ? (i_last - x) / 8 + 1 : 0;
}

__global__ __launch_bounds__(256, 2) void syrk_trailing128_kernel(double* __restrict__ A, int d, int k0,
                                                                  int Kd, int cb0, int cb1) {
  const int cbeg = cb0 * NB, cend = cb1 * NB;
  const int n_col_tiles = (cend - cbeg + kGemmTile - 1) / kGemmTile;
  const int n_band = (n_col_tiles + kTrailBand - 1) / kTrailBand;
  const int x = blockIdx.x & 7;
  int rem = blockIdx.x >> 3, band = 0;
  for (; band < n_band; ++band) {
    const int cnt = trail_band_rows(band, x, cbeg, cend) * kTrailBand;
    if (rem < cnt) break;
    rem -= cnt;
  }
  if (band == n_band) return;
  const int tj = band * kTrailBand + (rem & (kTrailBand - 1));
  if (tj >= n_col_tiles) return;
  const int row0 = (x + 8 * (rem / kTrailBand)) * kGemmTile;
  const int col0 = cbeg + tj * kGemmTile;
  if (row0 > col0 + kGemmTile - 1) return;      // wholly below the diagonal

  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  Acc128 q;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) q.c[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};
  const double* src_i[4];
  const double* src_j[4];
  gemm128_row_sources(A, d, row0, cend, k0, w, lane, src_i);
  gemm128_row_sources(A, d, col0, cend, k0, w, lane, src_j);
  gemm128_accumulate<true>(src_i, src_j, kGemmK, kGemmK, Kd / kGemmK, q);
  // read-modify-write, one row of tiles (16 values per lane) at a time, loads first
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    double old[16];
    acc128_for_each_in_row(i, [&](int j, int r, int row, int col) {
      const int gi = row0 + row, gj = col0 + col;
      const bool in = gi < cend && gj < cend && gj >= gi;
      old[4 * j + r] = A[in ? (long)gi * d + gj : 0L];
    });
    acc128_for_each_in_row(i, [&](int j, int r, int row, int col) {
      const int gi = row0 + row, gj = col0 + col;
      if (gi < cend && gj < cend && gj >= gi) A[(long)gi * d + gj] = old[4 * j + r] - q.c[i][j][r];
    });
  }
}

// Work-groups of a launch of the 128-tile update over column blocks [cb0, cb1): 8 dies times the
// longest list, which is die 0's.
static int trail128_grid(int cb0, int cb1) {
  const int cbeg = cb0 * NB, cend = cb1 * NB;
  const int n_col_tiles = (cend - cbeg + kGemmTile - 1) / kGemmTile;
  const int n_band = (n_col_tiles + kTrailBand - 1) / kTrailBand;
  int slots = 0;
  for (int band = 0; band < n_band; ++band) slots += trail_band_rows(band, 0, cbeg, cend) * kTrailBand;
  return 8 * slots;
}
// Below this many column blocks the 64-tile kernel has more work-groups to spread over the chip.
constexpr int kTrail128MinBlocks = 64;
// ... and a level of the inversion tree with fewer 128-tiles than this (two per compute unit)
constexpr long kInverse128MinTiles = 512;

// ---------------------------------------------------------------- invert -------------------
// Node `node` of tree depth `depth` over the block range [0, P): ranges are halved
// (left half gets the extra block).  Returns false if the path ends in a leaf earlier.
__device__ __forceinline__ bool tree_node(int P, int depth, int node, int& lo, int& mid, int& hi) {
  lo = 0;
  hi = P;
  for (int l = depth - 1; l >= 0; --l) {
    if (hi - lo < 2) return false;
    const int m = lo + (hi - lo + 1) / 2;
    if ((node >> l) & 1) lo = m; else hi = m;
  }
  if (hi - lo < 2) return false;
  mid = lo + (hi - lo + 1) / 2;
  return true;
}

// One 64 x 64 output tile of C = op(A) * op(B) in fp64, 256 threads, 4 x 4 per thread.
// MODE 1: tmp = R12 * U22      (B upper triangular: k-tiles 0..tj, diagonal tile masked)
// MODE 2: A12 = -U11 * tmp     (A upper triangular: k-tiles ti..M-1, diagonal tile masked)
template <int MODE>
__global__ __launch_bounds__(256) void tri_inverse_level_kernel(double* __restrict__ A, int d,
                                                                double* __restrict__ tmp, int ldt,
                                                                int P, int depth) {
  __shared__ double sa[NB][NB + 1];
  __shared__ double sb[NB][NB + 1];
  int lo, mid, hi;
  if (!tree_node(P, depth, blockIdx.z, lo, mid, hi)) return;
  const int Mb = mid - lo, Nb = hi - mid;        // in blocks
  const int ti = blockIdx.y, tj = blockIdx.x;
  if (ti >= Mb || tj >= Nb) return;
  const int tid = threadIdx.x;
  const int row0 = (lo + ti) * NB;               // global rows of the output tile
  const int col0 = (mid + tj) * NB;              // global cols of the output tile (in A)
  Quad64 q;
  quad_zero(q);
  const int kb_begin = (MODE == 1) ? 0 : ti;
  const int kb_end = (MODE == 1) ? tj + 1 : Mb;
  double va[16], vb[16];
  auto fetch = [&](int kb) {
    if (MODE == 1) {
      // A operand: R12[row0+i][(mid+kb)*NB + j];  B operand: U22[(mid+kb)*NB+i][col0+j]
      fetch_tile64(A, [&](int i, int j) { return row0 + i < d && (mid + kb) * NB + j < d; },
                   [&](int i, int j) { return (long)(row0 + i) * d + (mid + kb) * NB + j; }, va);
      fetch_tile64(A,
                   [&](int i, int j) {
                     const int br = (mid + kb) * NB + i, bc = col0 + j;
                     return br < d && bc < d && br <= bc;
                   },
                   [&](int i, int j) { return (long)((mid + kb) * NB + i) * d + col0 + j; }, vb);
    } else {
      // A operand: U11[row0+i][(lo+kb)*NB + j];  B operand: tmp[(lo+kb)*NB+i][tj*NB+j]
      fetch_tile64(A,
                   [&](int i, int j) {
                     const int gr = row0 + i, gc = (lo + kb) * NB + j;
                     return gr < d && gc < d && gr <= gc;
                   },
                   [&](int i, int j) { return (long)(row0 + i) * d + (lo + kb) * NB + j; }, va);
      fetch_tile64(tmp, [&](int i, int) { return (lo + kb) * NB + i < d; },
                   [&](int i, int j) { return (long)((lo + kb) * NB + i) * ldt + tj * NB + j; }, vb);
    }
  };
  if (kb_begin < kb_end) fetch(kb_begin);
  for (int kb = kb_begin; kb < kb_end; ++kb) {
    put_tile64(sa, va);
    put_tile64(sb, vb);
    __syncthreads();
    if (kb + 1 < kb_end) fetch(kb + 1);             // in flight during the products below
    quad_mfma_64<false>(sa, sb, q);
    __syncthreads();
  }
  quad_for_each(q, [&](int r, int c, double v) {
    const int i = row0 + r;
    if (i >= d) return;
    if (MODE == 1) {
      tmp[(long)i * ldt + tj * NB + c] = v;
    } else if (col0 + c < d) {
      A[(long)i * d + col0 + c] = -v;
    }
  });
}

// The same two products on the 128-tile engine (d a multiple of 64).  Tile (ti, tj) of 128 x 128:
//   MODE 1: tmp[rows][tj] = R12[rows][k] U22[k][tj], k over the columns of U22 up to the tile's last
//           (U22 is upper triangular; the block left of a diagonal block holds zeros);
//   MODE 2: U12[rows][tj] = -U11[rows][k] tmp[k][tj], k from the tile's first row on.
// A node with an odd number of blocks leaves half a tile hanging over: its rows / columns are
// clamped on the way in and skipped on the way out.
template <int MODE>
__global__ __launch_bounds__(256, 2) void tri_inverse_level128_kernel(double* __restrict__ A, int d,
                                                                      double* __restrict__ tmp, int ldt,
                                                                      int P, int depth) {
  int lo, mid, hi;
  if (!tree_node(P, depth, blockIdx.z, lo, mid, hi)) return;
  const int n_rows = (mid - lo) * NB, n_cols = (hi - mid) * NB;
  // Work-groups go to the 8 XCDs in turn (x fastest).  The tile column is rotated by the tile row:
  // otherwise, whenever the tile count per row is a multiple of 8, one XCD would get all the
  // longest (or shortest) K ranges, which grow with the column (MODE 1) or shrink with the row.
  // (Super-blocks of 4 x 4 tiles per XCD, for L2 reuse, were measured and were slower.)
  const int r_loc = blockIdx.y * kGemmTile;
  const int c_loc = (int)((blockIdx.x + blockIdx.y) % gridDim.x) * kGemmTile;   // inside the node
  if (r_loc >= n_rows || c_loc >= n_cols) return;
  const int row0 = lo * NB + r_loc, row_limit = mid * NB;     // global rows of the tile
  const int col0 = mid * NB + c_loc, col_limit = hi * NB;     // global columns of the tile (in A)
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  Acc128 q;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) q.c[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};
  const double* src_a[4];
  const double* src_b[4];
  if (MODE == 1) {
    const int k_begin = mid * NB;
    const int k_end = (col0 + kGemmTile < col_limit) ? col0 + kGemmTile : col_limit;
    gemm128_row_sources(A, d, row0, row_limit, k_begin, w, lane, src_a);
    gemm128_col_sources(A, d, k_begin, col0, col_limit, w, lane, src_b);
    gemm128_accumulate<false>(src_a, src_b, kGemmK, (long)kGemmK * d, (k_end - k_begin) / kGemmK, q);
  } else {
    const int k_begin = row0, k_end = row_limit;
    gemm128_row_sources(A, d, row0, row_limit, k_begin, w, lane, src_a);
    gemm128_col_sources(tmp, ldt, k_begin, c_loc, n_cols, w, lane, src_b);
    gemm128_accumulate<false>(src_a, src_b, kGemmK, (long)kGemmK * ldt, (k_end - k_begin) / kGemmK, q);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    acc128_for_each_in_row(i, [&](int j, int r, int row, int col) {
      const int gi = row0 + row;
      if (gi >= row_limit || c_loc + col >= n_cols) return;
      if (MODE == 1) tmp[(long)gi * ldt + c_loc + col] = q.c[i][j][r];
      else A[(long)gi * d + col0 + col] = -q.c[i][j][r];
    });
}

// U (fp32) <- upper triangle of A, zeros below.
__global__ __launch_bounds__(256) void prep_store_kernel(const double* __restrict__ A, int d,
                                                         float* __restrict__ U) {
  const long n = (long)d * d;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const int i = (int)(e / d), j = (int)(e % d);
    U[e] = (j >= i) ? (float)A[e] : 0.f;
  }
}

static int tree_depth(int P) {   // number of levels that contain at least one internal node
  int depth = 0, width = P;
  while (width >= 2) {
    width = (width + 1) / 2;
    ++depth;
  }
  return depth;
}

struct PrepLayout {
  size_t a_off, tmp_off, rdiag_off, r12_off, flag_off, scal_off, total;
  int P, ldt;
};

static PrepLayout prep_layout(int d) {
  PrepLayout L;
  L.P = bpdq_ceil_div(d, NB);
  L.ldt = ((L.P + 1) / 2) * NB;
  size_t off = 0;
  L.a_off = off;    off += bpdq_align_up((size_t)d * d * sizeof(double), 256);
  L.tmp_off = off;  off += bpdq_align_up((size_t)d * L.ldt * sizeof(double), 256);
  L.rdiag_off = off; off += bpdq_align_up((size_t)L.P * NB * NB * sizeof(double), 256);
  L.r12_off = off;  off += bpdq_align_up((size_t)L.P * NB * NB * sizeof(double), 256);
  L.flag_off = off; off += bpdq_align_up((size_t)L.P * sizeof(int), 256);
  L.scal_off = off; off += 256;
  L.total = off;
  return L;
}

#define BPDQ_TRY(expr)              \
  do {                              \
    const int rc_ = (expr);         \
    if (rc_ != 0) return rc_;       \
  } while (0)

// The trailing update of column blocks [cb0, cb1) by the factored columns [k0, k0 + depth).
static int launch_trailing(hipStream_t st, double* A, int d, int k0, int depth, int cb0, int cb1) {
  if (cb1 <= cb0) return 0;
  if (cb1 >= kTrail128MinBlocks && d % 2 == 0 && depth % 32 == 0 && k0 + depth <= d) {
    hipLaunchKernelGGL(syrk_trailing128_kernel, dim3(trail128_grid(cb0, cb1)), dim3(256), kGemmLdsBytes, st,
                       A, d, k0, depth, cb0, cb1);
  } else {
    const int tiles = (cb1 * (cb1 + 1) - cb0 * (cb0 + 1)) / 2;
    hipLaunchKernelGGL(syrk_trailing_kernel, dim3(tiles), dim3(256), 0, st, A, d, k0, depth, cb0, cb1);
  }
  BPDQ_LAUNCH_CHECK();
  return 0;
}

}  // namespace bpdq

using namespace bpdq;

extern "C" size_t bpdq_prepare_workspace_bytes(int d_in) {
  if (d_in <= 0) return 0;
  return prep_layout(d_in).total;
}

extern "C" int bpdq_prepare(const float* H, int d_in, float damp, float* U, unsigned char* dead,
                            int* info, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (!H) return -1;
  if (d_in <= 0) return -2;
  if (!(damp >= 0.f)) return -3;
  if (!U) return -4;
  if (!info) return -6;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return -7;
  const PrepLayout L = prep_layout(d_in);
  if (ws_bytes < L.total) return -8;
  char* base = static_cast<char*>(ws);
  double* A = reinterpret_cast<double*>(base + L.a_off);
  double* tmp = reinterpret_cast<double*>(base + L.tmp_off);
  double* Rdiag = reinterpret_cast<double*>(base + L.rdiag_off);
  double* scal = reinterpret_cast<double*>(base + L.scal_off);
  double* R12buf = reinterpret_cast<double*>(base + L.r12_off);
  int* pair_flag = reinterpret_cast<int*>(base + L.flag_off);
  const int d = d_in, P = L.P;
  BPDQ_HIP_TRY(bpdq_lds_limit<&panel_pair_kernel>(kPairLdsBytes));
  BPDQ_HIP_TRY(bpdq_lds_limit<&syrk_trailing128_kernel>(kGemmLdsBytes));
  BPDQ_HIP_TRY(bpdq_lds_limit<&tri_inverse_level128_kernel<1>>(kGemmLdsBytes));
  BPDQ_HIP_TRY(bpdq_lds_limit<&tri_inverse_level128_kernel<2>>(kGemmLdsBytes));

  hipLaunchKernelGGL(prep_diag_kernel, dim3(1), dim3(1024), 0, stream, H, d, damp, dead, scal, info);
  BPDQ_LAUNCH_CHECK();
  const int grid_el = (int)((((long)d * d + 255) / 256) < 65536 ? (((long)d * d + 255) / 256) : 65536);
  hipLaunchKernelGGL(prep_load_kernel, dim3(grid_el), dim3(256), 0, stream, H, d, scal, A);
  BPDQ_LAUNCH_CHECK();

  // outer panels of kOuter blocks, from the right; inside one, 64-column panels from the right
  constexpr int kOuter = 8;
  for (int ob1 = P; ob1 > 0; ob1 -= kOuter) {
    const int ob0 = ob1 > kOuter ? ob1 - kOuter : 0;
    int p = ob1 - 1;
    while (p >= ob0) {
      int first_blk, width;                  // blocks [first_blk, p] factored by this launch
      if (p - 1 >= ob0) {                    // a pair of panels
        const int b1 = p - 1, p1 = b1 * NB;
        const int nb2 = (d - p * NB < NB) ? d - p * NB : NB;
        hipLaunchKernelGGL(panel_pair_kernel, dim3(b1 > 0 ? b1 : 1), dim3(256), kPairLdsBytes, stream,
                           A, d, p1, nb2, b1, Rdiag + (size_t)b1 * NB * NB,
                           Rdiag + (size_t)p * NB * NB, R12buf + (size_t)p * NB * NB,
                           pair_flag + b1, pair_flag + p, info);
        first_blk = b1;
        width = NB + nb2;
      } else {                               // a single panel (odd count at the left edge)
        const int p0 = p * NB;
        const int nb = (d - p0 < NB) ? d - p0 : NB;
        hipLaunchKernelGGL(panel_factor_kernel, dim3(p > 0 ? p : 1), dim3(256), 0, stream, A, d, p0,
                           nb, p, Rdiag + (size_t)p * NB * NB, pair_flag + p, info);
        first_blk = p;
        width = nb;
      }
      BPDQ_LAUNCH_CHECK();
      if (first_blk > ob0) {
        const int tiles = (first_blk * (first_blk + 1) - ob0 * (ob0 + 1)) / 2;
        hipLaunchKernelGGL(syrk_trailing_kernel, dim3(tiles), dim3(256), 0, stream, A, d,
                           first_blk * NB, width, ob0, first_blk);
        BPDQ_LAUNCH_CHECK();
      }
      p = first_blk - 1;
    }
    if (ob0 > 0) {
      const int depth = (ob1 - ob0) * NB;
      BPDQ_TRY(launch_trailing(stream, A, d, ob0 * NB, depth, 0, ob0));
    }
  }

  hipLaunchKernelGGL(diag_inverse_kernel, dim3(P), dim3(256), 0, stream, Rdiag, R12buf, pair_flag, A, d);
  BPDQ_LAUNCH_CHECK();
  const int depth = tree_depth(P);
  for (int dd = depth - 1; dd >= 0; --dd) {
    // at depth dd a node spans at most ceil(P / 2^dd) blocks
    int span = P;
    for (int l = 0; l < dd; ++l) span = (span + 1) / 2;
    const int half = (span + 1) / 2;
    const long tiles128 = ((long)((half + 1) / 2) * ((half + 1) / 2)) << dd;
    if (d % NB == 0 && tiles128 >= kInverse128MinTiles) {
      dim3 grid((half + 1) / 2, (half + 1) / 2, 1 << dd);
      hipLaunchKernelGGL(tri_inverse_level128_kernel<1>, grid, dim3(256), kGemmLdsBytes, stream, A, d, tmp,
                         L.ldt, P, dd);
      BPDQ_LAUNCH_CHECK();
      hipLaunchKernelGGL(tri_inverse_level128_kernel<2>, grid, dim3(256), kGemmLdsBytes, stream, A, d, tmp,
                         L.ldt, P, dd);
      BPDQ_LAUNCH_CHECK();
      continue;
    }
    dim3 grid(half, half, 1 << dd);
    hipLaunchKernelGGL(tri_inverse_level_kernel<1>, grid, dim3(256), 0, stream, A, d, tmp, L.ldt, P, dd);
    BPDQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(tri_inverse_level_kernel<2>, grid, dim3(256), 0, stream, A, d, tmp, L.ldt, P, dd);
    BPDQ_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(prep_store_kernel, dim3(grid_el), dim3(256), 0, stream, A, d, U);
  BPDQ_LAUNCH_CHECK();
  return 0;
}
