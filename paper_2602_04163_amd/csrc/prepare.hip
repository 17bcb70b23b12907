// Step 2 of the pass: damping and U = chol(H^-1), H^-1 = U^T U with U upper triangular
// (paper Sec. 3.1, "Quantization Error Compensation").
//
// Route: with Ht = H + lambda I, factor Ht = R R^T with R UPPER triangular (a Cholesky
// factorisation that runs from the last column to the first).  Then
// Ht^-1 = R^-T R^-1 = (R^-1)^T (R^-1), so U = R^-1: one factorisation plus one triangular
// inverse (2/3 d^3 flops) and Ht^-1 is never formed.  Everything runs in fp64 inside the
// workspace; the result is rounded to fp32 once, on output.
//
//   factor : right-looking over 64-column panels from the right: every panel work-group factors
//            the diagonal block in registers and solves its 64 rows of R12 R22^T = A12.  The
//            trailing update A11 -= R12 R12^T (fp64 MFMA, upper 64 x 64 tiles) is two-level:
//            after each panel only inside the current 512-column outer panel, and once per
//            outer panel, with K = 512, on everything to its left.
//   invert : divide and conquer over block ranges, [R11 R12; 0 R22]^-1 =
//            [U11, -U11 R12 U22; 0, U22]; every tree level is two launches.
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
// 1 / x in fp64: hardware estimate + two Newton steps (the pivot reciprocal sits on the critical
// path of every column step).
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = fma(fma(-x, r, 1.0), r, r);
  r = fma(fma(-x, r, 1.0), r, r);
  return r;
}

// Panel step of the reversed Cholesky, one work-group (256 threads) per 64 rows of the panel.
//   (1) every work-group factors the 64 x 64 diagonal block D = R R^T (R upper, columns taken
//       from the last to the first) for itself: thread (ty, tx) keeps the 4 x 4 sub-block
//       rows 4ty.., cols 4tx.. in registers; per column one LDS broadcast of the current column,
//       one barrier, one reciprocal and a rank-1 update  a -= col col^T / pivot.
//   (2) rows [64 b, 64 b + 64) of the panel above the block: X R^T = A12 solved by substitution,
//       one thread per row, the row held in registers.
// Work-group 0 also writes R of the diagonal block to Rdiag (NB x NB, row-major, zero below the
// diagonal, identity-padded) and reports a non-positive pivot.
// Launch with max(p, 1) work-groups, p = number of 64-row blocks above the diagonal block.
__global__ __launch_bounds__(256) void panel_factor_kernel(double* __restrict__ A, int d, int p0,
                                                           int nb, int n_above,
                                                           double* __restrict__ Rdiag, int* info) {
  __shared__ double sR[NB][NB + 1];     // R (upper) of the diagonal block
  __shared__ double sA[NB][NB + 1];     // panel tile of this work-group
  __shared__ double col[2][NB];
  __shared__ double sInvD[NB];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;

  double a[4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int i = 4 * ty + r, j = 4 * tx + c;
      double v = (i == j) ? 1.0 : 0.0;              // identity padding of a ragged last block
      if (i < nb && j < nb)
        v = (j >= i) ? A[(long)(p0 + i) * d + p0 + j] : A[(long)(p0 + j) * d + p0 + i];
      a[r][c] = v;
    }
  // panel tile (coalesced), used after the factorisation
  const int r0 = blockIdx.x * NB;
  if (n_above > 0) {
    for (int e = tid; e < NB * NB; e += 256) {
      const int i = e / NB, j = e % NB;
      sA[i][j] = (r0 + i < p0 && j < nb) ? A[(long)(r0 + i) * d + p0 + j] : 0.0;
    }
  }

#pragma unroll 1
  for (int jb = NB / 4 - 1; jb >= 0; --jb) {
#pragma unroll
    for (int jj = 3; jj >= 0; --jj) {
      const int j = 4 * jb + jj;
      double* cbuf = col[j & 1];
      if (tx == jb) {
#pragma unroll
        for (int r = 0; r < 4; ++r) cbuf[4 * ty + r] = a[r][jj];
      }
      __syncthreads();
      double piv = cbuf[j];
      if (!(piv > 0.0)) {
        if (tid == 0 && blockIdx.x == 0) atomicCAS(info, 0, p0 + j + 1);
        piv = 1.0;
      }
      const double ip = fast_rcp(piv);
      double ci[4], cj[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) ci[r] = cbuf[4 * ty + r] * ip;
#pragma unroll
      for (int c = 0; c < 4; ++c) cj[c] = cbuf[4 * tx + c];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) a[r][c] = fma(-ci[r], cj[c], a[r][c]);
      if (tid < NB) {
        sR[tid][j] = (tid <= j) ? cbuf[tid] : 0.0;     // unscaled column; scaled after the loop
        if (tid == j) sInvD[j] = piv;
      }
    }
  }
  __syncthreads();
  // R[:, j] = column_j / sqrt(pivot_j): the square roots are taken once, off the critical path
  if (tid < NB) sInvD[tid] = 1.0 / sqrt(sInvD[tid]);
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    sR[i][j] *= sInvD[j];
  }
  __syncthreads();
  // R of the diagonal block goes to its own buffer: the block itself must stay untouched, because
  // work-groups of this launch that start later still have to read it
  if (blockIdx.x == 0) {
    for (int e = tid; e < NB * NB; e += 256) Rdiag[e] = sR[e / NB][e % NB];
  }
  if (n_above == 0) return;

  // (2) X R^T = A12 by substitution from the last column: x_j = rem_j / R_jj, then
  //     rem_k -= x_j R[k][j] for every k < j (independent updates: no serial dot product)
  if (tid < NB) {
    double x[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) x[j] = sA[tid][j];
#pragma unroll
    for (int j = NB - 1; j >= 0; --j) {
      x[j] *= sInvD[j];
#pragma unroll
      for (int k = 0; k < j; ++k) x[k] = fma(-x[j], sR[k][j], x[k]);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) sA[tid][j] = x[j];
  }
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    if (r0 + i < p0 && j < nb) A[(long)(r0 + i) * d + p0 + j] = sA[i][j];
  }
}

// Inverses of all diagonal blocks of R at once (one work-group per block, thread c solves
// R x = e_c by back substitution); the inverse replaces the diagonal block of A (upper part,
// zeros below), which until now still held the unfactored block.
__global__ __launch_bounds__(64) void diag_inverse_kernel(const double* __restrict__ Rdiag,
                                                          double* __restrict__ A, int d) {
  __shared__ double s[NB][NB + 1];
  __shared__ double x[NB][NB + 1];
  const int p0 = blockIdx.x * NB;
  const int nb = (d - p0 < NB) ? d - p0 : NB;
  const int c = threadIdx.x;
  const double* src = Rdiag + (long)blockIdx.x * NB * NB;
  for (int e = c; e < NB * NB; e += 64) {
    s[e / NB][e % NB] = src[e];
    x[e / NB][e % NB] = 0.0;
  }
  __syncthreads();
  x[c][c] = 1.0 / s[c][c];
  for (int i = c - 1; i >= 0; --i) {
    double acc = 0.0;
    for (int m = i + 1; m <= c; ++m) acc += s[i][m] * x[m][c];
    x[i][c] = -acc / s[i][i];
  }
  __syncthreads();
  for (int e = c; e < NB * NB; e += 64) {
    const int i = e / NB, j = e % NB;
    if (i < nb && j < nb) A[(long)(p0 + i) * d + p0 + j] = (j >= i) ? x[i][j] : 0.0;
  }
}

// 64 x 64 x 64 fp64 product on the matrix cores for a 256-thread work-group: wavefront w owns
// the 32 x 32 quadrant (w / 2, w % 2) as 2 x 2 tiles of v_mfma_f64_16x16x4_f64.
//   A operand: lane l holds A[m = l % 16][k = l / 16];  B operand: B[k = l / 16][n = l % 16];
//   D: register r of lane l is D[4 * r + l / 16][l % 16].
// sa is [m][k]; sb is [k][n], or [n][k] when B_T (second operand given by rows, as in a SYRK).
// With the 65-double row pitch every 16-lane group reads 16 distinct bank pairs.
typedef double f64x4 __attribute__((ext_vector_type(4)));

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
  for (int kc = k0; kc < k_end; kc += NB) {
    for (int e = tid; e < NB * NB; e += 256) {
      const int i = e / NB, k = e % NB;
      const bool in = kc + k < k_end;
      si[i][k] = in ? A[(long)(bi * NB + i) * d + kc + k] : 0.0;
      sj[i][k] = in ? A[(long)(bj * NB + i) * d + kc + k] : 0.0;
    }
    __syncthreads();
    quad_mfma_64<true>(si, sj, q);
    __syncthreads();
  }
  quad_for_each(q, [&](int r, int c, double v) {
    const int i = bi * NB + r, j = bj * NB + c;
    if (j >= i) A[(long)i * d + j] -= v;
  });
}

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
  for (int kb = kb_begin; kb < kb_end; ++kb) {
    for (int e = tid; e < NB * NB; e += 256) {
      const int i = e / NB, j = e % NB;
      double va, vb;
      if (MODE == 1) {
        // A operand: R12[row0+i][mid*NB + kb*NB + j];  B operand: U22[(mid+kb)*NB+i][col0+j]
        const int gr = row0 + i, gc = (mid + kb) * NB + j;
        va = (gr < d && gc < d) ? A[(long)gr * d + gc] : 0.0;
        const int br = (mid + kb) * NB + i, bc = col0 + j;
        vb = (br < d && bc < d && br <= bc) ? A[(long)br * d + bc] : 0.0;
      } else {
        // A operand: U11[row0+i][(lo+kb)*NB + j];  B operand: tmp[(lo+kb)*NB+i][tj*NB+j]
        const int gr = row0 + i, gc = (lo + kb) * NB + j;
        va = (gr < d && gc < d && gr <= gc) ? A[(long)gr * d + gc] : 0.0;
        const int br = (lo + kb) * NB + i;
        vb = (br < d) ? tmp[(long)br * ldt + tj * NB + j] : 0.0;
      }
      sa[i][j] = va;
      sb[i][j] = vb;
    }
    __syncthreads();
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
  size_t a_off, tmp_off, rdiag_off, scal_off, total;
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
  L.scal_off = off; off += 256;
  L.total = off;
  return L;
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
  const int d = d_in, P = L.P;

  hipLaunchKernelGGL(prep_diag_kernel, dim3(1), dim3(1024), 0, stream, H, d, damp, dead, scal, info);
  BPDQ_LAUNCH_CHECK();
  const int grid_el = (int)((((long)d * d + 255) / 256) < 65536 ? (((long)d * d + 255) / 256) : 65536);
  hipLaunchKernelGGL(prep_load_kernel, dim3(grid_el), dim3(256), 0, stream, H, d, scal, A);
  BPDQ_LAUNCH_CHECK();

  // outer panels of kOuter blocks, from the right; inside one, 64-column panels from the right
  constexpr int kOuter = 8;
  for (int ob1 = P; ob1 > 0; ob1 -= kOuter) {
    const int ob0 = ob1 > kOuter ? ob1 - kOuter : 0;
    for (int p = ob1 - 1; p >= ob0; --p) {
      const int p0 = p * NB;
      const int nb = (d - p0 < NB) ? d - p0 : NB;
      hipLaunchKernelGGL(panel_factor_kernel, dim3(p > 0 ? p : 1), dim3(256), 0, stream, A, d, p0,
                         nb, p, Rdiag + (size_t)p * NB * NB, info);
      BPDQ_LAUNCH_CHECK();
      if (p > ob0) {
        const int tiles = (p * (p + 1) - ob0 * (ob0 + 1)) / 2;
        hipLaunchKernelGGL(syrk_trailing_kernel, dim3(tiles), dim3(256), 0, stream, A, d, p0, nb,
                           ob0, p);
        BPDQ_LAUNCH_CHECK();
      }
    }
    if (ob0 > 0) {
      hipLaunchKernelGGL(syrk_trailing_kernel, dim3(ob0 * (ob0 + 1) / 2), dim3(256), 0, stream, A, d,
                         ob0 * NB, (ob1 - ob0) * NB, 0, ob0);
      BPDQ_LAUNCH_CHECK();
    }
  }

  hipLaunchKernelGGL(diag_inverse_kernel, dim3(P), dim3(64), 0, stream, Rdiag, A, d);
  BPDQ_LAUNCH_CHECK();
  const int depth = tree_depth(P);
  for (int dd = depth - 1; dd >= 0; --dd) {
    // at depth dd a node spans at most ceil(P / 2^dd) blocks
    int span = P;
    for (int l = 0; l < dd; ++l) span = (span + 1) / 2;
    const int half = (span + 1) / 2;
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
