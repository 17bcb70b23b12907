/*
 * bpdq.h -- C ABI of the BPDQ per-layer quantization pass for AMD MI355X (gfx950).
 *
 * BPDQ (Bit-Plane Decomposition Quantization on a variable grid) represents a linear
 * layer's weight as   What = REP(C_0) + sum_{i=1..k} REP(C_i) (.) B_i   (paper Eq. 1):
 * k binary planes B_i and k+1 real coefficients per (row, group of g input channels),
 * chosen to minimise || (W - What) X ||_F^2 = tr((W - What) H (W - What)^T)  (Eq. 2).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer owned by the caller unless marked "host".
 *    The library allocates nothing: scratch comes from the caller's workspace `ws`
 *    (256-byte aligned, at least *_workspace_bytes() long).
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and returns without synchronising.  Calls on one stream are
 *    ordered; a workspace must not be shared by calls that can run concurrently.
 *  - Matrices are dense row-major fp32 unless stated.
 *  - Return value: 0 = enqueued; -n = argument number n (1-based) is invalid;
 *    BPDQ_ERR_LAUNCH = a HIP call failed.  Numerical failure of bpdq_prepare is reported
 *    through its device-side `info`, LAPACK style.
 *  - Results are deterministic: no floating-point atomics anywhere.
 */
#ifndef BPDQ_H
#define BPDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BPDQ_ERR_LAUNCH (-100)
#define BPDQ_GRID_VARIABLE 0
#define BPDQ_GRID_UNIFORM 1

/* Knobs of the method (paper Sec. 4.1: k in {2,3,4}, g in {64,128,256}, 10 iterations,
 * alpha = 1e-4). */
typedef struct bpdq_params {
  int   bits;           /* k, number of bit-planes: 1..4                                      */
  int   group;          /* g: 32, 64, 128 or 256 (256 only with bits <= 3); must divide d_in  */
  int   block;          /* lazy-update block B; the effective block is max(B, g); g | B       */
  int   refine_iters;   /* T >= 0 iterations of (bit-plane update, refit, delta correction);
                           0 keeps the initialisation + one fit (Sec. 3.2)                    */
  float alpha;          /* relative ridge of the coefficient fit (Sec. 3.2, end): the
                           (k+1)x(k+1) normal matrix G gets alpha*tr(G)/(k+1) on its diagonal */
  int   grid;           /* BPDQ_GRID_VARIABLE: the method (variable grid, Sec. 3).
                           BPDQ_GRID_UNIFORM: the fixed-grid comparator of App. A -- levels
                           lo + s*{0..2^k-1} per (row, group) from the group's min/max, one
                           sweep, no fit (GPTQ on a uniform grid); refine_iters and alpha are
                           ignored, the coefficients returned are (lo, s, 2s, ...).             */
  int   coef_fp16;      /* storage precision of the coefficients (Table 1 counts 16 bits each).
                           0: fp32 throughout.  1: every coefficient is rounded to IEEE half
                           (nearest even) right after its fit, so the levels of the next bit-plane
                           update, What, E*, the scores and the compensation all belong to the
                           values that are stored; `coefs` still holds floats, each exactly a
                           half (bpdq_coefs_to_fp16 is then lossless).  Magnitudes above 65504
                           would become infinite: scale such a layer first.                    */
} bpdq_params;

/* Library version (major*10000 + minor*100 + patch). */
int bpdq_version(void);

/* ---- step 1: calibration Hessian (Sec. 3.1, text under Eq. 2: H = X X^T) ---------------
 * H += scale * Xc^T Xc for one chunk of tokens.
 *   Xc : n_tok x d_in, one token per row, row stride ldx floats (>= d_in).  This is the
 *        paper's X (d_in x N, one token per column) in column-major storage.
 *   H  : d_in x d_in.  Only the upper triangle (j >= i) is accumulated; pass
 *        symmetrize != 0 (e.g. on the last chunk) to mirror it into the lower triangle.
 *   scale : 2 reproduces the customary H = 2 X X^T; any positive factor gives the same
 *        planes and coefficients.
 *   ws : split-K partial sums and, for the default entry, the activations re-encoded as halves;
 *        bpdq_hessian_workspace_bytes(n_tok, d_in) bytes serve any of the three entries
 *        (about 4 * n_tok * d_in bytes plus the partial tiles).
 * Requirements: d_in % 4 == 0, ldx % 4 == 0, Xc and H 16-byte aligned, ws 256-byte aligned, n_tok >= 0.
 * Returns 0, or a negative code naming the offending argument (-1 Xc, -2 n_tok, -3 d_in,
 * -4 ldx, -6 H, -8 ws, -9 ws_bytes); nothing is launched then.
 *
 * Three kernels compute the same update; each result is bit-reproducible from call to call, they
 * are not bit-identical to one another (they differ by rounding), and each is checked against the
 * fp64 definition to 1e-5 relative Frobenius error.
 * bpdq_hessian_accumulate (the fastest) runs on the fp16 matrix cores: a streaming pre-pass finds
 *   every channel's largest magnitude in the call, scales the channel by the power of two that
 *   brings it into [2^13, 2^14) and cuts every scaled value into two halves h + l (22 significant
 *   bits); a product is the sum of the three half products of weight >= 2^-11, accumulated in fp32,
 *   and the result is scaled back exactly.  The error of a product is below 2^-21 of it -- above
 *   the 2^-24 of an fp32 product, far below the rounding of the fp32 accumulation over thousands of
 *   tokens.  Assumes finite X (an infinity or NaN yields NaN in its row and column).
 * bpdq_hessian_accumulate_bf16x3 runs on the bf16 matrix cores without a pre-pass: every value is
 *   cut exactly into three bf16 pieces inside the kernel and a product is the sum of the six piece
 *   products of weight >= 2^-16 (error below 2^-24 of a product).  About 1.5 times slower.
 *   Assumes |x| < 2^127.
 * bpdq_hessian_accumulate_f32 runs on the fp32 matrix cores (about 2.4 times slower). */
size_t bpdq_hessian_workspace_bytes(int n_tok, int d_in);
int bpdq_hessian_accumulate(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                            float* H, int symmetrize, void* ws, size_t ws_bytes, void* stream);
int bpdq_hessian_accumulate_bf16x3(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                                   float* H, int symmetrize, void* ws, size_t ws_bytes,
                                   void* stream);
int bpdq_hessian_accumulate_f32(const float* Xc, int n_tok, int d_in, int ldx, float scale,
                                float* H, int symmetrize, void* ws, size_t ws_bytes,
                                void* stream);

/* The same call with the kernel chosen by number, for measurement: ev_begin / ev_end (hipEvent_t
 * as void*, created by the caller with timing enabled, or NULL) are recorded on `stream`
 * immediately before the first and immediately after the last launch of the tile-product kernel
 * (a call of at most 524288 tokens on a layer of fewer than 1024 tiles is one launch: then the two
 * events bracket that kernel alone, without the pre-pass before it and the reduction after it).
 * Return codes as above with every argument number one higher (-1: unknown kernel). */
#define BPDQ_HESSIAN_F16X2 0
#define BPDQ_HESSIAN_BF16X3 1
#define BPDQ_HESSIAN_F32 2
int bpdq_hessian_accumulate_timed(int kernel, const float* Xc, int n_tok, int d_in, int ldx,
                                  float scale, float* H, int symmetrize, void* ws, size_t ws_bytes,
                                  void* stream, void* ev_begin, void* ev_end);

/* ---- step 2: damping and U = chol(H^-1) (Sec. 3.1, "Quantization Error Compensation") ---
 * Reads the upper triangle of H.  Channels with H_ii == 0 are marked dead[i] = 1 and get
 * H_ii = 1.  Then lambda = damp * mean_i(H_ii), Ht = H + lambda I, and U is the upper
 * triangular matrix with positive diagonal such that Ht^-1 = U^T U.
 *   U    : d_in x d_in fp32, full matrix written (strictly lower part = 0); may alias H.
 *   dead : d_in bytes.
 *   info : one device int: 0, or the 1-based index of a column whose pivot was not
 *          positive (Ht not positive definite; U is then undefined).
 * The factorisation runs in fp64 inside ws. */
size_t bpdq_prepare_workspace_bytes(int d_in);
int bpdq_prepare(const float* H, int d_in, float damp, float* U, unsigned char* dead,
                 int* info, void* ws, size_t ws_bytes, void* stream);

/* ---- steps 3-4: the group/column sweep with lazy block updates (Sec. 3.2, 3.3, App. B.3) -
 * For every block of max(B, g) columns, left to right, and every group of g columns in it:
 * 8-bit round-to-nearest initialisation of the planes from the group's current working
 * weights (Eq. 5), coefficient fit in the metric of the local factor (Eq. 6), then
 * refine_iters times: column-wise nearest-level bit-plane update with error propagation
 * (Eq. 3-4, 7-8), coefficient refit, delta correction (Eq. 9); the iterate with the smallest
 * ||E_group||_F^2 is kept (the initial state counts as iterate 0; ties keep the earliest).
 * Its propagation error reaches the columns not yet quantized exactly as
 * W'[:, end:] -= E_blk U[blk, end:] per block (and E* U[grp, rest of block] inside a block):
 * one GEMM per block for the far columns, applied one block late and overlapped with the next
 * sweep, while the groups of the next block read the pending terms directly from the kept E*.
 *   W       : d_out x d_in, read only.
 *   U, dead : from bpdq_prepare (dead may be NULL).
 *   planes  : uint32 [bits][d_out][d_in/32]; column c of plane B_i (i = 1..bits) is bit
 *             (c % 32) of word planes[i-1][r][c/32], least significant bit first.
 *   coefs   : float [bits+1][d_out][d_in/g]; index 0 is the bias C_0.
 *   W_hat   : float d_out x d_in, or NULL.  Equal to bpdq_dequant(planes, coefs) bit for bit.
 *   grp_err : double [d_in/g], ||E_group||_F^2 of the kept iterate; their sum is the layer
 *             objective tr((W-What) Ht (W-What)^T) (App. B.2).
 *   grp_iter: int [d_in/g], index of the kept iterate (0..refine_iters).
 * Requirements: d_in % group == 0, d_in % 32 == 0, group | max(block, group). */
size_t bpdq_quantize_workspace_bytes(int d_out, int d_in, const bpdq_params* p /* host */);
int bpdq_quantize_layer(const float* W, int d_out, int d_in, const float* U,
                        const unsigned char* dead, const bpdq_params* p /* host */,
                        uint32_t* planes, float* coefs, float* W_hat, double* grp_err,
                        int* grp_iter, void* ws, size_t ws_bytes, void* stream);

/* The lazy block update on its own (Eq. 4 applied to a whole block of finished columns, App. B.3
 * tail form), as bpdq_quantize_layer applies it inside the sweep:
 *     Wp[:, c_begin:c_end] -= E_blk U[k0:k0+Kd, c_begin:c_end]
 * on the fp32 matrix cores, in place.
 *   Et : the block's propagation coordinates, transposed: Kd x lde, row k holds E[:, k0 + k] for all
 *        d_out rows (lde >= d_out; the lde - d_out padding entries of a row are read and ignored).
 *   U  : the factor from bpdq_prepare, leading dimension ldu;  Wp: d_out x ldw working weights.
 * Requirements: lde, ldu multiples of 4; Et, U 16-byte aligned; c_begin, c_end multiples of 4.
 * Exposed for parity tests and for measuring this GEMM by itself. */
int bpdq_block_update(const float* Et, int lde, int Kd, const float* U, int ldu, int k0, float* Wp,
                      int ldw, int d_out, int c_begin, int c_end, void* stream);

/* Layers that share one input (q/k/v, up/gate) share H and U; stacked by rows they go through the
 * sweep in one call.  Every formula of the method is row-wise; only the choice of the kept
 * iterate is made per weight matrix (Sec. 3.3), so it is made per layer here:
 *   W       : the layers stacked by rows, d_out rows in all; planes / coefs / W_hat likewise.
 *   seg_end : host array of n_seg (1..8) ascending row boundaries, seg_end[n_seg-1] == d_out;
 *             every layer but the last must have a multiple of 16 rows.
 *   grp_err, grp_iter : [n_seg][d_in/g].
 * The results equal those of n_seg separate bpdq_quantize_layer calls bit for bit; the workspace
 * is bpdq_quantize_workspace_bytes(d_out, d_in, p). */
int bpdq_quantize_layers(const float* W, int d_out, int d_in, const float* U,
                         const unsigned char* dead, const bpdq_params* p /* host */, int n_seg,
                         const int* seg_end /* host */, uint32_t* planes, float* coefs,
                         float* W_hat, double* grp_err, int* grp_iter, void* ws, size_t ws_bytes,
                         void* stream);

/* ---- storage format helpers (Eq. 1) -------------------------------------------------------
 * codes : uint8 d_out x d_in, bit (i-1) of a code is B_i.  planes as above. */
int bpdq_pack_planes(const unsigned char* codes, int d_out, int d_in, int bits,
                     uint32_t* planes, void* stream);
/* W_hat[r][c] = ((C_0 + b_1 C_1) + b_2 C_2) + ... evaluated in fp32 in this order. */
int bpdq_dequant(const uint32_t* planes, const float* coefs, int d_out, int d_in, int bits,
                 int group, float* W_hat, void* stream);

/* Storage format with 16-bit coefficients: k plane bits per weight plus (k+1) halves per
 * (row, group), i.e. k + 16 (k+1) / g bits per weight (the BPW column of Table 1).
 * bpdq_coefs_to_fp16: out[i] = half(coefs[i]), round to nearest even, n values (uint16 bit
 * patterns).  bpdq_dequant_fp16: as bpdq_dequant with the coefficients read as halves; the sum
 * is evaluated in fp32 in the same order, so for a layer quantized with coef_fp16 = 1 it
 * reproduces that call's W_hat bit for bit. */
int bpdq_coefs_to_fp16(const float* coefs, long n, uint16_t* out, void* stream);
int bpdq_dequant_fp16(const uint32_t* planes, const uint16_t* coefs_h, int d_out, int d_in,
                      int bits, int group, float* W_hat, void* stream);

/* ---- serving side: y = What x for one token, straight from the stored format (Sec. 5) -------
 * Eq. 1 regrouped per (row, group G):
 *   y_r = sum_G ( C_0[r,G] S(G) + sum_i C_i[r,G] sum_{c in G} B_i[r,c] x_c ),  S(G) = sum_{c in G} x_c
 * so a weight costs no multiply: the inner sums come from a table of the 16 partial sums of every
 * 4 consecutive x values.  The planes are read once (bits/8 bytes per weight), the coefficients
 * as halves; fp32 accumulation in a fixed order.
 *   planes : as above;  coefs_h : half [bits+1][d_out][d_in/g];  x : float d_in;  y : float d_out.
 * Requirements: d_in % 32 == 0, 32 | group | d_in, x 16-byte aligned. */
int bpdq_gemv(const uint32_t* planes, const uint16_t* coefs_h, int d_out, int d_in, int bits,
              int group, const float* x, float* y, void* stream);

/* ---- channel ordering around the pass (Sec. 4.1) --------------------------------------------
 * The pass quantizes the columns left to right; a caller that wants another order permutes W and
 * H first and carries `perm` with the stored layer.
 * bpdq_channel_order: perm[i] = original index of the channel at position i.
 *   group_size = 1: channels in descending order of H_jj (GPTQ's desc_act, Sec. 4.1); equal
 *     values keep their index order.
 *   group_size = g (divides d_in): every block of g consecutive channels stays together and in
 *     order, blocks sorted by the descending sum of their H_jj (fp64, index order) -- a
 *     group-preserving stand-in for the reordering the paper's experiments take from another
 *     paper, not that method.
 *   H: d_in x d_in, only the diagonal is read.  perm: d_in ints.  ws: 8-byte aligned,
 *   bpdq_channel_order_workspace_bytes(d_in) bytes.
 * bpdq_gather_columns:   Wp[r][i] = W[r][perm[i]]            (Wp must not alias W)
 * bpdq_scatter_columns:  W[r][perm[i]] = Wp[r][i]            (inverse; e.g. W_hat back in place)
 * bpdq_gather_symmetric: Hp[i][j] = H[perm[i]][perm[j]]      (H full/symmetrized; no aliasing)
 * perm must be a permutation of 0..d_in-1 (not checked). */
size_t bpdq_channel_order_workspace_bytes(int d_in);
int bpdq_channel_order(const float* H, int d_in, int group_size, int* perm, void* ws,
                       size_t ws_bytes, void* stream);
/* bpdq_channel_order for callers that cannot allocate device memory and have no workspace to
 * hand over (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * same arguments and result, the sort keys live in a 256 KB device array built into the library
 * (one copy per GPU, held until the process ends).  No hipMalloc / hipFree, no workspace.
 *   Limit: d_in / group_size <= 32768 keys; more returns -2 and launches nothing.
 *   All calls on one GPU share that array: calls that may overlap on one GPU (different streams,
 *   different host threads) race and must be serialised by the caller.  Nothing of an earlier
 *   call's contents enters a later result.
 * Returns 0, -1 H, -2 d_in (or too many keys), -3 group_size, -4 perm, BPDQ_ERR_LAUNCH. */
int bpdq_channel_order_noalloc(const float* H, int d_in, int group_size, int* perm, void* stream);
int bpdq_gather_columns(const float* W, int d_out, int d_in, const int* perm, float* Wp,
                        void* stream);
int bpdq_scatter_columns(const float* Wp, int d_out, int d_in, const int* perm, float* W,
                         void* stream);
int bpdq_gather_symmetric(const float* H, int d_in, const int* perm, float* Hp, void* stream);

/* ---- measurement probes (not part of the method) ---------------------------------------------
 * Ceilings of the GPU the library runs on, for quoting a kernel against what the hardware
 * sustains as well as against its published peak.
 * bpdq_probe_mfma: a register-only loop of one matrix-core instruction, no memory traffic:
 *   kind 0 v_mfma_f32_32x32x2_f32, 1 v_mfma_f32_32x32x16_bf16, 2 v_mfma_f32_32x32x16_f16,
 *   3 v_mfma_f64_16x16x4_f64, 4 v_mfma_i32_32x32x32_i8 (ops instead of flops; normal operands are
 *   round(32 z) clamped to +-127);  data 0 zeros, 1 ones, 2 standard normal operand values (the
 *   sustained clock depends on the operand bits that toggle);  waves_per_simd 1 or 2;
 *   `groups` work-groups (256 = one per compute unit) of 4 * waves_per_simd wavefronts, each
 *   issuing 8 * iters instructions on a 2 x 4 grid of independent accumulator tiles (fp64: 16 * iters
 *   on 4 x 4).
 *   out: device floats, groups * 256 * waves_per_simd of them (keeps the results alive).
 *   flops (host, may be NULL): receives the flops the launch performs.  Time it with events.
 * bpdq_probe_copy: dst[i] = src[i], n_floats (multiple of 4) floats, 16-byte aligned: the plain
 *   streaming copy HBM counters and bandwidth are scaled by. */
int bpdq_probe_mfma(int kind, int data, int waves_per_simd, int groups, int iters, float* out,
                    double* flops /* host */, void* stream);
int bpdq_probe_copy(const float* src, float* dst, long n_floats, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BPDQ_H */
