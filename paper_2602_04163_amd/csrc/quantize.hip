// Steps 3-4 of the pass, host side: the loop over blocks and groups (paper Sec. 3.2, 3.3) with
// the schedule of the lazy block updates (Eq. 4 applied to whole blocks; App. B.3 tail form) and
// the storage helpers.  The per-group kernels live in group_sweep.h.
#include "group_sweep.h"

namespace bpdq {

// The lazy block update as a launch of its own (group sizes whose sweep kernel cannot share a CU
// with it): the same tail role, one 128 x 128 tile per work-group.
__global__ __launch_bounds__(TailGemm::kThreads) void tail_update_kernel(TailArgs ta, const float* __restrict__ U,
                                                                         int ldu, int lde, int ldw, int d_out) {
  tail_role(ta, U, ldu, lde, ldw, d_out);
}

int launch_tail_update(hipStream_t stream, TailArgs ta, const float* U, int ldu, int lde, int ldw,
                       int d_out, int n_tiles) {
  BPDQ_HIP_TRY(bpdq_lds_limit<&tail_update_kernel>(TailGemm::kLdsBytes));
  ta.first_wg = 0;
  ta.far_wgs = bpdq_ceil_div(lde, TailGemm::kTileM) * ta.far.tiles_n;
  hipLaunchKernelGGL(tail_update_kernel, dim3(n_tiles), dim3(TailGemm::kThreads), TailGemm::kLdsBytes,
                     stream, ta, U, ldu, lde, ldw, d_out);
  BPDQ_LAUNCH_CHECK();
  return 0;
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

__device__ __forceinline__ float coef_value(float c) { return c; }
__device__ __forceinline__ float coef_value(_Float16 c) { return (float)c; }

// Eq. 1 from the packed format, ((C_0 + b_1 C_1) + b_2 C_2) + ... in fp32; CT = float or half
template <typename CT>
__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t* __restrict__ planes,
                                                      const CT* __restrict__ coefs, int d_out,
                                                      int d_in, int bits, int group,
                                                      float* __restrict__ W_hat) {
  const int n_word = d_in / 32, n_grp = d_in / group;
  const long n = (long)d_out * d_in;
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
    const int r = (int)(e / d_in), c = (int)(e % d_in);
    const int gi = c / group;
    float v = coef_value(coefs[(long)r * n_grp + gi]);
    for (int i = 0; i < bits; ++i) {
      const uint32_t w = planes[((long)i * d_out + r) * n_word + c / 32];
      if ((w >> (c & 31)) & 1u) v = v + coef_value(coefs[((long)(i + 1) * d_out + r) * n_grp + gi]);
    }
    W_hat[e] = v;
  }
}

__global__ __launch_bounds__(256) void coefs_to_fp16_kernel(const float* __restrict__ coefs, long n,
                                                            _Float16* __restrict__ out) {
  for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256)
    out[e] = (_Float16)coefs[e];                 // v_cvt_f16_f32: round to nearest even
}

// ------------------------------------------------------------------ host side --------------
static int check_params(int d_out, int d_in, const bpdq_params* p) {
  if (!p) return 1;
  if (p->bits < 1 || p->bits > 4) return 1;
  if (p->group != 32 && p->group != 64 && p->group != 128 && p->group != 256) return 1;
  if (p->group == 256 && p->bits > 3) return 1;      // 4 planes at g = 256 are not built (see header)
  if (d_in % p->group || d_in % 32) return 1;
  const int B = p->block > p->group ? p->block : p->group;
  if (p->block < 1 || B % p->group) return 1;
  if (p->refine_iters < 0 || p->refine_iters > 63) return 1;
  if (!(p->alpha >= 0.f)) return 1;
  if (p->grid != BPDQ_GRID_VARIABLE && p->grid != BPDQ_GRID_UNIFORM) return 1;
  if (p->coef_fp16 != 0 && p->coef_fp16 != 1) return 1;
  if (d_out <= 0 || d_in <= 0) return 1;
  return 0;
}

static GroupLauncher pick_group(int k, int g) {
  if (g == 256) {
    switch (k) {
      case 1: return group256_k1();
      case 2: return group256_k2();
      case 3: return group256_k3();
    }
    return nullptr;
  }
  switch (k) {
    case 1: return pick_group_k1(g);
    case 2: return pick_group_k2(g);
    case 3: return pick_group_k3(g);
    case 4: return pick_group_k4(g);
  }
  return nullptr;
}

}  // namespace bpdq

using namespace bpdq;

extern "C" int bpdq_version(void) { return 100; }

extern "C" size_t bpdq_quantize_workspace_bytes(int d_out, int d_in, const bpdq_params* p) {
  if (check_params(d_out, d_in, p)) return 0;
  return quant_layout(d_out, d_in, *p).total;
}

static int quantize_rows(const float* W, int d_out, int d_in, const float* U,
                         const unsigned char* dead, const bpdq_params* p, const SegArgs& seg,
                         uint32_t* planes, float* coefs, float* W_hat, double* grp_err,
                         int* grp_iter, void* ws, size_t ws_bytes, hipStream_t stream) {
  const QuantLayout L = quant_layout(d_out, d_in, *p);
  if (ws_bytes < L.total) return -13;
  char* base = static_cast<char*>(ws);
  float* Wp = reinterpret_cast<float*>(base + L.wp_off);
  float* Eall = reinterpret_cast<float*>(base + L.eall_off);
  GroupLauncher group = pick_group(p->bits, p->group);
  if (!group) return -6;

  const long n = (long)d_out * d_in;
  const int grid = (int)((n / 4 + 255) / 256 < 65536 ? (n / 4 + 255) / 256 : 65536);
  hipLaunchKernelGGL(copy_in_kernel, dim3(grid), dim3(256), 0, stream, W, n, d_in, dead, Wp);
  BPDQ_LAUNCH_CHECK();

  // Blocks of B columns, groups of g inside.  W' only ever receives whole-block updates, one
  // block late: the first group launch of block q carries the update of block q-1 to the columns
  // beyond block q (tail role), and every group of block q reads the updates of block q-1 and of
  // the earlier groups of its own block left-looking from the committed E*.
  // Two levels (see TailArgs): with super-blocks of SBc columns, the update of a block of
  // super-block S reaches only to the end of super-block S + 1; the columns from super-block S + 2
  // on receive ONE update of depth SBc for all of super-block S, applied during the launches of
  // super-block S + 1: its first launch takes the columns of super-block S + 2 (the per-block
  // update of that launch, from the last block of S, ends where they begin), the other launches
  // share the columns beyond (which no per-block update of super-block S + 1 reaches).  Two
  // updates of one launch thus never meet, and a column has received every earlier block's term
  // before its own block starts.
  const int g = p->group, B = L.B;
  const int SBc = B >= 1024 ? B : B * (1024 / B);
  auto make_task = [&](int k0, int Kd, long c0, long c1) {
    TailTask t{};
    c0 = c0 < d_in ? c0 : d_in;
    c1 = c1 < d_in ? c1 : d_in;
    if (c1 > c0) {
      t.Et = Eall + (long)k0 * L.lde;
      t.Kd = Kd;
      t.k0 = k0;
      t.c_begin = (int)c0;
      t.c_end = (int)c1;
      t.tiles_n = bpdq_ceil_div((int)(c1 - c0), TailGemm::kTileN);
    }
    return t;
  };
  for (int b0 = 0; b0 < d_in; b0 += B) {
    const int b1 = b0 + B < d_in ? b0 + B : d_in;
    const int kp0 = b0 > 0 ? b0 - B : 0;
    const int sb0 = b0 / SBc * SBc;                         // start of this block's super-block
    for (int s0 = b0; s0 < b1; s0 += g) {
      TailArgs ta{};
      ta.Wp = Wp;
      if (s0 == b0 && b0 > 0)     // per-block update of block q-1: to the end of the super-block after its own
        ta.near = make_task(kp0, B, b1, ((long)(kp0 / SBc) + 2) * SBc);
      if (sb0 > 0) {
        // deep update of the previous super-block [sb0 - SBc, sb0), columns from sb0 + SBc on
        const int li = (s0 - sb0) / g, n_l = SBc / g;
        const long f0 = (long)sb0 + SBc, f1 = f0 + SBc;      // the next super-block's columns
        if (li == 0) {
          ta.far = make_task(sb0 - SBc, SBc, f0, f1);
        } else if (f1 < d_in) {
          const int cols = bpdq_ceil_div(bpdq_ceil_div(d_in - (int)f1, TailGemm::kTileN), n_l - 1) * TailGemm::kTileN;
          ta.far = make_task(sb0 - SBc, SBc, f1 + (long)(li - 1) * cols, f1 + (long)li * cols);
        }
      }
      const int rc = group(stream, Wp, d_out, d_in, U, s0, kp0, ta, seg, *p, L, base, planes, coefs,
                           W_hat, grp_err, grp_iter);
      if (rc) return rc;
    }
  }
  return 0;
}

extern "C" int bpdq_quantize_layer(const float* W, int d_out, int d_in, const float* U,
                                   const unsigned char* dead, const bpdq_params* p,
                                   uint32_t* planes, float* coefs, float* W_hat, double* grp_err,
                                   int* grp_iter, void* ws, size_t ws_bytes, void* stream_) {
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
  SegArgs seg{};
  seg.n_seg = 1;
  seg.wg_end[0] = bpdq_ceil_div(d_out, kRowsPerWG);
  return quantize_rows(W, d_out, d_in, U, dead, p, seg, planes, coefs, W_hat, grp_err, grp_iter, ws,
                       ws_bytes, static_cast<hipStream_t>(stream_));
}

extern "C" int bpdq_quantize_layers(const float* W, int d_out, int d_in, const float* U,
                                    const unsigned char* dead, const bpdq_params* p, int n_seg,
                                    const int* seg_end, uint32_t* planes, float* coefs,
                                    float* W_hat, double* grp_err, int* grp_iter, void* ws,
                                    size_t ws_bytes, void* stream_) {
  if (!W || (reinterpret_cast<uintptr_t>(W) & 15)) return -1;
  if (d_out <= 0) return -2;
  if (d_in <= 0 || d_in % 32) return -3;
  if (!U || (reinterpret_cast<uintptr_t>(U) & 15)) return -4;
  if (check_params(d_out, d_in, p)) return -6;
  if (n_seg < 1 || n_seg > kMaxSegments) return -7;
  if (!seg_end) return -8;
  SegArgs seg{};
  seg.n_seg = n_seg;
  int prev = 0;
  for (int s = 0; s < n_seg; ++s) {
    const int e = seg_end[s];
    // every layer but the last must end on a work-group boundary (16 rows)
    if (e <= prev || e > d_out || (s + 1 < n_seg && e % kRowsPerWG)) return -8;
    seg.wg_end[s] = bpdq_ceil_div(e, kRowsPerWG);
    prev = e;
  }
  if (prev != d_out) return -8;
  if (!planes) return -9;
  if (!coefs) return -10;
  if (!grp_err) return -12;
  if (!grp_iter) return -13;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255)) return -14;
  const int rc = quantize_rows(W, d_out, d_in, U, dead, p, seg, planes, coefs, W_hat, grp_err,
                               grp_iter, ws, ws_bytes, static_cast<hipStream_t>(stream_));
  return rc == -13 ? -15 : rc;
}

extern "C" int bpdq_block_update(const float* Et, int lde, int Kd, const float* U, int ldu, int k0,
                                 float* Wp, int ldw, int d_out, int c_begin, int c_end, void* stream_) {
  if (!Et || (reinterpret_cast<uintptr_t>(Et) & 15)) return -1;
  if (lde < d_out || lde % 4) return -2;
  if (Kd <= 0) return -3;
  if (!U || (reinterpret_cast<uintptr_t>(U) & 15)) return -4;
  if (ldu < c_end || ldu % 4) return -5;
  if (k0 < 0) return -6;
  if (!Wp) return -7;
  if (ldw < c_end) return -8;
  if (d_out <= 0) return -9;
  if (c_begin < 0 || c_begin % 4) return -10;
  if (c_end < c_begin || c_end % 4) return -11;
  if (c_end == c_begin) return 0;
  TailArgs ta{};
  ta.Wp = Wp;
  ta.near.Et = Et;
  ta.near.Kd = Kd;
  ta.near.k0 = k0;
  ta.near.c_begin = c_begin;
  ta.near.c_end = c_end;
  ta.near.tiles_n = bpdq_ceil_div(c_end - c_begin, TailGemm::kTileN);
  const int n_tiles = bpdq_ceil_div(lde, TailGemm::kTileM) * ta.near.tiles_n;
  return launch_tail_update(static_cast<hipStream_t>(stream_), ta, U, ldu, lde, ldw, d_out, n_tiles);
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

static int launch_dequant(const uint32_t* planes, const void* coefs, bool half, int d_out, int d_in,
                          int bits, int group, float* W_hat, hipStream_t stream) {
  if (!planes) return -1;
  if (!coefs) return -2;
  if (d_out <= 0) return -3;
  if (d_in <= 0 || d_in % 32) return -4;
  if (bits < 1 || bits > 4) return -5;
  if (group <= 0 || d_in % group) return -6;
  if (!W_hat) return -7;
  const long n = (long)d_out * d_in;
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  if (half) {
    hipLaunchKernelGGL(dequant_kernel<_Float16>, dim3(grid), dim3(256), 0, stream, planes,
                       static_cast<const _Float16*>(coefs), d_out, d_in, bits, group, W_hat);
  } else {
    hipLaunchKernelGGL(dequant_kernel<float>, dim3(grid), dim3(256), 0, stream, planes,
                       static_cast<const float*>(coefs), d_out, d_in, bits, group, W_hat);
  }
  BPDQ_LAUNCH_CHECK();
  return 0;
}

extern "C" int bpdq_dequant(const uint32_t* planes, const float* coefs, int d_out, int d_in,
                            int bits, int group, float* W_hat, void* stream_) {
  return launch_dequant(planes, coefs, false, d_out, d_in, bits, group, W_hat,
                        static_cast<hipStream_t>(stream_));
}

extern "C" int bpdq_dequant_fp16(const uint32_t* planes, const uint16_t* coefs_h, int d_out,
                                 int d_in, int bits, int group, float* W_hat, void* stream_) {
  if (coefs_h && (reinterpret_cast<uintptr_t>(coefs_h) & 1)) return -2;
  return launch_dequant(planes, coefs_h, true, d_out, d_in, bits, group, W_hat,
                        static_cast<hipStream_t>(stream_));
}

extern "C" int bpdq_coefs_to_fp16(const float* coefs, long n, uint16_t* out, void* stream_) {
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if (n < 0) return -2;
  if (n == 0) return 0;
  if (!coefs) return -1;
  if (!out || (reinterpret_cast<uintptr_t>(out) & 1)) return -3;
  const int grid = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  hipLaunchKernelGGL(coefs_to_fp16_kernel, dim3(grid), dim3(256), 0, stream, coefs, n,
                     reinterpret_cast<_Float16*>(out));
  BPDQ_LAUNCH_CHECK();
  return 0;
}
