// canz_soap_step / canz_soap_workspace_bytes: the SOAP step the paper runs through the same
// planner as Muon and Shampoo ("Generalization to Other Optimizers (Shampoo & SOAP)", App. C;
// App. B.3), per matrix (Adam in the eigenbasis of Shampoo's statistics):
//   M <- beta1 M + (1 - beta1) G;   G' = Q_L^T G Q_R,  M' = Q_L^T M Q_R;
//   V <- beta2 V + (1 - beta2) G'^2;   N' = m / (sqrt(v) + eps);   N = Q_L N' Q_R^T;
//   P <- P (1 - lr wd) - lr N  (or Delta W = -lr N);
//   L <- beta2 L + (1 - beta2) G G^T,  R <- beta2 R + (1 - beta2) G^T G;
//   on a refresh step  Q_L <- orthogonal factor of QR(L Q_L),  Q_R likewise.
// State and sums are fp32; the products run on v_mfma_f32_32x32x2_f32, with two exceptions on the bf16 matrix
// cores (the kernels of the Muon step, operands in its panel layout): the statistics of gradients that arrive as
// bf16 (their own values are the operands, every product is exact in fp32, the sums stay fp32), and, if the caller
// asks for it (bf16_rotations), the rotations with the bases, M and N' rounded to bf16.
//
// The products all take the form C[i][j] = sum_k P[i][k] Q[j][k].  The rotation into the basis
// runs right side first with its result written transposed, (G Q_R)^T = Q_R^T-rows times G-rows,
// so that the left side finds its second operand contiguous along k; the rotation back runs
// the same way round.  G and M travel through the rotation as two problems of one launch that
// share the basis operand; with a rotated momentum kept by the caller (mom_rot) only G is rotated
// and M' follows M' <- beta1 M' + (1 - beta1) G' in the Adam kernel.
//
// QR refresh: blocked Householder factorisation with panels of 32 columns, on the transposed
// matrix (a column of S = L Q is a contiguous row of the working copy).  Per panel: one workgroup
// per matrix finds the 32 reflectors (each wavefront owns whole columns of the panel, so the only
// block-wide synchronisation is two barriers per column), a second kernel forms the compact WY
// factors H = I - V T V^T, Y = V T^T, Y2 = V T, and two products update the trailing columns:
//   W = (columns) V,  (columns) -= W Y^T.
// Afterwards the orthogonal factor is accumulated from the last panel to the first with the same
// two products (and Y2).  Tile boundaries of these products are rounded down to multiples of 128;
// the extra rows and columns they touch either hold zeros in V (no effect) or are columns the
// factorisation has finished with (R is never needed: only Q is).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "canz.h"
#include "canz_internal.h"
#include "device_util.h"
#include "f32_mfma_gemm.h"
#include "kernels.h"
#include "panel_layout.h"

namespace canz {
namespace {

using namespace f32mfma;

constexpr int64_t MAX_EXTENT = 32768;
constexpr size_t BATCH_BYTES = size_t(32) << 30;   // working matrices of one launch batch: the more matrices share
                                                     // a batch, the more workgroups the panel kernel of a refresh has
constexpr int QB = 32;            // panel width of the QR factorisation
constexpr int QTH = 1024;         // threads of the panel kernel: 16 wavefronts
constexpr int QWAVES = QTH / 64;

// Where k_soap_load leaves its results: fp32 working copies and / or bf16 images in the panel layout
// (panel_layout.h; padded to multiples of 256, operands of the bf16 MFMA kernels), each in both orientations.
struct LoadOut {
  float *gm, *gmt;               // fp32: gm [nb][2][rp][cp] (G, then M) and gmt [nb][2][cp][rp]
  bool g32, m32;                 // which of their two planes are wanted
  __bf16 *gp, *gpt, *mp, *mpt;   // bf16 panels: G [nb][rp2][cp2], G^T [nb][cp2][rp2], M, M^T; nullptr: not wanted
  int64_t rp2, cp2;
};

// one 64 x 64 fp32 tile in LDS -> the 8-element chunks of its bf16 panel image, straight (dst rows = tile rows) or
// transposed (dst rows = tile columns); (r0, c0): the tile's place in the matrix, kc: row length of the image
__device__ __forceinline__ void tile_to_panels(const float (*tile)[65], __bf16* __restrict__ dst, int64_t r0, int64_t c0,
                                               int64_t kc, bool transposed, int t) {
  const int cv = (t & 7) * 8;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int rl = (t >> 3) + half * 32;
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(transposed ? tile[cv + e][rl] : tile[rl][cv + e]);
    *reinterpret_cast<bf16x8*>(dst + (transposed ? panel_chunk_off(c0 + rl, r0 + cv, kc) : panel_chunk_off(r0 + rl, c0 + cv, kc))) = o;
  }
}

// G (bf16 or fp32, whole or tp column fragments) and the momentum M <- beta1 M + (1 - beta1) G
// (fp32, dense, in the caller's buffer) -> working copies of both as `w` asks, zero outside rows x cols.
// One block per 64 x 64 tile of the padded matrix (padded to 256 if a bf16 image is wanted, else to 128).
// VEC: cols and cols / tp are multiples of 8, so a lane's 8 consecutive elements lie in one fragment and every
// access of the caller's arrays is a 16-byte vector.
template <bool VEC>
__global__ __launch_bounds__(NTH) void k_soap_load(Shape s, PtrTable grad, int grad_dtype, PtrTable mom, float beta1,
                                                    int64_t rp, int64_t cp, LoadOut w) {
  __shared__ float tg[64][65], tm[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const int wf = static_cast<int>(s.wfrag);
  const int64_t plane = rp * cp;
  float* gs = w.gm + static_cast<int64_t>(b) * 2 * plane;
  float* gt = w.gmt + static_cast<int64_t>(b) * 2 * plane;
  float* m = static_cast<float*>(mom.p[b]);
  if (VEC) {
    const int cv = (t & 7) * 8;
    f32x4 gv[2][2], mv[2][2];
    bool live[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {   // all loads first: the tables may alias as far as the compiler knows
      const int row = r0 + (t >> 3) + half * 32, col = c0 + cv;
      live[half] = row < s.rows && col < s.cols;
      gv[half][0] = gv[half][1] = mv[half][0] = mv[half][1] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (!live[half]) continue;
      const int f = col / wf;
      const int64_t at = static_cast<int64_t>(row) * wf + (col - f * wf);
      if (grad_dtype == CANZ_DT_BF16) {
        const bf16x8 g8 = *reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(grad.p[b * s.tp + f]) + at);
#pragma unroll
        for (int e = 0; e < 4; ++e) gv[half][0][e] = static_cast<float>(g8[e]), gv[half][1][e] = static_cast<float>(g8[4 + e]);
      } else {
        const f32x4* g4 = reinterpret_cast<const f32x4*>(static_cast<const float*>(grad.p[b * s.tp + f]) + at);
        gv[half][0] = g4[0], gv[half][1] = g4[1];
      }
      const f32x4* m4 = reinterpret_cast<const f32x4*>(m + static_cast<int64_t>(row) * s.cols + col);
      mv[half][0] = m4[0], mv[half][1] = m4[1];
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int rl = (t >> 3) + half * 32, row = r0 + rl, col = c0 + cv;
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          mv[half][q][e] = live[half] ? __builtin_fmaf(beta1, mv[half][q][e], (1.f - beta1) * gv[half][q][e]) : 0.f;
          tg[rl][cv + 4 * q + e] = gv[half][q][e];
          tm[rl][cv + 4 * q + e] = mv[half][q][e];
        }
      if (live[half]) {
        f32x4* m4 = reinterpret_cast<f32x4*>(m + static_cast<int64_t>(row) * s.cols + col);
        m4[0] = mv[half][0], m4[1] = mv[half][1];
      }
      if (row < rp && col < cp) {
        if (w.g32) {
          f32x4* o = reinterpret_cast<f32x4*>(gs + static_cast<int64_t>(row) * cp + col);
          o[0] = gv[half][0], o[1] = gv[half][1];
        }
        if (w.m32) {
          f32x4* o = reinterpret_cast<f32x4*>(gs + plane + static_cast<int64_t>(row) * cp + col);
          o[0] = mv[half][0], o[1] = mv[half][1];
        }
      }
    }
  } else {
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int row = r0 + r, col = c0 + c;
    float g = 0.f, mv = 0.f;
    if (row < s.rows && col < s.cols) {
      const int f = col / wf;
      const int64_t at = static_cast<int64_t>(row) * wf + (col - f * wf);
      g = grad_dtype == CANZ_DT_BF16 ? static_cast<float>(static_cast<const __bf16*>(grad.p[b * s.tp + f])[at])
                                     : static_cast<const float*>(grad.p[b * s.tp + f])[at];
      const int64_t am = static_cast<int64_t>(row) * s.cols + col;
      mv = __builtin_fmaf(beta1, m[am], (1.f - beta1) * g);
      m[am] = mv;
    }
    if (row < rp && col < cp) {
      if (w.g32) gs[static_cast<int64_t>(row) * cp + col] = g;
      if (w.m32) gs[plane + static_cast<int64_t>(row) * cp + col] = mv;
    }
    tg[r][c] = g;
    tm[r][c] = mv;
  }
  }
  __syncthreads();
  if (w.g32 || w.m32) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;  // r: column of G, c: row of G
      if (c0 + r < cp && r0 + c < rp) {
        if (w.g32) gt[static_cast<int64_t>(c0 + r) * rp + r0 + c] = tg[c][r];
        if (w.m32) gt[plane + static_cast<int64_t>(c0 + r) * rp + r0 + c] = tm[c][r];
      }
    }
  }
  const int64_t p2 = static_cast<int64_t>(b) * w.rp2 * w.cp2;
  if (w.gp) tile_to_panels(tg, w.gp + p2, r0, c0, w.cp2, false, t);
  if (w.gpt) tile_to_panels(tg, w.gpt + p2, r0, c0, w.rp2, true, t);
  if (w.mp) tile_to_panels(tm, w.mp + p2, r0, c0, w.cp2, false, t);
  if (w.mpt) tile_to_panels(tm, w.mpt + p2, r0, c0, w.rp2, true, t);
}

// Adam in the rotated space.  rot [nb][2][rp][cp] holds G' and (unless `incremental`) M'; V (dense,
// caller's) is updated in place; N' = (c1 M') / (sqrt(c2 V) + eps) goes to np [nb][rp][cp], or
// transposed to [nb][cp][rp]; zero outside rows x cols.  If the caller keeps the rotated momentum
// (`keep`, dense, mrot): incremental: M' = beta1 mrot + (1 - beta1) G'; either way mrot <- M'.
__global__ __launch_bounds__(NTH) void k_soap_adam(Shape s, PtrTable var, PtrTable mrot, bool keep, bool incremental,
                                                    const float* __restrict__ rot, int64_t rp, int64_t cp, float beta1,
                                                    float beta2, float c1, float c2, float eps, int transposed,
                                                    float* __restrict__ np) {
  __shared__ float tile[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const int64_t plane = rp * cp;
  const float* gr = rot + static_cast<int64_t>(b) * 2 * plane;
  float* v = static_cast<float*>(var.p[b]);
  float* out = np + static_cast<int64_t>(b) * plane;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int row = r0 + r, col = c0 + c;
    float n = 0.f;
    if (row < s.rows && col < s.cols) {
      const int64_t at = static_cast<int64_t>(row) * cp + col, av = static_cast<int64_t>(row) * s.cols + col;
      const float g = gr[at];
      float* mr = static_cast<float*>(mrot.p[b]);
      const float m = incremental ? __builtin_fmaf(beta1, mr[av], (1.f - beta1) * g) : gr[plane + at];
      if (keep) mr[av] = m;
      const float vn = __builtin_fmaf(beta2, v[av], (1.f - beta2) * (g * g));
      v[av] = vn;
      n = (c1 * m) / (sqrtf(c2 * vn) + eps);
    }
    if (transposed)
      tile[r][c] = n;
    else
      out[static_cast<int64_t>(row) * cp + col] = n;
  }
  if (!transposed) return;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    out[static_cast<int64_t>(c0 + r) * rp + r0 + c] = tile[c][r];
  }
}

// The caller's basis Q (d x d, dense fp32) -> padded working copies in both orientations, zero outside d x d: fp32
// [dp][dp] (if `f32`) and / or bf16 panels [dp2][dp2] (if given).  One block per 64 x 64 tile of the larger padding.
__global__ __launch_bounds__(NTH) void k_soap_load_basis(PtrTable q, int64_t d, int64_t dp, bool f32, float* __restrict__ straight,
                                                          float* __restrict__ transposed, int64_t dp2, __bf16* __restrict__ sp,
                                                          __bf16* __restrict__ tp) {
  __shared__ float tile[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const float* src = static_cast<const float*>(q.p[b]);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int64_t row = r0 + r, col = c0 + c;
    const float val = row < d && col < d ? src[row * d + col] : 0.f;
    if (f32 && row < dp && col < dp) straight[(b * dp + row) * dp + col] = val;
    tile[r][c] = val;
  }
  __syncthreads();
  if (f32) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;  // r: column of Q, c: row of Q
      if (c0 + r < dp && r0 + c < dp) transposed[(b * dp + c0 + r) * dp + r0 + c] = tile[c][r];
    }
  }
  if (sp) tile_to_panels(tile, sp + b * dp2 * dp2, r0, c0, dp2, false, t);
  if (tp) tile_to_panels(tile, tp + b * dp2 * dp2, r0, c0, dp2, true, t);
}

inline int64_t pad256(int64_t x) { return (x + PAD - 1) / PAD * PAD; }

// Adam in the rotated space on bf16 panels: G' (and, unless `incremental`, M') [rp2][cp2] panels in, N' panels
// out, straight [rp2][cp2] and / or transposed [cp2][rp2], zero outside rows x cols; V and the kept rotated
// momentum are the caller's dense fp32 arrays as in k_soap_adam.  One block per 64 x 64 tile: the panel chunks
// (8 consecutive elements of a row) go through LDS so that the dense fp32 arrays are read and written with one
// row of 64 elements per wavefront, whatever the row length of the caller's matrix.
__global__ __launch_bounds__(NTH) void k_soap_adam_bf16(Shape s, PtrTable var, PtrTable mrot, bool keep, bool incremental,
                                                         const __bf16* __restrict__ grot, const __bf16* __restrict__ mrot_p,
                                                         int64_t rp2, int64_t cp2, float beta1, float beta2, float c1,
                                                         float c2, float eps, __bf16* __restrict__ n_straight,
                                                         __bf16* __restrict__ n_transposed) {
  __shared__ float tg[64][65], tm[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const int64_t plane = rp2 * cp2;
  const __bf16* gp = grot + static_cast<int64_t>(b) * plane;
  float* v = static_cast<float*>(var.p[b]);
  float* mr = static_cast<float*>(mrot.p[b]);
  const int cv = (t & 7) * 8;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int rl = (t >> 3) + half * 32;
    const int64_t at = panel_chunk_off(r0 + rl, c0 + cv, cp2);
    const bf16x8 g8 = *reinterpret_cast<const bf16x8*>(gp + at);
#pragma unroll
    for (int e = 0; e < 8; ++e) tg[rl][cv + e] = static_cast<float>(g8[e]);
    if (!incremental) {
      const bf16x8 m8 = *reinterpret_cast<const bf16x8*>(mrot_p + static_cast<int64_t>(b) * plane + at);
#pragma unroll
      for (int e = 0; e < 8; ++e) tm[rl][cv + e] = static_cast<float>(m8[e]);
    }
  }
  __syncthreads();
  float vo[16], mo[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) {   // all old values first: one memory latency for the tile
    const int idx = e * NTH + t, row = r0 + (idx >> 6), col = c0 + (idx & 63);
    const bool in = row < s.rows && col < s.cols;
    const int64_t av = static_cast<int64_t>(row) * s.cols + col;
    vo[e] = in ? v[av] : 0.f;
    mo[e] = in && incremental ? mr[av] : 0.f;
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63, row = r0 + r, col = c0 + c;
    float n = 0.f;
    if (row < s.rows && col < s.cols) {
      const int64_t av = static_cast<int64_t>(row) * s.cols + col;
      const float g = tg[r][c];
      const float m = incremental ? __builtin_fmaf(beta1, mo[e], (1.f - beta1) * g) : tm[r][c];
      if (keep) mr[av] = m;
      const float vn = __builtin_fmaf(beta2, vo[e], (1.f - beta2) * (g * g));
      v[av] = vn;
      n = (c1 * m) / (sqrtf(c2 * vn) + eps);
    }
    tg[r][c] = n;   // the element this thread read
  }
  __syncthreads();
  if (n_straight) tile_to_panels(tg, n_straight + static_cast<int64_t>(b) * plane, r0, c0, cp2, false, t);
  if (n_transposed) tile_to_panels(tg, n_transposed + static_cast<int64_t>(b) * plane, r0, c0, rp2, true, t);
}

// S[row][col] <- S[col][row] for row > col of the caller's dense d x d matrices: the symmetric statistic is computed
// on and above the diagonal tiles only.  One block per 64 x 64 tile on or below the diagonal (blockIdx.y >= blockIdx.x).
__global__ __launch_bounds__(NTH) void k_soap_mirror(PtrTable stat, int64_t d) {
  __shared__ float tile[64][65];
  if (blockIdx.y < blockIdx.x) return;
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  float* m = static_cast<float*>(stat.p[b]);
#pragma unroll
  for (int e = 0; e < 16; ++e) {   // the tile above the diagonal that mirrors this one: rows c0.., columns r0..
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int64_t row = c0 + r, col = r0 + c;
    tile[r][c] = row < d && col < d ? m[row * d + col] : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int64_t row = r0 + r, col = c0 + c;
    if (row < d && col < row) m[row * d + col] = tile[c][r];
  }
}

// a[b][i] = (identity ? (row == col) : 0) for the [rows][ld] matrices of a batch
__global__ __launch_bounds__(NTH) void k_soap_fill(float* __restrict__ a, int64_t elems, int64_t ld, int identity) {
  float* ab = a + static_cast<int64_t>(blockIdx.y) * elems;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * NTH + threadIdx.x; i < elems; i += static_cast<int64_t>(gridDim.x) * NTH)
    ab[i] = identity && (i / ld) == (i % ld) ? 1.f : 0.f;
}

// Caller's basis Q (d x d, dense, columns are the vectors) <- the transposed working copy qt [dp][dp].
__global__ __launch_bounds__(NTH) void k_soap_store_q(PtrTable q, const float* __restrict__ qt, int64_t d, int64_t dp) {
  __shared__ float tile[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const float* src = qt + static_cast<int64_t>(b) * dp * dp;
  float* dst = static_cast<float*>(q.p[b]);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    tile[r][c] = src[static_cast<int64_t>(r0 + r) * dp + c0 + c];   // qt[col of Q][row of Q]
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int row = c0 + r, col = r0 + c;                          // row / column of Q
    if (row < d && col < d) dst[static_cast<int64_t>(row) * d + col] = tile[c][r];
  }
}

// One panel of the Householder QR factorisation: columns j0 .. j0 + 31 of the matrix whose
// column c is row c of wk (row length dp).  One workgroup of 16 wavefronts per matrix, two kernels.
// The first finds the reflectors:
//   vall row j0 + c  <- reflector v_c (zero before row j0 + c, 1 there),   tau[c] <- tau_c
// updating the panel's later columns as each reflector is found.  Columns at or beyond d (padding)
// and columns that are already zero below the diagonal get tau = 0 (H = I).  The second
// (k_qr_tfactor) accumulates V V^T (32 x 32, which T needs) on the matrix cores, each wavefront
// taking every 16th group of 32 rows, sums over the wavefronts in a fixed order, forms T column by
// column (H_0 ... H_31 = I - V T V^T), and writes
//   ybuf [dp][128]   <- Y  = V T^T, rows klo .. dp - 1   (H^T A = A - Y (V^T A))
//   y2   [dp][128]   <- Y2 = V T                          (H A = A - Y2 (V^T A)),
// both into the 32 columns `ycol`.. of a strip that holds the four panels of a block of 128 columns side by side.
//
// Blocks.  The four panels of a block are applied to the rows beyond the block in one go: with W_raw = X [V_0 .. V_3]
// (X: the rows to update), the W of panel b applied after panels a < b is W_b = W_raw,b - sum_{a<b} W_a C_ab,
// C_ab = Y_a^T V_b = T_a (V_a^T V_b), i.e. W = W_raw U with U = (I + C)^(-1), C strictly block upper triangular; then
// X -= W [Y_0 .. Y_3]^T.  When the orthogonal factor is accumulated the panels are applied last to first with Y2:
// W = W_raw U2, U2 = (I + C2)^(-1), C2_ab = Y2_a^T V_b = T_a^T (V_a^T V_b) for a > b.  k_qr_tfactor of panel `pos`
// of a block also forms V_a^T V_pos for the earlier panels a of the block and writes the blocks C_a,pos and
// C2_pos,a (it reads T_a from tbuf, where every panel leaves its T); k_qr_block_u turns them into U^T and U2^T.
//
// Column c2 of the panel belongs to wavefront (c2 - 1) mod 16 for the whole kernel: it alone reads and
// writes that column, so the columns need no synchronisation between wavefronts.  What the others
// need of step c is the reflector v_c, which its owner leaves in LDS (a basis has at most VMAX rows)
// together with tau_c.  Per step: every wavefront applies H_c to its own
// later columns; barrier; the owner of column c + 1 turns it into v_(c+1); barrier.  With v in LDS the
// barriers only have to order LDS traffic, so they do not wait for the stores in flight.
// Up to 3072 remaining rows the columns stay in registers for the whole kernel (k_qr_panel_regs);
// k_qr_panel_hybrid, for longer panels, keeps the first 2048 rows there and streams the rest from memory (L2) on every step.
constexpr int QBLK = 128;   // columns of a block: four panels
struct QrPanel {
  float* wk;
  float* vall;
  float* ybuf;     // this block's Y strip  [dp][128]
  float* y2;       // this block's Y2 strip [dp][128]
  float* tau;      // [nb][32] handed from the first kernel of a panel to the second
  float* tbuf;     // [nb][dp / 32][32][32]: T of every panel
  float* cbuf;     // [nb][2][128][128]: C (blocks above the diagonal) and C2 (below) of the block under way
  int64_t dp, d;
  int64_t s_wk, s_vall, s_y, s_y2, s_t;   // batch strides
  int j0, klo;
  int ycol;        // 32 * (position of the panel in its block)
};

constexpr int VMAX = 12288;   // rows of a reflector kept in LDS: the largest extent a side with a basis may have
constexpr int TLD = QB + 4;   // row length of the T factor in LDS (rows 16-byte aligned)

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// tau and the scale of v for a column with diagonal element al and sum of squares ss below it
__device__ __forceinline__ void reflector_of(bool live, float ss, float al, float& tau, float& scale) {
  tau = 0.f, scale = 0.f;
  if (live && ss > 0.f) {
    const float nrm = sqrtf(__builtin_fmaf(al, al, ss));
    const float beta = al >= 0.f ? -nrm : nrm;
    tau = (beta - al) / beta;
    scale = 1.f / (al - beta);
  }
}
// elements 4 q .. 4 q + 3 of v_c from those of the column
__device__ __forceinline__ f32x4 v_of(const f32x4& x, int q, int c, float scale) {
  f32x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int r = 4 * q + e;
    o[e] = r < c ? 0.f : (r == c ? 1.f : x[e] * scale);
  }
  return o;
}

// Sum over the 64 lanes through the data-parallel-primitive lanes of the vector ALU (no LDS crossbar
// round trips, which dominate a step of the register-resident panel kernel otherwise): an inclusive scan
// inside each row of 16 lanes (shifts by 1, 2, 4, 8, out-of-row sources read as 0), then the row totals
// are carried into the following rows (row_bcast:15 into rows 1 and 3, row_bcast:31 into rows 2 and 3);
// lane 63 holds the total, which every lane receives.
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, BOUND));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v += dpp_mov<0x111, 0xf, true>(v);    // row_shr:1
  v += dpp_mov<0x112, 0xf, true>(v);    // row_shr:2
  v += dpp_mov<0x114, 0xf, true>(v);    // row_shr:4
  v += dpp_mov<0x118, 0xf, true>(v);    // row_shr:8
  v += dpp_mov<0x142, 0xa, false>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_mov<0x143, 0xc, false>(v);   // row_bcast:31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Columns ka and / or kb (registers) <- H_c applied to them, v_c in LDS.
template <int XS, bool DO_A, bool DO_B>
__device__ __forceinline__ void apply_reflector(f32x4 (&ka)[XS], f32x4 (&kb)[XS], const f32x4* s_v4, int nvec, int lane,
                                                float tau) {
  constexpr bool HOLD_V = XS <= 8;
  f32x4 v[HOLD_V ? XS : 1];
  float da = 0.f, db = 0.f;
#pragma unroll
  for (int sl = 0; sl < XS; ++sl) {
    const int q = lane + 64 * sl;
    if (q < nvec) {
      const f32x4 y = s_v4[q];
      if (HOLD_V) v[sl] = y;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (DO_A) da = __builtin_fmaf(ka[sl][e], y[e], da);
        if (DO_B) db = __builtin_fmaf(kb[sl][e], y[e], db);
      }
    }
  }
  const float fa = DO_A ? tau * wave_sum_dpp(da) : 0.f;
  const float fb = DO_B ? tau * wave_sum_dpp(db) : 0.f;
#pragma unroll
  for (int sl = 0; sl < XS; ++sl) {
    const int q = lane + 64 * sl;
    if (q < nvec) {
      const f32x4 y = HOLD_V ? v[sl] : s_v4[q];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (DO_A) ka[sl][e] = __builtin_fmaf(-fa, y[e], ka[sl][e]);
        if (DO_B) kb[sl][e] = __builtin_fmaf(-fb, y[e], kb[sl][e]);
      }
    }
  }
}

// The first kernel of a panel with at most 256 XS remaining rows (XS = 8: 2048, XS = 12: 3072): every
// wavefront loads its two columns (wave + 1 and wave + 17) into registers once and keeps them there; a step
// reads v_c from LDS, and the owner of column c + 1 writes v_(c+1) to LDS and to the reflector array.  The
// columns are never written back: what the factorisation leaves in them is R, which nothing uses.
// With XS = 8 there is room to hold v_c in registers between the dot products and the updates.
template <int XS>
__global__ __launch_bounds__(QTH) void k_qr_panel_regs(QrPanel a) {
  __shared__ f32x4 s_v4[64 * XS];
  __shared__ float s_tau[QB];
  const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t dp = a.dp;
  const int j0 = a.j0;
  const int nvec = (static_cast<int>(dp) - j0) / 4;   // <= 64 XS
  const float* wk = a.wk + static_cast<int64_t>(b) * a.s_wk;
  float* vrows = a.vall + static_cast<int64_t>(b) * a.s_vall;
  const int ca = wave + 1, cb = wave + 1 + QWAVES;    // this wavefront's columns (cb only if < 32)
  f32x4 ka[XS], kb[XS];

  auto load_col = [&](f32x4 (&k)[XS], int c) {
    const f32x4* x = reinterpret_cast<const f32x4*>(wk + static_cast<int64_t>(j0 + c) * dp + j0);
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
      const int q = lane + 64 * sl;
      if (q < nvec) k[sl] = x[q];
    }
  };
  // sum of squares below row c and the element at row c, over the wavefront
  auto head = [&](const f32x4 (&k)[XS], int c, float& ss, float& al) {
    ss = 0.f, al = 0.f;
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
      const int q = lane + 64 * sl;
      if (q < nvec) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * q + e;
          if (r > c) ss += k[sl][e] * k[sl][e];
          if (r == c) al = k[sl][e];
        }
      }
    }
    ss = wave_sum_dpp(ss), al = wave_sum_dpp(al);
  };
  // column c (in k), whose head is (ss, al), becomes the reflector v_c: to LDS, to the reflector array, tau to LDS
  auto make_v = [&](const f32x4 (&k)[XS], int c, float ss, float al) {
    float tau, scale;
    reflector_of(j0 + c < a.d, ss, al, tau, scale);
    f32x4* vg = reinterpret_cast<f32x4*>(vrows + static_cast<int64_t>(j0 + c) * dp + j0);
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
      const int q = lane + 64 * sl;
      if (q < nvec) {
        const f32x4 o = v_of(k[sl], q, c, scale);
        s_v4[q] = o;
        vg[q] = o;
      }
    }
    if (lane == 0) s_tau[c] = tau;
  };

  if (wave == 0) {
    float ss, al;
    load_col(ka, 0);
    head(ka, 0, ss, al);
    make_v(ka, 0, ss, al);
  }
  load_col(ka, ca);
  if (cb < QB) load_col(kb, cb);
  lds_barrier();

  for (int c = 0; c < QB; ++c) {
    const float tau = s_tau[c];
    const bool do_a = ca > c, do_b = cb < QB && cb > c;
    if (tau != 0.f) {   // columns that have become reflectors are left alone
      if (do_a && do_b)
        apply_reflector<XS, true, true>(ka, kb, s_v4, nvec, lane, tau);
      else if (do_a)
        apply_reflector<XS, true, false>(ka, kb, s_v4, nvec, lane, tau);
      else if (do_b)
        apply_reflector<XS, false, true>(ka, kb, s_v4, nvec, lane, tau);
    }
    // the owner of column c + 1 takes its head while the others are still busy with their columns
    const bool owner = c + 1 < QB && wave == c % QWAVES;
    float ss = 0.f, al = 0.f;
    if (owner) {
      if (c + 1 == ca)
        head(ka, c + 1, ss, al);
      else
        head(kb, c + 1, ss, al);
    }
    lds_barrier();   // every wavefront has finished with v_c
    if (owner) {
      if (c + 1 == ca)
        make_v(ka, c + 1, ss, al);
      else
        make_v(kb, c + 1, ss, al);
    }
    lds_barrier();   // v_(c+1) and tau_(c+1) are in place
  }
  if (t < QB) (a.tau + static_cast<int64_t>(b) * QB)[t] = s_tau[t];
}

// The first kernel of a panel with more remaining rows than the registers hold: as k_qr_panel_regs, every wavefront
// keeps the first 256 XS rows of its two columns in registers for the whole kernel; the rows beyond are streamed
// from the working copy on every step (read for the dot product, read and written for the update: the wavefront's
// own stores, which it reads back itself).  v_c is in LDS at full length.
template <int XS>
__global__ __launch_bounds__(QTH) void k_qr_panel_hybrid(QrPanel a) {
  __shared__ f32x4 s_v4[VMAX / 4];
  __shared__ float s_tau[QB];
  constexpr int NR = 64 * XS;   // float4 of a column kept in registers
  constexpr int TU = 2;         // loads in flight per lane in the streaming loops
  const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t dp = a.dp;
  const int j0 = a.j0;
  const int nvec = (static_cast<int>(dp) - j0) / 4;   // > NR
  float* wk = a.wk + static_cast<int64_t>(b) * a.s_wk;
  float* vrows = a.vall + static_cast<int64_t>(b) * a.s_vall;
  auto col = [&](int c) { return reinterpret_cast<f32x4*>(wk + static_cast<int64_t>(j0 + c) * dp + j0); };
  const int ca = wave + 1, cb = wave + 1 + QWAVES;    // this wavefront's columns (cb only if < 32)
  f32x4 ka[XS], kb[XS];

  auto load_col = [&](f32x4 (&k)[XS], int c) {
    const f32x4* x = col(c);
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) k[sl] = x[lane + 64 * sl];
  };
  // sum of squares below row c and the element at row c (c < 32: it lies in the registers), over the wavefront
  auto head = [&](const f32x4 (&k)[XS], int c, float& ss, float& al) {
    ss = 0.f, al = 0.f;
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = 4 * (lane + 64 * sl) + e;
        if (r > c) ss += k[sl][e] * k[sl][e];
        if (r == c) al = k[sl][e];
      }
    }
    const f32x4* x = col(c);
    for (int q0 = NR + lane; q0 < nvec; q0 += 64 * TU) {
      f32x4 xv[TU];
#pragma unroll
      for (int u = 0; u < TU; ++u) xv[u] = x[min(q0 + 64 * u, nvec - 1)];   // in bounds; surplus loads unused
#pragma unroll
      for (int u = 0; u < TU; ++u)
        if (q0 + 64 * u < nvec)
#pragma unroll
          for (int e = 0; e < 4; ++e) ss += xv[u][e] * xv[u][e];
    }
    ss = wave_sum_dpp(ss), al = wave_sum_dpp(al);
  };
  // column c, whose head is (ss, al), becomes the reflector v_c: to LDS, to the reflector array, tau to LDS
  auto make_v = [&](const f32x4 (&k)[XS], int c, float ss, float al) {
    float tau, scale;
    reflector_of(j0 + c < a.d, ss, al, tau, scale);
    f32x4* vg = reinterpret_cast<f32x4*>(vrows + static_cast<int64_t>(j0 + c) * dp + j0);
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
      const int q = lane + 64 * sl;
      const f32x4 o = v_of(k[sl], q, c, scale);
      s_v4[q] = o;
      vg[q] = o;
    }
    const f32x4* x = col(c);
    for (int q = NR + lane; q < nvec; q += 64) {
      f32x4 o = x[q];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] *= scale;
      s_v4[q] = o;
      vg[q] = o;
    }
    if (lane == 0) s_tau[c] = tau;
  };
  // H_c applied to column c2, held in k and, beyond the registers, in memory
  auto apply = [&](f32x4 (&k)[XS], int c2, float tau) {
    f32x4* x = col(c2);
    float dot = 0.f;
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
      const f32x4 y = s_v4[lane + 64 * sl];
#pragma unroll
      for (int e = 0; e < 4; ++e) dot = __builtin_fmaf(k[sl][e], y[e], dot);
    }
    for (int q0 = NR + lane; q0 < nvec; q0 += 64 * TU) {
      f32x4 xv[TU];
#pragma unroll
      for (int u = 0; u < TU; ++u) xv[u] = x[min(q0 + 64 * u, nvec - 1)];
#pragma unroll
      for (int u = 0; u < TU; ++u) {
        const int q = q0 + 64 * u;
        if (q < nvec) {
          const f32x4 y = s_v4[q];
#pragma unroll
          for (int e = 0; e < 4; ++e) dot = __builtin_fmaf(xv[u][e], y[e], dot);
        }
      }
    }
    const float f = tau * wave_sum_dpp(dot);
#pragma unroll
    for (int sl = 0; sl < XS; ++sl) {
      const f32x4 y = s_v4[lane + 64 * sl];
#pragma unroll
      for (int e = 0; e < 4; ++e) k[sl][e] = __builtin_fmaf(-f, y[e], k[sl][e]);
    }
    for (int q0 = NR + lane; q0 < nvec; q0 += 64 * TU) {
      f32x4 xv[TU];
#pragma unroll
      for (int u = 0; u < TU; ++u) xv[u] = x[min(q0 + 64 * u, nvec - 1)];
#pragma unroll
      for (int u = 0; u < TU; ++u) {
        const int q = q0 + 64 * u;
        if (q < nvec) {
          const f32x4 y = s_v4[q];
#pragma unroll
          for (int e = 0; e < 4; ++e) xv[u][e] = __builtin_fmaf(-f, y[e], xv[u][e]);
          x[q] = xv[u];
        }
      }
    }
  };

  if (wave == 0) {
    float ss, al;
    load_col(ka, 0);
    head(ka, 0, ss, al);
    make_v(ka, 0, ss, al);
  }
  load_col(ka, ca);
  if (cb < QB) load_col(kb, cb);
  lds_barrier();

  for (int c = 0; c < QB; ++c) {
    const float tau = s_tau[c];
    if (tau != 0.f) {   // columns that have become reflectors are left alone
      if (ca > c) apply(ka, ca, tau);
      if (cb < QB && cb > c) apply(kb, cb, tau);
    }
    // the owner of column c + 1 takes its head while the others are still busy with their columns
    const bool owner = c + 1 < QB && wave == c % QWAVES;
    float ss = 0.f, al = 0.f;
    if (owner) {
      if (c + 1 == ca)
        head(ka, c + 1, ss, al);
      else
        head(kb, c + 1, ss, al);
    }
    lds_barrier();   // every wavefront has finished with v_c
    if (owner) {
      if (c + 1 == ca)
        make_v(ka, c + 1, ss, al);
      else
        make_v(kb, c + 1, ss, al);
    }
    lds_barrier();   // v_(c+1) and tau_(c+1) are in place
  }
  if (t < QB) (a.tau + static_cast<int64_t>(b) * QB)[t] = s_tau[t];
}

// Second kernel of a panel: T from the reflectors and their tau, then Y and Y2 (see above).
__global__ __launch_bounds__(QTH) void k_qr_tfactor(QrPanel a) {
  __shared__ float s_part[8 * 1024];
  __shared__ float s_g[QB][QB + 1];
  __shared__ __attribute__((aligned(16))) float s_t[QB][TLD], s_tt[QB][TLD];
  __shared__ float s_tau[QB];
  const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t dp = a.dp;
  const int j0 = a.j0;
  const int len = static_cast<int>(dp) - j0;
  const float* vrows = a.vall + static_cast<int64_t>(b) * a.s_vall;
  if (t < QB) s_tau[t] = (a.tau + static_cast<int64_t>(b) * QB)[t];
  // The products of a whole block run over the rows of the reflectors from the block's first column on: this panel's
  // reflectors are zero there, which the panel kernel (it writes them from column j0 on) has not stored.
  for (int e = t; e < QB * a.ycol; e += QTH) {
    const int r = e / a.ycol, q = e - r * a.ycol;
    (a.vall + static_cast<int64_t>(b) * a.s_vall)[static_cast<int64_t>(j0 + r) * dp + (j0 - a.ycol) + q] = 0.f;
  }

  // s_g <- U^T V on the matrix cores, V this panel's reflectors, U those of the panel that starts at row `ju` (this
  // panel itself for V V^T), summed over the rows j0 .. dp - 1 (V is zero before): lane l supplies rows l % 32 at k
  // and k + 4 (l / 32), four k per load
  auto gram = [&](int ju) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const float* vbase = vrows + static_cast<int64_t>(j0 + (lane & 31)) * dp + j0 + 4 * (lane >> 5);
    const float* ubase = vrows + static_cast<int64_t>(ju + (lane & 31)) * dp + j0 + 4 * (lane >> 5);
    const int nblk = len / 8;
    // a wavefront takes four consecutive blocks at a time (32 rows x 32 k: one whole 128-byte line per row)
    for (int kb0 = 4 * wave; kb0 < nblk; kb0 += 4 * QWAVES) {   // nblk is a multiple of 4
      f32x4 x[4], u4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = *reinterpret_cast<const f32x4*>(vbase + 8 * (kb0 + u));
#pragma unroll
      for (int u = 0; u < 4; ++u) u4[u] = *reinterpret_cast<const f32x4*>(ubase + 8 * (kb0 + u));
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(u4[u][e], x[u][e], acc, 0, 0, 0);
    }
    // sum over the wavefronts in a fixed order, eight at a time through LDS
    float* scratch = s_part;
    float total = 0.f;
    for (int round = 0; round < QWAVES / 8; ++round) {
      if ((wave >> 3) == round) {
#pragma unroll
        for (int r = 0; r < 16; ++r) scratch[(wave & 7) * 1024 + r * 64 + lane] = acc[r];
      }
      __syncthreads();
#pragma unroll
      for (int w = 0; w < 8; ++w) total += scratch[w * 1024 + t];
      __syncthreads();
    }
    const int r = t >> 6, l = t & 63;   // thread t holds accumulator register r of lane l
    s_g[8 * (r >> 2) + (r & 3) + 4 * (l >> 5)][l & 31] = total;
    __syncthreads();
  };
  gram(j0);

  // T, forward and column by column: T[c][c] = tau_c, T[0:c, c] = -tau_c T[0:c, 0:c] (V^T v_c)
  // (thread i keeps row i of T in registers; its entries left of the diagonal are zero, so the sums may start at 0)
  if (t < QB) {
    const int i = t;
    float trow[QB];
#pragma unroll
    for (int c = 0; c < QB; ++c) {
      float sum = 0.f;
#pragma unroll
      for (int l = 0; l < c; ++l) sum = __builtin_fmaf(trow[l], s_g[l][c], sum);
      const float val = i == c ? s_tau[c] : (i < c ? -s_tau[c] * sum : 0.f);
      trow[c] = val;
      s_t[i][c] = val;
      s_tt[c][i] = val;
    }
  }
  __syncthreads();
  {   // T for the later panels of the block
    float* tb = a.tbuf + static_cast<int64_t>(b) * a.s_t + static_cast<int64_t>(j0 / QB) * QB * QB;
    tb[t] = s_t[t >> 5][t & 31];
  }
  // the blocks of C and C2 that pair this panel with the earlier ones of its block
  for (int pa = 0; pa < a.ycol / QB; ++pa) {
    const int ja = j0 - a.ycol + pa * QB;
    __syncthreads();               // s_g is free again
    gram(ja);                      // s_g[i][j] = (V_a^T V)[i][j]
    const float* ta = a.tbuf + static_cast<int64_t>(b) * a.s_t + static_cast<int64_t>(ja / QB) * QB * QB;
    const int i = t >> 5, j = t & 31;
    float c = 0.f, c2 = 0.f;
#pragma unroll 8
    for (int l = 0; l < QB; ++l) {
      c = __builtin_fmaf(ta[i * QB + l], s_g[l][j], c);     // C_a,pos = T_a (V_a^T V)
      c2 = __builtin_fmaf(s_t[l][i], s_g[j][l], c2);        // C2_pos,a = T^T (V^T V_a) = T^T (V_a^T V)^T
    }
    float* cb = a.cbuf + static_cast<int64_t>(b) * 2 * QBLK * QBLK;
    cb[(pa * QB + i) * QBLK + a.ycol + j] = c;
    cb[QBLK * QBLK + (a.ycol + i) * QBLK + pa * QB + j] = c2;
  }

  // Y = V T^T and Y2 = V T on the matrix cores, 32 rows per wavefront and turn; blocks of rows before j0
  // (down to the tile boundary klo) are zero.  Lane l supplies V[r0 + l % 32][k] and T[l % 32][k] resp.
  // T[k][l % 32] for k = 2 kk + l / 32.
  float* ybuf = a.ybuf + static_cast<int64_t>(b) * a.s_y;
  float* y2 = a.y2 + static_cast<int64_t>(b) * a.s_y2;
  const int nrb = (static_cast<int>(dp) - a.klo) / 32;
  for (int rb = wave; rb < nrb; rb += QWAVES) {
    const int64_t r0 = a.klo + 32 * rb;
    f32x16 ay, ay2;
#pragma unroll
    for (int r = 0; r < 16; ++r) ay[r] = 0.f, ay2[r] = 0.f;
    if (r0 >= j0) {
      const float* vp = vrows + static_cast<int64_t>(j0 + (lane >> 5)) * dp + r0 + (lane & 31);
      float xa[QB / 2];
#pragma unroll
      for (int kk = 0; kk < QB / 2; ++kk) xa[kk] = vp[static_cast<int64_t>(2 * kk) * dp];
#pragma unroll
      for (int kk = 0; kk < QB / 2; ++kk) {
        ay = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[kk], s_tt[2 * kk + (lane >> 5)][lane & 31], ay, 0, 0, 0);
        ay2 = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[kk], s_t[2 * kk + (lane >> 5)][lane & 31], ay2, 0, 0, 0);
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t at = (r0 + 8 * (r >> 2) + (r & 3) + 4 * (lane >> 5)) * QBLK + a.ycol + (lane & 31);
      ybuf[at] = ay[r];
      y2[at] = ay2[r];
    }
  }
}

// U^T and U2^T of one block of four panels from the blocks of C (above the diagonal) and C2 (below) that the panels'
// T kernels left in cbuf: U = (I + C)^(-1) by U_ab = -C_ab - sum_{a<c<b} C_ac U_cb, U2 = (I + C2)^(-1) by
// U2_ab = -C2_ab - sum_{b<c<a} C2_ac U2_cb; identity blocks on the diagonal, zero on the other side.  One workgroup
// of 1024 threads per matrix; thread (i, j) computes element (i, j) of every 32 x 32 block.
__global__ __launch_bounds__(QTH) void k_qr_block_u(const float* __restrict__ cbuf, float* __restrict__ ut, float* __restrict__ u2t,
                                                    int64_t s_u2) {
  __shared__ float s_c[QBLK][QBLK + 1], s_u[QBLK][QBLK + 1];
  const int b = blockIdx.x, t = threadIdx.x, i = t >> 5, j = t & 31;
  for (int lower = 0; lower < 2; ++lower) {
    const float* c = cbuf + (static_cast<int64_t>(b) * 2 + lower) * QBLK * QBLK;
    for (int e = t; e < QBLK * QBLK; e += QTH) {
      const int r = e >> 7, q = e & 127;
      const bool live = lower ? (r >> 5) > (q >> 5) : (r >> 5) < (q >> 5);
      s_c[r][q] = live ? c[e] : 0.f;
      s_u[r][q] = r == q ? 1.f : 0.f;
    }
    __syncthreads();
    for (int k = 1; k < 4; ++k) {          // blocks at distance k from the diagonal
      for (int lo = 0; lo + k < 4; ++lo) {
        const int ba = lower ? lo + k : lo, bb = lower ? lo : lo + k;   // block row, block column
        float acc = s_c[ba * QB + i][bb * QB + j];
        for (int bc = lo + 1; bc < lo + k; ++bc)
#pragma unroll 8
          for (int l = 0; l < QB; ++l) acc = __builtin_fmaf(s_c[ba * QB + i][bc * QB + l], s_u[bc * QB + l][bb * QB + j], acc);
        s_u[ba * QB + i][bb * QB + j] = -acc;
      }
      __syncthreads();
    }
    float* out = lower ? u2t + static_cast<int64_t>(b) * s_u2 : ut + static_cast<int64_t>(b) * QBLK * QBLK;
    for (int e = t; e < QBLK * QBLK; e += QTH) out[e] = s_u[e & 127][e >> 7];   // transposed
    __syncthreads();
  }
}

struct Carve {   // float offsets into the workspace of one launch batch
  size_t gm, gmt, t1, rot, np, yt, ql, qlt, qr, qrt, stat, wk, vall, y2, ybuf, tau, wt, qt, tb, cb, ub, u2, total_bytes;
  // bf16 rotations (offsets in floats as well; each array holds bf16 panels padded to 256)
  size_t gp, gpt, mp, mpt, as_g, at_g, as_m, at_m, rg, rgt, rm, rmt, npn, npt, ys, yst, qlp, qltp, qrp, qrtp;
};

struct Sides {
  bool left, right;
};
Sides sides(const canz_soap_group& g, const canz_soap_hparams& hp) {
  return {g.rows <= hp.max_precond_dim, g.cols <= hp.max_precond_dim};
}
// Gradients that arrive as bf16 are exact operands of the bf16 matrix cores: the products of G G^T and G^T G are
// exact in fp32 and are accumulated in fp32, so the statistics lose nothing against the fp32 kernel and take
// a fraction of its time.
bool bf16_statistics(const canz_soap_group& g) { return g.grad_dtype == CANZ_DT_BF16; }

Carve carve(int64_t rows, int64_t cols, int nb, Sides u, bool refresh, bool bf16, bool stat16) {
  const size_t rp = pad128(rows), cp = pad128(cols);
  const size_t dm = std::max(u.left ? rp : 0, u.right ? cp : 0);
  Carve c{};
  size_t off = 0;
  auto take = [&](size_t floats) {
    const size_t at = off;
    off += align_up(floats * sizeof(float)) / sizeof(float);
    return at;
  };
  const size_t plane = rp * cp;
  c.gm = take(2 * nb * plane), c.gmt = take(2 * nb * plane);
  c.t1 = take(u.left && u.right ? 2 * nb * plane : 0);
  c.rot = take(2 * nb * plane);
  c.np = take(nb * plane);
  c.yt = take(u.left && u.right ? nb * plane : 0);
  c.ql = take(u.left ? nb * rp * rp : 0), c.qlt = take(u.left ? nb * rp * rp : 0);
  c.qr = take(u.right ? nb * cp * cp : 0), c.qrt = take(u.right ? nb * cp * cp : 0);
  c.stat = take(nb * dm * dm);
  if (refresh) {
    c.wk = take(nb * dm * dm);
    c.vall = take(nb * dm * dm);
    c.y2 = take(nb * dm * dm);         // dm / 128 blocks of [dm][128]
    c.ybuf = take(nb * dm * QBLK);     // the Y strip of the block under way
    c.tau = take(nb * QB);
    c.wt = take(2 * nb * dm * QBLK);   // W_raw and W of a block
    c.qt = take(nb * dm * dm);
    c.tb = take(nb * dm * QB);         // T of every panel
    c.cb = take(2 * nb * QBLK * QBLK); // C and C2 of the block under way
    c.ub = take(nb * QBLK * QBLK);     // U^T of the block under way
    c.u2 = take(nb * dm * QBLK);       // U2^T of every block
  }
  const size_t rp2 = pad256(rows), cp2 = pad256(cols), p2 = nb * rp2 * cp2 / 2;   // floats that hold a batch of panels
  if (bf16 || stat16) c.gp = take(bf16 || u.left ? p2 : 0), c.gpt = take(bf16 || u.right ? p2 : 0);
  if (bf16) {
    const bool both = u.left && u.right;
    c.mp = take(p2), c.mpt = take(p2);
    c.as_g = take(u.right ? p2 : 0), c.at_g = take(u.right ? p2 : 0), c.as_m = take(u.right ? p2 : 0), c.at_m = take(u.right ? p2 : 0);
    c.rg = take(u.left ? p2 : 0), c.rgt = take(u.left ? p2 : 0), c.rm = take(u.left ? p2 : 0), c.rmt = take(u.left ? p2 : 0);
    c.npn = take(p2), c.npt = take(p2);
    c.ys = take(both ? p2 : 0), c.yst = take(both ? p2 : 0);
    c.qlp = take(u.left ? nb * rp2 * rp2 / 2 : 0), c.qltp = take(u.left ? nb * rp2 * rp2 / 2 : 0);
    c.qrp = take(u.right ? nb * cp2 * cp2 / 2 : 0), c.qrtp = take(u.right ? nb * cp2 * cp2 / 2 : 0);
  }
  c.total_bytes = off * sizeof(float);
  return c;
}

int batch_cap(const canz_soap_group& g, const canz_soap_hparams& hp) {
  const size_t one = carve(g.rows, g.cols, 1, sides(g, hp), hp.refresh != 0, hp.bf16_rotations != 0, bf16_statistics(g)).total_bytes;
  const int64_t by_bytes = std::max<int64_t>(1, static_cast<int64_t>(BATCH_BYTES / one));
  return static_cast<int>(std::min<int64_t>(MAX_PTRS / g.tp, by_bytes));
}

int check_hparams(const canz_soap_hparams* hp) {
  if (!hp) return fail(CANZ_EINVAL, "null hparams");
  if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f))
    return fail(CANZ_EINVAL, "beta1 and beta2 must be in [0, 1)");
  if (!(hp->eps >= 0.f)) return fail(CANZ_EINVAL, "eps must be >= 0");
  if (hp->step < 1) return fail(CANZ_EINVAL, "step must be >= 1");
  if (hp->max_precond_dim < 1) return fail(CANZ_EINVAL, "max_precond_dim must be >= 1");
  if (hp->out_mode != CANZ_OUT_PARAM && hp->out_mode != CANZ_OUT_DELTA)
    return fail(CANZ_EUNSUPPORTED, "unknown out_mode %d", hp->out_mode);
  return CANZ_OK;
}

int check_group(const canz_soap_group& g, int idx, bool need_ptrs, const canz_soap_hparams& hp) {
  if (g.n_mats < 0) return fail(CANZ_EINVAL, "group %d: n_mats < 0", idx);
  if (g.rows < 1 || g.cols < 1) return fail(CANZ_EINVAL, "group %d: empty shape", idx);
  if (g.rows > MAX_EXTENT || g.cols > MAX_EXTENT)
    return fail(CANZ_ESHAPE, "group %d: extent above %lld", idx, static_cast<long long>(MAX_EXTENT));
  const Sides u = sides(g, hp);
  if ((u.left && g.rows > VMAX) || (u.right && g.cols > VMAX))
    return fail(CANZ_ESHAPE, "group %d: a side with a basis may have at most %d rows or columns (lower max_precond_dim)", idx, VMAX);
  if (!u.left && !u.right)
    return fail(CANZ_EUNSUPPORTED, "group %d: both extents exceed max_precond_dim (plain Adam is not part of this library)", idx);
  if (g.tp < 1 || g.tp > MAX_TP) return fail(CANZ_EINVAL, "group %d: tp must be in 1..%d", idx, MAX_TP);
  if (g.cols % g.tp) return fail(CANZ_ESHAPE, "group %d: cols not divisible by tp", idx);
  if (g.tp > 1 && (g.cols / g.tp) % 8) return fail(CANZ_ESHAPE, "group %d: fragment width not a multiple of 8", idx);
  if (g.grad_dtype != CANZ_DT_F32 && g.grad_dtype != CANZ_DT_BF16)
    return fail(CANZ_EUNSUPPORTED, "group %d: unknown grad_dtype", idx);
  if (g.out_dtype != CANZ_DT_F32 && g.out_dtype != CANZ_DT_BF16)
    return fail(CANZ_EUNSUPPORTED, "group %d: unknown out_dtype", idx);
  if (!need_ptrs || g.n_mats == 0) return CANZ_OK;
  if (!g.grad || !g.mom || !g.var || !g.out || (u.left && (!g.left || !g.qleft)) || (u.right && (!g.right || !g.qright)))
    return fail(CANZ_EINVAL, "group %d: null pointer table", idx);
  const int n_out = hp.out_mode == CANZ_OUT_DELTA ? g.n_mats * g.tp : g.n_mats;
  auto bad = [](const void* p) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
  for (int i = 0; i < g.n_mats * g.tp; ++i)
    if (bad(g.grad[i])) return fail(CANZ_EINVAL, "group %d: grad[%d] null or not 16-byte aligned", idx, i);
  for (int i = 0; i < g.n_mats; ++i) {
    if (bad(g.mom[i]) || bad(g.var[i]) || (g.mom_rot && bad(g.mom_rot[i])))
      return fail(CANZ_EINVAL, "group %d: moment %d null or not 16-byte aligned", idx, i);
    if (u.left && (bad(g.left[i]) || bad(g.qleft[i])))
      return fail(CANZ_EINVAL, "group %d: left state %d null or not 16-byte aligned", idx, i);
    if (u.right && (bad(g.right[i]) || bad(g.qright[i])))
      return fail(CANZ_EINVAL, "group %d: right state %d null or not 16-byte aligned", idx, i);
  }
  for (int i = 0; i < n_out; ++i)
    if (bad(g.out[i])) return fail(CANZ_EINVAL, "group %d: out[%d] null or not 16-byte aligned", idx, i);
  return CANZ_OK;
}

inline int64_t floor128(int64_t x) { return x / SB * SB; }

// Basis refresh of one side: q (caller's, d x d) <- Q factor of QR(S q), S = the padded statistic in
// `stat` [nb][dp][dp], qt_old [nb][dp][dp] the transposed padded copy of the current basis.
int refresh_side(void* const* q_tab, int first, int nb, int64_t d, int64_t dp, const float* stat, const float* qt_old,
                 float* ws, const Carve& c, const Shape& s, const OutSpec& o, hipStream_t st) {
  const PtrTable none{};
  const int64_t dd = dp * dp;
  float *wk = ws + c.wk, *vall = ws + c.vall, *y2 = ws + c.y2, *ybuf = ws + c.ybuf, *wt = ws + c.wt, *qt = ws + c.qt;
  const int64_t s_vall = dp * dp, s_y = dp * QB;
  auto fill = [&](float* p, int64_t elems, int64_t ld, int identity) {
    const unsigned blocks = static_cast<unsigned>(std::min<int64_t>(2048, (elems + NTH - 1) / NTH));
    hipLaunchKernelGGL(k_soap_fill, dim3(blocks, nb), dim3(NTH), 0, st, p, elems, ld, identity);
  };
  prof_mark(st, CANZ_KERNEL_SOAP_PANEL, true);
  fill(qt, dd, dp, 1);   // nothing else has to start from a known state: every row that is read is written first
  prof_mark(st, CANZ_KERNEL_SOAP_PANEL, false);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "refresh fill: %s", hipGetErrorString(e));

  // working copy, transposed: wk[c][r] = (S q)[r][c] = sum_k qt_old[c][k] S[r][k]
  ShGemm p0{};
  p0.M = dp, p0.N = dp, p0.K = dp, p0.ldp = dp, p0.ldq = dp, p0.sp = dd, p0.sq = dd;
  p0.P = qt_old, p0.Q = stat, p0.c = wk;
  CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(p0, nb, none, s, o, st)), "refresh product");

  // Blocks of 128 columns = four panels; all of a block's columns are rows of one 128-row tile of the working copy.
  // Inside the block every panel is applied to that tile alone (rank 32); to the rows beyond it the whole block is
  // applied at once (rank 128), which moves the trailing matrix through memory once per block instead of once per
  // panel.  A last block with fewer than four panels has no rows beyond it.
  float *ycat = ws + c.ybuf, *wraw = ws + c.wt, *wfix = ws + c.wt + static_cast<size_t>(nb) * dp * QBLK;
  float *tb = ws + c.tb, *cb = ws + c.cb, *ub = ws + c.ub, *u2 = ws + c.u2;
  const int64_t s_strip = dp * QBLK, s_t = dp * QB, s_u2 = dp * QBLK;
  // W = (rows lo .. lo + rows - 1 of m) [V of `width` columns from column j0 on], over the rows j0.. of the reflectors
  auto w_product = [&](const float* m, int64_t lo, int64_t rows_, int64_t j0, int64_t width, float* w_out) {
    ShGemm w{};
    w.M = rows_, w.N = width, w.K = dp - j0, w.ldp = dp, w.ldq = dp, w.sp = dd, w.sq = s_vall;
    w.P = m + lo * dp + j0, w.Q = vall + j0 * dp + j0;
    w.c = w_out + lo * QBLK, w.ldc = QBLK, w.sc = s_strip;
    return w;
  };
  // (rows lo .. lo + rows - 1, columns klo.. of m) -= W Y^T: W and Y are the columns ycol .. ycol + width - 1 of their strips
  auto sub_product = [&](float* m, int64_t lo, int64_t rows_, int64_t klo, const float* w_in, const float* y, int64_t sy,
                         int64_t ycol, int64_t width) {
    ShGemm u{};
    u.M = rows_, u.N = dp - klo, u.K = width, u.ldp = QBLK, u.ldq = QBLK, u.sp = s_strip, u.sq = sy;
    u.P = w_in + lo * QBLK + ycol, u.Q = y + klo * QBLK + ycol;
    u.c = m + lo * dp + klo, u.ldc = dp, u.sc = dd;
    return u;
  };
  // W = W_raw U for a whole block: wfix = wraw (rows lo..) times the transposed factor ut [128][128]
  auto fix_product = [&](int64_t lo, int64_t rows_, const float* ut, int64_t s_ut) {
    ShGemm f{};
    f.M = rows_, f.N = QBLK, f.K = QBLK, f.ldp = QBLK, f.ldq = QBLK, f.sp = s_strip, f.sq = s_ut;
    f.P = wraw + lo * QBLK, f.Q = ut;
    f.c = wfix + lo * QBLK, f.ldc = QBLK, f.sc = s_strip;
    return f;
  };
  // one panel with the rank-32 products: W into its 32 columns of wraw, then the update
  auto apply_panel = [&](float* m, int64_t lo, int64_t rows_, int64_t klo, int64_t j0, const float* y, int64_t sy, const char* what) -> int {
    const int64_t ycol = j0 % QBLK;
    ShGemm w = w_product(m, lo, rows_, j0, QB, wraw);
    w.c += ycol;
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false, QB>(w, nb, none, s, o, st)), what);
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_SUB, false>(sub_product(m, lo, rows_, klo, wraw, y, sy, ycol, QB), nb, none, s, o, st)), what);
    return CANZ_OK;
  };
  // a whole block with the rank-128 products
  auto apply_block = [&](float* m, int64_t lo, int64_t klo, int64_t jb, const float* y, int64_t sy, const float* ut, int64_t s_ut,
                         const char* what) -> int {
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(w_product(m, lo, dp - lo, jb, QBLK, wraw), nb, none, s, o, st)), what);
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(fix_product(lo, dp - lo, ut, s_ut), nb, none, s, o, st)), what);
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_SUB, false>(sub_product(m, lo, dp - lo, klo, wfix, y, sy, 0, QBLK), nb, none, s, o, st)), what);
    return CANZ_OK;
  };

  for (int64_t jb = 0; jb < d; jb += QBLK) {            // factorisation, block by block
    float* y2blk = y2 + (jb / QBLK) * dp * QBLK;
    const int64_t panels = std::min<int64_t>(4, (d - jb + QB - 1) / QB);
    for (int64_t pp = 0; pp < panels; ++pp) {
      const int64_t j0 = jb + pp * QB;
      QrPanel a{};
      a.wk = wk, a.vall = vall, a.ybuf = ycat, a.y2 = y2blk, a.tau = ws + c.tau, a.tbuf = tb, a.cbuf = cb;
      a.dp = dp, a.d = d, a.s_wk = dd, a.s_vall = s_vall, a.s_y = s_strip, a.s_y2 = dd, a.s_t = s_t;
      a.j0 = static_cast<int>(j0), a.klo = static_cast<int>(jb), a.ycol = static_cast<int>(pp * QB);
      prof_mark(st, CANZ_KERNEL_SOAP_PANEL, true);
      if (dp - j0 <= 64 * 4 * 8)
        hipLaunchKernelGGL(k_qr_panel_regs<8>, dim3(nb), dim3(QTH), 0, st, a);
      else if (dp - j0 <= 64 * 4 * 12)
        hipLaunchKernelGGL(k_qr_panel_regs<12>, dim3(nb), dim3(QTH), 0, st, a);
      else
        hipLaunchKernelGGL(k_qr_panel_hybrid<8>, dim3(nb), dim3(QTH), 0, st, a);
      hipLaunchKernelGGL(k_qr_tfactor, dim3(nb), dim3(QTH), 0, st, a);
      prof_mark(st, CANZ_KERNEL_SOAP_PANEL, false);
      if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "panel kernel: %s", hipGetErrorString(e));
      if (pp + 1 < panels)   // the later panels of the block: the block's own 128 rows
        if (int rc = apply_panel(wk, jb, QBLK, jb, j0, ycat, s_strip, "QR (panel update)")) return rc;
    }
    if (jb + QBLK >= dp) break;   // no columns after this block
    prof_mark(st, CANZ_KERNEL_SOAP_PANEL, true);
    hipLaunchKernelGGL(k_qr_block_u, dim3(nb), dim3(QTH), 0, st, cb, ub, u2 + (jb / QBLK) * QBLK * QBLK, s_u2);
    prof_mark(st, CANZ_KERNEL_SOAP_PANEL, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "block kernel: %s", hipGetErrorString(e));
    if (int rc = apply_block(wk, jb + QBLK, jb, jb, ycat, s_strip, ub, QBLK * QBLK, "QR (block update)")) return rc;
  }
  // Q = H(0) H(1) ... applied to the identity from the last block to the first; a last block without all four panels
  // (it has no U2) panel by panel
  for (int64_t jb = (d - 1) / QBLK * QBLK; jb >= 0; jb -= QBLK) {
    const float* y2blk = y2 + (jb / QBLK) * dp * QBLK;
    const int64_t panels = std::min<int64_t>(4, (d - jb + QB - 1) / QB);
    if (panels == 4 && jb + QBLK < dp) {
      if (int rc = apply_block(qt, jb, jb, jb, y2blk, dd, u2 + (jb / QBLK) * QBLK * QBLK, s_u2, "Q (block update)")) return rc;
    } else {
      for (int64_t pp = panels - 1; pp >= 0; --pp)
        if (int rc = apply_panel(qt, jb, dp - jb, jb, jb + pp * QB, y2blk, dd, "Q (panel update)")) return rc;
    }
  }
  PtrTable q{};
  for (int i = 0; i < nb; ++i) q.p[i] = q_tab[first + i];
  prof_mark(st, CANZ_KERNEL_SOAP_PANEL, true);
  hipLaunchKernelGGL(k_soap_store_q, dim3(static_cast<unsigned>(dp / 64), static_cast<unsigned>(dp / 64), static_cast<unsigned>(nb)),
                     dim3(NTH), 0, st, q, qt, d, dp);
  prof_mark(st, CANZ_KERNEL_SOAP_PANEL, false);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "basis store: %s", hipGetErrorString(e));
  return CANZ_OK;
}

// One launch batch: matrices first .. first + nb - 1 of group g.
int run_batch(const canz_soap_group& g, int first, int nb, const canz_soap_hparams& hp, float* ws, hipStream_t st) {
  const int64_t rp = pad128(g.rows), cp = pad128(g.cols), plane = rp * cp;
  const Sides u = sides(g, hp);
  const bool bf16 = hp.bf16_rotations != 0;
  const bool stat16 = bf16_statistics(g);
  const Carve c = carve(g.rows, g.cols, nb, u, hp.refresh != 0, bf16, stat16);
  Shape s{};
  s.rows = g.rows, s.cols = g.cols;
  s.m = std::min(g.rows, g.cols), s.n = std::max(g.rows, g.cols);
  s.mp = rp, s.np = cp;
  s.tall = g.rows > g.cols;
  s.tp = g.tp;
  s.wfrag = g.cols / g.tp;
  PtrTable grad{}, mom{}, var{}, none{};
  for (int i = 0; i < nb * g.tp; ++i) grad.p[i] = const_cast<void*>(g.grad[first * g.tp + i]);
  for (int i = 0; i < nb; ++i) mom.p[i] = g.mom[first + i], var.p[i] = g.var[first + i];
  OutSpec o{};
  const int per_out = hp.out_mode == CANZ_OUT_DELTA ? g.tp : 1;
  for (int i = 0; i < nb * per_out; ++i) o.out.p[i] = g.out[first * per_out + i];
  o.out_dtype = g.out_dtype;
  o.out_mode = hp.out_mode;
  o.decay = static_cast<float>(1.0 - static_cast<double>(hp.lr) * static_cast<double>(hp.weight_decay));
  o.neg_lr_scale = -hp.lr;

  float *gm = ws + c.gm, *gmt = ws + c.gmt, *t1 = ws + c.t1, *rot = ws + c.rot, *np = ws + c.np, *yt = ws + c.yt;
  float *ql = ws + c.ql, *qlt = ws + c.qlt, *qr = ws + c.qr, *qrt = ws + c.qrt, *stat = ws + c.stat;
  const dim3 tiles(static_cast<unsigned>(cp / 64), static_cast<unsigned>(rp / 64), static_cast<unsigned>(nb));

  // With a valid rotated momentum from the caller only G is rotated (M' follows its own recurrence in the rotated
  // space, which is the same linear map as long as the bases stand still); otherwise G and M.
  const bool incremental = g.mom_rot != nullptr && hp.mom_rot_valid != 0;
  // bf16 images in the panel layout (padded to 256): operands of the bf16 rotations and of the statistics
  const int64_t rp2 = pad256(g.rows), cp2 = pad256(g.cols), p2 = rp2 * cp2;
  const SplitWs no_split{nullptr, 0};
  auto pan = [&](size_t at) { return reinterpret_cast<__bf16*>(ws + at); };

  prof_mark(st, CANZ_KERNEL_SOAP_LOAD, true);
  {
    // fp32 copies: G for the fp32 rotations and the fp32 statistics, M for the fp32 rotations; bf16 images: G for the
    // bf16 rotations and statistics, M for the bf16 rotations of a step that rotates it (also the re-rotation of a
    // kept M' after a refresh)
    LoadOut w{};
    w.gm = gm, w.gmt = gmt;
    w.g32 = !bf16 || !stat16;
    w.m32 = !bf16;
    w.rp2 = rp2, w.cp2 = cp2;
    if (bf16 || (stat16 && u.left)) w.gp = pan(c.gp);
    if (bf16 || (stat16 && u.right)) w.gpt = pan(c.gpt);
    if (bf16 && (!incremental || (hp.refresh && g.mom_rot != nullptr))) w.mp = pan(c.mp), w.mpt = pan(c.mpt);
    const bool images = w.gp || w.gpt;
    const dim3 grid(static_cast<unsigned>((images ? cp2 : cp) / 64), static_cast<unsigned>((images ? rp2 : rp) / 64),
                    static_cast<unsigned>(nb));
    if (g.cols % 8 == 0 && s.wfrag % 8 == 0)
      hipLaunchKernelGGL(k_soap_load<true>, grid, dim3(NTH), 0, st, s, grad, g.grad_dtype, mom, hp.beta1, rp, cp, w);
    else
      hipLaunchKernelGGL(k_soap_load<false>, grid, dim3(NTH), 0, st, s, grad, g.grad_dtype, mom, hp.beta1, rp, cp, w);
  }
  // the bases: padded copies in both orientations, zero outside d x d: fp32 for the fp32 rotations and for the
  // refresh (which multiplies the new statistic with the old basis), bf16 images for the bf16 rotations
  auto load_basis = [&](void* const* tab, int64_t d, int64_t dp, float* straight, float* transposed, bool f32, int64_t dp2,
                        __bf16* sp, __bf16* tp) {
    PtrTable q{};
    for (int i = 0; i < nb; ++i) q.p[i] = tab[first + i];
    const unsigned side = static_cast<unsigned>((sp || tp ? dp2 : dp) / 64);
    hipLaunchKernelGGL(k_soap_load_basis, dim3(side, side, static_cast<unsigned>(nb)), dim3(NTH), 0, st, q, d, dp, f32, straight,
                       transposed, dp2, sp, tp);
  };
  const bool basis32 = !bf16 || hp.refresh;
  if (u.left) load_basis(g.qleft, g.rows, rp, ql, qlt, basis32, rp2, bf16 ? pan(c.qlp) : nullptr, bf16 ? pan(c.qltp) : nullptr);
  if (u.right) load_basis(g.qright, g.cols, cp, qr, qrt, basis32, cp2, bf16 ? pan(c.qrp) : nullptr, bf16 ? pan(c.qrtp) : nullptr);
  prof_mark(st, CANZ_KERNEL_SOAP_LOAD, false);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "load kernels: %s", hipGetErrorString(e));

  // rotation into the bases of `per` planes of each matrix's (G, M) pair, from plane `p0` on: problem p is
  // plane p0 + p % per of matrix p / per; consecutive problems of a matrix share the basis operand
  auto rotate_in = [&](int p0, int per) -> int {
    const int64_t step_ = per == 2 ? plane : 2 * plane, at = p0 * plane;
    const int count = per * nb;
    if (u.left && u.right) {
      ShGemm a{};   // t1 = (X Q_R)^T: [cp][rp]
      a.M = cp, a.N = rp, a.K = cp, a.ldp = cp, a.ldq = cp, a.sp = cp * cp, a.pdiv = per, a.sq = step_;
      a.P = qrt, a.Q = gm + at, a.c = t1 + at, a.ldc = rp, a.sc = step_;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(a, count, none, s, o, st)), "rotation (right)");
      ShGemm bq{};  // rot = Q_L^T (X Q_R): [rp][cp]
      bq.M = rp, bq.N = cp, bq.K = rp, bq.ldp = rp, bq.ldq = rp, bq.sp = rp * rp, bq.pdiv = per, bq.sq = step_;
      bq.P = qlt, bq.Q = t1 + at, bq.c = rot + at, bq.ldc = cp, bq.sc = step_;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(bq, count, none, s, o, st)), "rotation (left)");
    } else if (u.left) {
      ShGemm bq{};  // rot = Q_L^T X with X^T as the second operand
      bq.M = rp, bq.N = cp, bq.K = rp, bq.ldp = rp, bq.ldq = rp, bq.sp = rp * rp, bq.pdiv = per, bq.sq = step_;
      bq.P = qlt, bq.Q = gmt + at, bq.c = rot + at, bq.ldc = cp, bq.sc = step_;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(bq, count, none, s, o, st)), "rotation (left)");
    } else {
      ShGemm a{};   // rot = X Q_R
      a.M = rp, a.N = cp, a.K = cp, a.ldp = cp, a.ldq = cp, a.sp = step_, a.sq = cp * cp, a.qdiv = per;
      a.P = gm + at, a.Q = qrt, a.c = rot + at, a.ldc = cp, a.sc = step_;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(a, count, none, s, o, st)), "rotation (right)");
    }
    return CANZ_OK;
  };
  PtrTable mrot{};
  if (g.mom_rot)
    for (int i = 0; i < nb; ++i) mrot.p[i] = g.mom_rot[first + i];
  const double c1 = hp.bias_correction ? 1.0 / (1.0 - std::pow(static_cast<double>(hp.beta1), hp.step)) : 1.0;
  const double c2 = hp.bias_correction ? 1.0 / (1.0 - std::pow(static_cast<double>(hp.beta2), hp.step)) : 1.0;

  // shapes of the bf16 rotation products (first operand: a basis)
  const GemmDims right_dims{cp2, rp2, cp2, cp2, cp2, cp2 * cp2, p2, nb};   // (basis rows) x (matrix rows), k over columns
  const GemmDims left_dims{rp2, cp2, rp2, rp2, rp2, rp2 * rp2, p2, nb};    // (basis rows) x (matrix columns), k over rows
  if (bf16) {
    // The rotations on the bf16 matrix cores (fp32 accumulation): the bases, G (and M on a step that rotates it) and
    // N' are rounded to bf16 once each, the intermediate of a two-sided rotation once more; momentum, second
    // moment, the statistics' accumulation and the refresh stay in fp32.  The products reuse the update kernel of the
    // Muon step (it writes its result in both orientations, which is what the next product wants as its second
    // operand) and its last product (which writes the parameter update).
    // X' = Q_L^T X Q_R for X given as straight and transposed panels; the result as straight panels
    auto rotate_in16 = [&](const __bf16* xs, const __bf16* xt, size_t as_, size_t at_, size_t r_, size_t rt_,
                           const __bf16** result) -> int {
      if (u.right)   // as = (X Q_R)^T [cp2][rp2], at = X Q_R [rp2][cp2]
        CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_update_bf16(right_dims, pan(c.qrtp), xs, pan(as_), pan(at_), nullptr, no_split, st),
                 "rotation (right, bf16)");
      if (u.left)    // r = Q_L^T (.) [rp2][cp2] from the transposed image of what the right side left (or of X)
        CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE,
                 launch_update_bf16(left_dims, pan(c.qltp), u.right ? pan(as_) : xt, pan(r_), pan(rt_), nullptr, no_split, st),
                 "rotation (left, bf16)");
      *result = u.left ? pan(r_) : pan(at_);
      return CANZ_OK;
    };
    const __bf16 *g_rot = nullptr, *m_rot = nullptr;
    if (int rc = rotate_in16(pan(c.gp), pan(c.gpt), c.as_g, c.at_g, c.rg, c.rgt, &g_rot)) return rc;
    if (!incremental)
      if (int rc = rotate_in16(pan(c.mp), pan(c.mpt), c.as_m, c.at_m, c.rm, c.rmt, &m_rot)) return rc;
    const bool want_t = u.left && !u.right;   // the left side alone takes N'^T as its second operand
    const dim3 tiles2(static_cast<unsigned>(cp2 / 64), static_cast<unsigned>(rp2 / 64), static_cast<unsigned>(nb));
    prof_mark(st, CANZ_KERNEL_SOAP_ADAM, true);
    hipLaunchKernelGGL(k_soap_adam_bf16, tiles2, dim3(NTH), 0, st, s, var, mrot, g.mom_rot != nullptr, incremental, g_rot, m_rot,
                       rp2, cp2, hp.beta1, hp.beta2, static_cast<float>(c1), static_cast<float>(c2), hp.eps,
                       want_t ? nullptr : pan(c.npn), want_t ? pan(c.npt) : nullptr);
    prof_mark(st, CANZ_KERNEL_SOAP_ADAM, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "adam kernel: %s", hipGetErrorString(e));
    if (u.left && u.right) {
      // ys = (N' Q_R^T)^T [cp2][rp2]; then Q_L times it, into the caller's buffers
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_update_bf16(right_dims, pan(c.qrp), pan(c.npn), pan(c.ys), pan(c.yst), nullptr, no_split, st),
               "back rotation (right, bf16)");
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_final_bf16(left_dims, pan(c.qlp), pan(c.ys), nullptr, no_split, s, o, st),
               "back rotation (left, bf16)");
    } else if (u.left) {
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_final_bf16(left_dims, pan(c.qlp), pan(c.npt), nullptr, no_split, s, o, st),
               "back rotation (left, bf16)");
    } else {
      const GemmDims d{rp2, cp2, cp2, cp2, cp2, p2, cp2 * cp2, nb};   // N' [rp2][cp2] times Q_R^T
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_final_bf16(d, pan(c.npn), pan(c.qrp), nullptr, no_split, s, o, st),
               "back rotation (right, bf16)");
    }
  } else {
    if (int rc = rotate_in(0, incremental ? 1 : 2)) return rc;

    {
      const int transposed = u.left && !u.right;
      prof_mark(st, CANZ_KERNEL_SOAP_ADAM, true);
      hipLaunchKernelGGL(k_soap_adam, tiles, dim3(NTH), 0, st, s, var, mrot, g.mom_rot != nullptr, incremental, rot, rp, cp,
                         hp.beta1, hp.beta2, static_cast<float>(c1), static_cast<float>(c2), hp.eps, transposed, np);
      prof_mark(st, CANZ_KERNEL_SOAP_ADAM, false);
      if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "adam kernel: %s", hipGetErrorString(e));
    }

    // rotation back, the last product writes the update
    if (u.left && u.right) {
      ShGemm cq{};  // yt = (N' Q_R^T)^T: [cp][rp]
      cq.M = cp, cq.N = rp, cq.K = cp, cq.ldp = cp, cq.ldq = cp, cq.sp = cp * cp, cq.sq = plane;
      cq.P = qr, cq.Q = np, cq.c = yt;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(cq, nb, none, s, o, st)), "back rotation (right)");
      ShGemm dq{};
      dq.M = rp, dq.N = cp, dq.K = rp, dq.ldp = rp, dq.ldq = rp, dq.sp = rp * rp, dq.sq = plane;
      dq.P = ql, dq.Q = yt;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_OUT, false>(dq, nb, none, s, o, st)), "back rotation (left)");
    } else if (u.left) {
      ShGemm dq{};  // np holds N'^T
      dq.M = rp, dq.N = cp, dq.K = rp, dq.ldp = rp, dq.ldq = rp, dq.sp = rp * rp, dq.sq = plane;
      dq.P = ql, dq.Q = np;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_OUT, false>(dq, nb, none, s, o, st)), "back rotation (left)");
    } else {
      ShGemm cq{};
      cq.M = rp, cq.N = cp, cq.K = cp, cq.ldp = cp, cq.ldq = cp, cq.sp = plane, cq.sq = cp * cp;
      cq.P = np, cq.Q = qr;
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_OUT, false>(cq, nb, none, s, o, st)), "back rotation (right)");
    }

  }

  // statistics (and, on a refresh step, the new basis) side by side
  auto one_side = [&](void* const* stat_tab, void* const* q_tab, int64_t d, int64_t dp, int64_t kp, const float* side,
                      const float* qt_old, const __bf16* side16, int64_t d2, int64_t k2) -> int {
    PtrTable tab{};
    for (int i = 0; i < nb; ++i) tab.p[i] = stat_tab[first + i];
    if (stat16) {
      // S <- beta2 S + (1 - beta2) X X^T as the "last product" of the bf16 kernels: it updates the caller's dense
      // fp32 array in place as old * decay + factor * product, on and above the diagonal tiles; the rest is mirrored
      Shape sq{};
      sq.rows = d, sq.cols = d, sq.m = d, sq.n = d, sq.mp = d2, sq.np = d2, sq.tp = 1, sq.wfrag = d;
      OutSpec so{};
      so.out = tab, so.out_dtype = CANZ_DT_F32, so.out_mode = CANZ_OUT_PARAM, so.decay = hp.beta2, so.neg_lr_scale = 1.f - hp.beta2;
      const GemmDims sd{d2, d2, k2, k2, k2, d2 * k2, d2 * k2, nb};
      // Only the tiles on and above the diagonal, mirrored afterwards, where that pays: the products it saves (about
      // 0.65 us per 32-long k-step of a tile, a round of tiles on 256 CUs at a time) against one more pass over the
      // statistic at some 4 TB/s that does not overlap with anything.  Long sums win (25600 x 5120: 3.9 -> 1.3 ms),
      // short ones do not (3072 x 1024: the mirror pass costs what the products save).
      const int64_t t256 = d2 / 256;
      const double saved_us = static_cast<double>(t256 * (t256 - 1) / 2 * nb) / 256.0 * static_cast<double>(k2 / 32) * 0.65;
      const double mirror_us = 15.0 + static_cast<double>(d) * static_cast<double>(d) * nb * 4.0 / 4.0e6;
      if (saved_us > 1.5 * mirror_us) {
        CANZ_HIP(CANZ_KERNEL_SOAP_STAT, launch_final_sym_bf16(sd, side16, no_split, sq, so, st), "statistics kernel (bf16 operands)");
        prof_mark(st, CANZ_KERNEL_SOAP_STAT, true);
        const unsigned t64 = static_cast<unsigned>((d + 63) / 64);
        hipLaunchKernelGGL(k_soap_mirror, dim3(t64, t64, static_cast<unsigned>(nb)), dim3(NTH), 0, st, tab, d);
        prof_mark(st, CANZ_KERNEL_SOAP_STAT, false);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "statistic mirror: %s", hipGetErrorString(e));
      } else {
        CANZ_HIP(CANZ_KERNEL_SOAP_STAT, launch_final_bf16(sd, side16, side16, nullptr, no_split, sq, so, st),
                 "statistics kernel (bf16 operands)");
      }
      if (hp.refresh) {   // the padded copy the refresh multiplies the basis with (its transposed image lands in wk, unused)
        prof_mark(st, CANZ_KERNEL_SOAP_STAT, true);
        hipLaunchKernelGGL(k_sh_load, dim3(static_cast<unsigned>(dp / 64), static_cast<unsigned>(dp / 64), static_cast<unsigned>(nb)),
                           dim3(NTH), 0, st, sq, tab, static_cast<int>(CANZ_DT_F32), dp, dp, stat, ws + c.wk);
        prof_mark(st, CANZ_KERNEL_SOAP_STAT, false);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "statistic copy: %s", hipGetErrorString(e));
      }
    } else {
      ShGemm q{};
      q.M = dp, q.N = dp, q.K = kp, q.ldp = kp, q.ldq = kp, q.sp = 2 * plane, q.sq = 2 * plane;
      q.P = side, q.Q = side, q.c = hp.refresh ? stat : nullptr, q.d = d, q.beta = hp.beta2, q.gscale = 1.f - hp.beta2, q.eps = 0.f;
      CANZ_HIP(CANZ_KERNEL_SOAP_STAT, (launch_gemm<SE_STAT, true>(q, nb, tab, s, o, st)), "statistics kernel");
    }
    if (!hp.refresh) return CANZ_OK;
    return refresh_side(q_tab, first, nb, d, dp, stat, qt_old, ws, c, s, o, st);
  };
  if (u.left)
    if (int rc = one_side(g.left, g.qleft, g.rows, rp, cp, gm, qlt, pan(c.gp), rp2, cp2)) return rc;
  if (u.right)
    if (int rc = one_side(g.right, g.qright, g.cols, cp, rp, gmt, qrt, pan(c.gpt), cp2, rp2)) return rc;
  if (hp.refresh && g.mom_rot && bf16) {
    // the caller's rotated momentum follows the new bases, M' = Q_L^T M Q_R once more with the M of this step: bf16
    // operands as for every rotation of this mode; the last product leaves its fp32 sums in the caller's array
    prof_mark(st, CANZ_KERNEL_SOAP_LOAD, true);
    if (u.left) load_basis(g.qleft, g.rows, rp, ql, qlt, false, rp2, nullptr, pan(c.qltp));
    if (u.right) load_basis(g.qright, g.cols, cp, qr, qrt, false, cp2, nullptr, pan(c.qrtp));
    prof_mark(st, CANZ_KERNEL_SOAP_LOAD, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "basis load: %s", hipGetErrorString(e));
    Shape whole = s;
    whole.tp = 1, whole.wfrag = g.cols;
    OutSpec mo{};
    mo.out = mrot, mo.out_dtype = CANZ_DT_F32, mo.out_mode = CANZ_OUT_DELTA, mo.decay = 1.f, mo.neg_lr_scale = 1.f;
    if (u.left && u.right) {
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE,
               launch_update_bf16(right_dims, pan(c.qrtp), pan(c.mp), pan(c.as_m), pan(c.at_m), nullptr, no_split, st),
               "momentum re-rotation (right, bf16)");
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_final_bf16(left_dims, pan(c.qltp), pan(c.as_m), nullptr, no_split, whole, mo, st),
               "momentum re-rotation (left, bf16)");
    } else if (u.left) {
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_final_bf16(left_dims, pan(c.qltp), pan(c.mpt), nullptr, no_split, whole, mo, st),
               "momentum re-rotation (left, bf16)");
    } else {
      const GemmDims d{rp2, cp2, cp2, cp2, cp2, p2, cp2 * cp2, nb};   // M [rp2][cp2] times (Q_R^T)^T
      CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, launch_final_bf16(d, pan(c.mp), pan(c.qrtp), nullptr, no_split, whole, mo, st),
               "momentum re-rotation (right, bf16)");
    }
  } else if (hp.refresh && g.mom_rot) {
    // the same in fp32
    prof_mark(st, CANZ_KERNEL_SOAP_LOAD, true);
    if (u.left) load_basis(g.qleft, g.rows, rp, ql, qlt, true, rp2, nullptr, nullptr);
    if (u.right) load_basis(g.qright, g.cols, cp, qr, qrt, true, cp2, nullptr, nullptr);
    prof_mark(st, CANZ_KERNEL_SOAP_LOAD, false);
    if (int rc = rotate_in(1, 1)) return rc;
    prof_mark(st, CANZ_KERNEL_SOAP_ADAM, true);
    hipLaunchKernelGGL(k_unpad, tiles, dim3(NTH), 0, st, s, mrot, rot + plane, 2 * plane, cp);
    prof_mark(st, CANZ_KERNEL_SOAP_ADAM, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "momentum re-rotation: %s", hipGetErrorString(e));
  }
  return CANZ_OK;
}

// Consecutive groups of a call that agree in shape, tp, dtypes and in which tables they pass run as one group: every
// matrix is computed on its own whatever shares its launch, a refresh keeps only one workgroup per matrix busy in
// its panel kernel, and its products are small - the more matrices share a launch, the better the chip is filled.
struct MergedGroup {
  canz_soap_group g{};
  std::vector<const void*> grad;
  std::vector<void*> tab[8];   // mom, var, left, right, qleft, qright, out, mom_rot
};

void* const* const* tables_of(const canz_soap_group& g, void* const* (&out)[8]) {
  out[0] = g.mom, out[1] = g.var, out[2] = g.left, out[3] = g.right, out[4] = g.qleft, out[5] = g.qright, out[6] = g.out,
  out[7] = g.mom_rot;
  return out;
}

bool mergeable(const canz_soap_group& a, const canz_soap_group& b) {
  if (a.rows != b.rows || a.cols != b.cols || a.tp != b.tp || a.grad_dtype != b.grad_dtype || a.out_dtype != b.out_dtype) return false;
  if ((a.grad == nullptr) != (b.grad == nullptr)) return false;
  void* const* ta[8];
  void* const* tb[8];
  tables_of(a, ta), tables_of(b, tb);
  for (int k = 0; k < 8; ++k)
    if ((ta[k] == nullptr) != (tb[k] == nullptr)) return false;
  return true;
}

std::vector<MergedGroup> merge_groups(const canz_soap_group* g, int n_groups, const canz_soap_hparams& hp) {
  std::vector<MergedGroup> all;
  const auto append = [&](MergedGroup& m, const canz_soap_group& x) {
    void* const* t[8];
    tables_of(x, t);
    const int per_out = hp.out_mode == CANZ_OUT_DELTA ? x.tp : 1;
    if (x.grad) m.grad.insert(m.grad.end(), x.grad, x.grad + static_cast<size_t>(x.n_mats) * x.tp);
    for (int k = 0; k < 8; ++k)
      if (t[k]) m.tab[k].insert(m.tab[k].end(), t[k], t[k] + static_cast<size_t>(x.n_mats) * (k == 6 ? per_out : 1));
    m.g.n_mats += x.n_mats;
  };
  for (int i = 0; i < n_groups; ++i) {
    if (g[i].n_mats == 0) continue;
    if (all.empty() || !mergeable(all.back().g, g[i])) {
      all.emplace_back();
      all.back().g = g[i];
      all.back().g.n_mats = 0;
    }
    append(all.back(), g[i]);
  }
  for (MergedGroup& m : all) {   // the tables now stand still: point the group at them
    canz_soap_group& x = m.g;
    if (x.grad) x.grad = m.grad.data();
    if (x.mom) x.mom = m.tab[0].data();
    if (x.var) x.var = m.tab[1].data();
    if (x.left) x.left = m.tab[2].data();
    if (x.right) x.right = m.tab[3].data();
    if (x.qleft) x.qleft = m.tab[4].data();
    if (x.qright) x.qright = m.tab[5].data();
    if (x.out) x.out = m.tab[6].data();
    if (x.mom_rot) x.mom_rot = m.tab[7].data();
  }
  return all;
}

}  // namespace
}  // namespace canz

extern "C" int canz_soap_workspace_bytes(const canz_soap_group* g, int32_t n_groups, const canz_soap_hparams* hp,
                                         size_t* bytes_out) {
  using namespace canz;
  if (!bytes_out) return fail(CANZ_EINVAL, "null bytes_out");
  if (n_groups < 0 || (n_groups > 0 && !g)) return fail(CANZ_EINVAL, "bad group array");
  if (int rc = check_hparams(hp)) return rc;
  size_t need = ALIGN;
  for (int i = 0; i < n_groups; ++i)
    if (int rc = check_group(g[i], i, false, *hp)) return rc;
  for (const MergedGroup& m : merge_groups(g, n_groups, *hp))
    need = std::max(need, carve(m.g.rows, m.g.cols, std::min(m.g.n_mats, batch_cap(m.g, *hp)), sides(m.g, *hp), hp->refresh != 0,
                                hp->bf16_rotations != 0, bf16_statistics(m.g)).total_bytes);
  *bytes_out = need;
  return CANZ_OK;
}

extern "C" int canz_soap_step(const canz_soap_group* g, int32_t n_groups, const canz_soap_hparams* hp, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  using namespace canz;
  size_t need = 0;
  if (int rc = canz_soap_workspace_bytes(g, n_groups, hp, &need)) return rc;
  bool any = false;
  for (int i = 0; i < n_groups; ++i) {
    if (int rc = check_group(g[i], i, true, *hp)) return rc;
    any = any || g[i].n_mats > 0;
  }
  if (!any) return CANZ_OK;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (ALIGN - 1)))
    return fail(CANZ_EWORKSPACE, "workspace null or not 256-byte aligned");
  if (workspace_bytes < need)
    return fail(CANZ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (const MergedGroup& m : merge_groups(g, n_groups, *hp)) {
    const int cap = batch_cap(m.g, *hp);
    for (int first = 0; first < m.g.n_mats; first += cap)
      if (int rc = run_batch(m.g, first, std::min(cap, m.g.n_mats - first), *hp, static_cast<float*>(workspace), st)) return rc;
  }
  return CANZ_OK;
}
