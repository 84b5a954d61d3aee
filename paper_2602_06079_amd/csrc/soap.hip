// canz_soap_step / canz_soap_workspace_bytes: the SOAP step the paper runs through the same
// planner as Muon and Shampoo ("Generalization to Other Optimizers (Shampoo & SOAP)", App. C;
// App. B.3), per matrix (Adam in the eigenbasis of Shampoo's statistics):
//   M <- beta1 M + (1 - beta1) G;   G' = Q_L^T G Q_R,  M' = Q_L^T M Q_R;
//   V <- beta2 V + (1 - beta2) G'^2;   N' = m / (sqrt(v) + eps);   N = Q_L N' Q_R^T;
//   P <- P (1 - lr wd) - lr N  (or Delta W = -lr N);
//   L <- beta2 L + (1 - beta2) G G^T,  R <- beta2 R + (1 - beta2) G^T G;
//   on a refresh step  Q_L <- orthogonal factor of QR(L Q_L),  Q_R likewise.
// Everything is fp32 on v_mfma_f32_32x32x2_f32 (the products) and plain vector code.
//
// The products all take the form C[i][j] = sum_k P[i][k] Q[j][k].  The rotation into the basis
// runs right side first with its result written transposed, (G Q_R)^T = Q_R^T-rows times G-rows,
// so that the left side finds its second operand contiguous along k; the rotation back runs
// the same way round.  G and M travel through the rotation as two problems of one launch that
// share the basis operand.
//
// QR refresh: blocked Householder factorisation with panels of 32 columns, on the transposed
// matrix (a column of S = L Q is a contiguous row of the working copy).  One workgroup per
// matrix factors a panel in place (each wavefront owns whole columns of the panel, so the only
// block-wide synchronisation is two barriers per column); the trailing columns are updated,
// and afterwards the orthogonal factor is accumulated from the last panel to the first, with
// the compact WY form H = I - V T V^T through three products per panel:
//   Y = V [T^T | T]   (one small product against the panel's stored T),
//   W = (columns) V,  (columns) -= W Y^T.
// Tile boundaries of these products are rounded down to multiples of 128; the extra rows and
// columns they touch either hold zeros in V (no effect) or are columns the factorisation has
// finished with (R is never needed: only Q is).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>

#include "canz.h"
#include "canz_internal.h"
#include "device_util.h"
#include "f32_mfma_gemm.h"
#include "kernels.h"

namespace canz {
namespace {

using namespace f32mfma;

constexpr int64_t MAX_EXTENT = 32768;
constexpr size_t BATCH_BYTES = size_t(32) << 30;   // working matrices of one launch batch: the more matrices share
                                                     // a batch, the more workgroups the panel kernel of a refresh has
constexpr int QB = 32;            // panel width of the QR factorisation
constexpr int QTH = 1024;         // threads of the panel kernel: 16 wavefronts
constexpr int QWAVES = QTH / 64;

// G (bf16 or fp32, whole or tp column fragments) and the momentum M <- beta1 M + (1 - beta1) G
// (fp32, dense, in the caller's buffer) -> fp32 working copies of both, in both orientations,
// zero outside rows x cols: gm [nb][2][rp][cp] (G, then M) and gmt [nb][2][cp][rp].
__global__ __launch_bounds__(NTH) void k_soap_load(Shape s, PtrTable grad, int grad_dtype, PtrTable mom, float beta1,
                                                    int64_t rp, int64_t cp, float* __restrict__ gm, float* __restrict__ gmt) {
  __shared__ float tg[64][65], tm[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const int wf = static_cast<int>(s.wfrag);
  const int64_t plane = rp * cp;
  float* gs = gm + static_cast<int64_t>(b) * 2 * plane;
  float* gt = gmt + static_cast<int64_t>(b) * 2 * plane;
  float* m = static_cast<float*>(mom.p[b]);
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
    gs[static_cast<int64_t>(row) * cp + col] = g;
    gs[plane + static_cast<int64_t>(row) * cp + col] = mv;
    tg[r][c] = g;
    tm[r][c] = mv;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;  // r: column of G, c: row of G
    gt[static_cast<int64_t>(c0 + r) * rp + r0 + c] = tg[c][r];
    gt[plane + static_cast<int64_t>(c0 + r) * rp + r0 + c] = tm[c][r];
  }
}

// Adam in the rotated space.  rot [nb][2][rp][cp] holds G' and M'; V (dense, caller's) is updated
// in place; N' = (c1 M') / (sqrt(c2 V) + eps) goes to np [nb][rp][cp], or transposed to
// [nb][cp][rp]; zero outside rows x cols.
__global__ __launch_bounds__(NTH) void k_soap_adam(Shape s, PtrTable var, const float* __restrict__ rot, int64_t rp,
                                                    int64_t cp, float beta2, float c1, float c2, float eps, int transposed,
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
      const float g = gr[at], m = gr[plane + at];
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
// column c is row c of wk (row length dp).  One workgroup per matrix.
//   vall row j0 + c   <- reflector v_c (zero before row j0 + c, 1 there)
//   vkt  [dp][32]     <- the same reflectors, row r holds v_0[r] .. v_31[r]       (rows >= j0)
//   tt   [128][32]    <- rows 0..31 T, rows 32..63 T^T   (H_0 ... H_31 = I - V T V^T)
// and the panel's later columns are updated in place as each reflector is found.  Columns at or
// beyond d (padding) and columns that are already zero below the diagonal get tau = 0 (H = I).
struct QrPanel {
  float* wk;
  float* vall;
  float* vkt;
  float* tt;
  int64_t dp, d;
  int64_t s_wk, s_vall, s_vkt, s_tt;   // batch strides
  int j0;
};

// Dot product of two rows of nvec float4 over the lanes of a wavefront (each lane's share; the caller
// sums over the lanes).  QUN pairs of loads are issued before the first is used, so that a pass over a
// row costs a few memory round trips instead of one per 256 elements.
constexpr int QUN = 4;
__device__ __forceinline__ float row_dot(const f32x4* a, const f32x4* b, int nvec, int lane) {
  float dot = 0.f;
  for (int q0 = lane; q0 < nvec; q0 += 64 * QUN) {
    f32x4 x[QUN], y[QUN];
#pragma unroll
    for (int u = 0; u < QUN; ++u) {
      const int q = min(q0 + 64 * u, nvec - 1);     // in bounds; the surplus loads are not used
      x[u] = a[q];
      y[u] = b[q];
    }
#pragma unroll
    for (int u = 0; u < QUN; ++u)
      if (q0 + 64 * u < nvec) dot += (x[u][0] * y[u][0] + x[u][1] * y[u][1]) + (x[u][2] * y[u][2] + x[u][3] * y[u][3]);
  }
  return dot;
}

__global__ __launch_bounds__(QTH) void k_qr_panel(QrPanel a) {
  __shared__ float s_g[QB][QB + 1], s_t[QB][QB + 1], s_tau[QB], s_part[QWAVES], s_head[2];
  const int b = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t dp = a.dp;
  const int j0 = a.j0;
  const int nvec = static_cast<int>(dp - j0) / 4;             // float4 per row in the rows j0 .. dp - 1
  float* wk = a.wk + static_cast<int64_t>(b) * a.s_wk;
  float* vrows = a.vall + static_cast<int64_t>(b) * a.s_vall;
  auto col = [&](int c) { return reinterpret_cast<f32x4*>(wk + static_cast<int64_t>(j0 + c) * dp + j0); };
  auto vrow = [&](int c) { return reinterpret_cast<f32x4*>(vrows + static_cast<int64_t>(j0 + c) * dp + j0); };

  // head of column 0: sum of squares below the diagonal, and the diagonal element
  {
    float ss = 0.f;
    const f32x4* x = col(0);
    for (int q = t; q < nvec; q += QTH) {
      const f32x4 v = x[q];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (4 * q + e > 0) ss += v[e] * v[e];
    }
    ss = wave_sum(ss);
    if (lane == 0) s_part[wave] = ss;
    __syncthreads();
    if (t == 0) {
      float tot = 0.f;
      for (int w = 0; w < QWAVES; ++w) tot += s_part[w];
      s_head[0] = tot;
      s_head[1] = wk[static_cast<int64_t>(j0) * dp + j0];
    }
    __syncthreads();
  }

  for (int c = 0; c < QB; ++c) {
    const float ss = s_head[0], al = s_head[1];
    float tau = 0.f, scale = 0.f;
    if (j0 + c < a.d && ss > 0.f) {
      const float nrm = sqrtf(__builtin_fmaf(al, al, ss));
      const float beta = al >= 0.f ? -nrm : nrm;
      tau = (beta - al) / beta;
      scale = 1.f / (al - beta);
    }
    {
      const f32x4* x = col(c);
      f32x4* v = vrow(c);
      for (int q = t; q < nvec; q += QTH) {
        const f32x4 xv = x[q];
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * q + e;
          o[e] = r < c ? 0.f : (r == c ? 1.f : xv[e] * scale);
        }
        v[q] = o;
      }
      if (t == 0) s_tau[c] = tau;
    }
    __syncthreads();   // v_c is complete; every thread has read the head of column c

    for (int task = wave; task < QB - 1; task += QWAVES) {
      const f32x4* v = vrow(c);
      if (task < c) {                       // v_task . v_c for the triangular factor
        const float dot = wave_sum(row_dot(vrow(task), v, nvec, lane));
        if (lane == 0) s_g[task][c] = dot;
      } else {                              // column c2 <- H_c column c2
        const int c2 = task + 1;
        f32x4* x = col(c2);
        float f = 0.f;
        if (tau != 0.f) f = tau * wave_sum(row_dot(x, v, nvec, lane));
        const bool next = c2 == c + 1;      // this wavefront also takes the head of the next column
        if (tau != 0.f || next) {
          float ss2 = 0.f, al2 = 0.f;
          for (int q0 = lane; q0 < nvec; q0 += 64 * QUN) {
            f32x4 xv[QUN], y[QUN];
#pragma unroll
            for (int u = 0; u < QUN; ++u) {
              const int q = min(q0 + 64 * u, nvec - 1);
              xv[u] = x[q];
              y[u] = v[q];
            }
#pragma unroll
            for (int u = 0; u < QUN; ++u) {
              const int q = q0 + 64 * u;
              if (q < nvec) {
                if (tau != 0.f) {
#pragma unroll
                  for (int e = 0; e < 4; ++e) xv[u][e] = __builtin_fmaf(-f, y[u][e], xv[u][e]);
                  x[q] = xv[u];
                }
                if (next) {
#pragma unroll
                  for (int e = 0; e < 4; ++e) {
                    const int r = 4 * q + e;
                    if (r > c2) ss2 += xv[u][e] * xv[u][e];
                    if (r == c2) al2 = xv[u][e];
                  }
                }
              }
            }
          }
          if (next) {
            ss2 = wave_sum(ss2);
            al2 = wave_sum(al2);            // one lane holds the diagonal element, the others 0
            if (lane == 0) s_head[0] = ss2, s_head[1] = al2;
          }
        }
      }
    }
    __syncthreads();   // the panel is updated; the next head and the dot products are in LDS
  }

  // T, forward and column by column: T[c][c] = tau_c, T[0:c, c] = -tau_c T[0:c, 0:c] (V^T v_c)
  if (t < QB) {
    const int i = t;
    for (int c = 0; c < QB; ++c) {
      float val = 0.f;
      if (i == c) {
        val = s_tau[c];
      } else if (i < c) {
        float sum = 0.f;
        for (int l = i; l < c; ++l) sum = __builtin_fmaf(s_t[i][l], s_g[l][c], sum);
        val = -s_tau[c] * sum;
      }
      s_t[i][c] = val;
    }
  }
  __syncthreads();
  float* tt = a.tt + static_cast<int64_t>(b) * a.s_tt;
  for (int idx = t; idx < 2 * QB * QB; idx += QTH) {
    const int row = idx >> 5, l = idx & 31;
    tt[idx] = row < QB ? s_t[row][l] : s_t[l][row - QB];
  }
  float* vkt = a.vkt + static_cast<int64_t>(b) * a.s_vkt;
  for (int64_t r = j0 + t; r < dp; r += QTH) {
    float x[QB];
#pragma unroll
    for (int l = 0; l < QB; ++l) x[l] = vrows[static_cast<int64_t>(j0 + l) * dp + r];
    f32x4* dst = reinterpret_cast<f32x4*>(vkt + r * QB);
#pragma unroll
    for (int q = 0; q < QB / 4; ++q) {
      f32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = x[4 * q + e];
      dst[q] = o;
    }
  }
}

struct Carve {   // float offsets into the workspace of one launch batch
  size_t gm, gmt, t1, rot, np, yt, ql, qlt, qr, qrt, stat, wk, vall, vkt, tt, ybuf, wt, qt, total_bytes;
};

struct Sides {
  bool left, right;
};
Sides sides(const canz_soap_group& g, const canz_soap_hparams& hp) {
  return {g.rows <= hp.max_precond_dim, g.cols <= hp.max_precond_dim};
}

Carve carve(int64_t rows, int64_t cols, int nb, Sides u, bool refresh) {
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
    c.vall = take(nb * (dm + 96) * dm);
    c.vkt = take(nb * dm * dm);
    c.tt = take(nb * dm * 128);        // dm / 32 panels of [128][32]
    c.ybuf = take(nb * dm * 128);
    c.wt = take(nb * dm * 128);
    c.qt = take(nb * dm * dm);
  }
  c.total_bytes = off * sizeof(float);
  return c;
}

int batch_cap(const canz_soap_group& g, const canz_soap_hparams& hp) {
  const size_t one = carve(g.rows, g.cols, 1, sides(g, hp), hp.refresh != 0).total_bytes;
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
    if (bad(g.mom[i]) || bad(g.var[i])) return fail(CANZ_EINVAL, "group %d: moment %d null or not 16-byte aligned", idx, i);
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
  float *wk = ws + c.wk, *vall = ws + c.vall, *vkt = ws + c.vkt, *tt = ws + c.tt, *ybuf = ws + c.ybuf, *wt = ws + c.wt,
        *qt = ws + c.qt;
  const int64_t s_vall = (dp + 96) * dp, s_thin = dp * 128;
  auto fill = [&](float* p, int64_t elems, int64_t ld, int identity) {
    const unsigned blocks = static_cast<unsigned>(std::min<int64_t>(2048, (elems + NTH - 1) / NTH));
    hipLaunchKernelGGL(k_soap_fill, dim3(blocks, nb), dim3(NTH), 0, st, p, elems, ld, identity);
  };
  prof_mark(st, CANZ_KERNEL_SOAP_PANEL, true);
  fill(vall, s_vall, dp, 0);
  fill(vkt, dd, dp, 0);
  fill(tt, s_thin, 128, 0);
  fill(qt, dd, dp, 1);
  prof_mark(st, CANZ_KERNEL_SOAP_PANEL, false);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "refresh fill: %s", hipGetErrorString(e));

  // working copy, transposed: wk[c][r] = (S q)[r][c] = sum_k qt_old[c][k] S[r][k]
  ShGemm p0{};
  p0.M = dp, p0.N = dp, p0.K = dp, p0.ldp = dp, p0.ldq = dp, p0.sp = dd, p0.sq = dd;
  p0.P = qt_old, p0.Q = stat, p0.c = wk;
  CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(p0, nb, none, s, o, st)), "refresh product");

  // Y of panel j0: ybuf[r][0..31] = (V T^T)[r], ybuf[r][32..63] = (V T)[r], rows from klo on
  auto y_product = [&](int64_t j0, int64_t klo) {
    ShGemm y{};
    y.M = dp - klo, y.N = 128, y.K = QB, y.ldp = QB, y.ldq = QB, y.sp = dd, y.sq = s_thin;
    y.P = vkt + (j0 / QB) * dp * QB + klo * QB, y.Q = tt + (j0 / QB) * 128 * QB;
    y.c = ybuf + klo * 128, y.ldc = 128, y.sc = s_thin;
    return y;
  };
  // W = (rows lo.. of m) V_panel over the rows j0.. of the reflectors: wt[j][0..31]
  auto w_product = [&](const float* m, int64_t lo, int64_t j0) {
    ShGemm w{};
    w.M = dp - lo, w.N = 128, w.K = dp - j0, w.ldp = dp, w.ldq = dp, w.sp = dd, w.sq = s_vall;
    w.P = m + lo * dp + j0, w.Q = vall + j0 * dp + j0;
    w.c = wt + lo * 128, w.ldc = 128, w.sc = s_thin;
    return w;
  };
  // (rows lo.., columns klo.. of m) -= W Y^T with Y the columns ycol .. ycol + 31 of ybuf
  auto sub_product = [&](float* m, int64_t lo, int64_t klo, int ycol) {
    ShGemm u{};
    u.M = dp - lo, u.N = dp - klo, u.K = QB, u.ldp = 128, u.ldq = 128, u.sp = s_thin, u.sq = s_thin;
    u.P = wt + lo * 128, u.Q = ybuf + klo * 128 + ycol;
    u.c = m + lo * dp + klo, u.ldc = dp, u.sc = dd;
    return u;
  };

  for (int64_t j0 = 0; j0 < d; j0 += QB) {
    QrPanel a{};
    a.wk = wk, a.vall = vall, a.vkt = vkt + (j0 / QB) * dp * QB, a.tt = tt + (j0 / QB) * 128 * QB;
    a.dp = dp, a.d = d, a.s_wk = dd, a.s_vall = s_vall, a.s_vkt = dd, a.s_tt = s_thin;
    a.j0 = static_cast<int>(j0);
    prof_mark(st, CANZ_KERNEL_SOAP_PANEL, true);
    hipLaunchKernelGGL(k_qr_panel, dim3(nb), dim3(QTH), 0, st, a);
    prof_mark(st, CANZ_KERNEL_SOAP_PANEL, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "panel kernel: %s", hipGetErrorString(e));
    const int64_t jlo = floor128(j0 + QB), klo = floor128(j0);
    if (jlo >= dp) continue;   // no columns after this panel
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(y_product(j0, klo), nb, none, s, o, st)), "QR (Y)");
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(w_product(wk, jlo, j0), nb, none, s, o, st)), "QR (W)");
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_SUB, false>(sub_product(wk, jlo, klo, 0), nb, none, s, o, st)), "QR (update)");
  }
  // Q = H(0) H(1) ... applied to the identity from the last panel to the first
  for (int64_t j0 = (d - 1) / QB * QB; j0 >= 0; j0 -= QB) {
    const int64_t lo = floor128(j0);
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(y_product(j0, lo), nb, none, s, o, st)), "Q (Y)");
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_PLAIN, false>(w_product(qt, lo, j0), nb, none, s, o, st)), "Q (W)");
    CANZ_HIP(CANZ_KERNEL_SOAP_QR, (launch_gemm<SE_SUB, false>(sub_product(qt, lo, lo, QB), nb, none, s, o, st)), "Q (update)");
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
  const Carve c = carve(g.rows, g.cols, nb, u, hp.refresh != 0);
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

  prof_mark(st, CANZ_KERNEL_SOAP_LOAD, true);
  hipLaunchKernelGGL(k_soap_load, tiles, dim3(NTH), 0, st, s, grad, g.grad_dtype, mom, hp.beta1, rp, cp, gm, gmt);
  // the bases: padded copies in both orientations (q [d][d] dense -> q, q^T, zero outside d x d)
  auto load_basis = [&](void* const* tab, int64_t d, int64_t dp, float* straight, float* transposed) {
    Shape sq{};
    sq.rows = d, sq.cols = d, sq.tp = 1, sq.wfrag = d;
    PtrTable q{};
    for (int i = 0; i < nb; ++i) q.p[i] = tab[first + i];
    hipLaunchKernelGGL(k_sh_load, dim3(static_cast<unsigned>(dp / 64), static_cast<unsigned>(dp / 64), static_cast<unsigned>(nb)),
                       dim3(NTH), 0, st, sq, q, static_cast<int>(CANZ_DT_F32), dp, dp, straight, transposed);
  };
  if (u.left) load_basis(g.qleft, g.rows, rp, ql, qlt);
  if (u.right) load_basis(g.qright, g.cols, cp, qr, qrt);
  prof_mark(st, CANZ_KERNEL_SOAP_LOAD, false);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "load kernels: %s", hipGetErrorString(e));

  // rotation into the bases: G' and M' as problems 2 b and 2 b + 1 of one launch
  if (u.left && u.right) {
    ShGemm a{};   // t1 = (X Q_R)^T: [cp][rp]
    a.M = cp, a.N = rp, a.K = cp, a.ldp = cp, a.ldq = cp, a.sp = cp * cp, a.pdiv = 2, a.sq = plane;
    a.P = qrt, a.Q = gm, a.c = t1;
    CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(a, 2 * nb, none, s, o, st)), "rotation (right)");
    ShGemm bq{};  // rot = Q_L^T (X Q_R): [rp][cp]
    bq.M = rp, bq.N = cp, bq.K = rp, bq.ldp = rp, bq.ldq = rp, bq.sp = rp * rp, bq.pdiv = 2, bq.sq = plane;
    bq.P = qlt, bq.Q = t1, bq.c = rot;
    CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(bq, 2 * nb, none, s, o, st)), "rotation (left)");
  } else if (u.left) {
    ShGemm bq{};  // rot = Q_L^T X with X^T as the second operand
    bq.M = rp, bq.N = cp, bq.K = rp, bq.ldp = rp, bq.ldq = rp, bq.sp = rp * rp, bq.pdiv = 2, bq.sq = plane;
    bq.P = qlt, bq.Q = gmt, bq.c = rot;
    CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(bq, 2 * nb, none, s, o, st)), "rotation (left)");
  } else {
    ShGemm a{};   // rot = X Q_R
    a.M = rp, a.N = cp, a.K = cp, a.ldp = cp, a.ldq = cp, a.sp = plane, a.sq = cp * cp, a.qdiv = 2;
    a.P = gm, a.Q = qrt, a.c = rot;
    CANZ_HIP(CANZ_KERNEL_SOAP_ROTATE, (launch_gemm<SE_PLAIN, false>(a, 2 * nb, none, s, o, st)), "rotation (right)");
  }

  {
    const double c1 = hp.bias_correction ? 1.0 / (1.0 - std::pow(static_cast<double>(hp.beta1), hp.step)) : 1.0;
    const double c2 = hp.bias_correction ? 1.0 / (1.0 - std::pow(static_cast<double>(hp.beta2), hp.step)) : 1.0;
    const int transposed = u.left && !u.right;
    prof_mark(st, CANZ_KERNEL_SOAP_ADAM, true);
    hipLaunchKernelGGL(k_soap_adam, tiles, dim3(NTH), 0, st, s, var, rot, rp, cp, hp.beta2, static_cast<float>(c1),
                       static_cast<float>(c2), hp.eps, transposed, np);
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

  // statistics (and, on a refresh step, the new basis) side by side
  auto one_side = [&](void* const* stat_tab, void* const* q_tab, int64_t d, int64_t dp, int64_t kp, const float* side,
                      const float* qt_old) -> int {
    PtrTable tab{};
    for (int i = 0; i < nb; ++i) tab.p[i] = stat_tab[first + i];
    ShGemm q{};
    q.M = dp, q.N = dp, q.K = kp, q.ldp = kp, q.ldq = kp, q.sp = 2 * plane, q.sq = 2 * plane;
    q.P = side, q.Q = side, q.c = stat, q.d = d, q.beta = hp.beta2, q.gscale = 1.f - hp.beta2, q.eps = 0.f;
    CANZ_HIP(CANZ_KERNEL_SOAP_STAT, (launch_gemm<SE_STAT, true>(q, nb, tab, s, o, st)), "statistics kernel");
    if (!hp.refresh) return CANZ_OK;
    return refresh_side(q_tab, first, nb, d, dp, stat, qt_old, ws, c, s, o, st);
  };
  if (u.left)
    if (int rc = one_side(g.left, g.qleft, g.rows, rp, cp, gm, qlt)) return rc;
  if (u.right)
    if (int rc = one_side(g.right, g.qright, g.cols, cp, rp, gmt, qrt)) return rc;
  return CANZ_OK;
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
  for (int i = 0; i < n_groups; ++i) {
    if (int rc = check_group(g[i], i, false, *hp)) return rc;
    if (g[i].n_mats == 0) continue;
    need = std::max(need, carve(g[i].rows, g[i].cols, std::min(g[i].n_mats, batch_cap(g[i], *hp)), sides(g[i], *hp),
                                hp->refresh != 0).total_bytes);
  }
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
  for (int i = 0; i < n_groups; ++i) {
    const int cap = batch_cap(g[i], *hp);
    for (int first = 0; first < g[i].n_mats; first += cap)
      if (int rc = run_batch(g[i], first, std::min(cap, g[i].n_mats - first), *hp, static_cast<float*>(workspace), st)) return rc;
  }
  return CANZ_OK;
}
