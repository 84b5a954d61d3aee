// canz_shampoo_step / canz_shampoo_workspace_bytes: the Shampoo step the paper runs through
// the same planner as Muon ("Generalization to Other Optimizers (Shampoo & SOAP)", App. C;
// App. B.3), per matrix:
//   L <- beta L + G G^T,  R <- beta R + G^T G,
//   O = (L + eps I)^(-1/4) G (R + eps I)^(-1/4),  P <- P (1 - lr wd) - lr O  (or Delta W = -lr O).
// Everything is fp32 (the statistics span many orders of magnitude; bf16 would lose the small
// eigenvalues the inverse root amplifies), on v_mfma_f32_32x32x2_f32.
//
// All products have the form C[i][j] = sum_k P[i][k] Q[j][k] with both operands contiguous
// along k: the statistics are Gram products of G in its two orientations (both are written by
// the load kernel), and every matrix of the root iteration is a polynomial in the symmetric
// A = S + eps I, hence symmetric itself, so "times Q" and "times Q^T" coincide.  Symmetric
// products compute only the tiles on or above the diagonal and write the mirror tile from the
// same accumulators, which halves their work and keeps the iterates symmetric bit for bit.
//
// Inverse fourth root (coupled Newton iteration for the inverse p-th root, p = 4): from
// M = z A, X = z^(1/4) I with z = 5 / (2 ||A||_F), repeat T = (5 I - M) / 4, X <- X T,
// M <- T^4 M; M -> I and X -> A^(-1/4).  Four products per round: X T, T T, T^2 T^2, T^4 M (the
// last one also writes the next T).  The round count is fixed by the caller: no test of
// convergence is read back, so the step never synchronises and can be captured in a graph.
//
// Working extents are multiples of 128 (zero padding: the padded part of every iterate is a
// separate diagonal block that never mixes with the matrix and is multiplied by zeros at the end).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <vector>

#include "canz.h"
#include "canz_internal.h"
#include "device_util.h"
#include "kernels.h"

namespace canz {
namespace {

constexpr int SB = 128;          // block tile (rows and columns)
constexpr int SK = 32;           // k extent of one LDS stage: long enough that the next stage's global loads land under it
constexpr int NTH = 256;
constexpr int LDS_LD = SB + 5;   // odd row length: the k-major stores of a stage spread over all banks
constexpr int FLUSH = 16;        // stages (512 k) between folds of the running accumulator
constexpr int NPART = 64;        // partial sums per matrix of the Frobenius norm
constexpr int64_t MAX_EXTENT = 32768;
constexpr size_t BATCH_BYTES = size_t(8) << 30;
constexpr size_t ALIGN = 256;

inline int64_t pad128(int64_t x) { return (x + SB - 1) / SB * SB; }
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

enum { SE_STAT = 0, SE_PLAIN = 1, SE_MT = 2, SE_OUT = 3 };

struct ShGemm {
  int64_t M, N, K;      // multiples of 128, 128, 32
  int64_t ldp, ldq;     // row strides of P [M][K] and Q [N][K]
  int64_t sp, sq;       // batch strides
  const float* P;
  const float* Q;
  float* c;             // [nb][M][N] output, row stride N, batch stride M * N
  float* c2;            // SE_MT: the next T = 5/4 I - 1/4 C
  // SE_STAT: the caller's statistic (d x d, dense) is updated in place and A = S + eps I is written to c
  int64_t d;
  float beta, eps;
};

// Straight and (for off-diagonal tiles of a symmetric product) mirrored store of the 16 values
// a lane holds of a 32 x 32 accumulator tile: rows row0 + 8 (r / 4) + (r % 4), column col.
__device__ __forceinline__ void put16(float* C, int64_t ld, int row0, int col, const float (&v)[16], bool mirror) {
#pragma unroll
  for (int r = 0; r < 16; ++r) C[static_cast<int64_t>(row0 + 8 * (r >> 2) + (r & 3)) * ld + col] = v[r];
  if (mirror) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 q;
#pragma unroll
      for (int e = 0; e < 4; ++e) q[e] = v[4 * g + e];
      *reinterpret_cast<f32x4*>(C + static_cast<int64_t>(col) * ld + row0 + 8 * g) = q;
    }
  }
}

template <int EPI, bool SYM>
__global__ __launch_bounds__(NTH) void k_sh_gemm(ShGemm g, PtrTable stat, Shape s, OutSpec o) {
  __shared__ float sP[2][SK][LDS_LD];  // k-major: the lanes of one MFMA operand read consecutive rows
  __shared__ float sQ[2][SK][LDS_LD];

  const int tiles_m = static_cast<int>(g.M / SB), tiles_n = static_cast<int>(g.N / SB);
  const int per = SYM ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  const int b = blockIdx.x / per;
  int tix = blockIdx.x - b * per;
  int tm, tn;
  if (SYM) {
    // upper triangle row by row: row tm holds the columns tm .. tiles_m - 1
    tm = 0;
    for (int len = tiles_m; tix >= len; --len) tix -= len, ++tm;
    tn = tm + tix;
  } else {
    tm = tix / tiles_n;
    tn = tix - tm * tiles_n;
  }

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const float* Pg = g.P + static_cast<int64_t>(b) * g.sp + static_cast<int64_t>(tm) * SB * g.ldp;
  const float* Qg = g.Q + static_cast<int64_t>(b) * g.sq + static_cast<int64_t>(tn) * SB * g.ldq;

  const int ld_row = t >> 3, ld_k = (t & 7) * 4;  // rows ld_row + 32 x (x = 0..3), 4 consecutive k
  // Long sums of the statistics (k up to the other extent of the matrix, terms of one sign on the
  // diagonal) are folded into a second accumulator every FLUSH stages; the products of the root
  // iteration and the preconditioning accumulate in one go (their rounding, about 1e-5 relative,
  // is corrected by the following rounds and is far below the tolerance of the update).
  constexpr bool FOLD = EPI == SE_STAT;
  f32x16 acc[2][2], tot[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f, tot[i][j][r] = 0.f;

  // Two register sets: stage kt + 2 is requested while stage kt is multiplied and stage kt + 1
  // waits in the other set, so a request has two stage times (about 3.5 us) to land.
  f32x4 pv[2][4], qv[2][4];
  auto fetch = [&](int kt, int set) {
    const int64_t k0 = static_cast<int64_t>(kt) * SK + ld_k;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      pv[set][x] = *reinterpret_cast<const f32x4*>(Pg + static_cast<int64_t>(ld_row + 32 * x) * g.ldp + k0);
      qv[set][x] = *reinterpret_cast<const f32x4*>(Qg + static_cast<int64_t>(ld_row + 32 * x) * g.ldq + k0);
    }
  };
  auto stash = [&](int buf, int set) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        sP[buf][ld_k + c][ld_row + 32 * x] = pv[set][x][c];
        sQ[buf][ld_k + c][ld_row + 32 * x] = qv[set][x][c];
      }
  };
  // one stage: LDS buffer `buf` holds stage kt, register set `other` stage kt + 1, set `mine` is free
  const int nk = static_cast<int>(g.K / SK);   // a multiple of 4: K is a multiple of 128
  auto stage = [&](int kt, int buf, int mine, int other) {
    if (kt + 2 < nk) fetch(kt + 2, mine);
#pragma unroll
    for (int k = 0; k < SK; k += 2) {
      float fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = sP[buf][k + (lane >> 5)][wm * 64 + i * 32 + (lane & 31)];
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = sQ[buf][k + (lane >> 5)][wn * 64 + j * 32 + (lane & 31)];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (FOLD && ((kt + 1) % FLUSH == 0 || kt + 1 == nk)) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) tot[i][j][r] += acc[i][j][r], acc[i][j][r] = 0.f;
    }
    if (kt + 1 < nk) stash(buf ^ 1, other);
    __syncthreads();  // stage kt + 1 is complete in LDS; every wavefront is done reading stage kt
  };
  fetch(0, 0);
  fetch(1, 1);
  stash(0, 0);
  __syncthreads();
  for (int kt = 0; kt < nk; kt += 2) {
    stage(kt, 0, 0, 1);
    stage(kt + 1, 1, 1, 0);
  }
  if (!FOLD) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) tot[i][j] = acc[i][j];
  }

  const int row_base = tm * SB + wm * 64 + 4 * (lane >> 5);
  const int col_base = tn * SB + wn * 64 + (lane & 31);
  const bool mirror = SYM && tm != tn;
  const int64_t cb = static_cast<int64_t>(b) * g.M * g.N;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int row0 = row_base + i * 32, col = col_base + j * 32;
      float v[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = tot[i][j][r];
      if (EPI == SE_OUT) {
        store_out_tile(o, s, b, row0, col, v);
      } else if (EPI == SE_PLAIN) {
        put16(g.c + cb, g.N, row0, col, v, mirror);
      } else if (EPI == SE_MT) {
        put16(g.c + cb, g.N, row0, col, v, mirror);
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = (row0 + 8 * (r >> 2) + (r & 3) == col ? 1.25f : 0.f) - 0.25f * v[r];
        put16(g.c2 + cb, g.N, row0, col, v, mirror);
      } else {  // SE_STAT
        float* S = static_cast<float*>(stat.p[b]);
        const int d = static_cast<int>(g.d);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + 8 * (r >> 2) + (r & 3);
          float val = 0.f;
          if (row < d && col < d) {
            const int64_t at = static_cast<int64_t>(row) * d + col;
            val = v[r];
            if (g.beta != 0.f) val += g.beta * S[at];
            S[at] = val;
            if (mirror) S[static_cast<int64_t>(col) * d + row] = val;
            if (row == col) val += g.eps;
          }
          v[r] = val;
        }
        put16(g.c + cb, g.N, row0, col, v, mirror);
      }
    }
  }
}

template <int EPI, bool SYM>
hipError_t launch_gemm(const ShGemm& g, int nb, const PtrTable& stat, const Shape& s, const OutSpec& o, hipStream_t st) {
  const int64_t tm = g.M / SB, tn = g.N / SB;
  const int64_t blocks = (SYM ? tm * (tm + 1) / 2 : tm * tn) * nb;
  hipLaunchKernelGGL((k_sh_gemm<EPI, SYM>), dim3(static_cast<unsigned>(blocks)), dim3(NTH), 0, st, g, stat, s, o);
  return hipGetLastError();
}

// G (bf16 or fp32, whole or tp column fragments) -> fp32 working copies in both orientations,
// zero outside rows x cols.  One block per 64 x 64 tile; the transposed copy goes through LDS.
__global__ __launch_bounds__(NTH) void k_sh_load(Shape s, PtrTable grad, int grad_dtype, int64_t rp, int64_t cp,
                                                  float* __restrict__ gs, float* __restrict__ gt) {
  __shared__ float tile[64][65];
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const int wf = static_cast<int>(s.wfrag);
  float* gsb = gs + static_cast<int64_t>(b) * rp * cp;
  float* gtb = gt + static_cast<int64_t>(b) * rp * cp;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;
    const int row = r0 + r, col = c0 + c;
    float val = 0.f;
    if (row < s.rows && col < s.cols) {
      const int f = col / wf;
      const int64_t at = static_cast<int64_t>(row) * wf + (col - f * wf);
      val = grad_dtype == CANZ_DT_BF16 ? static_cast<float>(static_cast<const __bf16*>(grad.p[b * s.tp + f])[at])
                                       : static_cast<const float*>(grad.p[b * s.tp + f])[at];
    }
    gsb[static_cast<int64_t>(row) * cp + col] = val;
    tile[r][c] = val;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, r = idx >> 6, c = idx & 63;  // r: column of G, c: row of G
    gtb[static_cast<int64_t>(c0 + r) * rp + r0 + c] = tile[c][r];
  }
}

// partial[b][p] = sum of squares of the elements p, p + NPART * NTH, ... (in blocks of NTH) of A[b]
__global__ __launch_bounds__(NTH) void k_sh_sumsq(const float* __restrict__ a, int64_t elems, float* __restrict__ partial) {
  __shared__ float wsum[NTH / 64];
  const int b = blockIdx.y, p = blockIdx.x, t = threadIdx.x;
  const float* ab = a + static_cast<int64_t>(b) * elems;
  float ss = 0.f;
  for (int64_t i = static_cast<int64_t>(p) * NTH + t; i < elems; i += static_cast<int64_t>(NPART) * NTH) ss += ab[i] * ab[i];
  ss = wave_sum(ss);
  if ((t & 63) == 0) wsum[t >> 6] = ss;
  __syncthreads();
  if (t == 0) partial[b * NPART + p] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
}

// Start of the root iteration: z = 5 / (2 ||A||_F); M = z A; T = 5/4 I - 1/4 M; X = z^(1/4) I.
__global__ __launch_bounds__(NTH) void k_sh_init(const float* __restrict__ a, const float* __restrict__ partial,
                                                  int64_t dp, float* __restrict__ x, float* __restrict__ m,
                                                  float* __restrict__ tt) {
  const int b = blockIdx.y;
  double sum = 0.0;
  for (int i = 0; i < NPART; ++i) sum += static_cast<double>(partial[b * NPART + i]);
  const float nrm = static_cast<float>(sqrt(sum));
  const float z = nrm > 0.f ? 2.5f / nrm : 1.f;
  const float x0 = sqrtf(sqrtf(z));
  const int64_t elems = dp * dp, off = static_cast<int64_t>(b) * elems;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * NTH + threadIdx.x; i < elems; i += static_cast<int64_t>(gridDim.x) * NTH) {
    const bool diag = (i / dp) == (i % dp);
    const float mv = z * a[off + i];
    m[off + i] = mv;
    tt[off + i] = (diag ? 1.25f : 0.f) - 0.25f * mv;
    x[off + i] = diag ? x0 : 0.f;
  }
}

struct Carve {   // float offsets into the workspace of one launch batch
  size_t gs, gt, tmp, lroot, rroot, a, x[2], m[2], t, t2, t4, partial, total_bytes;
};

Carve carve(int64_t rows, int64_t cols, int nb) {
  const size_t rp = pad128(rows), cp = pad128(cols), dm = std::max(rp, cp);
  Carve c{};
  size_t off = 0;
  auto take = [&](size_t floats) {
    const size_t at = off;
    off += align_up(floats * sizeof(float)) / sizeof(float);
    return at;
  };
  c.gs = take(nb * rp * cp), c.gt = take(nb * rp * cp), c.tmp = take(nb * rp * cp);
  c.lroot = take(nb * rp * rp), c.rroot = take(nb * cp * cp);
  c.a = take(nb * dm * dm);
  c.x[0] = take(nb * dm * dm), c.x[1] = take(nb * dm * dm);
  c.m[0] = take(nb * dm * dm), c.m[1] = take(nb * dm * dm);
  c.t = take(nb * dm * dm), c.t2 = take(nb * dm * dm), c.t4 = take(nb * dm * dm);
  c.partial = take(static_cast<size_t>(nb) * NPART);
  c.total_bytes = off * sizeof(float);
  return c;
}

int batch_cap(const canz_shampoo_group& g) {
  const size_t one = carve(g.rows, g.cols, 1).total_bytes;
  const int64_t by_bytes = std::max<int64_t>(1, static_cast<int64_t>(BATCH_BYTES / one));
  return static_cast<int>(std::min<int64_t>(MAX_PTRS / g.tp, by_bytes));
}

int check_hparams(const canz_shampoo_hparams* hp) {
  if (!hp) return fail(CANZ_EINVAL, "null hparams");
  if (hp->root_iters < 1) return fail(CANZ_EINVAL, "root_iters must be >= 1");
  if (!(hp->eps >= 0.f)) return fail(CANZ_EINVAL, "eps must be >= 0");
  if (hp->out_mode != CANZ_OUT_PARAM && hp->out_mode != CANZ_OUT_DELTA)
    return fail(CANZ_EUNSUPPORTED, "unknown out_mode %d", hp->out_mode);
  return CANZ_OK;
}

int check_group(const canz_shampoo_group& g, int idx, bool need_ptrs, int out_mode) {
  if (g.n_mats < 0) return fail(CANZ_EINVAL, "group %d: n_mats < 0", idx);
  if (g.rows < 1 || g.cols < 1) return fail(CANZ_EINVAL, "group %d: empty shape", idx);
  if (g.rows > MAX_EXTENT || g.cols > MAX_EXTENT)
    return fail(CANZ_ESHAPE, "group %d: extent above %lld", idx, static_cast<long long>(MAX_EXTENT));
  if (g.tp < 1 || g.tp > MAX_TP) return fail(CANZ_EINVAL, "group %d: tp must be in 1..%d", idx, MAX_TP);
  if (g.cols % g.tp) return fail(CANZ_ESHAPE, "group %d: cols not divisible by tp", idx);
  if (g.tp > 1 && (g.cols / g.tp) % 8) return fail(CANZ_ESHAPE, "group %d: fragment width not a multiple of 8", idx);
  if (g.grad_dtype != CANZ_DT_F32 && g.grad_dtype != CANZ_DT_BF16)
    return fail(CANZ_EUNSUPPORTED, "group %d: unknown grad_dtype", idx);
  if (g.out_dtype != CANZ_DT_F32 && g.out_dtype != CANZ_DT_BF16)
    return fail(CANZ_EUNSUPPORTED, "group %d: unknown out_dtype", idx);
  if (!need_ptrs || g.n_mats == 0) return CANZ_OK;
  if (!g.grad || !g.left || !g.right || !g.out) return fail(CANZ_EINVAL, "group %d: null pointer table", idx);
  const int n_out = out_mode == CANZ_OUT_DELTA ? g.n_mats * g.tp : g.n_mats;
  auto bad = [](const void* p) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
  for (int i = 0; i < g.n_mats * g.tp; ++i)
    if (bad(g.grad[i])) return fail(CANZ_EINVAL, "group %d: grad[%d] null or not 16-byte aligned", idx, i);
  for (int i = 0; i < g.n_mats; ++i)
    if (bad(g.left[i]) || bad(g.right[i]))
      return fail(CANZ_EINVAL, "group %d: statistic %d null or not 16-byte aligned", idx, i);
  for (int i = 0; i < n_out; ++i)
    if (bad(g.out[i])) return fail(CANZ_EINVAL, "group %d: out[%d] null or not 16-byte aligned", idx, i);
  return CANZ_OK;
}

// One launch batch: matrices first .. first + nb - 1 of group g.
int run_batch(const canz_shampoo_group& g, int first, int nb, const canz_shampoo_hparams& hp, float* ws, hipStream_t st) {
  const int64_t rp = pad128(g.rows), cp = pad128(g.cols);
  const Carve c = carve(g.rows, g.cols, nb);
  Shape s{};
  s.rows = g.rows, s.cols = g.cols;
  s.m = std::min(g.rows, g.cols), s.n = std::max(g.rows, g.cols);
  s.mp = rp, s.np = cp;
  s.tall = g.rows > g.cols;
  s.tp = g.tp;
  s.wfrag = g.cols / g.tp;
  PtrTable grad{}, none{};
  for (int i = 0; i < nb * g.tp; ++i) grad.p[i] = const_cast<void*>(g.grad[first * g.tp + i]);
  OutSpec o{};
  const int per_out = hp.out_mode == CANZ_OUT_DELTA ? g.tp : 1;
  for (int i = 0; i < nb * per_out; ++i) o.out.p[i] = g.out[first * per_out + i];
  o.out_dtype = g.out_dtype;
  o.out_mode = hp.out_mode;
  o.decay = static_cast<float>(1.0 - static_cast<double>(hp.lr) * static_cast<double>(hp.weight_decay));
  o.neg_lr_scale = -hp.lr;

  float *gs = ws + c.gs, *gt = ws + c.gt, *tmp = ws + c.tmp;
  {
    const dim3 grid(static_cast<unsigned>(cp / 64), static_cast<unsigned>(rp / 64), static_cast<unsigned>(nb));
    prof_mark(st, CANZ_KERNEL_SH_LOAD, true);
    hipLaunchKernelGGL(k_sh_load, grid, dim3(NTH), 0, st, s, grad, g.grad_dtype, rp, cp, gs, gt);
    prof_mark(st, CANZ_KERNEL_SH_LOAD, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "load kernel: %s", hipGetErrorString(e));
  }

  // one side: statistic (d x d, in the caller's buffers) from the operand `side` [dp][kp], then
  // its inverse fourth root into `root`
  auto one_side = [&](void* const* stat_tab, int64_t d, int64_t dp, int64_t kp, const float* side, float* root) -> int {
    PtrTable stat{};
    for (int i = 0; i < nb; ++i) stat.p[i] = stat_tab[first + i];
    const int64_t dd = dp * dp;
    float *a = ws + c.a, *x[2] = {ws + c.x[0], ws + c.x[1]}, *m[2] = {ws + c.m[0], ws + c.m[1]};
    float *tt = ws + c.t, *t2 = ws + c.t2, *t4 = ws + c.t4, *partial = ws + c.partial;
    ShGemm q{};
    q.M = dp, q.N = dp, q.K = kp, q.ldp = kp, q.ldq = kp, q.sp = dp * kp, q.sq = dp * kp;
    q.P = side, q.Q = side, q.c = a, q.d = d, q.beta = hp.beta, q.eps = hp.eps;
    CANZ_HIP(CANZ_KERNEL_SH_STAT, (launch_gemm<SE_STAT, true>(q, nb, stat, s, o, st)), "statistics kernel");
    prof_mark(st, CANZ_KERNEL_SH_INIT, true);
    hipLaunchKernelGGL(k_sh_sumsq, dim3(NPART, nb), dim3(NTH), 0, st, a, dd, partial);
    const unsigned init_blocks = static_cast<unsigned>(std::min<int64_t>(4096, (dd + NTH - 1) / NTH));
    hipLaunchKernelGGL(k_sh_init, dim3(init_blocks, nb), dim3(NTH), 0, st, a, partial, dp, x[0], m[0], tt);
    prof_mark(st, CANZ_KERNEL_SH_INIT, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "root start: %s", hipGetErrorString(e));
    auto prod = [&](const float* P, const float* Q, float* C) {
      ShGemm r{};
      r.M = dp, r.N = dp, r.K = dp, r.ldp = dp, r.ldq = dp, r.sp = dd, r.sq = dd;
      r.P = P, r.Q = Q, r.c = C;
      return r;
    };
    int cur = 0;
    for (int it = 0; it < hp.root_iters; ++it) {
      const bool last = it + 1 == hp.root_iters;
      CANZ_HIP(CANZ_KERNEL_SH_ROOT, (launch_gemm<SE_PLAIN, true>(prod(x[cur], tt, last ? root : x[cur ^ 1]), nb, none, s, o, st)),
               "root kernel (X T)");
      if (last) break;
      CANZ_HIP(CANZ_KERNEL_SH_ROOT, (launch_gemm<SE_PLAIN, true>(prod(tt, tt, t2), nb, none, s, o, st)), "root kernel (T T)");
      CANZ_HIP(CANZ_KERNEL_SH_ROOT, (launch_gemm<SE_PLAIN, true>(prod(t2, t2, t4), nb, none, s, o, st)), "root kernel (T2 T2)");
      ShGemm r = prod(t4, m[cur], m[cur ^ 1]);
      r.c2 = tt;
      CANZ_HIP(CANZ_KERNEL_SH_ROOT, (launch_gemm<SE_MT, true>(r, nb, none, s, o, st)), "root kernel (T4 M)");
      cur ^= 1;
    }
    return CANZ_OK;
  };
  float *lroot = ws + c.lroot, *rroot = ws + c.rroot;
  if (int rc = one_side(g.left, g.rows, rp, cp, gs, lroot)) return rc;
  if (int rc = one_side(g.right, g.cols, cp, rp, gt, rroot)) return rc;

  // O = (L^(-1/4) G) R^(-1/4): P = L root, Q = G^T gives rows x cols; then P = that, Q = R root
  ShGemm a1{};
  a1.M = rp, a1.N = cp, a1.K = rp, a1.ldp = rp, a1.ldq = rp, a1.sp = rp * rp, a1.sq = rp * cp;
  a1.P = lroot, a1.Q = gt, a1.c = tmp;
  CANZ_HIP(CANZ_KERNEL_SH_APPLY, (launch_gemm<SE_PLAIN, false>(a1, nb, none, s, o, st)), "preconditioning kernel (left)");
  ShGemm a2{};
  a2.M = rp, a2.N = cp, a2.K = cp, a2.ldp = cp, a2.ldq = cp, a2.sp = rp * cp, a2.sq = cp * cp;
  a2.P = tmp, a2.Q = rroot;
  CANZ_HIP(CANZ_KERNEL_SH_APPLY, (launch_gemm<SE_OUT, false>(a2, nb, none, s, o, st)), "preconditioning kernel (right)");
  return CANZ_OK;
}

}  // namespace
}  // namespace canz

extern "C" int canz_shampoo_workspace_bytes(const canz_shampoo_group* g, int32_t n_groups, const canz_shampoo_hparams* hp,
                                            size_t* bytes_out) {
  using namespace canz;
  if (!bytes_out) return fail(CANZ_EINVAL, "null bytes_out");
  if (n_groups < 0 || (n_groups > 0 && !g)) return fail(CANZ_EINVAL, "bad group array");
  if (int rc = check_hparams(hp)) return rc;
  size_t need = ALIGN;
  for (int i = 0; i < n_groups; ++i) {
    if (int rc = check_group(g[i], i, false, hp->out_mode)) return rc;
    if (g[i].n_mats == 0) continue;
    need = std::max(need, carve(g[i].rows, g[i].cols, std::min(g[i].n_mats, batch_cap(g[i]))).total_bytes);
  }
  *bytes_out = need;
  return CANZ_OK;
}

extern "C" int canz_shampoo_step(const canz_shampoo_group* g, int32_t n_groups, const canz_shampoo_hparams* hp,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace canz;
  size_t need = 0;
  if (int rc = canz_shampoo_workspace_bytes(g, n_groups, hp, &need)) return rc;
  bool any = false;
  for (int i = 0; i < n_groups; ++i) {
    if (int rc = check_group(g[i], i, true, hp->out_mode)) return rc;
    any = any || g[i].n_mats > 0;
  }
  if (!any) return CANZ_OK;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (ALIGN - 1)))
    return fail(CANZ_EWORKSPACE, "workspace null or not 256-byte aligned");
  if (workspace_bytes < need)
    return fail(CANZ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (int i = 0; i < n_groups; ++i) {
    const int cap = batch_cap(g[i]);
    for (int first = 0; first < g[i].n_mats; first += cap)
      if (int rc = run_batch(g[i], first, std::min(cap, g[i].n_mats - first), *hp, static_cast<float*>(workspace), st)) return rc;
  }
  return CANZ_OK;
}
