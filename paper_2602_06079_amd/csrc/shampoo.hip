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
// same accumulators, which halves their work and keeps the iterates symmetric (bit for bit across
// tiles; inside a diagonal tile the two halves are rounded separately and agree to an ulp or two).
//
// Inverse fourth root (coupled Newton iteration for the inverse p-th root, p = 4): from
// M = z A, X = z^(1/4) I with z = 5 / (2 b), b an upper bound of the largest eigenvalue (see k_sh_init),
// repeat T = (5 I - M) / 4, X <- X T,
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
#include "f32_mfma_gemm.h"
#include "kernels.h"

namespace canz {
namespace {

using namespace f32mfma;

constexpr int NPART = 64;        // partial sums per matrix of the Frobenius norm
constexpr int64_t MAX_EXTENT = 32768;
constexpr size_t BATCH_BYTES = size_t(8) << 30;

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

// Start of the root iteration.  The iteration needs M = z A with eigenvalues in (0, 5); the closer the largest
// comes to 5/2 the fewer rounds the smallest needs to grow to 1.  ||A||_F bounds the largest eigenvalue of A,
// but loosely (by sqrt(d) for a flat spectrum: three and a half rounds at d = 3072); ||A'^4||_F^(1/4) with
// A' = A / ||A||_F is a bound too, at most d^(1/8) above it, for two products.
//   k_sh_prescale:  A' = A / ||A||_F
//   k_sh_init:      z' = 5 / (2 ||A'^4||_F^(1/4));  M = z' A';  T = 5/4 I - 1/4 M;  X = (z' / ||A||_F)^(1/4) I
__device__ __forceinline__ double sum_partials(const float* partial, int b) {
  double sum = 0.0;
  for (int i = 0; i < NPART; ++i) sum += static_cast<double>(partial[b * NPART + i]);
  return sum;
}

__global__ __launch_bounds__(NTH) void k_sh_prescale(const float* __restrict__ a, const float* __restrict__ partial,
                                                      int64_t elems, float* __restrict__ m) {
  const int b = blockIdx.y;
  const float nrm = static_cast<float>(sqrt(sum_partials(partial, b)));
  const float inv = nrm > 0.f ? 1.f / nrm : 0.f;
  const int64_t off = static_cast<int64_t>(b) * elems;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * NTH + threadIdx.x; i < elems; i += static_cast<int64_t>(gridDim.x) * NTH)
    m[off + i] = inv * a[off + i];
}

__global__ __launch_bounds__(NTH) void k_sh_init(const float* __restrict__ partial, const float* __restrict__ partial4,
                                                  int64_t dp, float* __restrict__ x, float* __restrict__ m,
                                                  float* __restrict__ tt) {
  const int b = blockIdx.y;
  const float nrm = static_cast<float>(sqrt(sum_partials(partial, b)));
  const float bound = static_cast<float>(pow(sum_partials(partial4, b), 0.125));   // ||A'^4||_F^(1/4) >= lambda_max(A')
  const float z = bound > 0.f ? 2.5f / bound : 1.f;
  const float x0 = nrm > 0.f ? sqrtf(sqrtf(z / nrm)) : 1.f;
  const int64_t elems = dp * dp, off = static_cast<int64_t>(b) * elems;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * NTH + threadIdx.x; i < elems; i += static_cast<int64_t>(gridDim.x) * NTH) {
    const bool diag = (i / dp) == (i % dp);
    const float mv = z * m[off + i];
    m[off + i] = mv;
    tt[off + i] = (diag ? 1.25f : 0.f) - 0.25f * mv;
    x[off + i] = diag ? x0 : 0.f;
  }
}

struct Carve {   // float offsets into the workspace of one launch batch
  size_t gs, gt, tmp, lroot, rroot, a, x[2], m[2], t, t2, t4, partial, partial4, total_bytes;
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
  c.partial4 = take(static_cast<size_t>(nb) * NPART);
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

int check_group(const canz_shampoo_group& g, int idx, bool need_ptrs, int out_mode, bool keep_roots) {
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
  if ((g.lroot == nullptr) != (g.rroot == nullptr)) return fail(CANZ_EINVAL, "group %d: one root table without the other", idx);
  if (keep_roots && !g.lroot) return fail(CANZ_EINVAL, "group %d: keep_roots needs the root tables", idx);
  const int n_out = out_mode == CANZ_OUT_DELTA ? g.n_mats * g.tp : g.n_mats;
  auto bad = [](const void* p) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
  for (int i = 0; i < g.n_mats * g.tp; ++i)
    if (bad(g.grad[i])) return fail(CANZ_EINVAL, "group %d: grad[%d] null or not 16-byte aligned", idx, i);
  for (int i = 0; i < g.n_mats; ++i)
    if (bad(g.left[i]) || bad(g.right[i]) || (g.lroot && (bad(g.lroot[i]) || bad(g.rroot[i]))))
      return fail(CANZ_EINVAL, "group %d: statistic or root %d null or not 16-byte aligned", idx, i);
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
  auto one_side = [&](void* const* stat_tab, void* const* root_tab, int64_t d, int64_t dp, int64_t kp, const float* side,
                      float* root) -> int {
    PtrTable stat{}, kept{};
    for (int i = 0; i < nb; ++i) stat.p[i] = stat_tab[first + i];
    if (root_tab)
      for (int i = 0; i < nb; ++i) kept.p[i] = root_tab[first + i];
    Shape sq{};   // the d x d matrices of this side, for the padded load and the dense store of a kept root
    sq.rows = d, sq.cols = d, sq.tp = 1, sq.wfrag = d;
    const dim3 sq_tiles(static_cast<unsigned>(dp / 64), static_cast<unsigned>(dp / 64), static_cast<unsigned>(nb));
    const int64_t dd = dp * dp;
    float *a = ws + c.a, *x[2] = {ws + c.x[0], ws + c.x[1]}, *m[2] = {ws + c.m[0], ws + c.m[1]};
    float *tt = ws + c.t, *t2 = ws + c.t2, *t4 = ws + c.t4, *partial = ws + c.partial, *partial4 = ws + c.partial4;
    ShGemm q{};
    q.M = dp, q.N = dp, q.K = kp, q.ldp = kp, q.ldq = kp, q.sp = dp * kp, q.sq = dp * kp;
    q.P = side, q.Q = side, q.c = hp.keep_roots ? nullptr : a, q.d = d, q.beta = hp.beta, q.gscale = 1.f, q.eps = hp.eps;
    CANZ_HIP(CANZ_KERNEL_SH_STAT, (launch_gemm<SE_STAT, true>(q, nb, stat, s, o, st)), "statistics kernel");
    if (hp.keep_roots) {   // the caller's root, padded (its transposed image, which equals it, goes to a free buffer)
      prof_mark(st, CANZ_KERNEL_SH_LOAD, true);
      hipLaunchKernelGGL(k_sh_load, sq_tiles, dim3(NTH), 0, st, sq, kept, static_cast<int>(CANZ_DT_F32), dp, dp, root, x[0]);
      prof_mark(st, CANZ_KERNEL_SH_LOAD, false);
      if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "root load: %s", hipGetErrorString(e));
      return CANZ_OK;
    }
    auto prod = [&](const float* P, const float* Q, float* C) {
      ShGemm r{};
      r.M = dp, r.N = dp, r.K = dp, r.ldp = dp, r.ldq = dp, r.sp = dd, r.sq = dd;
      r.P = P, r.Q = Q, r.c = C;
      return r;
    };
    const unsigned init_blocks = static_cast<unsigned>(std::min<int64_t>(4096, (dd + NTH - 1) / NTH));
    prof_mark(st, CANZ_KERNEL_SH_INIT, true);
    hipLaunchKernelGGL(k_sh_sumsq, dim3(NPART, nb), dim3(NTH), 0, st, a, dd, partial);
    hipLaunchKernelGGL(k_sh_prescale, dim3(init_blocks, nb), dim3(NTH), 0, st, a, partial, dd, m[0]);
    prof_mark(st, CANZ_KERNEL_SH_INIT, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "root start: %s", hipGetErrorString(e));
    CANZ_HIP(CANZ_KERNEL_SH_ROOT, (launch_gemm<SE_PLAIN, true>(prod(m[0], m[0], t2), nb, none, s, o, st)), "root start (A A)");
    CANZ_HIP(CANZ_KERNEL_SH_ROOT, (launch_gemm<SE_PLAIN, true>(prod(t2, t2, t4), nb, none, s, o, st)), "root start (A2 A2)");
    prof_mark(st, CANZ_KERNEL_SH_INIT, true);
    hipLaunchKernelGGL(k_sh_sumsq, dim3(NPART, nb), dim3(NTH), 0, st, t4, dd, partial4);
    hipLaunchKernelGGL(k_sh_init, dim3(init_blocks, nb), dim3(NTH), 0, st, partial, partial4, dp, x[0], m[0], tt);
    prof_mark(st, CANZ_KERNEL_SH_INIT, false);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "root start: %s", hipGetErrorString(e));
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
    if (root_tab) {
      prof_mark(st, CANZ_KERNEL_SH_LOAD, true);
      hipLaunchKernelGGL(k_unpad, sq_tiles, dim3(NTH), 0, st, sq, kept, root, dd, dp);
      prof_mark(st, CANZ_KERNEL_SH_LOAD, false);
      if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail(CANZ_EHIP, "root store: %s", hipGetErrorString(e));
    }
    return CANZ_OK;
  };
  float *lroot = ws + c.lroot, *rroot = ws + c.rroot;
  if (int rc = one_side(g.left, g.lroot, g.rows, rp, cp, gs, lroot)) return rc;
  if (int rc = one_side(g.right, g.rroot, g.cols, cp, rp, gt, rroot)) return rc;

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

// Consecutive groups of a call that agree in shape, tp, dtypes and in which tables they pass run as one group: every
// matrix is computed on its own whatever shares its launch, and the products of small matrices fill the chip only
// when many of them share one.
struct MergedGroup {
  canz_shampoo_group g{};
  std::vector<const void*> grad;
  std::vector<void*> tab[5];   // left, right, out, lroot, rroot
};

void tables_of(const canz_shampoo_group& g, void* const* (&out)[5]) {
  out[0] = g.left, out[1] = g.right, out[2] = g.out, out[3] = g.lroot, out[4] = g.rroot;
}

bool mergeable(const canz_shampoo_group& a, const canz_shampoo_group& b) {
  if (a.rows != b.rows || a.cols != b.cols || a.tp != b.tp || a.grad_dtype != b.grad_dtype || a.out_dtype != b.out_dtype) return false;
  if ((a.grad == nullptr) != (b.grad == nullptr)) return false;
  void* const* ta[5];
  void* const* tb[5];
  tables_of(a, ta), tables_of(b, tb);
  for (int k = 0; k < 5; ++k)
    if ((ta[k] == nullptr) != (tb[k] == nullptr)) return false;
  return true;
}

std::vector<MergedGroup> merge_groups(const canz_shampoo_group* g, int n_groups, int out_mode) {
  std::vector<MergedGroup> all;
  for (int i = 0; i < n_groups; ++i) {
    const canz_shampoo_group& x = g[i];
    if (x.n_mats == 0) continue;
    if (all.empty() || !mergeable(all.back().g, x)) {
      all.emplace_back();
      all.back().g = x;
      all.back().g.n_mats = 0;
    }
    MergedGroup& m = all.back();
    void* const* t[5];
    tables_of(x, t);
    const int per_out = out_mode == CANZ_OUT_DELTA ? x.tp : 1;
    if (x.grad) m.grad.insert(m.grad.end(), x.grad, x.grad + static_cast<size_t>(x.n_mats) * x.tp);
    for (int k = 0; k < 5; ++k)
      if (t[k]) m.tab[k].insert(m.tab[k].end(), t[k], t[k] + static_cast<size_t>(x.n_mats) * (k == 2 ? per_out : 1));
    m.g.n_mats += x.n_mats;
  }
  for (MergedGroup& m : all) {   // the tables now stand still: point the group at them
    canz_shampoo_group& x = m.g;
    if (x.grad) x.grad = m.grad.data();
    if (x.left) x.left = m.tab[0].data();
    if (x.right) x.right = m.tab[1].data();
    if (x.out) x.out = m.tab[2].data();
    if (x.lroot) x.lroot = m.tab[3].data();
    if (x.rroot) x.rroot = m.tab[4].data();
  }
  return all;
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
  for (int i = 0; i < n_groups; ++i)
    if (int rc = check_group(g[i], i, false, hp->out_mode, hp->keep_roots != 0)) return rc;
  for (const MergedGroup& m : merge_groups(g, n_groups, hp->out_mode))
    need = std::max(need, carve(m.g.rows, m.g.cols, std::min(m.g.n_mats, batch_cap(m.g))).total_bytes);
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
    if (int rc = check_group(g[i], i, true, hp->out_mode, hp->keep_roots != 0)) return rc;
    any = any || g[i].n_mats > 0;
  }
  if (!any) return CANZ_OK;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (ALIGN - 1)))
    return fail(CANZ_EWORKSPACE, "workspace null or not 256-byte aligned");
  if (workspace_bytes < need)
    return fail(CANZ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  for (const MergedGroup& m : merge_groups(g, n_groups, hp->out_mode)) {
    const int cap = batch_cap(m.g);
    for (int first = 0; first < m.g.n_mats; first += cap)
      if (int rc = run_batch(m.g, first, std::min(cap, m.g.n_mats - first), *hp, static_cast<float*>(workspace), st)) return rc;
  }
  return CANZ_OK;
}
