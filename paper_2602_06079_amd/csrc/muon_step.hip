// canz_muon_step / canz_muon_workspace_bytes: host side of the per-rank Muon step
// (Delta W = Muon_step(G, States), Sec. 4.1 stage (2); zero-communication owner update,
// Sec. 3.3 stage (2)).  Validates the groups, carves the caller's workspace and enqueues
// the kernels of each micro-group on the caller's stream:
//   momentum (+ TP gather, cast, norm partials) -> norm scale ->
//   ns_steps x { Gram, polynomial, update }  with the last update writing the caller's
//   buffers (+ TP scatter).  Nothing here allocates, copies to the device or synchronises.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <mutex>
#include <vector>

#include "canz.h"
#include "canz_internal.h"
#include "kernels.h"

namespace canz {

// ---- optional per-kernel timing (canz_profile_*): a pool of event pairs recorded around
// each launch on the step's own stream.  Process-wide state behind a mutex; while profiling is
// off a launch only reads one atomic flag.  Steps recorded from several threads at once would
// interleave their launches in one pool: the timing is meant for one benchmark thread.
namespace {
struct Profiler {
  std::atomic<bool> on{false};
  std::mutex lock;
  std::vector<hipEvent_t> ev;   // 2 per launch
  std::vector<int> kind;        // kind of each recorded launch
  size_t used = 0;              // launches recorded
};
Profiler g_prof;
}  // namespace

void prof_mark(hipStream_t st, int kind, bool begin) {
  if (!g_prof.on.load(std::memory_order_relaxed)) return;
  std::lock_guard<std::mutex> hold(g_prof.lock);
  if (g_prof.used * 2 + 1 >= g_prof.ev.size()) return;
  if (begin) {
    (void)hipEventRecord(g_prof.ev[g_prof.used * 2], st);
  } else {
    (void)hipEventRecord(g_prof.ev[g_prof.used * 2 + 1], st);
    g_prof.kind[g_prof.used] = kind;
    ++g_prof.used;
  }
}

}  // namespace canz

namespace canz {
namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline int64_t pad_up(int64_t x) { return (x + PAD - 1) / PAD * PAD; }

struct Carve {   // byte offsets of one launch batch's arrays, relative to its own base
  size_t xw, xt0, xt1, a, b, partial, scale, scale2, total;
};

Shape make_shape(const canz_group& g) {
  Shape s{};
  s.rows = g.rows, s.cols = g.cols;
  s.m = std::min(g.rows, g.cols), s.n = std::max(g.rows, g.cols);
  s.mp = pad_up(s.m), s.np = pad_up(s.n);
  s.tall = g.rows > g.cols;
  s.tp = g.tp;
  s.wfrag = g.cols / g.tp;
  return s;
}

Carve carve(const Shape& s, int nb, int precision) {
  const size_t esz = precision == CANZ_PREC_BF16 ? 2 : 4;
  const size_t x_bytes = align_up(static_cast<size_t>(nb) * s.mp * s.np * esz);
  const size_t a_bytes = align_up(static_cast<size_t>(nb) * s.mp * s.mp * esz);
  Carve c{};
  size_t off = 0;
  c.xw = off, off += x_bytes;
  c.xt0 = off, off += x_bytes;
  c.xt1 = off, off += x_bytes;
  c.a = off, off += a_bytes;
  c.b = off, off += a_bytes;
  c.partial = off, off += align_up(static_cast<size_t>(nb) * momentum_tiles(s) * sizeof(float));
  c.scale = off, off += align_up(nb * sizeof(float));
  c.scale2 = off, off += align_up(nb * sizeof(float));
  c.total = off;
  return c;
}

// scratch of the k-split, shared by all launches of a call (bf16 mode only)
size_t split_bytes(int precision) {
  return precision == CANZ_PREC_BF16 ? align_up(SPLIT_MAX_BLOCKS * SPLIT_BLOCK_BYTES) : 0;
}

int check_hparams(const canz_muon_hparams* hp) {
  if (!hp) return fail(CANZ_EINVAL, "null hparams");
  if (hp->ns_steps < 0) return fail(CANZ_EINVAL, "ns_steps must be >= 0");
  if (hp->scale_mode < CANZ_SCALE_NONE || hp->scale_mode > CANZ_SCALE_RMS)
    return fail(CANZ_EUNSUPPORTED, "unknown scale_mode %d", hp->scale_mode);
  if (hp->precision != CANZ_PREC_BF16 && hp->precision != CANZ_PREC_F32)
    return fail(CANZ_EUNSUPPORTED, "unknown precision %d", hp->precision);
  if (hp->out_mode != CANZ_OUT_PARAM && hp->out_mode != CANZ_OUT_DELTA)
    return fail(CANZ_EUNSUPPORTED, "unknown out_mode %d", hp->out_mode);
  return CANZ_OK;
}

int check_group(const canz_group& g, int idx, bool need_ptrs, int out_mode) {
  if (g.n_mats < 0) return fail(CANZ_EINVAL, "group %d: n_mats < 0", idx);
  if (g.rows < 1 || g.cols < 1) return fail(CANZ_EINVAL, "group %d: empty shape", idx);
  // 65535 grid rows of 64-row tiles in the element-wise kernels
  constexpr int64_t MAX_EXTENT = 65535 * 64;
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
  if (!g.grad || !g.mom || !g.out) return fail(CANZ_EINVAL, "group %d: null pointer table", idx);
  const int n_out = out_mode == CANZ_OUT_DELTA ? g.n_mats * g.tp : g.n_mats;
  auto bad = [](const void* p) { return p == nullptr || (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
  for (int i = 0; i < g.n_mats * g.tp; ++i)
    if (bad(g.grad[i])) return fail(CANZ_EINVAL, "group %d: grad[%d] null or not 16-byte aligned", idx, i);
  for (int i = 0; i < g.n_mats; ++i)
    if (bad(g.mom[i])) return fail(CANZ_EINVAL, "group %d: mom[%d] null or not 16-byte aligned", idx, i);
  for (int i = 0; i < n_out; ++i)
    if (bad(g.out[i])) return fail(CANZ_EINVAL, "group %d: out[%d] null or not 16-byte aligned", idx, i);
  return CANZ_OK;
}

double update_scale(const canz_group& g, int mode) {
  if (mode == CANZ_SCALE_ASPECT) return std::sqrt(std::max(1.0, static_cast<double>(g.rows) / static_cast<double>(g.cols)));
  if (mode == CANZ_SCALE_RMS) return 0.2 * std::sqrt(static_cast<double>(std::max(g.rows, g.cols)));
  return 1.0;
}

// Launch batches: consecutive matrices of the call that share dtypes and shape - up to a
// transpose, since the iteration runs on the wide orientation of either - are batched
// together, up to batch_cap() per launch, across micro-group boundaries (a matrix's result
// does not depend on its batch, and small matrices need the larger batch to fill the chip).
bool same_kind(const canz_group& a, const canz_group& b) {
  return std::min(a.rows, a.cols) == std::min(b.rows, b.cols) && std::max(a.rows, a.cols) == std::max(b.rows, b.cols) &&
         a.tp == b.tp && a.grad_dtype == b.grad_dtype && a.out_dtype == b.out_dtype;
}

// matrices of this kind per launch: bounded by the pointer tables (kernel arguments) and by
// the workspace a launch needs.  Small matrices go many to a launch, so that the persistent
// GEMM grids have whole rounds of tiles and the launch count stays low.
int batch_cap(const canz_group& g) {
  const Shape s = make_shape(g);
  const int64_t by_ptrs = MAX_PTRS / g.tp;
  const int64_t by_elems = std::max<int64_t>(1, MAX_BATCH_ELEMS / (s.mp * s.np));
  return static_cast<int>(std::min(by_ptrs, by_elems));
}

// calls fn(proto group, first group index, first matrix in it, count) for every launch batch
template <typename F>
int for_each_batch(const canz_group* g, int n_groups, F&& fn) {
  int proto = -1, count = 0, start_group = 0, start_mat = 0;
  for (int i = 0; i < n_groups; ++i) {
    for (int m = 0; m < g[i].n_mats; ++m) {
      if (count > 0 && (count == batch_cap(g[proto]) || !same_kind(g[proto], g[i]))) {
        if (int rc = fn(g[proto], start_group, start_mat, count)) return rc;
        count = 0;
      }
      if (count == 0) proto = i, start_group = i, start_mat = m;
      ++count;
    }
  }
  if (count > 0) return fn(g[proto], start_group, start_mat, count);
  return CANZ_OK;
}

// The matrices of one orientation inside a launch batch.
struct Part {
  const canz_group* proto = nullptr;
  std::vector<const void*> grad;
  std::vector<void*> mom, out;
  int n() const { return static_cast<int>(mom.size()); }
};

// One launch batch: part[0] holds its wide (rows <= cols) matrices, part[1] the tall ones of
// the transposed shape.  They occupy consecutive slots of the batch's workspace arrays, the
// wide ones first; the kernels that touch the caller's buffers (momentum, last product,
// apply) run once per part.
struct Batch {
  Part part[2];
  Shape s0{};     // shape of any member: the padded extents are those of the whole batch
  int nb = 0;
  int64_t update_tiles() const { return (s0.mp / PAD) * (s0.np / PAD) * nb; }
};

// Collects the launch batches of a call (pointers only when `with_ptrs`).
int collect_batches(const canz_group* g, int n_groups, int out_mode, bool with_ptrs, std::vector<Batch>& out) {
  return for_each_batch(g, n_groups, [&](const canz_group& proto, int gi, int mi, int count) {
    out.emplace_back();
    Batch& bt = out.back();
    bt.s0 = make_shape(proto);
    bt.nb = count;
    for (int left = count; left > 0; ++gi, mi = 0) {
      const canz_group& src = g[gi];
      const int take = std::min(left, src.n_mats - mi);
      if (take <= 0) continue;
      Part& p = bt.part[src.rows > src.cols ? 1 : 0];
      if (!p.proto) p.proto = &src;
      const int per_out = out_mode == CANZ_OUT_DELTA ? src.tp : 1;
      for (int m = mi; m < mi + take; ++m) {
        if (with_ptrs) {
          for (int f = 0; f < src.tp; ++f) p.grad.push_back(src.grad[m * src.tp + f]);
          for (int f = 0; f < per_out; ++f) p.out.push_back(src.out[m * per_out + f]);
        }
        p.mom.push_back(with_ptrs ? src.mom[m] : nullptr);
      }
      left -= take;
    }
    return CANZ_OK;
  });
}

// Launch batches that are too small to fill the chip on their own for long (fewer than 8
// rounds of update tiles on 256 CUs) are run together, up to MAX_KINDS of them: their Gram,
// polynomial and update products then share launches.  first[i] .. first[i + 1] are the
// batches of run i.  Only in bf16 mode; the fp32 verification path keeps one batch per run.
constexpr int64_t SMALL_BATCH_TILES = 8 * 256;
std::vector<int> group_runs(const std::vector<Batch>& batches, int precision) {
  std::vector<int> first;
  const int n = static_cast<int>(batches.size());
  for (int i = 0; i < n;) {
    first.push_back(i);
    int j = i + 1;
    if (precision == CANZ_PREC_BF16 && batches[i].update_tiles() < SMALL_BATCH_TILES) {
      int64_t elems = batches[i].s0.mp * batches[i].s0.np * batches[i].nb;
      while (j < n && j - i < MAX_KINDS && batches[j].update_tiles() < SMALL_BATCH_TILES) {
        const int64_t more = batches[j].s0.mp * batches[j].s0.np * batches[j].nb;
        if (elems + more > MAX_BATCH_ELEMS) break;
        elems += more;
        ++j;
      }
    }
    i = j;
  }
  first.push_back(n);
  return first;
}

size_t run_bytes(const std::vector<Batch>& batches, int lo, int hi, int precision) {
  size_t total = 0;
  for (int k = lo; k < hi; ++k) total += carve(batches[k].s0, batches[k].nb, precision).total;
  return total + split_bytes(precision);
}

// One run: the batches lo .. hi-1 side by side in the workspace, then the split scratch.
template <typename T>
int run_batches(const std::vector<Batch>& batches, int lo, int hi, const canz_muon_hparams& hp, char* ws,
                hipStream_t st) {
  constexpr bool is_bf16 = sizeof(T) == 2;
  const int nk = hi - lo;
  struct Kind {
    T *xw, *xt[2], *a, *bm;
    float *partial, *scale, *scale2;
    int64_t x_elems, a_elems;
    int tiles, nb;
    Shape s0, shape[2];
    OutSpec out[2];
    int first[2];
    GemmDims gram, poly, upd;
  };
  Kind kind[MAX_KINDS];
  size_t base = 0;
  for (int k = 0; k < nk; ++k) {
    const Batch& bt = batches[lo + k];
    Kind& kd = kind[k];
    const Carve c = carve(bt.s0, bt.nb, hp.precision);
    char* w = ws + base;
    kd.xw = reinterpret_cast<T*>(w + c.xw);
    kd.xt[0] = reinterpret_cast<T*>(w + c.xt0), kd.xt[1] = reinterpret_cast<T*>(w + c.xt1);
    kd.a = reinterpret_cast<T*>(w + c.a), kd.bm = reinterpret_cast<T*>(w + c.b);
    kd.partial = reinterpret_cast<float*>(w + c.partial);
    kd.scale = reinterpret_cast<float*>(w + c.scale), kd.scale2 = reinterpret_cast<float*>(w + c.scale2);
    base += c.total;
    const Shape& s = kd.s0 = bt.s0;
    kd.nb = bt.nb;
    kd.x_elems = s.mp * s.np, kd.a_elems = s.mp * s.mp;
    kd.tiles = momentum_tiles(s);
    kd.first[0] = 0, kd.first[1] = bt.part[0].n();
    kd.gram = GemmDims{s.mp, s.mp, s.np, s.np, s.np, kd.x_elems, kd.x_elems, bt.nb};
    kd.poly = GemmDims{s.mp, s.mp, s.mp, s.mp, s.mp, kd.a_elems, kd.a_elems, bt.nb};
    kd.upd = GemmDims{s.mp, s.np, s.mp, s.mp, s.mp, kd.a_elems, kd.x_elems, bt.nb};
  }
  const SplitWs split{reinterpret_cast<float*>(ws + base), SPLIT_MAX_BLOCKS};

  // momentum (+ gather, cast, both orientations, tile sums of U^2) per part, norm per batch
  for (int k = 0; k < nk; ++k) {
    const Batch& bt = batches[lo + k];
    Kind& kd = kind[k];
    for (int h = 0; h < 2; ++h) {
      const Part& part = bt.part[h];
      const int n = part.n();
      if (n == 0) continue;
      const canz_group& g = *part.proto;
      kd.shape[h] = make_shape(g);
      PtrTable grad{}, mom{};
      OutSpec& o = kd.out[h];
      o = OutSpec{};
      const int n_out = hp.out_mode == CANZ_OUT_DELTA ? n * g.tp : n;
      for (int i = 0; i < n * g.tp; ++i) grad.p[i] = const_cast<void*>(part.grad[i]);
      for (int i = 0; i < n; ++i) mom.p[i] = part.mom[i];
      for (int i = 0; i < n_out; ++i) o.out.p[i] = part.out[i];
      o.out_dtype = g.out_dtype;
      o.out_mode = hp.out_mode;
      o.decay = static_cast<float>(1.0 - static_cast<double>(hp.lr) * static_cast<double>(hp.weight_decay));
      o.neg_lr_scale = static_cast<float>(-static_cast<double>(hp.lr) * update_scale(g, hp.scale_mode));
      const int f = kd.first[h];
      CANZ_HIP(CANZ_KERNEL_MOMENTUM,
               launch_momentum<T>(kd.shape[h], n, grad, g.grad_dtype, mom, hp.beta, hp.nesterov, kd.xw + f * kd.x_elems,
                                  kd.xt[0] + f * kd.x_elems, kd.partial + static_cast<int64_t>(f) * kd.tiles, st),
               "momentum kernel");
    }
    CANZ_HIP(CANZ_KERNEL_NORM, launch_norm_scale(kd.nb, kd.tiles, kd.partial, hp.eps, kd.scale, kd.scale2, st),
             "norm kernel");
  }

  if (hp.ns_steps == 0) {
    for (int k = 0; k < nk; ++k)
      for (int h = 0; h < 2; ++h) {
        const int n = batches[lo + k].part[h].n();
        if (n == 0) continue;
        const Kind& kd = kind[k];
        const Shape& s = kd.shape[h];
        const T* straight = (s.tall ? kd.xt[0] : kd.xw) + kd.first[h] * kd.x_elems;
        const int64_t ld = s.tall ? s.mp : s.np;
        CANZ_HIP(CANZ_KERNEL_APPLY,
                 launch_apply<T>(s, n, straight, ld, kd.x_elems, kd.scale + kd.first[h], kd.out[h], st), "apply kernel");
      }
    return CANZ_OK;
  }

  const bool together = is_bf16 && nk > 1;   // shared launches for Gram, polynomial and update
  int cur = 0;
  for (int it = 0; it < hp.ns_steps; ++it) {
    const bool first_it = it == 0, last = it + 1 == hp.ns_steps;
    if (together) {
      GemmBatch gb{};
      gb.n = nk;
      for (int k = 0; k < nk; ++k)
        gb.pr[k] = GemmProblem{kind[k].gram, kind[k].xw, kind[k].xw, kind[k].a, nullptr, nullptr,
                               first_it ? kind[k].scale2 : nullptr};
      CANZ_HIP(CANZ_KERNEL_GRAM, launch_gram_bf16_multi(gb, st), "gram kernel");
      for (int k = 0; k < nk; ++k)
        gb.pr[k] = GemmProblem{kind[k].poly, kind[k].a, kind[k].a, kind[k].bm, nullptr, kind[k].a, nullptr};
      CANZ_HIP(CANZ_KERNEL_POLY, launch_poly_bf16_multi(gb, hp.a, hp.b, hp.c, st), "poly kernel");
      if (!last) {
        for (int k = 0; k < nk; ++k)
          gb.pr[k] = GemmProblem{kind[k].upd, kind[k].bm, kind[k].xt[cur], kind[k].xw, kind[k].xt[cur ^ 1], nullptr,
                                 first_it ? kind[k].scale : nullptr};
        CANZ_HIP(CANZ_KERNEL_UPDATE, launch_update_bf16_multi(gb, st), "update kernel");
      }
    }
    for (int k = 0; k < nk; ++k) {
      const Kind& kd = kind[k];
      const float* sc1 = first_it ? kd.scale : nullptr;
      const float* sc2 = first_it ? kd.scale2 : nullptr;
      if (!together) {
        if (is_bf16) {
          CANZ_HIP(CANZ_KERNEL_GRAM, launch_gram_bf16(kd.gram, kd.xw, kd.a, sc2, split, st), "gram kernel");
          CANZ_HIP(CANZ_KERNEL_POLY, launch_poly_bf16(kd.poly, kd.a, kd.bm, hp.a, hp.b, hp.c, split, st), "poly kernel");
          if (!last)
            CANZ_HIP(CANZ_KERNEL_UPDATE,
                     launch_update_bf16(kd.upd, kd.bm, kd.xt[cur], kd.xw, kd.xt[cur ^ 1], sc1, split, st), "update kernel");
        } else {
          CANZ_HIP(CANZ_KERNEL_GRAM, launch_gram_f32(kd.gram, kd.xw, kd.a, sc2, st), "gram kernel");
          CANZ_HIP(CANZ_KERNEL_POLY, launch_poly_f32(kd.poly, kd.a, kd.bm, hp.a, hp.b, hp.c, st), "poly kernel");
          if (!last)
            CANZ_HIP(CANZ_KERNEL_UPDATE, launch_update_f32(kd.upd, kd.bm, kd.xt[cur], kd.xw, kd.xt[cur ^ 1], sc1, st),
                     "update kernel");
        }
      }
      if (!last) continue;
      // last product, written in the caller's orientation: for the tall part the roles of
      // the polynomial and of X swap, so that C comes out as rows x cols
      for (int h = 0; h < 2; ++h) {
        const int n = batches[lo + k].part[h].n();
        if (n == 0) continue;
        const Shape& s = kd.s0;
        const T* bk = kd.bm + kd.first[h] * kd.a_elems;
        const T* xk = kd.xt[cur] + kd.first[h] * kd.x_elems;
        const float* sk = sc1 ? sc1 + kd.first[h] : nullptr;
        const bool tall = kd.shape[h].tall;
        GemmDims fin = tall ? GemmDims{s.np, s.mp, s.mp, s.mp, s.mp, kd.x_elems, kd.a_elems, n} : kd.upd;
        fin.nb = n;
        const void* P = tall ? static_cast<const void*>(xk) : static_cast<const void*>(bk);
        const void* Q = tall ? static_cast<const void*>(bk) : static_cast<const void*>(xk);
        if (is_bf16)
          CANZ_HIP(CANZ_KERNEL_FINAL, launch_final_bf16(fin, P, Q, sk, split, kd.shape[h], kd.out[h], st), "final kernel");
        else
          CANZ_HIP(CANZ_KERNEL_FINAL, launch_final_f32(fin, P, Q, sk, kd.shape[h], kd.out[h], st), "final kernel");
      }
    }
    cur ^= 1;
  }
  return CANZ_OK;
}

}  // namespace
}  // namespace canz

extern "C" int canz_muon_workspace_bytes(const canz_group* g, int32_t n_groups, const canz_muon_hparams* hp,
                                         size_t* bytes_out) {
  using namespace canz;
  if (!bytes_out) return fail(CANZ_EINVAL, "null bytes_out");
  if (n_groups < 0 || (n_groups > 0 && !g)) return fail(CANZ_EINVAL, "bad group array");
  if (int rc = check_hparams(hp)) return rc;
  size_t need = ALIGN;
  for (int i = 0; i < n_groups; ++i)
    if (int rc = check_group(g[i], i, false, hp->out_mode)) return rc;
  std::vector<Batch> batches;
  if (int rc = collect_batches(g, n_groups, hp->out_mode, false, batches)) return rc;
  const std::vector<int> first = group_runs(batches, hp->precision);
  for (size_t r = 0; r + 1 < first.size(); ++r)
    need = std::max(need, run_bytes(batches, first[r], first[r + 1], hp->precision));
  *bytes_out = need;
  return CANZ_OK;
}

namespace canz {
namespace {

// Validates the call and enqueues every run of launch batches on `st`, using `workspace`.
int muon_step_on(const canz_group* g, int32_t n_groups, const canz_muon_hparams* hp, void* workspace,
                 size_t workspace_bytes, hipStream_t st) {
  if (n_groups < 0 || (n_groups > 0 && !g)) return fail(CANZ_EINVAL, "bad group array");
  if (int rc = check_hparams(hp)) return rc;
  size_t need = 0;
  if (int rc = canz_muon_workspace_bytes(g, n_groups, hp, &need)) return rc;
  for (int i = 0; i < n_groups; ++i)
    if (int rc = check_group(g[i], i, true, hp->out_mode)) return rc;
  bool any = false;
  for (int i = 0; i < n_groups; ++i) any = any || g[i].n_mats > 0;
  if (!any) return CANZ_OK;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (ALIGN - 1)))
    return fail(CANZ_EWORKSPACE, "workspace null or not 256-byte aligned");
  if (workspace_bytes < need)
    return fail(CANZ_EWORKSPACE, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);

  char* ws = static_cast<char*>(workspace);
  std::vector<Batch> batches;
  if (int rc = collect_batches(g, n_groups, hp->out_mode, true, batches)) return rc;
  const std::vector<int> first = group_runs(batches, hp->precision);
  for (size_t r = 0; r + 1 < first.size(); ++r) {
    const int rc = hp->precision == CANZ_PREC_BF16 ? run_batches<__bf16>(batches, first[r], first[r + 1], *hp, ws, st)
                                                   : run_batches<float>(batches, first[r], first[r + 1], *hp, ws, st);
    if (rc) return rc;
  }
  return CANZ_OK;
}

// ---- workspace that lives in the library (canz_muon_step_static).  The array sits in the
// code object of this file; every device that loads the library holds its own copy at its own
// address until the process ends.  Host code never uses the array's name as an address: the
// device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[CANZ_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the current device (nullptr + error message on failure).
void* scratch_address() {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
    fail(CANZ_EHIP, "hipGetDevice: %s (device %d)", hipGetErrorString(err), dev);
    return nullptr;
  }
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !ptr) {
      fail(CANZ_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(err));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace
}  // namespace canz

extern "C" int canz_muon_step(const canz_group* g, int32_t n_groups, const canz_muon_hparams* hp, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  return canz::muon_step_on(g, n_groups, hp, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

extern "C" int canz_muon_step_static(const canz_group* g, int32_t n_groups, const canz_muon_hparams* hp,
                                     void* hip_stream) {
  using namespace canz;
  if (n_groups < 0 || (n_groups > 0 && !g)) return fail(CANZ_EINVAL, "bad group array");
  size_t need = 0;
  if (int rc = canz_muon_workspace_bytes(g, n_groups, hp, &need)) return rc;
  if (need > CANZ_STATIC_WORKSPACE_BYTES)
    return fail(CANZ_EWORKSPACE, "step needs %zu bytes of scratch, the built-in workspace holds %zu", need,
                static_cast<size_t>(CANZ_STATIC_WORKSPACE_BYTES));
  void* ptr = scratch_address();
  if (!ptr) return CANZ_EHIP;
  return muon_step_on(g, n_groups, hp, ptr, CANZ_STATIC_WORKSPACE_BYTES, static_cast<hipStream_t>(hip_stream));
}

extern "C" int canz_profile_enable(int32_t max_launches) {
  using namespace canz;
  if (max_launches < 1) return fail(CANZ_EINVAL, "max_launches must be >= 1");
  std::lock_guard<std::mutex> hold(g_prof.lock);
  while (g_prof.ev.size() < static_cast<size_t>(max_launches) * 2) {
    hipEvent_t e;
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) return fail(CANZ_EHIP, "hipEventCreate: %s", hipGetErrorString(err));
    g_prof.ev.push_back(e);
  }
  g_prof.kind.assign(g_prof.ev.size() / 2, 0);
  g_prof.used = 0;
  g_prof.on.store(true);
  return CANZ_OK;
}

extern "C" int canz_profile_collect(double* ms_out, int64_t* launches_out) {
  using namespace canz;
  if (!ms_out || !launches_out) return fail(CANZ_EINVAL, "null output pointer");
  for (int k = 0; k < CANZ_KERNEL_KINDS; ++k) ms_out[k] = 0.0, launches_out[k] = 0;
  std::lock_guard<std::mutex> hold(g_prof.lock);
  for (size_t i = 0; i < g_prof.used; ++i) {
    hipError_t err = hipEventSynchronize(g_prof.ev[2 * i + 1]);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]);
    if (err != hipSuccess) return fail(CANZ_EHIP, "profile event: %s", hipGetErrorString(err));
    ms_out[g_prof.kind[i]] += ms;
    launches_out[g_prof.kind[i]] += 1;
  }
  g_prof.used = 0;
  return CANZ_OK;
}

extern "C" int canz_profile_disable(void) {
  std::lock_guard<std::mutex> hold(canz::g_prof.lock);
  canz::g_prof.on.store(false);
  canz::g_prof.used = 0;
  return CANZ_OK;
}
