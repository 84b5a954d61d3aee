// Launchers of the device kernels behind canz_muon_step (internal, not part of the ABI).
//
// Working layout of one sub-batch of nb same-shape matrices (m = min(rows, cols),
// n = max(rows, cols), mp / np = m / n rounded up to PAD):
//   XW  [nb][mp][np]  the iterate X in its wide orientation, row-major
//   XT  [nb][np][mp]  the same values transposed (two buffers, ping-pong)
//   A,B [nb][mp][mp]  Gram matrix and the polynomial aI + bA + cAA
// Padding rows / columns hold zeros; zeros stay zero under the iteration, so the GEMM
// kernels run on the padded extents without bounds checks.  Both orientations are kept
// because every product then contracts over a contiguous index of both operands
// (C[i][j] = sum_k P[i][k] Q[j][k]), which is the operand form of the bf16 MFMA.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "canz_internal.h"

namespace canz {

constexpr int PAD = 256;           // working extents are multiples of this
constexpr int MAX_TP = 8;
constexpr int MAX_PTRS = 128;      // buffers per pointer table: a launch takes up to MAX_PTRS / tp matrices
// ... and no more than this many padded elements, which bounds the workspace of a launch
constexpr int64_t MAX_BATCH_ELEMS = int64_t(1) << 30;
constexpr int EW_TILE = 64;        // elementwise kernels work on 64 x 64 tiles

// Pointer tables travel as kernel arguments, so nothing is copied to the device.
struct PtrTable {
  void* p[MAX_PTRS];
};

struct Shape {
  int64_t rows, cols;   // caller's matrix
  int64_t m, n;         // min / max extent
  int64_t mp, np;       // padded
  int tall;             // rows > cols: the wide orientation is the transpose
  int tp;               // column fragments of grad / delta
  int64_t wfrag;        // cols / tp
};

// ---- per-kernel timing (canz_profile_*) --------------------------------------------
// Records an event on `st` before (begin) or after a launch of the given CANZ_KERNEL_* kind;
// does nothing while profiling is off.
void prof_mark(hipStream_t st, int kind, bool begin);

#define CANZ_HIP(kind, expr, what)                                                      \
  do {                                                                                  \
    ::canz::prof_mark(st, kind, true);                                                  \
    hipError_t err__ = (expr);                                                          \
    ::canz::prof_mark(st, kind, false);                                                 \
    if (err__ != hipSuccess) return ::canz::fail(CANZ_EHIP, "%s: %s", what, hipGetErrorString(err__)); \
  } while (0)

// ---- elementwise -----------------------------------------------------------------
// M <- beta M + G; U = M or G + beta M; U written (type T = bf16 or float) to XW and XT
// (padding zero-filled); per-tile sums of U^2 to partial[b][tile].
template <typename T>
hipError_t launch_momentum(const Shape& s, int nb, const PtrTable& grad, int grad_dtype,
                           const PtrTable& mom, float beta, int nesterov, T* xw, T* xt,
                           float* partial, hipStream_t st);
int momentum_tiles(const Shape& s);  // partial sums per matrix

// scale[b] = 1 / (sqrt(sum partial[b][*]) + eps), scale2[b] = scale[b]^2
hipError_t launch_norm_scale(int nb, int n_partial, const float* partial, float eps, float* scale,
                             float* scale2, hipStream_t st);

struct OutSpec {
  PtrTable out;
  int out_dtype;      // CANZ_DT_*
  int out_mode;       // CANZ_OUT_*
  float decay;        // 1 - lr * weight_decay
  float neg_lr_scale; // -lr * scale
};

// ns_steps == 0: O = scale[b] * U taken from the orientation that matches the caller's.
template <typename T>
hipError_t launch_apply(const Shape& s, int nb, const T* x_straight, int64_t ld, int64_t batch_stride,
                        const float* scale, const OutSpec& o, hipStream_t st);

// ---- bf16 MFMA GEMMs -------------------------------------------------------------
struct GemmDims {
  int64_t M, N, K;          // multiples of PAD
  int64_t ldp, ldq;         // row strides of P [M][K] and Q [N][K]
  int64_t sp, sq;           // batch strides
  int nb;
};
// Scratch for the k-split of left-over tiles: fp32 accumulators of up to max_blocks blocks
// (256 KiB each), written by the split launch and read by the kernel that finishes the tiles.
struct SplitWs {
  float* partial;
  int max_blocks;
};
constexpr int SPLIT_MAX_BLOCKS = 256;                       // CU count of MI355X; fewer blocks split on a smaller part
constexpr size_t SPLIT_BLOCK_BYTES = 256 * 256 * sizeof(float);
// Several products of one kind in one launch (matrices of different shapes): the persistent
// blocks walk the tiles of problem 0, then of problem 1, ...  Used for shares whose shape
// classes are too small to fill the chip on their own.
constexpr int MAX_KINDS = 4;
struct GemmProblem {
  GemmDims d;
  const void* p;       // first operand  [nb][M][K] panels
  const void* q;       // second operand [nb][N][K] panels
  void* c;             // output (UPDATE: the straight image)
  void* ct;            // UPDATE: the transposed image
  const void* aux;     // POLY: A
  const float* scale;  // per-matrix factor or nullptr
};
struct GemmBatch {
  int n;
  GemmProblem pr[MAX_KINDS];
};
hipError_t launch_gram_bf16_multi(const GemmBatch& g, hipStream_t st);
hipError_t launch_poly_bf16_multi(const GemmBatch& g, float ca, float cb, float cc, hipStream_t st);
hipError_t launch_update_bf16_multi(const GemmBatch& g, hipStream_t st);

// A = scale2[b] * X X^T                      (P = Q = XW)
hipError_t launch_gram_bf16(const GemmDims& d, const void* xw, void* a_out, const float* scale2, const SplitWs& w,
                            hipStream_t st);
// B = ca I + cb A + cc A A                   (P = Q = A, symmetric)
hipError_t launch_poly_bf16(const GemmDims& d, const void* a_in, void* b_out, float ca, float cb, float cc,
                            const SplitWs& w, hipStream_t st);
// X' = scale[b] * B X: XW' [mp][np] straight and XT' [np][mp] transposed  (P = B, Q = XT)
hipError_t launch_update_bf16(const GemmDims& d, const void* b_in, const void* xt_in, void* xw_out, void* xt_out,
                              const float* scale, const SplitWs& w, hipStream_t st);
// last step: O = scale[b] * P Q^T goes straight into the caller's buffers; the caller of
// this launcher orders the operands so that C is in the matrix's own orientation:
// wide matrix: P = B, Q = XT (C = B X);  tall matrix: P = XT, Q = B (C = X^T B = (B X)^T)
hipError_t launch_final_bf16(const GemmDims& d, const void* p, const void* q, const float* scale, const SplitWs& w,
                             const Shape& s, const OutSpec& o, hipStream_t st);
// the same for a symmetric result O = X X^T (M = N): only the tiles on and above the diagonal are computed and
// written; the elements below the diagonal tiles are left as they were (the caller mirrors them)
hipError_t launch_final_sym_bf16(const GemmDims& d, const void* x, const SplitWs& w, const Shape& s, const OutSpec& o,
                                 hipStream_t st);

// ---- fp32 verification GEMMs (same contracts, float storage) ----------------------
hipError_t launch_gram_f32(const GemmDims& d, const void* xw, void* a_out, const float* scale2, hipStream_t st);
hipError_t launch_poly_f32(const GemmDims& d, const void* a_in, void* b_out, float ca, float cb, float cc,
                           hipStream_t st);
hipError_t launch_update_f32(const GemmDims& d, const void* b_in, const void* xt_in, void* xw_out, void* xt_out,
                             const float* scale, hipStream_t st);
hipError_t launch_final_f32(const GemmDims& d, const void* p, const void* q, const float* scale,
                            const Shape& s, const OutSpec& o, hipStream_t st);

}  // namespace canz
