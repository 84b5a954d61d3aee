// Streaming kernels of the Muon step: momentum update fused with the (TP) gather, the
// cast into both working orientations and the Frobenius-norm partial sums; the norm
// scale; and the direct update used when no Newton-Schulz step is requested.
// These passes are HBM-bound: every global access is a 16-byte vector per lane on
// contiguous rows, the transpose goes through LDS, the reduction through wave shuffles.
#include "device_util.h"
#include "panel_layout.h"

namespace canz {
namespace {

constexpr int TILE = EW_TILE;     // 64 x 64 elements per block
constexpr int NTHREADS = 256;

template <typename T>
struct Vec8;
template <>
struct alignas(16) Vec8<float> {
  float v[8];
};
template <>
struct alignas(16) Vec8<__bf16> {
  __bf16 v[8];
};

// One block = one 64 x 64 tile of one matrix in the caller's orientation, extended over
// the padded extents (elements outside rows x cols are zeros and touch no caller memory).
// Step 2 of the operator: M <- beta M + G, U = M (or G + beta M); step 1 (TP gather) is
// the fragment lookup on the load.
template <typename T, bool VEC>
__global__ __launch_bounds__(NTHREADS) void k_momentum(Shape s, PtrTable grad, int grad_dtype, PtrTable mom,
                                                        float beta, int nesterov, T* __restrict__ xw,
                                                        T* __restrict__ xt, float* __restrict__ partial) {
  __shared__ float tile[TILE][TILE + 1];
  __shared__ float wsum[NTHREADS / 64];

  const int b = blockIdx.z;
  const int r0 = blockIdx.y * TILE, c0 = blockIdx.x * TILE;
  const int rows = static_cast<int>(s.rows), cols = static_cast<int>(s.cols);
  const int wf = static_cast<int>(s.wfrag);
  // straight = same orientation as the caller's matrix; transposed = the other one
  const int64_t pr = s.tall ? s.np : s.mp, pc = s.tall ? s.mp : s.np;
  T* straight = (s.tall ? xt : xw) + static_cast<int64_t>(b) * pr * pc;
  T* transposed = (s.tall ? xw : xt) + static_cast<int64_t>(b) * pr * pc;
  float* mptr = static_cast<float*>(mom.p[b]);

  const int t = threadIdx.x;
  const int cv = (t & 7) * 8;
  float ss = 0.f;
  // Phase 1: every load of both half-tiles is issued before the first store (the momentum
  // store of one half must not hold back the loads of the other: the buffers come from
  // pointer tables and may alias as far as the compiler knows).
  float g[2][8], mo[2][8];
  bool live[2];
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int row = r0 + (t >> 3) + half * 32, col = c0 + cv;
    live[half] = row < rows && col < cols;
#pragma unroll
    for (int e = 0; e < 8; ++e) g[half][e] = 0.f, mo[half][e] = 0.f;
    if (!live[half]) continue;
    if (VEC) {
      // cols and wfrag are multiples of 8 here: the vector lies in one fragment
      const int f = col / wf;
      const int64_t gi = static_cast<int64_t>(row) * wf + (col - f * wf);
      if (grad_dtype == CANZ_DT_BF16) {
        const bf16x8 gv = *reinterpret_cast<const bf16x8*>(static_cast<const __bf16*>(grad.p[b * s.tp + f]) + gi);
#pragma unroll
        for (int e = 0; e < 8; ++e) g[half][e] = static_cast<float>(gv[e]);
      } else {
        const f32x4* gp = reinterpret_cast<const f32x4*>(static_cast<const float*>(grad.p[b * s.tp + f]) + gi);
        const f32x4 g0 = gp[0], g1 = gp[1];
#pragma unroll
        for (int e = 0; e < 4; ++e) g[half][e] = g0[e], g[half][4 + e] = g1[e];
      }
      const f32x4* mp4 = reinterpret_cast<const f32x4*>(mptr + static_cast<int64_t>(row) * cols + col);
      const f32x4 m0 = mp4[0], m1 = mp4[1];
#pragma unroll
      for (int e = 0; e < 4; ++e) mo[half][e] = m0[e], mo[half][4 + e] = m1[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int c = col + e;
        if (c < cols) {
          const int f = c / wf;
          const int64_t gi = static_cast<int64_t>(row) * wf + (c - f * wf);
          g[half][e] = grad_dtype == CANZ_DT_BF16
                           ? static_cast<float>(static_cast<const __bf16*>(grad.p[b * s.tp + f])[gi])
                           : static_cast<const float*>(grad.p[b * s.tp + f])[gi];
          mo[half][e] = mptr[static_cast<int64_t>(row) * cols + c];
        }
      }
    }
  }
  // Phase 2: momentum, stores, working copies
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int rl = (t >> 3) + half * 32;
    const int row = r0 + rl, col = c0 + cv;
    float u[8], mn[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mn[e] = beta * mo[half][e] + g[half][e];
      u[e] = nesterov ? g[half][e] + beta * mn[e] : mn[e];
    }
    if (live[half]) {
      if (VEC) {
        f32x4 n0, n1;
#pragma unroll
        for (int e = 0; e < 4; ++e) n0[e] = mn[e], n1[e] = mn[4 + e];
        f32x4* mp4 = reinterpret_cast<f32x4*>(mptr + static_cast<int64_t>(row) * cols + col);
        mp4[0] = n0;
        mp4[1] = n1;
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (col + e < cols) mptr[static_cast<int64_t>(row) * cols + col + e] = mn[e];
      }
    }
    Vec8<T> o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      ss += u[e] * u[e];
      o.v[e] = from_f32<T>(u[e]);
      tile[rl][cv + e] = u[e];
    }
    *reinterpret_cast<Vec8<T>*>(straight + WorkLayout<T>::chunk_off(row, col, pc)) = o;
  }
  __syncthreads();
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int cl = (t >> 3) + half * 32;  // column of the tile = row of the transposed tile
    Vec8<T> o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.v[e] = from_f32<T>(tile[cv + e][cl]);
    *reinterpret_cast<Vec8<T>*>(transposed + WorkLayout<T>::chunk_off(c0 + cl, r0 + cv, pr)) = o;
  }
  // sum of squares of this tile, fixed order: lanes -> waves -> thread 0
  ss = wave_sum(ss);
  if ((t & 63) == 0) wsum[t >> 6] = ss;
  __syncthreads();
  if (t == 0) {
    const int tiles = gridDim.x * gridDim.y;
    partial[static_cast<int64_t>(b) * tiles + blockIdx.y * gridDim.x + blockIdx.x] =
        (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
  }
}

// Step 3 of the operator, as a scalar: 1 / (||U||_F + eps).  One block per matrix; the
// tile sums are added in fp64 in a fixed order, so the result does not depend on timing.
__global__ __launch_bounds__(NTHREADS) void k_norm_scale(int n_partial, const float* __restrict__ partial, float eps,
                                                          float* __restrict__ scale, float* __restrict__ scale2) {
  __shared__ double red[NTHREADS];
  const int b = blockIdx.x, t = threadIdx.x;
  double acc = 0.0;
  for (int i = t; i < n_partial; i += NTHREADS) acc += static_cast<double>(partial[static_cast<int64_t>(b) * n_partial + i]);
  red[t] = acc;
  __syncthreads();
  for (int w = NTHREADS / 2; w > 0; w >>= 1) {
    if (t < w) red[t] += red[t + w];
    __syncthreads();
  }
  if (t == 0) {
    const float sc = static_cast<float>(1.0 / (sqrt(red[0]) + static_cast<double>(eps)));
    scale[b] = sc;
    scale2[b] = sc * sc;
  }
}

// ns_steps == 0: O = scale * U, read back from the working copy in the caller's orientation.
template <typename T>
__global__ __launch_bounds__(NTHREADS) void k_apply(Shape s, const T* __restrict__ x, int64_t ld, int64_t batch_stride,
                                                     const float* __restrict__ scale, OutSpec o) {
  const int b = blockIdx.z;
  const float sc = scale[b];
  const T* xb = x + static_cast<int64_t>(b) * batch_stride;
  for (int row = blockIdx.y; row < s.rows; row += gridDim.y)
    for (int col = blockIdx.x * NTHREADS + threadIdx.x; col < s.cols; col += gridDim.x * NTHREADS)
      store_out(o, s, b, row, col, sc * static_cast<float>(xb[WorkLayout<T>::chunk_off(row, col & ~7, ld) + (col & 7)]));
}

}  // namespace

int momentum_tiles(const Shape& s) {
  return static_cast<int>((s.mp / TILE) * (s.np / TILE));
}

template <typename T>
hipError_t launch_momentum(const Shape& s, int nb, const PtrTable& grad, int grad_dtype, const PtrTable& mom,
                           float beta, int nesterov, T* xw, T* xt, float* partial, hipStream_t st) {
  const int64_t pr = s.tall ? s.np : s.mp, pc = s.tall ? s.mp : s.np;
  const dim3 grid(static_cast<unsigned>(pc / TILE), static_cast<unsigned>(pr / TILE), static_cast<unsigned>(nb));
  const bool vec = (s.cols % 8 == 0) && (s.wfrag % 8 == 0);
  if (vec)
    hipLaunchKernelGGL((k_momentum<T, true>), grid, dim3(NTHREADS), 0, st, s, grad, grad_dtype, mom, beta, nesterov,
                       xw, xt, partial);
  else
    hipLaunchKernelGGL((k_momentum<T, false>), grid, dim3(NTHREADS), 0, st, s, grad, grad_dtype, mom, beta, nesterov,
                       xw, xt, partial);
  return hipGetLastError();
}

template hipError_t launch_momentum<__bf16>(const Shape&, int, const PtrTable&, int, const PtrTable&, float, int,
                                            __bf16*, __bf16*, float*, hipStream_t);
template hipError_t launch_momentum<float>(const Shape&, int, const PtrTable&, int, const PtrTable&, float, int,
                                           float*, float*, float*, hipStream_t);

hipError_t launch_norm_scale(int nb, int n_partial, const float* partial, float eps, float* scale, float* scale2,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_norm_scale, dim3(nb), dim3(NTHREADS), 0, st, n_partial, partial, eps, scale, scale2);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_apply(const Shape& s, int nb, const T* x_straight, int64_t ld, int64_t batch_stride,
                        const float* scale, const OutSpec& o, hipStream_t st) {
  const unsigned gx = static_cast<unsigned>((s.cols + NTHREADS - 1) / NTHREADS);
  const dim3 grid(gx > 64 ? 64 : gx, static_cast<unsigned>(s.rows > 32768 ? 32768 : s.rows), static_cast<unsigned>(nb));
  hipLaunchKernelGGL((k_apply<T>), grid, dim3(NTHREADS), 0, st, s, x_straight, ld, batch_stride, scale, o);
  return hipGetLastError();
}
template hipError_t launch_apply<__bf16>(const Shape&, int, const __bf16*, int64_t, int64_t, const float*,
                                         const OutSpec&, hipStream_t);
template hipError_t launch_apply<float>(const Shape&, int, const float*, int64_t, int64_t, const float*,
                                        const OutSpec&, hipStream_t);

}  // namespace canz
