// Small device-side helpers shared by the kernels: bf16 conversion, wave / block
// reductions, and the store of one output element into the caller's buffers.
#pragma once
#include <hip/hip_runtime.h>

#include "canz.h"
#include "kernels.h"

namespace canz {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ __bf16 from_f32<__bf16>(float v) {
  return static_cast<__bf16>(v);  // round-to-nearest-even (v_cvt_pk_bf16_f32)
}

// Sum over the 64 lanes of a wavefront; every lane receives the total.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// The two places where an epilogue combines several terms, written once with the roundings
// pinned (one product, then one fused multiply-add), so that every kernel that produces the
// same element produces the same bits whatever its tile shape.
//   polynomial  a I + b A + c (A A)
__device__ __forceinline__ float poly_value(float a_elem, float aa_elem, float ca, float cb, float cc, bool diag) {
  const float v = __builtin_fmaf(cb, a_elem, cc * aa_elem);
  return diag ? v + ca : v;
}
//   update      old * decay + neg_lr_scale * O   (old = 0 gives Delta W = neg_lr_scale * O exactly)
__device__ __forceinline__ float apply_update(float old, float decay, float neg_lr_scale, float ortho) {
  return __builtin_fmaf(neg_lr_scale, ortho, old * decay);
}

// O (one element of the orthogonalised matrix, caller's orientation) -> caller's buffer.
//   CANZ_OUT_PARAM: P <- P * decay + neg_lr_scale * O       (Sec. 3.3 stage (2))
//   CANZ_OUT_DELTA: Delta W fragment <- neg_lr_scale * O     (Sec. 4.1 stage (3))
__device__ __forceinline__ void store_out(const OutSpec& o, const Shape& s, int b, int row, int col, float ortho) {
  const float delta = o.neg_lr_scale * ortho;
  if (o.out_mode == CANZ_OUT_PARAM) {
    const int64_t idx = static_cast<int64_t>(row) * s.cols + col;
    if (o.out_dtype == CANZ_DT_F32) {
      float* p = static_cast<float*>(o.out.p[b]);
      p[idx] = apply_update(p[idx], o.decay, o.neg_lr_scale, ortho);
    } else {
      __bf16* p = static_cast<__bf16*>(o.out.p[b]);
      p[idx] = static_cast<__bf16>(apply_update(static_cast<float>(p[idx]), o.decay, o.neg_lr_scale, ortho));
    }
  } else {
    const int wf = static_cast<int>(s.wfrag);
    const int f = col / wf;
    const int64_t idx = static_cast<int64_t>(row) * wf + (col - f * wf);
    if (o.out_dtype == CANZ_DT_F32) {
      static_cast<float*>(o.out.p[b * s.tp + f])[idx] = delta;
    } else {
      static_cast<__bf16*>(o.out.p[b * s.tp + f])[idx] = static_cast<__bf16>(delta);
    }
  }
}


// The same for the 16 accumulator values one lane holds of a 32 x 32 MFMA tile: rows
// row0 + 8 * (r / 4) + (r % 4), r = 0..15, one column.  All old parameter values are
// loaded before the first store, so the 16 read-modify-writes overlap instead of
// running as a chain of dependent memory round trips.
__device__ __forceinline__ void store_out_tile(const OutSpec& o, const Shape& s, int b, int row0, int col,
                                               const float (&ortho)[16]) {
  if (col >= s.cols) return;
  const int rows = static_cast<int>(s.rows);
  int ld = static_cast<int>(s.cols), c = col, tab = b;
  if (o.out_mode == CANZ_OUT_DELTA) {
    ld = static_cast<int>(s.wfrag);
    const int f = col / ld;
    c = col - f * ld;
    tab = b * s.tp + f;
  }
  void* base = o.out.p[tab];
  float val[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) val[r] = 0.f;
  if (o.out_mode == CANZ_OUT_PARAM) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = row0 + 8 * (r >> 2) + (r & 3);
      if (row < rows) {
        const int64_t idx = static_cast<int64_t>(row) * ld + c;
        val[r] = o.out_dtype == CANZ_DT_F32 ? static_cast<const float*>(base)[idx]
                                            : static_cast<float>(static_cast<const __bf16*>(base)[idx]);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = row0 + 8 * (r >> 2) + (r & 3);
    if (row < rows) {
      const int64_t idx = static_cast<int64_t>(row) * ld + c;
      const float v = apply_update(val[r], o.decay, o.neg_lr_scale, ortho[r]);
      if (o.out_dtype == CANZ_DT_F32)
        static_cast<float*>(base)[idx] = v;
      else
        static_cast<__bf16*>(base)[idx] = static_cast<__bf16>(v);
    }
  }
}


// Four consecutive columns at once (row length and col are multiples of 4, so the four
// elements are 16-byte aligned in fp32 buffers and lie in one TP fragment).
__device__ __forceinline__ f32x4 load_param4(const OutSpec& o, const Shape& s, int b, int row, int col) {
  const int64_t idx = static_cast<int64_t>(row) * s.cols + col;
  if (o.out_dtype == CANZ_DT_F32) return *reinterpret_cast<const f32x4*>(static_cast<const float*>(o.out.p[b]) + idx);
  const bf16x4 v = *reinterpret_cast<const bf16x4*>(static_cast<const __bf16*>(o.out.p[b]) + idx);
  f32x4 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) r[e] = static_cast<float>(v[e]);
  return r;
}

__device__ __forceinline__ void store_out4(const OutSpec& o, const Shape& s, int b, int row, int col, f32x4 val) {
  int ld = static_cast<int>(s.cols), c = col, tab = b;
  if (o.out_mode == CANZ_OUT_DELTA) {
    ld = static_cast<int>(s.wfrag);
    const int f = col / ld;
    c = col - f * ld;
    tab = b * s.tp + f;
  }
  const int64_t idx = static_cast<int64_t>(row) * ld + c;
  if (o.out_dtype == CANZ_DT_F32) {
    *reinterpret_cast<f32x4*>(static_cast<float*>(o.out.p[tab]) + idx) = val;
  } else {
    bf16x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = static_cast<__bf16>(val[e]);
    *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(o.out.p[tab]) + idx) = v;
  }
}

}  // namespace canz
