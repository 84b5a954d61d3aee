// fp32 verification path of the Newton-Schulz GEMMs: same contracts as the bf16 kernels
// (C[b][i][j] = sum_k P[b][i][k] Q[b][j][k], both operands contiguous along k, padded
// extents), float storage, v_mfma_f32_32x32x2_f32.  This path exists to separate kernel
// bugs from bf16 rounding; it is tiled plainly (128 x 128 x 16, 2 x 2 wavefronts of
// 64 x 64) and is not tuned.  Long sums are split: every FLUSH k-steps the running
// accumulator is folded into a second one, which keeps the rounding error of the
// K = 25600 Gram products near that of a blocked summation.
#include "device_util.h"

namespace canz {
namespace {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int NTHREADS = 256;
constexpr int LDS_LD = BM + 4;
constexpr int FLUSH = 32;  // k-tiles (512 k) between folds of the accumulator

enum { EPI_GRAM = 0, EPI_POLY = 1, EPI_UPDATE = 2, EPI_FINAL = 3 };

struct EpiArgs {
  void* c;
  void* ct;
  const void* aux;
  const float* scale;
  float ca, cb, cc;
};

template <int EPI>
__global__ __launch_bounds__(NTHREADS) void k_gemm_nt_f32(GemmDims d, const float* __restrict__ P,
                                                           const float* __restrict__ Q, EpiArgs e, Shape s,
                                                           OutSpec o) {
  __shared__ float sP[BK][LDS_LD];  // k-major: lanes of one MFMA operand read consecutive rows
  __shared__ float sQ[BK][LDS_LD];

  const int tiles_n = static_cast<int>(d.N / BN);
  const int tiles_m = static_cast<int>(d.M / BM);
  const int per_batch = tiles_m * tiles_n;
  const int bid = blockIdx.x;
  const int b = bid / per_batch;
  const int tix = bid - b * per_batch;
  const int tm = tix / tiles_n, tn = tix - tm * tiles_n;

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const float* Pg = P + static_cast<int64_t>(b) * d.sp + static_cast<int64_t>(tm) * BM * d.ldp;
  const float* Qg = Q + static_cast<int64_t>(b) * d.sq + static_cast<int64_t>(tn) * BN * d.ldq;

  const int ld_row = t >> 2, ld_k = (t & 3) * 4;  // rows ld_row and ld_row + 64, 4 consecutive k
  f32x16 acc[2][2], tot[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f, tot[i][j][r] = 0.f;

  const int nk = static_cast<int>(d.K / BK);
  for (int kt = 0; kt < nk; ++kt) {
    const int64_t k0 = static_cast<int64_t>(kt) * BK + ld_k;
    f32x4 p0 = *reinterpret_cast<const f32x4*>(Pg + static_cast<int64_t>(ld_row) * d.ldp + k0);
    f32x4 p1 = *reinterpret_cast<const f32x4*>(Pg + static_cast<int64_t>(ld_row + 64) * d.ldp + k0);
    f32x4 q0 = *reinterpret_cast<const f32x4*>(Qg + static_cast<int64_t>(ld_row) * d.ldq + k0);
    f32x4 q1 = *reinterpret_cast<const f32x4*>(Qg + static_cast<int64_t>(ld_row + 64) * d.ldq + k0);
    __syncthreads();  // previous tile fully consumed
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      sP[ld_k + c][ld_row] = p0[c];
      sP[ld_k + c][ld_row + 64] = p1[c];
      sQ[ld_k + c][ld_row] = q0[c];
      sQ[ld_k + c][ld_row + 64] = q1[c];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; k += 2) {
      float fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = sP[k + (lane >> 5)][wm * 64 + i * 32 + (lane & 31)];
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = sQ[k + (lane >> 5)][wn * 64 + j * 32 + (lane & 31)];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if ((kt + 1) % FLUSH == 0 || kt + 1 == nk) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) tot[i][j][r] += acc[i][j][r], acc[i][j][r] = 0.f;
    }
  }

  const float sc = e.scale ? e.scale[b] : 1.f;
  const int row_base = tm * BM + wm * 64 + 4 * (lane >> 5);
  const int col_base = tn * BN + wn * 64 + (lane & 31);
  const int64_t cb = static_cast<int64_t>(b) * d.M * d.N;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = col_base + j * 32;
      if (EPI == EPI_FINAL) {
        float v[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = tot[i][j][r] * sc;
        store_out_tile(o, s, b, row_base + i * 32, col, v);
        continue;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = row_base + i * 32 + (r >> 2) * 8 + (r & 3);
        const float v = tot[i][j][r] * sc;
        const int64_t idx = cb + static_cast<int64_t>(row) * d.N + col;
        if (EPI == EPI_GRAM) {
          static_cast<float*>(e.c)[idx] = v;
        } else if (EPI == EPI_POLY) {
          float r2 = e.cb * static_cast<const float*>(e.aux)[idx] + e.cc * v;
          if (row == col) r2 += e.ca;
          static_cast<float*>(e.c)[idx] = r2;
        } else if (EPI == EPI_UPDATE) {
          static_cast<float*>(e.c)[idx] = v;
          static_cast<float*>(e.ct)[cb + static_cast<int64_t>(col) * d.M + row] = v;
        }
      }
    }
  }
}

template <int EPI>
hipError_t launch(const GemmDims& d, const void* P, const void* Q, const EpiArgs& e, const Shape& s, const OutSpec& o,
                  hipStream_t st) {
  const int64_t blocks = (d.M / BM) * (d.N / BN) * d.nb;
  hipLaunchKernelGGL((k_gemm_nt_f32<EPI>), dim3(static_cast<unsigned>(blocks)), dim3(NTHREADS), 0, st, d,
                     static_cast<const float*>(P), static_cast<const float*>(Q), e, s, o);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gram_f32(const GemmDims& d, const void* xw, void* a_out, const float* scale2, hipStream_t st) {
  EpiArgs e{};
  e.c = a_out;
  e.scale = scale2;
  return launch<EPI_GRAM>(d, xw, xw, e, Shape{}, OutSpec{}, st);
}

hipError_t launch_poly_f32(const GemmDims& d, const void* a_in, void* b_out, float ca, float cb, float cc,
                           hipStream_t st) {
  EpiArgs e{};
  e.c = b_out;
  e.aux = a_in;
  e.ca = ca, e.cb = cb, e.cc = cc;
  return launch<EPI_POLY>(d, a_in, a_in, e, Shape{}, OutSpec{}, st);
}

hipError_t launch_update_f32(const GemmDims& d, const void* b_in, const void* xt_in, void* xw_out, void* xt_out,
                             const float* scale, hipStream_t st) {
  EpiArgs e{};
  e.c = xw_out;
  e.ct = xt_out;
  e.scale = scale;
  return launch<EPI_UPDATE>(d, b_in, xt_in, e, Shape{}, OutSpec{}, st);
}

hipError_t launch_final_f32(const GemmDims& d, const void* p, const void* q, const float* scale, const Shape& s,
                            const OutSpec& o, hipStream_t st) {
  EpiArgs e{};
  e.scale = scale;
  return launch<EPI_FINAL>(d, p, q, e, s, o, st);
}

}  // namespace canz
