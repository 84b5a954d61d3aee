// Batched bf16 MFMA GEMMs of the Newton-Schulz iteration (step 4 of the operator):
//   C[b][i][j] = sum_k P[b][i][k] * Q[b][j][k]        fp32 accumulate
// Both operands are contiguous along k (see kernels.h for why both orientations of X are
// kept), which is the lane layout v_mfma_f32_32x32x16_bf16 wants: lane l supplies 8
// consecutive k of row (l % 32), k-group (l / 32).
//
// Tiling: one 256-thread block (4 wavefronts, 2 x 2) owns a 256 x 256 tile of C; each
// wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32 accumulators per lane.  K is
// walked in steps of 64.  The 256 x 64 panels of P and Q are staged in LDS (32 KiB each)
// with the 16-byte chunk index XOR-swizzled by (row >> 1) & 7 so that the 16 lanes served
// per LDS cycle hit 16 different bank groups on both the b128 stores and the MFMA operand
// loads.  The next panel is fetched into registers while the current one is multiplied.
// Extents are multiples of 256 (zero padded by the producer), so there are no bounds
// checks on the operand side; only the final epilogue clips to the caller's shape.
#include "device_util.h"

namespace canz {
namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 256;
constexpr int CHUNKS = BK / 8;                 // 16-byte chunks per panel row
constexpr int LD_PASSES = BM * CHUNKS / NTHREADS;  // 8 loads of 16 B per thread and panel

enum { EPI_GRAM = 0, EPI_POLY = 1, EPI_UPDATE = 2, EPI_FINAL = 3 };

struct EpiArgs {
  void* c;                 // GRAM/POLY: [nb][M][N] bf16; UPDATE: XW' [nb][M][N]
  void* ct;                // UPDATE: XT' [nb][N][M]
  const void* aux;         // POLY: A [nb][M][N]
  const float* scale;      // per-matrix factor applied to the accumulator, or nullptr
  float ca, cb, cc;        // POLY coefficients
};

__device__ __forceinline__ int swz(int row, int chunk) {
  return (row * CHUNKS + (chunk ^ ((row >> 1) & (CHUNKS - 1)))) * 8;  // element offset in the panel
}

template <int EPI>
__global__ __launch_bounds__(NTHREADS) void k_gemm_nt_bf16(GemmDims d, const __bf16* __restrict__ P,
                                                            const __bf16* __restrict__ Q, EpiArgs e, Shape s,
                                                            OutSpec o) {
  __shared__ __attribute__((aligned(16))) __bf16 sP[BM * BK];
  __shared__ __attribute__((aligned(16))) __bf16 sQ[BN * BK];

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

  const __bf16* Pg = P + static_cast<int64_t>(b) * d.sp + static_cast<int64_t>(tm) * BM * d.ldp;
  const __bf16* Qg = Q + static_cast<int64_t>(b) * d.sq + static_cast<int64_t>(tn) * BN * d.ldq;

  // global -> register staging: thread t fetches chunk (t % 8) of rows (t / 8) + 32 * pass
  const int ld_row = t >> 3, ld_chunk = t & 7;
  bf16x8 rp[LD_PASSES], rq[LD_PASSES];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int p = 0; p < LD_PASSES; ++p) {
      const int row = ld_row + 32 * p;
      rp[p] = *reinterpret_cast<const bf16x8*>(Pg + static_cast<int64_t>(row) * d.ldp + k0 + ld_chunk * 8);
      rq[p] = *reinterpret_cast<const bf16x8*>(Qg + static_cast<int64_t>(row) * d.ldq + k0 + ld_chunk * 8);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int p = 0; p < LD_PASSES; ++p) {
      const int row = ld_row + 32 * p;
      *reinterpret_cast<bf16x8*>(sP + swz(row, ld_chunk)) = rp[p];
      *reinterpret_cast<bf16x8*>(sQ + swz(row, ld_chunk)) = rq[p];
    }
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frag_row = lane & 31, frag_kg = lane >> 5;
  const int nk = static_cast<int>(d.K / BK);
  fetch(0);
  stash();
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) fetch(static_cast<int64_t>(kt + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(sP + swz(wm * 128 + i * 32 + frag_row, kk * 2 + frag_kg));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(sQ + swz(wn * 128 + j * 32 + frag_row, kk * 2 + frag_kg));
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
    if (kt + 1 < nk) {
      stash();
      __syncthreads();
    }
  }

  // ---- epilogue.  Accumulator register r of lane l in MFMA tile (i, j) is element
  //      row = 8 * (r / 4) + 4 * (l / 32) + (r % 4),  col = l % 32   of that 32 x 32 tile.
  const float sc = e.scale ? e.scale[b] : 1.f;
  const int row_base = tm * BM + wm * 128 + 4 * (lane >> 5);
  const int col_base = tn * BN + wn * 128 + (lane & 31);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = col_base + j * 32;
#pragma unroll
      for (int rq4 = 0; rq4 < 4; ++rq4) {
        const int row0 = row_base + i * 32 + rq4 * 8;
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = acc[i][j][rq4 * 4 + q] * sc;
        if (EPI == EPI_GRAM) {
          __bf16* C = static_cast<__bf16*>(e.c) + static_cast<int64_t>(b) * d.M * d.N;
#pragma unroll
          for (int q = 0; q < 4; ++q) C[static_cast<int64_t>(row0 + q) * d.N + col] = static_cast<__bf16>(v[q]);
        } else if (EPI == EPI_POLY) {
          __bf16* C = static_cast<__bf16*>(e.c) + static_cast<int64_t>(b) * d.M * d.N;
          const __bf16* A = static_cast<const __bf16*>(e.aux) + static_cast<int64_t>(b) * d.M * d.N;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int64_t idx = static_cast<int64_t>(row0 + q) * d.N + col;
            float r = e.cb * static_cast<float>(A[idx]) + e.cc * v[q];
            if (row0 + q == col) r += e.ca;
            C[idx] = static_cast<__bf16>(r);
          }
        } else if (EPI == EPI_UPDATE) {
          __bf16* C = static_cast<__bf16*>(e.c) + static_cast<int64_t>(b) * d.M * d.N;
          __bf16* CT = static_cast<__bf16*>(e.ct) + static_cast<int64_t>(b) * d.M * d.N;
          bf16x4 pk;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            pk[q] = static_cast<__bf16>(v[q]);
            C[static_cast<int64_t>(row0 + q) * d.N + col] = pk[q];
          }
          *reinterpret_cast<bf16x4*>(CT + static_cast<int64_t>(col) * d.M + row0) = pk;
        } else {
          // (row, col) index the wide orientation [m][n]; the caller's matrix is its transpose if tall
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int wr = row0 + q, wc = col;
            const int orow = s.tall ? wc : wr, ocol = s.tall ? wr : wc;
            if (orow < s.rows && ocol < s.cols) store_out(o, s, b, orow, ocol, v[q]);
          }
        }
      }
    }
  }
}

template <int EPI>
hipError_t launch(const GemmDims& d, const void* P, const void* Q, const EpiArgs& e, const Shape& s, const OutSpec& o,
                  hipStream_t st) {
  const int64_t blocks = (d.M / BM) * (d.N / BN) * d.nb;
  hipLaunchKernelGGL((k_gemm_nt_bf16<EPI>), dim3(static_cast<unsigned>(blocks)), dim3(NTHREADS), 0, st, d,
                     static_cast<const __bf16*>(P), static_cast<const __bf16*>(Q), e, s, o);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gram_bf16(const GemmDims& d, const void* xw, void* a_out, const float* scale2, hipStream_t st) {
  EpiArgs e{};
  e.c = a_out;
  e.scale = scale2;
  return launch<EPI_GRAM>(d, xw, xw, e, Shape{}, OutSpec{}, st);
}

hipError_t launch_poly_bf16(const GemmDims& d, const void* a_in, void* b_out, float ca, float cb, float cc,
                            hipStream_t st) {
  EpiArgs e{};
  e.c = b_out;
  e.aux = a_in;
  e.ca = ca, e.cb = cb, e.cc = cc;
  return launch<EPI_POLY>(d, a_in, a_in, e, Shape{}, OutSpec{}, st);
}

hipError_t launch_update_bf16(const GemmDims& d, const void* b_in, const void* xt_in, void* xw_out, void* xt_out,
                              const float* scale, hipStream_t st) {
  EpiArgs e{};
  e.c = xw_out;
  e.ct = xt_out;
  e.scale = scale;
  return launch<EPI_UPDATE>(d, b_in, xt_in, e, Shape{}, OutSpec{}, st);
}

hipError_t launch_final_bf16(const GemmDims& d, const void* b_in, const void* xt_in, const float* scale,
                             const Shape& s, const OutSpec& o, hipStream_t st) {
  EpiArgs e{};
  e.scale = scale;
  return launch<EPI_FINAL>(d, b_in, xt_in, e, s, o, st);
}

}  // namespace canz
