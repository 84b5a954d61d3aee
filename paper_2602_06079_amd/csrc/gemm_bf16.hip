// Batched bf16 MFMA GEMMs of the Newton-Schulz iteration (step 4 of the operator):
//   C[b][i][j] = sum_k P[b][i][k] * Q[b][j][k]        fp32 accumulate
// Both operands are contiguous along k (see kernels.h for why both orientations of X are
// kept), which is the lane layout v_mfma_f32_32x32x16_bf16 wants: lane l supplies 8
// consecutive k of row (l % 32), k-group (l / 32).
//
// Tiling: one 256-thread block (4 wavefronts, 2 x 2) owns a 256 x 256 tile of C; each
// wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32 accumulators per lane (one
// wavefront per SIMD, 512 registers each).  K is walked in steps of 64.
//
// Operand staging: the 256 x 64 panels of P and Q go from global memory straight into LDS
// (global_load_lds_dwordx4: every lane fetches 16 bytes, a wavefront fills 1 KiB = 8 panel
// rows), into one of two 64 KiB stages.  Inside a panel row the 16-byte chunk index is
// XOR-swizzled by (row >> 1) & 7 - applied on the global side, by choosing which chunk a
// lane fetches - so that the ds_read_b128 operand loads of 16 consecutive rows hit 16
// different bank groups.
//
// Pipeline per k-step (one barrier): the panels of step t+1 are in flight while step t is
// multiplied; the MFMA operand fragments are double-buffered in registers, and the
// barrier sits before the last quarter of the step so that the fetch of step t+2 and the
// first fragments of step t+1 are issued under the remaining 16 MFMAs.
//
// Blocks are numbered so that the 32 blocks resident on one XCD (blockIdx % 8 selects the
// XCD) form a 4 x 8 patch of tiles of one matrix and share panels in that XCD's L2.
// Extents are multiples of 256 (zero padded by the producer), so there are no bounds
// checks on the operand side; only the final epilogue clips to the caller's shape.
#include "device_util.h"

namespace canz {
namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int NTHREADS = 256;
constexpr int CHUNKS = BK / 8;   // 16-byte chunks per panel row
constexpr int GROUP_M = 4;       // tile rows per raster band
constexpr int N_XCD = 8;

enum { EPI_GRAM = 0, EPI_POLY = 1, EPI_UPDATE = 2, EPI_FINAL = 3 };

struct EpiArgs {
  void* c;                 // GRAM/POLY: [nb][M][N] bf16; UPDATE: straight output [nb][M][N]
  void* ct;                // UPDATE: transposed output [nb][N][M]
  const void* aux;         // POLY: A [nb][M][N]
  const float* scale;      // per-matrix factor applied to the accumulator, or nullptr
  float ca, cb, cc;        // POLY coefficients
};

#define CANZ_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define CANZ_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ int swz(int row, int chunk) {
  return (row * CHUNKS + (chunk ^ ((row >> 1) & (CHUNKS - 1)))) * 8;  // element offset in the panel
}

template <int EPI>
__global__ __launch_bounds__(NTHREADS) void k_gemm_nt_bf16(GemmDims d, const __bf16* __restrict__ P,
                                                            const __bf16* __restrict__ Q, EpiArgs e, Shape s,
                                                            OutSpec o) {
  // four separate arrays (not one carved buffer): the compiler then knows that a fetch into
  // one stage does not alias the operand reads of the other and keeps them overlapped
  __shared__ __attribute__((aligned(1024))) __bf16 sP0[BM * BK];
  __shared__ __attribute__((aligned(1024))) __bf16 sQ0[BN * BK];
  __shared__ __attribute__((aligned(1024))) __bf16 sP1[BM * BK];
  __shared__ __attribute__((aligned(1024))) __bf16 sQ1[BN * BK];

  // ---- block -> (matrix, tile): XCD-contiguous numbering, then 4-row raster bands
  const int tiles_n = static_cast<int>(d.N / BN);
  const int tiles_m = static_cast<int>(d.M / BM);
  const int per_batch = tiles_m * tiles_n;
  int logical;
  {
    const int nblocks = gridDim.x, bid = blockIdx.x;
    const int per = nblocks / N_XCD, rem = nblocks % N_XCD;
    const int xcd = bid % N_XCD, q = bid / N_XCD;
    logical = xcd < rem ? xcd * (per + 1) + q : rem * (per + 1) + (xcd - rem) * per + q;
  }
  const int b = logical / per_batch;
  const int tix = logical - b * per_batch;
  int tm, tn;
  {
    const int band = tix / (GROUP_M * tiles_n);
    const int in_band = tix - band * GROUP_M * tiles_n;
    const int rows_here = min(GROUP_M, tiles_m - band * GROUP_M);
    tn = in_band / rows_here;
    tm = band * GROUP_M + (in_band - tn * rows_here);
  }

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const __bf16* Pg = P + static_cast<int64_t>(b) * d.sp + static_cast<int64_t>(tm) * BM * d.ldp;
  const __bf16* Qg = Q + static_cast<int64_t>(b) * d.sq + static_cast<int64_t>(tn) * BN * d.ldq;

  // ---- global -> LDS: wavefront w fills rows w*8 + 32*g .. +7 (g = 0..7) of both panels;
  //      lane l lands at row (l / 8), slot (l % 8) and therefore fetches chunk slot ^ swizzle.
  const int r8 = lane >> 3, slot = lane & 7;
  const int chunk = slot ^ (((wave & 1) << 2) | (r8 >> 1));
  const __bf16* pl = Pg + static_cast<int64_t>(wave * 8 + r8) * d.ldp + chunk * 8;
  const __bf16* ql = Qg + static_cast<int64_t>(wave * 8 + r8) * d.ldq + chunk * 8;
  const int64_t p_step = 32 * d.ldp, q_step = 32 * d.ldq;
  // one of the 16 direct loads of a stage: idx 0..7 -> P rows, 8..15 -> Q rows
  auto fetch_one = [&](__bf16* sP, __bf16* sQ, int64_t k0, int idx) {
    const int g = idx & 7;
    if (idx < 8)
      __builtin_amdgcn_global_load_lds(CANZ_GLB(pl + g * p_step + k0), CANZ_LDS(sP + (wave * 8 + g * 32) * BK), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds(CANZ_GLB(ql + g * q_step + k0), CANZ_LDS(sQ + (wave * 8 + g * 32) * BK), 16, 0, 0);
  };
  auto fetch = [&](__bf16* sP, __bf16* sQ, int64_t k0) {
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) fetch_one(sP, sQ, k0, idx);
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // MFMA operand fragments, double-buffered in registers: idx 0..3 -> rows of P, 4..7 -> rows of Q
  const int frag_row = lane & 31, frag_kg = lane >> 5;
  bf16x8 fa[2][4], fb[2][4];
  auto frag_one = [&](const __bf16* sP, const __bf16* sQ, int kk, int set, int idx) {
    if (idx < 4)
      fa[set][idx] = *reinterpret_cast<const bf16x8*>(sP + swz(wm * 128 + idx * 32 + frag_row, kk * 2 + frag_kg));
    else
      fb[set][idx - 4] =
          *reinterpret_cast<const bf16x8*>(sQ + swz(wn * 128 + (idx - 4) * 32 + frag_row, kk * 2 + frag_kg));
  };
  auto load_frags = [&](const __bf16* sP, const __bf16* sQ, int kk, int set) {
#pragma unroll
    for (int idx = 0; idx < 8; ++idx) frag_one(sP, sQ, kk, set, idx);
  };
  auto mma_one = [&](int set, int idx) {
    const int i = idx >> 2, j = idx & 3;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
  };

  const int nk = static_cast<int>(d.K / BK);  // even: K is a multiple of 256
  // The issue order below is pinned with scheduling fences.  A wavefront issues in order and
  // an MFMA occupies the matrix pipe for 32 cycles, so every other instruction is placed in
  // the shadow of one MFMA: one LDS operand load or one direct global->LDS load per MFMA.
  // Left to itself the compiler clusters the loads and the matrix pipe drains meanwhile.
#define CANZ_FENCE() __builtin_amdgcn_sched_barrier(0)
  // one k-step on stage (cP, cQ); the other stage (nP, nQ) holds step kt + 1.  The fetch
  // index is clamped instead of guarded (a branch here costs the compiler its knowledge of
  // which stage is in flight); the last two steps refetch the final panel into stages
  // nobody reads any more.
  auto k_step = [&](__bf16* cP, __bf16* cQ, const __bf16* nP, const __bf16* nQ, int kt) {
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) {
#pragma unroll
      for (int idx = 0; idx < 16; ++idx) {
        mma_one(kk & 1, idx);
        CANZ_FENCE();
        if (idx < 8) {
          frag_one(cP, cQ, kk + 1, (kk + 1) & 1, idx);  // lands under the 8 MFMAs that follow
          CANZ_FENCE();
        }
      }
    }
    __syncthreads();  // step kt+1 has landed everywhere; nobody reads (cP, cQ) any more
    const int64_t k2 = static_cast<int64_t>(min(kt + 2, nk - 1)) * BK;
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) {
      mma_one(1, idx);
      CANZ_FENCE();
      fetch_one(cP, cQ, k2, idx);
      CANZ_FENCE();
      if (idx < 8) {
        frag_one(nP, nQ, 0, 0, idx);
        CANZ_FENCE();
      }
    }
  };

  fetch(sP0, sQ0, 0);
  __syncthreads();
  fetch(sP1, sQ1, BK);
  load_frags(sP0, sQ0, 0, 0);
  for (int kt = 0; kt < nk; kt += 2) {
    k_step(sP0, sQ0, sP1, sQ1, kt);
    k_step(sP1, sQ1, sP0, sQ0, kt + 1);
  }
  __syncthreads();  // drains the clamped tail fetches before the block may retire
#undef CANZ_FENCE

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
      if (EPI == EPI_FINAL) {
        // the host orders the operands so that (row, col) is the caller's orientation
        float v[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = acc[i][j][r] * sc;
        store_out_tile(o, s, b, row_base + i * 32, col, v);
        continue;
      }
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
          float av[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) av[q] = static_cast<float>(A[static_cast<int64_t>(row0 + q) * d.N + col]);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float r = e.cb * av[q] + e.cc * v[q];
            if (row0 + q == col) r += e.ca;
            C[static_cast<int64_t>(row0 + q) * d.N + col] = static_cast<__bf16>(r);
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

hipError_t launch_final_bf16(const GemmDims& d, const void* p, const void* q, const float* scale, const Shape& s,
                             const OutSpec& o, hipStream_t st) {
  EpiArgs e{};
  e.scale = scale;
  return launch<EPI_FINAL>(d, p, q, e, s, o, st);
}

}  // namespace canz
