// fp32 products on v_mfma_f32_32x32x2_f32, shared by the Shampoo and SOAP steps (internal).
//
// All products have the form C[i][j] = sum_k P[i][k] Q[j][k] with both operands contiguous
// along k.  A product whose natural form is different is brought to this one by choosing
// which factor is P and which is Q (which decides whether C or its transpose is written) and
// by keeping the operands in the orientation their consumer needs.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "canz.h"
#include "device_util.h"
#include "kernels.h"

namespace canz {
namespace f32mfma {

constexpr int SB = 128;          // block tile (rows and columns)
constexpr int SK = 32;           // k extent of one LDS stage: long enough that the next stage's global loads land under it
constexpr int NTH = 256;
constexpr int LDS_LD = SB + 5;   // odd row length: the k-major stores of a stage spread over all banks
constexpr int FLUSH = 16;        // stages (512 k) between folds of the running accumulator
constexpr size_t ALIGN = 256;

inline int64_t pad128(int64_t x) { return (x + SB - 1) / SB * SB; }
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Epilogues: SE_STAT  S <- beta S + gscale C into the caller's dense statistic, S + eps I to c;
//            SE_PLAIN c = C;   SE_MT  c = C and c2 = 5/4 I - 1/4 C;   SE_OUT  the optimizer update
//            into the caller's parameters or Delta W fragments;   SE_SUB  c <- c - C.
enum { SE_STAT = 0, SE_PLAIN = 1, SE_MT = 2, SE_OUT = 3, SE_SUB = 4 };

struct ShGemm {
  int64_t M, N, K;      // multiples of 128, 128, 32
  int64_t ldp, ldq;     // row strides of P [M][K] and Q [N][K]
  int64_t sp, sq;       // batch strides: matrix b reads P + (b / pdiv) sp and Q + (b / qdiv) sq
  int pdiv, qdiv;       // 0 means 1; 2 lets two consecutive problems share an operand
  const float* P;
  const float* Q;
  float* c;             // output
  int64_t ldc, sc;      // its row and batch strides; 0, 0 means dense: N and M * N
  float* c2;            // SE_MT: the next T = 5/4 I - 1/4 C (strides as c)
  // SE_STAT: the caller's statistic (d x d, dense) is updated in place and A = S + eps I is written to c
  int64_t d;
  float beta, gscale, eps;
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

// BN = 128: 128 x 128 tiles, each wavefront a 64 x 64 quarter.  BN = 32 (for products whose N is 32, the
// width of a QR panel): 128 x 32 tiles, each wavefront a 32 x 32 block of rows.
template <int EPI, bool SYM, int BN>
__device__ __forceinline__ void sh_gemm_body(const ShGemm& g, const PtrTable& stat, const Shape& s, const OutSpec& o) {
  static_assert(BN == SB || (BN == 32 && !SYM), "tile widths: 128, or 32 for plain products");
  constexpr int NI = BN == SB ? 2 : 1;   // 32 x 32 MFMA tiles per wavefront, along M and along N
  constexpr int QX = BN / 32;            // 32-row groups of the Q tile
  __shared__ float sP[2][SK][LDS_LD];  // k-major: the lanes of one MFMA operand read consecutive rows
  __shared__ float sQ[2][SK][LDS_LD];

  const int tiles_m = static_cast<int>(g.M / SB), tiles_n = static_cast<int>(g.N / BN);
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
  const int wm = BN == SB ? wave >> 1 : wave, wn = BN == SB ? wave & 1 : 0;
  const float* Pg = g.P + static_cast<int64_t>(b / g.pdiv) * g.sp + static_cast<int64_t>(tm) * SB * g.ldp;
  const float* Qg = g.Q + static_cast<int64_t>(b / g.qdiv) * g.sq + static_cast<int64_t>(tn) * BN * g.ldq;

  const int ld_row = t >> 3, ld_k = (t & 7) * 4;  // rows ld_row + 32 x (x = 0..3), 4 consecutive k
  // Long sums of the statistics (k up to the other extent of the matrix, terms of one sign on the
  // diagonal) are folded into a second accumulator every FLUSH stages; the products of the root
  // iteration and the preconditioning accumulate in one go (their rounding, about 1e-5 relative,
  // is corrected by the following rounds and is far below the tolerance of the update).
  constexpr bool FOLD = EPI == SE_STAT;
  f32x16 acc[NI][NI], tot[NI][NI];
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
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
      if (x < QX) qv[set][x] = *reinterpret_cast<const f32x4*>(Qg + static_cast<int64_t>(ld_row + 32 * x) * g.ldq + k0);
    }
  };
  auto stash = [&](int buf, int set) {
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        sP[buf][ld_k + c][ld_row + 32 * x] = pv[set][x][c];
        if (x < QX) sQ[buf][ld_k + c][ld_row + 32 * x] = qv[set][x][c];
      }
  };
  // one stage: LDS buffer `buf` holds stage kt, register set `other` stage kt + 1, set `mine` is free
  const int nk = static_cast<int>(g.K / SK);   // >= 1
  auto stage = [&](int kt, int buf, int mine, int other) {
    if (kt + 2 < nk) fetch(kt + 2, mine);
#pragma unroll
    for (int k = 0; k < SK; k += 2) {
      float fa[NI], fb[NI];
#pragma unroll
      for (int i = 0; i < NI; ++i) fa[i] = sP[buf][k + (lane >> 5)][wm * 32 * NI + i * 32 + (lane & 31)];
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j] = sQ[buf][k + (lane >> 5)][wn * 64 + j * 32 + (lane & 31)];
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (FOLD && ((kt + 1) % FLUSH == 0 || kt + 1 == nk)) {
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) tot[i][j][r] += acc[i][j][r], acc[i][j][r] = 0.f;
    }
    if (kt + 1 < nk) stash(buf ^ 1, other);
    __syncthreads();  // stage kt + 1 is complete in LDS; every wavefront is done reading stage kt
  };
  fetch(0, 0);
  if (nk > 1) fetch(1, 1);
  stash(0, 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {   // pairs of stages without a test between them: the two halves schedule as one body
    stage(kt, 0, 0, 1);
    stage(kt + 1, 1, 1, 0);
  }
  if (kt < nk) stage(kt, 0, 0, 1);   // odd stage count (k = 32 (2 j + 1)): only the products of a QR panel
  if (!FOLD) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) tot[i][j] = acc[i][j];
  }

  const int row_base = tm * SB + wm * 32 * NI + 4 * (lane >> 5);
  const int col_base = tn * BN + wn * 64 + (lane & 31);
  const bool mirror = SYM && tm != tn;
  const int64_t cb = static_cast<int64_t>(b) * g.sc;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int row0 = row_base + i * 32, col = col_base + j * 32;
      float v[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = tot[i][j][r];
      if (EPI == SE_OUT) {
        store_out_tile(o, s, b, row0, col, v);
      } else if (EPI == SE_PLAIN) {
        put16(g.c + cb, g.ldc, row0, col, v, mirror);
      } else if (EPI == SE_SUB) {
        float* C = g.c + cb;
        float old[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) old[r] = C[static_cast<int64_t>(row0 + 8 * (r >> 2) + (r & 3)) * g.ldc + col];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = old[r] - v[r];
        put16(C, g.ldc, row0, col, v, false);
      } else if (EPI == SE_MT) {
        put16(g.c + cb, g.ldc, row0, col, v, mirror);
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = (row0 + 8 * (r >> 2) + (r & 3) == col ? 1.25f : 0.f) - 0.25f * v[r];
        put16(g.c2 + cb, g.ldc, row0, col, v, mirror);
      } else {  // SE_STAT
        float* S = static_cast<float*>(stat.p[b]);
        const int d = static_cast<int>(g.d);
        // all old values are requested before the first store, so that the 16 read-modify-writes overlap
        // instead of running as a chain of dependent memory round trips
        float old[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + 8 * (r >> 2) + (r & 3);
          old[r] = g.beta != 0.f && row < d && col < d ? S[static_cast<int64_t>(row) * d + col] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + 8 * (r >> 2) + (r & 3);
          float val = 0.f;
          if (row < d && col < d) {
            const int64_t at = static_cast<int64_t>(row) * d + col;
            val = g.gscale * v[r];
            if (g.beta != 0.f) val += g.beta * old[r];
            S[at] = val;
            if (mirror) S[static_cast<int64_t>(col) * d + row] = val;
            if (row == col) val += g.eps;
          }
          v[r] = val;
        }
        if (g.c == nullptr) continue;   // the padded copy is only wanted when something reads it
        put16(g.c + cb, g.ldc, row0, col, v, mirror);
      }
    }
  }
}

template <int EPI, bool SYM, int BN = SB>
__global__ __launch_bounds__(NTH) void k_sh_gemm(ShGemm g, PtrTable stat, Shape s, OutSpec o) {
  sh_gemm_body<EPI, SYM, BN>(g, stat, s, o);
}
// The statistics variant carries a second set of accumulators; left to itself the register allocator takes
// more than half of a SIMD's registers for it, which leaves one block per CU and nothing to cover its
// barriers and epilogue with (MFMA pipe 40 % busy).  Held to two wavefronts per SIMD it fits without spills.
// The other variants are left alone: under the same limit they lose their AGPR accumulators and 5 % of their rate.
template <int EPI, bool SYM, int BN = SB>
__global__ __launch_bounds__(NTH) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_sh_gemm_2w(ShGemm g, PtrTable stat, Shape s,
                                                                                             OutSpec o) {
  sh_gemm_body<EPI, SYM, BN>(g, stat, s, o);
}

template <int EPI, bool SYM, int BN = SB>
hipError_t launch_gemm(ShGemm g, int nb, const PtrTable& stat, const Shape& s, const OutSpec& o, hipStream_t st) {
  if (g.M < SB || g.N < BN || g.K < SK || g.M % SB || g.N % BN || g.K % SK || (SYM && g.M != g.N)) return hipErrorInvalidValue;
  if (g.ldc == 0) g.ldc = g.N, g.sc = g.M * g.N;
  if (g.pdiv == 0) g.pdiv = 1;
  if (g.qdiv == 0) g.qdiv = 1;
  const int64_t tm = g.M / SB, tn = g.N / BN;
  const int64_t blocks = (SYM ? tm * (tm + 1) / 2 : tm * tn) * nb;
  if constexpr (EPI == SE_STAT)
    hipLaunchKernelGGL((k_sh_gemm_2w<EPI, SYM, BN>), dim3(static_cast<unsigned>(blocks)), dim3(NTH), 0, st, g, stat, s, o);
  else
    hipLaunchKernelGGL((k_sh_gemm<EPI, SYM, BN>), dim3(static_cast<unsigned>(blocks)), dim3(NTH), 0, st, g, stat, s, o);
  return hipGetLastError();
}

// G (bf16 or fp32, whole or tp column fragments) -> fp32 working copies in both orientations,
// zero outside rows x cols.  One block per 64 x 64 tile; the transposed copy goes through LDS.
static __global__ __launch_bounds__(NTH) void k_sh_load(Shape s, PtrTable grad, int grad_dtype, int64_t rp, int64_t cp,
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

// dense rows x cols matrices of the caller <- the padded working copies src[b * stride] (row length cp)
static __global__ __launch_bounds__(NTH) void k_unpad(Shape s, PtrTable dst, const float* __restrict__ src, int64_t stride,
                                                     int64_t cp) {
  const int b = blockIdx.z, r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
  const float* from = src + static_cast<int64_t>(b) * stride;
  float* to = static_cast<float*>(dst.p[b]);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int idx = e * NTH + t, row = r0 + (idx >> 6), col = c0 + (idx & 63);
    if (row < s.rows && col < s.cols) to[static_cast<int64_t>(row) * s.cols + col] = from[static_cast<int64_t>(row) * cp + col];
  }
}

}  // namespace f32mfma
}  // namespace canz
