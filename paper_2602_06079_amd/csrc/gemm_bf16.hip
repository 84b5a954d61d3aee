// Batched bf16 MFMA GEMMs of the Newton-Schulz iteration (step 4 of the operator):
//   C[b][i][j] = sum_k P[b][i][k] * Q[b][j][k]        fp32 accumulate
// Both operands are contiguous along k (see kernels.h for why both orientations of X are
// kept), which is the lane layout v_mfma_f32_32x32x16_bf16 wants: lane l supplies 8
// consecutive k of row (l % 32), k-group (l / 32).  Operands and bf16 results live in the
// panel layout of panel_layout.h.
//
// Tiling: one 256-thread block (4 wavefronts, 2 x 2) owns a 256 x 256 tile of C; each
// wavefront owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256 fp32 accumulators per lane (one
// wavefront per SIMD, 512 registers each).  K is walked in steps of 32.
//
// Operand staging: a 256 x 32 panel is 16 KiB of contiguous memory that already has the
// bank-conflict-free LDS arrangement, so it goes from global memory straight into LDS as
// a linear copy (global_load_lds_dwordx4: a wavefront moves 1 KiB per instruction), into
// one of four 32 KiB stages (P panel + Q panel).
//
// Pipeline: moving 32 KiB per k-step from L2 into LDS takes about as long as the 32 MFMAs
// of the step, and a fetch needs more than a microsecond to land, so the ring is four
// stages deep: while step t is multiplied, steps t+1 .. t+3 are resident or in flight and
// step t+4 is being requested.  The MFMA operand fragments are double-buffered in
// registers.  A wavefront issues in order and an MFMA keeps the matrix pipe busy for 32
// cycles, so every other instruction is placed in the shadow of one MFMA: one LDS operand
// load after each of the first 8 MFMAs of a half-step, one direct load after every
// fourth.  One barrier per k-step, between its two half-steps: before it each wavefront
// waits for its own share of step t+1 (s_waitcnt vmcnt(16): the 16 younger loads of steps
// t+2 and t+3 may stay in flight); after it stage t is free for step t+4.
//
// Epilogue: the accumulators are re-arranged through LDS (free after the last step) into
// panel-layout images, one per wavefront, and leave as linear 16-byte-per-lane stores; the
// last product of the chain instead stages fp32 rows and applies the parameter update
// with 16-byte accesses on the caller's row-major buffers.
//
// Blocks are persistent (one per CU) and loop over tiles, so the stores of one tile's
// epilogue drain while the next tile is multiplied.  In every round the 32 blocks of one XCD
// (blockIdx % 8 selects the XCD) form a 4 x 8 patch of tiles of one matrix and share panels
// in that XCD's L2.
// Symmetric products (Gram, polynomial) run only the tiles on or above the diagonal and
// write the mirror image as well.  Extents are multiples of 256 (zero padded by the
// producer), so only the final epilogue clips to the caller's shape.
#include <algorithm>
#include <type_traits>

#include "device_util.h"
#include "panel_layout.h"

namespace canz {
namespace {

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int NTHREADS = 256;
constexpr int CHUNKS = BK / 8;   // 16-byte chunks per panel row
constexpr int GROUP_M = 4;       // tile rows per raster band
constexpr int N_XCD = 8;
static_assert(BM == PANEL_ROWS && BK == PANEL_K, "tile = panel");

enum { EPI_GRAM = 0, EPI_POLY = 1, EPI_UPDATE = 2, EPI_FINAL = 3, EPI_FINAL_SYM = 4 };
// EPI_FINAL_SYM: the last-product epilogue (the caller's dense buffers) over the tiles on and above the diagonal of a
// symmetric result only; the caller mirrors them into the lower triangle afterwards.
constexpr bool epi_symmetric(int epi) { return epi == EPI_GRAM || epi == EPI_POLY || epi == EPI_FINAL_SYM; }
constexpr bool epi_final(int epi) { return epi == EPI_FINAL || epi == EPI_FINAL_SYM; }

struct EpiArgs {
  void* c;                 // GRAM/POLY: [nb][M][N] panels; UPDATE: straight output [nb][M][N] panels
  void* ct;                // UPDATE: transposed output [nb][N][M] panels
  const void* aux;         // POLY: A [nb][M][N] panels
  const float* scale;      // per-matrix factor applied to the accumulator, or nullptr
  float ca, cb, cc;        // POLY coefficients
  // schedule of the persistent blocks (see launch()): full rounds of whole tiles, then the
  // `left` remaining tiles, each cut into `splits` k-slices that different blocks compute
  int full_rounds, left, splits, main_grid;
  float* partial;          // [gridDim][256 regs][256 threads] fp32 accumulators of the k-slices
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define CANZ_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define CANZ_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ int swz(int row, int chunk) {
  return (row * CHUNKS + (chunk ^ ((row >> 2) & (CHUNKS - 1)))) * 8;  // element offset in the panel
}

// value of the neighbouring lane (lane ^ 1), through the DPP quad permute [1, 0, 3, 2]
__device__ __forceinline__ unsigned lane_xor1(unsigned v) {
  return static_cast<unsigned>(__builtin_amdgcn_mov_dpp(static_cast<int>(v), 0xB1, 0xF, 0xF, false));
}

// logical tile index -> (matrix b, tile row tm, tile column tn)
template <int EPI>
__device__ __forceinline__ void decode_tile(int logical, int tiles_m, int tiles_n, int per_batch, int& b, int& tm,
                                            int& tn) {
  b = logical / per_batch;
  const int tix = logical - b * per_batch;
  if (epi_symmetric(EPI)) {
    // symmetric output: only tiles with tn >= tm exist (per_batch = nt (nt + 1) / 2); the
    // epilogue writes each off-diagonal tile twice, straight and mirrored.  Raster: bands of
    // 4 tile rows; inside the band starting at r0 the columns r0, r0+1, ... are walked one
    // after the other, column c holding the rows r0 .. min(r0 + 3, c).
    int rem = tix, band = 0;
    for (;;) {
      const int rows = min(GROUP_M, tiles_m - band * GROUP_M), cols = tiles_m - band * GROUP_M;
      const int cnt = rows * cols - rows * (rows - 1) / 2;
      if (rem < cnt) break;
      rem -= cnt;
      ++band;
    }
    const int r0 = band * GROUP_M;
    const int rows = min(GROUP_M, tiles_m - r0);
    const int tri = rows * (rows + 1) / 2;
    if (rem < tri) {
      int c = 0;
      while (rem >= c + 1) rem -= c + 1, ++c;
      tn = r0 + c;
      tm = r0 + rem;
    } else {
      rem -= tri;
      tn = r0 + rows + rem / rows;
      tm = r0 + rem % rows;
    }
  } else {
    // bands of 4 tile rows, walked column by column
    const int band = tix / (GROUP_M * tiles_n);
    const int in_band = tix - band * GROUP_M * tiles_n;
    const int rows_here = min(GROUP_M, tiles_m - band * GROUP_M);
    tn = in_band / rows_here;
    tm = band * GROUP_M + (in_band - tn * rows_here);
  }

}

// Epilogue of one 256 x 256 tile held in the accumulators of the block's four wavefronts
// (shared by the GEMM kernel and by the kernel that finishes k-split tiles).
// `stage`: this wavefront's private 32 KiB of LDS.
template <int EPI>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[4][4], __bf16* stage, int lane, int wm, int wn, int b,
                                              int tm, int tn, const GemmDims& d, const EpiArgs& e, const Shape& s,
                                              const OutSpec& o) {
  // ---- epilogue.  Accumulator register r of lane l in MFMA tile (it, jt) is element
  //      row = 32 it + 8 (r / 4) + 4 (l / 32) + (r % 4),  col = 32 jt + (l % 32)
  //      of the wavefront's 128 x 128 part.  Each wavefront stages through its own 32 KiB.
  const int lj = lane & 31, lh = lane >> 5;

  // scale (first iteration: folded normalisation), or the polynomial in A for EPI_POLY
  if (EPI == EPI_POLY) {
    // A is symmetric bit for bit (the Gram epilogue writes both halves from the same
    // accumulators), so element (i, j) is read as (j, i): the wavefront's part of the mirrored
    // tile is copied linearly into its staging area (global -> LDS, 16 bytes per lane) and is
    // then the transposed image, in which a lane's four consecutive rows are four consecutive k.
    const __bf16* A = static_cast<const __bf16*>(e.aux) + static_cast<int64_t>(b) * d.M * d.N;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      const __bf16* src = A + (static_cast<int64_t>(tn) * (d.M >> 5) + 8 * tm + 4 * wm + kb) * PANEL_ELEMS +
                          wn * 128 * PANEL_K + lane * 8;
#pragma unroll
      for (int x = 0; x < 8; ++x)
        __builtin_amdgcn_global_load_lds(CANZ_GLB(src + x * 512), CANZ_LDS(stage + kb * 4096 + x * 512), 16, 0, 0);
    }
    int a_base[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) a_base[g] = lj * 32 + ((g ^ ((lj >> 2) & 3)) << 3) + 4 * lh;
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0): the copy has landed
#pragma unroll
    for (int it = 0; it < 4; ++it)
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) {
        const int col = tn * BN + wn * 128 + jt * 32 + lj;
        const int row0 = tm * BM + wm * 128 + it * 32 + 4 * lh;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const bf16x4 av = *reinterpret_cast<const bf16x4*>(stage + it * 4096 + jt * 32 * 32 + a_base[g]);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            acc[it][jt][4 * g + q] =
                poly_value(static_cast<float>(av[q]), acc[it][jt][4 * g + q], e.ca, e.cb, e.cc, row0 + 8 * g + q == col);
          }
        }
      }
    // every read of the staging area is done before the images below overwrite it
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  } else if (e.scale) {
    const float sc = e.scale[b];
#pragma unroll
    for (int it = 0; it < 4; ++it)
#pragma unroll
      for (int jt = 0; jt < 4; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[it][jt][r] *= sc;
  }

  // the wavefront's part of an output tile in panel layout: four pieces of 8 KiB (the four
  // 32-wide k-blocks it covers), 128 rows each; LDS image == memory image
  auto flush_stage = [&](__bf16* out, int64_t row_block, int64_t kc, int64_t kblock0, int half_rows) {
    // out: matrix base; the wavefront's rows start at row_block * 256 + half_rows * 128
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      __bf16* dst = out + (row_block * (kc >> 5) + kblock0 + kb) * PANEL_ELEMS + half_rows * 128 * PANEL_K;
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(stage + kb * 4096 + (x * 64 + lane) * 8);
        *reinterpret_cast<u32x4*>(dst + (x * 64 + lane) * 8) = v;
      }
    }
  };

  if (!epi_final(EPI)) {
    // ---- straight image: element (i, j) of C is (row i, k = j) of the result's panels.
    // A 16-byte chunk is 8 consecutive j of one row, i.e. one value from each of 8 lanes:
    // neighbouring lanes exchange their packed pairs so that every lane writes two bf16 of
    // one row.
    __bf16* C = static_cast<__bf16*>(e.c) + static_cast<int64_t>(b) * d.M * d.N;
    // Staging offset = (lane-only base) + (compile-time part), so that the compiler keeps two
    // address registers instead of one per store.  Element (row_l, col_l) of the wavefront's
    // part, row_l = 32 it + 8 g + 2 p + 4 lh + odd (rp = 2 g + p), col_l = 32 jt + lj, lies in
    // k-block jt at row_l * 32 + ((chunk ^ swizzle) << 3) with chunk = lj >> 3 and
    // swizzle = (row_l >> 2) & 3 = 2 (g & 1) + lh: lane bits except for g & 1.
    // byte selector of v_perm_b32 over {theirs (bytes 4..7), mine (bytes 0..3)}
    const unsigned pair_sel = (lane & 1) ? 0x03020706u : 0x05040100u;
    int s_base[2];
#pragma unroll
    for (int g1 = 0; g1 < 2; ++g1)
      s_base[g1] = (4 * lh + (lane & 1)) * 32 + ((((lj >> 3) ^ (2 * g1 + lh)) & 3) << 3) + (lj & 6);
#pragma unroll
    for (int it = 0; it < 4; ++it)
#pragma unroll
      for (int jt = 0; jt < 4; ++jt)
#pragma unroll
        for (int rp = 0; rp < 8; ++rp) {  // register pairs (2 rp, 2 rp + 1): rows differ by one
          // both rows of this lane's column, packed; the even lane keeps the low halves of
          // the pair of lanes (row 2 rp), the odd lane the high halves (row 2 rp + 1)
          bf16x2 own;
          own[0] = static_cast<__bf16>(acc[it][jt][2 * rp]);
          own[1] = static_cast<__bf16>(acc[it][jt][2 * rp + 1]);
          const unsigned mine = __builtin_bit_cast(unsigned, own);
          const unsigned theirs = lane_xor1(mine);
          const unsigned pk = __builtin_amdgcn_perm(theirs, mine, pair_sel);
          const int g = rp >> 1, p = rp & 1;
          const int fixed = jt * 4096 + (it * 32 + 8 * g + 2 * p) * 32;
          *reinterpret_cast<unsigned*>(stage + fixed + s_base[g & 1]) = pk;
        }
    flush_stage(C, tm, d.N, 8 * tn + 4 * wn, wm);

    // ---- transposed image: element (i, j) is (row j, k = i) of CT (UPDATE) or of the mirror
    // tile of C (symmetric products).  A lane's 4 consecutive rows are half a chunk.
    const bool mirror = (EPI == EPI_GRAM || EPI == EPI_POLY);
    if (!mirror || tm != tn) {
      __bf16* CT = mirror ? C : static_cast<__bf16*>(e.ct) + static_cast<int64_t>(b) * d.M * d.N;
      // element (i_l, j_l) goes to row j_l = 32 jt + lj, k = i_l = 32 it + 8 g + 4 lh + q:
      // k-block it, chunk g, swizzle (lj >> 2) & 3: one lane base per g, the rest immediate
      int t_base[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) t_base[g] = lj * 32 + ((g ^ ((lj >> 2) & 3)) << 3) + 4 * lh;
#pragma unroll
      for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            bf16x4 pk;
#pragma unroll
            for (int q = 0; q < 4; ++q) pk[q] = static_cast<__bf16>(acc[it][jt][4 * g + q]);
            *reinterpret_cast<bf16x4*>(stage + it * 4096 + jt * 32 * 32 + t_base[g]) = pk;
          }
      flush_stage(CT, tn, d.M, 8 * tm + 4 * wm, wn);
    }
  } else {
    // ---- last product: O in the caller's orientation (the host orders the operands so).
    const int ld = static_cast<int>(o.out_mode == CANZ_OUT_DELTA ? s.wfrag : s.cols);
    if ((ld & 3) == 0) {
      // fp32 rows through LDS, 64 rows x 128 columns at a time; the column index is XOR-ed
      // with 32 on rows whose bit 2 is set so that the two half-waves hit different banks.
      // One instantiation per (output mode, output dtype): the branches stay outside the
      // unrolled code.
      auto run = [&](auto mode_tag, auto dtype_tag) {
        constexpr int MODE = decltype(mode_tag)::value, DTYPE = decltype(dtype_tag)::value;
        float* sf = reinterpret_cast<float*>(stage);
        int f_base[2], r_base[2];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          f_base[p] = 4 * lh * 128 + lj + 32 * (p ^ lh);
          r_base[p] = lh * 128 + ((lj * 4) ^ (p << 5));
        }
        // per-lane element offset of (row 0 of the wavefront's part, its 4 columns) in the
        // caller's buffer, and the buffer itself (TP: the fragment that holds these columns)
        const int col = tn * BN + wn * 128 + lj * 4;
        const bool col_ok = col < s.cols;
        int c_in = col, tab = b;
        if (MODE == CANZ_OUT_DELTA) {
          const int f = col_ok ? col / ld : 0;
          c_in = col - f * ld;
          tab = b * s.tp + f;
        }
        char* base = static_cast<char*>(o.out.p[col_ok ? tab : b * (MODE == CANZ_OUT_DELTA ? s.tp : 1)]);
        constexpr int ESZ = DTYPE == CANZ_DT_F32 ? 4 : 2;
        // whole 128 x 128 part inside the matrix (uniform over the wavefront): no predicates
        const bool inside = tm * BM + wm * 128 + 128 <= s.rows && tn * BN + wn * 128 + 128 <= s.cols;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const int row_base = tm * BM + wm * 128 + half * 64 + lh;
          auto stage_half = [&]() {
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
              for (int jt = 0; jt < 4; ++jt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                  // (32 jt + lj) ^ (32 lh) = lj + 32 (jt ^ lh): lane base per parity of jt
                  const int fixed = (i2 * 32 + 8 * (r >> 2) + (r & 3)) * 128 + (jt & ~1) * 32;
                  sf[fixed + f_base[jt & 1]] = acc[half * 2 + i2][jt][r];
                }
          };
          if (inside) {
            // The lane handles 4 columns of the 32 rows row_base + 2 i.  All old values of the
            // half are requested at once and every one of them is consumed before the first
            // store is issued: the half then costs one memory latency (with loads and stores
            // interleaved, each group of rows would wait for the stores of the one before).
            char* const ptr0 = base + (static_cast<int64_t>(row_base) * ld + c_in) * ESZ;
            const int64_t pitch2 = static_cast<int64_t>(2) * ld * ESZ;
            f32x4 val[32];
            if (MODE == CANZ_OUT_PARAM) {
#pragma unroll
              for (int i = 0; i < 32; ++i) {
                if (DTYPE == CANZ_DT_F32) {
                  val[i] = *reinterpret_cast<const f32x4*>(ptr0 + i * pitch2);
                } else {
                  const bf16x4 ob = *reinterpret_cast<const bf16x4*>(ptr0 + i * pitch2);
#pragma unroll
                  for (int q = 0; q < 4; ++q) val[i][q] = static_cast<float>(ob[q]);
                }
              }
            }
            __builtin_amdgcn_sched_barrier(0);
            stage_half();
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 32; ++i) {
              // row 2 i + lh of the staged half; bit 2 of that row is bit 1 of i
              const f32x4 v = *reinterpret_cast<const f32x4*>(sf + 2 * i * 128 + r_base[(i >> 1) & 1]);
#pragma unroll
              for (int q = 0; q < 4; ++q)
                val[i][q] = MODE == CANZ_OUT_PARAM ? apply_update(val[i][q], o.decay, o.neg_lr_scale, v[q])
                                                   : o.neg_lr_scale * v[q];
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 32; ++i) {
              if (DTYPE == CANZ_DT_F32) {
                *reinterpret_cast<f32x4*>(ptr0 + i * pitch2) = val[i];
              } else {
                bf16x4 rb;
#pragma unroll
                for (int q = 0; q < 4; ++q) rb[q] = static_cast<__bf16>(val[i][q]);
                *reinterpret_cast<bf16x4*>(ptr0 + i * pitch2) = rb;
              }
            }
            __builtin_amdgcn_sched_barrier(0);
            continue;
          }
          // ragged edge of the matrix: rows and columns checked one by one, 4 rows at a time
          stage_half();
#pragma unroll
          for (int x4 = 0; x4 < 8; ++x4) {  // loads of old values first
            f32x4 v[4], old[4];
            char* ptr[4];
            bool live[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              // lane reads 4 columns of row 2 (4 x4 + u) + lh; bit 2 of that row is bit 1 of u
              v[u] = *reinterpret_cast<const f32x4*>(sf + 2 * (x4 * 4 + u) * 128 + r_base[(u >> 1) & 1]);
              const int row = row_base + 2 * (x4 * 4 + u);
              live[u] = col_ok && row < s.rows;
              ptr[u] = base + (static_cast<int64_t>(row) * ld + c_in) * ESZ;
            }
            if (MODE == CANZ_OUT_PARAM) {
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                if (!live[u]) continue;
                if (DTYPE == CANZ_DT_F32) {
                  old[u] = *reinterpret_cast<const f32x4*>(ptr[u]);
                } else {
                  const bf16x4 ob = *reinterpret_cast<const bf16x4*>(ptr[u]);
#pragma unroll
                  for (int q = 0; q < 4; ++q) old[u][q] = static_cast<float>(ob[q]);
                }
              }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if (!live[u]) continue;
              f32x4 res;
#pragma unroll
              for (int q = 0; q < 4; ++q)
                res[q] = MODE == CANZ_OUT_PARAM ? apply_update(old[u][q], o.decay, o.neg_lr_scale, v[u][q])
                                                : o.neg_lr_scale * v[u][q];
              if (DTYPE == CANZ_DT_F32) {
                *reinterpret_cast<f32x4*>(ptr[u]) = res;
              } else {
                bf16x4 rb;
#pragma unroll
                for (int q = 0; q < 4; ++q) rb[q] = static_cast<__bf16>(res[q]);
                *reinterpret_cast<bf16x4*>(ptr[u]) = rb;
              }
            }
          }
        }
      };
      using P_ = std::integral_constant<int, CANZ_OUT_PARAM>;
      using D_ = std::integral_constant<int, CANZ_OUT_DELTA>;
      using F_ = std::integral_constant<int, CANZ_DT_F32>;
      using B_ = std::integral_constant<int, CANZ_DT_BF16>;
      if (o.out_mode == CANZ_OUT_PARAM) {
        if (o.out_dtype == CANZ_DT_F32) run(P_{}, F_{}); else run(P_{}, B_{});
      } else {
        if (o.out_dtype == CANZ_DT_F32) run(D_{}, F_{}); else run(D_{}, B_{});
      }
    } else {
      // unaligned row length: element-wise stores straight from the accumulators
#pragma unroll
      for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
          float v[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) v[r] = acc[it][jt][r];
          store_out_tile(o, s, b, tm * BM + wm * 128 + it * 32 + 4 * lh, tn * BN + wn * 128 + jt * 32 + lj, v);
        }
    }
  }
}

// Operands of a launch: one product (the usual case), or several of different shapes.
struct OneProblem {
  static constexpr bool multi = false;
  GemmDims d;
  const __bf16* P;
  const __bf16* Q;
};
struct ManyProblems {
  static constexpr bool multi = true;
  int n;
  int begin[MAX_KINDS + 1];  // first logical tile of each problem, then the total
  GemmProblem pr[MAX_KINDS];
};

template <int EPI, bool SPLIT, typename Args>
__global__ __launch_bounds__(NTHREADS) void k_gemm_nt_bf16(Args args, EpiArgs e_launch, Shape s, OutSpec o) {
  // one array per stage (not one carved buffer): the compiler then knows that a fetch into
  // one stage does not alias the operand reads of another and keeps them overlapped.
  // Elements [0, 8192) hold the P panel, [8192, 16384) the Q panel.
  constexpr int QOFF = BM * BK;
  __shared__ __attribute__((aligned(1024))) __bf16 st0[(BM + BN) * BK];
  __shared__ __attribute__((aligned(1024))) __bf16 st1[(BM + BN) * BK];
  __shared__ __attribute__((aligned(1024))) __bf16 st2[(BM + BN) * BK];
  __shared__ __attribute__((aligned(1024))) __bf16 st3[(BM + BN) * BK];

  // ---- persistent blocks: the grid is one block per CU (or fewer); block `bid` works on the
  //      logical tiles round * gridDim + slot(bid).  slot() makes the 32 blocks of one XCD
  //      (blockIdx % 8 selects the XCD) neighbours, so that in every round they form a 4 x 8
  //      patch of tiles of one matrix and share panels in that XCD's L2.
  GemmDims d{};
  const __bf16 *P = nullptr, *Q = nullptr;
  EpiArgs e = e_launch;
  if constexpr (!Args::multi) d = args.d, P = args.P, Q = args.Q;
  int tiles_n = static_cast<int>(d.N / BN);
  int tiles_m = static_cast<int>(d.M / BM);
  int per_batch = epi_symmetric(EPI) ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  int slot;
  {
    const int nblocks = gridDim.x, bid = blockIdx.x;
    const int per = nblocks / N_XCD, rem = nblocks % N_XCD;
    const int xcd = bid % N_XCD, q = bid / N_XCD;
    slot = xcd < rem ? xcd * (per + 1) + q : rem * (per + 1) + (xcd - rem) * per + q;
  }

  const int t = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  int nk_all = static_cast<int>(d.K / BK);  // multiple of 8: K is a multiple of 256

  for (int work = 0;; ++work) {
  // ---- what to do in this round: a whole tile, or one k-slice of a left-over tile.  When
  //      the tiles do not fill the last round, each left-over tile is cut along k so that the
  //      whole chip shares them (second launch); the slices' accumulators are parked in global
  //      memory and k_split_finish adds them up and runs the epilogue.
  // SPLIT = false: persistent blocks over whole tiles (the full rounds, plus the left-over
  // tiles if they are not split).  SPLIT = true: a second launch in which every block
  // computes one k-slice of one left-over tile and parks its accumulators.
  int logical, k_begin = 0, nk = nk_all;
  if (!SPLIT) {
    const int rounds = e.full_rounds + (e.splits == 1 && slot < e.left ? 1 : 0);
    if (work >= rounds) break;
    logical = work * e.main_grid + slot;
  } else {
    if (work > 0) break;
    const int l = slot / e.splits, sl = slot - l * e.splits;
    logical = e.full_rounds * e.main_grid + l;
    const int groups = nk_all / 4, base = groups / e.splits, extra = groups % e.splits;
    k_begin = 4 * (sl * base + min(sl, extra));
    nk = 4 * (base + (sl < extra ? 1 : 0));
  }
  // The lane id is made opaque once per tile: otherwise every lane-dependent address of the
  // loop body (hundreds of them) is hoisted out of the tile loop and kept alive in scratch.
  int lane = t & 63;
  asm volatile("" : "+v"(lane));
  if constexpr (Args::multi) {
    // which product this tile belongs to; its extents, operands and outputs
    int j = 0;
    while (j + 1 < args.n && logical >= args.begin[j + 1]) ++j;
    const GemmProblem& pr = args.pr[j];
    d = pr.d;
    P = static_cast<const __bf16*>(pr.p), Q = static_cast<const __bf16*>(pr.q);
    e.c = pr.c, e.ct = pr.ct, e.aux = pr.aux, e.scale = pr.scale;
    logical -= args.begin[j];
    tiles_n = static_cast<int>(d.N / BN), tiles_m = static_cast<int>(d.M / BM);
    per_batch = epi_symmetric(EPI) ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
    nk_all = static_cast<int>(d.K / BK);
    nk = nk_all;
  }
  int b, tm, tn;
  decode_tile<EPI>(logical, tiles_m, tiles_n, per_batch, b, tm, tn);

  // ---- global -> LDS: panel (tile row, k-step) is 16 KiB contiguous; wavefront w copies the
  //      1 KiB pieces w, w+4, w+8, w+12 of both panels, lane l the 16 bytes at l * 16.
  const int64_t nkb = d.K / BK;
  const __bf16* pl = P + static_cast<int64_t>(b) * d.sp + (static_cast<int64_t>(tm) * nkb + k_begin) * PANEL_ELEMS + wave * 512 + lane * 8;
  const __bf16* ql = Q + static_cast<int64_t>(b) * d.sq + (static_cast<int64_t>(tn) * nkb + k_begin) * PANEL_ELEMS + wave * 512 + lane * 8;
  // one of the 8 direct loads of a stage: idx 0..3 -> P pieces, 4..7 -> Q pieces
  auto fetch_one = [&](__bf16* st, int64_t kt, int idx) {
    const int g = idx & 3;
    if (idx < 4)
      __builtin_amdgcn_global_load_lds(CANZ_GLB(pl + kt * PANEL_ELEMS + g * 2048), CANZ_LDS(st + wave * 512 + g * 2048), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds(CANZ_GLB(ql + kt * PANEL_ELEMS + g * 2048), CANZ_LDS(st + QOFF + wave * 512 + g * 2048), 16, 0, 0);
  };
  auto fetch = [&](__bf16* st, int64_t kt) {
#pragma unroll
    for (int idx = 0; idx < 8; ++idx) fetch_one(st, kt, idx);
  };

  // not cleared: the first 16 MFMAs of a tile take the constant 0 as their addend
  f32x16 acc[4][4];

  // MFMA operand fragments, double-buffered in registers: idx 0..3 -> rows of P, 4..7 -> rows of Q
  const int frag_row = lane & 31, frag_kg = lane >> 5;
  bf16x8 fa[2][4], fb[2][4];
  auto frag_one = [&](const __bf16* st, int kk, int set, int idx) {
    if (idx < 4)
      fa[set][idx] = *reinterpret_cast<const bf16x8*>(st + swz(wm * 128 + idx * 32 + frag_row, kk * 2 + frag_kg));
    else
      fb[set][idx - 4] =
          *reinterpret_cast<const bf16x8*>(st + QOFF + swz(wn * 128 + (idx - 4) * 32 + frag_row, kk * 2 + frag_kg));
  };
  auto mma_one = [&](auto first, int set, int idx) {
    const int i = idx >> 2, j = idx & 3;
    if (decltype(first)::value) {
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], zero, 0, 0, 0);
    } else {
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    }
  };

  // The issue order below is pinned with scheduling fences (left to itself the compiler
  // clusters the loads and the matrix pipe drains meanwhile).
#define CANZ_FENCE() __builtin_amdgcn_sched_barrier(0)
  // One k-step on stage `cur`; `nxt` holds step kt+1, `prv` (free since the barrier of the
  // previous step) receives the Q panel of step kt+3, `cur` after this step's barrier the P
  // panel of step kt+4.  The loads of the whole tile are issued in the order P0 Q0 P1 Q1 ...;
  // in the middle of step kt the youngest is Q(kt+3), so "all but the 16 youngest have
  // landed" means that step kt+1 is complete.  The last four steps of a tile have nothing
  // left to request: they are separate instances (compile-time flags, no branch in the
  // body - a branch would cost the compiler its count of the loads in flight) with the
  // wait counts that follow from the shorter queue.
  using Yes = std::true_type;
  using No = std::false_type;
  auto k_step = [&](auto first, auto fetch_q, auto fetch_p, auto read_next, auto wait_code, __bf16* cur,
                    const __bf16* nxt, __bf16* prv, int kt) {
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) {
      mma_one(first, 0, idx);
      CANZ_FENCE();
      if (idx < 8) {
        frag_one(cur, 1, 1, idx);  // second half-step's operands, land under the next 8 MFMAs
        CANZ_FENCE();
      }
      if (decltype(fetch_q)::value && (idx & 3) == 2) {
        fetch_one(prv, kt + 3, 4 + (idx >> 2));  // Q panel of step kt+3
        CANZ_FENCE();
      }
    }
    // own share of step kt+1 has landed; this wavefront's reads of `cur` are complete.
    // simm16 = vmcnt[3:0] | expcnt 7 << 4 | lgkmcnt << 8 | vmcnt[5:4] << 14
    __builtin_amdgcn_s_waitcnt(decltype(wait_code)::value);
    __builtin_amdgcn_s_barrier();
    CANZ_FENCE();
#pragma unroll
    for (int idx = 0; idx < 16; ++idx) {
      mma_one(No{}, 1, idx);
      CANZ_FENCE();
      if (decltype(read_next)::value && idx < 8) {
        frag_one(nxt, 0, 0, idx);  // first operands of step kt+1
        CANZ_FENCE();
      }
      if (decltype(fetch_p)::value && (idx & 3) == 2) {
        fetch_one(cur, kt + 4, idx >> 2);  // P panel of step kt+4
        CANZ_FENCE();
      }
    }
  };
  using Vm16 = std::integral_constant<int, 0x4070>;  // vmcnt(16) lgkmcnt(0)
  using Vm8 = std::integral_constant<int, 0x0078>;   // vmcnt(8)  lgkmcnt(0)
  using Vm0 = std::integral_constant<int, 0x0070>;   // vmcnt(0)  lgkmcnt(0)

  // steps 0..2 whole and the P panel of step 3; its Q panel is the first request of step 0
  fetch(st0, 0);
  fetch(st1, 1);
  fetch(st2, 2);
#pragma unroll
  for (int idx = 0; idx < 4; ++idx) fetch_one(st3, 3, idx);
  __syncthreads();
#pragma unroll
  for (int idx = 0; idx < 8; ++idx) frag_one(st0, 0, 0, idx);
  // first four steps (the very first one starts the accumulators), whole groups of four,
  // last four steps; nk is a multiple of 4 and at least 8
  k_step(Yes{}, Yes{}, Yes{}, Yes{}, Vm16{}, st0, st1, st3, 0);
  k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st1, st2, st0, 1);
  k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st2, st3, st1, 2);
  k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st3, st0, st2, 3);
  for (int kt = 4; kt < nk - 4; kt += 4) {
    k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st0, st1, st3, kt);
    k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st1, st2, st0, kt + 1);
    k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st2, st3, st1, kt + 2);
    k_step(No{}, Yes{}, Yes{}, Yes{}, Vm16{}, st3, st0, st2, kt + 3);
  }
  {
    // the tail: Q(nk-1) is the last request; then the queue drains: 16, 8, 0 younger loads
    const int kt = nk - 4;
    k_step(No{}, Yes{}, No{}, Yes{}, Vm16{}, st0, st1, st3, kt);
    k_step(No{}, No{}, No{}, Yes{}, Vm8{}, st1, st2, st0, kt + 1);
    k_step(No{}, No{}, No{}, Yes{}, Vm0{}, st2, st3, st1, kt + 2);
    k_step(No{}, No{}, No{}, No{}, Vm0{}, st3, st0, st2, kt + 3);
  }
  __syncthreads();  // every wavefront is done with the stages; LDS is free for the epilogue
#undef CANZ_FENCE

  if (SPLIT) {
    // k-slice: park the accumulators (register r of thread t at [r][t]: coalesced stores);
    // k_split_finish adds the slices of each tile up and runs its epilogue.
    float* mine = e.partial + static_cast<int64_t>(slot) * (256 * NTHREADS) + t;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[((i * 4 + j) * 16 + r) * NTHREADS] = acc[i][j][r];
        __builtin_amdgcn_sched_barrier(0);
      }
    break;
  }

  {
    __bf16* stage = wave == 0 ? st0 : wave == 1 ? st1 : wave == 2 ? st2 : st3;
    tile_epilogue<EPI>(acc, stage, lane, wm, wn, b, tm, tn, d, e, s, o);
  }

  // the next tile's loads overwrite every wavefront's staging area: wait for all of them.
  // The global stores issued above keep draining while the next tile is multiplied.
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) only
  __builtin_amdgcn_s_barrier();
  }  // persistent work loop
}

// Finishes the tiles whose k range was split: one block per tile adds the parked slices
// (always in slice order, so the sum does not depend on timing) and runs the epilogue.
template <int EPI>
__global__ __launch_bounds__(NTHREADS) void k_split_finish(GemmDims d, EpiArgs e, Shape s, OutSpec o) {
  __shared__ __attribute__((aligned(1024))) __bf16 stg[4][(BM + BN) * BK];
  const int tiles_n = static_cast<int>(d.N / BN);
  const int tiles_m = static_cast<int>(d.M / BM);
  const int per_batch = epi_symmetric(EPI) ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  const int l = blockIdx.x;
  int b, tm, tn;
  decode_tile<EPI>(e.full_rounds * e.main_grid + l, tiles_m, tiles_n, per_batch, b, tm, tn);
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const float* first = e.partial + static_cast<int64_t>(l) * e.splits * (256 * NTHREADS) + t;
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f32x16 sum;
#pragma unroll
      for (int r = 0; r < 16; ++r) sum[r] = 0.f;
      for (int sl = 0; sl < e.splits; ++sl) {
        const float* p = first + static_cast<int64_t>(sl) * (256 * NTHREADS) + (i * 4 + j) * 16 * NTHREADS;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[r] += p[r * NTHREADS];
      }
      acc[i][j] = sum;
    }
  tile_epilogue<EPI>(acc, stg[wave], lane, wave >> 1, wave & 1, b, tm, tn, d, e, s, o);
}

// ---------------------------------------------------------------------------------------
// Small-product variant: 128 x 128 tiles, one block per tile, three resident blocks per CU.
//
// The persistent 256 x 256 kernel above is built for products with many rounds of long tiles.
// A launch with few tiles (the 0.6B-shaped shares: 260 Gram tiles for 256 CUs) leaves most
// of its last round idle and pays the un-overlapped prologue and epilogue of a tile on every
// short k range.  Here a tile is a quarter of that: four times as many blocks balance over
// the chip, 48 KiB of LDS and 64 accumulator registers per lane let three blocks share a CU, so
// that one block's loads and epilogue run under the others' MFMAs.  The price is twice the
// L2 -> LDS traffic per FLOP, which is why long products stay with the large tile.
// It therefore takes what the large kernel handles badly: launches with few tiles, and the
// left-over tiles behind the last full round of a launch with a short k range (each left-over
// 256 x 256 tile becomes four blocks here).
//
// Same operands (panel layout: the 128 rows of a tile are one contiguous 8 KiB half of a
// panel), same MFMA, same order of accumulation over k, same epilogue arithmetic: an element
// comes out with the same bits from either kernel.  Epilogues store straight from the
// accumulators (4 bytes per lane for the straight image after the lane-pair exchange, 8 bytes
// per lane for the transposed one): there is no LDS to spare for staging with three blocks
// per CU, and the stores of one block drain under the work of the others.  Only the last
// product, whose rows go to the caller's row-major buffers, stages them through the stages
// the k loop has left free.
constexpr int SM = 128;                  // tile rows and columns
constexpr int S_STAGE = 2 * SM * BK;     // elements per stage: P half-panel + Q half-panel (16 KiB)

template <int EPI, typename Args>
__global__ __launch_bounds__(NTHREADS, 3) void k_gemm_nt_bf16_small(Args args, EpiArgs e_launch, Shape s, OutSpec o) {
  __shared__ __attribute__((aligned(1024))) __bf16 sa[S_STAGE];
  __shared__ __attribute__((aligned(1024))) __bf16 sb[S_STAGE];
  __shared__ __attribute__((aligned(1024))) __bf16 sc[S_STAGE];

  GemmDims d{};
  const __bf16 *P = nullptr, *Q = nullptr;
  EpiArgs e = e_launch;
  // neighbouring tiles on one XCD (blockIdx % 8 selects the XCD): they share panels in its L2
  int logical;
  {
    const int nblocks = gridDim.x, bid = blockIdx.x;
    const int per = nblocks / N_XCD, rem = nblocks % N_XCD;
    const int xcd = bid % N_XCD, q = bid / N_XCD;
    logical = xcd < rem ? xcd * (per + 1) + q : rem * (per + 1) + (xcd - rem) * per + q;
  }
  // four consecutive blocks are the quadrants of one 256 x 256 tile of the large kernel's
  // numbering, starting at tile e.main_grid (the launcher's "first tile" here)
  const int quad = logical & 3;
  logical = e.main_grid + (logical >> 2);
  if constexpr (Args::multi) {
    int j = 0;
    while (j + 1 < args.n && logical >= args.begin[j + 1]) ++j;
    const GemmProblem& pr = args.pr[j];
    d = pr.d;
    P = static_cast<const __bf16*>(pr.p), Q = static_cast<const __bf16*>(pr.q);
    e.c = pr.c, e.ct = pr.ct, e.aux = pr.aux, e.scale = pr.scale;
    logical -= args.begin[j];
  } else {
    d = args.d, P = args.P, Q = args.Q;
  }
  const int tiles_m = static_cast<int>(d.M / BM), tiles_n = static_cast<int>(d.N / BN);
  const bool symmetric = epi_symmetric(EPI);
  const int per_batch = symmetric ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  int b, tm, tn;
  decode_tile<EPI>(logical, tiles_m, tiles_n, per_batch, b, tm, tn);
  // the lower-left quadrant of a diagonal tile of a symmetric product is the mirror of the upper-right one
  if (symmetric && tm == tn && quad == 2) return;
  tm = 2 * tm + (quad >> 1), tn = 2 * tn + (quad & 1);

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int nk = static_cast<int>(d.K / BK);
  const int64_t nkb = d.K / BK;

  // global -> LDS: a stage is 16 pieces of 1 KiB (8 of P, 8 of Q); wavefront w copies the
  // pieces w and w + 4 of both, lane l the 16 bytes at l * 16
  const __bf16* pl = P + static_cast<int64_t>(b) * d.sp + (static_cast<int64_t>(tm >> 1) * nkb) * PANEL_ELEMS +
                     (tm & 1) * (SM * BK) + wave * 512 + lane * 8;
  const __bf16* ql = Q + static_cast<int64_t>(b) * d.sq + (static_cast<int64_t>(tn >> 1) * nkb) * PANEL_ELEMS +
                     (tn & 1) * (SM * BK) + wave * 512 + lane * 8;
  auto fetch = [&](__bf16* st, int kt) {
    const int64_t off = static_cast<int64_t>(kt < nk ? kt : nk - 1) * PANEL_ELEMS;  // past the end: a harmless re-read
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      __builtin_amdgcn_global_load_lds(CANZ_GLB(pl + off + g * 2048), CANZ_LDS(st + wave * 512 + g * 2048), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(CANZ_GLB(ql + off + g * 2048), CANZ_LDS(st + SM * BK + wave * 512 + g * 2048), 16, 0, 0);
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frag_row = lane & 31, frag_kg = lane >> 5;
  auto multiply = [&](const __bf16* st) {
    bf16x8 fa[2][2], fb[2][2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[kk][i] = *reinterpret_cast<const bf16x8*>(st + swz(wm * 64 + i * 32 + frag_row, kk * 2 + frag_kg));
        fb[kk][i] = *reinterpret_cast<const bf16x8*>(st + SM * BK + swz(wn * 64 + i * 32 + frag_row, kk * 2 + frag_kg));
      }
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kk][i], fb[kk][j], acc[i][j], 0, 0, 0);
  };
  // One k-step on stage `cur`: the 4 loads of the following step may stay in flight; after the
  // barrier every wavefront has finished the step before, whose stage `nxt2` then receives step kt + 2.
  auto k_step = [&](const __bf16* cur, __bf16* nxt2, int kt) {
    __builtin_amdgcn_s_waitcnt(0x0074);  // vmcnt(4) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    fetch(nxt2, kt + 2);
    multiply(cur);
  };
  fetch(sa, 0);
  fetch(sb, 1);
  int kt = 0;
  for (; kt + 3 <= nk; kt += 3) {
    k_step(sa, sc, kt);
    k_step(sb, sa, kt + 1);
    k_step(sc, sb, kt + 2);
  }
  if (kt < nk) k_step(sa, sc, kt), ++kt;
  if (kt < nk) k_step(sb, sa, kt), ++kt;
  __builtin_amdgcn_s_waitcnt(0x0070);  // the re-reads past the end have landed before the block leaves

  // ---- epilogue.  Accumulator register r of lane l in MFMA tile (i, j): row 32 i + 8 (r / 4) + 4 (l / 32) + (r % 4),
  //      column 32 j + (l % 32) of the wavefront's 64 x 64 part.
  const int lj = lane & 31, lh = lane >> 5;
  const int row_w = tm * SM + wm * 64, col_w = tn * SM + wn * 64;
  if (EPI == EPI_POLY) {
    // A(i, j) is read as A(j, i) (symmetric bit for bit): the lane's four consecutive rows are
    // four consecutive k of row j, one 8-byte load
    const __bf16* A = static_cast<const __bf16*>(e.aux) + static_cast<int64_t>(b) * d.M * d.N;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = col_w + 32 * j + lj;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int row0 = row_w + 32 * i + 8 * g + 4 * lh;
          const bf16x4 av = *reinterpret_cast<const bf16x4*>(A + panel_chunk_off(col, row0 & ~7, d.M) + (row0 & 7));
#pragma unroll
          for (int q = 0; q < 4; ++q)
            acc[i][j][4 * g + q] = poly_value(static_cast<float>(av[q]), acc[i][j][4 * g + q], e.ca, e.cb, e.cc, row0 + q == col);
        }
      }
  } else if (e.scale) {
    const float sc1 = e.scale[b];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] *= sc1;
  }

  if (epi_final(EPI)) {
    const int ld = static_cast<int>(o.out_mode == CANZ_OUT_DELTA ? s.wfrag : s.cols);
    if ((ld & 3) != 0) {
      // unaligned row length: element-wise accesses straight from the accumulators
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          float v[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) v[r] = acc[i][j][r];
          store_out_tile(o, s, b, row_w + 32 * i + 4 * lh, col_w + 32 * j + lj, v);
        }
      return;
    }
    // The stages are free once every wavefront has left the k loop: each wavefront turns its
    // 64 x 64 part through 8 KiB of LDS, 32 rows at a time, into rows of fp32 and updates the
    // caller's buffer with 16-byte accesses (4 columns per lane, 16 lanes per row).
    __syncthreads();
    float* sf = reinterpret_cast<float*>(wave == 0 ? sa : wave == 1 ? sa + 4096 : wave == 2 ? sb : sb + 4096);
    const int col = col_w + (lane & 15) * 4;
    const bool col_ok = col < s.cols;
    int c_in = col, tab = b;
    if (o.out_mode == CANZ_OUT_DELTA) {
      const int f = col_ok ? col / ld : 0;
      c_in = col - f * ld;
      tab = b * s.tp + f;
    }
    char* base = static_cast<char*>(o.out.p[col_ok ? tab : b * (o.out_mode == CANZ_OUT_DELTA ? s.tp : 1)]);
    const int esz = o.out_dtype == CANZ_DT_F32 ? 4 : 2;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) sf[(8 * (r >> 2) + 4 * lh + (r & 3)) * 64 + 32 * j + lj] = acc[i][j][r];
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const int row_l = 4 * x + (lane >> 4);
        const f32x4 v = *reinterpret_cast<const f32x4*>(sf + row_l * 64 + (lane & 15) * 4);
        const int row = row_w + 32 * i + row_l;
        if (!col_ok || row >= s.rows) continue;
        char* ptr = base + (static_cast<int64_t>(row) * ld + c_in) * esz;
        f32x4 res;
        if (o.out_mode == CANZ_OUT_PARAM) {
          f32x4 old;
          if (o.out_dtype == CANZ_DT_F32) {
            old = *reinterpret_cast<const f32x4*>(ptr);
          } else {
            const bf16x4 ob = *reinterpret_cast<const bf16x4*>(ptr);
#pragma unroll
            for (int q = 0; q < 4; ++q) old[q] = static_cast<float>(ob[q]);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) res[q] = apply_update(old[q], o.decay, o.neg_lr_scale, v[q]);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) res[q] = o.neg_lr_scale * v[q];
        }
        if (o.out_dtype == CANZ_DT_F32) {
          *reinterpret_cast<f32x4*>(ptr) = res;
        } else {
          bf16x4 rb;
#pragma unroll
          for (int q = 0; q < 4; ++q) rb[q] = static_cast<__bf16>(res[q]);
          *reinterpret_cast<bf16x4*>(ptr) = rb;
        }
      }
      // the second half is staged in the same area (this wavefront's own: no barrier needed)
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    }
    return;
  }

  __bf16* C = static_cast<__bf16*>(e.c) + static_cast<int64_t>(b) * d.M * d.N;
  // straight image: (row i, k = j).  Neighbouring lanes exchange their packed pairs so that each
  // lane holds two consecutive columns of one row: the even lane of row 2 rp, the odd lane of row 2 rp + 1.
  const unsigned pair_sel = (lane & 1) ? 0x03020706u : 0x05040100u;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = col_w + 32 * j + (lj & ~1);
#pragma unroll
      for (int rp = 0; rp < 8; ++rp) {
        bf16x2 own;
        own[0] = static_cast<__bf16>(acc[i][j][2 * rp]);
        own[1] = static_cast<__bf16>(acc[i][j][2 * rp + 1]);
        const unsigned mine = __builtin_bit_cast(unsigned, own);
        const unsigned theirs = lane_xor1(mine);
        const unsigned pk = __builtin_amdgcn_perm(theirs, mine, pair_sel);
        const int row = row_w + 32 * i + 8 * (rp >> 1) + 4 * lh + 2 * (rp & 1) + (lane & 1);
        *reinterpret_cast<unsigned*>(C + panel_chunk_off(row, col & ~7, d.N) + (col & 7)) = pk;
      }
    }
  // transposed image: (row j, k = i) of CT (UPDATE) or of the mirror tile of C (symmetric products)
  if (!symmetric || tm != tn) {
    __bf16* CT = symmetric ? C : static_cast<__bf16*>(e.ct) + static_cast<int64_t>(b) * d.M * d.N;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = col_w + 32 * j + lj;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int row0 = row_w + 32 * i + 8 * g + 4 * lh;
          bf16x4 pk;
#pragma unroll
          for (int q = 0; q < 4; ++q) pk[q] = static_cast<__bf16>(acc[i][j][4 * g + q]);
          *reinterpret_cast<bf16x4*>(CT + panel_chunk_off(col, row0 & ~7, d.M) + (row0 & 7)) = pk;
        }
      }
  }
}

// Compute units of the current device.  The answer is cached per device in a plain array: the
// first calls from several threads may each query the attribute and store the same value
// (a benign race on an int that only ever takes one non-zero value).
int cu_count() {
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

// How a launch is divided between the two kernels.  Long products (k above SMALL_MAX_K; the small
// tile moves twice the bytes per FLOP) stay with the large kernel and its k-split.  Otherwise
// the large kernel runs the full rounds of one tile per CU, and the left-over tiles go to the
// small kernel when they would leave at least half of the chip idle for a whole tile time -
// which includes launches with no full round at all.
constexpr int64_t SMALL_MAX_K = 4096;
constexpr int64_t SMALL_ALL_MAX_K = 2048;   // polynomial products up to this k and under two rounds: small tiles only

template <int EPI>
int64_t tile_count(const GemmDims& d) {
  const int64_t tm = d.M / BM, tn = d.N / BN;
  return (epi_symmetric(EPI) ? tm * (tm + 1) / 2 : tm * tn) * d.nb;
}

// number of tiles [0, whole) for the large kernel; the rest, if any, for the small one
template <int EPI>
int64_t large_share(int64_t tiles, int64_t cus, int64_t longest_k) {
  const int64_t left = tiles % cus;
  if (longest_k > SMALL_MAX_K) return tiles;
  // a polynomial product (k = m, the shortest k range of the step) of less than two rounds runs faster on small
  // tiles throughout: 59.6 -> 52.4 us on 26 matrices of 1024 x 1024; the same rule costs the Gram product 7 %
  if (EPI == EPI_POLY && tiles < 2 * cus && longest_k <= SMALL_ALL_MAX_K) return 0;
  if (left == 0 || 2 * left > cus) return tiles;
  return tiles - left;
}

template <int EPI>
hipError_t launch(const GemmDims& d, const void* P, const void* Q, EpiArgs e, const SplitWs& w, const Shape& s,
                  const OutSpec& o, hipStream_t st) {
  // the k loop of both kernels takes whole panels in groups of four with a tail of four: K is a
  // multiple of 256 (the producers pad to PAD), hence at least 8 k-steps
  if (d.K < 8 * BK || d.K % (8 * BK) || d.M % BM || d.N % BN) return hipErrorInvalidValue;
  const int64_t tiles = tile_count<EPI>(d);
  const int64_t cus = cu_count();
  const OneProblem one{d, static_cast<const __bf16*>(P), static_cast<const __bf16*>(Q)};
  const int64_t whole_large = large_share<EPI>(tiles, cus, d.K);
  if (whole_large < tiles) {
    if (whole_large > 0) {
      e.full_rounds = static_cast<int>(whole_large / cus), e.left = 0, e.splits = 1, e.partial = nullptr;
      e.main_grid = static_cast<int>(cus);
      hipLaunchKernelGGL((k_gemm_nt_bf16<EPI, false, OneProblem>), dim3(static_cast<unsigned>(cus)), dim3(NTHREADS), 0, st,
                         one, e, s, o);
    }
    e.main_grid = static_cast<int>(whole_large);   // first tile of the small kernel
    hipLaunchKernelGGL((k_gemm_nt_bf16_small<EPI, OneProblem>), dim3(static_cast<unsigned>(4 * (tiles - whole_large))),
                       dim3(NTHREADS), 0, st, one, e, s, o);
    return hipGetLastError();
  }
  // full rounds of one tile per block, then the left-over tiles cut into k-slices (each at
  // least 8 k-steps long) so that they occupy as many blocks as fit
  e.full_rounds = static_cast<int>(tiles / cus);
  e.left = static_cast<int>(tiles % cus);
  e.splits = 1;
  if (e.left > 0 && w.partial) {
    const int64_t by_blocks = std::min<int64_t>(cus, w.max_blocks) / e.left;
    const int64_t by_k = (d.K / BK) / 8;
    const int64_t sp = std::max<int64_t>(1, std::min<int64_t>({by_blocks, by_k, 8}));
    // Splitting costs two more launches plus parking and re-reading the accumulators, about
    // 0.2 ms all told; a k-step takes about 0.65 us.  Split only where the part of a tile
    // time it saves, (1 - 1/sp) * k-steps, is clearly longer than that.
    if (sp > 1 && (d.K / BK) * (sp - 1) / sp >= 400) e.splits = static_cast<int>(sp);
  }
  e.partial = w.partial;
  // whole tiles: one persistent block per CU (fewer if there are fewer tiles)
  const int64_t whole = e.splits > 1 ? e.full_rounds * cus : tiles;
  e.main_grid = static_cast<int>(std::min<int64_t>(cus, std::max<int64_t>(whole, 1)));
  if (whole > 0)
    hipLaunchKernelGGL((k_gemm_nt_bf16<EPI, false, OneProblem>), dim3(static_cast<unsigned>(e.main_grid)), dim3(NTHREADS),
                       0, st, one, e, s, o);
  if (e.splits > 1) {
    hipLaunchKernelGGL((k_gemm_nt_bf16<EPI, true, OneProblem>), dim3(static_cast<unsigned>(e.left * e.splits)),
                       dim3(NTHREADS), 0, st, one, e, s, o);
    hipLaunchKernelGGL((k_split_finish<EPI>), dim3(static_cast<unsigned>(e.left)), dim3(NTHREADS), 0, st, d, e, s, o);
  }
  return hipGetLastError();
}

// Several products in one launch: whole tiles only (no k-split), one persistent block per CU.
template <int EPI>
hipError_t launch_multi(const GemmBatch& g, EpiArgs e, hipStream_t st) {
  const int64_t cus = cu_count();
  ManyProblems many{};
  many.n = g.n;
  int64_t tiles = 0, longest_k = 0;
  for (int j = 0; j < g.n; ++j) {
    many.begin[j] = static_cast<int>(tiles);
    many.pr[j] = g.pr[j];
    const GemmDims& d = g.pr[j].d;
    if (d.K < 8 * BK || d.K % (8 * BK) || d.M % BM || d.N % BN) return hipErrorInvalidValue;
    tiles += tile_count<EPI>(d);
    longest_k = std::max(longest_k, d.K);
  }
  for (int j = g.n; j <= MAX_KINDS; ++j) many.begin[j] = static_cast<int>(tiles);
  if (tiles == 0) return hipSuccess;
  const int64_t whole_large = large_share<EPI>(tiles, cus, longest_k);
  e.splits = 1;
  e.partial = nullptr;
  if (whole_large > 0) {
    e.full_rounds = static_cast<int>(whole_large / cus);
    e.left = static_cast<int>(whole_large % cus);
    e.main_grid = static_cast<int>(std::min<int64_t>(cus, whole_large));
    hipLaunchKernelGGL((k_gemm_nt_bf16<EPI, false, ManyProblems>), dim3(static_cast<unsigned>(e.main_grid)), dim3(NTHREADS),
                       0, st, many, e, Shape{}, OutSpec{});
  }
  if (whole_large < tiles) {
    e.main_grid = static_cast<int>(whole_large);   // first tile of the small kernel
    hipLaunchKernelGGL((k_gemm_nt_bf16_small<EPI, ManyProblems>), dim3(static_cast<unsigned>(4 * (tiles - whole_large))),
                       dim3(NTHREADS), 0, st, many, e, Shape{}, OutSpec{});
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gram_bf16_multi(const GemmBatch& g, hipStream_t st) { return launch_multi<EPI_GRAM>(g, EpiArgs{}, st); }

hipError_t launch_poly_bf16_multi(const GemmBatch& g, float ca, float cb, float cc, hipStream_t st) {
  EpiArgs e{};
  e.ca = ca, e.cb = cb, e.cc = cc;
  return launch_multi<EPI_POLY>(g, e, st);
}

hipError_t launch_update_bf16_multi(const GemmBatch& g, hipStream_t st) { return launch_multi<EPI_UPDATE>(g, EpiArgs{}, st); }

hipError_t launch_gram_bf16(const GemmDims& d, const void* xw, void* a_out, const float* scale2, const SplitWs& w,
                            hipStream_t st) {
  EpiArgs e{};
  e.c = a_out;
  e.scale = scale2;
  return launch<EPI_GRAM>(d, xw, xw, e, w, Shape{}, OutSpec{}, st);
}

hipError_t launch_poly_bf16(const GemmDims& d, const void* a_in, void* b_out, float ca, float cb, float cc,
                            const SplitWs& w, hipStream_t st) {
  EpiArgs e{};
  e.c = b_out;
  e.aux = a_in;
  e.ca = ca, e.cb = cb, e.cc = cc;
  return launch<EPI_POLY>(d, a_in, a_in, e, w, Shape{}, OutSpec{}, st);
}

hipError_t launch_update_bf16(const GemmDims& d, const void* b_in, const void* xt_in, void* xw_out, void* xt_out,
                              const float* scale, const SplitWs& w, hipStream_t st) {
  EpiArgs e{};
  e.c = xw_out;
  e.ct = xt_out;
  e.scale = scale;
  return launch<EPI_UPDATE>(d, b_in, xt_in, e, w, Shape{}, OutSpec{}, st);
}

hipError_t launch_final_bf16(const GemmDims& d, const void* p, const void* q, const float* scale, const SplitWs& w,
                             const Shape& s, const OutSpec& o, hipStream_t st) {
  EpiArgs e{};
  e.scale = scale;
  return launch<EPI_FINAL>(d, p, q, e, w, s, o, st);
}

hipError_t launch_final_sym_bf16(const GemmDims& d, const void* x, const SplitWs& w, const Shape& s, const OutSpec& o,
                                 hipStream_t st) {
  if (d.M != d.N) return hipErrorInvalidValue;
  return launch<EPI_FINAL_SYM>(d, x, x, EpiArgs{}, w, s, o, st);
}

}  // namespace canz
