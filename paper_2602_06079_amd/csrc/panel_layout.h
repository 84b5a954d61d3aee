// Storage layout of the bf16 working matrices (XW, XT, A, B) of the Newton-Schulz chain.
//
// Every one of them is only ever read as a GEMM operand "rows x k" whose 256 x 32 panels
// are copied verbatim into LDS.  So a matrix with R rows and KC columns (multiples of 256)
// is stored as a grid of such panels, [R / 256][KC / 32] panels of 16 KiB, and inside a
// panel exactly as the LDS image the MFMA operand loads want: row-major rows of 32
// elements (4 chunks of 16 bytes) with the chunk index XOR-ed by (row >> 2) & 3, which
// spreads the 16 rows one ds_read_b128 cycle serves over all 64 banks.
//   - a stage load is one contiguous 16 KiB read (full DRAM pages, full cache lines),
//   - a 256 x 256 output tile of a producer is one contiguous 128 KiB region, so the
//     epilogues assemble it in LDS and stream it out linearly.
// The fp32 verification path keeps plain row-major storage.
#pragma once
#include <cstdint>

namespace canz {

constexpr int PANEL_ROWS = 256;
constexpr int PANEL_K = 32;
constexpr int PANEL_ELEMS = PANEL_ROWS * PANEL_K;

// element offset of the 8-element chunk that holds (r, k8 .. k8 + 7); k8 is a multiple of 8
__host__ __device__ __forceinline__ int64_t panel_chunk_off(int64_t r, int64_t k8, int64_t kc) {
  return ((r >> 8) * (kc >> 5) + (k8 >> 5)) * PANEL_ELEMS + (r & 255) * PANEL_K +
         ((((k8 >> 3) & 3) ^ ((r >> 2) & 3)) << 3);
}

template <typename T>
struct WorkLayout;  // chunk_off(r, k8, kc): where the 8 elements (r, k8 ..) start
template <>
struct WorkLayout<__bf16> {
  __host__ __device__ static __forceinline__ int64_t chunk_off(int64_t r, int64_t k8, int64_t kc) {
    return panel_chunk_off(r, k8, kc);
  }
};
template <>
struct WorkLayout<float> {
  __host__ __device__ static __forceinline__ int64_t chunk_off(int64_t r, int64_t k8, int64_t kc) {
    return r * kc + k8;
  }
};

}  // namespace canz
