// A plain C++ consumer of libcanz.so: no Python, no torch.  Plans a small matrix set with
// the partitioner, allocates device buffers with hipMalloc, runs one optimizer step of the
// rank's share through the C ABI and writes inputs and results to a binary file, so that a
// test can check them against the CPU oracle.
//
//   c_abi_step <out.bin> <precision: 0 = bf16, 1 = fp32>
//
// File layout (little endian): int64 n, rows, cols; then per matrix four float32 arrays of
// rows*cols: gradient, parameter before, parameter after, momentum after.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "canz.h"

#define HIP_OK(call)                                                                         \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess) {                                                                  \
      std::fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));                 \
      return 2;                                                                              \
    }                                                                                        \
  } while (0)
#define CANZ_CHECK(call)                                                                     \
  do {                                                                                       \
    if ((call) != CANZ_OK) {                                                                 \
      std::fprintf(stderr, "%s failed: %s\n", #call, canz_last_error());                     \
      return 3;                                                                              \
    }                                                                                        \
  } while (0)

int main(int argc, char** argv) {
  if (argc < 3) {
    std::fprintf(stderr, "usage: %s <out.bin> <precision 0|1>\n", argv[0]);
    return 1;
  }
  const int precision = std::atoi(argv[2]);

  // 2 buckets of 3 matrices each, 2 ranks: run what rank 0 owns
  const int64_t rows[6] = {300, 300, 300, 300, 300, 300}, cols[6] = {200, 200, 200, 200, 200, 200};
  const int64_t bucket_off[3] = {0, 3, 6};
  int64_t cut[2 * 3], load[2];
  int32_t owner[6];
  CANZ_CHECK(canz_partition_alpha(6, rows, cols, nullptr, CANZ_COST_NUMEL, 2, bucket_off, 2, 1.0, cut, owner, load));
  const int32_t dtype[6] = {CANZ_DT_F32, CANZ_DT_F32, CANZ_DT_F32, CANZ_DT_F32, CANZ_DT_F32, CANZ_DT_F32};
  int64_t n_groups = 0, group_off[7], member[6];
  CANZ_CHECK(canz_microgroup_plan(6, rows, cols, dtype, owner, 0, 8, 0, &n_groups, group_off, member));
  if (n_groups != 1) {
    std::fprintf(stderr, "expected one micro-group, got %lld\n", static_cast<long long>(n_groups));
    return 4;
  }
  const int n = static_cast<int>(group_off[1] - group_off[0]);
  const int64_t R = rows[0], Ccols = cols[0], numel = R * Ccols;

  // deterministic inputs: a small linear congruential generator, values in (-0.02, 0.02)
  uint64_t state = 12345;
  auto next = [&]() {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (static_cast<double>(state >> 11) / 9007199254740992.0 - 0.5) * 0.04;
  };
  std::vector<std::vector<float>> grad(n), param(n);
  std::vector<const void*> d_grad(n);
  std::vector<void*> d_mom(n), d_out(n);
  for (int i = 0; i < n; ++i) {
    grad[i].resize(numel), param[i].resize(numel);
    for (auto& v : grad[i]) v = static_cast<float>(next());
    for (auto& v : param[i]) v = static_cast<float>(next());
    void *g = nullptr, *m = nullptr, *p = nullptr;
    HIP_OK(hipMalloc(&g, numel * 4));
    HIP_OK(hipMalloc(&m, numel * 4));
    HIP_OK(hipMalloc(&p, numel * 4));
    HIP_OK(hipMemcpy(g, grad[i].data(), numel * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(m, 0, numel * 4));
    HIP_OK(hipMemcpy(p, param[i].data(), numel * 4, hipMemcpyHostToDevice));
    d_grad[i] = g, d_mom[i] = m, d_out[i] = p;
  }

  canz_group grp{};
  grp.rows = R, grp.cols = Ccols, grp.n_mats = n, grp.tp = 1;
  grp.grad_dtype = CANZ_DT_F32, grp.out_dtype = CANZ_DT_F32;
  grp.grad = d_grad.data(), grp.mom = d_mom.data(), grp.out = d_out.data();
  canz_muon_hparams hp{};
  hp.beta = 0.95f, hp.lr = 0.02f, hp.weight_decay = 0.01f, hp.eps = 1e-7f;
  hp.nesterov = 0, hp.ns_steps = 5, hp.a = 3.4445f, hp.b = -4.7750f, hp.c = 2.0315f;
  hp.scale_mode = CANZ_SCALE_RMS, hp.precision = precision, hp.out_mode = CANZ_OUT_PARAM;

  size_t ws_bytes = 0;
  CANZ_CHECK(canz_muon_workspace_bytes(&grp, 1, &hp, &ws_bytes));
  void* ws = nullptr;
  HIP_OK(hipMalloc(&ws, ws_bytes));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));
  CANZ_CHECK(canz_muon_step(&grp, 1, &hp, ws, ws_bytes, stream));
  HIP_OK(hipStreamSynchronize(stream));

  std::FILE* f = std::fopen(argv[1], "wb");
  if (!f) return 5;
  const int64_t head[3] = {n, R, Ccols};
  std::fwrite(head, sizeof(int64_t), 3, f);
  std::vector<float> host(numel);
  for (int i = 0; i < n; ++i) {
    std::fwrite(grad[i].data(), 4, numel, f);
    std::fwrite(param[i].data(), 4, numel, f);
    HIP_OK(hipMemcpy(host.data(), d_out[i], numel * 4, hipMemcpyDeviceToHost));
    std::fwrite(host.data(), 4, numel, f);
    HIP_OK(hipMemcpy(host.data(), d_mom[i], numel * 4, hipMemcpyDeviceToHost));
    std::fwrite(host.data(), 4, numel, f);
  }
  std::fclose(f);
  for (int i = 0; i < n; ++i) {
    HIP_OK(hipFree(const_cast<void*>(d_grad[i])));
    HIP_OK(hipFree(d_mom[i]));
    HIP_OK(hipFree(d_out[i]));
  }
  HIP_OK(hipFree(ws));
  HIP_OK(hipStreamDestroy(stream));
  std::printf("c_abi_step: %d matrices of %lldx%lld, precision %d, workspace %zu bytes\n", n,
              static_cast<long long>(R), static_cast<long long>(Ccols), precision, ws_bytes);
  return 0;
}
