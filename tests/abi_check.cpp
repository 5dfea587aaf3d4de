// Stand-alone check of the C-ABI from a plain host program (no Python, no torch): device memory from
// hipMalloc, the three calls on a user-created stream, results compared with the CPU oracle.
// Built by __graft_entry__.build(); run by tests/test_gpu_parity.py::test_c_abi_from_a_plain_host_program.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "moe_rbf.h"

extern "C" {
int moe_ref_plan(int32_t, int32_t, int32_t, int32_t, int64_t, const int32_t *, int32_t *, int32_t *, int32_t *, int32_t *,
                 int32_t *, int32_t *, int32_t *);
int moe_ref_dispatch(int32_t, int32_t, int32_t, int32_t, const void *, const int32_t *, void *);
int moe_ref_combine(int32_t, int32_t, int32_t, int32_t, const void *, const float *, const int32_t *, void *);
}

#define HIP_OK(x)                                                                  \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      return 2;                                                                    \
    }                                                                              \
  } while (0)
#define MOE_OK_(x)                                                                          \
  do {                                                                                      \
    int r_ = (x);                                                                           \
    if (r_ != MOE_OK) {                                                                     \
      std::printf("%s -> %s [%s]\n", #x, moe_strerror(r_), moe_last_launch_error());        \
      return 3;                                                                             \
    }                                                                                       \
  } while (0)

template <typename T>
static T *dev(size_t n) {
  void *p = nullptr;
  if (hipMalloc(&p, n * sizeof(T) + 16) != hipSuccess) std::exit(4);
  return (T *)p;
}

static int run(int schedule, int T, int H, int k, int E, int R) {
  const int N = T * k;
  std::vector<uint16_t> X((size_t)T * H);
  std::vector<int32_t> K(N);
  std::vector<float> W(N);
  srand(7 + schedule);
  for (auto &v : X) v = (uint16_t)(0x3C00 + rand() % 0x0800);            // positive finite bf16 values below 1
  for (int i = 0; i < N; ++i) K[i] = rand() % 13 == 0 ? -1 : rand() % E;
  for (auto &v : W) v = (float)rand() / (float)RAND_MAX;

  moe_shape sh{};
  sh.T = T, sh.H = H, sh.k = k, sh.E = E, sh.R = R, sh.dtype = MOE_DTYPE_BF16, sh.schedule = schedule;
  size_t ws_bytes = 0;
  int64_t rows = 0;
  MOE_OK_(moe_workspace_bytes(&sh, &ws_bytes));
  MOE_OK_(moe_window_rows(&sh, &rows));

  hipStream_t st;
  HIP_OK(hipStreamCreate(&st));
  uint16_t *dX = dev<uint16_t>(X.size()), *dWin = dev<uint16_t>((size_t)rows * H), *dY = dev<uint16_t>(X.size());
  int32_t *dK = dev<int32_t>(N);
  float *dW = dev<float>(N);
  moe_plan_t pl{};
  pl.expert_count = dev<int32_t>(E), pl.rank_count = dev<int32_t>(R), pl.expert_offset = dev<int32_t>(E + 1);
  pl.region_base = dev<int32_t>(R + 1), pl.send_idx = dev<int32_t>(N), pl.row_map = dev<int32_t>(N);
  pl.status = dev<int32_t>(4), pl.workspace = dev<char>(ws_bytes), pl.workspace_bytes = ws_bytes;
  HIP_OK(hipMemcpyAsync(dX, X.data(), X.size() * 2, hipMemcpyHostToDevice, st));
  HIP_OK(hipMemcpyAsync(dK, K.data(), N * 4, hipMemcpyHostToDevice, st));
  HIP_OK(hipMemcpyAsync(dW, W.data(), N * 4, hipMemcpyHostToDevice, st));
  HIP_OK(hipMemsetAsync(dWin, 0, (size_t)rows * H * 2, st));

  int32_t resolved = 0;
  MOE_OK_(moe_resolve_schedule(&sh, &resolved));
  if (resolved == MOE_SCHEDULE_PREFILL) MOE_OK_(moe_plan(&sh, dK, &pl, st));
  MOE_OK_(moe_dispatch(&sh, dX, dK, &pl, dWin, st));
  MOE_OK_(moe_combine(&sh, dWin, dW, &pl, dY, st));                         // identity expert: window is its own output

  std::vector<int32_t> row_map(N), status(3);
  std::vector<uint16_t> win((size_t)rows * H), Y(X.size());
  HIP_OK(hipMemcpyAsync(row_map.data(), pl.row_map, N * 4, hipMemcpyDeviceToHost, st));
  HIP_OK(hipMemcpyAsync(status.data(), pl.status, 12, hipMemcpyDeviceToHost, st));
  HIP_OK(hipMemcpyAsync(win.data(), dWin, win.size() * 2, hipMemcpyDeviceToHost, st));
  HIP_OK(hipMemcpyAsync(Y.data(), dY, Y.size() * 2, hipMemcpyDeviceToHost, st));
  HIP_OK(hipStreamSynchronize(st));

  std::vector<int32_t> ce(E), cr(R), eo(E + 1), rb(R + 1), s(N), rm(N), rst(3);
  moe_ref_plan(T, k, E, R, 0, K.data(), ce.data(), cr.data(), eo.data(), rb.data(), s.data(), rm.data(), rst.data());
  std::vector<uint16_t> rwin((size_t)rows * H, 0), rY(X.size());
  moe_ref_dispatch(T, H, k, 2, X.data(), rm.data(), rwin.data());
  moe_ref_combine(T, H, k, MOE_DTYPE_BF16, rwin.data(), W.data(), rm.data(), rY.data());
  if (row_map != rm) return std::printf("row_map differs (schedule %d)\n", schedule), 1;
  if (status[0] != rst[0] || status[1] != rst[1] || status[2] != rst[2]) return std::printf("status differs\n"), 1;
  if (std::memcmp(win.data(), rwin.data(), win.size() * 2)) return std::printf("window differs\n"), 1;
  for (size_t i = 0; i < Y.size(); ++i) {
    const int d = (int)Y[i] - (int)rY[i];                                  // all values positive: plain code distance
    if (d < -1 || d > 1) return std::printf("Y differs at %zu: %04x vs %04x\n", i, Y[i], rY[i]), 1;
  }
  std::printf("schedule %d (resolved %d): T=%d H=%d k=%d E=%d R=%d ok\n", schedule, resolved, T, H, k, E, R);
  return 0;
}

int main() {
  int rc = run(MOE_SCHEDULE_PREFILL, 700, 1024, 8, 64, 8);
  if (rc) return rc;
  rc = run(MOE_SCHEDULE_DECODE, 100, 7168, 8, 256, 32);
  if (rc) return rc;
  rc = run(MOE_SCHEDULE_AUTO, 5000, 512, 4, 32, 4);
  if (rc) return rc;
  std::puts("abi_check: ok");
  return 0;
}
