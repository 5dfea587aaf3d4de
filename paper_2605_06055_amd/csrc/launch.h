// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <utility>

namespace moe_rbf {

// Device pointers of the plan state, passed by value to kernels.
struct PlanView {
  int32_t *expert_count;   // [E]
  int32_t *rank_count;     // [R]
  int32_t *expert_offset;  // [E+1]
  int32_t *region_base;    // [R+1]
  int32_t *send_idx;       // [N] or nullptr
  int32_t *row_map;        // [N]
  int32_t *status;         // [2]
  const int32_t *source_count;  // [R*E] or nullptr
  int32_t *recv_count;     // [E] or nullptr
  int32_t *recv_offset;    // [E+1] or nullptr
  int32_t *order;          // [2*N] (token, row) pairs in dispatch order, or nullptr
};

// Memory that the plan's spare workgroups read while it runs (moe_plan_t.prefetch), kept out of PlanView so
// that the latency-bound kernels that take a PlanView do not carry it in their arguments.
struct WarmRange {
  const void *ptr = nullptr;
  long long vecs = 0;      // 16-byte vectors
};

struct Dims {
  int32_t T, H, k, E, R, Er;
  int32_t me;       // this device's source rank
  int32_t N;        // T*k
  int32_t H16;      // 16-byte vectors per row
  int32_t dtype;
  int64_t stride;   // region_stride_rows (0 = tight)
  int32_t order_tiles;   // plan tiles per sorted stretch of the dispatch order list (0: the list is not used)
};

// Branches per plan tile for N routed branches (1024, doubled until at most 512 tiles remain) and the tile count.
int plan_tile_size(int64_t N);
int plan_tile_count(int64_t N);
// Does launch_plan read and write its tile_hist scratch for N branches?  (Small batches are planned by one
// launch that counts every id itself and may be given tile_hist == nullptr.)
bool plan_uses_workspace(int64_t N);
// Plan tiles per sorted stretch of the dispatch order list for this shape; 0 = dispatch walks the branches in
// token order and the list is neither written nor read.  Depends on the shape only, so that moe_plan, the
// decode-schedule dispatch (which leaves a plan) and the prefill-schedule dispatch agree.
int plan_order_tiles(const Dims &d);

hipError_t launch_plan_empty(const Dims &d, const PlanView &p, hipStream_t s);
hipError_t launch_plan(const Dims &d, const int32_t *K, const PlanView &p, int32_t *tile_hist, const WarmRange &warm,
                       hipStream_t s);
hipError_t launch_dispatch(const Dims &d, const void *x, const PlanView &p, void *window, hipStream_t s);
hipError_t launch_decode_dispatch(const Dims &d, const void *x, const int32_t *K, const PlanView &p, void *window,
                                  hipStream_t s);
hipError_t launch_dispatch_quant(const Dims &d, const void *x, const PlanView &p, void *window_q, float *window_scale,
                                 hipStream_t s);
hipError_t launch_decode_dispatch_quant(const Dims &d, const void *x, const int32_t *K, const PlanView &p,
                                        void *window_q, float *window_scale, hipStream_t s);
hipError_t launch_combine(const Dims &d, const void *expert_out, const float *W, const PlanView &p, void *y,
                          hipStream_t s);

// Typed launch that returns this launch's own error code (not a sticky one left by the caller's
// earlier runtime calls).  Arguments are converted to the kernel's parameter types first.
template <typename... P, typename... A, size_t... I>
inline hipError_t launch_impl(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t s,
                              std::index_sequence<I...>, A &&...a) {
  std::tuple<P...> params(std::forward<A>(a)...);
  void *argv[] = {(void *)&std::get<I>(params)...};
  return hipLaunchKernel((const void *)kernel, grid, block, argv, lds, s);
}
template <typename... P, typename... A>
inline hipError_t launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t s, A &&...a) {
  static_assert(sizeof...(P) == sizeof...(A), "kernel argument count");
  return launch_impl(kernel, grid, block, lds, s, std::index_sequence_for<P...>{}, std::forward<A>(a)...);
}

}  // namespace moe_rbf
