// C-ABI boundary of the library: argument validation on the host, then kernel launches on the
// caller's stream.  Nothing here allocates, copies between host and device, or synchronises.
#include <hip/hip_runtime.h>

#include <atomic>

#include "launch.h"
#include "moe_rbf.h"

using namespace moe_rbf;

// Scratch of moe_plan_static: the per-tile histograms that moe_plan keeps in the caller's plan->workspace.
// One copy per device, held until the process ends.  In host code this name is only a stand-in for the
// device array; its device address comes from hipGetSymbolAddress (static_scratch below).
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int elem_bytes(int dtype) { return dtype == MOE_DTYPE_BF16 ? 2 : 4; }

// Shape checks shared by every entry point.  Fills `d` on success.
int check_shape(const moe_shape *sh, Dims *d) {
  if (!sh) return MOE_ERR_NULL;
  if (sh->T < 0 || sh->H < 1 || sh->k < 1 || sh->E < 1 || sh->R < 1) return MOE_ERR_SHAPE;
  if (sh->E > MOE_MAX_EXPERTS || sh->E % sh->R != 0) return MOE_ERR_SHAPE;
  if (sh->dtype != MOE_DTYPE_BF16 && sh->dtype != MOE_DTYPE_F32) return MOE_ERR_SHAPE;
  if (sh->schedule != MOE_SCHEDULE_AUTO && sh->schedule != MOE_SCHEDULE_PREFILL &&
      sh->schedule != MOE_SCHEDULE_DECODE)
    return MOE_ERR_SHAPE;
  if (sh->rank_id < 0 || sh->rank_id >= sh->R || sh->region_stride_rows < 0) return MOE_ERR_SHAPE;
  const int64_t N = (int64_t)sh->T * sh->k;
  if (sh->schedule == MOE_SCHEDULE_DECODE && N > MOE_DECODE_MAX_BRANCHES) return MOE_ERR_SHAPE;
  const int64_t row_bytes = (int64_t)sh->H * elem_bytes(sh->dtype);
  if (row_bytes % 16 != 0) return MOE_ERR_ALIGN;
  if (N > INT32_MAX) return MOE_ERR_OVERFLOW;
  if (sh->region_stride_rows > 0 && (sh->region_stride_rows > INT32_MAX ||
                                     (int64_t)sh->R * sh->region_stride_rows > INT32_MAX))
    return MOE_ERR_OVERFLOW;
  // one workgroup per (token, 64-lane column chunk) or per (branch, 1/8 of a row): grids must fit in 31 bits
  if ((int64_t)sh->T * ((row_bytes / 16 + 63) / 64) > INT32_MAX || N * 8 > INT32_MAX) return MOE_ERR_OVERFLOW;
  if (d) {
    d->T = sh->T;
    d->H = sh->H;
    d->k = sh->k;
    d->E = sh->E;
    d->R = sh->R;
    d->Er = sh->E / sh->R;
    d->me = sh->rank_id;
    d->N = (int32_t)N;
    d->H16 = (int32_t)(row_bytes / 16);
    d->dtype = sh->dtype;
    d->stride = sh->region_stride_rows;
    d->order_tiles = 0;
  }
  return MOE_OK;
}

int resolve(const moe_shape *sh) {
  if (sh->schedule != MOE_SCHEDULE_AUTO) return sh->schedule;
  return (int64_t)sh->T * sh->k <= MOE_AUTO_DECODE_MAX_BRANCHES ? MOE_SCHEDULE_DECODE : MOE_SCHEDULE_PREFILL;
}

size_t workspace_need(const moe_shape *sh) {
  const int64_t N = (int64_t)sh->T * sh->k;
  const size_t b = (size_t)plan_tile_count(N) * (size_t)(sh->E + 1) * sizeof(int32_t);
  return (b + 255) / 256 * 256;
}

// Pointer checks for the plan tables that a call WRITES (need_tables) or only reads row_map from.
int check_plan(const moe_plan_t *pl, bool need_tables, PlanView *v) {
  if (!pl) return MOE_ERR_NULL;
  if (!pl->row_map) return MOE_ERR_NULL;
  if (need_tables && (!pl->expert_count || !pl->rank_count || !pl->expert_offset || !pl->region_base || !pl->status))
    return MOE_ERR_NULL;
  if (!aligned16(pl->row_map) || (pl->send_idx && !aligned16(pl->send_idx))) return MOE_ERR_ALIGN;
  if (need_tables && (!aligned16(pl->expert_count) || !aligned16(pl->rank_count) || !aligned16(pl->expert_offset) ||
                      !aligned16(pl->region_base) || !aligned16(pl->status)))
    return MOE_ERR_ALIGN;
  v->expert_count = pl->expert_count;
  v->rank_count = pl->rank_count;
  v->expert_offset = pl->expert_offset;
  v->region_base = pl->region_base;
  v->send_idx = pl->send_idx;
  v->row_map = pl->row_map;
  v->status = pl->status;
  v->source_count = need_tables ? pl->source_count : nullptr;
  v->recv_count = need_tables ? pl->recv_count : nullptr;
  v->recv_offset = need_tables ? pl->recv_offset : nullptr;
  v->order = pl->dispatch_order;
  if (!aligned16(pl->dispatch_order)) return MOE_ERR_ALIGN;

  if (need_tables && (!aligned16(pl->source_count) || !aligned16(pl->recv_count) || !aligned16(pl->recv_offset)))
    return MOE_ERR_ALIGN;
  return MOE_OK;
}

thread_local hipError_t g_last_hip_error = hipSuccess;

int launch_status(hipError_t e) {
  g_last_hip_error = e;
  return e == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}

// Do the byte ranges [a, a+na) and [b, b+nb) share a byte?
inline bool ranges_overlap(const void *a, uint64_t na, const void *b, uint64_t nb) {
  const uint64_t pa = (uint64_t)reinterpret_cast<uintptr_t>(a), pb = (uint64_t)reinterpret_cast<uintptr_t>(b);
  return na > 0 && nb > 0 && pa < pb + nb && pb < pa + na;
}

// Bytes of X / Y and (a lower bound of) the bytes of the window / expert_out buffer.  With several source
// ranks and tight windows the row count is device data (the sum of M); the T*k rows of this rank are
// then the part the host can be sure of.
inline uint64_t token_bytes(const Dims &d) { return (uint64_t)d.T * (uint64_t)d.H16 * 16u; }
inline uint64_t window_bytes(const Dims &d) {
  const uint64_t rows = d.stride > 0 ? (uint64_t)d.R * (uint64_t)d.stride : (uint64_t)d.N;
  return rows * (uint64_t)d.H16 * 16u;
}

// Device address of `scratch` on the current device, resolved once per device.
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

int static_scratch(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return launch_status(e);
  if (dev < 0 || dev >= kMaxDevices) return launch_status(hipErrorInvalidDevice);
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return launch_status(e);
    if (!p) return launch_status(hipErrorInvalidSymbol);
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread resolves the same address
  }
  *out = p;
  return MOE_OK;
}

// Common body of moe_plan and moe_plan_static.  own_scratch: the tile histograms go to the library's
// static device array instead of plan->workspace.
int plan_call(const moe_shape *shape, const int32_t *topk_idx, moe_plan_t *plan, void *stream, bool own_scratch) {
  Dims d;
  PlanView v;
  int rc = check_shape(shape, &d);
  if (rc != MOE_OK) return rc;
  if (!plan) return MOE_ERR_NULL;
  if (d.T > 0 && !topk_idx) return MOE_ERR_NULL;
  rc = check_plan(plan, true, &v);
  if (rc != MOE_OK) return rc;
  if (!aligned16(topk_idx)) return MOE_ERR_ALIGN;
  WarmRange warm;
  if (plan->prefetch && plan->prefetch_bytes > 0) {
    if (!aligned16(plan->prefetch) || plan->prefetch_bytes % 16 != 0) return MOE_ERR_ALIGN;
    const size_t bytes = plan->prefetch_bytes < (size_t)MOE_PREFETCH_MAX_BYTES ? plan->prefetch_bytes
                                                                                : (size_t)MOE_PREFETCH_MAX_BYTES;
    warm.ptr = plan->prefetch;
    warm.vecs = (long long)(bytes / 16);
  }
  d.order_tiles = v.order ? plan_order_tiles(d) : 0;
  hipStream_t s = (hipStream_t)stream;
  if (d.T == 0) return launch_status(launch_plan_empty(d, v, s));
  int32_t *tile_hist = nullptr;
  if (plan_uses_workspace(d.N)) {
    if (own_scratch) {
      if (workspace_need(shape) > (size_t)MOE_STATIC_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;
      void *p = nullptr;
      rc = static_scratch(&p);
      if (rc != MOE_OK) return rc;
      tile_hist = (int32_t *)p;
    } else {
      if (!plan->workspace || plan->workspace_bytes < workspace_need(shape)) return MOE_ERR_WORKSPACE;
      if (!aligned16(plan->workspace)) return MOE_ERR_ALIGN;
      tile_hist = (int32_t *)plan->workspace;
    }
  }
  return launch_status(launch_plan(d, topk_idx, v, tile_hist, warm, s));
}

}  // namespace

extern "C" {

int moe_workspace_bytes(const moe_shape *shape, size_t *out_bytes) {
  if (!out_bytes) return MOE_ERR_NULL;
  const int rc = check_shape(shape, nullptr);
  if (rc != MOE_OK) return rc;
  *out_bytes = workspace_need(shape);
  return MOE_OK;
}

int moe_window_rows(const moe_shape *shape, int64_t *out_rows) {
  if (!out_rows) return MOE_ERR_NULL;
  const int rc = check_shape(shape, nullptr);
  if (rc != MOE_OK) return rc;
  *out_rows = shape->region_stride_rows > 0 ? (int64_t)shape->R * shape->region_stride_rows
                                            : (int64_t)shape->T * shape->k;
  return MOE_OK;
}

int moe_resolve_schedule(const moe_shape *shape, int32_t *out_schedule) {
  if (!out_schedule) return MOE_ERR_NULL;
  const int rc = check_shape(shape, nullptr);
  if (rc != MOE_OK) return rc;
  *out_schedule = resolve(shape);
  return MOE_OK;
}

int moe_plan(const moe_shape *shape, const int32_t *topk_idx, moe_plan_t *plan, void *stream) {
  return plan_call(shape, topk_idx, plan, stream, false);
}

int moe_plan_static(const moe_shape *shape, const int32_t *topk_idx, moe_plan_t *plan, void *stream) {
  return plan_call(shape, topk_idx, plan, stream, true);
}

int moe_dispatch(const moe_shape *shape, const void *x, const int32_t *topk_idx, moe_plan_t *plan, void *window,
                 void *stream) {
  Dims d;
  PlanView v;
  int rc = check_shape(shape, &d);
  if (rc != MOE_OK) return rc;
  const bool decode = resolve(shape) == MOE_SCHEDULE_DECODE;
  if (!plan) return MOE_ERR_NULL;
  if (d.T > 0 && (!x || !window || (decode && !topk_idx))) return MOE_ERR_NULL;
  rc = check_plan(plan, decode, &v);
  if (rc != MOE_OK) return rc;
  if (!aligned16(x) || !aligned16(window) || (decode && !aligned16(topk_idx))) return MOE_ERR_ALIGN;
  if (ranges_overlap(x, token_bytes(d), window, window_bytes(d))) return MOE_ERR_OVERLAP;
  d.order_tiles = v.order ? plan_order_tiles(d) : 0;
  hipStream_t s = (hipStream_t)stream;
  if (d.T == 0) {
    return decode ? launch_status(launch_plan_empty(d, v, s)) : MOE_OK;
  }
  return launch_status(decode ? launch_decode_dispatch(d, x, topk_idx, v, window, s)
                              : launch_dispatch(d, x, v, window, s));
}

int moe_dispatch_quant(const moe_shape *shape, const void *x, const int32_t *topk_idx, moe_plan_t *plan,
                       void *window_q, float *window_scale, void *stream) {
  Dims d;
  PlanView v;
  int rc = check_shape(shape, &d);
  if (rc != MOE_OK) return rc;
  if (shape->dtype != MOE_DTYPE_BF16 || d.H16 > 4096) return MOE_ERR_SHAPE;
  const bool decode = resolve(shape) == MOE_SCHEDULE_DECODE;
  if (!plan) return MOE_ERR_NULL;
  if (d.T > 0 && (!x || !window_q || !window_scale || (decode && !topk_idx))) return MOE_ERR_NULL;
  rc = check_plan(plan, decode, &v);
  if (rc != MOE_OK) return rc;
  if (!aligned16(x) || !aligned16(window_q) || !aligned16(window_scale) || (decode && !aligned16(topk_idx)))
    return MOE_ERR_ALIGN;
  {
    const uint64_t rows = window_bytes(d) / ((uint64_t)d.H16 * 16u);
    if (ranges_overlap(x, token_bytes(d), window_q, rows * (uint64_t)d.H) ||
        ranges_overlap(x, token_bytes(d), window_scale, rows * sizeof(float)) ||
        ranges_overlap(window_q, rows * (uint64_t)d.H, window_scale, rows * sizeof(float)))
      return MOE_ERR_OVERLAP;
  }
  d.order_tiles = v.order ? plan_order_tiles(d) : 0;
  hipStream_t s = (hipStream_t)stream;
  if (d.T == 0) return decode ? launch_status(launch_plan_empty(d, v, s)) : MOE_OK;
  return launch_status(decode ? launch_decode_dispatch_quant(d, x, topk_idx, v, window_q, window_scale, s)
                              : launch_dispatch_quant(d, x, v, window_q, window_scale, s));
}

int moe_combine(const moe_shape *shape, const void *expert_out, const float *topk_w, const moe_plan_t *plan,
                void *y, void *stream) {
  Dims d;
  PlanView v;
  int rc = check_shape(shape, &d);
  if (rc != MOE_OK) return rc;
  if (!plan) return MOE_ERR_NULL;
  if (d.T > 0 && (!expert_out || !topk_w || !y)) return MOE_ERR_NULL;
  rc = check_plan(plan, false, &v);
  if (rc != MOE_OK) return rc;
  if (!aligned16(expert_out) || !aligned16(topk_w) || !aligned16(y)) return MOE_ERR_ALIGN;
  if (ranges_overlap(y, token_bytes(d), expert_out, window_bytes(d))) return MOE_ERR_OVERLAP;
  if (d.T == 0) return MOE_OK;
  return launch_status(launch_combine(d, expert_out, topk_w, v, y, (hipStream_t)stream));
}

const char *moe_last_launch_error(void) { return hipGetErrorString(g_last_hip_error); }

const char *moe_strerror(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_SHAPE: return "bad shape, dtype or schedule";
    case MOE_ERR_ALIGN: return "row bytes or a device pointer not 16-byte aligned";
    case MOE_ERR_OVERFLOW: return "branch or window row count exceeds int32";
    case MOE_ERR_WORKSPACE: return "plan workspace missing or too small";
    case MOE_ERR_LAUNCH: return "kernel launch failed";
    case MOE_ERR_OVERLAP: return "input and output buffers overlap";
    default: return "unknown status";
  }
}

}  // extern "C"
