// Combine: direct reading of expert outputs from the windows and local weighted reduction in token
// order (paper, Section 5.2 "Prefill Combine", Section 5.3 "Decode Combine"; second loop of
// Algorithms 1 and 2):  Y[t,:] = sum_j W[t,j] * Yexp[row_map[t,j], :].
//
// Work unit = (token, 16-byte output column); workgroups of one or two waves, or, for large launches, a
// persistent grid whose threads hold their results back until a round's loads are done.  A thread fetches its column from up to 8 window rows
// at once (8 independent 16-byte loads in flight per lane), folds them into fp32 accumulators in
// ascending j with one fused multiply-add per branch, rounds once and stores 16 bytes.  Every window
// row is read exactly once and Y is written exactly once, in token order: no un-permute buffer.
// Row ids and weights are uniform per workgroup and live in scalar registers.
#include <atomic>

#include "device_utils.h"
#include "launch.h"
#include "moe_rbf.h"

namespace moe_rbf {

#ifndef MOE_COMBINE_BLOCK
#define MOE_COMBINE_BLOCK 128
#endif

constexpr int kGather = 8;  // rows fetched together

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// two bf16 packed in a dword -> two floats (exact)
__device__ __forceinline__ float bf16_lo(unsigned u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __uint_as_float(u & 0xffff0000u); }
// two floats -> two bf16, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 f;
  f.x = lo;
  f.y = hi;
  return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}

template <int DT>
struct Acc;

template <>
struct Acc<MOE_DTYPE_BF16> {
  float a[8];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = 0.0f;
  }
  __device__ __forceinline__ void fma(float w, u32x4 y) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[2 * i] = __builtin_fmaf(w, bf16_lo(y[i]), a[2 * i]);
      a[2 * i + 1] = __builtin_fmaf(w, bf16_hi(y[i]), a[2 * i + 1]);
    }
  }
  __device__ __forceinline__ u32x4 result() const {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = pack_bf16(a[2 * i], a[2 * i + 1]);
    return r;
  }
};

template <>
struct Acc<MOE_DTYPE_F32> {
  float a[4];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = 0.0f;
  }
  __device__ __forceinline__ void fma(float w, u32x4 y) {
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = __builtin_fmaf(w, __uint_as_float(y[i]), a[i]);
  }
  __device__ __forceinline__ u32x4 result() const {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(a[i]);
    return r;
  }
};

// KFIX > 0: the routing degree is the compile-time constant KFIX (straight-line code, no bounds tests);
// KFIX == 0: any k, rows taken kGather at a time.
template <int BLOCK, int DT, int KFIX>
__global__ __launch_bounds__(BLOCK) void combine_rows_kernel(const u32x4 *__restrict__ Yexp,
                                                             const float *__restrict__ W,
                                                             const int32_t *__restrict__ row_map,
                                                             u32x4 *__restrict__ Y, int k_arg, int H16, int chunks) {
  const int k = KFIX > 0 ? KFIX : k_arg;
  const int t = blockIdx.x / chunks;
  const int c = blockIdx.x - t * chunks;
  const int col = c * BLOCK + threadIdx.x;
  if (col >= H16) return;
  // both arrays are 16-byte aligned (checked at the boundary): lets the scalar loads be wide
  const int32_t *rows = (const int32_t *)__builtin_assume_aligned(row_map, 16) + (size_t)t * k;
  const float *w = (const float *)__builtin_assume_aligned(W, 16) + (size_t)t * k;
  const u32x4 *base = Yexp + col;
  Acc<DT> acc;
  acc.zero();
  constexpr int G = KFIX > 0 ? (KFIX < kGather ? KFIX : kGather) : kGather;
  for (int j0 = 0; j0 < k; j0 += G) {
    int row[G];
    float wj[G];
    u32x4 y[G];
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const bool in = (KFIX > 0 && KFIX % G == 0) || j0 + u < k;
      row[u] = in ? uniform(rows[j0 + u]) : -1;
      wj[u] = in ? __uint_as_float(uniform(__float_as_uint(w[j0 + u]))) : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < G; ++u)
      y[u] = row[u] >= 0 ? load_stream(base + (size_t)row[u] * (size_t)H16) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < G; ++u)
      if (row[u] >= 0) acc.fma(wj[u], y[u]);
  }
  store_stream(Y + (size_t)t * (size_t)H16 + col, acc.result());
}

// Large launches: a persistent grid, one workgroup of 8 waves per compute unit, whose threads keep the results
// of R units in registers and store them only after the last row load of the round.  All waves run the same
// amount of work, so chip-wide the reads come first and the 11 % of writes follow in a burst instead of being
// mixed into the read stream (measured inside plan -> dispatch -> combine layers, H = 7168, k = 8, R = 28:
// T = 4096 179.3-180.0 against 184.4-185.3 us per layer, T = 8192 351.6 / 360.4, Zipf T = 16384 676.6 / 681.3).
// T = 4096 is exactly one round of 28 units per thread on 256 CUs.  Same arithmetic as combine_rows_kernel
// (ascending j, one fma per placed branch, one rounding).  Units (token, column) are numbered token-major over
// columns padded to a multiple of 64, so that a wave stays inside one token.
constexpr int kDeferBlock = 512;
constexpr int kDeferUnits = 28;

template <int DT, int KFIX>
__global__ __launch_bounds__(kDeferBlock) void combine_deferred_kernel(const u32x4 *__restrict__ Yexp,
                                                                       const float *__restrict__ W,
                                                                       const int32_t *__restrict__ row_map,
                                                                       u32x4 *__restrict__ Y, int k_arg, int H16,
                                                                       int cols_pad, int units, int dq, int dr,
                                                                       int first) {
  // this launch covers units [first, units)
  constexpr int R = kDeferUnits;
  const int k = KFIX > 0 ? KFIX : k_arg;
  constexpr int G = KFIX > 0 ? (KFIX < kGather ? KFIX : kGather) : kGather;
  const int nthreads = (int)gridDim.x * kDeferBlock;
  const int g = (int)blockIdx.x * kDeferBlock + (int)threadIdx.x;
  const int32_t *rm = (const int32_t *)__builtin_assume_aligned(row_map, 16);
  const float *wt = (const float *)__builtin_assume_aligned(W, 16);
  for (long long base = first; base < units; base += (long long)nthreads * R) {
    const long long u0 = base + g;
    const int t0 = (int)(u0 / cols_pad), col0 = (int)(u0 - (long long)t0 * cols_pad);
    u32x4 res[R];
    int t = t0, col = col0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (u0 + (long long)r * nthreads < units && col < H16) {     // the first test is uniform per wave
        const int ts = uniform(t);
        const int32_t *rows = rm + (size_t)ts * k;
        const float *w = wt + (size_t)ts * k;
        Acc<DT> acc;
        acc.zero();
        for (int j0 = 0; j0 < k; j0 += G) {
          int row[G];
          float wj[G];
          u32x4 y[G];
#pragma unroll
          for (int u = 0; u < G; ++u) {
            const bool in = (KFIX > 0 && KFIX % G == 0) || j0 + u < k;
            row[u] = in ? uniform(rows[j0 + u]) : -1;
            wj[u] = in ? __uint_as_float(uniform(__float_as_uint(w[j0 + u]))) : 0.0f;
          }
#pragma unroll
          for (int u = 0; u < G; ++u)
            y[u] = row[u] >= 0 ? load_stream(Yexp + (size_t)row[u] * (size_t)H16 + col) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
          for (int u = 0; u < G; ++u)
            if (row[u] >= 0) acc.fma(wj[u], y[u]);
        }
        res[r] = acc.result();
      }
      col += dr;
      t += dq;
      if (col >= cols_pad) col -= cols_pad, ++t;
    }
    t = t0, col = col0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (u0 + (long long)r * nthreads < units && col < H16) store_stream(Y + (size_t)t * (size_t)H16 + col, res[r]);
      col += dr;
      t += dq;
      if (col >= cols_pad) col -= cols_pad, ++t;
    }
  }
}

// Compute units of the current device (asked once per device; no allocation).  Calls may come from several host
// threads: the cache holds the same value whoever fills it.
static int device_cus() {
  static std::atomic<int> cus[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cus[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    cus[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

template <int DT>
static hipError_t launch_combine_deferred(const Dims &d, const void *expert_out, const float *W, const PlanView &p,
                                          void *y, int cols_pad, int units, hipStream_t s) {
  const int grid = device_cus();
  const int nthreads = grid * kDeferBlock;
  // Two rounds per launch: the workgroups drift apart over the rounds and reads and writes mix again; a kernel
  // boundary lines them up.  Measured inside layers, us per combine, one launch / one round per launch / two:
  // wide (4.6 rounds) 412 / 386 / 391, Zipf T = 16384 (4 rounds) 329 / 325 / 323, balanced T = 16384 332.5 / 331 / 329,
  // H = 4096: T = 8192 (1.1 rounds) 94.9 / 96.9 / 94.8, T = 16384 (2.3 rounds) 190.0 / 190.6 / 190.4.
  constexpr int kRoundsPerLaunch = 2;
  auto go = [&](auto kernel) {
    const long long per = (long long)nthreads * kDeferUnits * kRoundsPerLaunch;
    for (long long first = 0; first < units; first += per) {
      const long long end = first + per < units ? first + per : units;
      const hipError_t e = launch(kernel, dim3(grid), dim3(kDeferBlock), 0, s, (const u32x4 *)expert_out, W,
                                  (const int32_t *)p.row_map, (u32x4 *)y, d.k, d.H16, cols_pad, (int)end,
                                  nthreads / cols_pad, nthreads % cols_pad, (int)first);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  };
  switch (d.k) {
    case 8: return go(combine_deferred_kernel<DT, 8>);
    case 6: return go(combine_deferred_kernel<DT, 6>);
    default: return hipErrorInvalidValue;      // other routing degrees keep combine_rows_kernel (see launch_combine)
  }
}

template <int DT, int B>
static hipError_t launch_combine_dt(const Dims &d, const void *expert_out, const float *W, const PlanView &p, void *y,
                                    hipStream_t s) {
  const int chunks = (d.H16 + B - 1) / B;
  const dim3 grid((unsigned)d.T * (unsigned)chunks);
  auto go = [&](auto kernel) {
    return launch(kernel, grid, dim3(B), 0, s, (const u32x4 *)expert_out, W, (const int32_t *)p.row_map, (u32x4 *)y,
                  d.k, d.H16, chunks);
  };
  switch (d.k) {
    case 8: return go(combine_rows_kernel<B, DT, 8>);
    case 6: return go(combine_rows_kernel<B, DT, 6>);
    case 4: return go(combine_rows_kernel<B, DT, 4>);
    case 2: return go(combine_rows_kernel<B, DT, 2>);
    case 1: return go(combine_rows_kernel<B, DT, 1>);
    default: return go(combine_rows_kernel<B, DT, 0>);
  }
}

hipError_t launch_combine(const Dims &d, const void *expert_out, const float *W, const PlanView &p, void *y,
                          hipStream_t s) {
  // One-wave workgroups while the launch is small (latency-bound: every wave starts as early as possible),
  // two-wave workgroups once it streams.  Measured, H = 7168, k = 8, 64 / 128 threads: T = 128: 4.61 / 4.74 us,
  // T = 1024: 22.5 / 22.7, T = 2048: 43.1 / 43.0, T = 4096: 88.1 / 86.9.
  const bool small = (int64_t)d.T * d.H16 <= (int64_t)1536 * 1024;
  // Streaming launches with a routing degree of 6 or 8 take the deferred-store form.  Measured inside layers,
  // us per layer deferred / not: H = 7168: T = 2048 91.5 / 92.2, 3072 136.2 / 138.3, 4096 180.4 / 185.2,
  // 6144 264.9 / 267.7, 8192 348.1 / 355.2, 16384 702.9 / 713.1, Zipf 16384 673.5 / 681.8; H = 4096: T = 4096
  // 103.4 / 104.3, 16384 380.2 / 387.5, group-limited 32768 846.6 / 848.5; k = 4, T = 4096: 104.1 / 103.4 (no gain:
  // smaller degrees, and degrees without a compile-time form, whose results array the compiler would spill, stay).
  const int cols_pad = (d.H16 + 63) / 64 * 64;
  const long long units = (long long)d.T * cols_pad;
  if (!small && (d.k == 8 || d.k == 6) && units < 0x7fffffffLL)
    return d.dtype == MOE_DTYPE_BF16
               ? launch_combine_deferred<MOE_DTYPE_BF16>(d, expert_out, W, p, y, cols_pad, (int)units, s)
               : launch_combine_deferred<MOE_DTYPE_F32>(d, expert_out, W, p, y, cols_pad, (int)units, s);
  if (d.dtype == MOE_DTYPE_BF16)
    return small ? launch_combine_dt<MOE_DTYPE_BF16, 64>(d, expert_out, W, p, y, s)
                 : launch_combine_dt<MOE_DTYPE_BF16, MOE_COMBINE_BLOCK>(d, expert_out, W, p, y, s);
  return small ? launch_combine_dt<MOE_DTYPE_F32, 64>(d, expert_out, W, p, y, s)
               : launch_combine_dt<MOE_DTYPE_F32, MOE_COMBINE_BLOCK>(d, expert_out, W, p, y, s);
}

}  // namespace moe_rbf
