// Dispatch: direct placement of token rows into destination expert windows (paper, Section 5.2
// "Prefill Dispatch", Section 5.3 "Decode Dispatch"; first loop of Algorithms 1 and 2).
//
// Work unit = (token, column chunk).  A workgroup loads its chunk of row X[t] ONCE with 16-byte
// loads and stores it to the k destination rows, so the HBM traffic is the algorithmic one:
// T*H bytes read, T*k*H bytes written, no staging copy.  Destinations are whole contiguous rows,
// so every store instruction of a wave covers 1 KiB of consecutive addresses.
// No reuse exists between workgroups (each row segment is read once), so the order in which
// workgroups land on the 8 XCDs does not matter for L2.
//
// (That token-major fan-out is the decode kernel.  The prefill kernel is organised differently, see
// dispatch_slices_kernel.)
// Prefill schedule: the row map comes from moe_plan.
// Decode schedule : every workgroup rebuilds the plan values it needs from the routing ids in LDS
//   (histogram of all ids, histogram of the ids before its token, exclusive scan), so counts,
//   offsets, small offsets and payload placement happen in ONE launch with no grid-wide
//   synchronisation; the chunk-0 workgroup of a token records that token's s and row map and
//   workgroup 0 records the tables for combine.
#include "device_utils.h"
#include "launch.h"
#include "plan_tables.h"

namespace moe_rbf {

#ifndef MOE_DISPATCH_BLOCK
#define MOE_DISPATCH_BLOCK 128
#endif
#ifndef MOE_DISPATCH_VEC
#define MOE_DISPATCH_VEC 0   // 0 = pick from the row length
#endif
#ifndef MOE_DECODE_BLOCK
#define MOE_DECODE_BLOCK 128
#endif
#ifndef MOE_DECODE_VEC
#define MOE_DECODE_VEC 1
#endif
#ifndef MOE_DISPATCH_NT
#define MOE_DISPATCH_NT 1
#endif
#ifndef MOE_DISPATCH_SLICES
#define MOE_DISPATCH_SLICES 1
#endif
constexpr int kSlices = 8;   // column slices per row = XCDs per device
#if MOE_DISPATCH_NT
#define MOE_DISPATCH_STORE(p, v) store_stream(p, v)
#else
#define MOE_DISPATCH_STORE(p, v) (*(p) = (v))
#endif

constexpr int kRowBatch = 8;  // destination rows whose indices are fetched together

// Stores the V vectors held in v[] to every placed destination row of token t.
template <int BLOCK, int V>
__device__ __forceinline__ void scatter_rows(const u32x4 (&v)[V], const int32_t *rows, int k, u32x4 *window, int H16,
                                             int col0) {
  for (int j0 = 0; j0 < k; j0 += kRowBatch) {
    int row[kRowBatch];
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) row[u] = (j0 + u < k) ? uniform(rows[j0 + u]) : -1;
#pragma unroll
    for (int u = 0; u < kRowBatch; ++u) {
      if (row[u] < 0) continue;
      u32x4 *dst = window + (size_t)row[u] * (size_t)H16;
#pragma unroll
      for (int x = 0; x < V; ++x) {
        const int col = col0 + x * BLOCK;
        if (col < H16) MOE_DISPATCH_STORE(dst + col, v[x]);
      }
    }
  }
}

template <int BLOCK, int V>
__global__ __launch_bounds__(BLOCK) void dispatch_rows_kernel(const u32x4 *__restrict__ X,
                                                              const int32_t *__restrict__ row_map,
                                                              u32x4 *__restrict__ window, int k, int H16, int chunks) {
  const int t = blockIdx.x / chunks;
  const int c = blockIdx.x - t * chunks;
  const int col0 = c * (BLOCK * V) + threadIdx.x;
  const u32x4 *src = X + (size_t)t * (size_t)H16;
  u32x4 v[V];
#pragma unroll
  for (int x = 0; x < V; ++x) {
    const int col = col0 + x * BLOCK;
    v[x] = col < H16 ? load_stream(src + col) : u32x4{0u, 0u, 0u, 0u};
  }
  scatter_rows<BLOCK, V>(v, row_map + (size_t)t * k, k, window, H16, col0);
}

// Prefill dispatch, XCD-affine column slices.  Work unit = (branch n = t*k+j, column slice c of 8).
// Workgroup b handles slice c = b % 8 of branch n = b / 8.  Workgroups are handed to the 8 XCDs
// round-robin, so XCD c only ever touches column slice c: the k re-reads of X[t]'s slice by the k
// consecutive branches of a token hit in that XCD's L2 (X is fetched from HBM once), every wave issues
// a single 16-byte store per lane, and the 8 XCDs together lay down whole destination rows.
// (If the hardware maps workgroups differently the result is unchanged; only the L2 reuse is lost.)
template <int BLOCK, int J>
__global__ __launch_bounds__(BLOCK) void dispatch_slices_kernel(const u32x4 *__restrict__ X,
                                                                const int32_t *__restrict__ row_map,
                                                                u32x4 *__restrict__ window, int k, int H16, int slice,
                                                                int nslices) {
  const int g = blockIdx.x / nslices;
  const int c = blockIdx.x - g * nslices;
  const int n = g * J;                       // J consecutive branches of one token (J divides k)
  int row[J];
#pragma unroll
  for (int u = 0; u < J; ++u) row[u] = uniform(row_map[n + u]);
  const int t = n / k;
  const int end = min((c + 1) * slice, H16);
  const u32x4 *src = X + (size_t)t * (size_t)H16;
  for (int col = c * slice + threadIdx.x; col < end; col += BLOCK) {
    const u32x4 v = src[col];
#pragma unroll
    for (int u = 0; u < J; ++u)
      if (row[u] >= 0) MOE_DISPATCH_STORE(window + (size_t)row[u] * (size_t)H16 + col, v);
  }
}

template <int BLOCK, int V>
__global__ __launch_bounds__(BLOCK) void decode_dispatch_kernel(const u32x4 *__restrict__ X,
                                                                const int32_t *__restrict__ K,
                                                                u32x4 *__restrict__ window, Dims d, PlanView p,
                                                                int chunks) {
  extern __shared__ int lds[];
  const int E = d.E;
  int *total = lds;              // [E]   c^exp
  int *before = total + E;       // [E]   branches of expert e in earlier tokens
  int *g = before + E;           // [E+1] exclusive scan of total
  int *rows = g + E + 1;         // [k]   destination rows of this token
  int *misc = rows + d.k;        // [2]   {invalid ids, scratch counter}
  const int tid = threadIdx.x;
  const int t = blockIdx.x / chunks;
  const int c = blockIdx.x - t * chunks;

  // payload loads are issued first so that they are in flight while the plan is rebuilt
  const int col0 = c * (BLOCK * V) + tid;
  const u32x4 *src = X + (size_t)t * (size_t)d.H16;
  u32x4 v[V];
#pragma unroll
  for (int x = 0; x < V; ++x) {
    const int col = col0 + x * BLOCK;
    v[x] = col < d.H16 ? load_stream(src + col) : u32x4{0u, 0u, 0u, 0u};
  }

  for (int e = tid; e < 2 * E; e += BLOCK) lds[e] = 0;
  if (tid == 0) misc[0] = 0;
  __syncthreads();
  // counts of all ids, and of the ids with a smaller flat index than this token's first slot
  const int first = t * d.k;
  for (int i = tid; i < d.N; i += BLOCK) {
    const int e = K[i];
    if (e >= 0 && e < E) {
      atomicAdd(&total[e], 1);
      if (i < first) atomicAdd(&before[e], 1);
    } else if (e != -1) {
      atomicAdd(&misc[0], 1);
    }
  }
  __syncthreads();
  if (tid < kWave) wave_exclusive_scan_lds(total, g, E);
  __syncthreads();
  // small offset = earlier tokens' count + earlier slots of this token with the same id
  for (int j = tid; j < d.k; j += BLOCK) {
    const int e = K[first + j];
    int s = -1, row = -1;
    if (e >= 0 && e < E) {
      int dup = 0;
      for (int jp = 0; jp < j; ++jp) dup += (K[first + jp] == e);
      s = before[e] + dup;
      row = expert_first_row(g, e, d) + s;
      if (row >= region_row_limit(e, d)) row = -1;
    }
    rows[j] = row;
    if (c == 0) {
      if (p.send_idx) p.send_idx[first + j] = s;
      p.row_map[first + j] = row;
    }
  }
  if (blockIdx.x == 0) write_plan_tables(total, g, d, p, misc[0], misc + 1);
  __syncthreads();
  scatter_rows<BLOCK, V>(v, rows, d.k, window, d.H16, col0);
}

template <int BLOCK, int V>
static hipError_t launch_dispatch_cfg(const Dims &d, const void *x, const PlanView &p, void *window, hipStream_t s) {
  const int chunks = (d.H16 + BLOCK * V - 1) / (BLOCK * V);
  return launch(dispatch_rows_kernel<BLOCK, V>, dim3((unsigned)d.T * (unsigned)chunks), dim3(BLOCK), 0, s,
                (const u32x4 *)x, (const int32_t *)p.row_map, (u32x4 *)window, d.k, d.H16, chunks);
}

hipError_t launch_dispatch(const Dims &d, const void *x, const PlanView &p, void *window, hipStream_t s) {
  constexpr int B = MOE_DISPATCH_BLOCK;
#if MOE_DISPATCH_SLICES
  {
    // one wave per slice when a slice is <= 64 vectors; several branches of a token per workgroup when
    // a slice is short, so that the workgroup count stays within what the dispatcher sustains
    const int slice = (d.H16 + kSlices - 1) / kSlices;
    const int slice_bytes = slice * 16;
    const int want = slice <= 64 ? 4096 : 1792;
    int J = 1;
    while (J < 8 && J * slice_bytes < want && d.k % (2 * J) == 0) J *= 2;
    const dim3 grid((unsigned)(d.N / J) * (unsigned)kSlices);
    const u32x4 *xs = (const u32x4 *)x;
    u32x4 *win = (u32x4 *)window;
#define MOE_GO(B_, J_) \
  return launch(dispatch_slices_kernel<B_, J_>, grid, dim3(B_), 0, s, xs, (const int32_t *)p.row_map, win, d.k, d.H16, \
                slice, kSlices)
    if (J == 1) MOE_GO(128, 1);
    if (J == 2) MOE_GO(128, 2);
    if (J == 4) MOE_GO(128, 4);
    MOE_GO(128, 8);
#undef MOE_GO
  }
#endif
#if MOE_DISPATCH_VEC > 0
  return launch_dispatch_cfg<B, MOE_DISPATCH_VEC>(d, x, p, window, s);
#else
  // vectors per thread chosen so that a row splits into few, evenly filled chunks
  if (d.H16 % (B * 7) == 0) return launch_dispatch_cfg<B, 7>(d, x, p, window, s);
  if (d.H16 % (B * 4) == 0) return launch_dispatch_cfg<B, 4>(d, x, p, window, s);
  if (d.H16 >= B * 2) return launch_dispatch_cfg<B, 2>(d, x, p, window, s);
  return launch_dispatch_cfg<B, 1>(d, x, p, window, s);
#endif
}

hipError_t launch_decode_dispatch(const Dims &d, const void *x, const int32_t *K, const PlanView &p, void *window,
                                  hipStream_t s) {
  constexpr int B = MOE_DECODE_BLOCK, V = MOE_DECODE_VEC;
  const int chunks = (d.H16 + B * V - 1) / (B * V);
  const size_t lds = (size_t)(3 * d.E + 1 + d.k + 2) * sizeof(int);
  return launch(decode_dispatch_kernel<B, V>, dim3((unsigned)d.T * (unsigned)chunks), dim3(B), lds, s,
                (const u32x4 *)x, K, (u32x4 *)window, d, p, chunks);
}

}  // namespace moe_rbf
