// Dispatch: direct placement of token rows into destination expert windows (paper, Section 5.2
// "Prefill Dispatch", Section 5.3 "Decode Dispatch"; first loop of Algorithms 1 and 2).
// No staging copy exists: HBM traffic is T*H bytes read and T*k*H bytes written.
//
// Prefill schedule (row map from moe_plan): XCD-affine column slices, see dispatch_slices_kernel.
// Decode schedule: ONE launch.  Every workgroup rebuilds the plan values it needs from the routing
//   ids (LDS histogram of all ids with the count of ids before its token packed into the same word,
//   exclusive scan), so counts, offsets, small offsets and payload placement need no grid-wide
//   synchronisation; the chunk-0 workgroup of a token records that token's s and row map and
//   workgroup 0 records the tables that combine and the expert stage read.
//   The kernel is latency-bound (a few microseconds), so its hot path is kept small in code size:
//   rare paths are branched over.
#include "device_utils.h"
#include "launch.h"
#include "plan_tables.h"

namespace moe_rbf {

#ifndef MOE_DECODE_BLOCK
#define MOE_DECODE_BLOCK 448
#endif
#ifndef MOE_DECODE_VEC
#define MOE_DECODE_VEC 1
#endif

constexpr int kSlices = 8;   // column slices per row = XCDs per device

// Prefill dispatch.  Work unit = (J consecutive branches of one token, column slice c of 8).
// Workgroup b handles slice c = b % 8.  Workgroups are handed to the 8 XCDs round-robin, so XCD c only
// ever touches column slice c: the k re-reads of X[t]'s slice by the branches of a token hit in that
// XCD's L2 (X is fetched from HBM once), every wave issues few 16-byte stores per lane, and the 8 XCDs
// together lay down whole destination rows.  Stores are streaming (nontemporal) so that they do not
// evict the X slices from L2; loads are ordinary so that they stay.
// (If the hardware maps workgroups differently the result is unchanged; only the L2 reuse is lost.)
template <int BLOCK, int J>
__global__ __launch_bounds__(BLOCK) void dispatch_slices_kernel(const u32x4 *__restrict__ X,
                                                                const int32_t *__restrict__ row_map,
                                                                u32x4 *__restrict__ window, int k, int H16, int slice) {
  const int g = blockIdx.x / kSlices;
  const int c = blockIdx.x - g * kSlices;
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
      if (row[u] >= 0) store_stream(window + (size_t)row[u] * (size_t)H16 + col, v);
  }
}

// ---- decode -------------------------------------------------------------------------------------

// Rows of a token with more slots than one wave can rank with ballots (k > 64): plain loops.
__device__ __forceinline__ void decode_rows_large_k(const int *tok, const int *packed, const int *g, int *rows,
                                                 const Dims &d, const PlanView &p, int first, bool record) {
  for (int j = threadIdx.x; j < d.k; j += blockDim.x) {
    const int e = tok[j];
    int s = -1, row = -1;
    if (e >= 0 && e < d.E) {
      int dup = 0;
      for (int jp = 0; jp < j; ++jp) dup += (tok[jp] == e);
      s = (packed[e] >> 16) + dup;
      row = expert_first_row(g, e, d) + s;
      if (row >= region_row_limit(e, d)) row = -1;
    }
    rows[j] = row;
    if (record) {
      if (p.send_idx) p.send_idx[first + j] = s;
      p.row_map[first + j] = row;
    }
  }
}

template <int BLOCK, int V>
__global__ __launch_bounds__(BLOCK) void decode_dispatch_kernel(const u32x4 *__restrict__ X,
                                                                const int32_t *__restrict__ K,
                                                                u32x4 *__restrict__ window, Dims d, PlanView p,
                                                                int chunks) {
  extern __shared__ int lds[];
  const int E = d.E;
  int *total = lds;              // [E]   low half: c^exp; high half: branches of expert e with a flat index
                                 //       below this token's first slot
  int *g = total + E;            // [E+1] exclusive scan of c^exp
  int *rows = g + E + 1;         // [k]   destination rows of this token
  int *tok = rows + d.k;         // [k]   routing ids of this token
  int *misc = tok + d.k;         // [2]   {invalid ids, scratch counter}
  const int tid = threadIdx.x;
  const int t = blockIdx.x / chunks;
  const int c = blockIdx.x - t * chunks;
  const int first = t * d.k;

  // everything that comes from memory is requested up front: payload, all routing ids, own ids
  const int col0 = c * (BLOCK * V) + tid;
  const u32x4 *src = X + (size_t)t * (size_t)d.H16;
  u32x4 v[V];
#pragma unroll
  for (int x = 0; x < V; ++x) {
    const int col = col0 + x * BLOCK;
    v[x] = col < d.H16 ? load_stream(src + col) : u32x4{0u, 0u, 0u, 0u};
  }
  constexpr int kIds = 4;        // ids per thread and pass
  int id[kIds];
#pragma unroll
  for (int u = 0; u < kIds; ++u) {
    const int i = u * BLOCK + tid;
    id[u] = i < d.N ? K[i] : -1;
  }
  for (int j = tid; j < d.k; j += BLOCK) tok[j] = K[first + j];
  for (int e = tid; e < E; e += BLOCK) total[e] = 0;
  if (tid == 0) misc[0] = 0;
  __syncthreads();

  // one LDS atomic per id: +1 counts the id, +0x10000 also counts it as "before this token"
  // (T*k <= 8192, so neither half can overflow 16 bits)
  for (int i0 = 0; i0 < d.N; i0 += BLOCK * kIds) {
#pragma unroll
    for (int u = 0; u < kIds; ++u) {
      const int i = i0 + u * BLOCK + tid;
      const int e = i0 == 0 ? id[u] : (i < d.N ? K[i] : -1);
      if (e >= 0 && e < E) atomicAdd(&total[e], i < first ? 0x10001 : 1);
      else if (e != -1) atomicAdd(&misc[0], 1);
    }
  }
  __syncthreads();
  if (tid < kWave) wave_exclusive_scan_lds(total, g, E, 0xffff);
  __syncthreads();

  // small offset = count in earlier tokens + earlier slots of this token with the same id
  if (d.k <= kWave) {
    if (tid < kWave) {   // one wave: equal ids among the token's slots are found with ballots
      const bool in = tid < d.k;
      const int e = in ? tok[tid] : -1;
      const bool valid = e >= 0 && e < E;
      const unsigned long long peers = match_any(e, valid, id_bits(E));
      int s = -1, row = -1;
      if (valid) {
        s = (total[e] >> 16) + __popcll(peers & ((1ull << tid) - 1ull));
        row = expert_first_row(g, e, d) + s;
        if (row >= region_row_limit(e, d)) row = -1;
      }
      if (in) {
        rows[tid] = row;
        if (c == 0) {
          if (p.send_idx) p.send_idx[first + tid] = s;
          p.row_map[first + tid] = row;
        }
      }
    }
  } else {
    decode_rows_large_k(tok, total, g, rows, d, p, first, c == 0);
  }
  if (blockIdx.x == 0) write_plan_tables(total, g, d, p, misc[0], misc + 1, 0xffff);
  __syncthreads();

  // fan the chunk out to the token's destination rows; lane j of every wave holds row j of a batch of
  // up to 64 slots, so the loop reads LDS once and then only moves lanes into scalar registers
  for (int j0 = 0; j0 < d.k; j0 += kWave) {
    const int slot = j0 + (tid & (kWave - 1));
    const int mine = slot < d.k ? rows[slot] : -1;
    const int nb = min(kWave, d.k - j0);
    for (int j = 0; j < nb; ++j) {
      const int row = __builtin_amdgcn_readlane(mine, j);
      if (row < 0) continue;
      u32x4 *dst = window + (size_t)row * (size_t)d.H16;
#pragma unroll
      for (int x = 0; x < V; ++x) {
        const int col = col0 + x * BLOCK;
        if (col < d.H16) store_stream(dst + col, v[x]);
      }
    }
  }
}

hipError_t launch_dispatch(const Dims &d, const void *x, const PlanView &p, void *window, hipStream_t s) {
  // several branches of a token per workgroup when a slice is short, so that the number of workgroups
  // stays within what the dispatcher sustains
  const int slice = (d.H16 + kSlices - 1) / kSlices;
  const int slice_bytes = slice * 16;
  const int want = slice <= 64 ? 4096 : 1792;
  int J = 1;
  while (J < 8 && J * slice_bytes < want && d.k % (2 * J) == 0) J *= 2;
  const dim3 grid((unsigned)(d.N / J) * (unsigned)kSlices);
  const u32x4 *xs = (const u32x4 *)x;
  u32x4 *win = (u32x4 *)window;
  const int32_t *rm = p.row_map;
  switch (J) {
    case 1: return launch(dispatch_slices_kernel<128, 1>, grid, dim3(128), 0, s, xs, rm, win, d.k, d.H16, slice);
    case 2: return launch(dispatch_slices_kernel<128, 2>, grid, dim3(128), 0, s, xs, rm, win, d.k, d.H16, slice);
    case 4: return launch(dispatch_slices_kernel<128, 4>, grid, dim3(128), 0, s, xs, rm, win, d.k, d.H16, slice);
    default: return launch(dispatch_slices_kernel<128, 8>, grid, dim3(128), 0, s, xs, rm, win, d.k, d.H16, slice);
  }
}

hipError_t launch_decode_dispatch(const Dims &d, const void *x, const int32_t *K, const PlanView &p, void *window,
                                  hipStream_t s) {
  constexpr int B = MOE_DECODE_BLOCK, V = MOE_DECODE_VEC;
  const int chunks = (d.H16 + B * V - 1) / (B * V);
  const size_t lds = (size_t)(2 * d.E + 1 + 2 * d.k + 2) * sizeof(int);
  return launch(decode_dispatch_kernel<B, V>, dim3((unsigned)d.T * (unsigned)chunks), dim3(B), lds, s,
                (const u32x4 *)x, K, (u32x4 *)window, d, p, chunks);
}

}  // namespace moe_rbf
