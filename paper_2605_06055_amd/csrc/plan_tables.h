// Shared device code of the two schedules: turning the per-expert totals and their exclusive scan
// into the plan's count / offset tables (paper, Section 5.2 "Prefill Notify", single source rank).
#pragma once
#include "device_utils.h"
#include "launch.h"

namespace moe_rbf {

// First window row of expert e's block.  g = exclusive scan of the counts over ALL experts.
// Tight windows: region r starts where the previous one ends, so o[e] = g[e].
// Fixed stride : region r starts at r*stride and expert blocks are packed from there.
__device__ __forceinline__ int expert_first_row(const int *g, int e, const Dims &d) {
  if (d.stride <= 0) return g[e];
  const int r = e / d.Er;
  return (int)(r * d.stride) + g[e] - g[r * d.Er];
}

// First row past the rank region that holds expert e (no limit for tight windows).
__device__ __forceinline__ int region_row_limit(int e, const Dims &d) {
  return d.stride > 0 ? (int)((e / d.Er + 1) * d.stride) : 0x7fffffff;
}

// One workgroup writes expert_count, rank_count, expert_offset, region_base and status from LDS
// copies of total[0..E) and g[0..E].  Must be called by every thread of the workgroup.
// Branches dropped for capacity: rows of region r are packed, so exactly max(0, c_rank[r] - stride)
// of them fall past the region's end.
// Only the bits of total[] selected by `mask` are counts.
__device__ __forceinline__ void write_plan_tables(const int *total, const int *g, const Dims &d, const PlanView &p,
                                                  int n_invalid, int *lds_counter, int mask = -1) {
  const int nthreads = blockDim.x;
  const bool fixed = d.stride > 0;
  for (int e = threadIdx.x; e < d.E; e += nthreads) {
    p.expert_count[e] = total[e] & mask;
    p.expert_offset[e] = expert_first_row(g, e, d);
  }
  if (threadIdx.x == 0) {
    p.expert_offset[d.E] = expert_first_row(g, d.E - 1, d) + (total[d.E - 1] & mask);
    p.region_base[d.R] = fixed ? (int)(d.R * d.stride) : g[d.E];
    *lds_counter = 0;
  }
  __syncthreads();
  int dropped = 0;
  for (int r = threadIdx.x; r < d.R; r += nthreads) {
    const int c = g[(r + 1) * d.Er] - g[r * d.Er];
    p.rank_count[r] = c;
    p.region_base[r] = fixed ? (int)(r * d.stride) : g[r * d.Er];
    if (fixed && c > d.stride) dropped += c - (int)d.stride;
  }
  if (dropped) atomicAdd(lds_counter, dropped);
  __syncthreads();
  if (threadIdx.x == 0) {
    p.status[0] = n_invalid;
    p.status[1] = *lds_counter;
  }
}

}  // namespace moe_rbf
