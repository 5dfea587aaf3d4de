// Shared device code of the two schedules: turning per-expert counts into the plan's count / offset
// tables (paper, Section 5.2 "Prefill Notify"; Section 5.1, definition of the large offset o_{e,r}).
//
// Layout of the window: destination rank d owns a region; inside it the blocks of its experts follow
// each other; inside an expert's block the sub-blocks of the source ranks follow each other in rank
// order.  With
//   own[e]    = branches this rank sends to expert e                     (c^exp)
//   others[e] = branches all OTHER source ranks send to e                (column sum of M without row me)
//   pre[e]    = branches the source ranks BELOW this one send to e       (column sum of M over rows < me)
//   g         = exclusive scan over e of own + others
// the block of expert e starts at  B[e] = region_start(d) + g[e] - g[d*E_r]  and this rank's sub-block at
// o_{e,me} = B[e] + pre[e].  With one source rank others = pre = 0.
//
// Row numbers are int32.  With several sources the row total is device data (the sum of M); it is also
// accumulated in 64 bits, and when it reaches 2^31 no branch is placed and status[2] reports it.
#pragma once
#include "device_utils.h"
#include "launch.h"

namespace moe_rbf {

// First window row of expert e's whole block.  g = exclusive scan of the block sizes over ALL experts.
// Tight windows: region r starts where the previous one ends, so B[e] = g[e].
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

// Sums columns of a row-major int matrix src[rows][cols] with all threads of the workgroup: the columns
// are split over `parts` groups of threads that take every parts-th row; partial sums meet in LDS with
// integer atomics (counts: order-free).  all_sum[col] += sum over rows (without row `me` if SKIP_ME);
// before_sum[col] += sum over rows < me (if before_sum is given; only columns < before_cols).
// grand (optional, LDS, zeroed by the caller) += the sum of everything counted in all_sum, in 64 bits.
// The targets must hold their starting values before the call; the caller synchronises afterwards.
template <bool SKIP_ME>
__device__ __forceinline__ void sum_columns(const int32_t *__restrict__ src, int rows, int cols, int me,
                                            int *all_sum, int *before_sum, int before_cols,
                                            unsigned long long *grand = nullptr) {
  const int nthreads = blockDim.x;
  const int parts = max(1, nthreads / cols);
  const int tid = threadIdx.x;
  const bool live = parts == 1 || tid < parts * cols;      // every thread stays for the wave-wide sum below
  const int part = parts == 1 ? 0 : tid / cols;
  unsigned long long wide = 0;
  for (int col = parts == 1 ? tid : tid - part * cols; live && col < cols; col += nthreads) {
    int all = 0, bef = 0;
    const int32_t *p = src + col;
    for (int r0 = part; r0 < rows; r0 += parts * 16) {
      int v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int r = r0 + u * parts;
        v[u] = (r < rows && !(SKIP_ME && r == me)) ? p[(size_t)r * cols] : 0;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        all += v[u];
        wide += (unsigned)v[u];
        if (r0 + u * parts < me) bef += v[u];
      }
    }
    if (all) atomicAdd(&all_sum[col], all);
    if (before_sum && bef && col < before_cols) atomicAdd(&before_sum[col], bef);
  }
  if (grand) {                                             // one 64-bit LDS atomic per wave
    const unsigned long long wave_rows = wave_sum_u64(wide);
    if (lane_id() == 0 && wave_rows) atomicAdd(grand, wave_rows);
  }
}

// The tile histograms summed once for a workgroup that also emits the dispatch order list: besides the sums
// over all rows (all_sum) and over the rows in front of `me` (before_sum, columns < before_cols) it needs the
// same two sums restricted to the rows [st0, st1) of its stretch (st_all, st_before).  Same row split as
// sum_columns; one pass over the source instead of two.
__device__ __forceinline__ void sum_columns_stretch(const int32_t *__restrict__ src, int rows, int cols, int me,
                                                    int st0, int st1, int *all_sum, int *before_sum, int *st_all,
                                                    int *st_before, int before_cols) {
  const int nthreads = blockDim.x;
  const int parts = max(1, nthreads / cols);
  const int tid = threadIdx.x;
  if (parts > 1 && tid >= parts * cols) return;
  const int part = parts == 1 ? 0 : tid / cols;
  for (int col = parts == 1 ? tid : tid - part * cols; col < cols; col += nthreads) {
    int all = 0, bef = 0, s_all = 0, s_bef = 0;
    const int32_t *p = src + col;
    for (int r0 = part; r0 < rows; r0 += parts * 16) {
      int v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int r = r0 + u * parts;
        v[u] = r < rows ? p[(size_t)r * cols] : 0;
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int r = r0 + u * parts;
        const int in_stretch = (r >= st0 && r < st1) ? v[u] : 0;
        all += v[u];
        s_all += in_stretch;
        if (r < me) bef += v[u], s_bef += in_stretch;
      }
    }
    if (all) atomicAdd(&all_sum[col], all);
    if (s_all) atomicAdd(&st_all[col], s_all);
    if (col < before_cols) {
      if (bef) atomicAdd(&before_sum[col], bef);
      if (s_bef) atomicAdd(&st_before[col], s_bef);
    }
  }
}

// Do the rows of all sources together reach 2^31?  others_rows: 64-bit sum of the other sources' counts;
// all_rows_low: the int32 sum (possibly wrapped) of own + others; this rank's own count is below 2^31, so
// it is the difference of the two low words.
__device__ __forceinline__ bool rows_overflow(unsigned long long others_rows, int all_rows_low) {
  const unsigned own = (unsigned)all_rows_low - (unsigned)others_rows;
  return others_rows + own >= (1ull << 31);
}

// One workgroup writes expert_count, rank_count, expert_offset, region_base, recv_count, recv_offset and
// status from LDS copies of own[0..E) (count bits selected by `mask`), others/pre (nullptr with a single
// source rank) and g[0..E].  Must be called by every thread of the workgroup.
// Branches dropped for capacity: this rank's sub-block of expert e covers rows [o, o + own); the part at
// or past the region's end is dropped.  overflow: the row total does not fit in int32 (the offset tables
// are then meaningless and status[2] says so).
__device__ __forceinline__ void write_plan_tables(const int *own, const int *others, const int *pre, const int *g,
                                                  const Dims &d, const PlanView &p, int n_invalid, int *lds_counter,
                                                  bool overflow = false, int mask = -1) {
  const int nthreads = blockDim.x;
  const bool fixed = d.stride > 0;
  if (threadIdx.x == 0) *lds_counter = 0;
  __syncthreads();
  int dropped = 0;
  for (int e = threadIdx.x; e < d.E; e += nthreads) {
    const int c = own[e] & mask;
    const int block = expert_first_row(g, e, d);
    const int o = block + (pre ? pre[e] : 0);
    const int all = c + (others ? others[e] : 0);
    p.expert_count[e] = c;
    p.expert_offset[e] = o;
    if (p.recv_count) p.recv_count[e] = all;
    if (p.recv_offset) p.recv_offset[e] = block;
    if (fixed) dropped += min(c, max(0, o + c - region_row_limit(e, d)));
    if (e == d.E - 1) {
      p.expert_offset[d.E] = block + all;
      if (p.recv_offset) p.recv_offset[d.E] = block + all;
      p.region_base[d.R] = fixed ? (int)(d.R * d.stride) : g[d.E];
    }
  }
  for (int r = threadIdx.x; r < d.R; r += nthreads) {
    int c = 0;
    for (int e = r * d.Er; e < (r + 1) * d.Er; ++e) c += own[e] & mask;
    p.rank_count[r] = c;
    p.region_base[r] = fixed ? (int)(r * d.stride) : g[r * d.Er];
  }
  if (dropped) atomicAdd(lds_counter, dropped);
  __syncthreads();
  if (threadIdx.x == 0) {
    p.status[0] = n_invalid;
    p.status[1] = overflow ? 0 : *lds_counter;
    p.status[2] = overflow ? 1 : 0;
  }
}

// One workgroup builds the whole histogram from the routing ids themselves (counts only: LDS integer
// atomics) and writes the tables.  Used where no per-tile histograms exist: the fused decode dispatch and
// the single-launch plan.  LDS: 4E + 3 ints.  Must be called by every thread of the workgroup.
__device__ __forceinline__ void tables_from_ids_block(const int32_t *__restrict__ K, const Dims &d, const PlanView &p,
                                                    int *lds) {
  const int E = d.E, tid = threadIdx.x, nthreads = blockDim.x;
  int *total = lds;            // [E]
  int *g = total + E;          // [E+1]
  int *others = g + E + 1;     // [E]  several source ranks only
  int *pre = others + E;       // [E]
  int *misc = pre + E;         // [2]
  __shared__ unsigned long long others_rows;
  const bool multi = p.source_count != nullptr;
  for (int e = tid; e < E; e += nthreads) {
    total[e] = 0;
    others[e] = 0;
    pre[e] = 0;
  }
  if (tid == 0) misc[0] = 0, others_rows = 0;
  __syncthreads();
  for (int i = tid; i < d.N; i += nthreads) {
    const int e = K[i];
    if (e >= 0 && e < E) atomicAdd(&total[e], 1);
    else if (e != -1) atomicAdd(&misc[0], 1);
  }
  if (multi) sum_columns<true>(p.source_count, d.R, E, d.me, others, pre, E, &others_rows);
  __syncthreads();
  if (tid < kWave) wave_exclusive_scan_lds(total, g, E, -1, multi ? others : nullptr);
  __syncthreads();
  write_plan_tables(total, multi ? others : nullptr, multi ? pre : nullptr, g, d, p, misc[0], misc + 1,
                    multi && rows_overflow(others_rows, g[E]));
}

}  // namespace moe_rbf
