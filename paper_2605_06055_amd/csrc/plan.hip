// Prefill Layout + Notify for one source rank (paper, Section 5.2): per-expert and per-rank branch
// counts, large offsets o (exclusive scan of the counts inside each rank region), the stable small
// offset s of every branch and the row map o[K] + s.  No payload is touched.
//
// The small offset must be the number of EARLIER branches (smaller flat index t*k+j) with the same
// expert, so it cannot come from global atomics (arbitrary order).  It is built from counts per tile
// and a prefix over the tiles in front, the scheme the paper names for its Layout kernel:
//   pass 1  plan_tile_hist : one workgroup per tile of branches -> LDS histogram -> tile_hist[tile][E+1]
//                            (slot E counts ids outside [0,E) other than -1)
//   pass 2  plan_rank      : one workgroup (16 waves) per tile.  Column sums of tile_hist over earlier
//                            tiles give the tile's starting count per expert; every workgroup also forms
//                            the totals and their exclusive scan (cheap, E <= 1024), so there is no third
//                            launch.  Each wave owns a contiguous segment of the tile; segment histograms
//                            are prefix-summed over the waves with a DPP row scan, and inside a wave the
//                            rank among lanes holding the same id comes from ballots.  Integer LDS atomics
//                            are used for COUNTS only, which do not depend on order.  One extra workgroup
//                            writes the count/offset tables.
// Both kernels are latency-bound (a few microseconds): loads are requested before LDS is cleared and
// the serial chain is kept to three barriers.  Small batches skip pass 1 (see plan_rank_kernel with FUSED).
#include "device_utils.h"
#include "launch.h"
#include "plan_tables.h"

namespace moe_rbf {

constexpr int kPlanBlock = 1024;                  // 16 waves
constexpr int kPlanWaves = kPlanBlock / kWave;
constexpr int kPlanMinTile = kPlanBlock;          // one branch per thread
constexpr int kPlanMaxTiles = 512;

// Every pass-2 workgroup sums the histograms of all tiles, so many tiles cost more than long ones from about
// 200 000 branches on.  Measured, us per plan with tiles of 1024 / 2048 / 4096 branches: 32 768 branches
// 9.5 / 10.7 / 13.3, 131 072: 11.9 / 12.1 / 13.6, 262 144: 15.1 / 11.0 / 12.5.
int plan_tile_size(int64_t N) {
  int64_t tile = N >= 196608 ? 2 * kPlanMinTile : kPlanMinTile;
  while ((N + tile - 1) / tile > kPlanMaxTiles) tile *= 2;
  return (int)tile;
}
int plan_tile_count(int64_t N) {
  const int64_t tile = plan_tile_size(N);
  const int64_t tiles = (N + tile - 1) / tile;
  return tiles < 1 ? 1 : (int)tiles;
}

__global__ __launch_bounds__(kPlanBlock) void plan_tile_hist_kernel(const int32_t *__restrict__ K, int N, int E,
                                                                     int tile, int32_t *__restrict__ tile_hist) {
  extern __shared__ int hist[];  // [E+1]
  const long long start = (long long)blockIdx.x * tile;
  const long long end = min(start + (long long)tile, (long long)N);
  const long long i0 = start + threadIdx.x;
  const int first_id = i0 < end ? K[i0] : -1;     // requested before the histogram is cleared
  for (int e = threadIdx.x; e <= E; e += kPlanBlock) hist[e] = 0;
  __syncthreads();
  for (long long i = i0; i < end; i += kPlanBlock) {
    const int e = i == i0 ? first_id : K[i];
    if (e >= 0 && e < E) atomicAdd(&hist[e], 1);
    else if (e != -1) atomicAdd(&hist[E], 1);
  }
  __syncthreads();
  int32_t *out = tile_hist + (size_t)blockIdx.x * (E + 1);
  for (int e = threadIdx.x; e <= E; e += kPlanBlock) out[e] = hist[e];
}

// Inclusive prefix sum inside each row of 16 consecutive lanes (DPP row shifts).
__device__ __forceinline__ int row16_inclusive_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);
  return v;
}

// Pass 2.  Workgroups 0..tiles-1 rank one tile each; workgroup `tiles` writes the count/offset tables.
// A tile is split into 16 contiguous wave segments (64 branches each when the tile is 1024 branches).
// FUSED: there was no pass 1.  Every workgroup counts the ids outside its own tile itself (in front of the
// tile -> `before`, behind it -> `total`), which costs N LDS atomics per workgroup instead of a launch:
// worth it for batches of up to about twelve thousand branches.
// WARM: the grid carries spare workgroups that read the caller's prefetch range (compiled apart so that the
// usual plan carries none of it).
template <bool FUSED, bool WARM>
__global__ __launch_bounds__(kPlanBlock) void plan_rank_kernel(const int32_t *__restrict__ K,
                                                                const int32_t *__restrict__ tile_hist, int tiles,
                                                                int tile, Dims d, PlanView p, WarmRange warm) {
  extern __shared__ int lds[];
  const int E = d.E;
  int *total = lds;                    // [E+1]  c^exp, then the number of invalid ids
  int *g = total + E + 1;              // [E+1]  exclusive scan of the block sizes over all experts
  int *before = g + E + 1;             // [E]    branches of expert e in earlier tiles
  int *others = before + E;            // [E]    branches of the other source ranks (several sources only)
  int *pre = others + E;               // [E]    branches of the source ranks below this one
  int *wcur = pre + E;                 // [waves][E] segment histograms, then running s per wave segment
  int *misc = wcur + kPlanWaves * E;   // [2]    scratch
  // dispatch order list: counts inside this tile's sorted stretch (a run of d.order_tiles tiles)
  int *st_total = FUSED ? total : misc + 2;             // [E+1]  branches of expert e in the whole stretch
  int *st_before = FUSED ? before : st_total + E + 1;   // [E]    ... in the stretch's tiles in front of this one
  int *st_excl = misc + 2 + (E + 1) + E;                // [E+1]  exclusive scan of st_total over the experts
  __shared__ unsigned long long others_rows;   // rows of the other source ranks, 64-bit
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int me = blockIdx.x;
  const bool multi = p.source_count != nullptr;
  if (tid == 0) others_rows = 0;

  if (WARM && me > tiles) {            // spare workgroups: pull the caller's memory (normally X) into the caches
    constexpr int kPer = 8;            // vectors per thread and trip
    const u32x4 *src = (const u32x4 *)warm.ptr;
    const long long wgs = (long long)gridDim.x - tiles - 1, w = me - tiles - 1;
    const long long chunk = (warm.vecs + wgs - 1) / wgs;
    const long long lo = w * chunk, hi = min(lo + chunk, warm.vecs);
    unsigned acc = 0;
    for (long long i = lo + tid; i < hi; i += (long long)kPlanBlock * kPer) {
      u32x4 v[kPer];
#pragma unroll
      for (int u = 0; u < kPer; ++u)
        v[u] = i + (long long)u * kPlanBlock < hi ? src[i + (long long)u * kPlanBlock] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int u = 0; u < kPer; ++u) acc |= v[u][0];
    }
    asm volatile("" ::"v"(acc));       // the loads are kept although nothing uses their values
    return;
  }
  if (me == tiles) {                   // tables workgroup
    if (FUSED) {
      tables_from_ids_block(K, d, p, lds);
      return;
    }
    for (int e = tid; e <= E; e += kPlanBlock) total[e] = 0;
    for (int e = tid; e < 2 * E; e += kPlanBlock) others[e] = 0;     // others and pre
    __syncthreads();
    sum_columns<false>(tile_hist, tiles, E + 1, 0, total, nullptr, 0);
    if (multi) sum_columns<true>(p.source_count, d.R, E, d.me, others, pre, E, &others_rows);
    __syncthreads();
    if (wave == 0) wave_exclusive_scan_lds(total, g, E, -1, multi ? others : nullptr);
    __syncthreads();
    write_plan_tables(total, multi ? others : nullptr, multi ? pre : nullptr, g, d, p, total[E], misc,
                      multi && rows_overflow(others_rows, g[E]));
    return;
  }

  // The sorted stretch this tile belongs to (FUSED: the whole batch is one stretch)
  const bool ordered = d.order_tiles > 0;
  const int st0 = ordered ? (me / d.order_tiles) * d.order_tiles : 0;
  const int st1 = ordered ? min(tiles, st0 + d.order_tiles) : 0;
  const int seg = tile / kPlanWaves;
  const long long seg_start = (long long)me * tile + (long long)wave * seg;
  const int rounds = seg / kWave;
  // the first round's id is requested before anything else and stays in a register
  const long long i_first = seg_start + lane;
  const int id_first = i_first < d.N ? K[i_first] : -1;
  constexpr int kBatch = 8;            // FUSED: ids of other tiles, kBatch per thread and trip
  const int tile_start = me * tile;    // FUSED only runs with N <= tiles * tile well inside 31 bits
  const int tile_end = min(tile_start + tile, d.N);
  int other[kBatch];
  if (FUSED) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int i = u * kPlanBlock + tid;
      other[u] = (i < d.N && (i < tile_start || i >= tile_end)) ? K[i] : -1;
    }
  }

  for (int e = tid; e <= E; e += kPlanBlock) total[e] = 0;
  for (int e = tid; e < 3 * E; e += kPlanBlock) before[e] = 0;       // before, others and pre
  for (int x = tid; x < kPlanWaves * E; x += kPlanBlock) wcur[x] = 0;
  if (!FUSED && ordered)
    for (int e = tid; e < 2 * E + 1; e += kPlanBlock) st_total[e] = 0;                // st_total and st_before
  __syncthreads();
  if (FUSED) {
    for (int i0 = 0; i0 < d.N; i0 += kBatch * kPlanBlock) {
      int next[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {                 // the next trip's ids are requested first
        const int i = i0 + (kBatch + u) * kPlanBlock + tid;
        next[u] = (i < d.N && (i < tile_start || i >= tile_end)) ? K[i] : -1;
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int e = other[u];
        if (e >= 0 && e < E) atomicAdd(i0 + u * kPlanBlock + tid < tile_start ? &before[e] : &total[e], 1);
        other[u] = next[u];
      }
    }
  } else {
    if (ordered)
      sum_columns_stretch(tile_hist, tiles, E + 1, me, st0, st1, total, before, st_total, st_before, E);
    else
      sum_columns<false>(tile_hist, tiles, E + 1, me, total, before, E);
  }
  if (multi) sum_columns<true>(p.source_count, d.R, E, d.me, others, pre, E, &others_rows);
  // histogram of each wave's segment (counts only: atomics are order-free here)
  for (int rd = 0; rd < rounds; ++rd) {
    const long long i = seg_start + (long long)rd * kWave + lane;
    const int e = rd == 0 ? id_first : (i < d.N ? K[i] : -1);
    if (e >= 0 && e < E) atomicAdd(&wcur[wave * E + e], 1);
  }
  __syncthreads();
  if (!FUSED && wave == 0) wave_exclusive_scan_lds(total, g, E, -1, multi ? others : nullptr);
  if (!FUSED && ordered && wave == 1) wave_exclusive_scan_lds(st_total, st_excl, E);
  // exclusive prefix of the segment counts over the 16 waves, seeded with the count in earlier tiles:
  // element (e, w) sits in lane w of a 16-lane row, so one DPP row scan does it
  for (int x0 = 0; x0 < kPlanWaves * E; x0 += kPlanBlock) {
    const int x = x0 + tid;
    const int e = x / kPlanWaves, w = x % kPlanWaves;
    const bool in = x < kPlanWaves * E;
    const int c = in ? wcur[w * E + e] : 0;
    const int incl = row16_inclusive_scan(c);
    if (in) wcur[w * E + e] = before[e] + incl - c;
    // FUSED: total[e] held the ids behind the tile; the last wave's lane adds those in front and the tile's own
    if (FUSED && in && w == kPlanWaves - 1) total[e] += before[e] + incl;
  }
  __syncthreads();
  if (FUSED) {
    if (wave == 0) wave_exclusive_scan_lds(total, g, E, -1, multi ? others : nullptr);
    if (ordered && wave == 1) wave_exclusive_scan_lds(st_total, st_excl, E);
    __syncthreads();
  }

  // rows are int32: if the blocks of all sources together do not fit, nothing is placed
  const bool overflow = multi && rows_overflow(others_rows, g[E]);
  // stable ranks inside each wave segment: 64 branches per round, rounds in index order.  Lanes with
  // the same id all read the segment's running count, then the lowest of them advances it.
  const int bits = id_bits(E);
  int *mine = wcur + wave * E;
  for (int rd = 0; rd < rounds; ++rd) {
    const long long i = seg_start + (long long)rd * kWave + lane;
    const bool in = i < d.N;
    const int e = rd == 0 ? id_first : (in ? K[i] : -1);
    const bool valid = e >= 0 && e < E;
    const unsigned long long peers = match_any(e, valid, bits);
    int s = -1, row = -1;
    if (valid) {
      const int base = mine[e];
      const int rank = __popcll(peers & ((1ull << lane) - 1ull));
      if (rank == 0 && rounds > 1) mine[e] = base + __popcll(peers);   // LDS ops of a wave execute in order
      s = base + rank;
      row = expert_first_row(g, e, d) + pre[e] + s;                    // o_{e,me} + s
      if (row >= region_row_limit(e, d) || overflow) row = -1;
    }
    if (in) {
      if (p.send_idx) p.send_idx[i] = s;
      p.row_map[i] = row;
    }
    if (ordered) {
      // position of the branch among the counted branches of its stretch, sorted by (expert, flat index), i.e.
      // by window row; branches that are not counted leave the tail of the stretch's list, which is marked unused
      typedef int i32x2 __attribute__((ext_vector_type(2)));
      i32x2 *list = (i32x2 *)p.order;
      const long long st_base = (long long)st0 * tile;
      if (valid) list[st_base + st_excl[e] + st_before[e] + (s - before[e])] = i32x2{(int)i / d.k, row};
      if (in && (int)(i - st_base) >= st_excl[E]) list[i] = i32x2{-1, -1};
    }
    // the next round of this wave must see this round's counter updates
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// No tokens: the tables still describe the (possibly non-empty) blocks of the other source ranks.
__global__ __launch_bounds__(kPlanBlock) void plan_empty_kernel(Dims d, PlanView p) {
  extern __shared__ int lds[];
  const int E = d.E;
  int *total = lds;                    // [E]   zeros
  int *g = total + E;                  // [E+1]
  int *others = g + E + 1;             // [E]
  int *pre = others + E;               // [E]
  int *misc = pre + E;                 // [2]
  __shared__ unsigned long long others_rows;
  const bool multi = p.source_count != nullptr;
  for (int e = threadIdx.x; e < E; e += kPlanBlock) {
    total[e] = 0;
    others[e] = 0;
    pre[e] = 0;
  }
  if (threadIdx.x == 0) others_rows = 0;
  __syncthreads();
  if (multi) sum_columns<true>(p.source_count, d.R, E, d.me, others, pre, E, &others_rows);
  __syncthreads();
  if (threadIdx.x < kWave) wave_exclusive_scan_lds(total, g, E, -1, multi ? others : nullptr);
  __syncthreads();
  write_plan_tables(total, multi ? others : nullptr, multi ? pre : nullptr, g, d, p, 0, misc,
                    multi && rows_overflow(others_rows, g[E]));
}

hipError_t launch_plan_empty(const Dims &d, const PlanView &p, hipStream_t s) {
  const size_t lds = (size_t)(4 * d.E + 1 + 2) * sizeof(int);
  return launch(plan_empty_kernel, dim3(1), dim3(kPlanBlock), lds, s, d, p);
}

// Largest batch (in tiles of 1024 branches) planned with one launch.  Measured, E = 256, graph replay:
// one launch / two launches = 7.6 / 8.9 us at 8192 branches, 8.6 / 9.1 at 16384 (9.3 / 9.1 with Zipf
// routing, whose hot bins serialise the LDS atomics), 10.7 / 9.2 at 32768, 26 / 11.7 at 131072.
#ifndef MOE_PLAN_FUSED_MAX_TILES
#define MOE_PLAN_FUSED_MAX_TILES 12
#endif

bool plan_uses_workspace(int64_t N) { return N > (int64_t)MOE_PLAN_FUSED_MAX_TILES * kPlanMinTile; }

// Measured on the same buffers, k = 8 unless noted, us per LAYER (plan + dispatch + combine) with the list / in token
// order, with stretches of about 28 MB of X (3.5 MB per XCD, most of its L2), which did best:
//   H = 7168, balanced: T = 1536 69.3 / 75.4, 2048 94.4 / 97.6, 3072 134.3 / 136.2, 4096 171.3 / 181.1, 5120 221.6 / 220.8,
//             6144 258.5 / 263.7, 7168 309 / 303.6 (a loss), 8192 352.9 / 347.4 (a loss), 16384 702 / 691.5 (a loss);
//             Zipf routing: T = 4096 171.1 / 171.0, T = 16384 665 / 660 (a loss); k = 6, T = 4096: 134.6 / 137.2;
//             k = 4, T = 8192: 194.2 / 190.9 (a loss)
//   H = 6144: T = 4096 150.5 / 159.7, 6144 227.5 / 242.0, 8192 292.3 / 312.8
//   H = 8192: T = 4096 192.7 / 201.5, 6144 285.3 / 301.5;  H = 16384: T = 2048 203.7 / 204.6, 3072 289.8 / 303.0
//   H = 4096, balanced: T = 2048 59.1 / 61.6, 4096 108.4 / 109.4, 8192 204.4 / 208.5, 16384 390.1 / 418.7;
//             group-limited, E = 128: T = 8192 202.4 / 205.8, 16384 379.2 / 405.2, 32768 940 / 830 (a loss)
// A loop of dispatches alone gains more (T = 4096, H = 7168: 76.8 / 85.2 us).  Inside a layer the gain depends on
// X still being in the Infinity Cache when the dispatch starts (the list makes every token row be fetched at
// k scattered moments of its stretch), so the list is used
//   for rows of 12 KB or more while X holds at most 96 MiB and the window at most 770 MiB,
//   for narrower rows (8 to 12 KB, and 2 to 4 KB) with windows of up to 1100 MiB.
// Rows of 2 to 4 KB, us per layer with the list / in token order: H = 2048: T = 8192 105.4 / 108.0, 16384 197.0 / 204.3,
// 32768 388.6 / 407.6; H = 1024: T = 16384 110.0 / 113.4, 65536 405.7 / 426.0.  Rows in between: H = 3072: T = 8192
// 162.6 / 163.6, 16384 311.4 / 313.0; H = 2560, T = 8192: 145.6 / 138.5 (a loss).
int plan_order_tiles(const Dims &d) {
  const int64_t row_bytes = (int64_t)d.H16 * 16;
  // rows of 2 to 4 KB (slices of 16 to 32 vectors) and rows of at least 8 KB; in between (slices of 33 to 63
  // vectors, which fill neither one nor two units of a workgroup) and below, token order does as well or better
  if (d.N == 0 || d.H16 < 128 || (d.H16 > 256 && d.H16 < 512)) return 0;
#ifndef MOE_ORDER_LIMIT_SCALE
#define MOE_ORDER_LIMIT_SCALE 1          // tuning knob: scales all limits
#endif
  const int64_t mib = (int64_t)MOE_ORDER_LIMIT_SCALE << 20;
  const int64_t window = (int64_t)d.N * row_bytes, x = (int64_t)d.T * row_bytes;
  if (row_bytes < 12288 ? window > 1100 * mib : (window > 770 * mib || x > 96 * mib)) return 0;
  const int tile = plan_tile_size(d.N), tiles = plan_tile_count(d.N);
  if (!plan_uses_workspace(d.N)) return tiles;                      // single-launch plan: the batch is one stretch
  // stretches of about 28 MB of X, all of (nearly) the same length
  const int64_t most = ((int64_t)28 << 20) / row_bytes * d.k / tile;
  if (most < 1) return 1;
  const int64_t n = (tiles + most - 1) / most;
  return (int)((tiles + n - 1) / n);
}

template <bool FUSED>
static hipError_t launch_plan_rank(const Dims &d, const int32_t *K, const PlanView &p, const int32_t *tile_hist,
                                   int tiles, int tile, const WarmRange &warm, hipStream_t s) {
  const size_t lds = (size_t)(5 * d.E + 2 + kPlanWaves * d.E + 2 + 3 * d.E + 2) * sizeof(int);
  if (lds > 64 * 1024) {   // beyond the default dynamic LDS limit (E > ~800): raise it once per process
    static const hipError_t raised = [] {
      hipError_t e = hipFuncSetAttribute((const void *)plan_rank_kernel<FUSED, false>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
      return e != hipSuccess ? e
                             : hipFuncSetAttribute((const void *)plan_rank_kernel<FUSED, true>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    }();
    if (raised != hipSuccess) return raised;
  }
  if (!warm.ptr)
    return launch(plan_rank_kernel<FUSED, false>, dim3(tiles + 1), dim3(kPlanBlock), lds, s, K, tile_hist, tiles, tile,
                  d, p, warm);
  // spare workgroups for plan->prefetch: 8192 vectors (128 KB) each
  const unsigned spare = (unsigned)((warm.vecs + 8191) / 8192);
  return launch(plan_rank_kernel<FUSED, true>, dim3(tiles + 1 + spare), dim3(kPlanBlock), lds, s, K, tile_hist, tiles,
                tile, d, p, warm);
}

hipError_t launch_plan(const Dims &d, const int32_t *K, const PlanView &p, int32_t *tile_hist, const WarmRange &warm,
                       hipStream_t s) {
  const int tile = plan_tile_size(d.N);
  const int tiles = plan_tile_count(d.N);
  if (!plan_uses_workspace(d.N)) return launch_plan_rank<true>(d, K, p, nullptr, tiles, tile, warm, s);
  const size_t lds1 = (size_t)(d.E + 1) * sizeof(int);
  hipError_t err = launch(plan_tile_hist_kernel, dim3(tiles), dim3(kPlanBlock), lds1, s, K, d.N, d.E, tile, tile_hist);
  if (err != hipSuccess) return err;
  return launch_plan_rank<false>(d, K, p, tile_hist, tiles, tile, warm, s);
}

}  // namespace moe_rbf
