// Prefill Layout + Notify for one source rank (paper, Section 5.2): per-expert and per-rank branch
// counts, large offsets o (exclusive scan of the counts inside each rank region), the stable small
// offset s of every branch and the row map o[K] + s.  No payload is touched.
//
// The small offset must be the number of EARLIER branches (smaller flat index t*k+j) with the same
// expert, so it cannot come from global atomics (arbitrary order).  It is built the way the paper
// describes the Layout kernel -- per-block counting plus prefix accumulation over earlier blocks:
//   K1  plan_tile_hist : one workgroup per tile of branches -> LDS histogram -> tile_hist[tile][E+1]
//                        (slot E counts ids outside [0,E) other than -1)
//   K2  plan_rank      : one workgroup per tile; column sums of tile_hist over earlier tiles give the
//                        tile's starting count per expert; every workgroup also forms the totals and
//                        their exclusive scan (cheap, E <= 1024) so no third launch is needed; inside
//                        the tile each of the 4 waves owns a contiguous segment, segment histograms are
//                        prefix-summed in wave order, and inside a wave the rank among lanes holding the
//                        same id comes from ballots.  Integer LDS atomics are used for COUNTS only,
//                        which do not depend on order.
#include "device_utils.h"
#include "launch.h"
#include "plan_tables.h"

namespace moe_rbf {

constexpr int kPlanBlock = 256;                   // 4 waves
constexpr int kPlanWaves = kPlanBlock / kWave;
constexpr int kPlanMinTile = 1024;                // 4 rounds of 64 per wave
constexpr int kPlanMaxTiles = 512;

int plan_tile_size(int64_t N) {
  int64_t tile = kPlanMinTile;
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
  for (int e = threadIdx.x; e <= E; e += kPlanBlock) hist[e] = 0;
  __syncthreads();
  const long long start = (long long)blockIdx.x * tile;
  const long long end = min(start + (long long)tile, (long long)N);
  for (long long i = start + threadIdx.x; i < end; i += kPlanBlock) {
    const int e = K[i];
    if (e >= 0 && e < E) atomicAdd(&hist[e], 1);
    else if (e != -1) atomicAdd(&hist[E], 1);
  }
  __syncthreads();
  int32_t *out = tile_hist + (size_t)blockIdx.x * (E + 1);
  for (int e = threadIdx.x; e <= E; e += kPlanBlock) out[e] = hist[e];
}

// ROUNDS > 0: a wave's segment is ROUNDS*64 branches and its ids stay in registers between the
// counting pass and the ranking pass (tile = ROUNDS*256); ROUNDS == 0: any tile size, ids are re-read.
template <int ROUNDS>
__global__ __launch_bounds__(kPlanBlock) void plan_rank_kernel(const int32_t *__restrict__ K,
                                                                const int32_t *__restrict__ tile_hist, int tiles,
                                                                int tile, Dims d, PlanView p) {
  extern __shared__ int lds[];
  const int E = d.E;
  int *total = lds;                    // [E]    c^exp
  int *g = total + E;                  // [E+1]  exclusive scan of total over all experts
  int *off = g + E + 1;                // [E]    o[e]: first row of expert e
  int *lim = off + E;                  // [E]    first row past expert e's rank region
  int *before = lim + E;               // [E]    branches of expert e in earlier tiles
  int *wcur = before + E;              // [waves][E] segment histograms, then running s per wave
  int *misc = wcur + kPlanWaves * E;   // [2]    {invalid ids, scratch counter}
  const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
  const int me = blockIdx.x;
  const int seg = tile / kPlanWaves;
  const long long seg_start = (long long)me * tile + (long long)wave * seg;
  const int rounds = ROUNDS > 0 ? ROUNDS : seg / kWave;

  // this wave's ids: issued first so that their latency overlaps the histogram walk
  constexpr int R = ROUNDS > 0 ? ROUNDS : 1;
  int ids[R];
  if (ROUNDS > 0) {
#pragma unroll
    for (int rd = 0; rd < R; ++rd) {
      const long long i = seg_start + (long long)rd * kWave + lane;
      ids[rd] = i < d.N ? K[i] : -1;
    }
  }

  // column sums of the tile histograms: earlier tiles (start of this tile's streams) and all tiles;
  // 32 independent loads per batch
  for (int e = tid; e <= E; e += kPlanBlock) {
    int bef = 0, all = 0;
    const int32_t *col = tile_hist + e;
    for (int t0 = 0; t0 < tiles; t0 += 32) {
      int v[32];
#pragma unroll
      for (int u = 0; u < 32; ++u) v[u] = (t0 + u < tiles) ? col[(size_t)(t0 + u) * (E + 1)] : 0;
#pragma unroll
      for (int u = 0; u < 32; ++u) {
        all += v[u];
        if (t0 + u < me) bef += v[u];
      }
    }
    if (e < E) {
      total[e] = all;
      before[e] = bef;
    } else {
      misc[0] = all;
    }
  }
  for (int x = tid; x < kPlanWaves * E; x += kPlanBlock) wcur[x] = 0;
  __syncthreads();
  if (wave == 0) wave_exclusive_scan_lds(total, g, E);
  // histogram of each wave's contiguous segment (counts only: atomics are order-free here)
  for (int rd = 0; rd < rounds; ++rd) {
    int e;
    if (ROUNDS > 0) {
      e = ids[rd % R];
    } else {
      const long long i = seg_start + (long long)rd * kWave + lane;
      e = i < d.N ? K[i] : -1;
    }
    if (e >= 0 && e < E) atomicAdd(&wcur[wave * E + e], 1);
  }
  __syncthreads();
  // o and the region limit per expert; exclusive prefix of the segment counts over waves, seeded with
  // the count in earlier tiles: wcur[w][e] becomes the small offset of the first branch of expert e
  // in wave w's segment
  for (int e = tid; e < E; e += kPlanBlock) {
    off[e] = expert_first_row(g, e, d);
    lim[e] = region_row_limit(e, d);
    int run = before[e];
    for (int w = 0; w < kPlanWaves; ++w) {
      const int c = wcur[w * E + e];
      wcur[w * E + e] = run;
      run += c;
    }
  }
  __syncthreads();
  if (me == 0) write_plan_tables(total, g, d, p, misc[0], misc + 1);

  // stable ranks inside each wave segment: 64 branches per round, rounds in index order.  Among
  // lanes with the same id the lowest lane advances the running count and hands the old value out.
  const int bits = id_bits(E);
  int *mine = wcur + wave * E;
  for (int rd = 0; rd < rounds; ++rd) {
    const long long i = seg_start + (long long)rd * kWave + lane;
    const bool in = i < d.N;
    int e;
    if (ROUNDS > 0) e = ids[rd % R];
    else e = in ? K[i] : -1;
    const bool valid = e >= 0 && e < E;
    const unsigned long long peers = match_any(e, valid, bits);
    const int leader = valid ? __ffsll((long long)peers) - 1 : lane;
    int base = 0;
    if (valid && lane == leader) {
      base = mine[e];
      mine[e] = base + __popcll(peers);
    }
    base = __shfl(base, leader, kWave);
    int s = -1, row = -1;
    if (valid) {
      s = base + __popcll(peers & ((1ull << lane) - 1ull));
      row = off[e] + s;
      if (row >= lim[e]) row = -1;
    }
    if (in) {
      if (p.send_idx) p.send_idx[i] = s;
      p.row_map[i] = row;
    }
    // the next round of this wave must see this round's counter updates
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

__global__ void plan_empty_kernel(Dims d, PlanView p) {
  const bool fixed = d.stride > 0;
  for (int e = threadIdx.x; e < d.E; e += blockDim.x) {
    p.expert_count[e] = 0;
    p.expert_offset[e] = fixed ? (int)((e / d.Er) * d.stride) : 0;
  }
  for (int r = threadIdx.x; r < d.R; r += blockDim.x) {
    p.rank_count[r] = 0;
    p.region_base[r] = fixed ? (int)(r * d.stride) : 0;
  }
  if (threadIdx.x == 0) {
    p.expert_offset[d.E] = fixed ? (int)(((d.E - 1) / d.Er) * d.stride) : 0;
    p.region_base[d.R] = fixed ? (int)(d.R * d.stride) : 0;
    p.status[0] = 0;
    p.status[1] = 0;
  }
}

hipError_t launch_plan_empty(const Dims &d, const PlanView &p, hipStream_t s) {
  return launch(plan_empty_kernel, dim3(1), dim3(256), 0, s, d, p);
}

hipError_t launch_plan(const Dims &d, const int32_t *K, const PlanView &p, int32_t *tile_hist, hipStream_t s) {
  const int tile = plan_tile_size(d.N);
  const int tiles = plan_tile_count(d.N);
  const size_t lds1 = (size_t)(d.E + 1) * sizeof(int);
  hipError_t err = launch(plan_tile_hist_kernel, dim3(tiles), dim3(kPlanBlock), lds1, s, K, d.N, d.E, tile, tile_hist);
  if (err != hipSuccess) return err;
  const size_t lds2 = (size_t)(5 * d.E + 1 + kPlanWaves * d.E + 2) * sizeof(int);
  if (tile == kPlanMinTile)
    return launch(plan_rank_kernel<kPlanMinTile / kPlanBlock>, dim3(tiles), dim3(kPlanBlock), lds2, s, K, tile_hist,
                  tiles, tile, d, p);
  return launch(plan_rank_kernel<0>, dim3(tiles), dim3(kPlanBlock), lds2, s, K, tile_hist, tiles, tile, d, p);
}

}  // namespace moe_rbf
