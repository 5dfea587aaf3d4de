// Dispatch: direct placement of token rows into destination expert windows (paper, Section 5.2
// "Prefill Dispatch", Section 5.3 "Decode Dispatch"; first loop of Algorithms 1 and 2).
// No staging copy exists: HBM traffic is T*H bytes read and T*k*H bytes written.
//
// Prefill schedule (row map from moe_plan): XCD-affine column slices, see dispatch_slices_kernel.
// Decode schedule: ONE launch, no grid-wide synchronisation: every workgroup derives the rows of its
//   token from the routing ids themselves (see the decode section below).
#include "device_utils.h"
#include "launch.h"
#include "moe_rbf.h"
#include "plan_tables.h"
#include "quant.h"

namespace moe_rbf {

#ifndef MOE_DECODE_BLOCK
#define MOE_DECODE_BLOCK 512
#endif
#ifndef MOE_DECODE_VEC
#define MOE_DECODE_VEC 1
#endif

constexpr int kSlices = 8;   // column slices per row = XCDs per device

// Prefill dispatch.  Work unit = (J consecutive branches of one token, column slice c of 8); a workgroup
// holds U units.  Workgroup b handles slice c = b % 8.  Workgroups are handed to the 8 XCDs round-robin, so XCD c only
// ever touches column slice c: the k re-reads of X[t]'s slice by the branches of a token hit in that
// XCD's L2 (X is fetched from HBM once), every wave issues few 16-byte stores per lane, and the 8 XCDs
// together lay down whole destination rows.  Stores are streaming (nontemporal) so that they do not
// evict the X slices from L2; loads are ordinary so that they stay.
// (If the hardware maps workgroups differently the result is unchanged; only the L2 reuse is lost.)
template <int BLOCK, int J, int U>
__global__ __launch_bounds__(BLOCK) void dispatch_slices_kernel(const u32x4 *__restrict__ X,
                                                                const int32_t *__restrict__ row_map,
                                                                u32x4 *__restrict__ window, int k, int H16, int slice,
                                                                int N) {
  // U units per workgroup, each with BLOCK / U lanes: narrow slices (small H) still fill the workgroup
  constexpr int kLanes = BLOCK / U;
  const int unit = U == 1 ? 0 : (int)threadIdx.x / kLanes;
  const int lane = U == 1 ? (int)threadIdx.x : (int)threadIdx.x % kLanes;
  const int g = (blockIdx.x / kSlices) * U + unit;
  const int c = blockIdx.x % kSlices;
  const int n = g * J;                       // J consecutive branches of one token (J divides k)
  if (U > 1 && n >= N) return;
  int row[J];
#pragma unroll
  for (int u = 0; u < J; ++u) row[u] = kLanes % kWave == 0 ? uniform(row_map[n + u]) : row_map[n + u];
  const int t = n / k;
  const int end = min((c + 1) * slice, H16);
  const u32x4 *src = X + (size_t)t * (size_t)H16;
  for (int col = c * slice + lane; col < end; col += kLanes) {
    const u32x4 v = src[col];
#pragma unroll
    for (int u = 0; u < J; ++u)
      if (row[u] >= 0) store_stream(window + (size_t)row[u] * (size_t)H16 + col, v);
  }
}

// Prefill dispatch along the plan's order list: unit p copies column slice c of X[token] to window[row] for
// the p-th (token, row) pair.  The pairs are sorted by row inside stretches of tokens whose X slices fit the
// L2 of an XCD, so consecutive workgroups of an XCD write consecutive rows of one expert block and re-read
// tokens from L2.  U units per workgroup, each with 128 / U lanes, as in dispatch_slices_kernel.
template <int U>
__global__ __launch_bounds__(128) void dispatch_list_kernel(const u32x4 *__restrict__ X,
                                                            const int32_t *__restrict__ order,
                                                            u32x4 *__restrict__ window, int H16, int slice, int N) {
  typedef int i32x2 __attribute__((ext_vector_type(2)));
  constexpr int kLanes = 128 / U;
  const int unit = U == 1 ? 0 : (int)threadIdx.x / kLanes;
  const int lane = U == 1 ? (int)threadIdx.x : (int)threadIdx.x % kLanes;
  const int pidx = (blockIdx.x / kSlices) * U + unit;
  const int c = blockIdx.x % kSlices;
  if (pidx >= N) return;
  i32x2 pair = ((const i32x2 *)order)[pidx];
  if (kLanes % kWave == 0) pair = i32x2{uniform(pair[0]), uniform(pair[1])};
  const int t = pair[0], row = pair[1];
  if (t < 0 || row < 0) return;
  const int end = min((c + 1) * slice, H16);
  const u32x4 *src = X + (size_t)t * (size_t)H16;
  u32x4 *dst = window + (size_t)row * (size_t)H16;
  for (int col = c * slice + lane; col < end; col += kLanes) store_stream(dst + col, src[col]);
}

// ---- decode -------------------------------------------------------------------------------------
//
// Row of branch (t,j) with expert e:  region/expert base + #{ids i : lo <= K_i < e} + #{i < t*k+j : K_i = e}
// (lo = 0 and base = 0 for tight windows; lo = first expert of e's rank and base = rank*stride otherwise).
// Both terms are plain counts over the <= 8192 routing ids of the batch, so a payload workgroup gets
// them with compares on the ids it holds in registers, wave ballots (the counts land in scalar
// registers) and one LDS exchange between its waves: no histogram, no scan, one barrier.  The two
// counts of a slot travel packed in one word (low 16 bits: ids below e; high 16 bits: equal ids in
// front of the branch).
// One extra workgroup (the first, since it takes longest) builds the histogram and writes the tables for
// combine and the experts.


// QUANT: the workgroup holds a whole row (chunks == 1), quantises it once and fans the codes and the
// row's scale out instead of the bf16 payload.
// MULTI: plan->source_count is given (several source ranks); compiled apart so that the single-source
// kernel, which is latency-bound, carries none of that code.
// SB: slots of a token ranked together (one LDS exchange per SB slots).  The slots of a token may be split
// over `groups` workgroups (each ranks and stores only its own slots of the chunk): more, smaller
// workgroups spread the stores over all compute units and shorten each one's counting.
// GROUPS is a compile-time constant so that the index arithmetic in front of the first loads stays short.
template <int BLOCK, int V, int SB, int GROUPS, bool QUANT, bool MULTI>
__global__ __launch_bounds__(BLOCK) void decode_dispatch_kernel(const u32x4 *__restrict__ X,
                                                                const int32_t *__restrict__ K,
                                                                void *__restrict__ window_any,
                                                                float *__restrict__ window_scale, Dims d, PlanView p,
                                                                int chunks, int per_group) {
  constexpr int groups = GROUPS;
  extern __shared__ int lds[];                                  // tables workgroup; several-sources prefix tables
  __shared__ int part[(BLOCK / kWave) * SB];            // per-wave packed counts of a slot batch
  __shared__ int part_m[(BLOCK / kWave) * SB];          // per-wave rows of the other source ranks
  __shared__ int part_v[BLOCK / kWave];                         // per-wave number of ids inside [0,E)
  __shared__ unsigned long long part_w[BLOCK / kWave];          // per-wave rows of the other source ranks, 64-bit
  constexpr int kWaves = BLOCK / kWave;
  const int per_token = chunks * groups;
  if (blockIdx.x == 0) {                 // the tables workgroup goes first: it is the longest one
    tables_from_ids_block(K, d, p, lds);
    return;
  }
  const int b = (int)blockIdx.x - 1;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  // workgroup -> (token, chunk, slot group).  Workgroups go to the 8 XCDs round-robin: the workgroups of a
  // token are given to one XCD, whose L2 then serves their re-reads of the token row (the ragged tail of
  // tokens past a multiple of 8 is mapped plainly).
  int t, rem;
  {
    const int full = (d.T & ~7) * per_token;
    if (b >= full) {
      t = b / per_token;
      rem = b - t * per_token;
    } else if (chunks == 1) {             // the usual case: compile-time divisor
      const int q = b >> 3;
      t = (q / GROUPS) * 8 + (b & 7);
      rem = q % GROUPS;
    } else {
      const int q = b >> 3, tq = q / per_token;
      t = tq * 8 + (b & 7);
      rem = q - tq * per_token;
    }
  }
  const int c = rem / groups, grp = rem % groups;
  const int first = t * d.k;
  const int jg0 = grp * per_group, jg1 = min(d.k, jg0 + per_group);       // per_group: slots of a group, whole batches

  // everything that comes from memory is requested up front: payload, routing ids, own slots' ids
  const int col0 = c * (BLOCK * V) + tid;
  const u32x4 *src = X + (size_t)t * (size_t)d.H16;
  u32x4 v[V];
#pragma unroll
  for (int x = 0; x < V; ++x) {
    const int col = col0 + x * BLOCK;
    // read once by this workgroup: streaming, unless sibling workgroups of the token read it too
    v[x] = col < d.H16 ? (groups > 1 ? src[col] : load_stream(src + col)) : u32x4{0u, 0u, 0u, 0u};
  }
  constexpr int kIds = 4;        // ids per thread kept in registers (first kIds passes over K)
  int id[kIds];
#pragma unroll
  for (int u = 0; u < kIds; ++u) {
    const int i = u * BLOCK + tid;
    id[u] = i < d.N ? K[i] : -1;
  }
  u32x2 q[V];
  float scale = 0.0f;
  if (QUANT) {
    __shared__ float red[BLOCK / kWave];
    bool has[V];
#pragma unroll
    for (int x = 0; x < V; ++x) has[x] = col0 + x * BLOCK < d.H16;
    scale = quantise_row<BLOCK, V>(v, has, q, red);
  }

  // Several source ranks: rows of the other sources in front of a slot's sub-block =
  // (their rows in the experts below e, inside the region for fixed stride) + (rows of lower ranks for e),
  // i.e. sums over parts of the count matrix M.  A thread owns a few columns of M and keeps, per column, the
  // sum over the other ranks and the sum over the lower ranks; a slot's two terms are then masked sums of
  // these over the workgroup (wave reduction + the LDS exchange the id counts use anyway).
  constexpr bool multi = MULTI;
  constexpr int kCols = MULTI ? (MOE_MAX_EXPERTS + BLOCK - 1) / BLOCK : 1;     // columns a thread may own
  int col_all[kCols], col_pre[kCols], col_id[kCols];
#pragma unroll
  for (int q2 = 0; q2 < kCols; ++q2) col_all[q2] = col_pre[q2] = 0, col_id[q2] = -1;
  unsigned long long wave_rows = 0;                  // rows of the other sources counted by this wave's threads
  if (multi) {
    unsigned long long wide = 0;
    constexpr int kRows = 16;                       // rows of M requested together (8: 7.56 us, 16: 7.37, 32: 8.25 at T = 128, 32 sources)
    const int parts = max(1, BLOCK / d.E);          // threads per column when the matrix is narrow
    const int part = parts > 1 ? tid / d.E : 0;
#pragma unroll
    for (int q2 = 0; q2 < kCols; ++q2) {
      const int col = parts > 1 ? tid - part * d.E : tid + q2 * BLOCK;
      const bool live = parts > 1 ? (q2 == 0 && part < parts) : col < d.E;
      if (!live) continue;
      col_id[q2] = col;
      const int32_t *m = p.source_count + col;
      int all = 0, pre = 0;
      for (int r0 = part; r0 < d.R; r0 += parts * kRows) {
        int mv[kRows];
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          const int r = r0 + u * parts;
          mv[u] = (r < d.R && r != d.me) ? m[(size_t)r * d.E] : 0;
        }
#pragma unroll
        for (int u = 0; u < kRows; ++u) {
          all += mv[u];
          wide += (unsigned)mv[u];
          if (r0 + u * parts < d.me) pre += mv[u];
        }
      }
      col_all[q2] = all;
      col_pre[q2] = pre;
    }
    wave_rows = wave_sum_u64(wide);
  }
  bool overflow = false;                            // rows of all sources together do not fit in int32

  const bool fixed = d.stride > 0;
  for (int j0 = jg0; j0 < jg1; j0 += SB) {
    // lane u < SB of every wave owns slot j0+u
    const bool own = lane < SB && j0 + lane < jg1;
    const int my_e = own ? K[first + j0 + lane] : -1;
    const bool my_valid = my_e >= 0 && my_e < d.E;
    const int my_rank = my_valid ? my_e / d.Er : 0;
    const int my_lo = fixed ? my_rank * d.Er : 0;
    int e[SB], lo[SB], below[SB], front[SB];
#pragma unroll
    for (int u = 0; u < SB; ++u) {
      e[u] = __builtin_amdgcn_readlane(my_e, u);
      lo[u] = __builtin_amdgcn_readlane(my_lo, u);
      below[u] = 0;
      front[u] = 0;
    }
    // wave-wide counts by ballot: they land in scalar registers, no lane reduction is needed
    int n_valid = 0;
    for (int i0 = 0, pass = 0; i0 < d.N; i0 += BLOCK, ++pass) {
      const int i = i0 + tid;
      int x;
      if (pass < kIds) {
        x = id[0];
#pragma unroll
        for (int q = 1; q < kIds; ++q) x = pass == q ? id[q] : x;
      } else {
        x = i < d.N ? K[i] : -1;
      }
      const int ahead = first + j0 - i;               // slot u is behind id i  <=>  u + ahead > 0
      if (multi && j0 == jg0) n_valid += __popcll(__ballot((unsigned)x < (unsigned)d.E));
      // ids outside [0,E) never satisfy either test: as unsigned values they are huge (or x > e)
      if (fixed) {
#pragma unroll
        for (int u = 0; u < SB; ++u)
          below[u] += __popcll(__ballot((unsigned)(x - lo[u]) < (unsigned)(e[u] - lo[u])));
      } else {
#pragma unroll
        for (int u = 0; u < SB; ++u) below[u] += __popcll(__ballot((unsigned)x < (unsigned)e[u]));
      }
#pragma unroll
      for (int u = 0; u < SB; ++u)
        front[u] += __popcll(__ballot(x == e[u]) & __ballot(ahead + u > 0));   // two masks, and-ed as scalars
    }
    int mine_m = 0;                                   // lane u: this wave's rows of other sources in front of slot u
    if (multi) {
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        int cu = 0;
#pragma unroll
        for (int q2 = 0; q2 < kCols; ++q2) {
          cu += (unsigned)(col_id[q2] - lo[u]) < (unsigned)(e[u] - lo[u]) ? col_all[q2] : 0;
          cu += col_id[q2] == e[u] ? col_pre[q2] : 0;
        }
        const int tot = __builtin_amdgcn_readlane(wave_inclusive_scan(cu), kWave - 1);
        mine_m = lane == u ? tot : mine_m;
      }
    }
    if (j0 > jg0) __syncthreads();                      // the previous batch's exchange has been read
    {
      int mine = 0;                                   // lane u carries this wave's packed counts of slot u
#pragma unroll
      for (int u = 0; u < SB; ++u) mine = lane == u ? below[u] + (front[u] << 16) : mine;
      if (lane < SB) {
        part[wave * SB + lane] = mine;
        if (multi) part_m[wave * SB + lane] = mine_m;
      }
      if (multi && j0 == jg0 && lane == 0) part_v[wave] = n_valid, part_w[wave] = wave_rows;
    }
    __syncthreads();
    if (multi && j0 == jg0) {
      unsigned long long all_rows = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) all_rows += part_w[w] + (unsigned)part_v[w];
      overflow = all_rows >= (1ull << 31);
    }
    int packed = 0, ahead_m = 0;
    if (lane < SB) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) packed += part[w * SB + lane];
      if (multi)
#pragma unroll
        for (int w = 0; w < kWaves; ++w) ahead_m += part_m[w * SB + lane];
    }
    int s = -1, row = -1;
    if (own && my_valid) {
      s = packed >> 16;
      row = (fixed ? (int)(my_rank * d.stride) : 0) + (packed & 0xffff) + s;
      row += ahead_m;
      if ((fixed && row >= (int)((my_rank + 1) * d.stride)) || overflow) row = -1;
    }
    if (own && c == 0 && wave == 0) {
      if (p.send_idx) p.send_idx[first + j0 + lane] = s;
      p.row_map[first + j0 + lane] = row;
      if (d.order_tiles > 0) {          // a later prefill-schedule dispatch on this plan walks the order list
        p.order[2 * (first + j0 + lane)] = t;
        p.order[2 * (first + j0 + lane) + 1] = row;
      }
    }
    // fan the chunk out to this batch's destination rows
    const int nb = min(SB, jg1 - j0);
    for (int u = 0; u < nb; ++u) {
      const int r = __builtin_amdgcn_readlane(row, u);
      if (r < 0) continue;
      if (QUANT) {
        u32x2 *dst = (u32x2 *)window_any + (size_t)r * (size_t)d.H16;    // H bytes per row = H16 8-byte units
#pragma unroll
        for (int x = 0; x < V; ++x) {
          const int col = col0 + x * BLOCK;
          if (col < d.H16) __builtin_nontemporal_store(q[x], dst + col);
        }
        if (tid == 0) window_scale[r] = scale;
      } else {
        u32x4 *dst = (u32x4 *)window_any + (size_t)r * (size_t)d.H16;
#pragma unroll
        for (int x = 0; x < V; ++x) {
          const int col = col0 + x * BLOCK;
          if (col < d.H16) store_stream(dst + col, v[x]);
        }
      }
    }
  }
}

// Quantised dispatch with the row map from moe_plan: one workgroup per token holds the whole row,
// quantises it once and stores the codes and the scale to the k destination rows.
template <int BLOCK, int V>
__global__ __launch_bounds__(BLOCK) void dispatch_quant_rows_kernel(const u32x4 *__restrict__ X,
                                                                    const int32_t *__restrict__ row_map,
                                                                    u32x2 *__restrict__ window_q,
                                                                    float *__restrict__ window_scale, int k, int H16) {
  __shared__ float red[BLOCK / kWave];
  const int t = blockIdx.x, tid = threadIdx.x;
  const u32x4 *src = X + (size_t)t * (size_t)H16;
  u32x4 v[V];
  bool has[V];
#pragma unroll
  for (int x = 0; x < V; ++x) {
    const int col = tid + x * BLOCK;
    has[x] = col < H16;
    // ordinary loads, as in dispatch_slices_kernel: X may stay in the Infinity Cache from one layer to the next
    // (with streaming loads the headline dispatch takes 61-63 us instead of 47)
    v[x] = has[x] ? src[col] : u32x4{0u, 0u, 0u, 0u};
  }
  u32x2 q[V];
  const float scale = quantise_row<BLOCK, V>(v, has, q, red);
  const int32_t *rows = row_map + (size_t)t * k;
  for (int j0 = 0; j0 < k; j0 += 8) {
    int row[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) row[u] = j0 + u < k ? uniform(rows[j0 + u]) : -1;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (row[u] < 0) continue;
      u32x2 *dst = window_q + (size_t)row[u] * (size_t)H16;
#pragma unroll
      for (int x = 0; x < V; ++x)
        if (has[x]) __builtin_nontemporal_store(q[x], dst + tid + x * BLOCK);
      if (tid == 0) window_scale[row[u]] = scale;
    }
  }
}

template <int J, int U>
static hipError_t launch_dispatch_ju(const Dims &d, const void *x, const PlanView &p, void *window, int slice,
                                     hipStream_t s) {
  const unsigned units = (unsigned)(d.N / J);
  const dim3 grid((units + U - 1) / U * (unsigned)kSlices);
  return launch(dispatch_slices_kernel<128, J, U>, grid, dim3(128), 0, s, (const u32x4 *)x,
                (const int32_t *)p.row_map, (u32x4 *)window, d.k, d.H16, slice, d.N);
}

static hipError_t launch_dispatch_list(const Dims &d, const void *x, const PlanView &p, void *window, hipStream_t s) {
  // units per workgroup: as many as fit 128 lanes (a unit has as many lanes as its slice has vectors, rounded up
  // to a power of two, at least 16)
  const int slice = (d.H16 + kSlices - 1) / kSlices;
  const int U = slice > 64 ? 1 : slice > 32 ? 2 : slice > 16 ? 4 : 8;
  const dim3 grid(((unsigned)d.N + U - 1) / U * (unsigned)kSlices);
  auto go = [&](auto kernel) {
    return launch(kernel, grid, dim3(128), 0, s, (const u32x4 *)x, (const int32_t *)p.order, (u32x4 *)window, d.H16,
                  slice, d.N);
  };
  switch (U) {
    case 1: return go(dispatch_list_kernel<1>);
    case 2: return go(dispatch_list_kernel<2>);
    case 4: return go(dispatch_list_kernel<4>);
    default: return go(dispatch_list_kernel<8>);
  }
}

hipError_t launch_dispatch(const Dims &d, const void *x, const PlanView &p, void *window, hipStream_t s) {
  if (d.order_tiles > 0 && p.order) return launch_dispatch_list(d, x, p, window, s);
  // A workgroup should move a few KB, so that the grid stays within what the dispatcher sustains (about 3000
  // workgroups per microsecond), with its lanes busy.
  //   Normally one unit per workgroup; a unit takes J branches of its token until it moves 4 KB (1.75 KB
  //   when the slice fills both waves): one load feeds J stores.
  //   Slices of at most 16 columns (H <= 1024 for bf16), or of at most 32 when the routing degree does not
  //   allow enough branches per unit: a unit is as many lanes as the slice has columns (a power of two, at
  //   least 8) and 128 / lanes units, i.e. branches of neighbouring tokens, share the workgroup; J until it
  //   moves 8 KB.
  // Measured in a plan -> dispatch -> combine sequence, k = 8, us per dispatch, this rule / one unit only:
  //   H = 512, T = 131072: 212 / 544;  H = 1024, T = 131072: 466 / 828;  H = 2048, T = 65536: 436 / 459;
  //   H = 2048, k = 6, T = 8192: 37 / 58 (launches alone).
  const int slice = (d.H16 + kSlices - 1) / kSlices;
  const int slice_bytes = slice * 16;
  int lanes = 8;                                   // lanes of a unit
  while (lanes < 128 && lanes < slice) lanes *= 2;
  int want = slice <= 64 ? 4096 : 1792;
  int U = 1, J = 1;
  while (J < 8 && J * slice_bytes < want && d.k % (2 * J) == 0) J *= 2;
  // An X larger than the Infinity Cache (256 MiB) comes from HBM whatever ran before.  Reads that miss it are
  // slow while the chip is saturated with writes, and the units of a (token, slice) all wait on the same lines,
  // so fewer, larger units do better there: 2 branches per unit, 8 where a slice is a single wave.
  // Measured, k = 8, us per dispatch with this rule / without: H = 7168: T = 20480 501 / 752, 24576 632 / 915,
  // 32768 943 / 1292; H = 4096, T = 65536: 957 / 1064 (J = 4) / 1961 (J = 1).
  if ((int64_t)d.T * d.H16 * 16 > ((int64_t)256 << 20)) {
    const int most = slice <= 64 ? 8 : 2;
    while (J < most && d.k % (2 * J) == 0) J *= 2;
  }
  if (slice <= 16 || (slice <= 32 && J * slice_bytes < want)) {     // narrow, or the routing degree allows too few branches
    U = 128 / lanes;
    want = 8192;
    J = 1;
    while (J < 8 && U * J * slice_bytes < want && d.k % (2 * J) == 0) J *= 2;
  }
#define GO(J_, U_) if (J == J_ && U == U_) return launch_dispatch_ju<J_, U_>(d, x, p, window, slice, s)
  GO(1, 1); GO(2, 1); GO(4, 1); GO(8, 1);
  GO(1, 2); GO(2, 2); GO(4, 2); GO(8, 2);
  GO(1, 4); GO(2, 4); GO(4, 4); GO(8, 4);
  GO(1, 8); GO(2, 8); GO(4, 8); GO(8, 8);
  GO(1, 16); GO(2, 16); GO(4, 16); GO(8, 16);
#undef GO
  return hipErrorInvalidValue;
}

template <int B, int V, int SB, int G>
static hipError_t launch_decode_dispatch_shape(const Dims &d, const void *x, const int32_t *K, const PlanView &p,
                                               void *window, hipStream_t s) {
  const int chunks = (d.H16 + B * V - 1) / (B * V);
  const int per_group = ((d.k + G - 1) / G + SB - 1) / SB * SB;
  const size_t lds = (size_t)(4 * d.E + 1 + 2) * sizeof(int);
  const dim3 grid((unsigned)d.T * (unsigned)(chunks * G) + 1u);
  if (p.source_count)
    return launch(decode_dispatch_kernel<B, V, SB, G, false, true>, grid, dim3(B), lds, s, (const u32x4 *)x, K, window,
                  (float *)nullptr, d, p, chunks, per_group);
  return launch(decode_dispatch_kernel<B, V, SB, G, false, false>, grid, dim3(B), lds, s, (const u32x4 *)x, K, window,
                (float *)nullptr, d, p, chunks, per_group);
}

hipError_t launch_decode_dispatch(const Dims &d, const void *x, const int32_t *K, const PlanView &p, void *window,
                                  hipStream_t s) {
  // With a routing degree of at least 6 the slots of a token are split over 4 workgroups of 8 waves (2 slots
  // each), or over 2 (4 slots each) once the batch is so large that the counting, which every workgroup of a
  // token repeats over all ids, outweighs the better spread of the stores.  Measured, k = 8, us per dispatch
  // (one workgroup per token and chunk / two groups / four groups):
  //   H = 7168: T = 16: 3.9 / 3.5 / 3.5, T = 64: 4.2 / 4.0 / 4.1, T = 128: 5.4 / 4.9 / 4.8, T = 144: 6.0 / 5.5 / 5.2,
  //             T = 256: 8.8 / 8.0 / 7.7, T = 512: 16.3 / 14.6 / 14.5;
  //   H = 4096: T = 128: 4.7 / 4.2 / 4.2, T = 256: 6.3 / 5.7 / 6.2, T = 512: 11.0 / 11.2 / 12.4.
  // With several source ranks every workgroup also sums the columns of the count matrix, so two groups are the
  // better trade there (T = 128, 32 sources: 8.0 / 7.6 / 7.8 us with one / two / four groups).
  if (d.k >= 6) {
    if (d.N <= 1536 && !p.source_count) return launch_decode_dispatch_shape<512, 2, 2, 4>(d, x, K, p, window, s);
    return launch_decode_dispatch_shape<512, 2, 4, 2>(d, x, K, p, window, s);
  }
  // Few slots per token: one workgroup per token and chunk.  Every workgroup of a token repeats the
  // counting, so from about 900 branches on two vectors per lane (half as many chunks) win.
  if (d.H16 > MOE_DECODE_BLOCK && d.N >= 896)
    return launch_decode_dispatch_shape<MOE_DECODE_BLOCK, 2, 8, 1>(d, x, K, p, window, s);
  return launch_decode_dispatch_shape<MOE_DECODE_BLOCK, MOE_DECODE_VEC, 8, 1>(d, x, K, p, window, s);
}

// Whole-row workgroup shapes (threads, vectors per thread) covering H16 <= 4096, for the quantised kernels.
// Prefill: one workgroup per token.  (Smaller workgroups with more vectors per thread, and the slots of a token
// split over 2-4 workgroups as in the decode kernel, change the dispatch by less than 2 % either way.)
#define MOE_QUANT_ROW_SHAPES(GO) \
  if (d.H16 <= 256) GO(256, 1);  \
  else if (d.H16 <= 512) GO(512, 1);  \
  else if (d.H16 <= 1024) GO(1024, 1); \
  else if (d.H16 <= 2048) GO(1024, 2); \
  else GO(1024, 4)
// Decode: 8 waves where they cover the row, as for the unquantised kernel.
#define MOE_QUANT_DECODE_SHAPES(GO) \
  if (d.H16 <= 256) GO(256, 1);  \
  else if (d.H16 <= 512) GO(512, 1);  \
  else if (d.H16 <= 1024) GO(512, 2); \
  else if (d.H16 <= 2048) GO(1024, 2); \
  else GO(1024, 4)

hipError_t launch_dispatch_quant(const Dims &d, const void *x, const PlanView &p, void *window_q, float *window_scale,
                                 hipStream_t s) {
#define GO(B_, V_)                                                                                         \
  return launch(dispatch_quant_rows_kernel<B_, V_>, dim3((unsigned)d.T), dim3(B_), 0, s, (const u32x4 *)x, \
                (const int32_t *)p.row_map, (u32x2 *)window_q, window_scale, d.k, d.H16)
  MOE_QUANT_ROW_SHAPES(GO);
#undef GO
}

template <int B, int V, int SB, int G>
static hipError_t launch_decode_quant_shape(const Dims &d, const void *x, const int32_t *K, const PlanView &p,
                                            void *window_q, float *window_scale, hipStream_t s) {
  const size_t lds = (size_t)(4 * d.E + 1 + 2) * sizeof(int);
  const int per_group = ((d.k + G - 1) / G + SB - 1) / SB * SB;
  const dim3 grid((unsigned)d.T * (unsigned)G + 1u);
  if (p.source_count)
    return launch(decode_dispatch_kernel<B, V, SB, G, true, true>, grid, dim3(B), lds, s, (const u32x4 *)x, K, window_q,
                  window_scale, d, p, 1, per_group);
  return launch(decode_dispatch_kernel<B, V, SB, G, true, false>, grid, dim3(B), lds, s, (const u32x4 *)x, K, window_q,
                window_scale, d, p, 1, per_group);
}

// Slot groups as in launch_decode_dispatch.  Measured, k = 8, us per quantised dispatch, one workgroup of
// 1024 threads per token / this rule: H = 7168: T = 32: 5.1 / 3.8, T = 128: 6.0 / 5.1, T = 256: 7.4 / 6.9;
// H = 4096, T = 128: 5.3 / 4.5; H = 2048, T = 128: 5.1 / 4.2.
template <int B, int V>
static hipError_t launch_decode_quant_bv(const Dims &d, const void *x, const int32_t *K, const PlanView &p,
                                         void *window_q, float *window_scale, hipStream_t s) {
  if (d.k >= 6) {
    if (d.N <= 1536 && !p.source_count)
      return launch_decode_quant_shape<B, V, 2, 4>(d, x, K, p, window_q, window_scale, s);
    return launch_decode_quant_shape<B, V, 4, 2>(d, x, K, p, window_q, window_scale, s);
  }
  return launch_decode_quant_shape<B, V, 8, 1>(d, x, K, p, window_q, window_scale, s);
}

hipError_t launch_decode_dispatch_quant(const Dims &d, const void *x, const int32_t *K, const PlanView &p,
                                        void *window_q, float *window_scale, hipStream_t s) {
#define GO(B_, V_) return launch_decode_quant_bv<B_, V_>(d, x, K, p, window_q, window_scale, s)
  MOE_QUANT_DECODE_SHAPES(GO);
#undef GO
}

}  // namespace moe_rbf
