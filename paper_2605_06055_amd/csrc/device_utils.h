// Device-side helpers for the gfx950 kernels: 128-bit vector type, wave64 primitives.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe_rbf {

// 16-byte payload unit: one global_load/store_dwordx4 per lane.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() {
  return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Force a block-uniform value into a scalar register.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Number of bits needed to tell ids 0..E-1 apart.
__host__ __device__ inline int id_bits(int E) {
  int b = 0;
  while ((1 << b) < E) ++b;
  return b;
}

// For each lane with `valid`, the 64-bit mask of valid lanes in the wave that hold the same id.
// One ballot per id bit narrows the peer set.
__device__ __forceinline__ unsigned long long match_any(int id, bool valid, int bits) {
  unsigned long long mask = __ballot(valid);
  for (int b = 0; b < bits; ++b) {
    const bool bit = (id >> b) & 1;
    const unsigned long long m = __ballot(valid && bit);
    mask &= bit ? m : ~m;
  }
  return mask;
}

// Inclusive prefix sum across the 64 lanes of a wave with DPP row shifts and row broadcasts (no LDS
// traffic): shifts by 1,2,4,8 inside each row of 16 lanes, then the last lane of row 0/2 is added
// to row 1/3 and the last lane of the lower half to the upper half.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2 and 3
  return v;
}

// Sum of a 64-bit count (below 2^60) over the 64 lanes of a wave, as three 20-bit limbs through the DPP scan.
// Every lane of the wave must call; the result is uniform.
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
  const int l0 = (int)(v & 0xFFFFFu), l1 = (int)((v >> 20) & 0xFFFFFu), l2 = (int)(v >> 40);
  const unsigned s0 = (unsigned)__builtin_amdgcn_readlane(wave_inclusive_scan(l0), kWave - 1);
  const unsigned s1 = (unsigned)__builtin_amdgcn_readlane(wave_inclusive_scan(l1), kWave - 1);
  const unsigned s2 = (unsigned)__builtin_amdgcn_readlane(wave_inclusive_scan(l2), kWave - 1);
  return (unsigned long long)s0 + ((unsigned long long)s1 << 20) + ((unsigned long long)s2 << 40);
}

// Exclusive prefix sum of total[0..E) into g[0..E], g[E] = grand total; executed by ONE wave
// (all 64 lanes of it must call).  Each lane owns a run of consecutive experts; E <= 1024.
// Only the bits of total[] selected by `mask` are counts; `addend` (optional) is added element-wise.
__device__ __forceinline__ void wave_exclusive_scan_lds(const int *total, int *g, int E, int mask = -1,
                                                        const int *addend = nullptr) {
  constexpr int kMaxPer = 16;
  const int lane = lane_id();
  const int per = (E + kWave - 1) / kWave;
  const int b = lane * per;
  int c[kMaxPer];
#pragma unroll
  for (int x = 0; x < kMaxPer; ++x)
    c[x] = (x < per && b + x < E) ? (total[b + x] & mask) + (addend ? addend[b + x] : 0) : 0;
  int sum = 0;
#pragma unroll
  for (int x = 0; x < kMaxPer; ++x) sum += c[x];
  const int incl = wave_inclusive_scan(sum);
  int run = incl - sum;
#pragma unroll
  for (int x = 0; x < kMaxPer; ++x) {
    if (x < per && b + x < E) g[b + x] = run;
    run += c[x];
  }
  if (lane == kWave - 1) g[E] = incl;
}

// Streaming 16-byte accesses: the payload is touched once by these kernels.
__device__ __forceinline__ u32x4 load_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store_stream(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, p); }

}  // namespace moe_rbf
