// Row-wise quantisation of a token row for the quantised dispatch (paper, Section 5.2, end of "Prefill
// Dispatch"): row scales are kept in a separate float array indexed by window row.
// The paper names no format; this library uses OCP FP8 E4M3 codes with one fp32 scale per row:
//   amax = max |x| over the row, scale = amax / 448 (stored), q = e4m3(x * (448 / amax)), nearest even;
//   an all-zero row gets scale 1.
// A workgroup holds one whole row: V 16-byte vectors (8 bf16 each) per thread.
#pragma once
#include "device_utils.h"

namespace moe_rbf {

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max_step(float v) {
  const float o =
      __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false));
  return fmaxf(v, o);
}

__device__ __forceinline__ float wave_max_nonneg(float v) {   // maximum over the wave of values >= 0
  v = dpp_max_step<0x111, 0xf>(v);   // row_shr:1
  v = dpp_max_step<0x112, 0xf>(v);   // row_shr:2
  v = dpp_max_step<0x114, 0xf>(v);   // row_shr:4
  v = dpp_max_step<0x118, 0xf>(v);   // row_shr:8
  v = dpp_max_step<0x142, 0xa>(v);   // row_bcast:15
  v = dpp_max_step<0x143, 0xc>(v);   // row_bcast:31
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), kWave - 1));
}

// Quantises the row held by the workgroup.  v[x] is the thread's x-th vector (has[x] false past the row's
// end).  q[x] receives the 8 codes of vector x; the return value is the row's scale.
// red[] is LDS scratch of BLOCK/64 floats; contains a barrier.
template <int BLOCK, int V>
__device__ __forceinline__ float quantise_row(const u32x4 (&v)[V], const bool (&has)[V], u32x2 (&q)[V], float *red) {
  float amax = 0.0f;
#pragma unroll
  for (int x = 0; x < V; ++x) {
    if (!has[x]) continue;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      amax = fmaxf(amax, fabsf(__uint_as_float(v[x][i] << 16)));
      amax = fmaxf(amax, fabsf(__uint_as_float(v[x][i] & 0xffff0000u)));
    }
  }
  amax = wave_max_nonneg(amax);
  if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = amax;
  __syncthreads();
  float m = 0.0f;
#pragma unroll
  for (int w = 0; w < BLOCK / kWave; ++w) m = fmaxf(m, red[w]);
  const float scale = m == 0.0f ? 1.0f : m / 448.0f;
  const float inv = m == 0.0f ? 1.0f : 448.0f / m;
#pragma unroll
  for (int x = 0; x < V; ++x) {
    float f[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(v[x][i] << 16) * inv;
      f[2 * i + 1] = __uint_as_float(v[x][i] & 0xffff0000u) * inv;
    }
    int lo = 0, hi = 0;
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], lo, false);
    lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], hi, false);
    hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
    q[x] = u32x2{(unsigned)lo, (unsigned)hi};
  }
  return scale;
}

}  // namespace moe_rbf
