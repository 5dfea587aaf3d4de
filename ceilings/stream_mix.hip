// Plain streaming kernels that measure what the memory system of the device sustains for the two access
// mixes of the MoE path, independent of the library's kernels (measurement harness, not product code):
//
//   gather  : every output row is built from 8 input rows named by a table      (combine: 8 reads : 1 write)
//   scatter : every input row is copied to 8 output rows named by a table       (dispatch: 1 read : 8 writes)
//   read / write : one stream, nothing else.
//
// With the table  row(t, j) = 8 t + j  gather and scatter are purely sequential; with a table taken from a
// routing plan the rows are scattered over the expert blocks of a window exactly as in the MoE path.
// No arithmetic beyond an OR of the gathered vectors (so that every load is used); 16 bytes per lane.
// How workgroups are mapped to the data matters as much as the mix itself, so each kernel comes in several
// forms and the benchmark reports the best one:
//   map 0: workgroup b -> (row b / chunks, chunk b % chunks), a chunk being BLOCK vectors
//   map 1: workgroup b -> (column slice b % 8, row b / 8): with workgroups handed to the 8 XCDs round-robin,
//          XCD c only touches slice c of every row
//   map 2: XCD b % 8 owns a contiguous eighth of the (row, chunk) units and walks it in order
//   map 3 (gather only): one workgroup of 512 threads per compute unit; a thread works through units
//          u, u + threads, ... and holds the results of 28 of them in registers before it stores any
//          (all loads of a round first, then its stores)
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ u32x4 ld(const u32x4 *p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ void st(u32x4 *p, u32x4 v) {
  if (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// (row group, column range) of workgroup b.  `groups` row groups, `cols` vectors per row.
template <int BLOCK>
__device__ __forceinline__ void unit_of(int b, int map, int cols, int *g, int *c0, int *c1) {
  if (map == 1) {
    const int slice = (cols + 7) / 8;
    *g = b / 8;
    *c0 = (b % 8) * slice;
    *c1 = min(cols, *c0 + slice);
    return;
  }
  const int chunks = (cols + BLOCK - 1) / BLOCK;
  int u = b;
  if (map == 2) u = (b % 8) * ((int)gridDim.x / 8) + b / 8;
  *g = u / chunks;
  *c0 = (u % chunks) * BLOCK;
  *c1 = min(cols, *c0 + BLOCK);
}

template <int BLOCK, bool NT_LOAD>
__global__ __launch_bounds__(BLOCK) void gather8_kernel(const u32x4 *__restrict__ in, const int32_t *__restrict__ table,
                                                        u32x4 *__restrict__ out, int rows, int cols, int map) {
  int t, c0, c1;
  unit_of<BLOCK>(blockIdx.x, map, cols, &t, &c0, &c1);
  if (t >= rows) return;
  int r[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = __builtin_amdgcn_readfirstlane(table[(size_t)t * 8 + j]);
  for (int col = c0 + (int)threadIdx.x; col < c1; col += BLOCK) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = ld<NT_LOAD>(in + (size_t)r[j] * (size_t)cols + col);
    u32x4 acc = v[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) acc |= v[j];
    st<true>(out + (size_t)t * (size_t)cols + col, acc);
  }
}

// map 3: persistent grid, stores held back.  cols must be a multiple of 64 (a wave stays inside one row).
// The (row, column) of a thread's next unit is stepped, not divided out, so that nothing slow sits between
// the loads of one unit and those of the next.
__global__ __launch_bounds__(512) void gather8_held_kernel(const u32x4 *__restrict__ in, const int32_t *__restrict__ table,
                                                           u32x4 *__restrict__ out, int rows, int cols) {
  constexpr int kHeld = 28;
  const int step = (int)gridDim.x * 512, rows_per_step = step / cols, cols_per_step = step % cols;
  const long long units = (long long)rows * cols;
  for (long long first = (long long)blockIdx.x * 512 + threadIdx.x; first < units; first += (long long)step * kHeld) {
    const int t0 = (int)(first / cols), c0 = (int)(first - (long long)t0 * cols);
    u32x4 held[kHeld];
    int t = t0, c = c0;
#pragma unroll
    for (int i = 0; i < kHeld; ++i) {
      if (t < rows) {
        const int32_t *e = table + (size_t)__builtin_amdgcn_readfirstlane(t) * 8;
        int r[8];
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = __builtin_amdgcn_readfirstlane(e[j]);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = ld<true>(in + (size_t)r[j] * (size_t)cols + c);
        u32x4 acc = v[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) acc |= v[j];
        held[i] = acc;
      }
      c += cols_per_step, t += rows_per_step;
      if (c >= cols) c -= cols, ++t;
    }
    t = t0, c = c0;
#pragma unroll
    for (int i = 0; i < kHeld; ++i) {
      if (t < rows) st<true>(out + (size_t)t * (size_t)cols + c, held[i]);
      c += cols_per_step, t += rows_per_step;
      if (c >= cols) c -= cols, ++t;
    }
  }
}

// J table entries (destination rows) of one input row per workgroup; 8 entries per input row
template <int BLOCK, int J, bool NT_LOAD>
__global__ __launch_bounds__(BLOCK) void scatter8_kernel(const u32x4 *__restrict__ in, const int32_t *__restrict__ table,
                                                         u32x4 *__restrict__ out, int rows, int cols, int map) {
  int g, c0, c1;
  unit_of<BLOCK>(blockIdx.x, map, cols, &g, &c0, &c1);
  const int n = g * J;
  if (n >= rows * 8) return;
  const int t = n / 8;
  int r[J];
#pragma unroll
  for (int j = 0; j < J; ++j) r[j] = __builtin_amdgcn_readfirstlane(table[n + j]);
  for (int col = c0 + (int)threadIdx.x; col < c1; col += BLOCK) {
    const u32x4 v = ld<NT_LOAD>(in + (size_t)t * (size_t)cols + col);
#pragma unroll
    for (int j = 0; j < J; ++j) st<true>(out + (size_t)r[j] * (size_t)cols + col, v);
  }
}

// One stream over n vectors, one workgroup per BLOCK vectors.
template <int BLOCK, bool NT>
__global__ __launch_bounds__(BLOCK) void write_kernel(u32x4 *__restrict__ out, size_t n) {
  const size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
  if (i < n) st<NT>(out + i, u32x4{1u, 2u, 3u, 4u});
}
template <int BLOCK, bool NT>
__global__ __launch_bounds__(BLOCK) void read_kernel(const u32x4 *__restrict__ in, size_t n, u32x4 *__restrict__ sink) {
  const size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
  if (i >= n) return;
  const u32x4 v = ld<NT>(in + i);
  if (v[0] == 0x12345678u && v[1] == 0x9abcdef0u) sink[0] = v;     // never true for the benchmark's data
}

extern "C" {

// Every entry point returns the hipError_t of its launch (or hipErrorInvalidValue for an unknown form).
// table: device int32 [rows * 8], every entry inside the indexed buffer (the caller checks this).
// cols: 16-byte vectors per row.

int ceil_gather8(int block, int nt_load, int map, const void *in, const int32_t *table, void *out, int rows, int cols,
                 void *stream) {
  if (map == 3) {
    int dev = 0, cus = 0;
    if (rows < 1 || cols < 64 || cols % 64 != 0 || block != 512) return (int)hipErrorInvalidValue;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
      return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(gather8_held_kernel, dim3(cus), dim3(512), 0, (hipStream_t)stream, (const u32x4 *)in, table,
                       (u32x4 *)out, rows, cols);
    return (int)hipGetLastError();
  }
  const long long per = map == 1 ? 8 : (cols + block - 1) / block;
  long long units = (long long)rows * per;
  if (map == 2) units = (units + 7) / 8 * 8;
  if (rows < 1 || cols < 1 || units > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  const dim3 g((unsigned)units);
#define GO(B, L) hipLaunchKernelGGL((gather8_kernel<B, L>), g, dim3(B), 0, (hipStream_t)stream, (const u32x4 *)in, table, \
                                    (u32x4 *)out, rows, cols, map)
  if (block == 64) { if (nt_load) GO(64, true); else GO(64, false); }
  else if (block == 128) { if (nt_load) GO(128, true); else GO(128, false); }
  else return (int)hipErrorInvalidValue;
#undef GO
  return (int)hipGetLastError();
}

int ceil_scatter8(int per_unit, int nt_load, int map, const void *in, const int32_t *table, void *out, int rows, int cols,
                  void *stream) {
  constexpr int B = 128;
  const long long per = map == 1 ? 8 : (cols + B - 1) / B;
  long long units = (long long)rows * 8 / per_unit * per;
  if (map == 2) units = (units + 7) / 8 * 8;
  if (rows < 1 || cols < 1 || units > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  const dim3 g((unsigned)units);
#define GO(J, L) hipLaunchKernelGGL((scatter8_kernel<B, J, L>), g, dim3(B), 0, (hipStream_t)stream, (const u32x4 *)in, table, \
                                    (u32x4 *)out, rows, cols, map)
  if (per_unit == 1) { if (nt_load) GO(1, true); else GO(1, false); }
  else if (per_unit == 8) { if (nt_load) GO(8, true); else GO(8, false); }
  else return (int)hipErrorInvalidValue;
#undef GO
  return (int)hipGetLastError();
}

int ceil_write(int nt, void *out, size_t n_vec, void *stream) {
  constexpr int B = 256;
  const dim3 g((unsigned)((n_vec + B - 1) / B));
  if (nt) hipLaunchKernelGGL((write_kernel<B, true>), g, dim3(B), 0, (hipStream_t)stream, (u32x4 *)out, n_vec);
  else hipLaunchKernelGGL((write_kernel<B, false>), g, dim3(B), 0, (hipStream_t)stream, (u32x4 *)out, n_vec);
  return (int)hipGetLastError();
}

int ceil_read(int nt, const void *in, size_t n_vec, void *sink, void *stream) {
  constexpr int B = 128;
  const dim3 g((unsigned)((n_vec + B - 1) / B));
  if (nt) hipLaunchKernelGGL((read_kernel<B, true>), g, dim3(B), 0, (hipStream_t)stream, (const u32x4 *)in, n_vec, (u32x4 *)sink);
  else hipLaunchKernelGGL((read_kernel<B, false>), g, dim3(B), 0, (hipStream_t)stream, (const u32x4 *)in, n_vec, (u32x4 *)sink);
  return (int)hipGetLastError();
}

}  // extern "C"
