// Plain streaming kernels that measure what the memory system of the device sustains for the two access
// mixes of the MoE path, independent of the library's kernels (measurement harness, not product code):
//
//   gather  : every output row is built from NR input rows named by a table     (combine: 8 reads : 1 write)
//   scatter : every input row is copied to NW output rows named by a table      (dispatch: 1 read : 8 writes)
//
// With the table  row(t, j) = t * N + j  both are purely sequential streams; with a table taken from a
// routing plan the rows are scattered over the expert blocks of a window exactly as in the MoE path.
// No arithmetic beyond an OR of the gathered vectors (so that every load is used); 16 bytes per lane;
// streaming (nontemporal) accesses unless PLAIN.  Two launch forms: one workgroup per (row, 128-column
// chunk), and a persistent grid whose workgroups stride over those units.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool PLAIN>
__device__ __forceinline__ u32x4 ld(const u32x4 *p) {
  return PLAIN ? *p : __builtin_nontemporal_load(p);
}
template <bool PLAIN>
__device__ __forceinline__ void st(u32x4 *p, u32x4 v) {
  if (PLAIN) *p = v;
  else __builtin_nontemporal_store(v, p);
}

template <int N, bool PLAIN>
__global__ __launch_bounds__(128) void gather_kernel(const u32x4 *__restrict__ in, const int32_t *__restrict__ table,
                                                     u32x4 *__restrict__ out, int rows, int cols, int chunks) {
  const int units = rows * chunks;
  for (int unit = blockIdx.x; unit < units; unit += gridDim.x) {
    const int t = unit / chunks;
    const int col = (unit - t * chunks) * 128 + (int)threadIdx.x;
    if (col >= cols) continue;
    int r[N];
#pragma unroll
    for (int j = 0; j < N; ++j) r[j] = __builtin_amdgcn_readfirstlane(table[(size_t)t * N + j]);
    u32x4 v[N];
#pragma unroll
    for (int j = 0; j < N; ++j) v[j] = ld<PLAIN>(in + (size_t)r[j] * (size_t)cols + col);
    u32x4 acc = v[0];
#pragma unroll
    for (int j = 1; j < N; ++j) acc |= v[j];
    st<PLAIN>(out + (size_t)t * (size_t)cols + col, acc);
  }
}

template <int N, bool PLAIN>
__global__ __launch_bounds__(128) void scatter_kernel(const u32x4 *__restrict__ in, const int32_t *__restrict__ table,
                                                      u32x4 *__restrict__ out, int rows, int cols, int chunks) {
  const int units = rows * chunks;
  for (int unit = blockIdx.x; unit < units; unit += gridDim.x) {
    const int t = unit / chunks;
    const int col = (unit - t * chunks) * 128 + (int)threadIdx.x;
    if (col >= cols) continue;
    int r[N];
#pragma unroll
    for (int j = 0; j < N; ++j) r[j] = __builtin_amdgcn_readfirstlane(table[(size_t)t * N + j]);
    const u32x4 v = ld<PLAIN>(in + (size_t)t * (size_t)cols + col);
#pragma unroll
    for (int j = 0; j < N; ++j) st<PLAIN>(out + (size_t)r[j] * (size_t)cols + col, v);
  }
}

// Plain read-only and write-only streams over `n` 16-byte vectors (grid-stride).
__global__ __launch_bounds__(256) void read_kernel(const u32x4 *__restrict__ in, size_t n, u32x4 *__restrict__ sink) {
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    acc |= __builtin_nontemporal_load(in + i);
  if (acc[0] == 0x12345678u && acc[1] == 0x9abcdef0u) sink[0] = acc;     // never true for the benchmark's data
}
__global__ __launch_bounds__(256) void write_kernel(u32x4 *__restrict__ out, size_t n) {
  const u32x4 v = {1u, 2u, 3u, 4u};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
    __builtin_nontemporal_store(v, out + i);
}

extern "C" {

// kind: 0 = gather (table rows index `in`), 1 = scatter (table rows index `out`).  n_per_row: 1 or 8.
// table: device int32 [rows * n_per_row], every entry inside the indexed buffer (the caller's job).
// cols: 16-byte vectors per row.  grid: 0 = one workgroup per (row, chunk), else that many persistent workgroups.
// Returns the hipError_t of the launch.
int ceil_mix(int kind, int n_per_row, int plain, const void *in, const int32_t *table, void *out, int rows, int cols,
             int grid, void *stream) {
  const int chunks = (cols + 127) / 128;
  const long long units = (long long)rows * chunks;
  if (rows < 1 || cols < 1 || units > 0x7fffffffLL || (n_per_row != 1 && n_per_row != 8)) return (int)hipErrorInvalidValue;
  const dim3 g((unsigned)(grid > 0 ? grid : units)), b(128);
  hipStream_t s = (hipStream_t)stream;
  const u32x4 *i = (const u32x4 *)in;
  u32x4 *o = (u32x4 *)out;
#define GO(K, N, P) hipLaunchKernelGGL((K<N, P>), g, b, 0, s, i, table, o, rows, cols, chunks)
  if (kind == 0) {
    if (n_per_row == 8) { if (plain) GO(gather_kernel, 8, true); else GO(gather_kernel, 8, false); }
    else { if (plain) GO(gather_kernel, 1, true); else GO(gather_kernel, 1, false); }
  } else {
    if (n_per_row == 8) { if (plain) GO(scatter_kernel, 8, true); else GO(scatter_kernel, 8, false); }
    else { if (plain) GO(scatter_kernel, 1, true); else GO(scatter_kernel, 1, false); }
  }
#undef GO
  return (int)hipGetLastError();
}

int ceil_read(const void *in, size_t n_vec, void *sink, int grid, void *stream) {
  hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)in, n_vec, (u32x4 *)sink);
  return (int)hipGetLastError();
}

int ceil_write(void *out, size_t n_vec, int grid, void *stream) {
  hipLaunchKernelGGL(write_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (u32x4 *)out, n_vec);
  return (int)hipGetLastError();
}

}  // extern "C"
