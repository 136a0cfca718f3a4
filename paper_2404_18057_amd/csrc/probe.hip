// Bandwidth probes: a streaming read and a random 256-byte-row read.  They give
// the measured denominators for the two rooflines of the method (HBM for the K
// scan, the host link for the V pull; paper section 3.2, equations (3)-(4)).
#include "kc_internal.h"

namespace kc {
namespace {

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ p, size_t n16,
                                                         uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256 * 8;
  uint32_t acc = 0;
  for (size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x; i < n16; i += stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const size_t j = i + (size_t)u * 256;
      v[u] = j < n16 ? load_stream16(p + j) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // keeps the loads alive, practically never taken
}

__global__ __launch_bounds__(256) void probe_rows_kernel(const uint4* __restrict__ p,
                                                         unsigned long long total_rows,
                                                         long long n_rows,
                                                         uint32_t* __restrict__ sink) {
  const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const long long stride = (long long)gridDim.x * 16 * 8;
  uint32_t acc = 0;
  for (long long r0 = (long long)blockIdx.x * 16 * 8 + grp; r0 < n_rows; r0 += stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const long long r = r0 + (long long)u * 16;
      unsigned long long x = (unsigned long long)r * 0x9E3779B97F4A7C15ull;
      x ^= x >> 29;
      x *= 0xBF58476D1CE4E5B9ull;
      x ^= x >> 32;
      v[u] = r < n_rows ? p[(x % total_rows) * 16 + sub] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

}  // namespace

hipError_t launch_probe_read(const void* ptr, size_t bytes, uint32_t* sink, hipStream_t st) {
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 2047) / 2048;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                     static_cast<const uint4*>(ptr), n16, sink);
  return hipGetLastError();
}

hipError_t launch_probe_rows(const void* ptr, size_t total_rows, int64_t n_rows, uint32_t* sink,
                             hipStream_t st) {
  if (total_rows == 0 || n_rows <= 0) return hipSuccess;
  long long blocks = (n_rows + 127) / 128;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(probe_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                     static_cast<const uint4*>(ptr), (unsigned long long)total_rows,
                     (long long)n_rows, sink);
  return hipGetLastError();
}

}  // namespace kc
