// Measurement aid of the benchmark, built into a library of its own (libvq_bench.so): not part
// of the product's ABI.  Reads a buffer once with the same non-temporal 128-bit loads the GEMV
// kernels stream their indices with, and discards the data.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "../../include/vq_bench.h"

namespace {

typedef unsigned int probe_u32x4_t __attribute__((ext_vector_type(4)));

// Reads n16 16-byte pieces once and keeps the optimiser from dropping the loads.
__global__ __launch_bounds__(256) void stream_read_kernel(const probe_u32x4_t* __restrict__ p,
                                                          long long n16, unsigned* sink) {
  unsigned acc = 0;
  const long long stride = (long long)gridDim.x * 256 * 4;
  for (long long base = (long long)blockIdx.x * 256 * 4 + threadIdx.x; base < n16; base += stride) {
    probe_u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const long long i = base + u * 256;
      v[u] = i < n16 ? __builtin_nontemporal_load(p + i) : probe_u32x4_t{0, 0, 0, 0};
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u && sink) *sink = acc;   // never true for the fill patterns used; sink may be null
}

}  // namespace

extern "C" int vq_bench_stream_read(const void* buf, size_t bytes, void* stream) {
  if (!buf) return -1;
  if (reinterpret_cast<uintptr_t>(buf) & 15u) return -4;
  if (bytes == 0 || (bytes & 15)) return -6;
  hipLaunchKernelGGL(stream_read_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream,
                     (const probe_u32x4_t*)buf, (long long)(bytes / 16), (unsigned*)nullptr);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}
