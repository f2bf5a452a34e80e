// One-time re-layout: canonical indices -> device layout (see vq_device.h for the
// layout and the reason for it; Sec. 3.2: the index stream is organised for
// vector loads).  Codebooks are copied unchanged.  Off the hot path.
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

// One thread per (group, lane): gathers that lane's share of the group.
template <int K>
__global__ __launch_bounds__(256) void pack_idx_kernel(const uint8_t* __restrict__ canon,
                                                       uint8_t* __restrict__ dev, int n_cb,
                                                       long long n_groups) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long g = t >> 6;
  const int lane = (int)(t & 63);
  if (g >= n_groups) return;
  if (K == 16) {
    const long long rb = g / n_cb;
    const int c = (int)(g - rb * n_cb);
    const uint8_t* src = canon + g * 512 + lane;
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      lo |= (uint32_t)src[r * 64] << (8 * r);
      hi |= (uint32_t)src[(r + 4) * 64] << (8 * r);
    }
    uint8_t* dst = dev + rb * n_cb * 512 + k16_chunk_offset(c, n_cb, lane);
    *reinterpret_cast<uint2*>(dst) = make_uint2(lo, hi);
  } else {
    const uint8_t* src = canon + g * 1024 + 2 * lane;
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t a = *reinterpret_cast<const uint16_t*>(src + (2 * q) * 128);
      const uint32_t b = *reinterpret_cast<const uint16_t*>(src + (2 * q + 1) * 128);
      w[q] = a | (b << 16);
    }
    *reinterpret_cast<uint4*>(dev + g * 1024 + lane * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

__global__ __launch_bounds__(256) void copy16_kernel(const uint4* __restrict__ src,
                                                     uint4* __restrict__ dst, long long n16) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t < n16) dst[t] = src[t];
}

}  // namespace

hipError_t launch_pack(const vq_desc& d, const void* idx_canon, const void* cb_canon,
                       void* idx_dev, void* cb_dev, hipStream_t s) {
  const int n_cb = d.in_features / kGroupCols;
  const long long n_groups = (long long)(d.out_features / kGroupRows) * n_cb;
  const unsigned grid = (unsigned)((n_groups * 64 + 255) / 256);
  if (d.k == 16)
    hipLaunchKernelGGL(pack_idx_kernel<16>, dim3(grid), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_groups);
  else
    hipLaunchKernelGGL(pack_idx_kernel<256>, dim3(grid), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_groups);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long n16 = n_groups * d.k * 4 / 16;
  hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                     (const uint4*)cb_canon, (uint4*)cb_dev, n16);
  return hipGetLastError();
}

}  // namespace vq
