// One-time re-layout: canonical indices and codebooks -> device layout (see
// vq_device.h for the layout and the reason for it; Sec. 3.2: the index stream is
// organised for vector loads).  Off the hot path.
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

// One thread per (device group slot, lane): gathers that lane's share of the group.
// For k=16 the slots include the zero-filled pad group of row-blocks with an odd
// number of col-blocks.
template <int K>
__global__ __launch_bounds__(256) void pack_idx_kernel(const uint8_t* __restrict__ canon,
                                                       uint8_t* __restrict__ dev, int n_cb,
                                                       long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long slot = t >> 6;
  const int lane = (int)(t & 63);
  if (slot >= n_slots) return;
  if (K == 16) {
    const int slots_per_rb = 2 * k16_pairs(n_cb);
    const long long rb = slot / slots_per_rb;
    const int c = (int)(slot - rb * slots_per_rb);
    uint32_t words[2] = {0u, 0u};
    if (c < n_cb) {
      const uint8_t* src = canon + (rb * n_cb + c) * 512 + lane;   // canonical byte r*64 + lane
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const uint32_t byte = src[(4 * h + b) * 64];
          lo[b] = byte & 15u;
          hi[b] = byte >> 4;
        }
        words[h] = k16_encode_dword(lo, hi);
      }
    }
    uint8_t* dst = dev + rb * slots_per_rb * 512 + k16_chunk_offset(c, lane);
    *reinterpret_cast<uint2*>(dst) = make_uint2(words[0], words[1]);
  } else {
    const long long g = slot;
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

// Codebooks: canonical order; k=16 row-blocks with an odd number of col-blocks get a
// zero codebook for the pad group.  One thread per 16 bytes of the device array.
__global__ __launch_bounds__(256) void pack_cb_kernel(const uint4* __restrict__ src,
                                                      uint4* __restrict__ dst, int k, int n_cb,
                                                      long long n16) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n16) return;
  const int per_group = k / 4;                                  // 16-byte pieces per codebook
  const int slots_per_rb = k == 16 ? 2 * k16_pairs(n_cb) : n_cb;
  const long long slot = t / per_group;
  const int piece = (int)(t - slot * per_group);
  const long long rb = slot / slots_per_rb;
  const int c = (int)(slot - rb * slots_per_rb);
  dst[t] = c < n_cb ? src[(rb * n_cb + c) * per_group + piece] : make_uint4(0, 0, 0, 0);
}

// Reads n16 16-byte pieces once (non-temporal) and keeps the optimiser from dropping the loads.
typedef unsigned int probe_u32x4_t __attribute__((ext_vector_type(4)));
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

hipError_t launch_stream_read(const void* buf, size_t bytes, hipStream_t s) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(4096), dim3(256), 0, s,
                     (const probe_u32x4_t*)buf, (long long)(bytes / 16), (unsigned*)nullptr);
  return hipGetLastError();
}

hipError_t launch_pack(const vq_desc& d, const void* idx_canon, const void* cb_canon,
                       void* idx_dev, void* cb_dev, hipStream_t s) {
  const int n_cb = d.in_features / kGroupCols;
  const long long n_rb = d.out_features / kGroupRows;
  const long long n_slots = n_rb * (d.k == 16 ? 2 * k16_pairs(n_cb) : n_cb);
  const unsigned grid = (unsigned)((n_slots * 64 + 255) / 256);
  if (d.k == 16)
    hipLaunchKernelGGL(pack_idx_kernel<16>, dim3(grid), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots);
  else
    hipLaunchKernelGGL(pack_idx_kernel<256>, dim3(grid), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long n16 = n_slots * d.k * 4 / 16;
  hipLaunchKernelGGL(pack_cb_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                     (const uint4*)cb_canon, (uint4*)cb_dev, d.k, n_cb, n16);
  return hipGetLastError();
}

}  // namespace vq
