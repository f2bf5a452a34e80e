// Device-side helpers for the gfx950 kernels: index chunk addressing in the
// device layout, fp16-pair dot product, wave-level reductions.
//
// Device layout of the packed indices (what vq_pack_layout writes).  A group is
// 8 rows x 128 vectors.  Lane L of a wave owns the two vectors 2L, 2L+1 of every
// row of a group, so that its activations (x[4L..4L+3] of the group's columns)
// stay in two registers and one lane keeps 8 row accumulators.
//   4-bit (k=16): a lane's share of a group is 8 bytes, byte r = row r,
//     low nibble = vector 2L, high nibble = vector 2L+1 (= canonical byte
//     r*64 + L of the group).  Two horizontally adjacent groups (col-blocks
//     2p, 2p+1 of one row-block) are interleaved per lane: 16 bytes per lane,
//     1 KB per wave-wide 128-bit load.  If the number of col-blocks is odd the
//     last group of the row-block follows as 64 x 8 bytes.
//   8-bit (k=256): a lane's share is 16 bytes, byte 2r+e = row r, vector 2L+e
//     (= canonical byte r*128 + 2L + e); one group per wave-wide 128-bit load.
// Codebooks keep the canonical order (one dword per centroid).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vq {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
typedef float f16v_t __attribute__((ext_vector_type(16)));

// acc + c.lo*x.lo + c.hi*x.hi with fp32 accumulation (v_dot2_f32_f16).
__device__ __forceinline__ float dot2(uint32_t c, uint32_t x, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(h2_t, c), __builtin_bit_cast(h2_t, x), acc, false);
}

// Orders this wave's LDS writes before its later LDS reads (other lanes' data).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Byte offset of lane `lane`'s 8-byte share of 4-bit group (row-block base + ...).
__device__ __forceinline__ size_t k16_chunk_offset(int c, int n_cb, int lane) {
  const int n_pairs = n_cb >> 1;
  if (c < 2 * n_pairs) return (size_t)(c >> 1) * 1024 + lane * 16 + (c & 1) * 8;
  return (size_t)n_pairs * 1024 + lane * 8;
}

// Sum 8 per-lane row accumulators over the 64 lanes.  Returns, in every lane, the
// total of row (lane >> 3) & 7.  Halving exchange: 4 + 2 + 1 swaps, then 3 butterflies.
__device__ __forceinline__ float wave_reduce8(const float (&a)[8], int lane) {
  float b[4], c[2];
  bool up = lane & 32;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float send = up ? a[i] : a[i + 4];
    float keep = up ? a[i + 4] : a[i];
    b[i] = keep + __shfl_xor(send, 32);
  }
  up = lane & 16;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    float send = up ? b[i] : b[i + 2];
    float keep = up ? b[i + 2] : b[i];
    c[i] = keep + __shfl_xor(send, 16);
  }
  up = lane & 8;
  float send = up ? c[0] : c[1];
  float keep = up ? c[1] : c[0];
  float v = keep + __shfl_xor(send, 8);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 1);
  return v;
}

}  // namespace vq
