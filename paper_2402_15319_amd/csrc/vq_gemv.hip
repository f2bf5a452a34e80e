// Batch-1 product y = W x on vector-quantised W (Sec. 3.2: decode by table
// lookup, then matrix-vector multiply), fused: packed indices are streamed
// from HBM with 128-bit loads, each group's codebook is staged in LDS, and
// every looked-up fp16 pair goes straight into a fp32-accumulating dot2.
//
// Work decomposition: a workgroup has 4 waves.  A wave walks a strip of
// col-blocks of one row-block (8 rows); `splits` waves share a row-block and
// their partial sums meet in LDS, so the result is deterministic.
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

// Looks up the 8 vectors of one dword of 4-bit indices (4 rows x 2 vectors).
__device__ __forceinline__ void k16_dword(uint32_t w, const uint32_t* t, uint32_t x0, uint32_t x1,
                                          float* acc) {
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const uint32_t lo = (w >> (8 * r)) & 15u;
    const uint32_t hi = (w >> (8 * r + 4)) & 15u;
    acc[r] = dot2(t[lo], x0, acc[r]);
    acc[r] = dot2(t[hi], x1, acc[r]);
  }
}

// Looks up the 4 vectors of one dword of 8-bit indices (2 rows x 2 vectors).
__device__ __forceinline__ void k256_dword(uint32_t w, const uint32_t* t, uint32_t x0, uint32_t x1,
                                           float* acc) {
  acc[0] = dot2(t[w & 255u], x0, acc[0]);
  acc[0] = dot2(t[(w >> 8) & 255u], x1, acc[0]);
  acc[1] = dot2(t[(w >> 16) & 255u], x0, acc[1]);
  acc[1] = dot2(t[w >> 24], x1, acc[1]);
}

// k = 16: strip of col-block pairs [p0, p1) (+ the odd tail group) of row-block rb.
__device__ __forceinline__ void strip_k16(const GemvProblem& P, int rb, int split, int splits,
                                          int lane, uint32_t* lut, float (&acc)[8]) {
  const int n_cb = P.n_cb;
  const int n_pairs = n_cb >> 1;
  const int p0 = (n_pairs * split) / splits;
  const int p1 = (n_pairs * (split + 1)) / splits;
  const uint8_t* idx_rb = P.idx + (size_t)rb * n_cb * 512;
  const uint32_t* cb_rb = P.cb + (size_t)rb * n_cb * 16;
  const uint16_t* x = P.x;

  for (int pc = p0; pc < p1; pc += 8) {
    const int np = min(8, p1 - pc);
    // codebooks of the 2*np groups of this chunk: 32*np dwords, 4 per lane
    uint4 cbv = make_uint4(0, 0, 0, 0);
    if (lane * 4 < np * 32) cbv = *reinterpret_cast<const uint4*>(cb_rb + pc * 32 + lane * 4);
    wave_lds_sync();  // earlier lookups of this wave are done with the table
    *reinterpret_cast<uint4*>(lut + lane * 4) = cbv;
    wave_lds_sync();
#pragma unroll 4
    for (int q = 0; q < np; ++q) {
      const int p = pc + q;
      const uint4 w = *reinterpret_cast<const uint4*>(idx_rb + (size_t)p * 1024 + lane * 16);
      const uint2 xa = *reinterpret_cast<const uint2*>(x + (2 * p) * 256 + lane * 4);
      const uint2 xb = *reinterpret_cast<const uint2*>(x + (2 * p + 1) * 256 + lane * 4);
      const uint32_t* ta = lut + q * 32;
      k16_dword(w.x, ta, xa.x, xa.y, acc);
      k16_dword(w.y, ta, xa.x, xa.y, acc + 4);
      k16_dword(w.z, ta + 16, xb.x, xb.y, acc);
      k16_dword(w.w, ta + 16, xb.x, xb.y, acc + 4);
    }
  }
  if ((n_cb & 1) && split == splits - 1) {
    const int c = n_cb - 1;
    uint32_t cbv = 0;
    if (lane < 16) cbv = cb_rb[c * 16 + lane];
    wave_lds_sync();
    if (lane < 16) lut[lane] = cbv;
    wave_lds_sync();
    const uint2 w = *reinterpret_cast<const uint2*>(idx_rb + (size_t)n_pairs * 1024 + lane * 8);
    const uint2 xa = *reinterpret_cast<const uint2*>(x + c * 256 + lane * 4);
    k16_dword(w.x, lut, xa.x, xa.y, acc);
    k16_dword(w.y, lut, xa.x, xa.y, acc + 4);
  }
}

// k = 256: strip of col-blocks [c0, c1) of row-block rb; one group per iteration,
// the next group's loads are issued before the current one is consumed.
__device__ __forceinline__ void strip_k256(const GemvProblem& P, int rb, int split, int splits,
                                           int lane, uint32_t* lut, float (&acc)[8]) {
  const int n_cb = P.n_cb;
  const int c0 = (n_cb * split) / splits;
  const int c1 = (n_cb * (split + 1)) / splits;
  if (c0 >= c1) return;
  const uint8_t* idx_rb = P.idx + (size_t)rb * n_cb * 1024;
  const uint32_t* cb_rb = P.cb + (size_t)rb * n_cb * 256;
  const uint16_t* x = P.x;

  uint4 w = *reinterpret_cast<const uint4*>(idx_rb + (size_t)c0 * 1024 + lane * 16);
  uint4 cbv = *reinterpret_cast<const uint4*>(cb_rb + (size_t)c0 * 256 + lane * 4);
  uint2 xv = *reinterpret_cast<const uint2*>(x + c0 * 256 + lane * 4);
  for (int c = c0; c < c1; ++c) {
    uint4 wn = w, cbn = cbv;
    uint2 xn = xv;
    if (c + 1 < c1) {
      wn = *reinterpret_cast<const uint4*>(idx_rb + (size_t)(c + 1) * 1024 + lane * 16);
      cbn = *reinterpret_cast<const uint4*>(cb_rb + (size_t)(c + 1) * 256 + lane * 4);
      xn = *reinterpret_cast<const uint2*>(x + (c + 1) * 256 + lane * 4);
    }
    wave_lds_sync();
    *reinterpret_cast<uint4*>(lut + lane * 4) = cbv;
    wave_lds_sync();
    k256_dword(w.x, lut, xv.x, xv.y, acc);
    k256_dword(w.y, lut, xv.x, xv.y, acc + 2);
    k256_dword(w.z, lut, xv.x, xv.y, acc + 4);
    k256_dword(w.w, lut, xv.x, xv.y, acc + 6);
    w = wn;
    cbv = cbn;
    xv = xn;
  }
}

template <int K>
__global__ __launch_bounds__(256) void gemv_kernel(const GemvBatch batch) {
  __shared__ uint32_t lut_all[4][272];
  __shared__ float part[4][8];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wg = blockIdx.x;

  // which problem does this workgroup belong to (wg_begin is ascending)
  int lo = 0, hi = batch.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (batch.p[mid].wg_begin <= wg) lo = mid; else hi = mid;
  }
  const GemvProblem& P = batch.p[lo];
  const int splits = P.splits;
  const int rb_per_wg = 4 / splits;
  const int wg_local = wg - P.wg_begin;
  const int rb = wg_local * rb_per_wg + wave / splits;
  const int split = wave % splits;

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;

  if (rb < P.n_rb) {
    if (K == 16) strip_k16(P, rb, split, splits, lane, lut_all[wave], acc);
    else strip_k256(P, rb, split, splits, lane, lut_all[wave], acc);
  }

  const float v = wave_reduce8(acc, lane);
  if ((lane & 7) == 0) part[wave][lane >> 3] = v;
  __syncthreads();

  if ((int)threadIdx.x < rb_per_wg * 8) {
    const int rbi = threadIdx.x >> 3, r = threadIdx.x & 7;
    const int rbo = wg_local * rb_per_wg + rbi;
    if (rbo < P.n_rb) {
      float s = 0.f;
      for (int q = 0; q < splits; ++q) s += part[rbi * splits + q][r];
      const size_t o = (size_t)rbo * 8 + r;
      if (batch.y_f32) reinterpret_cast<float*>(P.y)[o] = s;
      else reinterpret_cast<_Float16*>(P.y)[o] = (_Float16)s;
    }
  }
}

}  // namespace

hipError_t launch_gemv(int k, const GemvBatch& batch, hipStream_t s) {
  const dim3 grid(batch.total_wgs), block(256);
  if (k == 16) hipLaunchKernelGGL(gemv_kernel<16>, grid, block, 0, s, batch);
  else hipLaunchKernelGGL(gemv_kernel<256>, grid, block, 0, s, batch);
  return hipGetLastError();
}

}  // namespace vq
