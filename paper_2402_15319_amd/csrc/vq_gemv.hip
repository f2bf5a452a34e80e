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

// Looks up the 4 vectors of one dword of 8-bit indices (2 rows x 2 vectors).
__device__ __forceinline__ void k256_dword(uint32_t w, const uint32_t* t, uint32_t x0, uint32_t x1,
                                           float* acc) {
  acc[0] = dot2(t[w & 255u], x0, acc[0]);
  acc[0] = dot2(t[(w >> 8) & 255u], x1, acc[0]);
  acc[1] = dot2(t[(w >> 16) & 255u], x0, acc[1]);
  acc[1] = dot2(t[w >> 24], x1, acc[1]);
}

// ---- k = 16 --------------------------------------------------------------
// A chunk is 4 col-block pairs (8 groups): 4 KB of indices, 512 B of codebooks and
// the matching activations, all fetched with one round of loads.  Two chunks
// (A/B) ping-pong so that one is in flight while the other is consumed.
struct ChunkK16 {
  uint4 w[4];     // slot s: the lane's 16 index bytes of pair p0+s (8 bytes if it is the odd tail)
  uint2 xa[4];    // activations of the first group of the slot
  uint2 xb[4];    // ... and of the second
  uint4 cbv;      // this lane's 16 bytes of the chunk's codebooks (lanes 0..31)
};

struct StripK16 {
  const uint8_t* idx_rb;   // row-block base of the indices, + lane*16 not applied
  const uint32_t* cb_rb;   // row-block base of the codebooks
  const uint16_t* x;
  int p1;                  // end of this strip's pair range
  int tail_c;              // col-block of the odd tail group handled by this strip, or -1
  int n_pairs;             // pairs in the whole row-block (locates the tail's bytes)
};

// A full chunk: 4 pairs, no conditions.
__device__ __forceinline__ void load_chunk_full(ChunkK16& c, const StripK16& S, int p, int lane) {
  c.cbv = make_uint4(0, 0, 0, 0);
  if (lane < 32) c.cbv = *reinterpret_cast<const uint4*>(S.cb_rb + (size_t)p * 32 + lane * 4);
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int q = p + s;
    c.w[s] = *reinterpret_cast<const uint4*>(S.idx_rb + (size_t)q * 1024 + lane * 16);
    c.xa[s] = *reinterpret_cast<const uint2*>(S.x + (2 * q) * 256 + lane * 4);
    c.xb[s] = *reinterpret_cast<const uint2*>(S.x + (2 * q + 1) * 256 + lane * 4);
  }
}

// Stages the chunk's codebooks in this wave's table region `lut` (LDS byte address
// `base`, 128 dwords) and consumes the chunk.
__device__ __forceinline__ void compute_chunk_full(const ChunkK16& c, uint32_t* lut, uint32_t base,
                                                   int lane, float (&acc)[8]) {
  if (lane < 32) *reinterpret_cast<uint4*>(lut + lane * 4) = c.cbv;
  wave_lds_sync();
  k16_group<0>(c.w[0].x, c.w[0].y, base, c.xa[0].x, c.xa[0].y, acc);
  k16_group<64>(c.w[0].z, c.w[0].w, base, c.xb[0].x, c.xb[0].y, acc);
  k16_group<128>(c.w[1].x, c.w[1].y, base, c.xa[1].x, c.xa[1].y, acc);
  k16_group<192>(c.w[1].z, c.w[1].w, base, c.xb[1].x, c.xb[1].y, acc);
  k16_group<256>(c.w[2].x, c.w[2].y, base, c.xa[2].x, c.xa[2].y, acc);
  k16_group<320>(c.w[2].z, c.w[2].w, base, c.xb[2].x, c.xb[2].y, acc);
  k16_group<384>(c.w[3].x, c.w[3].y, base, c.xa[3].x, c.xa[3].y, acc);
  k16_group<448>(c.w[3].z, c.w[3].w, base, c.xb[3].x, c.xb[3].y, acc);
}

// The ragged end of a strip: up to 3 pairs and/or the odd tail group, as 7 group slots
// (pair s -> slots 2s, 2s+1; the tail follows the last pair).  Absent slots get zero
// indices and zero activations, so they add exactly 0; all conditions are wave-uniform.
struct RaggedK16 {
  uint2 w[7];
  uint2 x[7];
  uint4 cbv;
};

__device__ __forceinline__ void load_ragged(RaggedK16& c, const StripK16& S, int p, int lane) {
  const int n_groups = 2 * (S.p1 - p) + (S.tail_c >= 0 ? 1 : 0);   // 1..7
  c.cbv = make_uint4(0, 0, 0, 0);
  if (lane * 16 < n_groups * 64)
    c.cbv = *reinterpret_cast<const uint4*>(S.cb_rb + (size_t)p * 32 + lane * 4);
#pragma unroll
  for (int g = 0; g < 7; ++g) {
    c.w[g] = make_uint2(0, 0);
    c.x[g] = make_uint2(0, 0);
    const int q = p + (g >> 1);
    if (q < S.p1) {
      c.w[g] = *reinterpret_cast<const uint2*>(S.idx_rb + (size_t)q * 1024 + lane * 16 + (g & 1) * 8);
      c.x[g] = *reinterpret_cast<const uint2*>(S.x + (2 * q + (g & 1)) * 256 + lane * 4);
    } else if (g == 2 * (S.p1 - p) && S.tail_c >= 0) {
      c.w[g] = *reinterpret_cast<const uint2*>(S.idx_rb + (size_t)S.n_pairs * 1024 + lane * 8);
      c.x[g] = *reinterpret_cast<const uint2*>(S.x + S.tail_c * 256 + lane * 4);
    }
  }
}

__device__ __forceinline__ void compute_ragged(const RaggedK16& c, int n_groups, uint32_t* lut,
                                               uint32_t base, int lane, float (&acc)[8]) {
  if (lane < 32) *reinterpret_cast<uint4*>(lut + lane * 4) = c.cbv;
  wave_lds_sync();
  k16_group<0>(c.w[0].x, c.w[0].y, base, c.x[0].x, c.x[0].y, acc);
  if (n_groups > 1) k16_group<64>(c.w[1].x, c.w[1].y, base, c.x[1].x, c.x[1].y, acc);
  if (n_groups > 2) k16_group<128>(c.w[2].x, c.w[2].y, base, c.x[2].x, c.x[2].y, acc);
  if (n_groups > 3) {
    k16_group<192>(c.w[3].x, c.w[3].y, base, c.x[3].x, c.x[3].y, acc);
    k16_group<256>(c.w[4].x, c.w[4].y, base, c.x[4].x, c.x[4].y, acc);
    k16_group<320>(c.w[5].x, c.w[5].y, base, c.x[5].x, c.x[5].y, acc);
    k16_group<384>(c.w[6].x, c.w[6].y, base, c.x[6].x, c.x[6].y, acc);
  }
}

// k = 16: pairs [p0, p1) (+ the odd tail group for the last split) of row-block rb.
// `lut` points at this wave's two 512-byte table regions.  The ragged end (if any) is
// done first, while the first full chunk is already in flight.
__device__ __forceinline__ void strip_k16(const GemvProblem& P, int rb, int split, int splits,
                                          int lane, uint32_t* lut, float (&acc)[8]) {
  const int n_cb = P.n_cb;
  const int n_pairs = n_cb >> 1;
  const int p0 = (n_pairs * split) / splits;
  StripK16 S;
  S.idx_rb = P.idx + (size_t)rb * n_cb * 512;
  S.cb_rb = P.cb + (size_t)rb * n_cb * 16;
  S.x = P.x;
  S.p1 = (n_pairs * (split + 1)) / splits;
  S.tail_c = ((n_cb & 1) && split == splits - 1) ? n_cb - 1 : -1;
  S.n_pairs = n_pairs;
  const int n_full = (S.p1 - p0) >> 2;              // full chunks
  const int p_rag = p0 + 4 * n_full;                // first pair of the ragged end
  const int rag_groups = 2 * (S.p1 - p_rag) + (S.tail_c >= 0 ? 1 : 0);
  const uint32_t base_a = lds_addr(lut), base_b = base_a + 512;

  ChunkK16 A, B;
  if (rag_groups > 0) {
    RaggedK16 R;
    load_ragged(R, S, p_rag, lane);
    if (n_full > 0) load_chunk_full(A, S, p0, lane);
    compute_ragged(R, rag_groups, lut + 128, base_b, lane, acc);
  } else if (n_full > 0) {
    load_chunk_full(A, S, p0, lane);
  }
  for (int t = 0; t < n_full; t += 2) {
    const int p = p0 + 4 * t;
    if (t + 1 < n_full) load_chunk_full(B, S, p + 4, lane);
    compute_chunk_full(A, lut, base_a, lane, acc);
    if (t + 2 < n_full) load_chunk_full(A, S, p + 8, lane);
    if (t + 1 < n_full) compute_chunk_full(B, lut + 128, base_b, lane, acc);
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
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform
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
