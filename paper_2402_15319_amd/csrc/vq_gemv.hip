// Batch-1 product y = W x on vector-quantised W (Sec. 3.2: decode by table
// lookup, then matrix-vector multiply), fused: packed indices are streamed
// from HBM with 128-bit loads, each group's codebook is staged in LDS, and
// every looked-up fp16 pair goes straight into a fp32-accumulating dot2.
//
// Work decomposition.  A workgroup has 4 waves; a wave owns a "strip": some or
// all col-blocks of one row-block (8 output rows).  A strip is consumed in
// chunks (k=16: 4 col-block pairs = 8 groups; k=256: 2 groups).  A chunk is one
// round of loads: its indices, its codebooks and its activations; two chunk
// buffers ping-pong so that one chunk is always in flight while the other is
// being consumed.  Absent parts of a ragged chunk are zero-filled (zero
// indices into a zeroed table times zero activations add exactly 0), so the
// consume step is branch-free.
//
// Two kernels share this code:
//   * gemv_stream_kernel (splits == 1): a persistent grid; every wave walks a
//     list of whole row-blocks, possibly across several matrices, and the first
//     chunk of its next row-block is already loading while the last chunk of
//     the current one is consumed.
//   * gemv_split_kernel (few row-blocks): one workgroup per `4/splits`
//     row-blocks; `splits` waves share a row-block and their partial sums meet
//     in LDS in a fixed order, so the result is deterministic.
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

// A strip as wave-uniform scalars.
struct Strip {
  const uint8_t* idx_rb;   // indices of the row-block
  const uint32_t* cb_rb;   // codebooks of the row-block (dwords)
  const uint16_t* x;
  int u;                   // next unit to load: col-block pair (k=16) or col-block (k=256)
  int u_end;               // end of the units, counting the odd tail group of k=16 as one
  int u_pairs_end;         // k=16: end of the full pairs of this strip
  int n_pairs;             // k=16: pairs in the whole row-block (locates the tail's bytes)
  int tail_c;              // k=16: col-block of the odd tail group in this strip, or -1
};

template <int K> struct Chunk;

// ---- k = 16 --------------------------------------------------------------
template <> struct Chunk<16> {
  static constexpr int kUnits = 4;       // col-block pairs per chunk
  static constexpr int kLutDwords = 128; // 8 groups x 16 centroids
  uint4 w[4];     // slot s: the lane's 16 index bytes of pair u+s (8 bytes + zeros for the tail)
  uint2 xa[4];    // activations of the first group of the slot
  uint2 xb[4];    // ... and of the second
  uint4 cbv;      // this lane's 16 bytes of the chunk's codebooks (lanes 0..31)

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    const int n_groups = 2 * max(0, min(4, S.u_pairs_end - u)) +
                         ((S.tail_c >= 0 && S.u_pairs_end - u >= 0 && S.u_pairs_end - u < 4) ? 1 : 0);
    cbv = make_uint4(0, 0, 0, 0);
    if (lane * 16 < n_groups * 64)
      cbv = *reinterpret_cast<const uint4*>(S.cb_rb + (size_t)u * 32 + lane * 4);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int q = u + s;
      w[s] = make_uint4(0, 0, 0, 0);
      xa[s] = make_uint2(0, 0);
      xb[s] = make_uint2(0, 0);
      if (q < S.u_pairs_end) {
        w[s] = *reinterpret_cast<const uint4*>(S.idx_rb + (size_t)q * 1024 + lane * 16);
        xa[s] = *reinterpret_cast<const uint2*>(S.x + (2 * q) * 256 + lane * 4);
        xb[s] = *reinterpret_cast<const uint2*>(S.x + (2 * q + 1) * 256 + lane * 4);
      } else if (q == S.u_pairs_end && S.tail_c >= 0) {
        const uint2 t = *reinterpret_cast<const uint2*>(S.idx_rb + (size_t)S.n_pairs * 1024 + lane * 8);
        w[s] = make_uint4(t.x, t.y, 0, 0);
        xa[s] = *reinterpret_cast<const uint2*>(S.x + S.tail_c * 256 + lane * 4);
      }
    }
  }

  // Stages the codebooks in this wave's table region (`lut`, LDS byte address `base`)
  // and consumes the chunk.
  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, int lane,
                                          float (&acc)[8]) const {
    if (lane < 32) *reinterpret_cast<uint4*>(lut + lane * 4) = cbv;
    wave_lds_sync();
    k16_group<0>(w[0].x, w[0].y, base, xa[0].x, xa[0].y, acc);
    k16_group<64>(w[0].z, w[0].w, base, xb[0].x, xb[0].y, acc);
    k16_group<128>(w[1].x, w[1].y, base, xa[1].x, xa[1].y, acc);
    k16_group<192>(w[1].z, w[1].w, base, xb[1].x, xb[1].y, acc);
    k16_group<256>(w[2].x, w[2].y, base, xa[2].x, xa[2].y, acc);
    k16_group<320>(w[2].z, w[2].w, base, xb[2].x, xb[2].y, acc);
    k16_group<384>(w[3].x, w[3].y, base, xa[3].x, xa[3].y, acc);
    k16_group<448>(w[3].z, w[3].w, base, xb[3].x, xb[3].y, acc);
  }
};

// ---- k = 256 -------------------------------------------------------------
template <> struct Chunk<256> {
  static constexpr int kUnits = 2;        // groups per chunk
  static constexpr int kLutDwords = 512;  // 2 groups x 256 centroids
  uint4 w[2];     // the lane's 16 index bytes of group u+s
  uint2 xv[2];    // its activations
  uint4 cbv[2];   // the lane's 16 bytes of the group's codebook

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int c = u + s;
      w[s] = make_uint4(0, 0, 0, 0);
      xv[s] = make_uint2(0, 0);
      cbv[s] = make_uint4(0, 0, 0, 0);
      if (c < S.u_end) {
        w[s] = *reinterpret_cast<const uint4*>(S.idx_rb + (size_t)c * 1024 + lane * 16);
        cbv[s] = *reinterpret_cast<const uint4*>(S.cb_rb + (size_t)c * 256 + lane * 4);
        xv[s] = *reinterpret_cast<const uint2*>(S.x + c * 256 + lane * 4);
      }
    }
  }

  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, int lane,
                                          float (&acc)[8]) const {
    *reinterpret_cast<uint4*>(lut + lane * 4) = cbv[0];
    *reinterpret_cast<uint4*>(lut + 256 + lane * 4) = cbv[1];
    wave_lds_sync();
    k256_group<0>(w[0].x, w[0].y, w[0].z, w[0].w, base, xv[0].x, xv[0].y, acc);
    k256_group<1024>(w[1].x, w[1].y, w[1].z, w[1].w, base, xv[1].x, xv[1].y, acc);
  }
};

// Strip (row-block rb, K-split `split` of `splits`) of problem P.
template <int K>
__device__ __forceinline__ Strip make_strip(const GemvProblem& P, int rb, int split, int splits) {
  Strip S;
  const int n_cb = P.n_cb;
  S.x = P.x;
  if (K == 16) {
    const int n_pairs = n_cb >> 1;
    S.idx_rb = P.idx + (size_t)rb * n_cb * 512;
    S.cb_rb = P.cb + (size_t)rb * n_cb * 16;
    S.u = (n_pairs * split) / splits;
    S.u_pairs_end = (n_pairs * (split + 1)) / splits;
    S.n_pairs = n_pairs;
    S.tail_c = ((n_cb & 1) && split == splits - 1) ? n_cb - 1 : -1;
    S.u_end = S.u_pairs_end + (S.tail_c >= 0 ? 1 : 0);
  } else {
    S.idx_rb = P.idx + (size_t)rb * n_cb * 1024;
    S.cb_rb = P.cb + (size_t)rb * n_cb * 256;
    S.u = (n_cb * split) / splits;
    S.u_end = (n_cb * (split + 1)) / splits;
    S.u_pairs_end = S.u_end;
    S.n_pairs = 0;
    S.tail_c = -1;
  }
  return S;
}

__device__ __forceinline__ void store_rows(void* y, int y_f32, int rb, int lane, float v) {
  // after wave_reduce8 every lane holds the total of row (lane >> 3) & 7
  if ((lane & 7) == 0) {
    const size_t o = (size_t)rb * 8 + (lane >> 3);
    if (y_f32) reinterpret_cast<float*>(y)[o] = v;
    else reinterpret_cast<_Float16*>(y)[o] = (_Float16)v;
  }
}

// Which problem does work item `item` belong to (item_begin is ascending, p[0].item_begin = 0).
__device__ __forceinline__ int find_problem(const GemvBatch& batch, int item) {
  int lo = 0, hi = batch.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (batch.p[mid].wg_begin <= item) lo = mid; else hi = mid;
  }
  return lo;
}

// ---- persistent streaming kernel (one wave per row-block) ------------------
// Work item i of the launch = row-block (i - p.wg_begin) of problem p (here wg_begin
// counts row-blocks).  Wave `gw` of `n_waves` handles items gw, gw + n_waves, ...
template <int K>
struct Cursor {
  Strip S;          // strip being loaded from
  void* y;
  int rb;
  int item;         // current item, or >= total when exhausted
};

template <int K>
__device__ __forceinline__ bool open_item(const GemvBatch& batch, Cursor<K>& C) {
  if (C.item >= batch.total_wgs) return false;
  const int pi = find_problem(batch, C.item);
  const GemvProblem& P = batch.p[pi];
  C.rb = C.item - P.wg_begin;
  C.y = P.y;
  C.S = make_strip<K>(P, C.rb, 0, 1);
  return true;
}

template <int K>
__global__ __launch_bounds__(256) void gemv_stream_kernel(const GemvBatch batch) {
  __shared__ __attribute__((aligned(16))) uint32_t lut_all[4][2 * Chunk<K>::kLutDwords];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_waves = gridDim.x * 4;
  uint32_t* lut_a = lut_all[wave];
  uint32_t* lut_b = lut_a + Chunk<K>::kLutDwords;
  const uint32_t base_a = lds_addr(lut_a), base_b = lds_addr(lut_b);

  // The loader runs one chunk ahead of the consumer; both walk the same item sequence.
  Cursor<K> L;                       // where the next load comes from
  L.item = blockIdx.x * 4 + wave;
  bool l_ok = open_item<K>(batch, L);
  // consumer side: (y, rb, chunks left) of the item being consumed
  void* c_y = L.y;
  int c_rb = L.rb;
  int c_left = l_ok ? (L.S.u_end - L.S.u + Chunk<K>::kUnits - 1) / Chunk<K>::kUnits : 0;

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;

  Chunk<K> A, B;
  // helper semantics (written out twice below for the two buffers):
  //   load next chunk of L into buffer; advance L (to the next item when the strip ends)
#define VQ_LOAD_NEXT(BUF, OK)                                            \
  do {                                                                   \
    OK = l_ok;                                                           \
    if (l_ok) {                                                          \
      BUF.load(L.S, L.S.u, lane);                                        \
      L.S.u += Chunk<K>::kUnits;                                         \
      if (L.S.u >= L.S.u_end) {                                          \
        L.item += n_waves;                                               \
        l_ok = open_item<K>(batch, L);                                   \
      }                                                                  \
    }                                                                    \
  } while (0)
  //   consume a buffer; when it was the last chunk of its item: reduce, store, move on
#define VQ_CONSUME(BUF, LUT, BASE)                                       \
  do {                                                                   \
    BUF.consume(LUT, BASE, lane, acc);                                   \
    if (--c_left == 0) {                                                 \
      const float v = wave_reduce8(acc, lane);                           \
      store_rows(c_y, batch.y_f32, c_rb, lane, v);                       \
      _Pragma("unroll") for (int r = 0; r < 8; ++r) acc[r] = 0.f;        \
      c_item += n_waves;                                                 \
      if (c_item < batch.total_wgs) {                                    \
        const GemvProblem& Pn = batch.p[find_problem(batch, c_item)];    \
        c_rb = c_item - Pn.wg_begin;                                     \
        c_y = Pn.y;                                                      \
        const Strip Sn = make_strip<K>(Pn, c_rb, 0, 1);                  \
        c_left = (Sn.u_end - Sn.u + Chunk<K>::kUnits - 1) / Chunk<K>::kUnits; \
      }                                                                  \
    }                                                                    \
  } while (0)

  int c_item = L.item;
  bool a_ok, b_ok;
  VQ_LOAD_NEXT(A, a_ok);
  while (a_ok) {
    VQ_LOAD_NEXT(B, b_ok);
    VQ_CONSUME(A, lut_a, base_a);
    VQ_LOAD_NEXT(A, a_ok);
    if (!b_ok) break;
    VQ_CONSUME(B, lut_b, base_b);
  }
#undef VQ_LOAD_NEXT
#undef VQ_CONSUME
}

// ---- split-K kernel (few row-blocks) ---------------------------------------
template <int K>
__global__ __launch_bounds__(256) void gemv_split_kernel(const GemvBatch batch) {
  __shared__ __attribute__((aligned(16))) uint32_t lut_all[4][2 * Chunk<K>::kLutDwords];
  __shared__ float part[4][8];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wg = blockIdx.x;
  const GemvProblem& P = batch.p[find_problem(batch, wg)];
  const int splits = P.splits;
  const int rb_per_wg = 4 / splits;
  const int wg_local = wg - P.wg_begin;
  const int rb = wg_local * rb_per_wg + wave / splits;
  const int split = wave % splits;
  uint32_t* lut_a = lut_all[wave];
  uint32_t* lut_b = lut_a + Chunk<K>::kLutDwords;
  const uint32_t base_a = lds_addr(lut_a), base_b = lds_addr(lut_b);

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;

  if (rb < P.n_rb) {
    Strip S = make_strip<K>(P, rb, split, splits);
    if (S.u < S.u_end) {
      constexpr int U = Chunk<K>::kUnits;
      Chunk<K> A, B;
      A.load(S, S.u, lane);
      for (int u = S.u; u < S.u_end; u += 2 * U) {
        if (u + U < S.u_end) B.load(S, u + U, lane);
        A.consume(lut_a, base_a, lane, acc);
        if (u + 2 * U < S.u_end) A.load(S, u + 2 * U, lane);
        if (u + U < S.u_end) B.consume(lut_b, base_b, lane, acc);
      }
    }
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

int gemv_stream_resident_wgs(int k) {
  // Occupancy of the persistent kernel, asked once per device and kernel (a pure function
  // of the code object and the device; caching it keeps the hot path free of runtime queries).
  static int cached[2][16];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) dev = 0;
  int& slot = cached[k == 16 ? 0 : 1][dev];
  if (slot == 0) {
    int per_cu = 0, cus = 0;
    hipError_t e = k == 16
        ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_stream_kernel<16>, 256, 0)
        : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_stream_kernel<256>, 256, 0);
    if (e != hipSuccess || per_cu < 1) per_cu = 2;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
      cus = 256;
    (void)hipGetLastError();
    slot = per_cu * cus;
  }
  return slot;
}

hipError_t launch_gemv(int k, const GemvBatch& batch, int stream_mode, int grid_wgs,
                       hipStream_t s) {
  const dim3 grid(grid_wgs), block(256);
  if (stream_mode) {
    if (k == 16) hipLaunchKernelGGL(gemv_stream_kernel<16>, grid, block, 0, s, batch);
    else hipLaunchKernelGGL(gemv_stream_kernel<256>, grid, block, 0, s, batch);
  } else {
    if (k == 16) hipLaunchKernelGGL(gemv_split_kernel<16>, grid, block, 0, s, batch);
    else hipLaunchKernelGGL(gemv_split_kernel<256>, grid, block, 0, s, batch);
  }
  return hipGetLastError();
}

}  // namespace vq
