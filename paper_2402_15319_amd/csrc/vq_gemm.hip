// Batched / prefill product Y[out,B] = W X[in,B] on vector-quantised W: the one
// place on this path that is a dense contraction.  Each workgroup decodes tiles
// of W (table lookup, Sec. 3.2) into LDS as fp16 and feeds them to the fp16
// matrix cores with fp32 accumulation.
//
// Tile: 32 rows (4 row-blocks, one per wave to decode) x 128 batch columns
// (one 32x32 MFMA accumulator per wave), K walked one col-block (256) at a time
// in four 64-deep sub-steps.  X is batch-contiguous, while the MFMA operands
// want 4 consecutive k per lane, so X is interleaved in registers on its way to
// LDS as Xs[k/4][n][k%4].
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

constexpr int MT = 32;    // rows per workgroup
constexpr int NT = 128;   // batch columns per workgroup
constexpr int WS = 264;   // LDS row stride of the decoded W tile, in halfs (256 + 8 pad)
constexpr int KS = 64;    // k per sub-step

template <int K>
__global__ __launch_bounds__(256) void gemm_kernel(const uint8_t* __restrict__ idx,
                                                   const uint32_t* __restrict__ cb,
                                                   const uint16_t* __restrict__ X, int B, int ldx,
                                                   void* __restrict__ Y, int ldy, int y_f32,
                                                   int n_rb, int n_cb, int n_tiles_n) {
  __shared__ __attribute__((aligned(16))) uint16_t Wt[MT * WS];
  __shared__ __attribute__((aligned(16))) uint32_t Xs[(KS / 4) * NT * 2];
  __shared__ __attribute__((aligned(16))) uint32_t lut_all[4][K];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int mt = blockIdx.x / n_tiles_n;
  const int nt = blockIdx.x - mt * n_tiles_n;
  uint32_t* lut = lut_all[wave];

  const int rb = mt * 4 + wave;          // the row-block this wave decodes
  const bool rb_ok = rb < n_rb;
  uint16_t* wrow = Wt + (wave * 8) * WS + lane * 4;

  // X staging role of this thread: k-quad kq (4 rows of X), 8 batch columns from n0
  const int kq = tid >> 4;
  const int n0 = nt * NT + (tid & 15) * 8;
  const bool n_ok = n0 < B;

  f16v_t acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  for (int c = 0; c < n_cb; ++c) {
    __syncthreads();   // all MFMA reads of Wt / Xs from the previous col-block are done
    // ---- decode this wave's group (rb, c) into Wt rows [8*wave, 8*wave+8)
    if (rb_ok) {
      const long long g = (long long)rb * n_cb + c;
      if (K == 16) {
        const int slots = 2 * k16_pairs(n_cb);
        if (lane < 16) lut[lane] = cb[((size_t)rb * slots + c) * 16 + lane];
        const uint2 w = *reinterpret_cast<const uint2*>(idx + (size_t)rb * slots * 512 +
                                                        k16_chunk_offset(c, lane));
        wave_lds_sync();
        const char* lutb = reinterpret_cast<const char*>(lut);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          uint32_t a, b;
          k16_split_dword(h ? w.y : w.x, a, b);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const uint32_t lo = *reinterpret_cast<const uint32_t*>(lutb + ((a >> (8 * r)) & 0xffu));
            const uint32_t hi = *reinterpret_cast<const uint32_t*>(lutb + ((b >> (8 * r)) & 0xffu));
            *reinterpret_cast<uint2*>(wrow + (4 * h + r) * WS) = make_uint2(lo, hi);
          }
        }
      } else {
        *reinterpret_cast<uint4*>(lut + lane * 4) =
            *reinterpret_cast<const uint4*>(cb + g * 256 + lane * 4);
        const uint4 w = *reinterpret_cast<const uint4*>(idx + g * 1024 + lane * 16);
        wave_lds_sync();
        const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const uint32_t half = ws[r >> 1] >> (16 * (r & 1));
          *reinterpret_cast<uint2*>(wrow + r * WS) =
              make_uint2(lut[half & 255u], lut[(half >> 8) & 255u]);
        }
      }
    } else {
#pragma unroll
      for (int r = 0; r < 8; ++r) *reinterpret_cast<uint2*>(wrow + r * WS) = make_uint2(0u, 0u);
    }

    for (int sub = 0; sub < 256 / KS; ++sub) {
      if (sub) __syncthreads();   // MFMA reads of Xs from the previous sub-step are done
      // ---- stage X rows [k0, k0+4) x columns [n0, n0+8), interleaved to [n][k%4]
      {
        uint4 r0 = make_uint4(0, 0, 0, 0), r1 = r0, r2 = r0, r3 = r0;
        if (n_ok) {
          const uint16_t* src = X + (size_t)(c * 256 + sub * KS + kq * 4) * ldx + n0;
          r0 = *reinterpret_cast<const uint4*>(src);
          r1 = *reinterpret_cast<const uint4*>(src + ldx);
          r2 = *reinterpret_cast<const uint4*>(src + 2 * (size_t)ldx);
          r3 = *reinterpret_cast<const uint4*>(src + 3 * (size_t)ldx);
        }
        const uint32_t a0[4] = {r0.x, r0.y, r0.z, r0.w}, a1[4] = {r1.x, r1.y, r1.z, r1.w};
        const uint32_t a2[4] = {r2.x, r2.y, r2.z, r2.w}, a3[4] = {r3.x, r3.y, r3.z, r3.w};
        uint32_t* dst = Xs + (kq * NT + (tid & 15) * 8) * 2;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint4 o;
          o.x = (a0[q] & 0xffffu) | (a1[q] << 16);          // n = 2q   : k+0, k+1
          o.y = (a2[q] & 0xffffu) | (a3[q] << 16);          //            k+2, k+3
          o.z = (a0[q] >> 16) | (a1[q] & 0xffff0000u);      // n = 2q+1
          o.w = (a2[q] >> 16) | (a3[q] & 0xffff0000u);
          *reinterpret_cast<uint4*>(dst + q * 4) = o;
        }
      }
      __syncthreads();
      // ---- 8 MFMAs of depth 8: A = decoded W (row lane%32), B = X (column lane%32)
#pragma unroll
      for (int mf = 0; mf < KS / 8; ++mf) {
        const h4_t a = *reinterpret_cast<const h4_t*>(Wt + (lane & 31) * WS + sub * KS + mf * 8 +
                                                      4 * (lane >> 5));
        const h4_t b = *reinterpret_cast<const h4_t*>(
            Xs + ((mf * 2 + (lane >> 5)) * NT + wave * 32 + (lane & 31)) * 2);
        acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, acc, 0, 0, 0);
      }
    }
  }

  // ---- store: accumulator register i holds row 8*(i/4) + 4*(lane/32) + i%4, column lane%32
  const int n = nt * NT + wave * 32 + (lane & 31);
  if (n < B) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = mt * MT + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
      if (row < n_rb * 8) {
        const size_t o = (size_t)row * ldy + n;
        if (y_f32) reinterpret_cast<float*>(Y)[o] = acc[i];
        else reinterpret_cast<_Float16*>(Y)[o] = (_Float16)acc[i];
      }
    }
  }
}

}  // namespace

hipError_t launch_gemm(const vq_desc& d, const void* idx_dev, const void* cb_dev, const void* X,
                       int B, int ldx, void* Y, int ldy, int y_f32, hipStream_t s) {
  const int n_rb = d.out_features / kGroupRows, n_cb = d.in_features / kGroupCols;
  const int tiles_m = (n_rb + 3) / 4, tiles_n = (B + NT - 1) / NT;
  const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
  if (d.k == 16)
    hipLaunchKernelGGL(gemm_kernel<16>, grid, block, 0, s, (const uint8_t*)idx_dev,
                       (const uint32_t*)cb_dev, (const uint16_t*)X, B, ldx, Y, ldy, y_f32, n_rb,
                       n_cb, tiles_n);
  else
    hipLaunchKernelGGL(gemm_kernel<256>, grid, block, 0, s, (const uint8_t*)idx_dev,
                       (const uint32_t*)cb_dev, (const uint16_t*)X, B, ldx, Y, ldy, y_f32, n_rb,
                       n_cb, tiles_n);
  return hipGetLastError();
}

}  // namespace vq
