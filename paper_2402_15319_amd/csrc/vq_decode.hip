// Dense reconstruction W[out,in] (fp16, row-major) from the device layout:
// the decode step of Sec. 3.2 on its own, W[r, c+t] = cb[g][I_g[v]][t], a pure
// copy of 16-bit patterns.  One wave per group; a row of a group is written as
// one contiguous 512-byte segment.
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

// K: 16 or 256 with fp16 codebooks, kFmtK16I8 for k = 16 with int8 tables and a scale per group
// (32 bytes per group slot, then one fp16 scale per slot behind all the tables), kFmtD1K16 for
// scalar codebooks (16 fp16 values per group; a byte of indices looks up a pair of them), kFmtD1K4
// for 2-bit scalar codebooks with one table per row (a nibble of indices looks up a pair).
template <int K>
__global__ __launch_bounds__(256) void decode_kernel(const uint8_t* __restrict__ idx,
                                                     const uint32_t* __restrict__ cb,
                                                     uint16_t* __restrict__ W, int n_cb,
                                                     long long n_groups, int in_features, int rpc) {
  // (k = 16 with blockwise normalisation: 16 table entries, then the group's 16 levels)
  __shared__ uint32_t lut_all[4][K == kFmtK16I8 ? 16 : (K == kFmtK16BN || K == kFmtK16I8H || K == kFmtK32) ? 32 : (K == kFmtD1K16 || K == kFmtK256I8) ? 256 : K == kFmtK256I8BN ? 272 : K == kFmtD1K4 ? 128 : K];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint32_t* lut = lut_all[wave];
  const long long g = (long long)blockIdx.x * 4 + wave;
  if (g >= n_groups) return;   // whole waves leave; no workgroup barrier below
  const long long rb = g / n_cb;
  const int c = (int)(g - rb * n_cb);
  uint16_t* out = W + (size_t)rb * 8 * in_features + (size_t)c * 256 + lane * 4;

  if (K == kFmtD1K4) {   // a 16-entry pair table per row: lane L builds entries 2*(L&7), +1 of row L >> 3
    const int slots = 2 * k16_pairs(n_cb);
    const uint8_t* rec = reinterpret_cast<const uint8_t*>(cb) + (size_t)(rb * slots + c) * kD1K4SlotTabBytes;
    const uint32_t q4 = *reinterpret_cast<const uint32_t*>(rec + (lane >> 3) * 4);
    const _Float16 scale = __builtin_bit_cast(
        _Float16, *reinterpret_cast<const uint16_t*>(rec + kD1K4ScaleOffset + (lane >> 3) * 2));
    const int j = 2 * (lane & 7);
    *reinterpret_cast<uint2*>(lut + 2 * lane) =
        make_uint2(k64_dequant_pair(d1k4_pair(q4, j), scale), k64_dequant_pair(d1k4_pair(q4, j + 1), scale));
    const uint2 w = *reinterpret_cast<const uint2*>(idx + rb * slots * 512 + k16_chunk_offset(c, lane));
    wave_lds_sync();
    const char* lutb = reinterpret_cast<const char*>(lut);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t a, b;
      k16_split_dword(h ? w.y : w.x, a, b);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const char* row_tab = lutb + (4 * h + r) * 64;
        const uint32_t lo = *reinterpret_cast<const uint32_t*>(row_tab + ((a >> (8 * r)) & 0xffu));
        const uint32_t hi = *reinterpret_cast<const uint32_t*>(row_tab + ((b >> (8 * r)) & 0xffu));
        *reinterpret_cast<uint2*>(out + (size_t)(4 * h + r) * in_features) = make_uint2(lo, hi);
      }
    }
  } else if (K == 16 || K == kFmtK16I8 || K == kFmtK16BN || K == kFmtK16I8H || K == kFmtK32) {
    const int slots = 2 * k16_pairs(n_cb);                  // group slots per row-block
    uint32_t cw = 0;                                        // BN: the lane's block codes, row r in bits [4r, 4r+4)
    uint32_t plane = 0;                                     // k = 32: the lane's fifth bits of the pair
    if (K == 16) {
      if (lane < 16) lut[lane] = cb[(rb * slots + c) * 16 + lane];
    } else if (K == kFmtK32) {      // a 32-entry table per group; fifth bits behind the nibbles of the whole matrix
      const long long n_rb = n_groups / n_cb;
      const uint8_t* tb = reinterpret_cast<const uint8_t*>(cb);
      if (lane < 32) {
        const uint16_t* sc = reinterpret_cast<const uint16_t*>(tb + (size_t)n_rb * slots * 64);
        lut[lane] = k64_dequant_pair(*reinterpret_cast<const uint16_t*>(tb + (size_t)(rb * slots + c) * 64 + lane * 2),
                                     __builtin_bit_cast(_Float16, sc[rb * slots + c]));
      }
      plane = reinterpret_cast<const uint32_t*>(idx + (size_t)n_rb * slots * 512)[(rb * (slots / 2) + (c >> 1)) * 64 + lane];
    } else if (K == kFmtK16I8H) {   // groups of 4 rows: the table of rows 0..3, then that of rows 4..7
      const long long n_rb = n_groups / n_cb;
      const uint8_t* tb = reinterpret_cast<const uint8_t*>(cb);
      if (lane < 32) {
        const uint16_t* sc = reinterpret_cast<const uint16_t*>(tb + (size_t)n_rb * slots * 64);
        lut[lane] = k64_dequant_pair(*reinterpret_cast<const uint16_t*>(tb + (size_t)(rb * slots + c) * 64 + lane * 2),
                                     __builtin_bit_cast(_Float16, sc[(rb * slots + c) * 2 + (lane >> 4)]));
      }
    } else {
      const long long n_rb = n_groups / n_cb;
      const uint8_t* tb = reinterpret_cast<const uint8_t*>(cb);
      if (lane < 16) {
        const uint8_t* tq = tb + (size_t)(rb * slots + c) * 32;
        const uint16_t* sc = reinterpret_cast<const uint16_t*>(tb + (size_t)n_rb * slots * 32);
        lut[lane] = k64_dequant_pair(*reinterpret_cast<const uint16_t*>(tq + lane * 2),
                                     __builtin_bit_cast(_Float16, sc[rb * slots + c]));
      }
      if (K == kFmtK16BN) {
        const size_t n_slots = (size_t)n_rb * slots;
        if (lane < 16)
          lut[16 + lane] = 0x10001u * reinterpret_cast<const uint16_t*>(tb + k16bn_level_offset(n_slots))[(rb * slots + c) * 16 + lane];
        cw = reinterpret_cast<const uint32_t*>(tb + k16bn_code_offset(n_slots))[((rb * slots + c) >> 1) * 16 + 2 * (lane >> 3) + (c & 1)];
      }
    }
    const uint2 w = *reinterpret_cast<const uint2*>(idx + rb * slots * 512 + k16_chunk_offset(c, lane));
    wave_lds_sync();
    const char* lutb = reinterpret_cast<const char*>(lut);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t a, b;
      k16_split_dword(h ? w.y : w.x, a, b);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const char* lut_h = lutb + (K == kFmtK16I8H ? 64 * h : 0);
        uint32_t lo = *reinterpret_cast<const uint32_t*>(lut_h + ((a >> (8 * r)) & 0xffu) +
                                                         (K == kFmtK32 ? 64 * k32_plane_bit(plane, c & 1, 4 * h + r, 0) : 0));
        uint32_t hi = *reinterpret_cast<const uint32_t*>(lut_h + ((b >> (8 * r)) & 0xffu) +
                                                         (K == kFmtK32 ? 64 * k32_plane_bit(plane, c & 1, 4 * h + r, 1) : 0));
        if (K == kFmtK16BN) {   // times the scale of the row's 32-weight block: one more fp16 rounding
          const h2_t sc = __builtin_bit_cast(h2_t, lut[16 + ((cw >> (4 * (4 * h + r))) & 15u)]);
          lo = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, lo) * sc);
          hi = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, hi) * sc);
        }
        *reinterpret_cast<uint2*>(out + (size_t)(4 * h + r) * in_features) = make_uint2(lo, hi);
      }
    }
  } else {
    uint32_t cw = 0;         // block-normalised: the lane's block codes, row r in bits [4r, 4r+4)
    if (K == kFmtK256I8 || K == kFmtK256I8BN) {   // int8 table of group (rb / rpc, c): lane L dequantises entries 4L .. 4L+3
      const uint8_t* tab = reinterpret_cast<const uint8_t*>(cb);
      const long long gt = (rb / rpc) * n_cb + c, n_tabs = (n_groups / n_cb / rpc) * n_cb;
      if (K == kFmtK256I8BN) {
        if (lane < 16)
          lut[256 + lane] = 0x10001u * reinterpret_cast<const uint16_t*>(tab + wide_bn_level_offset((size_t)n_tabs, 512))[gt * 16 + lane];
        cw = reinterpret_cast<const uint32_t*>(tab + wide_bn_code_offset((size_t)n_tabs, 512))
                 [(rb * k16_pairs(n_cb) + (c >> 1)) * 16 + 2 * (lane >> 3) + (c & 1)];
      }
      const uint2 q = *reinterpret_cast<const uint2*>(tab + gt * 512 + lane * 8);
      const _Float16 scale = __builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(tab + n_tabs * 512)[gt]);
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(q.x, scale), k64_dequant_pair(q.x >> 16, scale),
                     k64_dequant_pair(q.y, scale), k64_dequant_pair(q.y >> 16, scale));
    } else if (K == kFmtD1K16) {
      const uint8_t* cg = reinterpret_cast<const uint8_t*>(cb) + g * 32;
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          d1_pair_entries(*reinterpret_cast<const uint2*>(cg + (lane & 3) * 8),
                          *reinterpret_cast<const uint16_t*>(cg + (lane >> 2) * 2));
    } else {
      *reinterpret_cast<uint4*>(lut + lane * 4) = *reinterpret_cast<const uint4*>(cb + g * 256 + lane * 4);
    }
    const uint4 w = *reinterpret_cast<const uint4*>(idx + g * 1024 + lane * 16);
    wave_lds_sync();
    const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t half = ws[r >> 1] >> (16 * (r & 1));
      uint32_t lo = lut[half & 255u], hi = lut[(half >> 8) & 255u];
      if (K == kFmtK256I8BN) {   // times the scale of the row's 32-weight block: one more fp16 rounding
        const uint32_t sc = lut[256 + ((cw >> (4 * r)) & 15u)];
        lo = scale_pair(lo, sc);
        hi = scale_pair(hi, sc);
      }
      *reinterpret_cast<uint2*>(out + (size_t)r * in_features) = make_uint2(lo, hi);
    }
  }
}

// k = 64 (6-bit indices, int8 tables with a scale): one wave per (8-row block, col-block).
// Lane L dequantises table entry L (fp16(scale * q), one rounding) and then copies.  BN: every
// copied pair is first multiplied by the scale of its 32-weight block (one more fp16 rounding).
// MODE 0: k = 64; 1: with blockwise normalisation (BN); 2: d = 1, k = 8 (entry L of the pair table is
// built from the group's 8 int8 values); 3: d = 1, k = 8 with blockwise normalisation.
template <int MODE>
__global__ __launch_bounds__(256) void decode64_kernel(const uint8_t* __restrict__ idx,
                                                       const uint8_t* __restrict__ tab,
                                                       uint16_t* __restrict__ W, int n_cb,
                                                       long long n_items, int in_features, int rpc) {
  constexpr bool BN = MODE == 1 || MODE == 3, D1 = MODE >= 2;
  constexpr int tab_bytes = D1 ? (BN ? kD1K8NQuadTabBytes : kD1K8QuadTabBytes) : BN ? kK64NQuadTabBytes : kK64QuadTabBytes;
  constexpr int level_offset = D1 ? kD1K8NLevelOffset : kK64NLevelOffset;
  __shared__ uint32_t lut_all[4][BN ? 80 : 64];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint32_t* lut = lut_all[wave];
  const long long item = (long long)blockIdx.x * 4 + wave;
  if (item >= n_items) return;   // whole waves leave; no workgroup barrier below
  const long long rb8 = item / n_cb;
  const int c = (int)(item - rb8 * n_cb);
  const int n_quads = k64_quads(n_cb), q = c >> 2, j = c & 3;
  const uint8_t* tq = tab + (size_t)((rb8 / rpc) * n_quads + q) * tab_bytes;
  uint32_t cw = 0;
  if (BN) {
    const long long n_rb8 = n_items / n_cb;
    if (lane < 16) lut[64 + lane] = *reinterpret_cast<const uint16_t*>(tq + level_offset + j * 32 + lane * 2) * 0x10001u;
    cw = *reinterpret_cast<const uint32_t*>(tab + (size_t)(n_rb8 / rpc) * n_quads * tab_bytes +
                                            (size_t)(rb8 * n_quads + q) * kK64NQuadCodeBytes + (lane >> 3) * 16 + j * 4);
  }
  const uint32_t two = D1 ? d1k8_pair(*reinterpret_cast<const uint2*>(tq + j * 8), lane)
                          : (uint32_t)*reinterpret_cast<const uint16_t*>(tq + j * 128 + lane * 2);
  const _Float16 scale = __builtin_bit_cast(
      _Float16, *reinterpret_cast<const uint16_t*>(tq + (D1 ? kD1K8ScaleOffset : 512) + 2 * j));
  lut[lane] = k64_dequant_pair(two, scale);
  const uint8_t* iq = idx + (size_t)(rb8 * n_quads + q) * kK64QuadIdxBytes + lane * 16;
  uint32_t d[12];
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    const uint4 v = *reinterpret_cast<const uint4*>(iq + p * 1024);
    d[4 * p] = v.x; d[4 * p + 1] = v.y; d[4 * p + 2] = v.z; d[4 * p + 3] = v.w;
  }
  uint32_t d0 = 0, d1 = 0, d2 = 0;
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
    if (jj == j) { d0 = d[3 * jj]; d1 = d[3 * jj + 1]; d2 = d[3 * jj + 2]; }
  wave_lds_sync();
  const unsigned long long lo = d0 | ((unsigned long long)d1 << 32);
  uint16_t* out = W + (size_t)rb8 * 8 * in_features + (size_t)c * 256 + lane * 4;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    uint32_t id[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int pos = 6 * (2 * r + e);
      unsigned long long v = pos < 64 ? lo >> pos : (unsigned long long)(d2 >> (pos - 64));
      if (pos < 64 && pos > 58) v |= (unsigned long long)d2 << (64 - pos);
      id[e] = (uint32_t)v & 63u;
    }
    uint32_t p0 = lut[id[0]], p1 = lut[id[1]];
    if (BN) {
      const h2_t sc = __builtin_bit_cast(h2_t, lut[64 + ((cw >> (4 * r)) & 15u)]);
      p0 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, p0) * sc);
      p1 = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, p1) * sc);
    }
    *reinterpret_cast<uint2*>(out + (size_t)r * in_features) = make_uint2(p0, p1);
  }
}

// d = 4 (k = 256, int8 tables with a scale): one wave per (8-row block, col-block).  Lane L
// dequantises table entries 4L .. 4L+3 into the wave's 2 KB table, then copies one 8-byte entry
// per row (its vector: columns 4L .. 4L+3).
// MODE 1 (F16): fp16 tables (2 KB per group) instead of int8 tables with a scale; MODE 2 (BN):
// int8 tables with blockwise normalisation (every copied vector times the scale of its block).
template <int MODE>
__global__ __launch_bounds__(256) void decode_d4_kernel(const uint8_t* __restrict__ idx,
                                                        const uint8_t* __restrict__ tab,
                                                        uint16_t* __restrict__ W, int n_cb,
                                                        long long n_items, int in_features, int rpc) {
  constexpr bool F16 = MODE == 1, BN = MODE == 2;
  __shared__ __attribute__((aligned(16))) uint2 lut_all[4][256];
  __shared__ uint32_t lev_all[4][16];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  uint2* lut = lut_all[wave];
  uint32_t* lev = lev_all[wave];
  const long long item = (long long)blockIdx.x * 4 + wave;
  if (item >= n_items) return;   // whole waves leave; no workgroup barrier below
  const long long rb8 = item / n_cb;
  const int c = (int)(item - rb8 * n_cb);
  const long long n_groups = (n_items / n_cb / rpc) * n_cb;
  const long long g = (rb8 / rpc) * n_cb + c;
  if constexpr (F16) {
    const uint4* src = reinterpret_cast<const uint4*>(tab + g * 2048 + lane * 32);
    *reinterpret_cast<uint4*>(lut + 4 * lane) = src[0];
    *reinterpret_cast<uint4*>(lut + 4 * lane + 2) = src[1];
  } else {
    const uint4 q = *reinterpret_cast<const uint4*>(tab + g * 1024 + lane * 16);
    const _Float16 scale = __builtin_bit_cast(_Float16, reinterpret_cast<const uint16_t*>(tab + n_groups * 1024)[g]);
    lut[4 * lane] = d4_dequant_entry(q.x, scale);
    lut[4 * lane + 1] = d4_dequant_entry(q.y, scale);
    lut[4 * lane + 2] = d4_dequant_entry(q.z, scale);
    lut[4 * lane + 3] = d4_dequant_entry(q.w, scale);
  }
  const int n_pairs = (n_cb + 1) >> 1;
  uint32_t cw = 0;
  if constexpr (BN) {
    if (lane < 16)
      lev[lane] = 0x10001u * reinterpret_cast<const uint16_t*>(tab + wide_bn_level_offset((size_t)n_groups, 1024))[g * 16 + lane];
    cw = reinterpret_cast<const uint32_t*>(tab + wide_bn_code_offset((size_t)n_groups, 1024))
             [(rb8 * n_pairs + (c >> 1)) * 16 + 2 * (lane >> 3) + (c & 1)];
  }
  const uint2 w = *reinterpret_cast<const uint2*>(idx + (size_t)(rb8 * n_pairs + (c >> 1)) * 1024 + lane * 16 + (c & 1) * 8);
  wave_lds_sync();
  uint16_t* out = W + (size_t)rb8 * 8 * in_features + (size_t)c * 256 + lane * 4;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const uint32_t j = ((r < 4 ? w.x : w.y) >> (8 * (r & 3))) & 0xffu;
    uint2 t = lut[j];
    if constexpr (BN) {
      const uint32_t sc = lev[(cw >> (4 * r)) & 15u];
      t = make_uint2(scale_pair(t.x, sc), scale_pair(t.y, sc));
    }
    *reinterpret_cast<uint2*>(out + (size_t)r * in_features) = t;
  }
}

}  // namespace

hipError_t launch_decode(const vq_desc& d, const void* idx_dev, const void* cb_dev, void* W,
                         hipStream_t s) {
  const int n_cb = d.in_features / kGroupCols;
  const long long n_groups = (long long)(d.out_features / kGroupRows) * n_cb;   // 8-row items
  const unsigned grid = (unsigned)((n_groups + 3) / 4);
  const int fmt = format_tag(d);
  if (fmt == kFmtD4 || fmt == kFmtD4F16 || fmt == kFmtD4BN) {
#define VQ_DECODE_D4(MODE)                                                                            \
    hipLaunchKernelGGL(decode_d4_kernel<MODE>, dim3(grid), dim3(256), 0, s, (const uint8_t*)idx_dev, \
                       (const uint8_t*)cb_dev, (uint16_t*)W, n_cb, n_groups, d.in_features,          \
                       d.group_rows / kGroupRows)
    if (fmt == kFmtD4) VQ_DECODE_D4(0);
    else if (fmt == kFmtD4F16) VQ_DECODE_D4(1);
    else VQ_DECODE_D4(2);
#undef VQ_DECODE_D4
    return hipGetLastError();
  }
  if (fmt == 64 || fmt == kFmtK64BN || fmt == kFmtD1K8 || fmt == kFmtD1K8BN) {
#define VQ_DECODE64(MODE)                                                                            \
    hipLaunchKernelGGL(decode64_kernel<MODE>, dim3(grid), dim3(256), 0, s, (const uint8_t*)idx_dev, \
                       (const uint8_t*)cb_dev, (uint16_t*)W, n_cb, n_groups, d.in_features,         \
                       d.group_rows / kGroupRows)
    if (fmt == 64) VQ_DECODE64(0);
    else if (fmt == kFmtK64BN) VQ_DECODE64(1);
    else if (fmt == kFmtD1K8BN) VQ_DECODE64(3);
    else VQ_DECODE64(2);
#undef VQ_DECODE64
    return hipGetLastError();
  }
#define VQ_DECODE(K)                                                                                \
  hipLaunchKernelGGL(decode_kernel<K>, dim3(grid), dim3(256), 0, s, (const uint8_t*)idx_dev,       \
                     (const uint32_t*)cb_dev, (uint16_t*)W, n_cb, n_groups, d.in_features,          \
                     d.group_rows >= kGroupRows ? d.group_rows / kGroupRows : 1)
  if (fmt == kFmtK16I8) VQ_DECODE(kFmtK16I8);
  else if (fmt == kFmtK16I8H) VQ_DECODE(kFmtK16I8H);
  else if (fmt == kFmtK32) VQ_DECODE(kFmtK32);
  else if (fmt == kFmtK16BN) VQ_DECODE(kFmtK16BN);
  else if (fmt == kFmtD1K16) VQ_DECODE(kFmtD1K16);
  else if (fmt == kFmtD1K4) VQ_DECODE(kFmtD1K4);
  else if (fmt == kFmtK256I8) VQ_DECODE(kFmtK256I8);
  else if (fmt == kFmtK256I8BN) VQ_DECODE(kFmtK256I8BN);
  else if (fmt == 16) VQ_DECODE(16);
  else VQ_DECODE(256);
#undef VQ_DECODE
  return hipGetLastError();
}

}  // namespace vq
