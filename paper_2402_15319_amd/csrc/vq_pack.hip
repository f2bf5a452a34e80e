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
// row_groups = 1: the canonical groups are single rows (1 x 256, 64 bytes each, row-major), as in
// the scalar 2-bit format, instead of 8 x 256 blocks; row_groups = 4: groups of 4 rows (256 bytes
// each), two per block.
template <int K>
__global__ __launch_bounds__(256) void pack_idx_kernel(const uint8_t* __restrict__ canon,
                                                       uint8_t* __restrict__ dev, int n_cb,
                                                       long long n_slots, int row_groups, int rpc) {
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
      // canonical byte r*64 + lane of the block, or byte `lane` of the group of row rb*8 + r
      const uint8_t* src = row_groups == 1 ? canon + (rb * 8 * n_cb + c) * 64 + lane
                           : row_groups == 4 ? canon + (rb * 2 * n_cb + c) * 256 + lane
                                             : canon + (rb * n_cb + c) * 512 + lane;
      const size_t row_stride = row_groups == 1 ? (size_t)n_cb * 64 : 64;
      const size_t half_skip = row_groups == 4 ? (size_t)(n_cb - 1) * 256 : 0;   // rows 4..7: the group below
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        uint32_t lo[4], hi[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const uint32_t byte = src[(4 * h + b) * row_stride + h * half_skip];
          lo[b] = byte & 15u;
          hi[b] = byte >> 4;
        }
        words[h] = k16_encode_dword(lo, hi);
      }
    }
    uint8_t* dst = dev + rb * slots_per_rb * 512 + k16_chunk_offset(c, lane);
    *reinterpret_cast<uint2*>(dst) = make_uint2(words[0], words[1]);
  } else {
    // slot = (8-row block rb, col-block c); its 1 KB sits in canonical group (rb / rpc, c) of
    // rpc 8-row blocks (rpc = 1: the group itself)
    const long long g = slot;
    const long long rb = slot / n_cb;
    const int c = (int)(slot - rb * n_cb);
    const long long grow = rb / rpc;
    const int sub = (int)(rb - grow * rpc);
    const uint8_t* src = canon + ((grow * n_cb + c) * rpc + sub) * 1024 + 2 * lane;
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
// zero codebook for the pad group.  One thread per 16 bytes of the device array; a codebook
// is `per_group` such pieces and a row-block has `slots_per_rb` group slots.
__global__ __launch_bounds__(256) void pack_cb_kernel(const uint4* __restrict__ src,
                                                      uint4* __restrict__ dst, int per_group,
                                                      int slots_per_rb, int n_cb, long long n16) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n16) return;
  const long long slot = t / per_group;
  const int piece = (int)(t - slot * per_group);
  const long long rb = slot / slots_per_rb;
  const int c = (int)(slot - rb * slots_per_rb);
  dst[t] = c < n_cb ? src[(rb * n_cb + c) * per_group + piece] : make_uint4(0, 0, 0, 0);
}

// k = 16 with int8 tables: 32 bytes per group slot (zero for the pad group), then one fp16
// scale per slot.  One thread per dword of tables; the first n_slots threads also copy a scale.
__global__ __launch_bounds__(256) void pack_tab16_kernel(const uint32_t* __restrict__ q_canon,
                                                         const uint16_t* __restrict__ scale_canon,
                                                         uint32_t* __restrict__ dev, int n_cb,
                                                         long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_slots * 8) return;
  const int slots_per_rb = 2 * k16_pairs(n_cb);
  {
    const long long slot = t >> 3;
    const int piece = (int)(t & 7);
    const long long rb = slot / slots_per_rb;
    const int c = (int)(slot - rb * slots_per_rb);
    dev[t] = c < n_cb ? q_canon[(rb * n_cb + c) * 8 + piece] : 0u;
  }
  if (t < n_slots) {
    const long long rb = t / slots_per_rb;
    const int c = (int)(t - rb * slots_per_rb);
    reinterpret_cast<uint16_t*>(dev + n_slots * 8)[t] = c < n_cb ? scale_canon[rb * n_cb + c] : (uint16_t)0;
  }
}

// k = 16 with int8 tables and groups of 4 rows: 64 bytes per group slot (the table of rows 0..3,
// then that of rows 4..7; zero for the pad group), then two fp16 scales per slot.  Canonical
// group of half-block (rb, half) and col-block c: (2 * rb + half) * n_cb + c.  One thread per
// dword of tables; the first 2 * n_slots threads also copy a scale.
__global__ __launch_bounds__(256) void pack_tab16h_kernel(const uint32_t* __restrict__ q_canon,
                                                          const uint16_t* __restrict__ scale_canon,
                                                          uint32_t* __restrict__ dev, int n_cb,
                                                          long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_slots * 16) return;
  const int slots_per_rb = 2 * k16_pairs(n_cb);
  {
    const long long slot = t >> 4;
    const int half = (int)(t >> 3) & 1, piece = (int)(t & 7);
    const long long rb = slot / slots_per_rb;
    const int c = (int)(slot - rb * slots_per_rb);
    dev[t] = c < n_cb ? q_canon[((2 * rb + half) * n_cb + c) * 8 + piece] : 0u;
  }
  if (t < n_slots * 2) {
    const long long slot = t >> 1;
    const int half = (int)(t & 1);
    const long long rb = slot / slots_per_rb;
    const int c = (int)(slot - rb * slots_per_rb);
    reinterpret_cast<uint16_t*>(dev + n_slots * 16)[t] = c < n_cb ? scale_canon[(2 * rb + half) * n_cb + c] : (uint16_t)0;
  }
}

// k = 16 with blockwise normalisation: the levels and block codes behind tables and scales.
// Levels: canonical lev[group][16] fp16 -> 8 dwords per slot (zero for the pad slot).  Codes:
// canonical code[r][c/32] (two per byte, even block in the low nibble, 4*n_cb bytes per row) ->
// 16 dwords per col-block pair: dword 2*b + e = codes of block b of the pair's col-block e, row r
// in bits [4r, 4r+4).  One thread per (slot, j < 8): level dword j and the code dword of block j.
__global__ __launch_bounds__(256) void pack_bn16_kernel(const uint32_t* __restrict__ lev_canon,
                                                        const uint8_t* __restrict__ code_canon,
                                                        uint32_t* __restrict__ lev_dev,
                                                        uint32_t* __restrict__ code_dev, int n_cb,
                                                        long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_slots * 8) return;
  const int slots_per_rb = 2 * k16_pairs(n_cb);
  const long long slot = t >> 3;
  const int j = (int)(t & 7);
  const long long rb = slot / slots_per_rb;
  const int c = (int)(slot - rb * slots_per_rb);
  const bool ok = c < n_cb;
  lev_dev[t] = ok ? lev_canon[(rb * n_cb + c) * 8 + j] : 0u;
  uint32_t w = 0;
  if (ok) {
    const int blk = c * 8 + j;                       // block index inside the row
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t byte = code_canon[(size_t)(rb * 8 + r) * (4 * n_cb) + (blk >> 1)];
      w |= ((blk & 1) ? byte >> 4 : byte & 15u) << (4 * r);
    }
  }
  // slot = rb * slots_per_rb + c: pair c / 2, col-block e = c & 1 of the pair
  code_dev[(slot >> 1) * 16 + 2 * j + (c & 1)] = w;
}

// k = 32: one thread per (col-block pair, lane): the lane's two 8-byte nibble shares (the low four
// bits of its 16 indices in each col-block, in the k = 16 layout) and its dword of fifth bits.
// Canonical group: a little-endian stream of 5-bit fields, vector v of row r at bit 5 * (128 r + v).
__global__ __launch_bounds__(256) void pack_idx32_kernel(const uint8_t* __restrict__ canon,
                                                         uint8_t* __restrict__ nib_dev,
                                                         uint32_t* __restrict__ plane_dev, int n_cb,
                                                         long long n_pair_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long ps = t >> 6;                 // (row-block, pair)
  const int lane = (int)(t & 63);
  if (ps >= n_pair_slots) return;
  const int n_pairs = k16_pairs(n_cb);
  const long long rb = ps / n_pairs;
  const int p = (int)(ps - rb * n_pairs);
  uint32_t bits[2][16];
  uint32_t words[2][2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int c = 2 * p + e;
    const bool ok = c < n_cb;
    const uint8_t* g = canon + (size_t)(rb * n_cb + (ok ? c : 0)) * 640;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t lo[4], hi[4];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int r = 4 * h + b;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          const int bit0 = 5 * (128 * r + 2 * lane + tt);
          const uint32_t two = g[bit0 >> 3] | ((uint32_t)g[(bit0 >> 3) + ((bit0 & 7) > 3 ? 1 : 0)] << 8);
          const uint32_t v = ok ? (two >> (bit0 & 7)) & 31u : 0u;
          (tt ? hi : lo)[b] = v & 15u;
          bits[e][2 * r + tt] = v >> 4;
        }
      }
      words[e][h] = k16_encode_dword(lo, hi);
    }
  }
  *reinterpret_cast<uint4*>(nib_dev + ps * 1024 + lane * 16) = make_uint4(words[0][0], words[0][1], words[1][0], words[1][1]);
  plane_dev[ps * 64 + lane] = k32_plane_encode(bits[0], bits[1]);
}

// k = 32 tables: 64 bytes per group slot (zero for the pad group), then one fp16 scale per slot.
// One thread per dword of tables; the first n_slots threads also copy a scale.
__global__ __launch_bounds__(256) void pack_tab32_kernel(const uint32_t* __restrict__ q_canon,
                                                         const uint16_t* __restrict__ scale_canon,
                                                         uint32_t* __restrict__ dev, int n_cb,
                                                         long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_slots * 16) return;
  const int slots_per_rb = 2 * k16_pairs(n_cb);
  {
    const long long slot = t >> 4;
    const int piece = (int)(t & 15);
    const long long rb = slot / slots_per_rb;
    const int c = (int)(slot - rb * slots_per_rb);
    dev[t] = c < n_cb ? q_canon[(rb * n_cb + c) * 16 + piece] : 0u;
  }
  if (t < n_slots) {
    const long long rb = t / slots_per_rb;
    const int c = (int)(t - rb * slots_per_rb);
    reinterpret_cast<uint16_t*>(dev + n_slots * 16)[t] = c < n_cb ? scale_canon[rb * n_cb + c] : (uint16_t)0;
  }
}

// Block codes of the formats with tall groups (d = 4; d = 2 with k = 256 and int8 tables): the
// same 64 bytes per (8-row block, pair of col-blocks) as above.  One thread per (8-row block,
// col-block slot, block j < 8); the slot of an absent last col-block gets zeros.
__global__ __launch_bounds__(256) void pack_codes_pair_kernel(const uint8_t* __restrict__ code_canon,
                                                              uint32_t* __restrict__ code_dev, int n_cb,
                                                              long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_slots * 8) return;
  const int slots_per_rb = 2 * k16_pairs(n_cb);
  const long long slot = t >> 3;
  const int j = (int)(t & 7);
  const long long rb = slot / slots_per_rb;
  const int c = (int)(slot - rb * slots_per_rb);
  uint32_t w = 0;
  if (c < n_cb) {
    const int blk = c * 8 + j;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t byte = code_canon[(size_t)(rb * 8 + r) * (4 * n_cb) + (blk >> 1)];
      w |= ((blk & 1) ? byte >> 4 : byte & 15u) << (4 * r);
    }
  }
  code_dev[(slot >> 1) * 16 + 2 * j + (c & 1)] = w;
}

// d = 1, k = 4: per (8-row block, col-block slot) 48 bytes: the 4 int8 values of each of the 8
// rows, then the 8 rows' fp16 scales (zero for the pad slot).  Canonical group of row R and
// col-block c: R * n_cb + c.  One thread per (slot, row).
__global__ __launch_bounds__(256) void pack_tab_d1k4_kernel(const uint32_t* __restrict__ q_canon,
                                                            const uint16_t* __restrict__ scale_canon,
                                                            uint8_t* __restrict__ dev, int n_cb,
                                                            long long n_slots) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n_slots * 8) return;
  const long long slot = t >> 3;
  const int r = (int)(t & 7);
  const int slots_per_rb = 2 * k16_pairs(n_cb);
  const long long rb = slot / slots_per_rb;
  const int c = (int)(slot - rb * slots_per_rb);
  const bool ok = c < n_cb;
  const long long g = (rb * 8 + r) * n_cb + c;
  uint8_t* rec = dev + (size_t)slot * kD1K4SlotTabBytes;
  reinterpret_cast<uint32_t*>(rec)[r] = ok ? q_canon[g] : 0u;
  reinterpret_cast<uint16_t*>(rec + kD1K4ScaleOffset)[r] = ok ? scale_canon[g] : (uint16_t)0;
}

// ---- k = 64: 6-bit indices, int8 tables with a scale per group, groups of 8*rpc rows -------
// One thread per (8-row block, quad of col-blocks, lane): gathers the lane's 4 x 16 indices
// from the canonical little-endian 6-bit stream of their groups and re-packs them as four
// 96-bit streams (index 2*row + e at bits [6i, 6i+6)), written as three 16-byte planes.
__global__ __launch_bounds__(256) void pack_idx64_kernel(const uint8_t* __restrict__ canon,
                                                         uint8_t* __restrict__ dev, int n_cb,
                                                         long long n_rb8, int rpc) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long slot = t >> 6;
  const int lane = (int)(t & 63);
  const int n_quads = k64_quads(n_cb);
  if (slot >= n_rb8 * n_quads) return;
  const long long rb8 = slot / n_quads;
  const int q = (int)(slot - rb8 * n_quads);
  const long long grow = rb8 / rpc;              // row of groups
  const int sub = (int)(rb8 - grow * rpc);       // 8-row block inside the group
  const size_t group_bytes = (size_t)rpc * 8 * 96;   // rows x 128 vectors x 6 bits
  uint32_t d[12];
#pragma unroll
  for (int i = 0; i < 12; ++i) d[i] = 0u;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = 4 * q + j;
    if (c >= n_cb) continue;
    const uint8_t* g = canon + (size_t)(grow * n_cb + c) * group_bytes;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int v = (sub * 8 + (i >> 1)) * 128 + 2 * lane + (i & 1);
      const int bit = 6 * v, b = bit >> 3, sh = bit & 7;
      uint32_t val = g[b] >> sh;
      if (sh > 2) val |= (uint32_t)g[b + 1] << (8 - sh);   // the field continues in the next byte
      val &= 63u;
      const int pos = 6 * i, dw = 3 * j + (pos >> 5), off = pos & 31;
      d[dw] |= val << off;
      if (off > 26) d[dw + 1] |= val >> (32 - off);
    }
  }
#pragma unroll
  for (int p = 0; p < 3; ++p)
    *reinterpret_cast<uint4*>(dev + ((size_t)slot * 3 + p) * 1024 + lane * 16) =
        make_uint4(d[4 * p], d[4 * p + 1], d[4 * p + 2], d[4 * p + 3]);
}

// Tables: per (row of groups, quad) four int8 tables of 128 bytes, then their four scales;
// with blockwise normalisation (level_canon != nullptr, 672-byte records) also the four
// col-blocks' 16 fp16 levels.
__global__ __launch_bounds__(256) void pack_tab64_kernel(const uint8_t* __restrict__ q_canon,
                                                         const uint16_t* __restrict__ scale_canon,
                                                         const uint16_t* __restrict__ level_canon,
                                                         uint8_t* __restrict__ dev, int n_cb,
                                                         long long n_grow) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long slot = t >> 6;
  const int lane = (int)(t & 63);
  const int n_quads = k64_quads(n_cb);
  if (slot >= n_grow * n_quads) return;
  const long long grow = slot / n_quads;
  const int q = (int)(slot - grow * n_quads);
  const int c = 4 * q + (lane >> 4);
  uint8_t* dst = dev + (size_t)slot * (level_canon ? kK64NQuadTabBytes : kK64QuadTabBytes);
  if (level_canon) {
    reinterpret_cast<uint16_t*>(dst + kK64NLevelOffset)[lane] =
        c < n_cb ? level_canon[(grow * n_cb + c) * 16 + (lane & 15)] : (uint16_t)0;
    if (lane < 8) reinterpret_cast<uint16_t*>(dst + kK64NLevelOffset + 128)[lane] = 0;   // padding
  }
  const uint2 v = c < n_cb
      ? *reinterpret_cast<const uint2*>(q_canon + (size_t)(grow * n_cb + c) * 128 + (lane & 15) * 8)
      : make_uint2(0u, 0u);
  *reinterpret_cast<uint2*>(dst + lane * 8) = v;
  if (lane < 8) {
    const int cs = 4 * q + lane;
    reinterpret_cast<uint16_t*>(dst + 512)[lane] =
        (lane < 4 && cs < n_cb) ? scale_canon[grow * n_cb + cs] : (uint16_t)0;
  }
}

// d = 1, k = 8: per (row of groups, quad) four tables of 8 int8 values, four fp16 scales, padding
// (48 bytes).  One thread per record.
// With blockwise normalisation (level_canon != nullptr): 176-byte records, the four col-blocks'
// 16 fp16 levels behind the 48 bytes.
__global__ __launch_bounds__(256) void pack_tab_d1k8_kernel(const uint8_t* __restrict__ q_canon,
                                                            const uint16_t* __restrict__ scale_canon,
                                                            const uint16_t* __restrict__ level_canon,
                                                            uint8_t* __restrict__ dev, int n_cb,
                                                            long long n_grow) {
  const long long slot = (long long)blockIdx.x * 256 + threadIdx.x;
  const int n_quads = k64_quads(n_cb);
  if (slot >= n_grow * n_quads) return;
  const long long grow = slot / n_quads;
  const int q = (int)(slot - grow * n_quads);
  uint8_t* dst = dev + (size_t)slot * (level_canon ? kD1K8NQuadTabBytes : kD1K8QuadTabBytes);
  if (level_canon) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = 4 * q + j;
      uint4* lv = reinterpret_cast<uint4*>(dst + kD1K8NLevelOffset + j * 32);
      const uint4* src = reinterpret_cast<const uint4*>(level_canon + (size_t)(grow * n_cb + (c < n_cb ? c : 0)) * 16);
      lv[0] = c < n_cb ? src[0] : make_uint4(0, 0, 0, 0);
      lv[1] = c < n_cb ? src[1] : make_uint4(0, 0, 0, 0);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = 4 * q + j;
    const bool ok = c < n_cb;
    *reinterpret_cast<uint2*>(dst + j * 8) =
        ok ? *reinterpret_cast<const uint2*>(q_canon + (size_t)(grow * n_cb + c) * 8) : make_uint2(0u, 0u);
    reinterpret_cast<uint16_t*>(dst + kD1K8ScaleOffset)[j] = ok ? scale_canon[grow * n_cb + c] : (uint16_t)0;
  }
  *reinterpret_cast<uint2*>(dst + 40) = make_uint2(0u, 0u);
}

// Block codes: canonical code[r][c/32] (two per byte, even block in the low nibble, 4*n_cb
// bytes per row) -> per (8-row block, quad) 32 dwords, dword 4*b + j = codes of block b of
// col-block 4q + j, row r in bits [4r, 4r+4).  One thread per dword.
__global__ __launch_bounds__(256) void pack_codes64_kernel(const uint8_t* __restrict__ canon,
                                                           uint32_t* __restrict__ dev, int n_cb,
                                                           long long n_rb8) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const int n_quads = k64_quads(n_cb);
  if (t >= n_rb8 * n_quads * 32) return;
  const long long slot = t >> 5;
  const int b = (int)(t & 31) >> 2, j = (int)(t & 3);
  const long long rb8 = slot / n_quads;
  const int q = (int)(slot - rb8 * n_quads);
  const int c = 4 * q + j;
  uint32_t w = 0;
  if (c < n_cb) {
    const int blk = c * 8 + b;                       // block index inside the row
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t byte = canon[(size_t)(rb8 * 8 + r) * (4 * n_cb) + (blk >> 1)];
      w |= ((blk & 1) ? byte >> 4 : byte & 15u) << (4 * r);
    }
  }
  dev[t] = w;
}

// d = 4 indices: canonical group (row of groups, c) holds group_rows x 64 bytes, byte r*64 + L =
// row r, vector L.  One thread per (8-row block, pair of col-blocks, lane).
__global__ __launch_bounds__(256) void pack_idx_d4_kernel(const uint8_t* __restrict__ canon,
                                                          uint8_t* __restrict__ dev, int n_cb,
                                                          long long n_rb8, int rpc) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long slot = t >> 6;
  const int lane = (int)(t & 63);
  const int n_pairs = (n_cb + 1) >> 1;
  if (slot >= n_rb8 * n_pairs) return;
  const long long rb8 = slot / n_pairs;
  const int p = (int)(slot - rb8 * n_pairs);
  const long long grow = rb8 / rpc;
  const int sub = (int)(rb8 - grow * rpc);
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = 2 * p + h;
    if (c >= n_cb) continue;
    const uint8_t* g = canon + (size_t)(grow * n_cb + c) * ((size_t)rpc * 8 * 64) + (size_t)sub * 8 * 64 + lane;
#pragma unroll
    for (int r = 0; r < 8; ++r) w[2 * h + (r >> 2)] |= (uint32_t)g[r * 64] << (8 * (r & 3));
  }
  *reinterpret_cast<uint4*>(dev + (size_t)slot * 1024 + lane * 16) = make_uint4(w[0], w[1], w[2], w[3]);
}

// Plain copy of n16 16-byte pieces (the last one may be partial in the source: src_bytes).
__global__ __launch_bounds__(256) void copy16_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                     long long n16, long long src_bytes) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= n16) return;
  if ((t + 1) * 16 <= src_bytes) {
    reinterpret_cast<uint4*>(dst)[t] = reinterpret_cast<const uint4*>(src)[t];
  } else {
    for (int i = 0; i < 16; ++i) dst[t * 16 + i] = t * 16 + i < src_bytes ? src[t * 16 + i] : (uint8_t)0;
  }
}

}  // namespace

hipError_t launch_pack(const vq_desc& d, const void* idx_canon, const void* cb_canon,
                       void* idx_dev, void* cb_dev, hipStream_t s) {
  const int n_cb = d.in_features / kGroupCols;
  const long long n_rb = d.out_features / kGroupRows;
  if (d.d == 4) {
    const int rpc = d.group_rows / kGroupRows;
    const long long n_groups = (long long)(d.out_features / d.group_rows) * n_cb;
    const int n_pairs = (n_cb + 1) / 2;
    hipLaunchKernelGGL(pack_idx_d4_kernel, dim3((unsigned)((n_rb * n_pairs * 64 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_rb, rpc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // int8 tables (a multiple of 16 bytes), then the scales; or fp16 tables alone: copied as they are.
    // Blockwise normalisation: the padded scales and the levels are copied too, the codes are regrouped.
    const bool bn = d.codebook_dtype == VQ_I8_BN;
    const long long src_bytes = d.codebook_dtype == VQ_F16 ? n_groups * 2048
                                : bn ? (long long)wide_bn_code_offset((size_t)n_groups, 1024) : n_groups * 1024 + 2 * n_groups;
    const long long n16 = (src_bytes + 15) / 16;
    hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)cb_canon, (uint8_t*)cb_dev, n16, src_bytes);
    e = hipGetLastError();
    if (e != hipSuccess || !bn) return e;
    const long long n_slots = n_rb * 2 * n_pairs;
    hipLaunchKernelGGL(pack_codes_pair_kernel, dim3((unsigned)((n_slots * 8 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)cb_canon + src_bytes, (uint32_t*)((uint8_t*)cb_dev + src_bytes), n_cb, n_slots);
    return hipGetLastError();
  }
  if (d.k == 64 || (d.d == 1 && d.k == 8)) {   // 6-bit fields: k = 64, or two 3-bit indices of d = 1
    const int rpc = d.group_rows / kGroupRows;
    const long long n_grow = d.out_features / d.group_rows;
    const int n_quads = k64_quads(n_cb);
    hipLaunchKernelGGL(pack_idx64_kernel, dim3((unsigned)((n_rb * n_quads * 64 + 255) / 256)), dim3(256),
                       0, s, (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_rb, rpc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (d.d == 1) {   // k = 8 scalar tables: 8 bytes per group, padded to 16 in total, then the scales
      const size_t q8 = ((size_t)n_grow * n_cb * 8 + 15) / 16 * 16;
      const bool bn8 = d.codebook_dtype == VQ_I8_BN;
      const size_t s8 = ((size_t)n_grow * n_cb * 2 + 15) / 16 * 16;        // levels follow the padded scales
      const uint8_t* canon8 = (const uint8_t*)cb_canon;
      hipLaunchKernelGGL(pack_tab_d1k8_kernel, dim3((unsigned)((n_grow * n_quads + 255) / 256)), dim3(256), 0, s,
                         canon8, (const uint16_t*)(canon8 + q8),
                         bn8 ? (const uint16_t*)(canon8 + q8 + s8) : (const uint16_t*)nullptr,
                         (uint8_t*)cb_dev, n_cb, n_grow);
      e = hipGetLastError();
      if (e != hipSuccess || !bn8) return e;
      hipLaunchKernelGGL(pack_codes64_kernel, dim3((unsigned)((n_rb * n_quads * 32 + 255) / 256)), dim3(256),
                         0, s, canon8 + q8 + s8 + (size_t)n_grow * n_cb * 32,
                         (uint32_t*)((uint8_t*)cb_dev + (size_t)n_grow * n_quads * kD1K8NQuadTabBytes), n_cb, n_rb);
      return hipGetLastError();
    }
    const size_t q_bytes = ((size_t)n_grow * n_cb * 128 + 15) / 16 * 16;   // scales follow the tables
    const bool bn = d.codebook_dtype == VQ_I8_BN;
    const size_t s_bytes = ((size_t)n_grow * n_cb * 2 + 15) / 16 * 16;     // levels follow the padded scales
    const uint8_t* canon = (const uint8_t*)cb_canon;
    hipLaunchKernelGGL(pack_tab64_kernel, dim3((unsigned)((n_grow * n_quads * 64 + 255) / 256)),
                       dim3(256), 0, s, canon, (const uint16_t*)(canon + q_bytes),
                       bn ? (const uint16_t*)(canon + q_bytes + s_bytes) : (const uint16_t*)nullptr,
                       (uint8_t*)cb_dev, n_cb, n_grow);
    e = hipGetLastError();
    if (e != hipSuccess || !bn) return e;
    hipLaunchKernelGGL(pack_codes64_kernel, dim3((unsigned)((n_rb * n_quads * 32 + 255) / 256)), dim3(256),
                       0, s, canon + q_bytes + s_bytes + (size_t)n_grow * n_cb * 32,
                       (uint32_t*)((uint8_t*)cb_dev + (size_t)n_grow * n_quads * kK64NQuadTabBytes), n_cb, n_rb);
    return hipGetLastError();
  }
  const int fmt = format_tag(d);
  if (fmt == kFmtK256I8 || fmt == kFmtK256I8BN) {   // indices as for k = 256, gathered from groups of rpc 8-row blocks; tables copied
    const int rpc = d.group_rows / kGroupRows;
    const long long n_slots = n_rb * n_cb;
    const long long n_groups = (long long)(d.out_features / d.group_rows) * n_cb;
    hipLaunchKernelGGL(pack_idx_kernel<256>, dim3((unsigned)((n_slots * 64 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots, 0, rpc);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // tables (a multiple of 16), then scales; blockwise normalisation: + padding and levels, codes regrouped
    const bool bn = fmt == kFmtK256I8BN;
    const long long src_bytes = bn ? (long long)wide_bn_code_offset((size_t)n_groups, 512) : n_groups * 512 + 2 * n_groups;
    const long long n16 = (src_bytes + 15) / 16;
    hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)cb_canon, (uint8_t*)cb_dev, n16, src_bytes);
    e = hipGetLastError();
    if (e != hipSuccess || !bn) return e;
    const long long n_code_slots = n_rb * 2 * k16_pairs(n_cb);
    hipLaunchKernelGGL(pack_codes_pair_kernel, dim3((unsigned)((n_code_slots * 8 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)cb_canon + src_bytes, (uint32_t*)((uint8_t*)cb_dev + src_bytes), n_cb, n_code_slots);
    return hipGetLastError();
  }
  const int slots_per_rb = (fmt == 16 || fmt == kFmtK16I8 || fmt == kFmtK16BN || fmt == kFmtK16I8H || fmt == kFmtK32 || fmt == kFmtD1K4) ? 2 * k16_pairs(n_cb) : n_cb;
  const long long n_slots = n_rb * slots_per_rb;
  if (fmt == kFmtK32) {
    const long long n_pair_slots = n_slots / 2;
    hipLaunchKernelGGL(pack_idx32_kernel, dim3((unsigned)((n_pair_slots * 64 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev,
                       (uint32_t*)((uint8_t*)idx_dev + (size_t)n_pair_slots * 1024), n_cb, n_pair_slots);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t q_bytes = ((size_t)n_rb * n_cb * 64 + 15) / 16 * 16;   // scales follow the tables
    hipLaunchKernelGGL(pack_tab32_kernel, dim3((unsigned)((n_slots * 16 + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)cb_canon, (const uint16_t*)((const uint8_t*)cb_canon + q_bytes),
                       (uint32_t*)cb_dev, n_cb, n_slots);
    return hipGetLastError();
  }
  if (fmt == kFmtD1K4) {
    hipLaunchKernelGGL(pack_idx_kernel<16>, dim3((unsigned)((n_slots * 64 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots, 1, 1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t q_bytes = ((size_t)d.out_features * n_cb * 4 + 15) / 16 * 16;   // scales follow the values
    hipLaunchKernelGGL(pack_tab_d1k4_kernel, dim3((unsigned)((n_slots * 8 + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)cb_canon, (const uint16_t*)((const uint8_t*)cb_canon + q_bytes),
                       (uint8_t*)cb_dev, n_cb, n_slots);
    return hipGetLastError();
  }
  if (fmt == kFmtK16I8H) {
    hipLaunchKernelGGL(pack_idx_kernel<16>, dim3((unsigned)((n_slots * 64 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots, 4, 1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t q_bytes = ((size_t)n_rb * 2 * n_cb * 32 + 15) / 16 * 16;   // scales follow the tables
    hipLaunchKernelGGL(pack_tab16h_kernel, dim3((unsigned)((n_slots * 16 + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)cb_canon, (const uint16_t*)((const uint8_t*)cb_canon + q_bytes),
                       (uint32_t*)cb_dev, n_cb, n_slots);
    return hipGetLastError();
  }
  if (fmt == kFmtK16I8 || fmt == kFmtK16BN) {
    hipLaunchKernelGGL(pack_idx_kernel<16>, dim3((unsigned)((n_slots * 64 + 255) / 256)), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots, 0, 1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t q_bytes = ((size_t)n_rb * n_cb * 32 + 15) / 16 * 16;      // scales follow the tables
    hipLaunchKernelGGL(pack_tab16_kernel, dim3((unsigned)((n_slots * 8 + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)cb_canon, (const uint16_t*)((const uint8_t*)cb_canon + q_bytes),
                       (uint32_t*)cb_dev, n_cb, n_slots);
    e = hipGetLastError();
    if (e != hipSuccess || fmt == kFmtK16I8) return e;
    // blockwise normalisation: levels follow the scales (padded to 16 bytes), codes follow the levels;
    // the bytes between the scales and the levels of the device buffer (up to 15) are never read
    const size_t s_bytes = ((size_t)n_rb * n_cb * 2 + 15) / 16 * 16;
    const uint8_t* canon = (const uint8_t*)cb_canon;
    const uint8_t* lev_canon = canon + q_bytes + s_bytes;
    hipLaunchKernelGGL(pack_bn16_kernel, dim3((unsigned)((n_slots * 8 + 255) / 256)), dim3(256), 0, s,
                       (const uint32_t*)lev_canon, lev_canon + (size_t)n_rb * n_cb * 32,
                       (uint32_t*)((uint8_t*)cb_dev + k16bn_level_offset((size_t)n_slots)),
                       (uint32_t*)((uint8_t*)cb_dev + k16bn_code_offset((size_t)n_slots)), n_cb, n_slots);
    return hipGetLastError();
  }
  const unsigned grid = (unsigned)((n_slots * 64 + 255) / 256);
  if (fmt == 16)
    hipLaunchKernelGGL(pack_idx_kernel<16>, dim3(grid), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots, 0, 1);
  else   // k = 256 bytes, or d = 1: a byte holds the two 4-bit indices of a column pair
    hipLaunchKernelGGL(pack_idx_kernel<256>, dim3(grid), dim3(256), 0, s,
                       (const uint8_t*)idx_canon, (uint8_t*)idx_dev, n_cb, n_slots, 0, 1);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int per_group = d.k * d.d * 2 / 16;                      // 16-byte pieces of one fp16 codebook
  const long long n16 = n_slots * per_group;
  hipLaunchKernelGGL(pack_cb_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                     (const uint4*)cb_canon, (uint4*)cb_dev, per_group, slots_per_rb, n_cb, n16);
  return hipGetLastError();
}

}  // namespace vq
