// Batched / prefill product Y[out,B] = W X[in,B] on vector-quantised W: the one
// place on this path that is a dense contraction.  Each workgroup decodes tiles
// of W (table lookup, Sec. 3.2) into LDS as fp16 and feeds them to the fp16
// matrix cores (v_mfma_f32_32x32x16_f16) with fp32 accumulation.
//
// A workgroup has 4 (or 8) waves and owns an MT x NT tile of Y, MT = 32*RBW (x 2) rows.  K is
// walked one col-block (256 columns) at a time:
//   * every wave decodes RBW groups (its own row-blocks of the tile) of the
//     col-block into the LDS tile Wt[MT][256]: indices and codebooks were loaded
//     into registers one col-block earlier, all 16 lookups of a lane are issued
//     before the first result is used;
//   * X is batch-contiguous, while an MFMA operand wants 8 consecutive k per lane.
//     gemm_kernel (NT = 128 / 256) copies X sub-tiles to LDS unchanged (16-byte loads, four
//     sub-tiles ahead in registers, 16-byte LDS stores) and forms the operand with the
//     transposing LDS read ds_read_b64_tr_b16; the col-block is consumed in 64- / 32-deep
//     sub-steps through two X buffers (one barrier per sub-step), wave w owns a quarter of
//     the batch columns and 32*RBW rows (RBW x NT/128 accumulator tiles); with WM = 2 the
//     workgroup has 8 waves and twice the rows, the second four waves taking the lower half;
//   * gemm_tiny_kernel (16 x 16 tiles, a private X tile per wave) and gemm_small_kernel
//     (32 x 32 tiles, bandwidth-bound batches) copy X the same way.
#include <atomic>
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

typedef _Float16 h8_t __attribute__((ext_vector_type(8)));

constexpr int WS = 256;   // LDS row stride of the decoded W tile, in halfs (no padding)

// The W tile is stored without padding; 16-byte chunk q of row m lives at chunk q ^ (m & 15),
// so the 16 lanes of one LDS pass of a 128-bit operand read (rows m..m+15, same k: 256 bytes,
// all 64 banks) and the lanes of a decode write (same row, consecutive columns) all hit
// distinct banks.  (With q ^ (m & 7) rows m and m + 8 shared their banks and every operand
// read took two passes: 8.6 against 4.7 clocks per wave-wide read in a micro-benchmark.)
__device__ __forceinline__ int wt_half_index(int m, int k) {   // k in halfs
  return m * WS + ((((k >> 3) ^ (m & 15)) << 3) | (k & 7));
}

// K is the kernel format tag: 16 / 256 (fp16 codebooks), 64 (6-bit indices, int8 tables with a
// scale per group, groups of 8*rpc rows), kFmtK16I8 (k = 16 with int8 tables).
template <int K> constexpr int lut_dwords() {
  // BN: 64 centroids + 16 levels; d = 4: 256 entries of 4 halfs; scalar 2-bit: 8 rows x 16 pair entries
  return K == kFmtK16I8 ? 16 : (K == kFmtK16BN || K == kFmtK16I8H || K == kFmtK32) ? 32 : (K == kFmtD1K16 || K == kFmtK256I8) ? 256 : K == kFmtK256I8BN ? 272 : (K == kFmtK64BN || K == kFmtD1K8BN) ? 80 : (K == kFmtD4 || K == kFmtD4F16 || K == kFmtD4BN) ? 512 : K == kFmtD1K8 ? 64 : K == kFmtD1K4 ? 128 : K;
}

// What one wave needs to decode one group: the lane's index bytes and codebook piece.
template <int K> struct GroupRegs;
template <> struct GroupRegs<16> {
  uint2 w;
  uint32_t cbv;   // lanes 0..15: one centroid each
};
template <> struct GroupRegs<256> {
  uint4 w;
  uint4 cbv;      // 4 centroids per lane
};
template <> struct GroupRegs<64> {
  uint32_t d0, d1, d2;   // the lane's 16 six-bit indices of the 8-row block
  uint32_t two;          // int8 pair of table entry `lane`
  uint32_t sc;           // the group's fp16 scale
};
template <> struct GroupRegs<kFmtD1K8> {
  uint32_t d0, d1, d2, two, sc;   // as for k = 64: `two` is pair-table entry `lane`, built from the 8 values
};
template <> struct GroupRegs<kFmtK64BN> {
  uint32_t d0, d1, d2, two, sc;   // as for k = 64
  uint32_t cw;           // the lane's block codes of this col-block, row r in bits [4r, 4r+4)
  uint32_t lev;          // block-scale level lane & 15 (fp16)
};
template <> struct GroupRegs<kFmtD1K8BN> {
  uint32_t d0, d1, d2, two, sc, cw, lev;   // as for d = 1, k = 8, plus the block scales
};
template <> struct GroupRegs<kFmtD4> {
  uint2 w;        // the lane's 8 index bytes (one vector per row)
  uint4 q;        // table entries 4*lane .. 4*lane+3 (int8 x 4 each)
  uint32_t sc;    // the group's fp16 scale
};
template <> struct GroupRegs<kFmtD4BN> {
  uint2 w;
  uint4 q;
  uint32_t sc;    // as for d = 4 with int8 tables
  uint32_t cw;    // the lane's block codes of this col-block, row r in bits [4r, 4r+4)
  uint32_t lev;   // block-scale level lane & 15 (fp16)
};
template <> struct GroupRegs<kFmtK256I8BN> {
  uint4 w;
  uint2 q;
  uint32_t sc;    // as for k = 256 with int8 tables
  uint32_t cw, lev;
};
template <> struct GroupRegs<kFmtD4F16> {
  uint2 w;
  uint4 q0, q1;   // table entries 4*lane .. 4*lane+3 (fp16 x 4 each)
};
template <> struct GroupRegs<kFmtD1K16> {
  uint4 w;
  uint2 clo;      // scalars 4*(lane%4) .. +3 of the group's 16
  uint32_t chi;   // scalar lane/4
};
template <> struct GroupRegs<kFmtK256I8> {
  uint4 w;
  uint2 q;        // table entries 4*lane .. 4*lane+3 (int8 pairs)
  uint32_t sc;    // the group's fp16 scale
};
template <> struct GroupRegs<kFmtD1K4> {
  uint2 w;
  uint32_t q4;           // the 4 int8 values of row lane >> 3
  uint32_t sc;           // ... and its fp16 scale
};
template <> struct GroupRegs<kFmtK16I8> {
  uint2 w;
  uint32_t two;          // int8 pair of table entry lane & 15
  uint32_t sc;
};
template <> struct GroupRegs<kFmtK16I8H> {
  uint2 w;
  uint32_t two;          // int8 pair of entry lane & 15 of table (lane >> 4) & 1 (rows 0..3 / rows 4..7)
  uint32_t sc;           // that table's scale
};
template <> struct GroupRegs<kFmtK32> {
  uint2 w;               // the low four bits of the lane's 16 indices, as for k = 16
  uint32_t plane;        // the fifth bits of the lane's indices in both col-blocks of the pair
  uint32_t two;          // int8 pair of table entry lane & 31
  uint32_t sc;
  int slot;              // which col-block of the pair
};
template <> struct GroupRegs<kFmtK16BN> {
  uint2 w;
  uint32_t two, sc;      // as for k = 16 with int8 tables
  uint32_t cw;           // the lane's block codes of this col-block, row r in bits [4r, 4r+4)
  uint32_t lev;          // block-scale level lane & 15 (fp16)
};

template <int K>
__device__ __forceinline__ void load_group(GroupRegs<K>& g, const uint8_t* idx, const uint32_t* cb,
                                           long long rb, int c, int n_cb, int lane, int n_rb,
                                           int rpc) {
  if constexpr (K == 16) {
    const int slots = 2 * k16_pairs(n_cb);
    g.w = *reinterpret_cast<const uint2*>(idx + (size_t)rb * slots * 512 + k16_chunk_offset(c, lane));
    g.cbv = cb[((size_t)rb * slots + c) * 16 + (lane & 15)];
  } else if constexpr (K == kFmtK16I8 || K == kFmtK16BN) {
    const int slots = 2 * k16_pairs(n_cb);
    const uint8_t* tabs = reinterpret_cast<const uint8_t*>(cb);
    g.w = *reinterpret_cast<const uint2*>(idx + (size_t)rb * slots * 512 + k16_chunk_offset(c, lane));
    g.two = *reinterpret_cast<const uint16_t*>(tabs + ((size_t)rb * slots + c) * 32 + (lane & 15) * 2);
    g.sc = reinterpret_cast<const uint16_t*>(tabs + (size_t)n_rb * slots * 32)[(size_t)rb * slots + c];
    if constexpr (K == kFmtK16BN) {
      const size_t n_slots = (size_t)n_rb * slots, slot = (size_t)rb * slots + c;
      g.lev = reinterpret_cast<const uint16_t*>(tabs + k16bn_level_offset(n_slots))[slot * 16 + (lane & 15)];
      g.cw = reinterpret_cast<const uint32_t*>(tabs + k16bn_code_offset(n_slots))[(slot >> 1) * 16 + 2 * (lane >> 3) + (c & 1)];
    }
  } else if constexpr (K == kFmtK32) {
    const int slots = 2 * k16_pairs(n_cb);
    const uint8_t* tabs = reinterpret_cast<const uint8_t*>(cb);
    const size_t slot = (size_t)rb * slots + c;
    g.w = *reinterpret_cast<const uint2*>(idx + (size_t)rb * slots * 512 + k16_chunk_offset(c, lane));
    g.plane = reinterpret_cast<const uint32_t*>(idx + (size_t)n_rb * slots * 512)[(slot >> 1) * 64 + lane];
    g.two = *reinterpret_cast<const uint16_t*>(tabs + slot * 64 + (lane & 31) * 2);
    g.sc = reinterpret_cast<const uint16_t*>(tabs + (size_t)n_rb * slots * 64)[slot];
    g.slot = c & 1;
  } else if constexpr (K == kFmtK16I8H) {
    const int slots = 2 * k16_pairs(n_cb);
    const uint8_t* tabs = reinterpret_cast<const uint8_t*>(cb);
    const size_t slot = (size_t)rb * slots + c;
    g.w = *reinterpret_cast<const uint2*>(idx + (size_t)rb * slots * 512 + k16_chunk_offset(c, lane));
    g.two = *reinterpret_cast<const uint16_t*>(tabs + slot * 64 + (lane & 31) * 2);
    g.sc = reinterpret_cast<const uint16_t*>(tabs + (size_t)n_rb * slots * 64)[slot * 2 + ((lane >> 4) & 1)];
  } else if constexpr (K == kFmtD1K4) {
    const int slots = 2 * k16_pairs(n_cb);
    const uint8_t* rec = reinterpret_cast<const uint8_t*>(cb) + ((size_t)rb * slots + c) * kD1K4SlotTabBytes;
    g.w = *reinterpret_cast<const uint2*>(idx + (size_t)rb * slots * 512 + k16_chunk_offset(c, lane));
    g.q4 = *reinterpret_cast<const uint32_t*>(rec + (lane >> 3) * 4);
    g.sc = *reinterpret_cast<const uint16_t*>(rec + kD1K4ScaleOffset + (lane >> 3) * 2);
  } else if constexpr (K == kFmtD4F16) {
    const uint8_t* tab = reinterpret_cast<const uint8_t*>(cb);
    const size_t gi = (size_t)(rb / rpc) * n_cb + c;
    g.w = *reinterpret_cast<const uint2*>(idx + ((size_t)rb * ((n_cb + 1) >> 1) + (c >> 1)) * 1024 + lane * 16 + (c & 1) * 8);
    g.q0 = *reinterpret_cast<const uint4*>(tab + gi * 2048 + lane * 32);
    g.q1 = *reinterpret_cast<const uint4*>(tab + gi * 2048 + lane * 32 + 16);
  } else if constexpr (K == kFmtD4 || K == kFmtD4BN) {
    const uint8_t* tab = reinterpret_cast<const uint8_t*>(cb);
    const size_t gi = (size_t)(rb / rpc) * n_cb + c, n_groups = (size_t)(n_rb / rpc) * n_cb;
    g.w = *reinterpret_cast<const uint2*>(idx + ((size_t)rb * ((n_cb + 1) >> 1) + (c >> 1)) * 1024 + lane * 16 + (c & 1) * 8);
    g.q = *reinterpret_cast<const uint4*>(tab + gi * 1024 + lane * 16);
    g.sc = reinterpret_cast<const uint16_t*>(tab + n_groups * 1024)[gi];
    if constexpr (K == kFmtD4BN) {
      g.lev = reinterpret_cast<const uint16_t*>(tab + wide_bn_level_offset(n_groups, 1024))[gi * 16 + (lane & 15)];
      g.cw = reinterpret_cast<const uint32_t*>(tab + wide_bn_code_offset(n_groups, 1024))
                 [((size_t)rb * ((n_cb + 1) >> 1) + (c >> 1)) * 16 + 2 * (lane >> 3) + (c & 1)];
    }
  } else if constexpr (K == kFmtK256I8 || K == kFmtK256I8BN) {
    const uint8_t* tab = reinterpret_cast<const uint8_t*>(cb);
    const size_t gt = (size_t)(rb / rpc) * n_cb + c, n_tabs = (size_t)(n_rb / rpc) * n_cb;
    g.w = *reinterpret_cast<const uint4*>(idx + ((size_t)rb * n_cb + c) * 1024 + lane * 16);
    g.q = *reinterpret_cast<const uint2*>(tab + gt * 512 + lane * 8);
    g.sc = reinterpret_cast<const uint16_t*>(tab + n_tabs * 512)[gt];
    if constexpr (K == kFmtK256I8BN) {
      g.lev = reinterpret_cast<const uint16_t*>(tab + wide_bn_level_offset(n_tabs, 512))[gt * 16 + (lane & 15)];
      g.cw = reinterpret_cast<const uint32_t*>(tab + wide_bn_code_offset(n_tabs, 512))
                 [((size_t)rb * ((n_cb + 1) >> 1) + (c >> 1)) * 16 + 2 * (lane >> 3) + (c & 1)];
    }
  } else if constexpr (K == kFmtD1K16) {
    const size_t gi = (size_t)rb * n_cb + c;
    const uint8_t* cg = reinterpret_cast<const uint8_t*>(cb) + gi * 32;
    g.w = *reinterpret_cast<const uint4*>(idx + gi * 1024 + lane * 16);
    g.clo = *reinterpret_cast<const uint2*>(cg + (lane & 3) * 8);
    g.chi = *reinterpret_cast<const uint16_t*>(cg + (lane >> 2) * 2);
  } else if constexpr (K == 64 || K == kFmtK64BN || K == kFmtD1K8 || K == kFmtD1K8BN) {
    constexpr int tab_bytes = K == 64 ? kK64QuadTabBytes : K == kFmtD1K8 ? kD1K8QuadTabBytes
                              : K == kFmtD1K8BN ? kD1K8NQuadTabBytes : kK64NQuadTabBytes;
    constexpr int level_offset = K == kFmtD1K8BN ? kD1K8NLevelOffset : kK64NLevelOffset;
    const int n_quads = k64_quads(n_cb), q = c >> 2, j = c & 3;
    const uint8_t* iq = idx + ((size_t)rb * n_quads + q) * kK64QuadIdxBytes + lane * 16;
    const int w0 = 3 * j, w1 = 3 * j + 1, w2 = 3 * j + 2;     // the lane's dwords of col-block j
    g.d0 = *reinterpret_cast<const uint32_t*>(iq + (w0 >> 2) * 1024 + (w0 & 3) * 4);
    g.d1 = *reinterpret_cast<const uint32_t*>(iq + (w1 >> 2) * 1024 + (w1 & 3) * 4);
    g.d2 = *reinterpret_cast<const uint32_t*>(iq + (w2 >> 2) * 1024 + (w2 & 3) * 4);
    const uint8_t* tq = reinterpret_cast<const uint8_t*>(cb) +
                        ((size_t)(rb / rpc) * n_quads + q) * tab_bytes;
    if constexpr (K == kFmtD1K8 || K == kFmtD1K8BN) {
      g.two = d1k8_pair(*reinterpret_cast<const uint2*>(tq + j * 8), lane);
      g.sc = *reinterpret_cast<const uint16_t*>(tq + kD1K8ScaleOffset + 2 * j);
    } else {
      g.two = *reinterpret_cast<const uint16_t*>(tq + j * 128 + lane * 2);
      g.sc = *reinterpret_cast<const uint16_t*>(tq + 512 + 2 * j);
    }
    if constexpr (K == kFmtK64BN || K == kFmtD1K8BN) {
      g.lev = *reinterpret_cast<const uint16_t*>(tq + level_offset + j * 32 + (lane & 15) * 2);
      g.cw = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(cb) +
                                                (size_t)(n_rb / rpc) * n_quads * tab_bytes +
                                                ((size_t)rb * n_quads + q) * kK64NQuadCodeBytes +
                                                (lane >> 3) * 16 + j * 4);
    }
  } else {
    const size_t gi = (size_t)rb * n_cb + c;
    g.w = *reinterpret_cast<const uint4*>(idx + gi * 1024 + lane * 16);
    g.cbv = *reinterpret_cast<const uint4*>(cb + gi * 256 + lane * 4);
  }
}

template <int K> __device__ __forceinline__ uint32_t g_level2(const GroupRegs<K>&) { return 0u; }
template <> __device__ __forceinline__ uint32_t g_level2<kFmtD4BN>(const GroupRegs<kFmtD4BN>& g) { return g.lev * 0x10001u; }

// Decodes one group into rows [m0, m0+8) of the W tile (lane L owns columns 4L..4L+3).
template <int K>
__device__ __forceinline__ void decode_group(const GroupRegs<K>& g, uint32_t* lut, uint16_t* Wt,
                                             int m0, int lane) {
  const char* lutb = reinterpret_cast<const char*>(lut);
  uint32_t v[16];
  if constexpr (K == kFmtD4 || K == kFmtD4F16 || K == kFmtD4BN) {
    uint2* lut2 = reinterpret_cast<uint2*>(lut);
    if constexpr (K == kFmtD4F16) {
      *reinterpret_cast<uint4*>(lut2 + 4 * lane) = g.q0;
      *reinterpret_cast<uint4*>(lut2 + 4 * lane + 2) = g.q1;
    } else {
      const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)g.sc);
      lut2[4 * lane] = d4_dequant_entry(g.q.x, scale);
      lut2[4 * lane + 1] = d4_dequant_entry(g.q.y, scale);
      lut2[4 * lane + 2] = d4_dequant_entry(g.q.z, scale);
      lut2[4 * lane + 3] = d4_dequant_entry(g.q.w, scale);
    }
    // d = 4 with block scales: the table fills the wave's whole region, so the 16 levels stay in
    // registers (lane L holds level L & 15, the value in both halves) and a lane fetches the one
    // its code selects with a cross-lane read.
    const uint32_t lev2 = K == kFmtD4BN ? g_level2(g) : 0u;
    wave_lds_sync();
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint2 t = lut2[((r < 4 ? g.w.x : g.w.y) >> (8 * (r & 3))) & 0xffu];
      v[2 * r] = t.x;
      v[2 * r + 1] = t.y;
      if constexpr (K == kFmtD4BN) {     // times the block scale of the lane's 32-weight block
        const uint32_t sc = (uint32_t)__builtin_amdgcn_ds_bpermute((int)(((g.cw >> (4 * r)) & 15u) << 2), (int)lev2);
        v[2 * r] = scale_pair(t.x, sc);
        v[2 * r + 1] = scale_pair(t.y, sc);
      }
    }
  } else if constexpr (K == 64 || K == kFmtK64BN || K == kFmtD1K8 || K == kFmtD1K8BN) {
    lut[lane] = k64_dequant_pair(g.two, __builtin_bit_cast(_Float16, (uint16_t)g.sc));
    if constexpr (K == kFmtK64BN || K == kFmtD1K8BN) {
      if (lane < 16) lut[64 + lane] = g.lev * 0x10001u;
    }
    wave_lds_sync();
    const unsigned long long lo = g.d0 | ((unsigned long long)g.d1 << 32);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int pos = 6 * i;
      unsigned long long t = pos < 64 ? lo >> pos : (unsigned long long)(g.d2 >> (pos - 64));
      if (pos < 64 && pos > 58) t |= (unsigned long long)g.d2 << (64 - pos);
      v[i] = lut[(uint32_t)t & 63u];
    }
    if constexpr (K == kFmtK64BN || K == kFmtD1K8BN) {     // times the block scale of the lane's 32-weight block, per row
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const h2_t sc = __builtin_bit_cast(h2_t, lut[64 + ((g.cw >> (4 * r)) & 15u)]);
        v[2 * r] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, v[2 * r]) * sc);
        v[2 * r + 1] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, v[2 * r + 1]) * sc);
      }
    }
  } else if constexpr (K == kFmtD1K4) {   // lane L: entries 2*(L&7), +1 of row L >> 3; row r looks up in table r
    const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)g.sc);
    const int j = 2 * (lane & 7);
    *reinterpret_cast<uint2*>(lut + 2 * lane) =
        make_uint2(k64_dequant_pair(d1k4_pair(g.q4, j), scale), k64_dequant_pair(d1k4_pair(g.q4, j + 1), scale));
    wave_lds_sync();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t a, b;
      k16_split_dword(h ? g.w.y : g.w.x, a, b);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const char* row_tab = lutb + (4 * h + r) * 64;
        v[8 * h + 2 * r] = *reinterpret_cast<const uint32_t*>(row_tab + ((a >> (8 * r)) & 0xffu));
        v[8 * h + 2 * r + 1] = *reinterpret_cast<const uint32_t*>(row_tab + ((b >> (8 * r)) & 0xffu));
      }
    }
  } else if constexpr (K == 16 || K == kFmtK16I8 || K == kFmtK16BN || K == kFmtK16I8H || K == kFmtK32) {
    if constexpr (K == 16) {
      if (lane < 16) lut[lane] = g.cbv;
    } else if constexpr (K == kFmtK16I8H || K == kFmtK32) {
      if (lane < 32) lut[lane] = k64_dequant_pair(g.two, __builtin_bit_cast(_Float16, (uint16_t)g.sc));
    } else {
      if (lane < 16) lut[lane] = k64_dequant_pair(g.two, __builtin_bit_cast(_Float16, (uint16_t)g.sc));
      if constexpr (K == kFmtK16BN) {
        if (lane < 16) lut[16 + lane] = g.lev * 0x10001u;   // the level in both halves
      }
    }
    const auto& q = g;
    wave_lds_sync();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint32_t a, b;
      k16_split_dword(h ? q.w.y : q.w.x, a, b);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const char* lut_h = lutb + (K == kFmtK16I8H ? 64 * h : 0);   // groups of 4 rows: rows 4..7 use the second table
        uint32_t oa = (a >> (8 * r)) & 0xffu, ob = (b >> (8 * r)) & 0xffu;
        if constexpr (K == kFmtK32) {                                // the fifth bit selects the upper half of the table
          oa += 64 * k32_plane_bit(q.plane, q.slot, 4 * h + r, 0);
          ob += 64 * k32_plane_bit(q.plane, q.slot, 4 * h + r, 1);
        }
        v[8 * h + 2 * r] = *reinterpret_cast<const uint32_t*>(lut_h + oa);
        v[8 * h + 2 * r + 1] = *reinterpret_cast<const uint32_t*>(lut_h + ob);
      }
    }
    if constexpr (K == kFmtK16BN) {     // times the block scale of the lane's 32-weight block, per row
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const h2_t sc = __builtin_bit_cast(h2_t, lut[16 + ((q.cw >> (4 * r)) & 15u)]);
        v[2 * r] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, v[2 * r]) * sc);
        v[2 * r + 1] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, v[2 * r + 1]) * sc);
      }
    }
  } else {
    const auto& q = g;
    if constexpr (K == kFmtD1K16) {
      *reinterpret_cast<uint4*>(lut + lane * 4) = d1_pair_entries(q.clo, q.chi);
    } else if constexpr (K == kFmtK256I8 || K == kFmtK256I8BN) {
      const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)q.sc);
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(q.q.x, scale), k64_dequant_pair(q.q.x >> 16, scale),
                     k64_dequant_pair(q.q.y, scale), k64_dequant_pair(q.q.y >> 16, scale));
      if constexpr (K == kFmtK256I8BN) {
        if (lane < 16) lut[256 + lane] = q.lev * 0x10001u;
      }
    } else {
      *reinterpret_cast<uint4*>(lut + lane * 4) = q.cbv;
    }
    wave_lds_sync();
    const uint32_t ws[4] = {q.w.x, q.w.y, q.w.z, q.w.w};
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = lut[(ws[i >> 2] >> (8 * (i & 3))) & 0xffu];
    if constexpr (K == kFmtK256I8BN) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const uint32_t sc = lut[256 + ((q.cw >> (4 * r)) & 15u)];
        v[2 * r] = scale_pair(v[2 * r], sc);
        v[2 * r + 1] = scale_pair(v[2 * r + 1], sc);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 8; ++r)
    *reinterpret_cast<uint2*>(Wt + wt_half_index(m0 + r, 4 * lane)) = make_uint2(v[2 * r], v[2 * r + 1]);
}

// ---- X staging (all three kernels) ------------------------------------------------------
// An X sub-tile lives in LDS as it is in memory, Xs[k][NT] halfs with the batch index
// contiguous, and the matrix-core operand (8 consecutive k of one column per lane) is formed by
// the transposing LDS read ds_read_b64_tr_b16.  In each block of 16 lanes, lane i hands in the
// address of 4 consecutive halfs, row i / 4 and column fragment i % 4 of a 4 x 16 tile, and
// gets back column i of that tile (4 rows).  The LDS serves a 64-bit read 32 lanes (256 bytes,
// all 64 banks) at a time, i.e. two such tiles, 32 bytes apart in the same four rows: gemm_kernel
// stores the 32-byte chunk c of row k at chunk c ^ 2 * (k & 3), which sends the four rows of the
// even tile to the four even chunks of an aligned group of eight and those of the odd tile to
// the odd ones (with c ^ (k & 3) the two tiles shared four chunks and every read took two
// passes: 4.4 against 2.7 clocks per wave-wide read in a micro-benchmark).
typedef short s4_t __attribute__((ext_vector_type(4)));
typedef short s8_t __attribute__((ext_vector_type(8)));

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
struct XRows {
  u32x4_t r[4];   // 16 bytes (8 batch columns) of four rows of the sub-tile, one per pass
};

// Rows row0 + j * RPP (j = 0..3) are wave-uniform; voff is the lane's part in bytes.
template <int RPP, int PASSES = 4>
__device__ __forceinline__ void load_xrows(XRows& p, const uint16_t* X, long long row0, int ldx,
                                           uint32_t voff) {
  const char* base = reinterpret_cast<const char*>(X) + (size_t)row0 * ldx * 2;
#pragma unroll
  for (int j = 0; j < PASSES; ++j)
    p.r[j] = *reinterpret_cast<const u32x4_t*>(base + (size_t)j * RPP * ldx * 2 + voff);
}
template <int RPP, int NT, int PASSES = 4>
__device__ __forceinline__ void store_xrows(const XRows& p, char* dst) {
#pragma unroll
  for (int j = 0; j < PASSES; ++j) *reinterpret_cast<u32x4_t*>(dst + j * RPP * NT * 2) = p.r[j];
}
// 8 consecutive k of the lane's column from two 4-row tiles at lo and hi.
__device__ __forceinline__ h8_t read_x_operand2(const char* lo_src, const char* hi_src) {
  typedef s4_t __attribute__((address_space(3))) * lds_s4_ptr;
  const s4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(lo_src));
  const s4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(hi_src));
  return __builtin_bit_cast(h8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// 8 consecutive k (two 4-row tiles, 4 * NT * 2 bytes apart) of the lane's column.
template <int NT>
__device__ __forceinline__ h8_t read_x_operand(const char* src) {
  typedef s4_t __attribute__((address_space(3))) * lds_s4_ptr;
  const s4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(src));
  const s4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(src + 4 * NT * 2));
  return __builtin_bit_cast(h8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

template <int K, int RBW, int NT, int WM = 1>
__global__ __launch_bounds__(256 * WM, WM == 1 ? 2 : 1) void gemm_kernel(const uint8_t* __restrict__ idx,
                                                   const uint32_t* __restrict__ cb,
                                                   const uint16_t* __restrict__ X, int B, int ldx,
                                                   void* __restrict__ Y, int ldy, int y_f32,
                                                   int n_rb, int n_cb, int n_tiles_n, int rpc,
                                                   int rb0, int rb_end) {
  // the launch covers row-blocks [rb0, rb_end) of the matrix's n_rb; tile rows count from rb0
  static_assert(NT == 128 || NT == 256 || (NT == 512 && WM == 2), "column tile");
  constexpr int MT = 32 * RBW * WM;
  constexpr int KS = 8192 / NT;                  // k per X sub-tile: 64 or 32
  constexpr int NSUB = 256 / KS;                 // sub-steps per col-block: 4 or 8
  constexpr int NB = NT / 128;                   // 32-column accumulator tiles per wave
  constexpr int D = NT == 512 ? 2 : 4;           // X pieces in flight per thread (sub-tiles ahead; registers are short at 512 columns)
  static_assert(NSUB % D == 0, "ring slot must be a compile-time constant");
  __shared__ __attribute__((aligned(16))) uint16_t Wt[MT * WS];
  __shared__ __attribute__((aligned(16))) uint32_t Xs_all[2][4096];     // [KS][NT] halfs each

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wc = wave & 3, wr = wave >> 2;       // column quarter, row half
  const int mt = blockIdx.x / n_tiles_n;
  const int nt = blockIdx.x - mt * n_tiles_n;

  // X staging role: a sub-tile is copied in 4 passes of RPP rows; the thread owns 16 bytes
  // (8 batch columns from n_loc) of row x_row of every pass.  Columns at or beyond B are
  // loaded from column 0 instead: they only reach accumulator columns that are never written.
  constexpr int RPP = 2048 * WM / NT;            // rows per pass
  constexpr int PASSES = 4 / WM;
  const int x_row = tid / (NT / 8);
  const int n_loc = (tid % (NT / 8)) * 8;
  const int n_glob = nt * NT + n_loc;
  const int x_row_wave = wave * (512 / NT);      // first row of the wave inside a pass
  const int xs_off = x_row * NT * 2 + ((((n_loc >> 4) ^ (2 * (x_row & 3))) << 5) | ((n_loc & 8) << 1));
  uint32_t x_voff = (uint32_t)(((x_row - x_row_wave) * ldx + (n_glob < B ? n_glob : 0)) * 2);
  asm volatile("" : "+v"(x_voff));   // keep it one 32-bit register next to scalar row bases
  // operand role: lane i of a 16-lane block addresses row i / 4, fragment i % 4 of a 4 x 16 tile
  int xr_off[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int kq = (lane & 15) >> 2;
    const int chunk = ((wc * NB + b) * 32 + (lane & 16)) >> 4;
    xr_off[b] = (8 * (lane >> 5) + kq) * NT * 2 + ((chunk ^ (2 * kq)) << 5) + (lane & 3) * 8;
  }
  const int n_subtiles = n_cb * NSUB;

  f16v_t acc[RBW][NB];
#pragma unroll
  for (int a = 0; a < RBW; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // prologue: registers for col-block 0, X sub-tile 0 into buffer 0, sub-tiles 1..D in flight
  GroupRegs<K> g[RBW];
  long long rbs[RBW];
  bool rb_ok[RBW];
#pragma unroll
  for (int a = 0; a < RBW; ++a) {
    rbs[a] = rb0 + (long long)mt * (4 * RBW * WM) + wave * RBW + a;
    rb_ok[a] = rbs[a] < rb_end;
    load_group<K>(g[a], idx, cb, rb_ok[a] ? rbs[a] : 0, 0, n_cb, lane, n_rb, rpc);
  }
  XRows ring[D];   // slot t % D holds sub-tile t + 1 when sub-step t starts
  {
    XRows first;
    load_xrows<RPP, PASSES>(first, X, x_row_wave, ldx, x_voff);
#pragma unroll
    for (int i = 0; i < D; ++i)
      load_xrows<RPP, PASSES>(ring[i], X, (long long)min(i + 1, n_subtiles - 1) * KS + x_row_wave, ldx, x_voff);
    store_xrows<RPP, NT, PASSES>(first, reinterpret_cast<char*>(Xs_all[0]) + xs_off);
  }
  int cur = 0;   // X buffer the next MFMA step reads

  for (int c = 0; c < n_cb; ++c) {
    // every wave is past its MFMA reads of Wt (barrier at the end of the last sub-step); the
    // tables live in the X buffer that is idle while a col-block is being decoded
    uint32_t* lut = Xs_all[1 - cur] + wave * lut_dwords<K>();
    static_assert(4 * WM * lut_dwords<K>() <= 4096, "the waves' tables must fit in one X buffer");
#pragma unroll
    for (int a = 0; a < RBW; ++a) {
      const int m0 = (wave * RBW + a) * 8;
      if (rb_ok[a]) {
        decode_group<K>(g[a], lut, Wt, m0, lane);
      } else {
#pragma unroll
        for (int r = 0; r < 8; ++r)
          *reinterpret_cast<uint2*>(Wt + wt_half_index(m0 + r, 4 * lane)) = make_uint2(0u, 0u);
      }
      // next col-block's registers (clamped on the last one: a harmless re-read)
      load_group<K>(g[a], idx, cb, rb_ok[a] ? rbs[a] : 0, min(c + 1, n_cb - 1), n_cb, lane, n_rb, rpc);
    }
    __syncthreads();   // Wt of this col-block and the X sub-tile in Xs[cur] are complete

#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
      const char* Xs = reinterpret_cast<const char*>(Xs_all[cur]);
      // stage sub-tile t + 1 (loaded D sub-steps ago) into the other buffer while this one is
      // multiplied (after the last sub-tile this rewrites it: nobody reads that copy), and start
      // loading sub-tile t + 1 + D into the slot it leaves
      const int t = c * NSUB + sub;
      XRows& slot = ring[sub % D];
      store_xrows<RPP, NT, PASSES>(slot, reinterpret_cast<char*>(Xs_all[cur ^ 1]) + xs_off);
      load_xrows<RPP, PASSES>(slot, X, (long long)min(t + 1 + D, n_subtiles - 1) * KS + x_row_wave, ldx, x_voff);
      // wave w: batch columns [32*NB*w, 32*NB*(w+1)), all MT rows, the KS k of this sub-step
#pragma unroll
      for (int kk = 0; kk < KS / 16; ++kk) {
        h8_t bv[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
          bv[b] = read_x_operand<NT>(Xs + xr_off[b] + 16 * kk * NT * 2);
#pragma unroll
        for (int a = 0; a < RBW; ++a) {
          const h8_t av = *reinterpret_cast<const h8_t*>(
              Wt + wt_half_index(wr * 32 * RBW + 32 * a + (lane & 31), sub * KS + 16 * kk + 8 * (lane >> 5)));
#pragma unroll
          for (int b = 0; b < NB; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv[b], acc[a][b], 0, 0, 0);
        }
      }
      __syncthreads();   // reads of Xs[cur] (and, on the last sub-step, of Wt) done; Xs[cur^1] complete
      cur ^= 1;
    }
  }

  // ---- store: accumulator register i holds row 8*(i/4) + 4*(lane/32) + i%4, column lane%32
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    const int n = nt * NT + (wc * NB + b) * 32 + (lane & 31);
    if (n < B) {
#pragma unroll
      for (int a = 0; a < RBW; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = rb0 * 8 + mt * MT + wr * 32 * RBW + 32 * a + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
          if (row < rb_end * 8) {
            const size_t o = (size_t)row * ldy + n;
            if (y_f32) reinterpret_cast<float*>(Y)[o] = acc[a][b][i];
            else reinterpret_cast<_Float16*>(Y)[o] = (_Float16)acc[a][b][i];
          }
        }
    }
  }
}

// ---- tiny batches (B <= 16 per workgroup column): latency- and bandwidth-bound --------
// 16 rows (two row-blocks) x 16 batch columns per workgroup, v_mfma_f32_16x16x32_f16.  The
// four waves split K by col-block (wave w takes col-blocks w, w+4, ...) and share nothing
// until the end: each wave decodes its two groups into a private LDS tile Wt[16][256],
// copies its X tile unchanged into a private Xt[256 k][16 columns] (the matrix-core operand is
// formed by the transposing LDS read), and multiplies; there is
// no workgroup barrier inside the K loop, so the waves of a CU run out of step and hide
// each other's latencies.  Indices, codebooks and X of the wave's next col-block load
// into registers while the current one is processed.  The four partial 16 x 16 tiles meet
// in LDS at the end.  Many small workgroups (out/16 per 16 columns) keep every CU streaming.
typedef float f4v_t __attribute__((ext_vector_type(4)));
constexpr int kTinyXRows = 64;                 // rows of X a wave stages at a time
constexpr int kTinyXPasses = kTinyXRows / 32;  // 32-row passes (1 KB each) per staging step

template <int K>
__global__ __launch_bounds__(256, 2) void gemm_tiny_kernel(const uint8_t* __restrict__ idx,
                                                           const uint32_t* __restrict__ cb,
                                                           const uint16_t* __restrict__ X, int B,
                                                           int ldx, void* __restrict__ Y, int ldy,
                                                           int y_f32, int n_rb, int n_cb, int rpc) {
  __shared__ __attribute__((aligned(16))) uint16_t Wt_all[4][16 * WS];
  // [k][16 columns], as in memory; a quarter of a col-block at a time, which keeps the workgroup
  // under a third of the LDS for every format but d = 4 (three workgroups per CU; fewer than 170
  // registers, so the registers allow three as well)
  __shared__ __attribute__((aligned(16))) uint16_t Xt_all[4][kTinyXRows * 16];
  __shared__ __attribute__((aligned(16))) uint32_t lut_all[4][2 * lut_dwords<K>()];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint16_t* Wt = Wt_all[wave];
  uint16_t* Xt = Xt_all[wave];
  uint32_t* lut = lut_all[wave];

  const long long rb0 = 2ll * blockIdx.x;
  const long long rb1 = min(rb0 + 1, (long long)n_rb - 1);   // odd tail: decoded twice, stored once
  const int n0 = blockIdx.y * 16;

  // X of a col-block (256 rows x 16 columns) is copied to LDS unchanged in 8 passes of 32 rows:
  // the lane owns 16 bytes (8 columns: half `xh`) of row lane / 2 of every pass, so a pass is
  // one coalesced 1 KB load when ldx = 16.  A half that lies beyond the row (ldx < 16 columns
  // from n0) is not loaded; columns between B and ldx hold whatever X holds there and only
  // reach accumulator columns that are never written.
  const int xh = lane & 1;
  const bool x_ok = n0 + 8 * xh + 8 <= ldx;
  const size_t x_lane = (size_t)(lane >> 1) * ldx + (x_ok ? n0 + 8 * xh : 0);
  // Inside a pass of 32 rows, row r sits at position r ^ 4 if r & 8 (rows 8..11 and 12..15 trade
  // places): the LDS serves a 64-bit read 32 lanes at a time, i.e. the 4 x 16 tiles of two
  // 16-lane blocks, whose rows are 8 apart (256 bytes: the same banks) without the swap.
  const int xs_row = lane >> 1;
  const int xs_off = (xs_row ^ ((xs_row & 8) >> 1)) * 32 + xh * 16;   // bytes inside Xt
  // operand role (ds_read_b64_tr_b16): lane i of a 16-lane block addresses row i / 4, fragment
  // i % 4 of a 4 x 16 tile and receives column i; rows 8q + kq (first read) and 8q + kq + 4
  const int xr_base = (8 * (lane >> 4) + ((lane & 15) >> 2)) * 32 + (lane & 3) * 8;
  const int xr_swap = ((lane >> 4) & 1) * 128;                  // odd q: the two reads trade places
  const int xr_lo = xr_base + xr_swap, xr_hi = xr_base + 128 - xr_swap;
  f4v_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  GroupRegs<K> g[2][2];
  u32x4_t xr[2][8];

  // every load is issued whether or not the col-block exists (clamped), so that the number
  // of loads in flight is static and the waits stay partial
#define VQ_ISSUE(SLOT, C)                                                              \
  {                                                                                    \
    const int cc = min((C), n_cb - 1);                                                 \
    load_group<K>(g[SLOT][0], idx, cb, rb0, cc, n_cb, lane, n_rb, rpc);                           \
    load_group<K>(g[SLOT][1], idx, cb, rb1, cc, n_cb, lane, n_rb, rpc);                           \
    _Pragma("unroll") for (int j = 0; j < 8; ++j)                                      \
      xr[SLOT][j] = *reinterpret_cast<const u32x4_t*>(X + ((size_t)cc * 256 + 32 * j) * ldx + x_lane); \
  }
#define VQ_PROCESS(SLOT)                                                               \
  {                                                                                    \
    decode_group<K>(g[SLOT][0], lut, Wt, 0, lane);                                     \
    decode_group<K>(g[SLOT][1], lut + lut_dwords<K>(), Wt, 8, lane);                                 \
    _Pragma("unroll") for (int hf = 0; hf < 8 / kTinyXPasses; ++hf) {                  \
      _Pragma("unroll") for (int j = 0; j < kTinyXPasses; ++j)                         \
        *reinterpret_cast<u32x4_t*>(reinterpret_cast<char*>(Xt) + 1024 * j + xs_off) = \
            x_ok ? xr[SLOT][kTinyXPasses * hf + j] : u32x4_t{0u, 0u, 0u, 0u};          \
      wave_lds_sync();                                                                 \
      _Pragma("unroll") for (int kk = 0; kk < kTinyXPasses; ++kk) {                    \
        const int k0 = 32 * (kTinyXPasses * hf + kk) + 8 * (lane >> 4);                \
        const h8_t av = *reinterpret_cast<const h8_t*>(Wt + wt_half_index(lane & 15, k0)); \
        const h8_t bv = read_x_operand2(reinterpret_cast<const char*>(Xt) + 1024 * kk + xr_lo,  \
                                        reinterpret_cast<const char*>(Xt) + 1024 * kk + xr_hi); \
        if (kk & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0); \
        else acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);     \
      }                                                                                \
    }                                                                                  \
  }

  VQ_ISSUE(0, wave)
  for (int c = wave; c < n_cb; c += 8) {
    VQ_ISSUE(1, c + 4)
    VQ_PROCESS(0)
    VQ_ISSUE(0, c + 8)
    if (c + 4 < n_cb) VQ_PROCESS(1)
  }
#undef VQ_ISSUE
#undef VQ_PROCESS

  // four partial 16 x 16 tiles -> LDS -> sum -> Y   (lane l holds rows 4*(l/16)+i, column l%16)
  __syncthreads();
  float* part = reinterpret_cast<float*>(Wt_all[0]);      // 4 x 256 floats
  const f4v_t acc = acc0 + acc1;
#pragma unroll
  for (int i = 0; i < 4; ++i) part[wave * 256 + (4 * (lane >> 4) + i) * 16 + (lane & 15)] = acc[i];
  __syncthreads();
  {
    const int m = tid >> 4, nl = tid & 15;
    const float sum = part[tid] + part[256 + tid] + part[512 + tid] + part[768 + tid];
    const long long row = rb0 * 8 + m;
    const int n = n0 + nl;
    if (row < (long long)n_rb * 8 && n < B) {
      const size_t off = (size_t)row * ldy + n;
      if (y_f32) reinterpret_cast<float*>(Y)[off] = sum;
      else reinterpret_cast<_Float16*>(Y)[off] = (_Float16)sum;
    }
  }
}

template <int K>
hipError_t launch_tiny(const vq_desc& d, const void* idx_dev, const void* cb_dev, const void* X,
                       int B, int ldx, void* Y, int ldy, int y_f32, hipStream_t s) {
  const int n_rb = d.out_features / kGroupRows, n_cb = d.in_features / kGroupCols;
  const dim3 grid((unsigned)((n_rb + 1) / 2), (unsigned)((B + 15) / 16));
  hipLaunchKernelGGL((gemm_tiny_kernel<K>), grid, dim3(256), 0, s, (const uint8_t*)idx_dev,
                     (const uint32_t*)cb_dev, (const uint16_t*)X, B, ldx, Y, ldy, y_f32, n_rb, n_cb, d.group_rows / kGroupRows);
  return hipGetLastError();
}

// ---- small batches (B <= 32): bandwidth-bound ---------------------------------
// 32 rows x 32 batch columns per workgroup (many workgroups, so that every CU streams
// weights); the whole col-block of X is staged at once and wave w multiplies its own
// quarter of k; the four partial tiles meet in LDS at the end.  W tile and X tile are
// double-buffered: decoding col-block c+1 overlaps the MFMAs of col-block c and one
// barrier per col-block is enough.
template <int K>
__global__ __launch_bounds__(256, 2) void gemm_small_kernel(const uint8_t* __restrict__ idx,
                                                            const uint32_t* __restrict__ cb,
                                                            const uint16_t* __restrict__ X, int B,
                                                            int ldx, void* __restrict__ Y, int ldy,
                                                            int y_f32, int n_rb, int n_cb,
                                                            int n_tiles_n, int rpc) {
  constexpr int MT = 32, NT = 32;
  __shared__ __attribute__((aligned(16))) uint16_t Wt_all[2][MT * WS];
  // X tile [256 k][32 n] halfs as in memory; the 32-byte chunk c of row k sits at c ^ ((k >> 1) & 1),
  // which puts the four rows of a transposing read into four different bank groups
  __shared__ __attribute__((aligned(16))) uint32_t Xs_all[2][4096];
  __shared__ __attribute__((aligned(16))) uint32_t lut_all[4][lut_dwords<K>()];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int mt = blockIdx.x / n_tiles_n;
  const int nt = blockIdx.x - mt * n_tiles_n;
  uint32_t* lut = lut_all[wave];

  // X staging role: the col-block's tile is copied unchanged in 4 passes of 64 rows; the thread
  // owns 16 bytes (8 batch columns from n_loc) of row x_row of every pass.  A piece that lies
  // beyond the row (ldx) is not loaded; columns between B and ldx only reach accumulator
  // columns that are never written.
  const int x_row = tid >> 2;
  const int n_loc = (tid & 3) * 8;
  const int n_glob = nt * NT + n_loc;
  const bool x_ok = n_glob + 8 <= ldx;
  const size_t x_lane = (size_t)x_row * ldx + (x_ok ? n_glob : 0);
  const int xs_off = x_row * 64 + ((((n_loc >> 4) ^ ((x_row >> 1) & 1)) << 5) | ((n_loc & 8) << 1));   // bytes
  // operand role (ds_read_b64_tr_b16): lane i of a 16-lane block addresses row i / 4, fragment
  // i % 4 of a 4 x 16 tile and receives column i; rows 8 * (lane / 32) + 0..7 of a 16-deep step
  const int xr_kq = (lane & 15) >> 2;
  const int xr_off = (8 * (lane >> 5) + xr_kq) * 64 + (((((lane >> 4) & 1) ^ ((xr_kq >> 1) & 1))) << 5) + (lane & 3) * 8;

  f16v_t acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  const long long rb = (long long)mt * 4 + wave;
  const bool rb_ok = rb < n_rb;
  const long long rb_ld = rb_ok ? rb : 0;
  const int m0 = wave * 8;

  // Few workgroups are resident per CU here, so memory latency is hidden by depth
  // instead: a ring of D col-blocks (indices, codebook and the X piece) is kept in
  // flight in registers.  Loads are unconditional (clamped to the last col-block) so
  // that the compiler can count them and wait only for the oldest.
#define VQ_LOAD_X(j, c)                                                                         \
  _Pragma("unroll") for (int pass = 0; pass < 4; ++pass)                                        \
    xp[j].r[pass] = *reinterpret_cast<const u32x4_t*>(X + ((size_t)(c) * 256 + 64 * pass) * ldx + x_lane);
  constexpr int D = 4;
  GroupRegs<K> g[D];
  XRows xp[D];
#pragma unroll
  for (int j = 0; j < D; ++j) {
    const int cj = min(j, n_cb - 1);
    load_group<K>(g[j], idx, cb, rb_ld, cj, n_cb, lane, n_rb, rpc);
    VQ_LOAD_X(j, cj)
  }

  // Ring slot j (col-block c) -> LDS buffer j & 1 (D is even); with REFILL the slot is
  // then reloaded with col-block c + D.  Everything that loads is branch-free: col-blocks
  // past the end are clamped reads whose tiles are staged but never multiplied.
#define VQ_STAGE(j, c, REFILL)                                                                  \
  {                                                                                             \
    uint16_t* Wt_w = Wt_all[(j) & 1];                                                           \
    if (rb_ok) {                                                                                \
      decode_group<K>(g[j], lut, Wt_w, m0, lane);                                               \
    } else {                                                                                    \
      _Pragma("unroll") for (int r = 0; r < 8; ++r)                                             \
          *reinterpret_cast<uint2*>(Wt_w + wt_half_index(m0 + r, 4 * lane)) = make_uint2(0u, 0u); \
    }                                                                                           \
    _Pragma("unroll") for (int pass = 0; pass < 4; ++pass)                                      \
      *reinterpret_cast<u32x4_t*>(reinterpret_cast<char*>(Xs_all[(j) & 1]) + 4096 * pass + xs_off) = \
          x_ok ? xp[j].r[pass] : u32x4_t{0u, 0u, 0u, 0u};                                       \
    if (REFILL) {                                                                               \
      const int cn = min((c) + D, n_cb - 1);                                                    \
      load_group<K>(g[j], idx, cb, rb_ld, cn, n_cb, lane, n_rb, rpc);                           \
      VQ_LOAD_X(j, cn)                                                                          \
    }                                                                                           \
  }
  // multiply col-block c (staged in buffer j & 1) if it exists, then release the buffer
#define VQ_MULTIPLY(j, c)                                                                       \
  {                                                                                             \
    if ((c) < n_cb) {                                                                           \
      const uint16_t* Wt = Wt_all[(j) & 1];                                                     \
      const char* Xs = reinterpret_cast<const char*>(Xs_all[(j) & 1]);                          \
      _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                        \
        const int k16 = wave * 4 + kk;                                                          \
        const h8_t bv = read_x_operand<NT>(Xs + 1024 * k16 + xr_off);                           \
        const h8_t av = *reinterpret_cast<const h8_t*>(                                         \
            Wt + wt_half_index(lane & 31, 16 * k16 + 8 * (lane >> 5)));                         \
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc, 0, 0, 0);                     \
      }                                                                                         \
    }                                                                                           \
    __syncthreads();                                                                            \
  }

  const int n_pad = (n_cb + D - 1) / D * D;
  VQ_STAGE(0, 0, true)
  __syncthreads();
  int c0 = 0;
  for (; c0 + D < n_pad; c0 += D) {
    VQ_STAGE(1, c0 + 1, true) VQ_MULTIPLY(0, c0)
    VQ_STAGE(2, c0 + 2, true) VQ_MULTIPLY(1, c0 + 1)
    VQ_STAGE(3, c0 + 3, true) VQ_MULTIPLY(2, c0 + 2)
    VQ_STAGE(0, c0 + 4, true) VQ_MULTIPLY(3, c0 + 3)
  }
  VQ_STAGE(1, c0 + 1, false) VQ_MULTIPLY(0, c0)
  VQ_STAGE(2, c0 + 2, false) VQ_MULTIPLY(1, c0 + 1)
  VQ_STAGE(3, c0 + 3, false) VQ_MULTIPLY(2, c0 + 2)
  VQ_MULTIPLY(3, c0 + 3)
#undef VQ_STAGE
#undef VQ_MULTIPLY
#undef VQ_LOAD_X
  static_assert(D == 4, "the unrolled ring above is written for four slots");

  // four partial 32 x 32 tiles (one per wave) -> LDS -> sum -> Y
  float* part = reinterpret_cast<float*>(Wt_all[0]);      // 4 x 32 x 32 floats = 16 KB
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int m = 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
    part[(wave * MT + m) * 32 + (lane & 31)] = acc[i];
  }
  __syncthreads();
  for (int e = tid; e < MT * 32; e += 256) {
    const int m = e >> 5, nl = e & 31;
    const float sum = part[e] + part[MT * 32 + e] + part[2 * MT * 32 + e] + part[3 * MT * 32 + e];
    const int row = mt * MT + m, n = nt * NT + nl;
    if (row < n_rb * 8 && n < B) {
      const size_t o = (size_t)row * ldy + n;
      if (y_f32) reinterpret_cast<float*>(Y)[o] = sum;
      else reinterpret_cast<_Float16*>(Y)[o] = (_Float16)sum;
    }
  }
}

template <int K>
hipError_t launch_small(const vq_desc& d, const void* idx_dev, const void* cb_dev, const void* X,
                        int B, int ldx, void* Y, int ldy, int y_f32, hipStream_t s) {
  const int n_rb = d.out_features / kGroupRows, n_cb = d.in_features / kGroupCols;
  const int tiles_m = (n_rb + 3) / 4, tiles_n = (B + 31) / 32;
  hipLaunchKernelGGL((gemm_small_kernel<K>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, s,
                     (const uint8_t*)idx_dev, (const uint32_t*)cb_dev, (const uint16_t*)X, B, ldx, Y,
                     ldy, y_f32, n_rb, n_cb, tiles_n, d.group_rows / kGroupRows);
  return hipGetLastError();
}

// Row-blocks [rb0, rb_end) of the matrix (rb_end < 0: all of it).
template <int K, int RBW, int NT, int WM = 1>
hipError_t launch_one(const vq_desc& d, const void* idx_dev, const void* cb_dev, const void* X, int B,
                      int ldx, void* Y, int ldy, int y_f32, hipStream_t s, int rb0 = 0, int rb_end = -1) {
  const int n_rb = d.out_features / kGroupRows, n_cb = d.in_features / kGroupCols;
  if (rb_end < 0) rb_end = n_rb;
  const int tiles_m = (rb_end - rb0 + 4 * RBW * WM - 1) / (4 * RBW * WM), tiles_n = (B + NT - 1) / NT;
  hipLaunchKernelGGL((gemm_kernel<K, RBW, NT, WM>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256 * WM), 0, s,
                     (const uint8_t*)idx_dev, (const uint32_t*)cb_dev, (const uint16_t*)X, B, ldx, Y,
                     ldy, y_f32, n_rb, n_cb, tiles_n, d.group_rows / kGroupRows, rb0, rb_end);
  return hipGetLastError();
}

// Compute units of the current device: the 8-wave tiles run one workgroup per CU, so their time
// moves in whole rounds of that many tiles.  Asked once per device, then cached.
int device_cus() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  int cus = cached[dev].load(std::memory_order_relaxed);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
      (void)hipGetLastError();
      return 256;
    }
    cached[dev].store(cus, std::memory_order_relaxed);
  }
  return cus;
}

// Large batches on the 128-row tiles: 128 x 512 tiles decode W once per 512 batch columns instead
// of once per 256 and take 1.73 times as long as 128 x 256 tiles for twice the area, but a launch
// pays for whole rounds of one workgroup per CU.  So the first m_a tile rows run with 512-column
// tiles and the rest with 256-column tiles in a second launch, m_a chosen so that both launches
// fill their rounds best (m_a = 0: 256-column tiles only).  Same units as launch_gemm's estimates:
// microseconds at in_features = 4096, scaled by kscale = in_features / 4096 (a tile's time is its
// K loop); the 3 us of the second launch do not scale.
template <int K>
hipError_t launch_wide(const vq_desc& d, const void* idx_dev, const void* cb_dev, const void* X, int B,
                       int ldx, void* Y, int ldy, int y_f32, hipStream_t s) {
  // the 512-column tile needs 128 accumulator registers per wave: most formats fit the 256
  // registers or spill up to four of them; the block-normalised ones would spill seven to ten and
  // keep 256 columns
  if constexpr (K == kFmtK64BN || K == kFmtK16BN || K == kFmtD1K8BN || K == kFmtD4BN || K == kFmtK256I8BN) {
    return launch_one<K, 2, 256, 2>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);
  } else {
  const int n_rb = d.out_features / kGroupRows;
  const long long rows128 = (n_rb + 15) / 16, cols256 = (B + 255) / 256, cols512 = (B + 511) / 512;
  int m_a = 0;
  const long long cus = device_cus();
  const double kscale = (double)d.in_features / 4096.0;
  double best = 79.0 * kscale * (double)((rows128 * cols256 + cus - 1) / cus);
  for (long long m = 1; m <= rows128; ++m) {
    const long long rest = rows128 - m;
    const double t = 137.0 * kscale * (double)((m * cols512 + cus - 1) / cus) +
                     (rest > 0 ? 3.0 + 79.0 * kscale * (double)((rest * cols256 + cus - 1) / cus) : 0.0);
    if (t < best) {
      best = t;
      m_a = (int)m;
    }
  }
  if (m_a == 0) return launch_one<K, 2, 256, 2>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);
  const int rb_split = m_a * 16 < n_rb ? m_a * 16 : n_rb;
  hipError_t e = launch_one<K, 2, 512, 2>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s, 0, rb_split);
  if (e != hipSuccess || rb_split == n_rb) return e;
  return launch_one<K, 2, 256, 2>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s, rb_split, n_rb);
  }
}

}  // namespace

hipError_t launch_gemm(const vq_desc& d, const void* idx_dev, const void* cb_dev, const void* X,
                       int B, int ldx, void* Y, int ldy, int y_f32, hipStream_t s) {
  // B <= 16: 16 x 16 tiles, barrier-free (gemm_tiny_kernel).  It re-decodes W once per 16
  // columns, which still pays at 32 columns when the matrix is too short to fill the CUs
  // with the 32-row tiles of the other kernels (4096 x 4096 at B = 48 / 64: 15.0 / 22.5 us with
  // it, 13.7 / 13.9 us with the 32 x 32 tiles).  Then 32 x 32 tiles (gemm_small_kernel,
  // bandwidth-bound) while they are few enough to run in about one wave of workgroups, then
  // gemm_kernel with 32 x 128 tiles while those fit the CUs once, and beyond that the cheapest
  // of four tilings by a small cost model: 64 x 128 and 64 x 256 (4 waves, two workgroups per
  // CU: time grows almost linearly with the tile count) and 128 x 128 and 128 x 256 (8 waves, one
  // workgroup per CU: half the X traffic per product, but time moves in whole rounds of 256
  // one tile per CU).  The constants are microseconds measured at in_features = 4096 on 4096- and
  // 11008-row matrices, B = 512..4096, on 256 CUs.  A tile's time is its K loop, so every term
  // scales with in_features and only the ratios matter here; the 4-wave tiles run two per CU, so
  // their per-tile slope scales with 256 / CUs.
  const int n_rb = d.out_features / kGroupRows;
  const bool short_matrix = n_rb < 1024;
  const bool tiny = B <= 16 || (B <= 32 && short_matrix);
  const long long tiles_small = (long long)((n_rb + 3) / 4) * ((B + 31) / 32);
  const long long rows64 = (n_rb + 7) / 8, rows128 = (n_rb + 15) / 16;
  const long long cols128 = (B + 127) / 128, cols256 = (B + 255) / 256;
  const long long cus = device_cus();
  const bool small = B <= 32 || tiles_small <= 3 * cus;
  const bool one_round_32x128 = rows64 * cols128 <= cus / 2;
  const double per_cu = 256.0 / (double)cus;
  const double est[4] = {20.0 + 0.11 * per_cu * (double)(rows64 * cols128),              // 64 x 128
                         35.0 + 0.165 * per_cu * (double)(rows64 * cols256),             // 64 x 256
                         54.0 * (double)((rows128 * cols128 + cus - 1) / cus),           // 128 x 128
                         79.0 * (double)((rows128 * cols256 + cus - 1) / cus)};          // 128 x 256
  int best = 0;
  for (int i = 1; i < 4; ++i)
    if (est[i] < est[best]) best = i;
#define VQ_GEMM_DISPATCH(K)                                                                       \
  {                                                                                               \
    if (tiny) return launch_tiny<K>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);             \
    if (small) return launch_small<K>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);           \
    if (one_round_32x128)                                                                         \
      return launch_one<K, 1, 128>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);              \
    if (best == 0) return launch_one<K, 2, 128>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s); \
    if (best == 1) return launch_one<K, 2, 256>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s); \
    if (best == 2)                                                                                \
      return launch_one<K, 2, 128, 2>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);           \
    return launch_wide<K>(d, idx_dev, cb_dev, X, B, ldx, Y, ldy, y_f32, s);                       \
  }
  const int fmt = format_tag(d);
  if (fmt == 64) VQ_GEMM_DISPATCH(64)
  if (fmt == kFmtK16I8) VQ_GEMM_DISPATCH(kFmtK16I8)
  if (fmt == kFmtK16BN) VQ_GEMM_DISPATCH(kFmtK16BN)
  if (fmt == kFmtD1K16) VQ_GEMM_DISPATCH(kFmtD1K16)
  if (fmt == kFmtK64BN) VQ_GEMM_DISPATCH(kFmtK64BN)
  if (fmt == kFmtD4) VQ_GEMM_DISPATCH(kFmtD4)
  if (fmt == kFmtK16I8H) VQ_GEMM_DISPATCH(kFmtK16I8H)
  if (fmt == kFmtK32) VQ_GEMM_DISPATCH(kFmtK32)
  if (fmt == kFmtD4F16) VQ_GEMM_DISPATCH(kFmtD4F16)
  if (fmt == kFmtD4BN) VQ_GEMM_DISPATCH(kFmtD4BN)
  if (fmt == kFmtK256I8BN) VQ_GEMM_DISPATCH(kFmtK256I8BN)
  if (fmt == kFmtD1K8) VQ_GEMM_DISPATCH(kFmtD1K8)
  if (fmt == kFmtD1K8BN) VQ_GEMM_DISPATCH(kFmtD1K8BN)
  if (fmt == kFmtD1K4) VQ_GEMM_DISPATCH(kFmtD1K4)
  if (fmt == kFmtK256I8) VQ_GEMM_DISPATCH(kFmtK256I8)
  if (fmt == 16) VQ_GEMM_DISPATCH(16)
  VQ_GEMM_DISPATCH(256)
#undef VQ_GEMM_DISPATCH
}

}  // namespace vq
