// Kernels of the batch-1 product y = W x on vector-quantised W, shared by the two translation
// units that instantiate them: without (vq_gemv.hip) and with (vq_gemv_lora.hip) the low-rank
// adapter epilogue.  See vq_gemv.hip for the work decomposition.
#pragma once
#include <atomic>
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

// A strip as wave-uniform scalars.  Units are col-block pairs (k=16, scalar 2-bit), quads (6-bit
// fields) or col-blocks (k=256).
struct Strip {
  const uint8_t* idx_rb;   // indices of the row-block
  const uint32_t* cb_rb;   // codebooks / int8 tables of the row-block (dwords)
  const uint16_t* sc_rb;   // fp16 scales of the row-block's groups (k=16 with int8 tables)
  const uint8_t* codes_rb; // 4-bit block codes of the row-block (blockwise normalisation)
  const uint8_t* lev_rb;   // fp16 block-scale levels of the row-block's groups (k=16 with blockwise normalisation)
  const uint16_t* x;
  int u;                   // next unit to load
  int u_end;               // end of this strip's units
  int chunks_left;         // chunks still to load
  int n_cb;                // col-blocks of the matrix (k=16: the pad group has no activations)
};

// Every chunk issues the same loads whatever its shape: absent units read a harmless
// in-bounds address.  The loads of one chunk overlap the consumption of the other, and
// the compiler can only keep a partial vmcnt wait (instead of waiting for every
// outstanding load) if the number of loads in flight is static.  For k=16 absent units
// are also *consumed*: their table and activations are zero, so they add exactly 0 and
// the consume step has no branches (branches around the inline-asm blocks cost register
// copies of all 8 accumulators at every merge).
__device__ __forceinline__ uint2 zero_unless(bool keep, uint2 v) {
  return keep ? v : make_uint2(0, 0);
}
__device__ __forceinline__ uint32_t zero_unless(bool keep, uint32_t v) { return keep ? v : 0u; }
__device__ __forceinline__ uint4 zero_unless(bool keep, uint4 v) {
  return keep ? v : make_uint4(0, 0, 0, 0);
}
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// Streaming (non-temporal) 16-byte load: index and codebook bytes are used exactly once.
__device__ __forceinline__ uint4 stream_load16(const void* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// ---- chunks with activations in registers (split-K kernel) ------------------
template <int K> struct Chunk;

// k = 16.  MODE 1 (I8): the tables are int8 with a scale per group (32 + 2 bytes per group instead
// of 64), dequantised into the LDS table when the chunk is consumed.  MODE 2 (BN): blockwise
// normalisation on top (16 block-scale levels per group next to the tables in LDS, a 4-bit code
// per 32 weights); the plain C++ inner block replaces the hand-scheduled one.
// MODE 3 (H4): int8 tables for groups of 4 rows: two tables per 8-row block and col-block (rows
// 0..3, rows 4..7), 64 + 4 bytes per slot; the hand-scheduled block reads rows 4..7 from the second.
// MODE 4 (K32): k = 32, 5-bit indices: 64 bytes of int8 table per group (staged like the two tables
// of a 4-row-group slot) and a plane of fifth bits next to the nibbles (one dword per lane and pair).
template <int MODE> struct Chunk16T {
  static constexpr bool I8 = MODE >= 1, BN = MODE == 2, K32 = MODE == 4, H4 = MODE == 3 || K32;   // H4: 64 bytes of tables per slot
  static constexpr int kUnits = 4;        // col-block pairs per chunk
  static constexpr int kLutDwords = (BN || H4) ? 256 : 128;  // 8 groups x 16 centroids (+ 8 x 16 levels, or x 2 tables)
  uint4 ev;       // K32: the lane's fifth-bit plane dwords of pairs u .. u+3
  uint4 w[4];     // slot s: the lane's 16 index bytes of pair u+s
  uint2 xa[4];    // activations of the first group of the slot
  uint2 xb[4];    // ... and of the second
  uint4 cbv;      // fp16: this lane's 16 bytes of the chunk's codebooks (lanes 0..31)
  uint32_t tab;   // int8: this lane's two centroid pairs (4 bytes of the chunk's tables)
  uint32_t tab2;  // H4: two more (the lane holds 8 bytes of the chunk's 512 bytes of tables)
  uint32_t sc;    // int8: the fp16 scale of the group those pairs belong to
  uint2 cw[4];    // BN: the lane's block codes of the two groups of pair u+s
  uint32_t lev;   // BN: levels 2*(lane%8), +1 of group lane/8 of the chunk (two fp16)
  int np;         // pairs present (wave-uniform)

  // The chunk's tables: pairs u .. u+np-1 of the row-block (np may be 0: nothing is kept).
  __device__ __forceinline__ void load_tables(const Strip& S, int u, int lane, int np_) {
    const int u_ld = np_ > 0 ? u : 0;
    if constexpr (H4) {
      const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)u_ld * 128;
      const uint2 t2 = zero_unless(lane * 8 < np_ * 128,
                                   *reinterpret_cast<const uint2*>(tq + min(lane * 8, max(np_ * 128 - 8, 0))));
      tab = t2.x;
      tab2 = t2.y;
      sc = K32 ? S.sc_rb[u_ld * 2 + min(lane >> 3, max(2 * np_ - 1, 0))]     // one scale per 64-byte table
               : S.sc_rb[u_ld * 4 + min(lane >> 2, max(4 * np_ - 1, 0))];
    } else if constexpr (I8) {
      const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)u_ld * 64;
      tab = zero_unless(lane * 4 < np_ * 64,
                        *reinterpret_cast<const uint32_t*>(tq + min(lane * 4, max(np_ * 64 - 4, 0))));
      sc = S.sc_rb[u_ld * 2 + min(lane >> 3, max(2 * np_ - 1, 0))];
      if constexpr (BN)
        lev = zero_unless(lane * 4 < np_ * 64,
                          *reinterpret_cast<const uint32_t*>(S.lev_rb + (size_t)u_ld * 64 + min(lane * 4, max(np_ * 64 - 4, 0))));
    } else {
      const int cb_off = min(lane * 4, max(np_ * 32 - 4, 0));
      cbv = zero_unless(lane * 4 < np_ * 32, stream_load16(S.cb_rb + (size_t)u_ld * 32 + cb_off));
    }
  }
  __device__ __forceinline__ void stage_tables(uint32_t* lut, int lane) const {
    if constexpr (H4) {
      const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(tab, scale), k64_dequant_pair(tab >> 16, scale),
                     k64_dequant_pair(tab2, scale), k64_dequant_pair(tab2 >> 16, scale));
    } else if constexpr (I8) {
      const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
      *reinterpret_cast<uint2*>(lut + lane * 2) =
          make_uint2(k64_dequant_pair(tab, scale), k64_dequant_pair(tab >> 16, scale));
      if constexpr (BN)   // each level as a dword with the fp16 value in both halves
        *reinterpret_cast<uint2*>(lut + 128 + lane * 2) = make_uint2((lev & 0xffffu) * 0x10001u, (lev >> 16) * 0x10001u);
    } else {
      if (lane < 32) *reinterpret_cast<uint4*>(lut + lane * 4) = cbv;
    }
  }

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    np = max(0, min(4, S.u_end - u));
    load_tables(S, u, lane, np);
    if constexpr (K32) {
      uint32_t e[4];
#pragma unroll
      for (int s = 0; s < 4; ++s)
        e[s] = *reinterpret_cast<const uint32_t*>(S.codes_rb + (size_t)(s < np ? u + s : 0) * 256 + lane * 4);
      ev = make_uint4(e[0], e[1], e[2], e[3]);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const bool ok = s < np;
      const int q = ok ? u + s : 0;                              // pair 0 always exists
      const bool ok_b = ok && 2 * q + 1 < S.n_cb;                // the pad group has no x
      w[s] = stream_load16(S.idx_rb + (size_t)q * 1024 + lane * 16);
      if constexpr (BN) cw[s] = *reinterpret_cast<const uint2*>(S.codes_rb + (size_t)q * 64 + (lane >> 3) * 8);
      xa[s] = zero_unless(ok, *reinterpret_cast<const uint2*>(S.x + (2 * q) * 256 + lane * 4));
      xb[s] = zero_unless(ok_b, *reinterpret_cast<const uint2*>(S.x + (ok_b ? 2 * q + 1 : 0) * 256 + lane * 4));
    }
  }

  // Stages the codebooks in this wave's table region (`lut`, LDS byte address `base`)
  // and consumes the chunk.
  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, int lane,
                                          float (&acc)[8]) const {
    stage_tables(lut, lane);
    wave_lds_sync();
    if constexpr (BN) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (s == 2 && np <= 2) break;      // short strips of a finely split row-block: half the work
        k16_group_scaled(w[s].x, w[s].y, cw[s].x, lut + 32 * s, lut + 128 + 32 * s, xa[s].x, xa[s].y, acc);
        k16_group_scaled(w[s].z, w[s].w, cw[s].y, lut + 32 * s + 16, lut + 128 + 32 * s + 16, xb[s].x, xb[s].y, acc);
      }
      return;
    }
    if constexpr (K32) {
      const uint32_t es[4] = {ev.x, ev.y, ev.z, ev.w};
      const uint32_t hb = 0x40404040u;
#define VQ_K32(S, OFFA)                                                                                     \
      {                                                                                                     \
        uint32_t e0, e1, e2, e3;                                                                            \
        k32_plane_sets<0>(es[S], e0, e1, e2, e3);                                                           \
        k32_group<OFFA>(w[S].x, w[S].y, e0, e1, e2, e3, hb, base, xa[S].x, xa[S].y, acc);                   \
        k32_plane_sets<1>(es[S], e0, e1, e2, e3);                                                           \
        k32_group<OFFA + 128>(w[S].z, w[S].w, e0, e1, e2, e3, hb, base, xb[S].x, xb[S].y, acc);             \
      }
      VQ_K32(0, 0) VQ_K32(1, 256)
      acc_hazard_fence();
      if (np <= 2) return;
      VQ_K32(2, 512) VQ_K32(3, 768)
#undef VQ_K32
      acc_hazard_fence();
      return;
    }
    constexpr int T = H4 ? 128 : 64, HS = H4 ? 64 : 0;   // bytes of tables per group slot; rows 4..7
    k16_group<0, 0, HS>(w[0].x, w[0].y, base, xa[0].x, xa[0].y, acc);
    k16_group<T, 0, HS>(w[0].z, w[0].w, base, xb[0].x, xb[0].y, acc);
    k16_group<2 * T, 0, HS>(w[1].x, w[1].y, base, xa[1].x, xa[1].y, acc);
    k16_group<3 * T, 0, HS>(w[1].z, w[1].w, base, xb[1].x, xb[1].y, acc);
    acc_hazard_fence();       // before the branch: the compiler may copy accumulators at it
    if (np <= 2) return;      // short strips of a finely split row-block: half the work
    k16_group<4 * T, 0, HS>(w[2].x, w[2].y, base, xa[2].x, xa[2].y, acc);
    k16_group<5 * T, 0, HS>(w[2].z, w[2].w, base, xb[2].x, xb[2].y, acc);
    k16_group<6 * T, 0, HS>(w[3].x, w[3].y, base, xa[3].x, xa[3].y, acc);
    k16_group<7 * T, 0, HS>(w[3].z, w[3].w, base, xb[3].x, xb[3].y, acc);
    acc_hazard_fence();
  }
};
template <> struct Chunk<16> : Chunk16T<0> {};
template <> struct Chunk<kFmtK16I8H> : Chunk16T<3> {};
template <> struct Chunk<kFmtK32> : Chunk16T<4> {};
template <> struct Chunk<kFmtK16I8> : Chunk16T<1> {};
template <> struct Chunk<kFmtK16BN> : Chunk16T<2> {};

// d = 1, k = 4 (2-bit indices, a codebook per row of a col-block): the index bytes and the inner
// block of k = 16, with a 16-entry pair table per row.  A chunk is 2 col-block pairs = 4 blocks of
// 8 rows x 256 columns; lane L builds entries 8*(L&1) .. +7 of the table of (block, row) = L >> 1.
template <> struct Chunk<kFmtD1K4> {
  static constexpr int kUnits = 2;
  static constexpr int kLutDwords = 512;   // 4 blocks x 8 rows x 16 entries
  uint4 w[2];
  uint2 xa[2], xb[2];
  uint32_t tab;   // the 4 int8 values of (block, row) = lane >> 1
  uint32_t sc;    // ... and its fp16 scale
  int np;

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    np = max(0, min(2, S.u_end - u));
    const int u_ld = np > 0 ? u : 0;
    const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)u_ld * (2 * kD1K4SlotTabBytes);
    const int blk = min(lane >> 4, max(2 * np - 1, 0)), row = (lane >> 1) & 7;
    const bool ok = (lane >> 4) < 2 * np;
    tab = zero_unless(ok, *reinterpret_cast<const uint32_t*>(tq + blk * kD1K4SlotTabBytes + row * 4));
    sc = zero_unless(ok, (uint32_t)*reinterpret_cast<const uint16_t*>(tq + blk * kD1K4SlotTabBytes + kD1K4ScaleOffset + row * 2));
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const bool oks = s < np;
      const int q = oks ? u + s : 0;
      const bool ok_b = oks && 2 * q + 1 < S.n_cb;
      w[s] = stream_load16(S.idx_rb + (size_t)q * 1024 + lane * 16);
      xa[s] = zero_unless(oks, *reinterpret_cast<const uint2*>(S.x + (2 * q) * 256 + lane * 4));
      xb[s] = zero_unless(ok_b, *reinterpret_cast<const uint2*>(S.x + (ok_b ? 2 * q + 1 : 0) * 256 + lane * 4));
    }
  }

  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, int lane, float (&acc)[8]) const {
    const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
    uint4 e0, e1;
    d1k4_entries(k64_dequant_pair(tab, scale), k64_dequant_pair(tab >> 16, scale), lane & 1, e0, e1);
    *reinterpret_cast<uint4*>(lut + lane * 8) = e0;
    *reinterpret_cast<uint4*>(lut + lane * 8 + 4) = e1;
    wave_lds_sync();
    k16_group<0, 64>(w[0].x, w[0].y, base, xa[0].x, xa[0].y, acc);
    k16_group<512, 64>(w[0].z, w[0].w, base, xb[0].x, xb[0].y, acc);
    k16_group<1024, 64>(w[1].x, w[1].y, base, xa[1].x, xa[1].y, acc);
    k16_group<1536, 64>(w[1].z, w[1].w, base, xb[1].x, xb[1].y, acc);
    acc_hazard_fence();
  }
};

// k = 256 (D1 = false), and d = 1 with k = 16 (D1 = true): the same index bytes and inner
// block; D1 builds the 256-entry pair table from the group's 16 scalars instead of loading it.
template <bool D1> struct Chunk256T {
  static constexpr int kUnits = 2;        // groups per chunk
  static constexpr int kLutDwords = 512;  // 2 groups x 256 table entries
  uint4 w[2];     // the lane's 16 index bytes of group u+s
  uint2 xv[2];    // its activations
  uint4 cbv[2];   // k = 256: the lane's 16 bytes of the group's codebook
  uint2 clo[2];   // d = 1: scalars 4*(lane%4) .. +3 of the group
  uint32_t chi[2];   // d = 1: scalar lane/4

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const bool ok = u + s < S.u_end;
      const int c = ok ? u + s : 0;
      w[s] = stream_load16(S.idx_rb + (size_t)c * 1024 + lane * 16);
      if constexpr (D1) {
        const uint8_t* cg = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)c * 32;
        clo[s] = zero_unless(ok, *reinterpret_cast<const uint2*>(cg + (lane & 3) * 8));
        chi[s] = zero_unless(ok, (uint32_t)*reinterpret_cast<const uint16_t*>(cg + (lane >> 2) * 2));
      } else {
        cbv[s] = zero_unless(ok, stream_load16(S.cb_rb + (size_t)c * 256 + lane * 4));
      }
      xv[s] = zero_unless(ok, *reinterpret_cast<const uint2*>(S.x + c * 256 + lane * 4));
    }
  }

  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, int lane,
                                          float (&acc)[8]) const {
    *reinterpret_cast<uint4*>(lut + lane * 4) = D1 ? d1_pair_entries(clo[0], chi[0]) : cbv[0];
    *reinterpret_cast<uint4*>(lut + 256 + lane * 4) = D1 ? d1_pair_entries(clo[1], chi[1]) : cbv[1];
    wave_lds_sync();
    k256_group<0>(w[0].x, w[0].y, w[0].z, w[0].w, base, xv[0].x, xv[0].y, acc);
    k256_group<1024>(w[1].x, w[1].y, w[1].z, w[1].w, base, xv[1].x, xv[1].y, acc);
    acc_hazard_fence();
  }
};
template <> struct Chunk<256> : Chunk256T<false> {};
template <> struct Chunk<kFmtD1K16> : Chunk256T<true> {};

// k = 64 with int8 tables.  BN: blockwise normalisation on top (16 block-scale levels per
// group, a 4-bit code per 32 weights); the plain C++ inner block replaces the hand-scheduled one.
// MODE 2: d = 1, k = 8: the 64-entry pair table is built from the group's 8 int8 values; MODE 3:
// the same with blockwise normalisation.
template <int MODE> struct Chunk64T {
  static constexpr bool BN = MODE == 1 || MODE == 3, D1 = MODE >= 2;
  static constexpr int kUnits = 1;        // quads of 4 col-blocks per chunk
  static constexpr int kLutDwords = BN ? 320 : 256;  // 4 groups x 64 centroids (+ 4 x 16 levels)
  static constexpr int kTabBytes = D1 ? (BN ? kD1K8NQuadTabBytes : kD1K8QuadTabBytes) : BN ? kK64NQuadTabBytes : kK64QuadTabBytes;
  static constexpr int kScaleOffset = D1 ? kD1K8ScaleOffset : 512;
  static constexpr int kLevelOffset = D1 ? kD1K8NLevelOffset : kK64NLevelOffset;
  uint4 w[3];     // the lane's three index planes of the quad
  uint2 xv[4];    // activations of the quad's four col-blocks
  uint2 tab;      // 4 int8 centroid pairs: entries 4*(lane%16).. of table lane/16
  uint32_t sc;    // that table's fp16 scale (low 16 bits)
  uint4 cw;       // BN: the lane's block codes, one dword per col-block
  uint32_t lev;   // BN: level lane%16 of col-block lane/16 (fp16)

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    const bool ok = u < S.u_end;
    const int q = ok ? u : 0;
    const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)q * kTabBytes;
    tab = zero_unless(ok, *reinterpret_cast<const uint2*>(tq + (D1 ? (lane >> 4) * 8 : lane * 8)));
    sc = *reinterpret_cast<const uint16_t*>(tq + kScaleOffset + (lane >> 4) * 2);
    if constexpr (BN) {
      lev = zero_unless(ok, (uint32_t)*reinterpret_cast<const uint16_t*>(tq + kLevelOffset + lane * 2));
      cw = *reinterpret_cast<const uint4*>(S.codes_rb + (size_t)q * kK64NQuadCodeBytes + (lane >> 3) * 16);
    }
#pragma unroll
    for (int p = 0; p < 3; ++p)
      w[p] = stream_load16(S.idx_rb + (size_t)q * kK64QuadIdxBytes + p * 1024 + lane * 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool okx = ok && 4 * q + j < S.n_cb;
      xv[j] = zero_unless(okx, *reinterpret_cast<const uint2*>(S.x + (okx ? 4 * q + j : 0) * 256 + lane * 4));
    }
  }

  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, int lane,
                                          float (&acc)[8]) const {
    const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
    if constexpr (D1) {
      const int e = 4 * (lane & 15);
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(d1k8_pair(tab, e), scale), k64_dequant_pair(d1k8_pair(tab, e + 1), scale),
                     k64_dequant_pair(d1k8_pair(tab, e + 2), scale), k64_dequant_pair(d1k8_pair(tab, e + 3), scale));
    } else {
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(tab.x, scale), k64_dequant_pair(tab.x >> 16, scale),
                     k64_dequant_pair(tab.y, scale), k64_dequant_pair(tab.y >> 16, scale));
    }
    if constexpr (BN) lut[256 + lane] = lev * 0x10001u;   // the level in both halves
    wave_lds_sync();
    const uint32_t d[12] = {w[0].x, w[0].y, w[0].z, w[0].w, w[1].x, w[1].y,
                            w[1].z, w[1].w, w[2].x, w[2].y, w[2].z, w[2].w};
    if constexpr (BN) {
      const uint32_t cws[4] = {cw.x, cw.y, cw.z, cw.w};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        k64_group_scaled(d[3 * j], d[3 * j + 1], d[3 * j + 2], cws[j], lut + 64 * j, lut + 256 + 16 * j,
                         xv[j].x, xv[j].y, acc);
    } else {
#define VQ_G64(J)                                                                              \
      k64_group<256 * J>(d[3 * J], d[3 * J + 1], d[3 * J + 2],                                 \
                         __builtin_amdgcn_alignbit(d[3 * J + 1], d[3 * J], 30),                \
                         __builtin_amdgcn_alignbit(d[3 * J + 2], d[3 * J + 1], 28), base,      \
                         xv[J].x, xv[J].y, acc);
      VQ_G64(0) VQ_G64(1) VQ_G64(2) VQ_G64(3)
#undef VQ_G64
      acc_hazard_fence();
    }
  }
};
template <> struct Chunk<64> : Chunk64T<0> {};
template <> struct Chunk<kFmtK64BN> : Chunk64T<1> {};
template <> struct Chunk<kFmtD1K8> : Chunk64T<2> {};
template <> struct Chunk<kFmtD1K8BN> : Chunk64T<3> {};

// Strip (row-block rb, K-split `split` of `splits`) of problem P; may be empty.
template <int K>
__device__ __forceinline__ Strip make_strip(const GemvProblem& P, int rb, int split, int splits) {
  Strip S;
  const int n_cb = P.n_cb;
  S.x = P.x;
  S.n_cb = n_cb;
  S.sc_rb = nullptr;
  S.codes_rb = nullptr;
  S.lev_rb = nullptr;
  if (K == 16 || K == kFmtK16I8 || K == kFmtK16BN || K == kFmtK16I8H || K == kFmtK32) {
    const int n_pairs = k16_pairs(n_cb);
    S.idx_rb = P.idx + (size_t)rb * n_pairs * 1024;
    if (K == 16) {
      S.cb_rb = P.cb + (size_t)rb * n_pairs * 32;
    } else if (K == kFmtK32) {      // a 64-byte table per group slot, then all the scales; fifth bits behind all nibbles
      S.cb_rb = P.cb + (size_t)rb * n_pairs * 32;
      S.sc_rb = reinterpret_cast<const uint16_t*>(P.cb + (size_t)P.n_rb * n_pairs * 32) +
                (size_t)rb * n_pairs * 2;
      S.codes_rb = P.idx + (size_t)P.n_rb * n_pairs * 1024 + (size_t)rb * n_pairs * 256;
    } else if (K == kFmtK16I8H) {   // two 32-byte tables per group slot, then all the scales (4 bytes per slot)
      S.cb_rb = P.cb + (size_t)rb * n_pairs * 32;
      S.sc_rb = reinterpret_cast<const uint16_t*>(P.cb + (size_t)P.n_rb * n_pairs * 32) +
                (size_t)rb * n_pairs * 4;
    } else {   // int8 tables: 32 bytes per group slot, then all the scales (2 bytes per slot)
      S.cb_rb = P.cb + (size_t)rb * n_pairs * 16;
      S.sc_rb = reinterpret_cast<const uint16_t*>(P.cb + (size_t)P.n_rb * n_pairs * 16) +
                (size_t)rb * n_pairs * 2;
      if (K == kFmtK16BN) {   // levels (32 bytes per slot) and codes (64 bytes per pair) behind the scales
        const size_t n_slots = (size_t)P.n_rb * n_pairs * 2;
        const uint8_t* tb = reinterpret_cast<const uint8_t*>(P.cb);
        S.lev_rb = tb + k16bn_level_offset(n_slots) + (size_t)rb * n_pairs * 64;
        S.codes_rb = tb + k16bn_code_offset(n_slots) + (size_t)rb * n_pairs * 64;
      }
    }
    S.u = (n_pairs * split) / splits;
    S.u_end = (n_pairs * (split + 1)) / splits;
    S.chunks_left = (S.u_end - S.u + 3) >> 2;
  } else if (K == kFmtD1K4) {   // pairs as for k = 16; two 48-byte table records per pair
    const int n_pairs = k16_pairs(n_cb);
    S.idx_rb = P.idx + (size_t)rb * n_pairs * 1024;
    S.cb_rb = P.cb + (size_t)rb * n_pairs * (2 * kD1K4SlotTabBytes / 4);
    S.u = (n_pairs * split) / splits;
    S.u_end = (n_pairs * (split + 1)) / splits;
    S.chunks_left = (S.u_end - S.u + 1) >> 1;
  } else if (K == 64 || K == kFmtK64BN || K == kFmtD1K8 || K == kFmtD1K8BN) {
    const int n_quads = k64_quads(n_cb);
    constexpr int tab_bytes = K == 64 ? kK64QuadTabBytes : K == kFmtD1K8 ? kD1K8QuadTabBytes
                              : K == kFmtD1K8BN ? kD1K8NQuadTabBytes : kK64NQuadTabBytes;
    S.idx_rb = P.idx + (size_t)rb * n_quads * kK64QuadIdxBytes;
    S.cb_rb = P.cb + (size_t)(rb / P.rb_per_cb) * n_quads * (tab_bytes / 4);
    if (K == kFmtK64BN || K == kFmtD1K8BN)   // the codes follow the table records of all group rows
      S.codes_rb = reinterpret_cast<const uint8_t*>(P.cb) +
                   (size_t)(P.n_rb / P.rb_per_cb) * n_quads * tab_bytes +
                   (size_t)rb * n_quads * kK64NQuadCodeBytes;
    S.u = (n_quads * split) / splits;
    S.u_end = (n_quads * (split + 1)) / splits;
    S.chunks_left = S.u_end - S.u;
  } else {
    S.idx_rb = P.idx + (size_t)rb * n_cb * 1024;
    S.cb_rb = P.cb + (size_t)rb * n_cb * (K == kFmtD1K16 ? 8 : 256);   // dwords per group's codebook
    S.u = (n_cb * split) / splits;
    S.u_end = (n_cb * (split + 1)) / splits;
    S.chunks_left = (S.u_end - S.u + 1) >> 1;
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

// ---- low-rank adapter epilogue: y = W x + B (A x) ---------------------------------------------
// After wave_reduce8 lane L holds the total of row r = (L >> 3) & 7 of its row-block; the 8 lanes
// j = L & 7 of a row share the adapter term: lane j holds B[row][8j .. 8j+7] (one 16-byte load,
// issued together with the loads of the row-block's last chunk) and t[8j .. 8j+7] (t = A x, fp32,
// loaded once per problem); lanes with 8j >= rank hold zeros.  Eight fp32 multiply-adds, then
// the same three lane exchanges that end wave_reduce8.
template <bool LORA> struct BatchOf { using type = GemvBatch; };
template <> struct BatchOf<true> { using type = GemvBatchLora; };
__device__ __forceinline__ const GemvBatch& base_of(const GemvBatch& b) { return b; }
__device__ __forceinline__ const GemvBatch& base_of(const GemvBatchLora& b) { return b.base; }

__device__ __forceinline__ uint4 lora_load_b(const LoraProblem& L, const void* fallback, int rb, int lane) {
  const int r = (lane >> 3) & 7, j = lane & 7;
  const bool ok = 8 * j < L.rank;
  const void* p = ok ? static_cast<const void*>(L.B + ((size_t)rb * 8 + r) * L.rank + 8 * j) : fallback;
  return zero_unless(ok, *reinterpret_cast<const uint4*>(p));
}
__device__ __forceinline__ void lora_load_t(const LoraProblem& L, const void* fallback, int lane, float (&tv)[8]) {
  const int j = lane & 7;
  const bool ok = 8 * j < L.rank;
  const float4* p = reinterpret_cast<const float4*>(ok ? static_cast<const void*>(L.t + 8 * j) : fallback);
  const float4 a = p[0], b = p[1];
  tv[0] = ok ? a.x : 0.f; tv[1] = ok ? a.y : 0.f; tv[2] = ok ? a.z : 0.f; tv[3] = ok ? a.w : 0.f;
  tv[4] = ok ? b.x : 0.f; tv[5] = ok ? b.y : 0.f; tv[6] = ok ? b.z : 0.f; tv[7] = ok ? b.w : 0.f;
}
__device__ __forceinline__ float lora_term(uint4 lb, const float (&tv)[8]) {
  const uint32_t w[4] = {lb.x, lb.y, lb.z, lb.w};
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const h2_t h = __builtin_bit_cast(h2_t, w[i]);
    s = __builtin_fmaf((float)h.x, tv[2 * i], s);
    s = __builtin_fmaf((float)h.y, tv[2 * i + 1], s);
  }
  s += dpp_read<0x141>(s);      // row_half_mirror: the other quad of the row's 8 lanes
  s += dpp_read<0x4E>(s);       // quad_perm [2,3,0,1]
  s += dpp_read<0xB1>(s);       // quad_perm [1,0,3,2]
  return s;
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

// ---- persistent streaming kernel -------------------------------------------
// The launch's work is the concatenation of all row-blocks of all problems, measured in
// groups (a row-block of problem p costs n_cb[p] groups; cost_begin[p] is the prefix
// sum).  Workgroup g of G takes the row-blocks whose first group falls in
// [g*C/G, (g+1)*C/G): contiguous row-blocks, balanced to within one row-block.  Inside
// a problem the workgroup keeps x in LDS (staged once), and its waves draw row-blocks
// from an LDS counter, so a wave that finishes early takes the next one.  Each wave
// keeps two chunk buffers in flight across row-block boundaries.
//
// Chunks of the streaming kernel hold no activations: the inner blocks read them from
// the workgroup's LDS copy of x (natural order, read 64 bits per lane), which is followed
// by zeroed col-blocks that the absent units of a ragged chunk read.
template <int K> struct ChunkS;

template <int MODE> struct ChunkS16T {
  static constexpr bool I8 = MODE >= 1, BN = MODE == 2, K32 = MODE == 4, H4 = MODE == 3 || K32;   // see Chunk16T
  static constexpr int kUnits = 4;
  static constexpr int kLutDwords = (BN || H4) ? 256 : 128;
  uint4 ev;        // K32: fifth-bit plane dwords of the chunk's pairs
  uint4 w[4];
  uint4 cbv;       // fp16 codebooks (lanes 0..31), or
  uint32_t tab2;   // H4: see Chunk16T
  uint32_t tab;    // two int8 centroid pairs and
  uint32_t sc;     // their group's fp16 scale
  uint2 cw[4];     // BN: see Chunk16T
  uint32_t lev;
  int u0;          // first pair (locates the activations in LDS), wave-uniform

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    const int np = max(0, min(4, S.u_end - u));
    u0 = u;
    const int u_ld = np > 0 ? u : 0;
    if constexpr (H4) {
      const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)u_ld * 128;
      const uint2 t2 = zero_unless(lane * 8 < np * 128,
                                   *reinterpret_cast<const uint2*>(tq + min(lane * 8, max(np * 128 - 8, 0))));
      tab = t2.x;
      tab2 = t2.y;
      sc = K32 ? S.sc_rb[u_ld * 2 + min(lane >> 3, max(2 * np - 1, 0))]
               : S.sc_rb[u_ld * 4 + min(lane >> 2, max(4 * np - 1, 0))];
      if constexpr (K32) {
        uint32_t e[4];
#pragma unroll
        for (int s = 0; s < 4; ++s)
          e[s] = *reinterpret_cast<const uint32_t*>(S.codes_rb + (size_t)(s < np ? u + s : 0) * 256 + lane * 4);
        ev = make_uint4(e[0], e[1], e[2], e[3]);
      }
    } else if constexpr (I8) {
      const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)u_ld * 64;
      tab = zero_unless(lane * 4 < np * 64,
                        *reinterpret_cast<const uint32_t*>(tq + min(lane * 4, max(np * 64 - 4, 0))));
      sc = S.sc_rb[u_ld * 2 + min(lane >> 3, max(2 * np - 1, 0))];
      if constexpr (BN) {
        lev = zero_unless(lane * 4 < np * 64,
                          *reinterpret_cast<const uint32_t*>(S.lev_rb + (size_t)u_ld * 64 + min(lane * 4, max(np * 64 - 4, 0))));
#pragma unroll
        for (int s = 0; s < 4; ++s)
          cw[s] = *reinterpret_cast<const uint2*>(S.codes_rb + (size_t)(s < np ? u + s : 0) * 64 + (lane >> 3) * 8);
      }
    } else {
      const int cb_off = min(lane * 4, max(np * 32 - 4, 0));
      cbv = zero_unless(lane * 4 < np * 32, stream_load16(S.cb_rb + (size_t)u_ld * 32 + cb_off));
    }
    // uniform base + 32-bit lane offset: the opaque copy keeps the zero-extension next to the
    // load, where it folds into the scalar-base addressing mode (no 64-bit vector adds)
    uint32_t voff = (uint32_t)lane * 16u;
    asm volatile("" : "+v"(voff));
#pragma unroll
    for (int s = 0; s < 4; ++s)
      w[s] = stream_load16(S.idx_rb + (size_t)(s < np ? u + s : 0) * 1024 + voff);
  }

  // x_s: the workgroup's LDS copy of x (natural order: lane L's 4 halfs of col-block c
  // are the 8 bytes at c*512 + 8L, so a wave-wide 64-bit read is conflict-free).  The
  // read for block b+1 is issued before block b, so only the first one is waited for.
  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, const uint32_t* x_s, int lane,
                                          float (&acc)[8]) const {
    if constexpr (H4) {
      const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(tab, scale), k64_dequant_pair(tab >> 16, scale),
                     k64_dequant_pair(tab2, scale), k64_dequant_pair(tab2 >> 16, scale));
    } else if constexpr (I8) {
      const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
      *reinterpret_cast<uint2*>(lut + lane * 2) =
          make_uint2(k64_dequant_pair(tab, scale), k64_dequant_pair(tab >> 16, scale));
      if constexpr (BN)
        *reinterpret_cast<uint2*>(lut + 128 + lane * 2) = make_uint2((lev & 0xffffu) * 0x10001u, (lev >> 16) * 0x10001u);
    } else {
      if (lane < 32) *reinterpret_cast<uint4*>(lut + lane * 4) = cbv;
    }
    wave_lds_sync();
    const uint2* xp = reinterpret_cast<const uint2*>(x_s) + u0 * 128 + lane;   // 64 uint2 per col-block
    if constexpr (BN) {       // absent pairs: zero tables and levels against the zeroed col-blocks behind x
      uint2 x0 = xp[0], x1 = xp[64];
      k16_group_bn<0, 512>(w[0].x, w[0].y, cw[0].x, base, x0.x, x0.y, acc);
      x0 = xp[128];
      k16_group_bn<64, 576>(w[0].z, w[0].w, cw[0].y, base, x1.x, x1.y, acc);
      x1 = xp[192];
      k16_group_bn<128, 640>(w[1].x, w[1].y, cw[1].x, base, x0.x, x0.y, acc);
      x0 = xp[256];
      k16_group_bn<192, 704>(w[1].z, w[1].w, cw[1].y, base, x1.x, x1.y, acc);
      x1 = xp[320];
      k16_group_bn<256, 768>(w[2].x, w[2].y, cw[2].x, base, x0.x, x0.y, acc);
      x0 = xp[384];
      k16_group_bn<320, 832>(w[2].z, w[2].w, cw[2].y, base, x1.x, x1.y, acc);
      x1 = xp[448];
      k16_group_bn<384, 896>(w[3].x, w[3].y, cw[3].x, base, x0.x, x0.y, acc);
      k16_group_bn<448, 960>(w[3].z, w[3].w, cw[3].y, base, x1.x, x1.y, acc);
      acc_hazard_fence();
      return;
    }
    if constexpr (K32) {      // absent pairs: zero tables against the zeroed col-blocks behind x
      const uint32_t es[4] = {ev.x, ev.y, ev.z, ev.w};
      const uint32_t hb = 0x40404040u;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint2 xa = xp[128 * s], xb = xp[128 * s + 64];
        const uint32_t wa0 = s == 0 ? w[0].x : s == 1 ? w[1].x : s == 2 ? w[2].x : w[3].x;
        const uint32_t wa1 = s == 0 ? w[0].y : s == 1 ? w[1].y : s == 2 ? w[2].y : w[3].y;
        const uint32_t wb0 = s == 0 ? w[0].z : s == 1 ? w[1].z : s == 2 ? w[2].z : w[3].z;
        const uint32_t wb1 = s == 0 ? w[0].w : s == 1 ? w[1].w : s == 2 ? w[2].w : w[3].w;
        uint32_t e0, e1, e2, e3;
        k32_plane_sets<0>(es[s], e0, e1, e2, e3);
        if (s == 0) k32_group<0>(wa0, wa1, e0, e1, e2, e3, hb, base, xa.x, xa.y, acc);
        else if (s == 1) k32_group<256>(wa0, wa1, e0, e1, e2, e3, hb, base, xa.x, xa.y, acc);
        else if (s == 2) k32_group<512>(wa0, wa1, e0, e1, e2, e3, hb, base, xa.x, xa.y, acc);
        else k32_group<768>(wa0, wa1, e0, e1, e2, e3, hb, base, xa.x, xa.y, acc);
        k32_plane_sets<1>(es[s], e0, e1, e2, e3);
        if (s == 0) k32_group<128>(wb0, wb1, e0, e1, e2, e3, hb, base, xb.x, xb.y, acc);
        else if (s == 1) k32_group<384>(wb0, wb1, e0, e1, e2, e3, hb, base, xb.x, xb.y, acc);
        else if (s == 2) k32_group<640>(wb0, wb1, e0, e1, e2, e3, hb, base, xb.x, xb.y, acc);
        else k32_group<896>(wb0, wb1, e0, e1, e2, e3, hb, base, xb.x, xb.y, acc);
      }
      acc_hazard_fence();
      return;
    }
    constexpr int T = H4 ? 128 : 64, HS = H4 ? 64 : 0;   // bytes of tables per group slot; rows 4..7
    uint2 x0 = xp[0], x1 = xp[64];
    k16_group<0, 0, HS>(w[0].x, w[0].y, base, x0.x, x0.y, acc);
    x0 = xp[128];
    k16_group<T, 0, HS>(w[0].z, w[0].w, base, x1.x, x1.y, acc);
    x1 = xp[192];
    k16_group<2 * T, 0, HS>(w[1].x, w[1].y, base, x0.x, x0.y, acc);
    x0 = xp[256];
    k16_group<3 * T, 0, HS>(w[1].z, w[1].w, base, x1.x, x1.y, acc);
    x1 = xp[320];
    k16_group<4 * T, 0, HS>(w[2].x, w[2].y, base, x0.x, x0.y, acc);
    x0 = xp[384];
    k16_group<5 * T, 0, HS>(w[2].z, w[2].w, base, x1.x, x1.y, acc);
    x1 = xp[448];
    k16_group<6 * T, 0, HS>(w[3].x, w[3].y, base, x0.x, x0.y, acc);
    k16_group<7 * T, 0, HS>(w[3].z, w[3].w, base, x1.x, x1.y, acc);
    acc_hazard_fence();
  }
};
template <> struct ChunkS<16> : ChunkS16T<0> {};
template <> struct ChunkS<kFmtK16I8H> : ChunkS16T<3> {};
template <> struct ChunkS<kFmtK32> : ChunkS16T<4> {};
template <> struct ChunkS<kFmtK16I8> : ChunkS16T<1> {};
template <> struct ChunkS<kFmtK16BN> : ChunkS16T<2> {};

template <> struct ChunkS<kFmtD1K4> {
  static constexpr int kUnits = 2;
  static constexpr int kLutDwords = 512;
  uint4 w[2];
  uint32_t tab, sc;   // see Chunk<kFmtD1K4>
  int u0;             // first pair

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    const int np = max(0, min(2, S.u_end - u));
    u0 = u;
    const int u_ld = np > 0 ? u : 0;
    const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)u_ld * (2 * kD1K4SlotTabBytes);
    const int blk = min(lane >> 4, max(2 * np - 1, 0)), row = (lane >> 1) & 7;
    tab = zero_unless((lane >> 4) < 2 * np,
                      *reinterpret_cast<const uint32_t*>(tq + blk * kD1K4SlotTabBytes + row * 4));
    sc = zero_unless((lane >> 4) < 2 * np,
                     (uint32_t)*reinterpret_cast<const uint16_t*>(tq + blk * kD1K4SlotTabBytes + kD1K4ScaleOffset + row * 2));
    uint32_t voff = (uint32_t)lane * 16u;      // see ChunkS<16>::load
    asm volatile("" : "+v"(voff));
#pragma unroll
    for (int s = 0; s < 2; ++s)
      w[s] = stream_load16(S.idx_rb + (size_t)(s < np ? u + s : 0) * 1024 + voff);
  }

  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, const uint32_t* x_s, int lane,
                                          float (&acc)[8]) const {
    const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
    uint4 e0, e1;
    d1k4_entries(k64_dequant_pair(tab, scale), k64_dequant_pair(tab >> 16, scale), lane & 1, e0, e1);
    *reinterpret_cast<uint4*>(lut + lane * 8) = e0;
    *reinterpret_cast<uint4*>(lut + lane * 8 + 4) = e1;
    wave_lds_sync();
    const uint2* xp = reinterpret_cast<const uint2*>(x_s) + u0 * 128 + lane;
    uint2 x0 = xp[0], x1 = xp[64];
    k16_group<0, 64>(w[0].x, w[0].y, base, x0.x, x0.y, acc);
    x0 = xp[128];
    k16_group<512, 64>(w[0].z, w[0].w, base, x1.x, x1.y, acc);
    x1 = xp[192];
    k16_group<1024, 64>(w[1].x, w[1].y, base, x0.x, x0.y, acc);
    k16_group<1536, 64>(w[1].z, w[1].w, base, x1.x, x1.y, acc);
    acc_hazard_fence();
  }
};

template <bool D1> struct ChunkS256T {
  static constexpr int kUnits = 2;
  static constexpr int kLutDwords = 512;
  uint4 w[2];
  uint4 cbv[2];
  uint2 clo[2];      // d = 1: see Chunk256T
  uint32_t chi[2];
  int u0;          // first col-block

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    u0 = u;
    uint32_t voff = (uint32_t)lane * 16u;      // see ChunkS<16>::load
    asm volatile("" : "+v"(voff));
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const bool ok = u + s < S.u_end;
      const int c = ok ? u + s : 0;
      w[s] = stream_load16(S.idx_rb + (size_t)c * 1024 + voff);
      if constexpr (D1) {
        const uint8_t* cg = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)c * 32;
        clo[s] = zero_unless(ok, *reinterpret_cast<const uint2*>(cg + (lane & 3) * 8));
        chi[s] = zero_unless(ok, (uint32_t)*reinterpret_cast<const uint16_t*>(cg + (lane >> 2) * 2));
      } else {
        cbv[s] = zero_unless(ok, stream_load16(reinterpret_cast<const uint8_t*>(S.cb_rb + (size_t)c * 256) + voff));
      }
    }
  }

  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, const uint32_t* x_s, int lane,
                                          float (&acc)[8]) const {
    *reinterpret_cast<uint4*>(lut + lane * 4) = D1 ? d1_pair_entries(clo[0], chi[0]) : cbv[0];
    *reinterpret_cast<uint4*>(lut + 256 + lane * 4) = D1 ? d1_pair_entries(clo[1], chi[1]) : cbv[1];
    wave_lds_sync();
    const uint2* xp = reinterpret_cast<const uint2*>(x_s) + u0 * 64 + lane;
    const uint2 x0 = xp[0], x1 = xp[64];
    k256_group<0>(w[0].x, w[0].y, w[0].z, w[0].w, base, x0.x, x0.y, acc);
    k256_group<1024>(w[1].x, w[1].y, w[1].z, w[1].w, base, x1.x, x1.y, acc);
    acc_hazard_fence();
  }
};
template <> struct ChunkS<256> : ChunkS256T<false> {};
template <> struct ChunkS<kFmtD1K16> : ChunkS256T<true> {};

template <int MODE> struct ChunkS64T {
  static constexpr bool BN = MODE == 1 || MODE == 3, D1 = MODE >= 2;
  static constexpr int kUnits = 1;
  static constexpr int kLutDwords = BN ? 320 : 256;
  static constexpr int kTabBytes = D1 ? (BN ? kD1K8NQuadTabBytes : kD1K8QuadTabBytes) : BN ? kK64NQuadTabBytes : kK64QuadTabBytes;
  static constexpr int kScaleOffset = D1 ? kD1K8ScaleOffset : 512;
  static constexpr int kLevelOffset = D1 ? kD1K8NLevelOffset : kK64NLevelOffset;
  uint4 w[3];
  uint2 tab;
  uint32_t sc;
  uint4 cw;        // BN: see Chunk64T
  uint32_t lev;
  int u0;          // the quad (locates the activations in LDS), wave-uniform

  __device__ __forceinline__ void load(const Strip& S, int u, int lane) {
    const bool ok = u < S.u_end;
    const int q = ok ? u : 0;
    u0 = u;
    const uint8_t* tq = reinterpret_cast<const uint8_t*>(S.cb_rb) + (size_t)q * kTabBytes;
    uint32_t voff = (uint32_t)lane * 16u;      // see ChunkS<16>::load
    asm volatile("" : "+v"(voff));
    tab = zero_unless(ok, *reinterpret_cast<const uint2*>(tq + (D1 ? (uint32_t)(lane >> 4) * 8u : voff >> 1)));
    sc = *reinterpret_cast<const uint16_t*>(tq + kScaleOffset + (lane >> 4) * 2);
    if constexpr (BN) {
      lev = zero_unless(ok, (uint32_t)*reinterpret_cast<const uint16_t*>(tq + kLevelOffset + lane * 2));
      cw = *reinterpret_cast<const uint4*>(S.codes_rb + (size_t)q * kK64NQuadCodeBytes + (lane >> 3) * 16);
    }
#pragma unroll
    for (int p = 0; p < 3; ++p)
      w[p] = stream_load16(S.idx_rb + (size_t)q * kK64QuadIdxBytes + p * 1024 + voff);
  }

  // An absent quad is consumed with a zero table against the zeroed col-blocks behind x.
  __device__ __forceinline__ void consume(uint32_t* lut, uint32_t base, const uint32_t* x_s, int lane,
                                          float (&acc)[8]) const {
    const _Float16 scale = __builtin_bit_cast(_Float16, (uint16_t)sc);
    if constexpr (D1) {
      const int e = 4 * (lane & 15);
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(d1k8_pair(tab, e), scale), k64_dequant_pair(d1k8_pair(tab, e + 1), scale),
                     k64_dequant_pair(d1k8_pair(tab, e + 2), scale), k64_dequant_pair(d1k8_pair(tab, e + 3), scale));
    } else {
      *reinterpret_cast<uint4*>(lut + lane * 4) =
          make_uint4(k64_dequant_pair(tab.x, scale), k64_dequant_pair(tab.x >> 16, scale),
                     k64_dequant_pair(tab.y, scale), k64_dequant_pair(tab.y >> 16, scale));
    }
    if constexpr (BN) lut[256 + lane] = lev * 0x10001u;
    wave_lds_sync();
    const uint2* xp = reinterpret_cast<const uint2*>(x_s) + u0 * 256 + lane;   // 64 uint2 per col-block
    const uint32_t d[12] = {w[0].x, w[0].y, w[0].z, w[0].w, w[1].x, w[1].y,
                            w[1].z, w[1].w, w[2].x, w[2].y, w[2].z, w[2].w};
    if constexpr (BN) {
      uint2 x0 = xp[0], x1 = xp[64];
#define VQ_G64N(J, X, CW)                                                                      \
      k64_group_bn<256 * J, 1024 + 64 * J>(d[3 * J], d[3 * J + 1], d[3 * J + 2],               \
                         __builtin_amdgcn_alignbit(d[3 * J + 1], d[3 * J], 30),                \
                         __builtin_amdgcn_alignbit(d[3 * J + 2], d[3 * J + 1], 28), CW, base,  \
                         X.x, X.y, acc);
      VQ_G64N(0, x0, cw.x)
      x0 = xp[128];
      VQ_G64N(1, x1, cw.y)
      x1 = xp[192];
      VQ_G64N(2, x0, cw.z)
      VQ_G64N(3, x1, cw.w)
#undef VQ_G64N
      acc_hazard_fence();
    } else {
      uint2 x0 = xp[0], x1 = xp[64];
#define VQ_G64(J, X)                                                                           \
      k64_group<256 * J>(d[3 * J], d[3 * J + 1], d[3 * J + 2],                                 \
                         __builtin_amdgcn_alignbit(d[3 * J + 1], d[3 * J], 30),                \
                         __builtin_amdgcn_alignbit(d[3 * J + 2], d[3 * J + 1], 28), base,      \
                         X.x, X.y, acc);
      VQ_G64(0, x0)
      x0 = xp[128];
      VQ_G64(1, x1)
      x1 = xp[192];
      VQ_G64(2, x0)
      VQ_G64(3, x1)
#undef VQ_G64
      acc_hazard_fence();
    }
  }
};
template <> struct ChunkS<64> : ChunkS64T<0> {};
template <> struct ChunkS<kFmtK64BN> : ChunkS64T<1> {};
template <> struct ChunkS<kFmtD1K8> : ChunkS64T<2> {};
template <> struct ChunkS<kFmtD1K8BN> : ChunkS64T<3> {};

// Zeroed col-blocks kept behind x in LDS (absent units of a ragged chunk read them).
constexpr int kXPadColBlocks = 8;

// Waves per workgroup of the streaming kernel: 8 share one LDS copy of x, which lets 24
// waves (6 per SIMD) fit on a CU next to 3 copies of a 22 KB x.
constexpr int kStreamWaves = 8;

template <int K, bool LORA>
__global__ __launch_bounds__(kStreamWaves * 64) void gemv_stream_kernel(const typename BatchOf<LORA>::type arg) {
  const GemvBatch& batch = base_of(arg);
  // dynamic LDS: [kStreamWaves x 2 table regions][row-block counter][x of the current problem]
  extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
  constexpr int kLut = ChunkS<K>::kLutDwords;
  uint32_t* const counter = smem + kStreamWaves * 2 * kLut;          // 4 dwords reserved
  uint32_t* const x_s = counter + 4;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t* lut_a = smem + wave * 2 * kLut;
  uint32_t* lut_b = lut_a + kLut;
  const uint32_t base_a = lds_addr(lut_a), base_b = lds_addr(lut_b);

  const int lo = (int)((long long)blockIdx.x * batch.total_cost / gridDim.x);
  const int hi = (int)((long long)(blockIdx.x + 1) * batch.total_cost / gridDim.x);
  int pi;
  {  // last problem that starts at or before lo
    int lo_p = 0, hi_p = batch.count;
    while (hi_p - lo_p > 1) {
      const int mid = (lo_p + hi_p) >> 1;
      if (batch.p[mid].cost_begin <= lo) lo_p = mid; else hi_p = mid;
    }
    pi = lo_p;
  }

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;

  for (; pi < batch.count; ++pi) {
    const GemvProblem& P = batch.p[pi];
    const int c0 = P.cost_begin;
    if (c0 >= hi) break;
    const int n_cb = P.n_cb;
    const int c1 = c0 + P.n_rb * n_cb;
    const int rb_lo = (max(lo, c0) - c0 + n_cb - 1) / n_cb;
    const int rb_hi = (min(hi, c1) - c0 + n_cb - 1) / n_cb;
    if (rb_lo >= rb_hi) continue;

    // ---- the workgroup enters problem pi: stage x, reset the row-block counter
    __syncthreads();                       // everyone is done with the previous x
    {
      // x, then kXPadColBlocks col-blocks of zeros
      const uint4* xg = reinterpret_cast<const uint4*>(P.x);
      uint4* xl = reinterpret_cast<uint4*>(x_s);
      const int n16 = n_cb * 32;           // 16-byte pieces of x
      for (int i = threadIdx.x; i < n16 + kXPadColBlocks * 32; i += kStreamWaves * 64)
        xl[i] = i < n16 ? xg[i] : make_uint4(0, 0, 0, 0);
      if (threadIdx.x == 0) counter[0] = rb_lo + kStreamWaves;   // waves start on rb_lo + wave
    }
    __syncthreads();

    // ---- per-wave pipeline over row-blocks drawn from the counter
    int l_rb = rb_lo + wave;
    bool l_ok = l_rb < rb_hi;
    int s_rb = l_ok ? l_rb : rb_lo;       // the row-block S describes (always a valid one)
    Strip S = make_strip<K>(P, s_rb, 0, 1);
    float tv[8];
    uint4 a_lb = make_uint4(0, 0, 0, 0), b_lb = a_lb;
    if constexpr (LORA) lora_load_t(arg.l[pi], P.x, lane, tv);
    if (!l_ok) {              // park on a valid row-block with nothing left to load
      S.u = S.u_end;
      S.chunks_left = 0;
    }
    void* const y = P.y;

    ChunkS<K> A, B;
    bool a_ok, b_ok, a_last = false, b_last = false;
    (void)tv; (void)a_lb; (void)b_lb; (void)s_rb;
    int a_rb = 0, b_rb = 0;

    // The loads are issued whether or not a chunk is left (an exhausted strip makes them
    // harmless dummy reads): a branch around them would hide the number of loads in
    // flight from the compiler, which would then wait for all of them before every use.
#define VQ_LOAD_NEXT(BUF, OK, LAST, RB, LB)                                      \
    do {                                                                         \
      OK = l_ok;                                                                 \
      BUF.load(S, S.u, lane);                                                    \
      if constexpr (LORA) LB = lora_load_b(arg.l[pi], P.x, s_rb, lane);          \
      if (l_ok) {                                                                \
        S.u += ChunkS<K>::kUnits;                                                \
        LAST = --S.chunks_left == 0;                                             \
        RB = l_rb;                                                               \
        if (LAST) {                                                              \
          uint32_t nxt = 0;                                                      \
          if (lane == 0) nxt = atomicAdd(counter, 1u);                           \
          l_rb = __builtin_amdgcn_readfirstlane(nxt);                            \
          l_ok = l_rb < rb_hi;                                                   \
          if (l_ok) { s_rb = l_rb; S = make_strip<K>(P, l_rb, 0, 1); }           \
        }                                                                        \
      }                                                                          \
    } while (0)
#define VQ_CONSUME(BUF, LUT, BASE, LAST, RB, LB)                                 \
    do {                                                                         \
      __builtin_amdgcn_s_setprio(1);   /* lookups and dot products ahead of other waves' load set-up */ \
      BUF.consume(LUT, BASE, x_s, lane, acc);                                    \
      __builtin_amdgcn_s_setprio(0);                                             \
      if (LAST) {                                                                \
        float v = wave_reduce8(acc, lane);                                       \
        if constexpr (LORA) v += lora_term(LB, tv);                              \
        store_rows(y, batch.y_f32, RB, lane, v);                                 \
        _Pragma("unroll") for (int r = 0; r < 8; ++r) acc[r] = 0.f;              \
      }                                                                          \
    } while (0)

    VQ_LOAD_NEXT(A, a_ok, a_last, a_rb, a_lb);
    while (a_ok) {
      VQ_LOAD_NEXT(B, b_ok, b_last, b_rb, b_lb);
      VQ_CONSUME(A, lut_a, base_a, a_last, a_rb, a_lb);
      VQ_LOAD_NEXT(A, a_ok, a_last, a_rb, a_lb);
      if (!b_ok) break;
      VQ_CONSUME(B, lut_b, base_b, b_last, b_rb, b_lb);
    }
#undef VQ_LOAD_NEXT
#undef VQ_CONSUME
  }
}

// A chunk's lookups and dot products at wave priority 1: waves whose data has arrived go ahead
// of waves that are still setting up their loads.  Worth 7 % on the launches of a decoder layer
// (852 -> 794 us for the 128 launches of a 7B pass), which are latency-bound.
template <typename C>
__device__ __forceinline__ void consume_at_priority(const C& chunk, uint32_t* lut, uint32_t base,
                                                    int lane, float (&acc)[8]) {
  __builtin_amdgcn_s_setprio(1);
  chunk.consume(lut, base, lane, acc);
  __builtin_amdgcn_s_setprio(0);
}

// ---- split-K kernel (few row-blocks) ---------------------------------------
// UP > 0: the host guarantees that no strip of the launch is longer than UP chunks (1, 2 or 3); all
// of a wave's chunks are then loaded at once, so the wave waits for memory once instead of once
// per chunk (4096 x 11008 with k = 256: three chunks per wave), and with UP = 1 the second chunk
// buffer and its registers disappear.  UP = 0: strips of any length, two chunk buffers ping-pong.
// WPW: waves per workgroup, 4 or 8 (8 when 8 waves share a row-block).
template <int K, int UP, int WPW, bool LORA>
__global__ __launch_bounds__(64 * WPW) void gemv_split_kernel(const typename BatchOf<LORA>::type arg) {
  const GemvBatch& batch = base_of(arg);
  __shared__ __attribute__((aligned(16))) uint32_t lut_all[WPW][(UP == 1 ? 1 : 2) * Chunk<K>::kLutDwords];
  __shared__ float part[WPW][8];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wg = blockIdx.x;
  const int pi = find_problem(batch, wg);
  const GemvProblem& P = batch.p[pi];
  const int splits = P.splits;
  const int rb_per_wg = WPW / splits;
  const int wg_local = wg - P.wg_begin;
  const int rb = wg_local * rb_per_wg + wave / splits;
  const int split = wave % splits;
  uint32_t* lut_a = lut_all[wave];
  uint32_t* lut_b = lut_a + (UP == 1 ? 0 : Chunk<K>::kLutDwords);
  const uint32_t base_a = lds_addr(lut_a), base_b = lds_addr(lut_b);

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;

  float tv[8];
  uint4 lb = make_uint4(0, 0, 0, 0);
  (void)tv; (void)lb;
  if constexpr (LORA) {      // issued ahead of the chunk loads, used after the reduction
    lora_load_t(arg.l[pi], P.x, lane, tv);
    lb = lora_load_b(arg.l[pi], P.x, rb < P.n_rb ? rb : 0, lane);
  }

  if (rb < P.n_rb) {
    Strip S = make_strip<K>(P, rb, split, splits);
    if constexpr (UP == 1) {
      if (S.chunks_left > 0) {
        Chunk<K> A;
        A.load(S, S.u, lane);
        consume_at_priority(A, lut_a, base_a, lane, acc);
      }
    } else if constexpr (UP > 1) {
      if (S.chunks_left > 0) {
        constexpr int U = Chunk<K>::kUnits;
        Chunk<K> C[UP];
#pragma unroll
        for (int i = 0; i < UP; ++i) C[i].load(S, S.u + i * U, lane);   // past the strip's end: dummy loads, zero data
        consume_at_priority(C[0], lut_a, base_a, lane, acc);
        if (S.chunks_left > 1) consume_at_priority(C[1], lut_b, base_b, lane, acc);
        if constexpr (UP > 2) {
          if (S.chunks_left > 2) consume_at_priority(C[2], lut_a, base_a, lane, acc);
        }
      }
    } else if (S.chunks_left > 0) {
      constexpr int U = Chunk<K>::kUnits;
      Chunk<K> A, B;
      A.load(S, S.u, lane);
      while (true) {
        // invariant: A holds the chunk at S.u, chunks_left counts it
        const bool more1 = S.chunks_left > 1;
        if (more1) { --S.chunks_left; B.load(S, S.u + U, lane); ++S.chunks_left; }
        consume_at_priority(A, lut_a, base_a, lane, acc);
        if (!more1) break;
        S.u += U; --S.chunks_left;            // B is now current
        const bool more2 = S.chunks_left > 1;
        if (more2) { --S.chunks_left; A.load(S, S.u + U, lane); ++S.chunks_left; }
        consume_at_priority(B, lut_b, base_b, lane, acc);
        if (!more2) break;
        S.u += U; --S.chunks_left;            // A is current again
      }
    }
  }

  acc_hazard_fence();
  float v = wave_reduce8(acc, lane);
  if constexpr (LORA) {
    const float lo = lora_term(lb, tv);      // all lanes take part in the exchanges
    if (split == 0) v += lo;
  }
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

// Calls F<tag>() for the kernel format tag `fmt`.
#define VQ_FMT_SWITCH(fmt, F)                 \
  switch (fmt) {                              \
    case 16: F(16); break;                    \
    case 64: F(64); break;                    \
    case kFmtK16I8: F(kFmtK16I8); break;      \
    case kFmtK16I8H: F(kFmtK16I8H); break;    \
    case kFmtK32: F(kFmtK32); break;          \
    case kFmtD1K16: F(kFmtD1K16); break;      \
    case kFmtK64BN: F(kFmtK64BN); break;      \
    case kFmtK16BN: F(kFmtK16BN); break;      \
    case kFmtD1K8BN: F(kFmtD1K8BN); break;    \
    case kFmtD1K8: F(kFmtD1K8); break;        \
    case kFmtD1K4: F(kFmtD1K4); break;        \
    default: F(256); break;                   \
  }

namespace {

inline size_t stream_lds_bytes_impl(int fmt, int max_n_cb) {
  int lut_dwords = 0;
#define VQ_F(K) lut_dwords = ChunkS<K>::kLutDwords
  VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  return (size_t)kStreamWaves * 2 * lut_dwords * 4 + 16 + (size_t)(max_n_cb + kXPadColBlocks) * 512;
}

// Slot of a kernel format tag in per-format tables (the formats VQ_FMT_SWITCH knows; 256 is the default).
constexpr int kStreamFormats = 12;
inline int stream_format_slot(int fmt) {
  switch (fmt) {
    case 16: return 0;
    case 64: return 1;
    case kFmtK16I8: return 3;
    case kFmtD1K16: return 4;
    case kFmtK64BN: return 5;
    case kFmtD1K8: return 6;
    case kFmtD1K4: return 7;
    case kFmtK16BN: return 8;
    case kFmtD1K8BN: return 9;
    case kFmtK16I8H: return 10;
    case kFmtK32: return 11;
    default: return 2;
  }
}

// Workgroups of the persistent kernel that fit on the current device at once.
// Occupancy of the persistent kernel for this LDS size: a pure function of the code object
// and the device, asked of the runtime once per (device, format, size) and cached (the one
// piece of state the library keeps).  The slots are atomics: two threads that fill the same
// slot at once store the same value.  The query enqueues nothing on any stream.
template <bool LORA> int stream_resident_wgs_impl(int fmt, int max_n_cb) {
  static std::atomic<int> cached[kStreamFormats][16][kStreamMaxColBlocks + 1];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) dev = 0;
  const int fi = stream_format_slot(fmt);
  int slot = cached[fi][dev][max_n_cb].load(std::memory_order_relaxed);
  if (slot == 0) {
    int per_cu = 0, cus = 0;
    const size_t lds = stream_lds_bytes_impl(fmt, max_n_cb);
    const int threads = kStreamWaves * 64;
    hipError_t e = hipSuccess;
#define VQ_F(K) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gemv_stream_kernel<K, LORA>, threads, lds)
    VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
    const bool ok = e == hipSuccess && per_cu >= 1 &&
                    hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus >= 1;
    if (!ok) {
      // A refused query is not an error of the call: any grid size gives the right result, a
      // small one only runs slower.  Nothing is cached, so the next call asks again.
      (void)hipGetLastError();
      return 256;
    }
    slot = per_cu * cus;
    cached[fi][dev][max_n_cb].store(slot, std::memory_order_relaxed);
  }
  return slot;
}

inline int chunk_units_impl(int fmt) {
  int units = 0;
#define VQ_F(K) units = Chunk<K>::kUnits
  VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  return units;
}

template <bool LORA>
hipError_t launch_gemv_impl(int fmt, const typename BatchOf<LORA>::type& batch, int mode, int grid_wgs,
                            int max_n_cb, hipStream_t s, int wpw) {
  const dim3 grid(grid_wgs), block(64 * wpw);
  if (mode == 1) {
    const size_t lds = stream_lds_bytes_impl(fmt, max_n_cb);
    const dim3 sblock(kStreamWaves * 64);
#define VQ_F(K) hipLaunchKernelGGL((gemv_stream_kernel<K, LORA>), grid, sblock, lds, s, batch)
    VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  } else if (mode == 2) {
#define VQ_F(K)                                                                                   \
  if (wpw == 8) hipLaunchKernelGGL((gemv_split_kernel<K, 1, 8, LORA>), grid, block, 0, s, batch); \
  else hipLaunchKernelGGL((gemv_split_kernel<K, 1, 4, LORA>), grid, block, 0, s, batch)
    VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  } else if (wpw != 8) {
    return hipErrorInvalidValue;    // strips longer than one chunk are always shared by 8 waves
  } else if (mode == 3) {
#define VQ_F(K) hipLaunchKernelGGL((gemv_split_kernel<K, 2, 8, LORA>), grid, block, 0, s, batch)
    VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  } else if (mode == 4) {
#define VQ_F(K) hipLaunchKernelGGL((gemv_split_kernel<K, 3, 8, LORA>), grid, block, 0, s, batch)
    VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  } else {
#define VQ_F(K) hipLaunchKernelGGL((gemv_split_kernel<K, 0, 8, LORA>), grid, block, 0, s, batch)
    VQ_FMT_SWITCH(fmt, VQ_F)
#undef VQ_F
  }
  return hipGetLastError();
}

}  // namespace
}  // namespace vq
