// Device-side helpers for the gfx950 kernels: index chunk addressing in the
// device layout, fp16-pair dot product, wave-level reductions.
//
// Device layout of the packed indices (what vq_pack_layout writes).  A group is
// 8 rows x 128 vectors.  Lane L of a wave owns the two vectors 2L, 2L+1 of every
// row of a group, so that its activations (x[4L..4L+3] of the group's columns)
// are two dwords and one lane keeps 8 row accumulators.
//   4-bit (k=16): a lane's share of a group is 8 bytes = 2 dwords of 4 rows each.
//     Inside a dword, row b's two indices lo (vector 2L) and hi (vector 2L+1) are
//     stored pre-scaled for the table lookup: bits [8b+5:8b+2] = lo, bits
//     [8b+7:8b+6] = hi[1:0], bits [8b'+1:8b'] = hi[3:2] with b' = (b+1) mod 4.  Then
//     w & 0x3c3c3c3c holds 4*lo in every byte and ror(w,4) & 0x3c3c3c3c holds 4*hi:
//     three VALU instructions per 8 indices.  Two horizontally adjacent groups
//     (col-blocks 2p, 2p+1 of one row-block) are interleaved per lane: 16 bytes per
//     lane, 1 KB per wave-wide 128-bit load.  A row-block always holds
//     ceil(n_cb/2) such pairs: if the number of col-blocks is odd, the missing
//     group is stored as zero indices with an all-zero codebook, so it adds
//     exactly 0 and no kernel needs a special case.
//   8-bit (k=256): a lane's share is 16 bytes, byte 2r+e = row r, vector 2L+e
//     (= canonical byte r*128 + 2L + e); one group per wave-wide 128-bit load.
// Codebooks keep the canonical order (one dword per centroid), padded as above.
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

typedef __attribute__((address_space(3))) uint32_t lds_u32;

// LDS byte address of a pointer into a __shared__ array, made wave-uniform (SGPR).
__device__ __forceinline__ uint32_t lds_addr(const uint32_t* p) {
  const uint32_t a = (uint32_t)(uintptr_t)(lds_u32*)p;
  return __builtin_amdgcn_readfirstlane(a);
}

// Wait states between the last v_dot2c of an inline-asm block and ordinary VALU code
// that reads the accumulators.
__device__ __forceinline__ void acc_hazard_fence() { asm volatile("s_nop 3" ::: "memory"); }

// Orders this wave's LDS writes before its later LDS reads (other lanes' data).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The pre-scaled 4-bit layout of a dword (4 rows x 2 vectors): a = 4 * index of vector 2L in each
// byte, b = 4 * index of vector 2L + 1.
__device__ __forceinline__ void k16_split_dword(uint32_t w, uint32_t& a, uint32_t& b) {
  a = w & 0x3c3c3c3cu;
  b = __builtin_amdgcn_alignbit(w, w, 4) & 0x3c3c3c3cu;
}

// ---------------------------------------------------------------------------
// k = 16 inner block: all 16 lookups + dot products of one lane's share of one
// group (two dwords = 8 rows x 2 vectors), hand-scheduled.
//
//   w0, w1   the lane's 8 index bytes (byte r: low nibble = vector 2L, high = 2L+1)
//   base     LDS byte address of this wave's table region (wave-uniform, SGPR)
//   OFF      byte offset of the group's 16-entry table inside the region (immediate)
//   x0, x1   fp16 pairs of the activations of vectors 2L and 2L+1
//   acc      the 8 row accumulators (fp32)
//
// Per dword, w & 0x3c3c3c3c and ror(w, 4) & 0x3c3c3c3c leave index*4 of the two
// vectors of each row in the four bytes (see the layout above); one SDWA add per
// lookup then picks a byte and adds the table base, and the table offset rides in
// the ds_read immediate: 2.4 VALU instructions per vector including the dot2.  LDS reads are kept 8-12
// deep ahead of the dot products (lgkmcnt is a 4-bit counter).  A dot2c result
// may be consumed by the next dot2c at once, but other VALU instructions need
// wait states the compiler cannot see inside an asm statement: callers run
// acc_hazard_fence() after the last block of a straight run of blocks, i.e. before any
// point where the compiler may place code of its own that reads an accumulator (a loop
// edge or branch merge can make it copy accumulators between registers).
#define VQ_SDWA_RD(R, T, B, ROW)                                                          \
  "v_add_u32_sdwa " R ", %[base], " T                                                     \
  " dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_" #B "\n"            \
  "ds_read_b32 " R ", " R " offset:%[off]+" #ROW "*%[rs]+(" #ROW "/4)*%[hs]\n"
#define VQ_MASKS(W)                                  \
  "v_and_b32 %[ta], 0x3c3c3c3c, " W "\n"             \
  "v_alignbit_b32 %[tb], " W ", " W ", 4\n"          \
  "v_and_b32 %[tb], 0x3c3c3c3c, %[tb]\n"
#define VQ_DOT(ACC, R, X) "v_dot2c_f32_f16 " ACC ", " R ", " X "\n"

// RS: byte distance between the tables of consecutive rows (0: the 8 rows share one table;
// 64: a 16-entry table per row, the scalar 2-bit format).  HS: byte distance between the table
// of rows 0..3 and that of rows 4..7 (64 for groups of 4 rows, else 0).
template <int OFF, int RS = 0, int HS = 0>
__device__ __forceinline__ void k16_group(uint32_t w0, uint32_t w1, uint32_t base, uint32_t x0,
                                          uint32_t x1, float (&acc)[8]) {
  uint32_t ta, tb, r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11;
  asm volatile(
      VQ_MASKS("%[w0]")
      VQ_SDWA_RD("%[r0]", "%[ta]", 0, 0) VQ_SDWA_RD("%[r1]", "%[tb]", 0, 0)
      VQ_SDWA_RD("%[r2]", "%[ta]", 1, 1) VQ_SDWA_RD("%[r3]", "%[tb]", 1, 1)
      VQ_SDWA_RD("%[r4]", "%[ta]", 2, 2) VQ_SDWA_RD("%[r5]", "%[tb]", 2, 2)
      VQ_SDWA_RD("%[r6]", "%[ta]", 3, 3) VQ_SDWA_RD("%[r7]", "%[tb]", 3, 3)
      VQ_MASKS("%[w1]")
      VQ_SDWA_RD("%[r8]", "%[ta]", 0, 4) VQ_SDWA_RD("%[r9]", "%[tb]", 0, 4)
      VQ_SDWA_RD("%[r10]", "%[ta]", 1, 5) VQ_SDWA_RD("%[r11]", "%[tb]", 1, 5)
      "s_waitcnt lgkmcnt(4)\n"
      VQ_DOT("%[a0]", "%[r0]", "%[x0]") VQ_DOT("%[a1]", "%[r2]", "%[x0]")
      VQ_DOT("%[a2]", "%[r4]", "%[x0]") VQ_DOT("%[a3]", "%[r6]", "%[x0]")
      VQ_DOT("%[a0]", "%[r1]", "%[x1]") VQ_DOT("%[a1]", "%[r3]", "%[x1]")
      VQ_DOT("%[a2]", "%[r5]", "%[x1]") VQ_DOT("%[a3]", "%[r7]", "%[x1]")
      VQ_SDWA_RD("%[r0]", "%[ta]", 2, 6) VQ_SDWA_RD("%[r1]", "%[tb]", 2, 6)
      VQ_SDWA_RD("%[r2]", "%[ta]", 3, 7) VQ_SDWA_RD("%[r3]", "%[tb]", 3, 7)
      "s_waitcnt lgkmcnt(4)\n"
      VQ_DOT("%[a4]", "%[r8]", "%[x0]") VQ_DOT("%[a5]", "%[r10]", "%[x0]")
      VQ_DOT("%[a4]", "%[r9]", "%[x1]") VQ_DOT("%[a5]", "%[r11]", "%[x1]")
      "s_waitcnt lgkmcnt(0)\n"
      VQ_DOT("%[a6]", "%[r0]", "%[x0]") VQ_DOT("%[a7]", "%[r2]", "%[x0]")
      VQ_DOT("%[a6]", "%[r1]", "%[x1]") VQ_DOT("%[a7]", "%[r3]", "%[x1]")
      : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]),
        [a4] "+v"(acc[4]), [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]),
        [ta] "=&v"(ta), [tb] "=&v"(tb), [r0] "=&v"(r0), [r1] "=&v"(r1), [r2] "=&v"(r2),
        [r3] "=&v"(r3), [r4] "=&v"(r4), [r5] "=&v"(r5), [r6] "=&v"(r6), [r7] "=&v"(r7),
        [r8] "=&v"(r8), [r9] "=&v"(r9), [r10] "=&v"(r10), [r11] "=&v"(r11)
      : [w0] "v"(w0), [w1] "v"(w1), [base] "s"(base), [x0] "v"(x0), [x1] "v"(x1), [off] "n"(OFF), [rs] "n"(RS), [hs] "n"(HS)
      : "memory");
}
// k = 32 (5-bit indices): the low four bits of every index are stored exactly as for k = 16, the
// fifth bits in a separate plane (see the layout in vq_internal.h); the caller shifts the lane's
// plane dword so that e0 .. e3 carry, at bits 6, 14, 22 and 30, the fifth bits of (rows 0..3,
// vector 2L), (rows 0..3, vector 2L+1), (rows 4..7, vector 2L), (rows 4..7, vector 2L+1).  One
// v_and_or_b32 per four lookups merges them into the "4 * index" bytes (a byte then holds
// 4 * (index mod 16) + 64 * (index / 16) = 4 * index); the rest is the k = 16 block on a
// 32-entry table.  hb: 0x40404040 in a scalar register.
#define VQ_MASKS32(W, EA, EB)                        \
  VQ_MASKS(W)                                        \
  "v_and_or_b32 %[ta], " EA ", %[hb], %[ta]\n"       \
  "v_and_or_b32 %[tb], " EB ", %[hb], %[tb]\n"
template <int OFF>
__device__ __forceinline__ void k32_group(uint32_t w0, uint32_t w1, uint32_t e0, uint32_t e1, uint32_t e2,
                                          uint32_t e3, uint32_t hb, uint32_t base, uint32_t x0, uint32_t x1,
                                          float (&acc)[8]) {
  uint32_t ta, tb, r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11;
  asm volatile(
      VQ_MASKS32("%[w0]", "%[e0]", "%[e1]")
      VQ_SDWA_RD("%[r0]", "%[ta]", 0, 0) VQ_SDWA_RD("%[r1]", "%[tb]", 0, 0)
      VQ_SDWA_RD("%[r2]", "%[ta]", 1, 1) VQ_SDWA_RD("%[r3]", "%[tb]", 1, 1)
      VQ_SDWA_RD("%[r4]", "%[ta]", 2, 2) VQ_SDWA_RD("%[r5]", "%[tb]", 2, 2)
      VQ_SDWA_RD("%[r6]", "%[ta]", 3, 3) VQ_SDWA_RD("%[r7]", "%[tb]", 3, 3)
      VQ_MASKS32("%[w1]", "%[e2]", "%[e3]")
      VQ_SDWA_RD("%[r8]", "%[ta]", 0, 4) VQ_SDWA_RD("%[r9]", "%[tb]", 0, 4)
      VQ_SDWA_RD("%[r10]", "%[ta]", 1, 5) VQ_SDWA_RD("%[r11]", "%[tb]", 1, 5)
      "s_waitcnt lgkmcnt(4)\n"
      VQ_DOT("%[a0]", "%[r0]", "%[x0]") VQ_DOT("%[a1]", "%[r2]", "%[x0]")
      VQ_DOT("%[a2]", "%[r4]", "%[x0]") VQ_DOT("%[a3]", "%[r6]", "%[x0]")
      VQ_DOT("%[a0]", "%[r1]", "%[x1]") VQ_DOT("%[a1]", "%[r3]", "%[x1]")
      VQ_DOT("%[a2]", "%[r5]", "%[x1]") VQ_DOT("%[a3]", "%[r7]", "%[x1]")
      VQ_SDWA_RD("%[r0]", "%[ta]", 2, 6) VQ_SDWA_RD("%[r1]", "%[tb]", 2, 6)
      VQ_SDWA_RD("%[r2]", "%[ta]", 3, 7) VQ_SDWA_RD("%[r3]", "%[tb]", 3, 7)
      "s_waitcnt lgkmcnt(4)\n"
      VQ_DOT("%[a4]", "%[r8]", "%[x0]") VQ_DOT("%[a5]", "%[r10]", "%[x0]")
      VQ_DOT("%[a4]", "%[r9]", "%[x1]") VQ_DOT("%[a5]", "%[r11]", "%[x1]")
      "s_waitcnt lgkmcnt(0)\n"
      VQ_DOT("%[a6]", "%[r0]", "%[x0]") VQ_DOT("%[a7]", "%[r2]", "%[x0]")
      VQ_DOT("%[a6]", "%[r1]", "%[x1]") VQ_DOT("%[a7]", "%[r3]", "%[x1]")
      : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]),
        [a4] "+v"(acc[4]), [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]),
        [ta] "=&v"(ta), [tb] "=&v"(tb), [r0] "=&v"(r0), [r1] "=&v"(r1), [r2] "=&v"(r2),
        [r3] "=&v"(r3), [r4] "=&v"(r4), [r5] "=&v"(r5), [r6] "=&v"(r6), [r7] "=&v"(r7),
        [r8] "=&v"(r8), [r9] "=&v"(r9), [r10] "=&v"(r10), [r11] "=&v"(r11)
      : [w0] "v"(w0), [w1] "v"(w1), [e0] "v"(e0), [e1] "v"(e1), [e2] "v"(e2), [e3] "v"(e3), [hb] "s"(hb),
        [base] "s"(base), [x0] "v"(x0), [x1] "v"(x1), [off] "n"(OFF), [rs] "n"(0), [hs] "n"(0)
      : "memory");
}
#undef VQ_MASKS32
#undef VQ_SDWA_RD
#undef VQ_MASKS
#undef VQ_DOT

// The four shifted copies of a fifth-bit plane dword that k32_group takes, for the first (SLOT 0)
// or second (SLOT 1) col-block of a pair: set j of slot 0 sits at bits 6 - j of every byte, set j
// of slot 1 at bits 2 - j (j < 3) and at bit 7 (j = 3).
template <int SLOT>
__device__ __forceinline__ void k32_plane_sets(uint32_t e, uint32_t& e0, uint32_t& e1, uint32_t& e2, uint32_t& e3) {
  if constexpr (SLOT == 0) {
    e0 = e; e1 = e << 1; e2 = e << 2; e3 = e << 3;
  } else {
    e0 = e << 4; e1 = e << 5; e2 = e << 6; e3 = e >> 1;
  }
}
// The fifth bit of the index of (row r, vector 2L + t) of slot SLOT in a plane dword (plain form of the above).
__device__ __forceinline__ uint32_t k32_plane_bit(uint32_t e, int slot, int r, int t) {
  const int j = 2 * (r >> 2) + t;                      // the set
  const int pos = slot == 0 ? 6 - j : (j < 3 ? 2 - j : 7);
  return (e >> (8 * (r & 3) + pos)) & 1u;
}
__device__ __forceinline__ uint32_t k32_plane_encode(const uint32_t bits_a[16], const uint32_t bits_b[16]) {
  // bits_x[2 * r + t]: the fifth bit of (row r, vector 2L + t) of the pair's first / second col-block
  uint32_t e = 0;
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int j = 2 * (r >> 2) + t;
      e |= (bits_a[2 * r + t] & 1u) << (8 * (r & 3) + 6 - j);
      e |= (bits_b[2 * r + t] & 1u) << (8 * (r & 3) + (j < 3 ? 2 - j : 7));
    }
  return e;
}

// k = 16 inner block with blockwise normalisation, hand-scheduled (the streaming kernel's
// version of k16_group_scaled): per row the two centroid pairs and the row's block scale (a dword
// with the fp16 level in both halves, selected by the row's 4-bit code in cw) are looked up, both
// pairs are multiplied by the scale (one rounding: exactly the decoded weight) and go into the
// dot products.  Index bytes as in k16_group; the codes are spread once per block into two dwords
// of pre-scaled bytes (ca: 4 * code of rows 0, 2, 4, 6; cb: of rows 1, 3, 5, 7), so every address
// is one SDWA add.  Rows r + 4 are requested as soon as row r has been consumed: 9 to 12 LDS reads
// in flight.  OFF: byte offset of the group's table, LOFF: of its 16 level dwords.
#define VQ_B16_RD(R, T, B, OFF)                                                          \
  "v_add_u32_sdwa " R ", %[base], " T                                                    \
  " dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_" #B "\n"           \
  "ds_read_b32 " R ", " R " offset:" OFF "\n"
#define VQ_B16_ROW(RA, RB, RS, TA, TB, B, C, CB)                                         \
  VQ_B16_RD(RA, TA, B, "%[off]") VQ_B16_RD(RB, TB, B, "%[off]") VQ_B16_RD(RS, C, CB, "%[loff]")
#define VQ_B16_USE(ACC, RA, RB, RS)                      \
  "v_pk_mul_f16 " RA ", " RA ", " RS "\n"                \
  "v_pk_mul_f16 " RB ", " RB ", " RS "\n"                \
  "v_dot2c_f32_f16 " ACC ", " RA ", %[x0]\n"             \
  "v_dot2c_f32_f16 " ACC ", " RB ", %[x1]\n"
template <int OFF, int LOFF>
__device__ __forceinline__ void k16_group_bn(uint32_t w0, uint32_t w1, uint32_t cw, uint32_t base,
                                             uint32_t x0, uint32_t x1, float (&acc)[8]) {
  uint32_t r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11;
  const uint32_t ca = (cw << 2) & 0x3c3c3c3cu, cb = (cw >> 2) & 0x3c3c3c3cu;
  uint32_t ta0, tb0, ta1, tb1;
  k16_split_dword(w0, ta0, tb0);
  k16_split_dword(w1, ta1, tb1);
  asm volatile(
      VQ_B16_ROW("%[r0]", "%[r1]", "%[r2]", "%[ta0]", "%[tb0]", 0, "%[ca]", 0)
      VQ_B16_ROW("%[r3]", "%[r4]", "%[r5]", "%[ta0]", "%[tb0]", 1, "%[cb]", 0)
      VQ_B16_ROW("%[r6]", "%[r7]", "%[r8]", "%[ta0]", "%[tb0]", 2, "%[ca]", 1)
      VQ_B16_ROW("%[r9]", "%[r10]", "%[r11]", "%[ta0]", "%[tb0]", 3, "%[cb]", 1)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_B16_USE("%[a0]", "%[r0]", "%[r1]", "%[r2]")
      VQ_B16_ROW("%[r0]", "%[r1]", "%[r2]", "%[ta1]", "%[tb1]", 0, "%[ca]", 2)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_B16_USE("%[a1]", "%[r3]", "%[r4]", "%[r5]")
      VQ_B16_ROW("%[r3]", "%[r4]", "%[r5]", "%[ta1]", "%[tb1]", 1, "%[cb]", 2)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_B16_USE("%[a2]", "%[r6]", "%[r7]", "%[r8]")
      VQ_B16_ROW("%[r6]", "%[r7]", "%[r8]", "%[ta1]", "%[tb1]", 2, "%[ca]", 3)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_B16_USE("%[a3]", "%[r9]", "%[r10]", "%[r11]")
      VQ_B16_ROW("%[r9]", "%[r10]", "%[r11]", "%[ta1]", "%[tb1]", 3, "%[cb]", 3)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_B16_USE("%[a4]", "%[r0]", "%[r1]", "%[r2]")
      "s_waitcnt lgkmcnt(6)\n"
      VQ_B16_USE("%[a5]", "%[r3]", "%[r4]", "%[r5]")
      "s_waitcnt lgkmcnt(3)\n"
      VQ_B16_USE("%[a6]", "%[r6]", "%[r7]", "%[r8]")
      "s_waitcnt lgkmcnt(0)\n"
      VQ_B16_USE("%[a7]", "%[r9]", "%[r10]", "%[r11]")
      : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]),
        [a4] "+v"(acc[4]), [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]),
        [r0] "=&v"(r0), [r1] "=&v"(r1), [r2] "=&v"(r2), [r3] "=&v"(r3), [r4] "=&v"(r4),
        [r5] "=&v"(r5), [r6] "=&v"(r6), [r7] "=&v"(r7), [r8] "=&v"(r8), [r9] "=&v"(r9),
        [r10] "=&v"(r10), [r11] "=&v"(r11)
      : [ta0] "v"(ta0), [tb0] "v"(tb0), [ta1] "v"(ta1), [tb1] "v"(tb1), [ca] "v"(ca), [cb] "v"(cb),
        [base] "s"(base), [x0] "v"(x0), [x1] "v"(x1), [off] "n"(OFF), [loff] "n"(LOFF)
      : "memory");
}
#undef VQ_B16_RD
#undef VQ_B16_ROW
#undef VQ_B16_USE

// ---------------------------------------------------------------------------
// d = 1, k = 16 (scalar codebooks): a byte of the index stream holds the 4-bit indices of two
// neighbouring columns, low nibble first, and is used as one index into the 256-entry table
// of fp16 pairs T[j] = (c[j % 16], c[j / 16]).  A lane builds entries 4L..4L+3: `lo` holds
// c[4*(L%4) .. 4*(L%4)+3] (8 bytes at byte offset 8*(L%4) of the group's 32-byte codebook),
// `hi` holds c[L/4] in its low half (2 bytes at offset 2*(L/4)).
__device__ __forceinline__ uint4 d1_pair_entries(uint2 lo, uint32_t hi) {
  const uint32_t h = hi << 16;
  return make_uint4((lo.x & 0xffffu) | h, (lo.x >> 16) | h, (lo.y & 0xffffu) | h, (lo.y >> 16) | h);
}

// ---------------------------------------------------------------------------
// k = 256 inner block: the 16 lookups + dot products of one lane's share of one
// group (four dwords; byte 2r+e = row r, vector 2L+e), hand-scheduled like
// k16_group.  Address = base + OFF + 4*index: one v_bfe_u32 and one
// v_lshl_add_u32 per lookup (3 VALU instructions per vector with the dot2).
#define VQ_BFE_RD(R, W, BIT, OFF)                        \
  "v_bfe_u32 " R ", " W ", " #BIT ", 8\n"                \
  "v_lshl_add_u32 " R ", " R ", 2, %[base]\n"            \
  "ds_read_b32 " R ", " R " offset:" OFF "\n"
#define VQ_DOT(ACC, R, X) "v_dot2c_f32_f16 " ACC ", " R ", " X "\n"

template <int OFF>
__device__ __forceinline__ void k256_group(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3,
                                           uint32_t base, uint32_t x0, uint32_t x1,
                                           float (&acc)[8]) {
  uint32_t r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11;
  asm volatile(
      VQ_BFE_RD("%[r0]", "%[w0]", 0, "%[off]") VQ_BFE_RD("%[r1]", "%[w0]", 8, "%[off]")
      VQ_BFE_RD("%[r2]", "%[w0]", 16, "%[off]") VQ_BFE_RD("%[r3]", "%[w0]", 24, "%[off]")
      VQ_BFE_RD("%[r4]", "%[w1]", 0, "%[off]") VQ_BFE_RD("%[r5]", "%[w1]", 8, "%[off]")
      VQ_BFE_RD("%[r6]", "%[w1]", 16, "%[off]") VQ_BFE_RD("%[r7]", "%[w1]", 24, "%[off]")
      VQ_BFE_RD("%[r8]", "%[w2]", 0, "%[off]") VQ_BFE_RD("%[r9]", "%[w2]", 8, "%[off]")
      VQ_BFE_RD("%[r10]", "%[w2]", 16, "%[off]") VQ_BFE_RD("%[r11]", "%[w2]", 24, "%[off]")
      "s_waitcnt lgkmcnt(8)\n"
      VQ_DOT("%[a0]", "%[r0]", "%[x0]") VQ_DOT("%[a1]", "%[r2]", "%[x0]")
      VQ_DOT("%[a0]", "%[r1]", "%[x1]") VQ_DOT("%[a1]", "%[r3]", "%[x1]")
      VQ_BFE_RD("%[r0]", "%[w3]", 0, "%[off]") VQ_BFE_RD("%[r1]", "%[w3]", 8, "%[off]")
      VQ_BFE_RD("%[r2]", "%[w3]", 16, "%[off]") VQ_BFE_RD("%[r3]", "%[w3]", 24, "%[off]")
      "s_waitcnt lgkmcnt(8)\n"
      VQ_DOT("%[a2]", "%[r4]", "%[x0]") VQ_DOT("%[a3]", "%[r6]", "%[x0]")
      VQ_DOT("%[a2]", "%[r5]", "%[x1]") VQ_DOT("%[a3]", "%[r7]", "%[x1]")
      "s_waitcnt lgkmcnt(4)\n"
      VQ_DOT("%[a4]", "%[r8]", "%[x0]") VQ_DOT("%[a5]", "%[r10]", "%[x0]")
      VQ_DOT("%[a4]", "%[r9]", "%[x1]") VQ_DOT("%[a5]", "%[r11]", "%[x1]")
      "s_waitcnt lgkmcnt(0)\n"
      VQ_DOT("%[a6]", "%[r0]", "%[x0]") VQ_DOT("%[a7]", "%[r2]", "%[x0]")
      VQ_DOT("%[a6]", "%[r1]", "%[x1]") VQ_DOT("%[a7]", "%[r3]", "%[x1]")
      : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]),
        [a4] "+v"(acc[4]), [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]),
        [r0] "=&v"(r0), [r1] "=&v"(r1), [r2] "=&v"(r2), [r3] "=&v"(r3), [r4] "=&v"(r4),
        [r5] "=&v"(r5), [r6] "=&v"(r6), [r7] "=&v"(r7), [r8] "=&v"(r8), [r9] "=&v"(r9),
        [r10] "=&v"(r10), [r11] "=&v"(r11)
      : [w0] "v"(w0), [w1] "v"(w1), [w2] "v"(w2), [w3] "v"(w3), [base] "s"(base), [x0] "v"(x0),
        [x1] "v"(x1), [off] "n"(OFF)
      : "memory");
}
#undef VQ_BFE_RD
#undef VQ_DOT

// ---------------------------------------------------------------------------
// k = 64 inner block (6-bit indices): the lane's 16 indices of one 8-row block of a group
// are a little-endian 6-bit stream in three dwords d0..d2, index i = 2*row + e (vector
// 2L+e) at bits [6i, 6i+6).  Fields 5 and 10 straddle a dword boundary; the caller passes
// them aligned to bit 0 in t5 = alignbit(d1, d0, 30) and t10 = alignbit(d2, d1, 28).
// Per lookup: v_bfe_u32, v_lshl_add_u32 (index*4 + table base), ds_read_b32, v_dot2c.
#define VQ_BF6_RD(R, W, BIT, OFF)                        \
  "v_bfe_u32 " R ", " W ", " #BIT ", 6\n"                \
  "v_lshl_add_u32 " R ", " R ", 2, %[base]\n"            \
  "ds_read_b32 " R ", " R " offset:" OFF "\n"
#define VQ_DOT(ACC, R, X) "v_dot2c_f32_f16 " ACC ", " R ", " X "\n"

template <int OFF>
__device__ __forceinline__ void k64_group(uint32_t d0, uint32_t d1, uint32_t d2, uint32_t t5,
                                          uint32_t t10, uint32_t base, uint32_t x0, uint32_t x1,
                                          float (&acc)[8]) {
  uint32_t r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11;
  asm volatile(
      VQ_BF6_RD("%[r0]", "%[d0]", 0, "%[off]") VQ_BF6_RD("%[r1]", "%[d0]", 6, "%[off]")
      VQ_BF6_RD("%[r2]", "%[d0]", 12, "%[off]") VQ_BF6_RD("%[r3]", "%[d0]", 18, "%[off]")
      VQ_BF6_RD("%[r4]", "%[d0]", 24, "%[off]") VQ_BF6_RD("%[r5]", "%[t5]", 0, "%[off]")
      VQ_BF6_RD("%[r6]", "%[d1]", 4, "%[off]") VQ_BF6_RD("%[r7]", "%[d1]", 10, "%[off]")
      VQ_BF6_RD("%[r8]", "%[d1]", 16, "%[off]") VQ_BF6_RD("%[r9]", "%[d1]", 22, "%[off]")
      VQ_BF6_RD("%[r10]", "%[t10]", 0, "%[off]") VQ_BF6_RD("%[r11]", "%[d2]", 2, "%[off]")
      "s_waitcnt lgkmcnt(8)\n"
      VQ_DOT("%[a0]", "%[r0]", "%[x0]") VQ_DOT("%[a1]", "%[r2]", "%[x0]")
      VQ_DOT("%[a0]", "%[r1]", "%[x1]") VQ_DOT("%[a1]", "%[r3]", "%[x1]")
      VQ_BF6_RD("%[r0]", "%[d2]", 8, "%[off]") VQ_BF6_RD("%[r1]", "%[d2]", 14, "%[off]")
      VQ_BF6_RD("%[r2]", "%[d2]", 20, "%[off]") VQ_BF6_RD("%[r3]", "%[d2]", 26, "%[off]")
      "s_waitcnt lgkmcnt(8)\n"
      VQ_DOT("%[a2]", "%[r4]", "%[x0]") VQ_DOT("%[a3]", "%[r6]", "%[x0]")
      VQ_DOT("%[a2]", "%[r5]", "%[x1]") VQ_DOT("%[a3]", "%[r7]", "%[x1]")
      "s_waitcnt lgkmcnt(4)\n"
      VQ_DOT("%[a4]", "%[r8]", "%[x0]") VQ_DOT("%[a5]", "%[r10]", "%[x0]")
      VQ_DOT("%[a4]", "%[r9]", "%[x1]") VQ_DOT("%[a5]", "%[r11]", "%[x1]")
      "s_waitcnt lgkmcnt(0)\n"
      VQ_DOT("%[a6]", "%[r0]", "%[x0]") VQ_DOT("%[a7]", "%[r2]", "%[x0]")
      VQ_DOT("%[a6]", "%[r1]", "%[x1]") VQ_DOT("%[a7]", "%[r3]", "%[x1]")
      : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]),
        [a4] "+v"(acc[4]), [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]),
        [r0] "=&v"(r0), [r1] "=&v"(r1), [r2] "=&v"(r2), [r3] "=&v"(r3), [r4] "=&v"(r4),
        [r5] "=&v"(r5), [r6] "=&v"(r6), [r7] "=&v"(r7), [r8] "=&v"(r8), [r9] "=&v"(r9),
        [r10] "=&v"(r10), [r11] "=&v"(r11)
      : [d0] "v"(d0), [d1] "v"(d1), [d2] "v"(d2), [t5] "v"(t5), [t10] "v"(t10), [base] "s"(base),
        [x0] "v"(x0), [x1] "v"(x1), [off] "n"(OFF)
      : "memory");
}
#undef VQ_BF6_RD
#undef VQ_DOT

// k = 64 inner block with blockwise normalisation, hand-scheduled like k64_group: per row the
// two centroid pairs and the lane's block scale (a dword with the fp16 level in both halves,
// selected by the row's 4-bit code in cw) are looked up, both pairs are multiplied by the scale
// (v_pk_mul_f16: one rounding, exactly the decoded weight) and go into the dot products.  The
// lookups of row r + 4 are issued as soon as row r has been consumed, so 9 to 12 LDS reads are
// always in flight.  OFF: byte offset of the col-block's table, LOFF: of its 16 level dwords.
// The codes are spread once per block into two dwords of pre-scaled bytes (ca: 4 * code of rows
// 0, 2, 4, 6; cb: of rows 1, 3, 5, 7), so that a level's address is one SDWA add.
#define VQ_BN_RD(R, W, BIT, WIDTH, OFF)                  \
  "v_bfe_u32 " R ", " W ", " #BIT ", " #WIDTH "\n"       \
  "v_lshl_add_u32 " R ", " R ", 2, %[base]\n"            \
  "ds_read_b32 " R ", " R " offset:" OFF "\n"
#define VQ_BN_ROW(RA, WA, BA, RB, WB, BB, RS, ROW)                                       \
  VQ_BN_RD(RA, WA, BA, 6, "%[off]") VQ_BN_RD(RB, WB, BB, 6, "%[off]")                    \
  "v_add_u32_sdwa " RS ", %[base], %[c" #ROW "]"                                          \
  " dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_" VQ_BN_BYTE_##ROW "\n" \
  "ds_read_b32 " RS ", " RS " offset:%[loff]\n"
#define VQ_BN_BYTE_0 "0"
#define VQ_BN_BYTE_1 "0"
#define VQ_BN_BYTE_2 "1"
#define VQ_BN_BYTE_3 "1"
#define VQ_BN_BYTE_4 "2"
#define VQ_BN_BYTE_5 "2"
#define VQ_BN_BYTE_6 "3"
#define VQ_BN_BYTE_7 "3"
#define VQ_BN_USE(ACC, RA, RB, RS)                       \
  "v_pk_mul_f16 " RA ", " RA ", " RS "\n"                \
  "v_pk_mul_f16 " RB ", " RB ", " RS "\n"                \
  "v_dot2c_f32_f16 " ACC ", " RA ", %[x0]\n"             \
  "v_dot2c_f32_f16 " ACC ", " RB ", %[x1]\n"

template <int OFF, int LOFF>
__device__ __forceinline__ void k64_group_bn(uint32_t d0, uint32_t d1, uint32_t d2, uint32_t t5,
                                             uint32_t t10, uint32_t cw, uint32_t base, uint32_t x0,
                                             uint32_t x1, float (&acc)[8]) {
  uint32_t r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11;
  const uint32_t ca = (cw << 2) & 0x3c3c3c3cu, cb = (cw >> 2) & 0x3c3c3c3cu;
  asm volatile(
      VQ_BN_ROW("%[r0]", "%[d0]", 0, "%[r1]", "%[d0]", 6, "%[r2]", 0)
      VQ_BN_ROW("%[r3]", "%[d0]", 12, "%[r4]", "%[d0]", 18, "%[r5]", 1)
      VQ_BN_ROW("%[r6]", "%[d0]", 24, "%[r7]", "%[t5]", 0, "%[r8]", 2)
      VQ_BN_ROW("%[r9]", "%[d1]", 4, "%[r10]", "%[d1]", 10, "%[r11]", 3)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_BN_USE("%[a0]", "%[r0]", "%[r1]", "%[r2]")
      VQ_BN_ROW("%[r0]", "%[d1]", 16, "%[r1]", "%[d1]", 22, "%[r2]", 4)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_BN_USE("%[a1]", "%[r3]", "%[r4]", "%[r5]")
      VQ_BN_ROW("%[r3]", "%[t10]", 0, "%[r4]", "%[d2]", 2, "%[r5]", 5)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_BN_USE("%[a2]", "%[r6]", "%[r7]", "%[r8]")
      VQ_BN_ROW("%[r6]", "%[d2]", 8, "%[r7]", "%[d2]", 14, "%[r8]", 6)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_BN_USE("%[a3]", "%[r9]", "%[r10]", "%[r11]")
      VQ_BN_ROW("%[r9]", "%[d2]", 20, "%[r10]", "%[d2]", 26, "%[r11]", 7)
      "s_waitcnt lgkmcnt(9)\n"
      VQ_BN_USE("%[a4]", "%[r0]", "%[r1]", "%[r2]")
      "s_waitcnt lgkmcnt(6)\n"
      VQ_BN_USE("%[a5]", "%[r3]", "%[r4]", "%[r5]")
      "s_waitcnt lgkmcnt(3)\n"
      VQ_BN_USE("%[a6]", "%[r6]", "%[r7]", "%[r8]")
      "s_waitcnt lgkmcnt(0)\n"
      VQ_BN_USE("%[a7]", "%[r9]", "%[r10]", "%[r11]")
      : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3]),
        [a4] "+v"(acc[4]), [a5] "+v"(acc[5]), [a6] "+v"(acc[6]), [a7] "+v"(acc[7]),
        [r0] "=&v"(r0), [r1] "=&v"(r1), [r2] "=&v"(r2), [r3] "=&v"(r3), [r4] "=&v"(r4),
        [r5] "=&v"(r5), [r6] "=&v"(r6), [r7] "=&v"(r7), [r8] "=&v"(r8), [r9] "=&v"(r9),
        [r10] "=&v"(r10), [r11] "=&v"(r11)
      : [d0] "v"(d0), [d1] "v"(d1), [d2] "v"(d2), [t5] "v"(t5), [t10] "v"(t10),
        [c0] "v"(ca), [c1] "v"(cb), [c2] "v"(ca), [c3] "v"(cb), [c4] "v"(ca), [c5] "v"(cb), [c6] "v"(ca),
        [c7] "v"(cb), [base] "s"(base), [x0] "v"(x0), [x1] "v"(x1), [off] "n"(OFF), [loff] "n"(LOFF)
      : "memory");
}
#undef VQ_BN_RD
#undef VQ_BN_ROW
#undef VQ_BN_USE
#undef VQ_BN_BYTE_0
#undef VQ_BN_BYTE_1
#undef VQ_BN_BYTE_2
#undef VQ_BN_BYTE_3
#undef VQ_BN_BYTE_4
#undef VQ_BN_BYTE_5
#undef VQ_BN_BYTE_6
#undef VQ_BN_BYTE_7

// ---- 6-bit / int8-table device layout (k = 64) -------------------------------------------
// Indices: per (8-row block, quad of 4 col-blocks) three planes of 1 KB; the lane's 48 bytes
// are planes' bytes [16p, 16p+16), and col-block j of the quad is its dwords 3j..3j+2 (the
// 6-bit stream described at k64_group).  Tables: per (group row, quad) 528 bytes: four
// tables of 64 int8 pairs (128 B each), four fp16 scales, 8 bytes of padding.  Quads past
// the last col-block hold zero indices, zero tables and zero scales.
constexpr int kK64QuadIdxBytes = 3072;
constexpr int kK64QuadTabBytes = 528;
// With blockwise normalisation (appendix "Blockwise data normalization"; blocks of 32 weights,
// i.e. the 4 columns of 8 neighbouring lanes): the table record grows to 672 bytes, bytes
// [528, 656) being the four col-blocks' 16 fp16 block-scale levels; and behind all table records
// sit the 4-bit block codes, 128 bytes per (8-row block, quad): dword 4*b + j holds the codes of
// block b (lanes 8b .. 8b+7) of col-block j, row r in bits [4r, 4r+4), so a lane's four dwords
// are one 16-byte load.
// d = 1, k = 8 (3-bit indices; two neighbouring indices form the 6-bit index of the pair table
// T[j] = (c[j % 8], c[j / 8])): indices as for k = 64; the table record of a (group row, quad)
// is 48 bytes: four tables of 8 int8 values, four fp16 scales, 8 bytes of padding.
constexpr int kD1K8QuadTabBytes = 48;
constexpr int kD1K8ScaleOffset = 32;
// ... with blockwise normalisation: the 48-byte record, then the four col-blocks' 16 fp16 levels;
// the block codes behind all records exactly as for k = 64.
constexpr int kD1K8NQuadTabBytes = 176;
constexpr int kD1K8NLevelOffset = 48;
constexpr int kK64NQuadTabBytes = 672;
constexpr int kK64NLevelOffset = 528;
constexpr int kK64NQuadCodeBytes = 128;
__host__ __device__ __forceinline__ int k64_quads(int n_cb) { return (n_cb + 3) >> 2; }

// Centroid pair from two int8 table entries and the group's scale (Sec. 3.1: table and
// scale factor per group): the integers convert to fp16 exactly and one fp16 multiply
// rounds the exact product once, to nearest even.
__device__ __forceinline__ uint32_t k64_dequant_pair(uint32_t two_bytes, _Float16 scale) {
  h2_t v;
  v.x = (_Float16)(short)(signed char)(two_bytes & 0xffu);
  v.y = (_Float16)(short)(signed char)((two_bytes >> 8) & 0xffu);
  v = v * h2_t{scale, scale};
  return __builtin_bit_cast(uint32_t, v);
}

// k = 64 inner block with block scales, written in plain C++ (the compiler schedules it and
// takes care of the dot-product hazards itself): per row the lane's block scale S (fp16, both
// halves of a dword) is looked up from the 16 levels at lev[], both looked-up centroid pairs
// are multiplied by it (one fp16 rounding: exactly the decoded weight) and go into the dot2.
// tab: this col-block's 64-entry table, lev: its 16 level dwords, cw: the lane's code dword.
__device__ __forceinline__ void k64_group_scaled(uint32_t d0, uint32_t d1, uint32_t d2, uint32_t cw,
                                                 const uint32_t* tab, const uint32_t* lev,
                                                 uint32_t x0, uint32_t x1, float (&acc)[8]) {
  const unsigned long long lo = d0 | ((unsigned long long)d1 << 32);
  const h2_t xa = __builtin_bit_cast(h2_t, x0), xb = __builtin_bit_cast(h2_t, x1);
  uint32_t t[16], sv[8];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int pos = 6 * i;
    unsigned long long f = pos < 64 ? lo >> pos : (unsigned long long)(d2 >> (pos - 64));
    if (pos < 64 && pos > 58) f |= (unsigned long long)d2 << (64 - pos);
    t[i] = tab[(uint32_t)f & 63u];
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) sv[r] = lev[(cw >> (4 * r)) & 15u];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const h2_t sc = __builtin_bit_cast(h2_t, sv[r]);
    const h2_t ta = __builtin_bit_cast(h2_t, t[2 * r]) * sc;
    const h2_t tb = __builtin_bit_cast(h2_t, t[2 * r + 1]) * sc;
    acc[r] = __builtin_amdgcn_fdot2(ta, xa, acc[r], false);
    acc[r] = __builtin_amdgcn_fdot2(tb, xb, acc[r], false);
  }
}

// One fp16 pair times a block scale held in both halves of a dword (one rounding per half).
__device__ __forceinline__ uint32_t scale_pair(uint32_t pair, uint32_t scale2) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2_t, pair) * __builtin_bit_cast(h2_t, scale2));
}

// k = 256 inner block with block scales, in plain C++ like k64_group_scaled: w0 .. w3 hold the
// lane's 16 index bytes of one group (byte 2r + e = row r, vector 2L + e), cw its block codes
// (row r in bits [4r, 4r+4)), tab the group's 256 dequantised entries, lev its 16 level dwords.
__device__ __forceinline__ void k256_group_scaled(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3,
                                                  uint32_t cw, const uint32_t* tab, const uint32_t* lev,
                                                  uint32_t x0, uint32_t x1, float (&acc)[8]) {
  const uint32_t ws[4] = {w0, w1, w2, w3};
  const h2_t xa = __builtin_bit_cast(h2_t, x0), xb = __builtin_bit_cast(h2_t, x1);
  uint32_t t[16], sv[8];
#pragma unroll
  for (int i = 0; i < 16; ++i) t[i] = tab[(ws[i >> 2] >> (8 * (i & 3))) & 0xffu];
#pragma unroll
  for (int r = 0; r < 8; ++r) sv[r] = lev[(cw >> (4 * r)) & 15u];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    acc[r] = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2_t, scale_pair(t[2 * r], sv[r])), xa, acc[r], false);
    acc[r] = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2_t, scale_pair(t[2 * r + 1], sv[r])), xb, acc[r], false);
  }
}

// ---- d = 4 device layout (k = 256, int8 tables) ---------------------------------------------
// A lane owns ONE vector per row of a group: columns 4L .. 4L+3, one index byte.  Indices:
// per (8-row block, pair of col-blocks) 1 KB; the lane's 16 bytes are its 8 row bytes of the
// first col-block, then of the second (zero if the matrix has an odd number of col-blocks).
// Tables: as in the canonical buffer, 1 KB of int8 (256 entries x 4) per group in group order,
// then one fp16 scale per group.
__device__ __forceinline__ uint2 d4_dequant_entry(uint32_t four_bytes, _Float16 scale) {
  return make_uint2(k64_dequant_pair(four_bytes, scale), k64_dequant_pair(four_bytes >> 16, scale));
}

// d = 1, k = 8: the int8 pair (c[e % 8], c[e / 8]) of pair-table entry e from the group's 8 values.
__device__ __forceinline__ uint32_t d1k8_pair(uint2 c8, int e) {
  const uint32_t lo = ((e & 4) ? c8.y : c8.x) >> (8 * (e & 3));
  const uint32_t hi = ((e & 32) ? c8.y : c8.x) >> (8 * ((e >> 3) & 3));
  return (lo & 0xffu) | ((hi & 0xffu) << 8);
}

// d = 1, k = 4 (2-bit indices, one codebook of 4 int8 values + fp16 scale per row of a
// col-block): two neighbouring indices form the 4-bit index of the row's pair table
// T[j] = (c[j % 4], c[j / 4]); indices in the 4-bit device layout above.  Tables: per (8-row
// block, col-block slot) 48 bytes: the 8 rows' 4 values, then the 8 rows' scales.
constexpr int kD1K4SlotTabBytes = 48;
constexpr int kD1K4ScaleOffset = 32;
// The int8 pair (c[j % 4], c[j / 4]) of pair-table entry j from a row's 4 values.
__device__ __forceinline__ uint32_t d1k4_pair(uint32_t c4, int j) {
  return ((c4 >> (8 * (j & 3))) & 0xffu) | (((c4 >> (8 * (j >> 2))) & 0xffu) << 8);
}
// Entries 8*half .. 8*half+7 of a row's pair table from its dequantised values p01 = (c0, c1),
// p23 = (c2, c3): the low halves run through c0..c3 twice, the high half is c[2*half], then c[2*half+1].
__device__ __forceinline__ void d1k4_entries(uint32_t p01, uint32_t p23, int half, uint4& e0, uint4& e1) {
  const uint32_t hp = half ? p23 : p01;
  const uint32_t ha = hp << 16, hb = hp & 0xffff0000u;
  const uint32_t c0 = p01 & 0xffffu, c1 = p01 >> 16, c2 = p23 & 0xffffu, c3 = p23 >> 16;
  e0 = make_uint4(c0 | ha, c1 | ha, c2 | ha, c3 | ha);
  e1 = make_uint4(c0 | hb, c1 | hb, c2 | hb, c3 | hb);
}

// Pairs of col-blocks a k=16 row-block is stored as (the last one half-empty if n_cb is odd).
__host__ __device__ __forceinline__ int k16_pairs(int n_cb) { return (n_cb + 1) >> 1; }

// Byte offset, inside its row-block, of lane `lane`'s 8-byte share of 4-bit group c.
__device__ __forceinline__ size_t k16_chunk_offset(int c, int lane) {
  return (size_t)(c >> 1) * 1024 + lane * 16 + (c & 1) * 8;
}

// One device dword of 4-bit indices from its 4 (lo, hi) index pairs, and back to
// "4*index per byte" form (a: the lo indices, b: the hi indices).
__device__ __forceinline__ uint32_t k16_encode_dword(const uint32_t lo[4], const uint32_t hi[4]) {
  uint32_t w = 0;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    w |= (lo[b] << 2) << (8 * b);
    w |= (hi[b] & 3u) << (8 * b + 6);
    w |= (hi[b] >> 2) << (8 * ((b + 1) & 3));
  }
  return w;
}

// ---- k = 16 with int8 tables and blockwise normalisation: device layout of the table buffer ----
// (S = group slots of the matrix = row-blocks x 2 x col-block pairs; pad slots are all zero)
//   [0, 32 S)              int8 tables, 32 bytes per slot                      (as without BN)
//   [32 S, 34 S)           one fp16 scale per slot                             (as without BN)
//   [A, A + 32 S)          A = 34 S rounded up to 16: the slot's 16 fp16 levels
//   [A + 32 S, A + 64 S)   block codes, 64 bytes per col-block pair: dword 2b + e holds the codes of
//                          block b (lanes 8b .. 8b+7: 32 columns) of the pair's col-block e, row r in
//                          bits [4r, 4r+4): a lane's codes of a pair are one 8-byte load
// (offsets: k16bn_level_offset, k16bn_code_offset, k16bn_table_bytes in vq_internal.h)

// k = 16 inner block with block scales, in plain C++ like k64_group_scaled: w0 / w1 hold rows
// 0..3 / 4..7 in the pre-scaled 4-bit layout, cw the lane's code dword; tab: the group's 16-entry
// table, lev: its 16 level dwords (fp16 in both halves).  Each looked-up centroid pair is
// multiplied by the row's block scale (one fp16 rounding: exactly the decoded weight).
__device__ __forceinline__ void k16_group_scaled(uint32_t w0, uint32_t w1, uint32_t cw, const uint32_t* tab,
                                                 const uint32_t* lev, uint32_t x0, uint32_t x1,
                                                 float (&acc)[8]) {
  const h2_t xa = __builtin_bit_cast(h2_t, x0), xb = __builtin_bit_cast(h2_t, x1);
  const char* tb = reinterpret_cast<const char*>(tab);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    uint32_t a, b;
    k16_split_dword(h ? w1 : w0, a, b);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const h2_t sc = __builtin_bit_cast(h2_t, lev[(cw >> (4 * (4 * h + r))) & 15u]);
      const h2_t ta = __builtin_bit_cast(h2_t, *reinterpret_cast<const uint32_t*>(tb + ((a >> (8 * r)) & 0xffu))) * sc;
      const h2_t tv = __builtin_bit_cast(h2_t, *reinterpret_cast<const uint32_t*>(tb + ((b >> (8 * r)) & 0xffu))) * sc;
      acc[4 * h + r] = __builtin_amdgcn_fdot2(ta, xa, acc[4 * h + r], false);
      acc[4 * h + r] = __builtin_amdgcn_fdot2(tv, xb, acc[4 * h + r], false);
    }
  }
}


// Sum 8 per-lane row accumulators over the 64 lanes.  Returns, in every lane, the
// total of row (lane >> 3) & 7.  Halving exchange without LDS traffic: the two
// cross-row steps use the gfx950 lane-swap instructions (v_permlane32_swap exchanges
// the upper half of its first operand with the lower half of its second, so that
// "first + second" adds lanes l and l^32 of one accumulator in the lower half and of
// the other accumulator in the upper half; v_permlane16_swap does the same for the
// odd rows of the first operand and the even rows of the second), the steps inside
// a row of 16 lanes use DPP.  The s_nop around the swaps are the wait states between a
// VALU write and a lane swap (and back) that the compiler cannot see inside asm.
template <int CTRL> __device__ __forceinline__ float dpp_read(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_reduce8(const float (&a)[8], int lane) {
  float b[4], c[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float lo = a[i], hi = a[i + 4];
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(lo), "+v"(hi));
    b[i] = lo + hi;            // lanes 0..31: row i, lanes 32..63: row i + 4
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    float lo = b[i], hi = b[i + 2];
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(lo), "+v"(hi));
    c[i] = lo + hi;            // even rows of 16 lanes: row i (+4), odd rows: row i + 2 (+4)
  }
  const bool up = lane & 8;
  const float send = up ? c[0] : c[1];
  const float keep = up ? c[1] : c[0];
  float v = keep + dpp_read<0x128>(send);      // row_ror:8 = lane ^ 8 inside a row of 16
  v += dpp_read<0x141>(v);                      // row_half_mirror: the other quad of the 8 lanes
  v += dpp_read<0x4E>(v);                       // quad_perm [2,3,0,1]
  v += dpp_read<0xB1>(v);                       // quad_perm [1,0,3,2]
  return v;
}

}  // namespace vq
