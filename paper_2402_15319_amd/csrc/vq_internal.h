// Internal declarations shared by the translation units of libvq (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/vq.h"

namespace vq {

constexpr int kGroupRows = 8;
constexpr int kGroupCols = 256;
constexpr int kMaxProblemsPerLaunch = 256;  // the problem table travels in the kernel arguments (14 KB)
// Kernel format tags: the codebook size for d = 2 with fp16 codebooks (16, 256) and for k = 64
// (always int8 tables); k = 16 with int8 tables and the scalar (d = 1) format have tags of
// their own.  d = 1, k = 16: two neighbouring 4-bit indices form one byte, which indexes a
// 256-entry table of fp16 pairs T[j] = (c[j % 16], c[j / 16]) that the kernels build in LDS from
// the group's 16 scalars; from there on the work is that of d = 2, k = 256.
constexpr int kFmtK16I8 = 1016;
constexpr int kFmtK16I8H = 1416;   // k = 16, int8 tables + scale, groups of 4 rows x 256 columns (two tables per 8-row block)
constexpr int kFmtK32 = 1032;     // k = 32 (5-bit indices), int8 tables + scale, 8 x 256 groups.  Indices: the low four bits
                                  // of every index in the k = 16 layout (1 KB per col-block pair); behind the nibbles of
                                  // the whole matrix, the fifth bits: 256 bytes per (8-row block, pair), one dword per
                                  // lane (bit positions: k32_plane_encode in vq_device.h).  Tables: 64 bytes per group
                                  // slot, then one fp16 scale per slot.
constexpr int kFmtK256I8 = 1256;   // d = 2, k = 256, int8 tables + scale, groups of 64, 128 or 256 rows x 256 columns
constexpr int kFmtD1K16 = 2016;
constexpr int kFmtK64BN = 3064;   // k = 64, int8 tables + scale, blockwise normalisation (blocks of 32)
constexpr int kFmtD1K8BN = 3008;  // d = 1, k = 8, int8 values + scale, blockwise normalisation
constexpr int kFmtK16BN = 3016;   // k = 16, int8 tables + scale, blockwise normalisation (blocks of 32)
constexpr int kFmtD1K8 = 2008;     // d = 1, k = 8 (3-bit indices), int8 values + scale: pairs index a 64-entry pair table
constexpr int kFmtD1K4 = 2004;     // d = 1, k = 4 (2-bit indices), int8 values + scale, one codebook per row of a
                                   // col-block (groups of 1 x 256): pairs index a 16-entry pair table per row
constexpr int kFmtD4 = 4256;      // d = 4, k = 256 (one index byte per 4 weights), int8 tables + scale,
                                  // groups of 64, 128 or 256 rows x 256 columns
constexpr int kFmtD4F16 = 4257;   // the same with fp16 tables (2 KB per group, no scale)
constexpr int kFmtD4BN = 4258;    // d = 4 with int8 tables + scale and blockwise normalisation (blocks of 32)
constexpr int kFmtK256I8BN = 1257;   // d = 2, k = 256 with int8 tables + scale and blockwise normalisation
inline int format_tag(const vq_desc& d) {
  if (d.d == 1) return d.k == 8 ? (d.codebook_dtype == VQ_I8_BN ? kFmtD1K8BN : kFmtD1K8) : d.k == 4 ? kFmtD1K4 : kFmtD1K16;
  if (d.d == 4) return d.codebook_dtype == VQ_F16 ? kFmtD4F16 : d.codebook_dtype == VQ_I8_BN ? kFmtD4BN : kFmtD4;
  if (d.codebook_dtype == VQ_I8_BN) return d.k == 16 ? kFmtK16BN : d.k == 256 ? kFmtK256I8BN : kFmtK64BN;
  if (d.k == 16 && d.codebook_dtype == VQ_I8) return d.group_rows == 4 ? kFmtK16I8H : kFmtK16I8;
  if (d.k == 32) return kFmtK32;
  if (d.k == 256 && d.codebook_dtype == VQ_I8) return kFmtK256I8;
  return d.k;
}
// k = 16 with int8 tables and blockwise normalisation: byte offsets of the levels and of the block
// codes inside the device-layout table buffer of a matrix with n_slots group slots, and its size
// (the layout itself is described in vq_device.h).
__host__ __device__ constexpr size_t k16bn_level_offset(size_t n_slots) { return (34 * n_slots + 15) / 16 * 16; }
__host__ __device__ constexpr size_t k16bn_code_offset(size_t n_slots) { return k16bn_level_offset(n_slots) + 32 * n_slots; }
__host__ __device__ constexpr size_t k16bn_table_bytes(size_t n_slots) { return k16bn_code_offset(n_slots) + 32 * n_slots; }
// The formats whose tables are shared by 64 or more rows (d = 4, and d = 2 with k = 256 and int8
// tables), with blockwise normalisation: the table buffer is the canonical one up to and including
// the levels (tables of tab_bytes each, scales padded to 16 bytes, 32 bytes of levels per group);
// then 64 bytes of block codes per (8-row block, pair of col-blocks): dword 2b + e holds the codes
// of block b (lanes 8b .. 8b+7) of the pair's col-block e, row r in bits [4r, 4r+4).
__host__ __device__ constexpr size_t wide_bn_level_offset(size_t n_groups, size_t tab_bytes) {
  return n_groups * tab_bytes + (2 * n_groups + 15) / 16 * 16;
}
__host__ __device__ constexpr size_t wide_bn_code_offset(size_t n_groups, size_t tab_bytes) {
  return wide_bn_level_offset(n_groups, tab_bytes) + 32 * n_groups;
}
constexpr int kStreamMaxColBlocks = 96;   // widest x the streaming kernel stages in LDS (48 KB)

// One matrix-vector product as the kernels see it (lives in the kernel arguments).
struct GemvProblem {
  const uint8_t* idx;   // device-layout indices
  const uint32_t* cb;   // codebooks, one dword (fp16 pair) per centroid
  const uint16_t* x;    // fp16 activations
  void* y;              // fp16 or fp32 output
  int32_t n_rb;         // row-blocks  (out / 8)
  int32_t n_cb;         // col-blocks  (in / 256)
  int32_t wg_begin;     // first work item of this problem inside the launch (see launch_gemv)
  int32_t splits;       // waves sharing one row-block: 1, 2, 4 or 8
  int32_t cost_begin;   // groups of all earlier problems of the launch (streaming kernel)
  int32_t rb_per_cb;    // 8-row blocks that share one codebook (group_rows / 8)
};

struct GemvBatch {
  int32_t count;
  int32_t y_f32;
  int32_t total_wgs;    // work items in the launch
  int32_t total_cost;   // groups in the launch
  GemvProblem p[kMaxProblemsPerLaunch];
};

// Low-rank adapter of one problem (y = W x + B (A x)): what the GEMV epilogue needs.
struct LoraProblem {
  const uint16_t* B;    // fp16 [out, rank] row-major
  const float* t;       // t = A x, fp32 [rank] (written by the adapter's first kernel)
  int32_t rank;         // 0 (no adapter) or a multiple of 8 up to kMaxLoraRank
  int32_t pad;
};
constexpr int kMaxLoraRank = 64;
constexpr int kLoraWorkspaceFloats = kMaxLoraRank;   // fp32 slots of workspace per problem

struct GemvBatchLora {
  GemvBatch base;
  LoraProblem l[kMaxProblemsPerLaunch];
};

// t = A x of every problem of a launch: one wave per row of A.
struct LoraDownProblem {
  const uint16_t* A;    // fp16 [rank, in] row-major
  const uint16_t* x;    // fp16 [in]
  float* t;             // fp32 [rank]
  int32_t in_features;
  int32_t row_begin;    // rows of A of all earlier problems of the launch
};
struct LoraDownBatch {
  int32_t count;
  int32_t total_rows;
  LoraDownProblem p[kMaxProblemsPerLaunch];
};

// Launchers (each returns the hipError_t of its launch).
hipError_t launch_pack(const vq_desc& d, const void* idx_canon, const void* cb_canon,
                       void* idx_dev, void* cb_dev, hipStream_t s);
hipError_t launch_decode(const vq_desc& d, const void* idx_dev, const void* cb_dev,
                         void* W, hipStream_t s);
// mode 1: persistent streaming kernel (total_cost/cost_begin are used, grid_wgs workgroups, x
// of up to max_n_cb col-blocks staged in LDS); mode 0: split-K kernel, wg_begin/total_wgs count
// workgroups (= grid_wgs); modes 2, 3, 4: split-K kernel for launches whose strips all fit in one,
// two or three chunks (all of them loaded at once);
// wpw: waves per workgroup of the split-K kernel (4, or 8 when 8 waves share a row-block; strips
// longer than one chunk only occur with 8).
hipError_t launch_gemv(int fmt, const GemvBatch& batch, int mode, int grid_wgs,
                       int max_n_cb, hipStream_t s, int wpw);
// The same kernels with the low-rank adapter term added to every row before it is stored, and
// the kernel that computes t = A x for the problems of a launch.
hipError_t launch_gemv_lora(int fmt, const GemvBatchLora& batch, int mode, int grid_wgs,
                            int max_n_cb, hipStream_t s, int wpw);
int gemv_stream_resident_wgs_lora(int fmt, int max_n_cb);
hipError_t launch_lora_down(const LoraDownBatch& batch, hipStream_t s);
// Dynamic LDS of the persistent GEMV kernel for x of up to max_n_cb col-blocks.
size_t gemv_stream_lds_bytes(int fmt, int max_n_cb);
// Workgroups of the persistent GEMV kernel that fit on the current device at once.
int gemv_stream_resident_wgs(int fmt, int max_n_cb);
// Units (col-block pairs, quads or col-blocks, by format) that one chunk of the GEMV kernels holds.
int gemv_chunk_units(int fmt);
// d = 4, and d = 2 with k = 256 and int8 tables: GEMV kernels of their own (a workgroup of 8 waves
// owns 64 rows and shares the group's dequantised table; see vq_gemv_d4.hip).
// fmt: kFmtD4, kFmtD4F16 or kFmtD4BN; kFmtK256I8 or kFmtK256I8BN.
hipError_t launch_gemv_d4(const GemvBatch& batch, int total_wgs, hipStream_t s, int fmt);
hipError_t launch_gemv_k256i8(const GemvBatch& batch, int total_wgs, hipStream_t s, int fmt);
hipError_t launch_gemv_d4_lora(const GemvBatchLora& batch, int total_wgs, hipStream_t s, int fmt);
hipError_t launch_gemv_k256i8_lora(const GemvBatchLora& batch, int total_wgs, hipStream_t s, int fmt);
hipError_t launch_gemm(const vq_desc& d, const void* idx_dev, const void* cb_dev,
                       const void* X, int B, int ldx, void* Y, int ldy, int y_f32,
                       hipStream_t s);

// E- and M-step of the codebook initialisation (d in {1, 2, 4}, k in {4, 8, 16, 32, 64, 256}, groups
// of 1, 4, 8, 16, 32, 64, 128 or 256 rows x 256 columns; one row only with k * d <= 64, 4 rows
// only with d <= 2).
hipError_t launch_em_assign(const vq_desc& d, const void* W, const void* hdiag, const void* cb,
                            void* assign, hipStream_t s);
hipError_t launch_em_update(const vq_desc& d, const void* W, const void* hdiag, const void* assign,
                            void* cb_out, hipStream_t s);

}  // namespace vq
