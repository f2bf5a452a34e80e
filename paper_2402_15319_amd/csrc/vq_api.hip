// C ABI of libvq: argument validation on the host, then one launch per call (two for the
// widest batched products).  Nothing here allocates or synchronises; the only state the
// library keeps is a cache of device-dependent launch parameters (compute units, resident
// workgroups of the streaming kernel, the address of the static adapter scratch).
#include <stddef.h>
#include <string.h>
#include <atomic>
#include "vq_internal.h"

namespace {

using namespace vq;

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// The representations the kernels implement (d = 2 unless stated):
//   fp16 codebooks, 8 x 256 groups, k = 16 (4-bit indices) or 256 (8-bit);
//   int8 tables with one fp16 scale per group: k = 64 (6-bit indices), groups of 8, 16 or 32
//   rows x 256 columns (32 rows = the 8,192-weight groups of Sec. 5.1), or k = 16 with 8 x 256
//   groups (2.125 bits per value), or k = 256 with groups of 64, 128 or 256 rows x 256 columns
//   (128 rows: the 2D 4.125 row of the appendix table); k = 64 and k = 16 also with blockwise
//   normalisation (VQ_I8_BN);
//   d = 1 (scalar codebooks): k = 16 fp16 values per 8 x 256 group, 4-bit indices (4.125 bits
//   per value, the overhead of the 1D 4.125 row of the appendix table of VQ configurations);
//   d = 1, k = 8: 3-bit indices, 8 int8 values + scale per group of 8, 16 or 32 rows x 256 columns
//   (32 rows: the 1D 3.125 row of that table);
//   d = 1, k = 4: 2-bit indices, 4 int8 values + scale per row of a 256-column block (groups of
//   1 x 256: the 1D 2.125 row of that table);
//   d = 4: k = 256 (one index byte per 4 weights), int8 tables with a scale, groups of 64, 128 or
//   256 rows x 256 columns (128 and 256: the 4D 2.25 and 2.125 rows of that table); also with fp16
//   tables (2 KB per group).
bool is_i8(const vq_desc& d) { return d.codebook_dtype == VQ_I8 || d.codebook_dtype == VQ_I8_BN; }
bool is_bn(const vq_desc& d) { return d.codebook_dtype == VQ_I8_BN; }

int check_desc(const vq_desc* d) {
  if (!d) return VQ_ERR_NULL;
  if (d->out_features <= 0 || d->in_features <= 0 || d->group_rows <= 0 || d->group_cols <= 0 ||
      d->d <= 0 || d->k <= 0 || d->index_bits <= 0 || d->index_bits > 16)
    return VQ_ERR_BAD_DESC;
  if (!is_pow2(d->k) || d->k != (1 << d->index_bits)) return VQ_ERR_BAD_DESC;
  if (d->group_cols % d->d) return VQ_ERR_BAD_DESC;
  if (d->codebook_dtype != VQ_F16 && !is_i8(*d)) return VQ_ERR_UNSUPPORTED;
  if ((d->d != 2 && d->d != 1 && d->d != 4) || d->group_cols != kGroupCols) return VQ_ERR_UNSUPPORTED;
  if (d->d == 1) {
    if (d->k == 8) {          // 3-bit indices, int8 values + scale (also block-normalised), group heights of the k = 64 format
      if (!is_i8(*d)) return VQ_ERR_UNSUPPORTED;
      if (d->group_rows != 8 && d->group_rows != 16 && d->group_rows != 32) return VQ_ERR_UNSUPPORTED;
    } else if (d->k == 4) {   // 2-bit indices, int8 values + scale, one codebook per row of a col-block
      if (d->codebook_dtype != VQ_I8 || d->group_rows != 1) return VQ_ERR_UNSUPPORTED;
      if (d->out_features % kGroupRows) return VQ_ERR_UNSUPPORTED;
    } else if (d->k != 16 || is_i8(*d) || d->group_rows != kGroupRows) {
      return VQ_ERR_UNSUPPORTED;
    }
  } else if (d->d == 4) {                     // int8 tables with a scale (also block-normalised), or fp16 tables
    if (d->k != 256) return VQ_ERR_UNSUPPORTED;
    if (d->group_rows != 64 && d->group_rows != 128 && d->group_rows != 256) return VQ_ERR_UNSUPPORTED;
  } else if (is_i8(*d)) {
    if (d->k == 64) {
      if (d->group_rows != 8 && d->group_rows != 16 && d->group_rows != 32) return VQ_ERR_UNSUPPORTED;
    } else if (d->k == 16) {                  // 8 x 256 groups, with or without blockwise normalisation; or 4 x 256 groups
      if (d->group_rows != kGroupRows && !(d->group_rows == 4 && !is_bn(*d))) return VQ_ERR_UNSUPPORTED;
    } else if (d->k == 32) {                  // 5-bit indices (the 2.5-bits-per-dimension rows): 8 x 256 groups
      if (d->group_rows != kGroupRows || is_bn(*d)) return VQ_ERR_UNSUPPORTED;
    } else if (d->k == 256) {                 // the 4-bits-per-dimension 2D setting: large groups share a table
      if (d->group_rows != 64 && d->group_rows != 128 && d->group_rows != 256) return VQ_ERR_UNSUPPORTED;
    } else {
      return VQ_ERR_UNSUPPORTED;
    }
  } else {
    if (d->k != 16 && d->k != 256) return VQ_ERR_UNSUPPORTED;
    if (d->group_rows != kGroupRows) return VQ_ERR_UNSUPPORTED;
  }
  if (d->out_features % d->group_rows || d->out_features % kGroupRows || d->in_features % kGroupCols)
    return VQ_ERR_UNSUPPORTED;
  // index arithmetic inside the kernels uses 32-bit element offsets into x / rows
  if ((long long)d->out_features * d->in_features > (1ll << 40)) return VQ_ERR_UNSUPPORTED;
  return VQ_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

void sizes(const vq_desc& d, size_t* idx_bytes, size_t* cb_bytes) {
  const size_t n_groups = (size_t)(d.out_features / d.group_rows) * (d.in_features / d.group_cols);
  const size_t vecs = (size_t)d.group_rows * d.group_cols / d.d;
  if (idx_bytes) *idx_bytes = n_groups * (vecs * d.index_bits / 8);
  if (cb_bytes) {
    if (is_bn(d))   // tables and scales padded to 16 bytes each, 16 fp16 levels per group, 4-bit codes
      *cb_bytes = (n_groups * (size_t)d.k * d.d + 15) / 16 * 16 + (2 * n_groups + 15) / 16 * 16 +
                  32 * n_groups + (size_t)d.out_features * (d.in_features / 32) / 2;
    else if (is_i8(d))   // int8 tables padded to 16 bytes, then one fp16 scale per group
      *cb_bytes = (n_groups * (size_t)d.k * d.d + 15) / 16 * 16 + 2 * n_groups;
    else
      *cb_bytes = n_groups * (size_t)d.k * d.d * 2;
  }
}

// Units a row-block of `n_cb` col-blocks is cut into (what the strips of the GEMV kernels count).
int strip_units(int fmt, int n_cb) {
  return (fmt == 16 || fmt == kFmtK16I8 || fmt == kFmtK16BN || fmt == kFmtK16I8H || fmt == kFmtK32 || fmt == kFmtD1K4) ? (n_cb + 1) / 2 : (fmt == 64 || fmt == kFmtK64BN || fmt == kFmtD1K8 || fmt == kFmtD1K8BN) ? (n_cb + 3) / 4 : n_cb;
}

int hip_status(hipError_t e) { return e == hipSuccess ? VQ_OK : VQ_ERR_HIP; }

// The quantiser kernels work on fp32 weights and codebooks; codebook_dtype plays no part.
int check_em_desc(const vq_desc* d) {
  if (!d) return VQ_ERR_NULL;
  if (d->out_features <= 0 || d->in_features <= 0 || d->group_rows <= 0 || d->group_cols <= 0 ||
      d->d <= 0 || d->k <= 0 || d->index_bits <= 0 || d->index_bits > 16)
    return VQ_ERR_BAD_DESC;
  if (!is_pow2(d->k) || d->k != (1 << d->index_bits)) return VQ_ERR_BAD_DESC;
  if ((d->d != 1 && d->d != 2 && d->d != 4) || d->group_cols != kGroupCols) return VQ_ERR_UNSUPPORTED;
  if (d->k != 4 && d->k != 8 && d->k != 16 && d->k != 32 && d->k != 64 && d->k != 256) return VQ_ERR_UNSUPPORTED;
  const int gr = d->group_rows;
  if (gr != 1 && gr != 4 && gr != 8 && gr != 16 && gr != 32 && gr != 64 && gr != 128 && gr != 256) return VQ_ERR_UNSUPPORTED;
  if (gr == 1 && d->k * d->d > 64) return VQ_ERR_UNSUPPORTED;   // a codebook per row: small codebooks only
  if (gr == 4 && d->d == 4) return VQ_ERR_UNSUPPORTED;          // groups of 4 rows: d = 1 or 2
  if (d->out_features % (gr > kGroupRows ? gr : kGroupRows) || d->in_features % kGroupCols) return VQ_ERR_UNSUPPORTED;
  if ((long long)d->out_features * d->in_features > (1ll << 40)) return VQ_ERR_UNSUPPORTED;
  return VQ_OK;
}

// Scratch of vq_gemv_lora_multi_static: t = A x of up to kStaticLoraProblems products, in place of
// the caller's workspace.  One copy per GPU, held until the process ends.  In host code the
// array's name is only a handle; its device address on the current GPU comes from
// hipGetSymbolAddress and is what kernels and copies are given.
constexpr int kStaticLoraProblems = kMaxProblemsPerLaunch;
static __device__ __align__(256) float scratch[kStaticLoraProblems * kLoraWorkspaceFloats];   // 64 KB
constexpr int kMaxDevices = 64;
std::atomic<float*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current GPU (asked once per device, then cached).
int static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return VQ_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return VQ_ERR_UNSUPPORTED;
  float* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) {
      (void)hipGetLastError();
      return VQ_ERR_HIP;
    }
    p = static_cast<float*>(sym);
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread computes the same address
  }
  *out = p;
  return VQ_OK;
}

// The body of vq_gemv_multi and of its variants with a low-rank adapter (lora != NULL: t_ws is
// device memory for kLoraWorkspaceFloats floats per problem, t = A x of problem i at slot i).
int gemv_multi_impl(int count, const vq_desc* descs, const void* const* idx_dev,
                    const void* const* cb_dev, const void* const* x_f16, void* const* y,
                    int y_dtype, void* stream, const vq_lora_desc* lora, float* t_ws,
                    bool validate_only = false) {
  if (count < 1 || count > 65536) return VQ_ERR_BAD_ARG;
  if (!descs || !idx_dev || !cb_dev || !x_f16 || !y) return VQ_ERR_NULL;
  if (y_dtype != VQ_F16 && y_dtype != VQ_F32) return VQ_ERR_BAD_ARG;
  for (int i = 0; i < count; ++i) {
    const int st = check_desc(&descs[i]);
    if (st != VQ_OK) return st;
    if (format_tag(descs[i]) != format_tag(descs[0])) return VQ_ERR_BAD_ARG;
    if (!idx_dev[i] || !cb_dev[i] || !x_f16[i] || !y[i]) return VQ_ERR_NULL;
    if (!aligned16(idx_dev[i]) || !aligned16(cb_dev[i]) || !aligned16(x_f16[i]) || !aligned16(y[i]))
      return VQ_ERR_ALIGN;
    if (x_f16[i] == (const void*)y[i]) return VQ_ERR_BAD_ARG;
    if (lora) {
      const vq_lora_desc& l = lora[i];
      if (l.rank < 0 || l.rank > kMaxLoraRank || (l.rank & 7)) return VQ_ERR_BAD_ARG;
      if (l.rank > 0) {
        if (!l.A_f16 || !l.B_f16) return VQ_ERR_NULL;
        if (!aligned16(l.A_f16) || !aligned16(l.B_f16)) return VQ_ERR_ALIGN;
      }
    }
  }
  if (validate_only) return VQ_OK;
  for (int first = 0; first < count; first += kMaxProblemsPerLaunch) {
    const int n = count - first < kMaxProblemsPerLaunch ? count - first : kMaxProblemsPerLaunch;
    long long rb_launch = 0;
    for (int i = 0; i < n; ++i) rb_launch += descs[first + i].out_features / kGroupRows;
    int max_n_cb = 0;
    for (int i = 0; i < n; ++i) {
      const int c = descs[first + i].in_features / kGroupCols;
      if (c > max_n_cb) max_n_cb = c;
    }
    const int fmt = format_tag(descs[0]);
    if (lora) {   // t = A x of the launch's problems first, on the same stream
      static_assert(sizeof(LoraDownBatch) <= 16384, "kernel arguments");
      LoraDownBatch down;
      memset(&down, 0, offsetof(LoraDownBatch, p));
      int rows = 0, m = 0;
      for (int i = 0; i < n; ++i) {
        const vq_lora_desc& l = lora[first + i];
        if (l.rank == 0) continue;
        LoraDownProblem& dp = down.p[m++];
        dp.A = (const uint16_t*)l.A_f16;
        dp.x = (const uint16_t*)x_f16[first + i];
        dp.t = t_ws + (size_t)(first + i) * kLoraWorkspaceFloats;
        dp.in_features = descs[first + i].in_features;
        dp.row_begin = rows;
        rows += l.rank;
      }
      down.count = m;
      down.total_rows = rows;
      if (m > 0 && launch_lora_down(down, (hipStream_t)stream) != hipSuccess) return VQ_ERR_HIP;
    }
    const bool d4 = fmt == kFmtD4 || fmt == kFmtD4F16 || fmt == kFmtD4BN;
    if (d4 || fmt == kFmtK256I8 || fmt == kFmtK256I8BN) {   // one workgroup per 64 rows, see vq_gemv_d4.hip
      GemvBatchLora both;                       // 20 KB on the stack; only the used entries are filled
      GemvBatch& batch = both.base;
      memset(&batch, 0, offsetof(GemvBatch, p) + (size_t)n * sizeof(GemvProblem));
      if (lora) {
        for (int i = 0; i < n; ++i) {
          LoraProblem& lp = both.l[i];
          lp.B = (const uint16_t*)lora[first + i].B_f16;
          lp.t = t_ws + (size_t)(first + i) * kLoraWorkspaceFloats;
          lp.rank = lora[first + i].rank;
          lp.pad = 0;
        }
      }
      batch.count = n;
      batch.y_f32 = (y_dtype == VQ_F32);
      long long wgs = 0;
      for (int i = 0; i < n; ++i) {
        const vq_desc& d = descs[first + i];
        GemvProblem& p = batch.p[i];
        p.idx = (const uint8_t*)idx_dev[first + i];
        p.cb = (const uint32_t*)cb_dev[first + i];
        p.x = (const uint16_t*)x_f16[first + i];
        p.y = y[first + i];
        p.n_rb = d.out_features / kGroupRows;
        p.n_cb = d.in_features / kGroupCols;
        p.splits = 1;
        p.rb_per_cb = d.group_rows / kGroupRows;
        p.wg_begin = (int32_t)wgs;
        wgs += p.n_rb / 8;
      }
      if (wgs > 0x7fffffffll) return VQ_ERR_UNSUPPORTED;
      batch.total_wgs = (int32_t)wgs;
      const hipError_t e =
          lora ? (d4 ? launch_gemv_d4_lora(both, (int)wgs, (hipStream_t)stream, fmt)
                     : launch_gemv_k256i8_lora(both, (int)wgs, (hipStream_t)stream, fmt))
               : (d4 ? launch_gemv_d4(batch, (int)wgs, (hipStream_t)stream, fmt)
                     : launch_gemv_k256i8(batch, (int)wgs, (hipStream_t)stream, fmt));
      if (e != hipSuccess) return VQ_ERR_HIP;
      continue;
    }
    const long long stream_from = 4096;   // row-blocks from which the persistent kernel pays
    // Split-K kernel: `splits` waves share a row-block.  A wave is most efficient with exactly
    // one full chunk (its fixed costs are spread over 8 groups and nothing is double-buffered),
    // so take the fewest waves per row-block whose strips still fit in one chunk, and 8 if no
    // choice does (measured on the q/k/v, o, gate/up and down launches of a 7B layer).  If every
    // strip fits in one chunk the one-chunk variant of the kernel is used (half the registers).
    // 8 waves per row-block (workgroups of 8 waves) pay on the wide matrices: one call on
    // 11008 x 4096 with k = 256 went from 11.6 to 9.8 us, on 4096 x 11008 from 13.4 to 12.1 us
    // (k = 16: 7.7 to 7.1 us); 16 waves per row-block were slower again.
    int splits = 8, strip_chunks = 0;   // strip_chunks: chunks of the longest strip
    {
      int max_units = 0;
      for (int i = 0; i < n; ++i) {
        const int units = strip_units(fmt, descs[first + i].in_features / kGroupCols);
        max_units = units > max_units ? units : max_units;
      }
      const int cu = gemv_chunk_units(fmt);
      for (int sp = 1; sp <= 8; sp <<= 1) {
        if ((max_units + sp - 1) / sp <= cu) {
          splits = sp;
          break;
        }
      }
      strip_chunks = ((max_units + splits - 1) / splits + cu - 1) / cu;
    }
    const int wpw = splits == 8 ? 8 : 4;   // waves per workgroup of the split-K kernel
    // many row-blocks: the persistent streaming kernel
    const bool stream_mode = rb_launch >= stream_from && max_n_cb <= kStreamMaxColBlocks &&
                             gemv_stream_lds_bytes(fmt, max_n_cb) <= 65536;
    GemvBatchLora both;                    // 20 KB on the stack; only the used entries are filled
    GemvBatch& batch = both.base;
    memset(&batch, 0, offsetof(GemvBatch, p) + (size_t)n * sizeof(GemvProblem));
    batch.count = n;
    batch.y_f32 = (y_dtype == VQ_F32);
    if (lora) {
      for (int i = 0; i < n; ++i) {
        LoraProblem& lp = both.l[i];
        lp.B = (const uint16_t*)lora[first + i].B_f16;
        lp.t = t_ws + (size_t)(first + i) * kLoraWorkspaceFloats;
        lp.rank = lora[first + i].rank;
        lp.pad = 0;
      }
    }
    long long items = 0;   // row-blocks (stream mode) or workgroups (split mode)
    long long cost = 0;    // groups
    for (int i = 0; i < n; ++i) {
      const vq_desc& d = descs[first + i];
      GemvProblem& p = batch.p[i];
      p.idx = (const uint8_t*)idx_dev[first + i];
      p.cb = (const uint32_t*)cb_dev[first + i];
      p.x = (const uint16_t*)x_f16[first + i];
      p.y = y[first + i];
      p.n_rb = d.out_features / kGroupRows;
      p.n_cb = d.in_features / kGroupCols;
      p.splits = stream_mode ? 1 : splits;
      p.rb_per_cb = d.group_rows / kGroupRows;
      p.wg_begin = (int32_t)items;
      p.cost_begin = (int32_t)cost;
      cost += (long long)p.n_rb * p.n_cb;
      const int rb_per_wg = wpw / p.splits;
      items += stream_mode ? p.n_rb : (p.n_rb + rb_per_wg - 1) / rb_per_wg;
    }
    if (items > 0x7fffffffll || cost > 0x3fffffffll) return VQ_ERR_UNSUPPORTED;
    batch.total_wgs = (int32_t)items;
    batch.total_cost = (int32_t)cost;
    int grid = (int)items;
    if (stream_mode) {
      const long long want = (items + 7) / 8;   // at least one row-block per wave
      const int resident = lora ? gemv_stream_resident_wgs_lora(fmt, max_n_cb) : gemv_stream_resident_wgs(fmt, max_n_cb);
      grid = (int)(want < resident ? want : resident);
    }
    // up to three chunks per strip: all loaded at once (modes 2..4); longer strips: two buffers ping-pong
    const int mode = stream_mode ? 1 : strip_chunks <= 3 ? 1 + strip_chunks : 0;
    const hipError_t e = lora ? launch_gemv_lora(fmt, both, mode, grid, max_n_cb, (hipStream_t)stream, wpw)
                              : launch_gemv(fmt, batch, mode, grid, max_n_cb, (hipStream_t)stream, wpw);
    if (e != hipSuccess) return VQ_ERR_HIP;
  }
  return VQ_OK;
}


}  // namespace

extern "C" {

const char* vq_status_string(int status) {
  switch (status) {
    case VQ_OK: return "VQ_OK";
    case VQ_ERR_NULL: return "VQ_ERR_NULL: required pointer is NULL";
    case VQ_ERR_BAD_DESC: return "VQ_ERR_BAD_DESC: inconsistent descriptor";
    case VQ_ERR_UNSUPPORTED: return "VQ_ERR_UNSUPPORTED: configuration not implemented";
    case VQ_ERR_ALIGN: return "VQ_ERR_ALIGN: pointer or leading dimension misaligned";
    case VQ_ERR_HIP: return "VQ_ERR_HIP: HIP runtime error at launch";
    case VQ_ERR_BAD_ARG: return "VQ_ERR_BAD_ARG: scalar argument out of range";
    default: return "unknown vq_status";
  }
}

int vq_version(void) { return 2; }

int vq_canonical_bytes(const vq_desc* desc, size_t* idx_bytes, size_t* cb_bytes) {
  // The canonical format is defined for any consistent descriptor, also ones the
  // kernels do not implement.
  if (!desc) return VQ_ERR_NULL;
  const int st = check_desc(desc);
  if (st == VQ_ERR_BAD_DESC) return st;
  if (desc->out_features % desc->group_rows || desc->in_features % desc->group_cols)
    return VQ_ERR_UNSUPPORTED;
  if (((size_t)desc->group_rows * desc->group_cols / desc->d * desc->index_bits) % 8)
    return VQ_ERR_UNSUPPORTED;
  if (desc->codebook_dtype != VQ_F16 && !is_i8(*desc)) return VQ_ERR_UNSUPPORTED;
  if (is_bn(*desc) && desc->group_cols % 32) return VQ_ERR_UNSUPPORTED;
  sizes(*desc, idx_bytes, cb_bytes);
  return VQ_OK;
}

int vq_layout_bytes(const vq_desc* desc, size_t* idx_bytes, size_t* cb_bytes) {
  const int st = check_desc(desc);
  if (st != VQ_OK) return st;
  // 4-bit row-blocks are stored as whole col-block pairs (an odd last one is padded)
  const size_t n_rb = desc->out_features / kGroupRows;
  const size_t n_cb = desc->in_features / kGroupCols;
  if (desc->k == 64) {   // quads of 4 col-blocks: 3 KB of indices per 8-row block, 528 B of tables per group row
    const size_t n_quads = (n_cb + 3) / 4;
    if (idx_bytes) *idx_bytes = n_rb * n_quads * 3072;
    if (cb_bytes)   // with blockwise normalisation: 672-byte records, then 128 bytes of codes per (8-row block, quad)
      *cb_bytes = is_bn(*desc) ? (size_t)(desc->out_features / desc->group_rows) * n_quads * 672 + n_rb * n_quads * 128
                               : (size_t)(desc->out_features / desc->group_rows) * n_quads * 528;
    return VQ_OK;
  }
  if (desc->d == 4) {    // 1 KB of indices per (8-row block, pair of col-blocks); tables as in the canonical buffer
    const size_t n_groups = (size_t)(desc->out_features / desc->group_rows) * n_cb;
    if (idx_bytes) *idx_bytes = n_rb * ((n_cb + 1) / 2) * 1024;
    if (cb_bytes)   // with blockwise normalisation: + 32 bytes of levels per group and 64 of codes per (8-row block, pair)
      *cb_bytes = is_bn(*desc) ? wide_bn_code_offset(n_groups, 1024) + n_rb * ((n_cb + 1) / 2) * 64
                  : is_i8(*desc) ? n_groups * 1024 + (2 * n_groups + 15) / 16 * 16 : n_groups * 2048;
    return VQ_OK;
  }
  if (desc->d == 1 && desc->k == 8) {   // indices as for k = 64; 48-byte table records per (group row, quad)
    const size_t n_quads = (n_cb + 3) / 4;
    if (idx_bytes) *idx_bytes = n_rb * n_quads * 3072;
    if (cb_bytes)   // with blockwise normalisation: 176-byte records, then 128 bytes of codes per (8-row block, quad)
      *cb_bytes = is_bn(*desc) ? (size_t)(desc->out_features / desc->group_rows) * n_quads * 176 + n_rb * n_quads * 128
                               : (size_t)(desc->out_features / desc->group_rows) * n_quads * 48;
    return VQ_OK;
  }
  if (desc->d == 2 && desc->k == 256 && is_i8(*desc)) {   // 1 KB of indices per (8-row block, col-block); tables as canonical
    const size_t n_groups = (size_t)(desc->out_features / desc->group_rows) * n_cb;
    if (idx_bytes) *idx_bytes = n_rb * n_cb * 1024;
    if (cb_bytes)
      *cb_bytes = is_bn(*desc) ? wide_bn_code_offset(n_groups, 512) + n_rb * ((n_cb + 1) / 2) * 64
                               : n_groups * 512 + (2 * n_groups + 15) / 16 * 16;
    return VQ_OK;
  }
  if (desc->d == 1 && desc->k == 4) {   // indices as for k = 16; a 48-byte table record per (8-row block, col-block slot)
    const size_t slots = 2 * ((n_cb + 1) / 2);
    if (idx_bytes) *idx_bytes = n_rb * slots * 512;
    if (cb_bytes) *cb_bytes = n_rb * slots * 48;
    return VQ_OK;
  }
  if (desc->d == 1) {    // 1 KB of indices and 16 fp16 scalars per group
    if (idx_bytes) *idx_bytes = n_rb * n_cb * 1024;
    if (cb_bytes) *cb_bytes = n_rb * n_cb * 32;
    return VQ_OK;
  }
  if (desc->k == 32) {   // nibbles as for k = 16 plus a plane of fifth bits (640 bytes per slot); 64-byte tables + scale
    const size_t slots32 = 2 * ((n_cb + 1) / 2);
    if (idx_bytes) *idx_bytes = n_rb * slots32 * 640;
    if (cb_bytes) *cb_bytes = n_rb * slots32 * 66;
    return VQ_OK;
  }
  const size_t slots = desc->k == 16 ? 2 * ((n_cb + 1) / 2) : n_cb;
  if (idx_bytes) *idx_bytes = n_rb * slots * (1024 * (size_t)desc->index_bits / 8);
  if (cb_bytes)   // k = 16 with blockwise normalisation: levels and block codes behind tables and scales
    *cb_bytes = is_bn(*desc) ? k16bn_table_bytes(n_rb * slots)
                : is_i8(*desc) ? n_rb * slots * (desc->group_rows == 4 ? 68 : 34)   // 4-row groups: two tables and scales per slot
                               : n_rb * slots * (size_t)desc->k * 4;
  return VQ_OK;
}

int vq_pack_layout(const vq_desc* desc, const void* idx_canon, const void* cb_canon,
                   void* idx_dev, void* cb_dev, void* stream) {
  const int st = check_desc(desc);
  if (st != VQ_OK) return st;
  if (!idx_canon || !cb_canon || !idx_dev || !cb_dev) return VQ_ERR_NULL;
  if (!aligned16(idx_canon) || !aligned16(cb_canon) || !aligned16(idx_dev) || !aligned16(cb_dev))
    return VQ_ERR_ALIGN;
  if (idx_canon == idx_dev || cb_canon == cb_dev) return VQ_ERR_BAD_ARG;
  return hip_status(launch_pack(*desc, idx_canon, cb_canon, idx_dev, cb_dev, (hipStream_t)stream));
}

int vq_gemv_multi(int count, const vq_desc* descs, const void* const* idx_dev,
                  const void* const* cb_dev, const void* const* x_f16, void* const* y,
                  int y_dtype, void* stream) {
  return gemv_multi_impl(count, descs, idx_dev, cb_dev, x_f16, y, y_dtype, stream, nullptr, nullptr);
}

int vq_lora_workspace_bytes(int count, size_t* bytes) {
  if (count < 1 || count > 65536) return VQ_ERR_BAD_ARG;
  if (!bytes) return VQ_ERR_NULL;
  *bytes = (size_t)count * kLoraWorkspaceFloats * sizeof(float);
  return VQ_OK;
}

int vq_gemv_lora_multi(int count, const vq_desc* descs, const void* const* idx_dev,
                       const void* const* cb_dev, const void* const* x_f16, const vq_lora_desc* lora,
                       void* workspace, size_t workspace_bytes, void* const* y, int y_dtype,
                       void* stream) {
  if (count < 1 || count > 65536) return VQ_ERR_BAD_ARG;
  if (!lora || !workspace) return VQ_ERR_NULL;
  if (!aligned16(workspace)) return VQ_ERR_ALIGN;
  if (workspace_bytes < (size_t)count * kLoraWorkspaceFloats * sizeof(float)) return VQ_ERR_BAD_ARG;
  return gemv_multi_impl(count, descs, idx_dev, cb_dev, x_f16, y, y_dtype, stream, lora, (float*)workspace);
}

int vq_gemv_lora_multi_static(int count, const vq_desc* descs, const void* const* idx_dev,
                              const void* const* cb_dev, const void* const* x_f16,
                              const vq_lora_desc* lora, void* const* y, int y_dtype, void* stream) {
  if (count < 1 || count > kStaticLoraProblems) return VQ_ERR_BAD_ARG;   // beyond the static scratch
  if (!lora) return VQ_ERR_NULL;
  float* t_ws = nullptr;
  // validate everything else first, so that argument errors need no GPU
  const int st = gemv_multi_impl(count, descs, idx_dev, cb_dev, x_f16, y, y_dtype, stream, lora, nullptr, true);
  if (st != VQ_OK) return st;
  const int sp = static_scratch(&t_ws);
  if (sp != VQ_OK) return sp;
  return gemv_multi_impl(count, descs, idx_dev, cb_dev, x_f16, y, y_dtype, stream, lora, t_ws, false);
}

int vq_gemv_lora(const vq_desc* desc, const void* idx_dev, const void* cb_dev, const void* x_f16,
                 const void* A_f16, const void* B_f16, int rank, void* workspace,
                 size_t workspace_bytes, void* y, int y_dtype, void* stream) {
  if (!desc) return VQ_ERR_NULL;
  const vq_lora_desc l = {A_f16, B_f16, rank, 0};
  return vq_gemv_lora_multi(1, desc, &idx_dev, &cb_dev, &x_f16, &l, workspace, workspace_bytes, &y, y_dtype, stream);
}

int vq_gemv(const vq_desc* desc, const void* idx_dev, const void* cb_dev, const void* x_f16,
            void* y, int y_dtype, void* stream) {
  if (!desc) return VQ_ERR_NULL;
  return vq_gemv_multi(1, desc, &idx_dev, &cb_dev, &x_f16, &y, y_dtype, stream);
}

int vq_gemm_batched(const vq_desc* desc, const void* idx_dev, const void* cb_dev,
                    const void* X_f16, int B, int ldx, void* Y, int ldy, int y_dtype,
                    void* stream) {
  const int st = check_desc(desc);
  if (st != VQ_OK) return st;
  if (!idx_dev || !cb_dev || !X_f16 || !Y) return VQ_ERR_NULL;
  if (y_dtype != VQ_F16 && y_dtype != VQ_F32) return VQ_ERR_BAD_ARG;
  if (B < 1 || B > 65536) return VQ_ERR_BAD_ARG;
  if (ldx < B || ldy < B) return VQ_ERR_BAD_ARG;
  if ((ldx & 7) || (ldy & 7)) return VQ_ERR_ALIGN;
  if (!aligned16(idx_dev) || !aligned16(cb_dev) || !aligned16(X_f16) || !aligned16(Y))
    return VQ_ERR_ALIGN;
  if (X_f16 == (const void*)Y) return VQ_ERR_BAD_ARG;
  return hip_status(launch_gemm(*desc, idx_dev, cb_dev, X_f16, B, ldx, Y, ldy,
                                y_dtype == VQ_F32, (hipStream_t)stream));
}

int vq_decode_dense(const vq_desc* desc, const void* idx_dev, const void* cb_dev, void* W_f16,
                    void* stream) {
  const int st = check_desc(desc);
  if (st != VQ_OK) return st;
  if (!idx_dev || !cb_dev || !W_f16) return VQ_ERR_NULL;
  if (!aligned16(idx_dev) || !aligned16(cb_dev) || !aligned16(W_f16)) return VQ_ERR_ALIGN;
  return hip_status(launch_decode(*desc, idx_dev, cb_dev, W_f16, (hipStream_t)stream));
}

int vq_em_assign(const vq_desc* desc, const void* W_f32, const void* hdiag_f32, const void* cb_f32,
                 void* assign_u8, void* stream) {
  const int st = check_em_desc(desc);
  if (st != VQ_OK) return st;
  if (!W_f32 || !hdiag_f32 || !cb_f32 || !assign_u8) return VQ_ERR_NULL;
  if (!aligned16(W_f32) || !aligned16(hdiag_f32) || !aligned16(cb_f32) || !aligned16(assign_u8))
    return VQ_ERR_ALIGN;
  return hip_status(launch_em_assign(*desc, W_f32, hdiag_f32, cb_f32, assign_u8, (hipStream_t)stream));
}

int vq_em_update(const vq_desc* desc, const void* W_f32, const void* hdiag_f32, const void* assign_u8,
                 void* cb_f32_out, void* stream) {
  const int st = check_em_desc(desc);
  if (st != VQ_OK) return st;
  if (!W_f32 || !hdiag_f32 || !assign_u8 || !cb_f32_out) return VQ_ERR_NULL;
  if (!aligned16(W_f32) || !aligned16(hdiag_f32) || !aligned16(assign_u8) || !aligned16(cb_f32_out))
    return VQ_ERR_ALIGN;
  return hip_status(launch_em_update(*desc, W_f32, hdiag_f32, assign_u8, cb_f32_out, (hipStream_t)stream));
}

}  // extern "C"
