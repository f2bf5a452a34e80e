// Host-only stand-ins for the kernel launchers of libvq, for the sanitizer build of the host
// logic (tests/test_host_sanitizers.py).  Nothing here touches a GPU: every launcher checks the
// launch parameters it is handed against what the kernels assume of them and aborts with a
// message on the first violation; the API source (descriptor checks, size formulas, problem
// tables, kernel choice) is the real one, compiled with AddressSanitizer and UBSan on the host.
#include <cstdio>
#include <cstdlib>

#include "../../paper_2402_15319_amd/csrc/vq_internal.h"

namespace vq {
namespace {

long long g_launches = 0;

#define REQUIRE(cond, ...)                                        \
  do {                                                            \
    if (!(cond)) {                                                \
      std::fprintf(stderr, "launcher stub: %s violated: ", #cond); \
      std::fprintf(stderr, __VA_ARGS__);                          \
      std::fprintf(stderr, "\n");                                 \
      std::abort();                                               \
    }                                                             \
  } while (0)

// Units one chunk of the GEMV kernels holds: 4 col-block pairs (k = 16), 2 pairs (d = 1, k = 4),
// one quad of col-blocks (the k = 64 layouts), 2 col-blocks (the k = 256 layouts).
int chunk_units(int fmt) {
  return (fmt == 16 || fmt == kFmtK16I8 || fmt == kFmtK16BN || fmt == kFmtK16I8H || fmt == kFmtK32) ? 4 : (fmt == 64 || fmt == kFmtK64BN || fmt == kFmtD1K8 || fmt == kFmtD1K8BN) ? 1 : 2;
}

int strip_units(int fmt, int n_cb) {
  return (fmt == 16 || fmt == kFmtK16I8 || fmt == kFmtK16BN || fmt == kFmtK16I8H || fmt == kFmtK32 || fmt == kFmtD1K4) ? (n_cb + 1) / 2
         : (fmt == 64 || fmt == kFmtK64BN || fmt == kFmtD1K8 || fmt == kFmtD1K8BN) ? (n_cb + 3) / 4 : n_cb;
}

void check_problem(const GemvProblem& p, int i) {
  REQUIRE(p.idx && p.cb && p.x && p.y, "problem %d has a null pointer", i);
  REQUIRE(p.n_rb > 0 && p.n_cb > 0, "problem %d: n_rb %d n_cb %d", i, p.n_rb, p.n_cb);
  REQUIRE(p.rb_per_cb >= 1 && p.n_rb % p.rb_per_cb == 0 || p.rb_per_cb == 0, "problem %d: rb_per_cb %d n_rb %d", i,
          p.rb_per_cb, p.n_rb);
}

void check_gemv(int fmt, const GemvBatch& b, int mode, int grid_wgs, int max_n_cb, int wpw) {
  ++g_launches;
  REQUIRE(b.count >= 1 && b.count <= kMaxProblemsPerLaunch, "count %d", b.count);
  REQUIRE(b.y_f32 == 0 || b.y_f32 == 1, "y_f32 %d", b.y_f32);
  REQUIRE(mode >= 0 && mode <= 4, "mode %d", mode);
  REQUIRE(grid_wgs >= 1, "grid %d", grid_wgs);
  REQUIRE(wpw == 4 || wpw == 8, "wpw %d", wpw);
  long long items = 0, cost = 0;
  for (int i = 0; i < b.count; ++i) {
    const GemvProblem& p = b.p[i];
    check_problem(p, i);
    REQUIRE(p.n_cb <= max_n_cb, "problem %d: n_cb %d > max_n_cb %d", i, p.n_cb, max_n_cb);
    REQUIRE(p.wg_begin == items, "problem %d: wg_begin %d, expected %lld", i, p.wg_begin, items);
    REQUIRE(p.cost_begin == cost, "problem %d: cost_begin %d, expected %lld", i, p.cost_begin, cost);
    cost += (long long)p.n_rb * p.n_cb;
    if (mode == 1) {
      REQUIRE(p.splits == 1, "streaming kernel with splits %d", p.splits);
      items += p.n_rb;
    } else {
      REQUIRE(p.splits == 1 || p.splits == 2 || p.splits == 4 || p.splits == 8, "splits %d", p.splits);
      REQUIRE(p.splits <= wpw, "splits %d > waves per workgroup %d", p.splits, wpw);
      const int rb_per_wg = wpw / p.splits;
      items += (p.n_rb + rb_per_wg - 1) / rb_per_wg;
      // chunks of the longest strip: what the kernel variant (mode) is compiled for
      const int units = strip_units(fmt, p.n_cb);
      const int per_strip = (units + p.splits - 1) / p.splits;
      const int chunks = (per_strip + chunk_units(fmt) - 1) / chunk_units(fmt);
      if (mode >= 2) REQUIRE(chunks <= mode - 1, "problem %d: strips of %d chunks in mode %d", i, chunks, mode);
    }
  }
  REQUIRE(b.total_wgs == items, "total_wgs %d, expected %lld", b.total_wgs, items);
  REQUIRE(b.total_cost == cost, "total_cost %d, expected %lld", b.total_cost, cost);
  if (mode == 1) {
    REQUIRE(max_n_cb <= kStreamMaxColBlocks, "max_n_cb %d in the streaming kernel", max_n_cb);
    REQUIRE((long long)grid_wgs * 8 <= items + 7, "streaming grid %d for %lld row-blocks: a wave without a row-block", grid_wgs, items);
  } else {
    REQUIRE(grid_wgs == items, "split-K grid %d, %lld workgroups of work", grid_wgs, items);
    if (mode == 0 || mode == 3 || mode == 4) REQUIRE(wpw == 8, "mode %d with %d waves per workgroup", mode, wpw);
  }
}

void check_adapters(const GemvBatchLora& batch) {
  for (int i = 0; i < batch.base.count; ++i) {
    const LoraProblem& l = batch.l[i];
    REQUIRE(l.rank >= 0 && l.rank <= kMaxLoraRank && l.rank % 8 == 0, "problem %d: rank %d", i, l.rank);
    REQUIRE(l.rank == 0 || (l.B && l.t), "problem %d: adapter with a null pointer", i);
  }
}

}  // namespace

long long stub_launch_count() { return g_launches; }

hipError_t launch_pack(const vq_desc&, const void* a, const void* b, void* c, void* d, hipStream_t) {
  ++g_launches;
  REQUIRE(a && b && c && d, "pack with a null pointer");
  return hipSuccess;
}
hipError_t launch_decode(const vq_desc&, const void* a, const void* b, void* W, hipStream_t) {
  ++g_launches;
  REQUIRE(a && b && W, "decode with a null pointer");
  return hipSuccess;
}
hipError_t launch_gemv(int fmt, const GemvBatch& batch, int mode, int grid_wgs, int max_n_cb, hipStream_t, int wpw) {
  check_gemv(fmt, batch, mode, grid_wgs, max_n_cb, wpw);
  return hipSuccess;
}
hipError_t launch_gemv_lora(int fmt, const GemvBatchLora& batch, int mode, int grid_wgs, int max_n_cb, hipStream_t,
                            int wpw) {
  check_gemv(fmt, batch.base, mode, grid_wgs, max_n_cb, wpw);
  REQUIRE(fmt != kFmtD4 && fmt != kFmtD4F16 && fmt != kFmtD4BN && fmt != kFmtK256I8 && fmt != kFmtK256I8BN,
          "split-K / streaming launch for format %d", fmt);
  check_adapters(batch);
  return hipSuccess;
}
int gemv_stream_resident_wgs_lora(int, int) { return 512; }
int gemv_stream_resident_wgs(int, int) { return 768; }
hipError_t launch_lora_down(const LoraDownBatch& b, hipStream_t) {
  ++g_launches;
  REQUIRE(b.count >= 1 && b.count <= kMaxProblemsPerLaunch, "count %d", b.count);
  int rows = 0;
  for (int i = 0; i < b.count; ++i) {
    const LoraDownProblem& p = b.p[i];
    REQUIRE(p.A && p.x && p.t, "adapter problem %d has a null pointer", i);
    REQUIRE(p.row_begin == rows, "adapter problem %d: row_begin %d, expected %d", i, p.row_begin, rows);
    REQUIRE(p.in_features > 0 && p.in_features % 8 == 0, "adapter problem %d: in_features %d", i, p.in_features);
    REQUIRE(i + 1 == b.count || b.p[i + 1].row_begin > p.row_begin, "adapter problem %d has no rows", i);
    rows = i + 1 < b.count ? b.p[i + 1].row_begin : b.total_rows;
  }
  REQUIRE(b.total_rows > b.p[b.count - 1].row_begin, "last adapter problem has no rows");
  return hipSuccess;
}
size_t gemv_stream_lds_bytes(int, int max_n_cb) { return 8 * 2048 + (size_t)(max_n_cb + 8) * 512; }
int gemv_chunk_units(int fmt) { return chunk_units(fmt); }
static hipError_t check_wide(const GemvBatch& b, int total_wgs) {
  ++g_launches;
  long long wgs = 0;
  for (int i = 0; i < b.count; ++i) {
    check_problem(b.p[i], i);
    REQUIRE(b.p[i].n_rb % 8 == 0, "problem %d: %d row-blocks do not make whole 64-row workgroups", i, b.p[i].n_rb);
    REQUIRE(b.p[i].wg_begin == wgs, "problem %d: wg_begin", i);
    wgs += b.p[i].n_rb / 8;
  }
  REQUIRE(total_wgs == wgs && b.total_wgs == wgs, "total_wgs %d", total_wgs);
  return hipSuccess;
}
hipError_t launch_gemv_d4(const GemvBatch& b, int total_wgs, hipStream_t, int fmt) {
  REQUIRE(fmt == kFmtD4 || fmt == kFmtD4F16 || fmt == kFmtD4BN, "d = 4 launch for format %d", fmt);
  return check_wide(b, total_wgs);
}
hipError_t launch_gemv_k256i8(const GemvBatch& b, int total_wgs, hipStream_t, int fmt) {
  REQUIRE(fmt == kFmtK256I8 || fmt == kFmtK256I8BN, "k = 256 int8-table launch for format %d", fmt);
  return check_wide(b, total_wgs);
}
hipError_t launch_gemv_d4_lora(const GemvBatchLora& b, int total_wgs, hipStream_t s, int fmt) {
  check_adapters(b);
  return launch_gemv_d4(b.base, total_wgs, s, fmt);
}
hipError_t launch_gemv_k256i8_lora(const GemvBatchLora& b, int total_wgs, hipStream_t s, int fmt) {
  check_adapters(b);
  return launch_gemv_k256i8(b.base, total_wgs, s, fmt);
}
hipError_t launch_gemm(const vq_desc& d, const void* a, const void* b, const void* X, int B, int ldx, void* Y, int ldy,
                       int y_f32, hipStream_t) {
  ++g_launches;
  REQUIRE(a && b && X && Y, "gemm with a null pointer");
  REQUIRE(B >= 1 && ldx >= B && ldy >= B && ldx % 8 == 0, "gemm B %d ldx %d ldy %d", B, ldx, ldy);
  REQUIRE(y_f32 == 0 || y_f32 == 1, "y_f32 %d", y_f32);
  REQUIRE(d.out_features % 8 == 0 && d.in_features % 256 == 0, "gemm shape");
  return hipSuccess;
}
hipError_t launch_em_assign(const vq_desc& d, const void* W, const void* h, const void* cb, void* a, hipStream_t) {
  ++g_launches;
  REQUIRE(W && h && cb && a, "E-step with a null pointer");
  REQUIRE(d.group_rows == 1 || (d.group_rows == 4 && d.d <= 2) || d.group_rows % 8 == 0, "E-step group_rows %d", d.group_rows);
  return hipSuccess;
}
hipError_t launch_em_update(const vq_desc& d, const void* W, const void* h, const void* a, void* cb, hipStream_t) {
  ++g_launches;
  REQUIRE(W && h && cb && a, "M-step with a null pointer");
  REQUIRE(d.group_rows == 1 || (d.group_rows == 4 && d.d <= 2) || d.group_rows % 8 == 0, "M-step group_rows %d", d.group_rows);
  return hipSuccess;
}

}  // namespace vq
