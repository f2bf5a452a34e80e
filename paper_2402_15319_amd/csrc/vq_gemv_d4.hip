// Batch-1 product y = W x for four-dimensional vector quantisation (Sec. 2.1 with d = 4; the
// 4D rows of the appendix table of VQ configurations): k = 256, one index byte per 4 weights,
// int8 tables with a scale (Sec. 3.1), groups of 64, 128 or 256 rows x 256 columns; also with fp16
// tables, and with blockwise normalisation on top of the int8 tables.
//
// A table is 256 entries x 4 values, far too large to rebuild per 8-row strip (a strip holds
// 512 bytes of indices per col-block, the table is 1 KB), so the unit of work is a workgroup of
// 8 waves that owns 64 consecutive rows (8 row-blocks of ONE group row): per pair of col-blocks
// the 512 threads dequantise the two tables once (one entry each: int8 x 4 -> fp16 x 4, times
// the scale, 8 bytes into LDS), a barrier, and every wave does its 16 lookups per lane (one
// 8-byte LDS read returns the four weights of a vector) and 32 dot2 steps.  The tables are
// double-buffered, so one barrier per pair of col-blocks is enough; indices, activations and
// the next table entry are loaded one step ahead.  A lane owns columns 4L .. 4L+3 of a
// col-block and keeps 8 row accumulators, reduced over the wave at the end exactly as in the
// other GEMV kernels.
#include "vq_gemv_impl.h"

namespace vq {
namespace {

__device__ __forceinline__ int find_problem_d4(const GemvBatch& batch, int item) {
  int lo = 0, hi = batch.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (batch.p[mid].wg_begin <= item) lo = mid; else hi = mid;
  }
  return lo;
}

struct D4Step {
  uint4 w;        // the lane's 8 + 8 index bytes of the pair
  uint2 xa, xb;   // its activations in the two col-blocks
  uint2 q;        // this thread's table entry of col-block (tid >> 8) of the pair: 4 int8 in .x, or 4 fp16
  uint32_t sc;    // int8 tables: that table's fp16 scale
  uint2 cw;       // blockwise normalisation: the lane's block codes in the two col-blocks (row r in bits [4r, 4r+4))
  uint32_t lv;    // ... and level (tid & 15) of this thread's table (fp16)
};

// MODE 1 (F16): the tables are fp16 (2 KB per group, copied to LDS as they are) instead of int8
// with a scale.  MODE 2 (BN): int8 tables with blockwise normalisation (appendix "Blockwise data
// normalization"): the group's 16 block-scale levels sit next to its table in LDS, and per row
// the looked-up vector is multiplied by the scale of the lane's 32-weight block before the dot2.
template <bool LORA, int MODE>
__global__ __launch_bounds__(512) void gemv_d4_kernel(const typename BatchOf<LORA>::type arg) {
  constexpr bool F16 = MODE == 1, BN = MODE == 2;
  const GemvBatch& batch = base_of(arg);
  __shared__ __attribute__((aligned(16))) uint2 tabs[2][2][256];   // [buffer][col-block of the pair][entry]
  __shared__ uint32_t levs[2][2][16];                               // BN: the tables' levels, the value in both halves
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pi = find_problem_d4(batch, blockIdx.x);
  const GemvProblem& P = batch.p[pi];
  const int oct = blockIdx.x - P.wg_begin;          // which 64 rows
  const int n_cb = P.n_cb, n_pairs = (n_cb + 1) >> 1;
  const int rb = oct * 8 + wave;                    // n_rb is a multiple of 8 (groups are >= 64 rows)
  const long long grow = (long long)(oct * 8) / P.rb_per_cb;
  const uint8_t* tab = reinterpret_cast<const uint8_t*>(P.cb);
  const long long n_groups = (long long)(P.n_rb / P.rb_per_cb) * n_cb;
  const uint16_t* scales = reinterpret_cast<const uint16_t*>(tab + n_groups * 1024);   // int8 tables only
  const uint16_t* levels = reinterpret_cast<const uint16_t*>(tab + wide_bn_level_offset((size_t)n_groups, 1024));
  const uint8_t* codes_lane = tab + wide_bn_code_offset((size_t)n_groups, 1024) + (size_t)rb * n_pairs * 64 + (lane >> 3) * 8;
  (void)levels; (void)codes_lane;
  const uint8_t* idx_lane = P.idx + (size_t)rb * n_pairs * 1024 + lane * 16;
  const uint16_t* x_lane = P.x + lane * 4;
  const int h = tid >> 8, e = tid & 255;            // table duty of this thread

  auto load = [&](int p, D4Step& s) {
    const int c0 = 2 * p, c1 = 2 * p + 1;
    const bool ok1 = c1 < n_cb;
    const int cme = (h == 0 || ok1) ? c0 + h : c0;  // an absent second col-block re-reads the first (not used)
    const long long g = grow * n_cb + cme;
    s.w = *reinterpret_cast<const uint4*>(idx_lane + (size_t)p * 1024);
    s.xa = *reinterpret_cast<const uint2*>(x_lane + (size_t)c0 * 256);
    const uint2 xb = *reinterpret_cast<const uint2*>(x_lane + (size_t)(ok1 ? c1 : c0) * 256);
    s.xb = ok1 ? xb : make_uint2(0u, 0u);
    if constexpr (F16) {
      s.q = *reinterpret_cast<const uint2*>(tab + g * 2048 + e * 8);
      s.sc = 0;
    } else {
      s.q = make_uint2(*reinterpret_cast<const uint32_t*>(tab + g * 1024 + e * 4), 0u);
      s.sc = scales[g];
    }
    if constexpr (BN) {
      s.cw = *reinterpret_cast<const uint2*>(codes_lane + (size_t)p * 64);
      s.lv = levels[g * 16 + (e & 15)];
    }
  };

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;
  float tv[8];
  uint4 lb = make_uint4(0, 0, 0, 0);
  (void)tv; (void)lb; (void)pi;
  if constexpr (LORA) {      // issued ahead of the main loop, used after the reduction
    lora_load_t(arg.l[pi], P.x, lane, tv);
    lb = lora_load_b(arg.l[pi], P.x, rb, lane);
  }

  D4Step cur, nxt;
  load(0, cur);
  for (int p = 0; p < n_pairs; ++p) {
    load(p + 1 < n_pairs ? p + 1 : p, nxt);         // one step ahead (a harmless re-read at the end)
    const int buf = p & 1;
    const bool mine = h == 0 || 2 * p + 1 < n_cb;   // the absent col-block of an odd matrix gets a zero table
    tabs[buf][h][e] = !mine ? make_uint2(0u, 0u)
                      : F16 ? cur.q : d4_dequant_entry(cur.q.x, __builtin_bit_cast(_Float16, (uint16_t)cur.sc));
    if constexpr (BN) {
      if (e < 16) levs[buf][h][e] = mine ? cur.lv * 0x10001u : 0u;
    }
    __syncthreads();   // tables of this step complete; the other buffer is free again (see header)
    const uint2* T0 = tabs[buf][0];
    const uint2* T1 = tabs[buf][1];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t j0 = ((r < 4 ? cur.w.x : cur.w.y) >> (8 * (r & 3))) & 0xffu;
      const uint32_t j1 = ((r < 4 ? cur.w.z : cur.w.w) >> (8 * (r & 3))) & 0xffu;
      uint2 t0 = T0[j0], t1 = T1[j1];
      if constexpr (BN) {
        const uint32_t s0 = levs[buf][0][(cur.cw.x >> (4 * r)) & 15u], s1 = levs[buf][1][(cur.cw.y >> (4 * r)) & 15u];
        t0 = make_uint2(scale_pair(t0.x, s0), scale_pair(t0.y, s0));
        t1 = make_uint2(scale_pair(t1.x, s1), scale_pair(t1.y, s1));
      }
      acc[r] = dot2(t0.x, cur.xa.x, acc[r]);
      acc[r] = dot2(t0.y, cur.xa.y, acc[r]);
      acc[r] = dot2(t1.x, cur.xb.x, acc[r]);
      acc[r] = dot2(t1.y, cur.xb.y, acc[r]);
    }
    cur = nxt;
  }

  float v = wave_reduce8(acc, lane);   // every lane: the total of row (lane >> 3) & 7
  if constexpr (LORA) v += lora_term(lb, tv);
  if ((lane & 7) == 0) {
    const size_t o = (size_t)rb * 8 + (lane >> 3);
    if (batch.y_f32) reinterpret_cast<float*>(P.y)[o] = v;
    else reinterpret_cast<_Float16*>(P.y)[o] = (_Float16)v;
  }
}

// ---- d = 2, k = 256, int8 tables with a scale, groups of 64, 128 or 256 rows ---------------
// The 4-bits-per-dimension 2D setting of the appendix table of VQ configurations: a 256-entry
// table is worth its bytes only when many rows share it, so the work is cut as above: 8 waves
// own 64 rows of one group row, per pair of col-blocks the 512 threads dequantise the two
// tables once (one entry each: two int8 times the scale, one dword into LDS), a barrier, and
// every wave runs the k = 256 inner block (16 lookups and 16 dot2 per col-block and lane) on
// its own 8 rows.  Indices are laid out as for k = 256 with fp16 codebooks (1 KB per 8-row
// block and col-block); the tables keep the canonical order (512 bytes per group, then scales).
struct K256Step {
  uint4 w0, w1;   // the lane's 16 index bytes in the two col-blocks of the pair
  uint2 xa, xb;   // its activations there
  uint32_t q;     // this thread's table entry (2 int8) of col-block (tid >> 8) of the pair
  uint32_t sc;    // that table's fp16 scale
  uint2 cw;       // blockwise normalisation: the lane's block codes in the two col-blocks
  uint32_t lv;    // ... and level (tid & 15) of this thread's table (fp16)
};

// BN: with blockwise normalisation; the plain C++ inner block replaces the hand-scheduled one.
template <bool LORA, bool BN>
__global__ __launch_bounds__(512) void gemv_k256i8_kernel(const typename BatchOf<LORA>::type arg) {
  const GemvBatch& batch = base_of(arg);
  __shared__ __attribute__((aligned(16))) uint32_t tabs[2][2][256];   // [buffer][col-block of the pair][entry]
  __shared__ uint32_t levs[2][2][16];                                  // BN: the tables' levels, the value in both halves
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pi = find_problem_d4(batch, blockIdx.x);
  const GemvProblem& P = batch.p[pi];
  const int oct = blockIdx.x - P.wg_begin;          // which 64 rows
  const int n_cb = P.n_cb, n_pairs = (n_cb + 1) >> 1;
  const int rb = oct * 8 + wave;
  const long long grow = (long long)(oct * 8) / P.rb_per_cb;
  const uint8_t* tab = reinterpret_cast<const uint8_t*>(P.cb);
  const long long n_groups = (long long)(P.n_rb / P.rb_per_cb) * n_cb;
  const uint16_t* scales = reinterpret_cast<const uint16_t*>(tab + n_groups * 512);
  const uint16_t* levels = reinterpret_cast<const uint16_t*>(tab + wide_bn_level_offset((size_t)n_groups, 512));
  const uint8_t* codes_lane = tab + wide_bn_code_offset((size_t)n_groups, 512) + (size_t)rb * n_pairs * 64 + (lane >> 3) * 8;
  (void)levels; (void)codes_lane;
  const uint8_t* idx_lane = P.idx + (size_t)rb * n_cb * 1024 + lane * 16;
  const uint16_t* x_lane = P.x + lane * 4;
  const int h = tid >> 8, e = tid & 255;            // table duty of this thread

  auto load = [&](int p, K256Step& s) {
    const int c0 = 2 * p, c1 = 2 * p + 1;
    const bool ok1 = c1 < n_cb;
    const int c1_ld = ok1 ? c1 : c0;                // an absent second col-block re-reads the first (not used)
    const long long g = grow * n_cb + (h == 0 ? c0 : c1_ld);
    s.w0 = *reinterpret_cast<const uint4*>(idx_lane + (size_t)c0 * 1024);
    s.w1 = *reinterpret_cast<const uint4*>(idx_lane + (size_t)c1_ld * 1024);
    s.xa = *reinterpret_cast<const uint2*>(x_lane + (size_t)c0 * 256);
    const uint2 xb = *reinterpret_cast<const uint2*>(x_lane + (size_t)c1_ld * 256);
    s.xb = ok1 ? xb : make_uint2(0u, 0u);
    s.q = *reinterpret_cast<const uint16_t*>(tab + g * 512 + e * 2);
    s.sc = scales[g];
    if constexpr (BN) {
      s.cw = *reinterpret_cast<const uint2*>(codes_lane + (size_t)p * 64);
      s.lv = levels[g * 16 + (e & 15)];
    }
  };

  float acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0.f;
  float tv[8];
  uint4 lb = make_uint4(0, 0, 0, 0);
  (void)tv; (void)lb; (void)pi;
  if constexpr (LORA) {      // issued ahead of the main loop, used after the reduction
    lora_load_t(arg.l[pi], P.x, lane, tv);
    lb = lora_load_b(arg.l[pi], P.x, rb, lane);
  }

  K256Step cur, nxt;
  load(0, cur);
  for (int p = 0; p < n_pairs; ++p) {
    load(p + 1 < n_pairs ? p + 1 : p, nxt);         // one step ahead (a harmless re-read at the end)
    const int buf = p & 1;
    const bool mine = h == 0 || 2 * p + 1 < n_cb;   // the absent col-block of an odd matrix gets a zero table
    tabs[buf][h][e] = mine ? k64_dequant_pair(cur.q, __builtin_bit_cast(_Float16, (uint16_t)cur.sc)) : 0u;
    if constexpr (BN) {
      if (e < 16) levs[buf][h][e] = mine ? cur.lv * 0x10001u : 0u;
    }
    __syncthreads();   // tables of this step complete; the other buffer is free again
    if constexpr (BN) {
      k256_group_scaled(cur.w0.x, cur.w0.y, cur.w0.z, cur.w0.w, cur.cw.x, tabs[buf][0], levs[buf][0], cur.xa.x, cur.xa.y, acc);
      k256_group_scaled(cur.w1.x, cur.w1.y, cur.w1.z, cur.w1.w, cur.cw.y, tabs[buf][1], levs[buf][1], cur.xb.x, cur.xb.y, acc);
    } else {
      const uint32_t base = lds_addr(&tabs[buf][0][0]);
      k256_group<0>(cur.w0.x, cur.w0.y, cur.w0.z, cur.w0.w, base, cur.xa.x, cur.xa.y, acc);
      k256_group<1024>(cur.w1.x, cur.w1.y, cur.w1.z, cur.w1.w, base, cur.xb.x, cur.xb.y, acc);
      acc_hazard_fence();
    }
    cur = nxt;
  }

  float v = wave_reduce8(acc, lane);   // every lane: the total of row (lane >> 3) & 7
  if constexpr (LORA) v += lora_term(lb, tv);
  if ((lane & 7) == 0) {
    const size_t o = (size_t)rb * 8 + (lane >> 3);
    if (batch.y_f32) reinterpret_cast<float*>(P.y)[o] = v;
    else reinterpret_cast<_Float16*>(P.y)[o] = (_Float16)v;
  }
}

}  // namespace

#define VQ_LAUNCH_WIDE(...) hipLaunchKernelGGL((__VA_ARGS__), dim3((unsigned)total_wgs), dim3(512), 0, s, batch)

hipError_t launch_gemv_k256i8(const GemvBatch& batch, int total_wgs, hipStream_t s, int fmt) {
  if (fmt == kFmtK256I8BN) VQ_LAUNCH_WIDE(gemv_k256i8_kernel<false, true>);
  else if (fmt == kFmtK256I8) VQ_LAUNCH_WIDE(gemv_k256i8_kernel<false, false>);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_gemv_d4(const GemvBatch& batch, int total_wgs, hipStream_t s, int fmt) {
  if (fmt == kFmtD4F16) VQ_LAUNCH_WIDE(gemv_d4_kernel<false, 1>);
  else if (fmt == kFmtD4BN) VQ_LAUNCH_WIDE(gemv_d4_kernel<false, 2>);
  else if (fmt == kFmtD4) VQ_LAUNCH_WIDE(gemv_d4_kernel<false, 0>);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// The same kernels with the low-rank adapter term added to every row before it is stored.
hipError_t launch_gemv_k256i8_lora(const GemvBatchLora& batch, int total_wgs, hipStream_t s, int fmt) {
  if (fmt == kFmtK256I8BN) VQ_LAUNCH_WIDE(gemv_k256i8_kernel<true, true>);
  else if (fmt == kFmtK256I8) VQ_LAUNCH_WIDE(gemv_k256i8_kernel<true, false>);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_gemv_d4_lora(const GemvBatchLora& batch, int total_wgs, hipStream_t s, int fmt) {
  if (fmt == kFmtD4F16) VQ_LAUNCH_WIDE(gemv_d4_kernel<true, 1>);
  else if (fmt == kFmtD4BN) VQ_LAUNCH_WIDE(gemv_d4_kernel<true, 2>);
  else if (fmt == kFmtD4) VQ_LAUNCH_WIDE(gemv_d4_kernel<true, 0>);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
#undef VQ_LAUNCH_WIDE

}  // namespace vq
