// Batch-1 product y = W x on vector-quantised W (Sec. 3.2: decode by table
// lookup, then matrix-vector multiply), fused: packed indices are streamed
// from HBM with 128-bit loads, each group's codebook is staged in LDS, and
// every looked-up fp16 pair goes straight into a fp32-accumulating dot2.
//
// Work decomposition.  A workgroup has 4 waves; a wave owns a "strip": some or
// all col-blocks of one row-block (8 output rows).  A strip is consumed in
// chunks (k=16: 4 col-block pairs = 8 groups; k=256: 2 groups).  A chunk is one
// round of loads: its indices, its codebooks and its activations; two chunk
// buffers ping-pong so that one chunk is always in flight while the other is
// being consumed.  Absent parts of a ragged chunk are zero-filled (zero
// indices into a zeroed table times zero activations add exactly 0), so the
// consume step is branch-free.
//
// Two kernels share this code:
//   * gemv_stream_kernel (many row-blocks): a persistent grid; a workgroup owns a
//     contiguous, cost-balanced run of row-blocks, possibly across several
//     matrices, keeps x in LDS, and each of its waves has the first chunk of its
//     next row-block loading while the last chunk of the current one is consumed.
//   * gemv_split_kernel (few row-blocks): workgroups of 4 (or 8) waves; `splits`
//     (1, 2, 4 or 8) waves share a row-block and their partial sums meet in LDS in
//     a fixed order, so the result is deterministic.
#include "vq_gemv_impl.h"

namespace vq {

size_t gemv_stream_lds_bytes(int fmt, int max_n_cb) { return stream_lds_bytes_impl(fmt, max_n_cb); }
int gemv_stream_resident_wgs(int fmt, int max_n_cb) { return stream_resident_wgs_impl<false>(fmt, max_n_cb); }
int gemv_chunk_units(int fmt) { return chunk_units_impl(fmt); }

hipError_t launch_gemv(int fmt, const GemvBatch& batch, int mode, int grid_wgs, int max_n_cb,
                       hipStream_t s, int wpw) {
  return launch_gemv_impl<false>(fmt, batch, mode, grid_wgs, max_n_cb, s, wpw);
}

}  // namespace vq
