// y = W x + B (A x): the frozen vector-quantised base matrix with a low-rank adapter next to it
// (Sec. 5, "Combination of GPTVQ with LoRA adapters").  Two launches on one stream: t = A x
// (rank <= 64 dot products of length in_features, fp32), then the GEMV kernels of vq_gemv.hip
// instantiated with the adapter epilogue, which adds B[row, :] . t to every row total before
// it is stored.
#include "vq_gemv_impl.h"

namespace vq {
namespace {

// One wave per row of A: 8 halfs per lane and step, fp32 multiply-adds, lanes summed at the end.
__global__ __launch_bounds__(256) void lora_down_kernel(const LoraDownBatch batch) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= batch.total_rows) return;
  int lo = 0, hi = batch.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (batch.p[mid].row_begin <= row) lo = mid; else hi = mid;
  }
  const LoraDownProblem& P = batch.p[lo];
  const int i = row - P.row_begin;
  const uint4* a = reinterpret_cast<const uint4*>(P.A + (size_t)i * P.in_features);
  const uint4* x = reinterpret_cast<const uint4*>(P.x);
  float s = 0.f;
  for (int c = lane; c < P.in_features / 8; c += 64) {
    const uint4 av = a[c], xv = x[c];
    s = dot2(av.x, xv.x, s);
    s = dot2(av.y, xv.y, s);
    s = dot2(av.z, xv.z, s);
    s = dot2(av.w, xv.w, s);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  if (lane == 0) P.t[i] = s;
}

}  // namespace

hipError_t launch_lora_down(const LoraDownBatch& batch, hipStream_t s) {
  if (batch.total_rows == 0) return hipSuccess;
  hipLaunchKernelGGL(lora_down_kernel, dim3((batch.total_rows + 3) / 4), dim3(256), 0, s, batch);
  return hipGetLastError();
}

int gemv_stream_resident_wgs_lora(int fmt, int max_n_cb) { return stream_resident_wgs_impl<true>(fmt, max_n_cb); }

hipError_t launch_gemv_lora(int fmt, const GemvBatchLora& batch, int mode, int grid_wgs, int max_n_cb,
                            hipStream_t s, int wpw) {
  return launch_gemv_impl<true>(fmt, batch, mode, grid_wgs, max_n_cb, s, wpw);
}

}  // namespace vq
