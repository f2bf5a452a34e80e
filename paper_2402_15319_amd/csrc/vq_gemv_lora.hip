// y = W x + B (A x): the frozen vector-quantised base matrix with a low-rank adapter next to it
// (Sec. 5, "Combination of GPTVQ with LoRA adapters").  Two launches on one stream: t = A x
// (rank <= 64 dot products of length in_features, fp32), then the GEMV kernels of vq_gemv.hip
// instantiated with the adapter epilogue, which adds B[row, :] . t to every row total before
// it is stored.
#include "vq_gemv_impl.h"

namespace vq {
namespace {

// One workgroup of four waves per row of A.  A thread owns every 256th piece of 8 halfs; its
// first four pieces (rows of up to 8,192 columns) are all loaded before the first is used, so a
// row costs one round trip to memory.  fp32 multiply-adds, lanes summed by a halving exchange,
// the four waves' sums added in wave order: a fixed order, the same result on every call.
__global__ __launch_bounds__(256) void lora_down_kernel(const LoraDownBatch batch) {
  __shared__ float part[4];
  const int tid = threadIdx.x;
  const int row = blockIdx.x;
  int lo = 0, hi = batch.count;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (batch.p[mid].row_begin <= row) lo = mid; else hi = mid;
  }
  const LoraDownProblem& P = batch.p[lo];
  const int i = row - P.row_begin;
  const int n8 = P.in_features / 8;
  const uint4* a = reinterpret_cast<const uint4*>(P.A + (size_t)i * P.in_features);
  const uint4* x = reinterpret_cast<const uint4*>(P.x);
  const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
  uint4 av[4], xv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = tid + 256 * j;
    av[j] = c < n8 ? a[c] : zero;
    xv[j] = c < n8 ? x[c] : zero;
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    s = dot2(av[j].x, xv[j].x, s);
    s = dot2(av[j].y, xv[j].y, s);
    s = dot2(av[j].z, xv[j].z, s);
    s = dot2(av[j].w, xv[j].w, s);
  }
  for (int c = tid + 1024; c < n8; c += 256) {
    const uint4 aw = a[c], xw = x[c];
    s = dot2(aw.x, xw.x, s);
    s = dot2(aw.y, xw.y, s);
    s = dot2(aw.z, xw.z, s);
    s = dot2(aw.w, xw.w, s);
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  if ((tid & 63) == 0) part[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) P.t[i] = ((part[0] + part[1]) + part[2]) + part[3];
}

}  // namespace

hipError_t launch_lora_down(const LoraDownBatch& batch, hipStream_t s) {
  if (batch.total_rows == 0) return hipSuccess;
  hipLaunchKernelGGL(lora_down_kernel, dim3(batch.total_rows), dim3(256), 0, s, batch);
  return hipGetLastError();
}

int gemv_stream_resident_wgs_lora(int fmt, int max_n_cb) { return stream_resident_wgs_impl<true>(fmt, max_n_cb); }

hipError_t launch_gemv_lora(int fmt, const GemvBatchLora& batch, int mode, int grid_wgs, int max_n_cb,
                            hipStream_t s, int wpw) {
  return launch_gemv_impl<true>(fmt, batch, mode, grid_wgs, max_n_cb, s, wpw);
}

}  // namespace vq
