// Quantiser side: the E- and M-step of the Hessian-weighted EM that initialises a group's
// codebook (paragraph "Codebook Initialization": eq. "hessian_e_step" and the closed form
// below eq. "hessian_m_step"); the E-step is also the VQ_quant operation of Algorithm 2.
//
//   E-step:  a_i = argmin_m  sum_t h[c+t] * (x_i[t] - c_m[t])^2
//   M-step:  c_m[t] = sum_{i in I_m} h[c_i+t] * x_i[t] / sum_{i in I_m} h[c_i+t]   (0 if the sum of weights is 0)
//
// with x_i = W[r, c .. c+d-1] and h[c] = 1 / [H^-1]_cc, the diagonal weight of column c.
// em_assign_kernel / em_update_kernel: d = 2, groups of 8 x 256 weights.  One wave per group, lane
// L owns columns 4L .. 4L+3 (two vectors) of the group's 8 rows, exactly as in the matrix-vector
// kernels.  em_assign_any_kernel / em_update_any_kernel: d = 1, 2 or 4 and groups of 1, 8, 16, ...
// 256 rows x 256 columns (every group shape the decode formats use), the same lane ownership.
//
// The E-step is a decision taken in floating point, so its arithmetic is fixed: binary32,
// every operation rounded on its own (no fused multiply-add), in the order subtract, square,
// times weight, add; the smallest distance wins, the lowest m wins a tie.  The M-step sums in
// binary32 in a fixed order (a lane's 16 vectors one after the other, then lanes 0..63), so it is
// deterministic.
#include "vq_device.h"
#include "vq_internal.h"

namespace vq {
namespace {

template <int K>
__global__ __launch_bounds__(256) void em_assign_kernel(const float* __restrict__ W,
                                                        const float* __restrict__ hdiag,
                                                        const float* __restrict__ cb,
                                                        uint8_t* __restrict__ assign, int n_cb,
                                                        long long n_groups, int in_features) {
#pragma clang fp contract(off)
  __shared__ __attribute__((aligned(16))) float2 cbs_all[4][K];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float2* cbs = cbs_all[wave];
  const long long g = (long long)blockIdx.x * 4 + wave;
  if (g >= n_groups) return;   // whole waves leave; no workgroup barrier below
  const long long rb = g / n_cb;
  const int c = (int)(g - rb * n_cb);

  const float2* cg = reinterpret_cast<const float2*>(cb) + g * K;
#pragma unroll
  for (int i = 0; i < (K + 63) / 64; ++i)
    if (i * 64 + lane < K) cbs[i * 64 + lane] = cg[i * 64 + lane];
  const float4 h = *reinterpret_cast<const float4*>(hdiag + (size_t)c * 256 + lane * 4);
  float4 x[8];
#pragma unroll
  for (int r = 0; r < 8; ++r)
    x[r] = *reinterpret_cast<const float4*>(W + (size_t)(rb * 8 + r) * in_features + (size_t)c * 256 + lane * 4);
  wave_lds_sync();

  float best[16];
  uint32_t arg[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    best[v] = __builtin_inff();
    arg[v] = 0;
  }
  for (int m = 0; m < K; ++m) {
    const float2 cm = cbs[m];   // the same address in every lane: one broadcast read
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const float ea0 = x[r].x - cm.x, ea1 = x[r].y - cm.y;
      const float eb0 = x[r].z - cm.x, eb1 = x[r].w - cm.y;
      const float da = h.x * (ea0 * ea0) + h.y * (ea1 * ea1);
      const float db = h.z * (eb0 * eb0) + h.w * (eb1 * eb1);
      if (da < best[2 * r]) { best[2 * r] = da; arg[2 * r] = m; }
      if (db < best[2 * r + 1]) { best[2 * r + 1] = db; arg[2 * r + 1] = m; }
    }
  }
#pragma unroll
  for (int r = 0; r < 8; ++r)
    *reinterpret_cast<uint16_t*>(assign + (size_t)(rb * 8 + r) * (in_features / 2) + (size_t)c * 128 + lane * 2) =
        (uint16_t)(arg[2 * r] | (arg[2 * r + 1] << 8));
}

constexpr int kRedStride = 68;   // floats per lane row of the reduction buffer: 16-byte aligned, conflict-free

template <int K>
__global__ __launch_bounds__(128) void em_update_kernel(const float* __restrict__ W,
                                                        const float* __restrict__ hdiag,
                                                        const uint8_t* __restrict__ assign,
                                                        float* __restrict__ cb_out, int n_cb,
                                                        long long n_groups, int in_features) {
  __shared__ __attribute__((aligned(16))) float red_all[2][64 * kRedStride];
  __shared__ float tot_all[2][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* red = red_all[wave];
  float* tot = tot_all[wave];
  const long long g = (long long)blockIdx.x * 2 + wave;
  if (g >= n_groups) return;   // whole waves leave; no workgroup barrier below
  const long long rb = g / n_cb;
  const int c = (int)(g - rb * n_cb);

  const float4 h = *reinterpret_cast<const float4*>(hdiag + (size_t)c * 256 + lane * 4);
  float4 hx[8];
  uint32_t aa[8], ab[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const float4 x = *reinterpret_cast<const float4*>(W + (size_t)(rb * 8 + r) * in_features + (size_t)c * 256 + lane * 4);
    hx[r] = make_float4(h.x * x.x, h.y * x.y, h.z * x.z, h.w * x.w);
    const uint32_t a2 = *reinterpret_cast<const uint16_t*>(assign + (size_t)(rb * 8 + r) * (in_features / 2) +
                                                           (size_t)c * 128 + lane * 2);
    aa[r] = a2 & 0xffu;
    ab[r] = a2 >> 8;
  }

  float4* row = reinterpret_cast<float4*>(red + lane * kRedStride);   // this lane's 16 x 4 partial sums
  for (int m0 = 0; m0 < K; m0 += 16) {
    // this lane's part of (numerator t=0, numerator t=1, weight t=0, weight t=1) of 16
    // centroids: its 16 vectors are added one after the other (rows 0..7, the vector on
    // columns 4L, 4L+1 before the one on 4L+2, 4L+3) into the slot their assignment selects
#pragma unroll
    for (int j = 0; j < 16; ++j) row[j] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const uint32_t ja = aa[r] - m0, jb = ab[r] - m0;
      if (ja < 16u) {   // also keeps an out-of-range assignment byte out of the table
        float4 t = row[ja];
        t.x += hx[r].x; t.y += hx[r].y; t.z += h.x; t.w += h.y;
        row[ja] = t;
      }
      if (jb < 16u) {
        float4 t = row[jb];
        t.x += hx[r].z; t.y += hx[r].w; t.z += h.z; t.w += h.w;
        row[jb] = t;
      }
    }
    wave_lds_sync();
    // lane j owns quantity j of the 64: sum over the 64 lanes in lane order
    float s = 0.f;
    for (int l = 0; l < 64; ++l) s += red[l * kRedStride + lane];
    tot[lane] = s;
    wave_lds_sync();
    if (lane < 32) {
      const int j = lane >> 1, t = lane & 1;
      const float num = tot[4 * j + t], den = tot[4 * j + 2 + t];
      cb_out[(g * K + m0 + j) * 2 + t] = den != 0.f ? num / den : 0.f;
    }
    wave_lds_sync();   // tot and red are rewritten by the next 16 centroids
  }
}


// ---- any dimensionality and group height ---------------------------------------------------
// E-step.  One wave per (8-row block, col-block); the codebook is that of the group the block
// lies in (NCB = 1), one codebook per row (NCB = 8: groups of one row) or one per 4 rows (NCB = 2).
// D values per centroid, 4 / D vectors per row and lane.  Same arithmetic as em_assign_kernel:
// unfused binary32, sum over t in order.
template <int K, int D, int NCB>
__global__ __launch_bounds__(256) void em_assign_any_kernel(const float* __restrict__ W,
                                                            const float* __restrict__ hdiag,
                                                            const float* __restrict__ cb,
                                                            uint8_t* __restrict__ assign, int n_cb,
                                                            long long n_blocks, int in_features,
                                                            int group_rows) {
#pragma clang fp contract(off)
  constexpr int V = 4 / D;                 // vectors per row and lane
  constexpr int RPC = 8 / NCB;             // rows of the block that share a codebook
  __shared__ __attribute__((aligned(16))) float cbs_all[4][NCB * K * D];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* cbs = cbs_all[wave];
  const long long b = (long long)blockIdx.x * 4 + wave;
  if (b >= n_blocks) return;   // whole waves leave; no workgroup barrier below
  const long long rb = b / n_cb;
  const int c = (int)(b - rb * n_cb);

#pragma unroll
  for (int q = 0; q < NCB; ++q) {
    const long long g = ((rb * 8 + q * RPC) / group_rows) * n_cb + c;
    const float* cg = cb + g * (K * D);
    for (int i = lane; i < K * D; i += 64) cbs[q * K * D + i] = cg[i];
  }
  const float4 h4 = *reinterpret_cast<const float4*>(hdiag + (size_t)c * 256 + lane * 4);
  const float h[4] = {h4.x, h4.y, h4.z, h4.w};
  float x[8][4];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const float4 t = *reinterpret_cast<const float4*>(W + (size_t)(rb * 8 + r) * in_features + (size_t)c * 256 + lane * 4);
    x[r][0] = t.x; x[r][1] = t.y; x[r][2] = t.z; x[r][3] = t.w;
  }
  wave_lds_sync();

  float best[8 * V];
  uint32_t arg[8 * V];
#pragma unroll
  for (int v = 0; v < 8 * V; ++v) {
    best[v] = __builtin_inff();
    arg[v] = 0;
  }
  for (int m = 0; m < K; ++m) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const float* cm = cbs + (r / RPC) * K * D + m * D;   // the same address in every lane: broadcast reads
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const float e0 = x[r][v * D] - cm[0];
        float dist = h[v * D] * (e0 * e0);
#pragma unroll
        for (int t = 1; t < D; ++t) {
          const float e = x[r][v * D + t] - cm[t];
          dist = dist + h[v * D + t] * (e * e);
        }
        if (dist < best[r * V + v]) { best[r * V + v] = dist; arg[r * V + v] = m; }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    uint8_t* a = assign + (size_t)(rb * 8 + r) * (in_features / D) + (size_t)c * (256 / D) + lane * V;
    if constexpr (V == 4)
      *reinterpret_cast<uint32_t*>(a) = arg[4 * r] | (arg[4 * r + 1] << 8) | (arg[4 * r + 2] << 16) | (arg[4 * r + 3] << 24);
    else if constexpr (V == 2)
      *reinterpret_cast<uint16_t*>(a) = (uint16_t)(arg[2 * r] | (arg[2 * r + 1] << 8));
    else
      *a = (uint8_t)arg[r];
  }
}

// M-step.  One wave per group of n_rows rows (group_rows, or 1) x 256 columns.  A lane keeps the
// partial sums of 64 quantities in its LDS row: (numerator[D], weight[D]) of 32 / D centroids; the
// group's rows are walked once per such set of centroids (row after row, a lane's vectors left to
// right), then lane q sums quantity q over the 64 lanes in lane order: a fixed order, deterministic.
template <int K, int D>
__global__ __launch_bounds__(128) void em_update_any_kernel(const float* __restrict__ W,
                                                            const float* __restrict__ hdiag,
                                                            const uint8_t* __restrict__ assign,
                                                            float* __restrict__ cb_out, int n_cb,
                                                            long long n_groups, int in_features,
                                                            int n_rows) {
  constexpr int V = 4 / D;
  constexpr int CP = 32 / D;               // centroids per pass
  __shared__ __attribute__((aligned(16))) float red_all[2][64 * kRedStride];
  __shared__ float tot_all[2][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* red = red_all[wave];
  float* tot = tot_all[wave];
  const long long g = (long long)blockIdx.x * 2 + wave;
  if (g >= n_groups) return;   // whole waves leave; no workgroup barrier below
  const long long gr = g / n_cb;
  const int c = (int)(g - gr * n_cb);
  const long long row0 = gr * n_rows;

  const float4 h4 = *reinterpret_cast<const float4*>(hdiag + (size_t)c * 256 + lane * 4);
  const float h[4] = {h4.x, h4.y, h4.z, h4.w};
  float* row = red + lane * kRedStride;
  for (int m0 = 0; m0 < K; m0 += CP) {
#pragma unroll
    for (int j = 0; j < 64; ++j) row[j] = 0.f;
    for (int r = 0; r < n_rows; ++r) {
      const float4 t = *reinterpret_cast<const float4*>(W + (size_t)(row0 + r) * in_features + (size_t)c * 256 + lane * 4);
      const float x[4] = {t.x, t.y, t.z, t.w};
      const uint8_t* ap = assign + (size_t)(row0 + r) * (in_features / D) + (size_t)c * (256 / D) + lane * V;
      uint32_t a[V];
      if constexpr (V == 4) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(ap);
        a[0] = w & 0xffu; a[1] = (w >> 8) & 0xffu; a[2] = (w >> 16) & 0xffu; a[3] = w >> 24;
      } else if constexpr (V == 2) {
        const uint32_t w = *reinterpret_cast<const uint16_t*>(ap);
        a[0] = w & 0xffu; a[1] = w >> 8;
      } else {
        a[0] = *ap;
      }
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const uint32_t j = a[v] - m0;
        if (j < (uint32_t)CP && a[v] < (uint32_t)K) {   // also keeps an out-of-range assignment byte out of the table
          float* slot = row + j * 2 * D;
#pragma unroll
          for (int tt = 0; tt < D; ++tt) {
            slot[tt] += h[v * D + tt] * x[v * D + tt];
            slot[D + tt] += h[v * D + tt];
          }
        }
      }
    }
    wave_lds_sync();
    float s = 0.f;
    for (int l = 0; l < 64; ++l) s += red[l * kRedStride + lane];
    tot[lane] = s;
    wave_lds_sync();
    if (lane < CP * D) {
      const int j = lane / D, t = lane % D;
      if (m0 + j < K) {
        const float num = tot[j * 2 * D + t], den = tot[j * 2 * D + D + t];
        cb_out[(g * K + m0 + j) * D + t] = den != 0.f ? num / den : 0.f;
      }
    }
    wave_lds_sync();   // tot and red are rewritten by the next set of centroids
  }
}

}  // namespace

// Calls F(K) for the codebook size k (4, 8, 16, 64 or 256).
#define VQ_EM_K_SWITCH(k, F) \
  switch (k) {               \
    case 4: F(4); break;     \
    case 8: F(8); break;     \
    case 16: F(16); break;   \
    case 32: F(32); break;   \
    case 64: F(64); break;   \
    default: F(256); break;  \
  }

hipError_t launch_em_assign(const vq_desc& d, const void* W, const void* hdiag, const void* cb, void* assign,
                            hipStream_t s) {
  const int k = d.k, out_features = d.out_features, in_features = d.in_features;
  const int n_cb = in_features / kGroupCols;
  const long long n_blocks = (long long)(out_features / kGroupRows) * n_cb;
  const unsigned grid = (unsigned)((n_blocks + 3) / 4);
  if (d.d == 2 && d.group_rows == kGroupRows && (k == 16 || k == 64 || k == 256)) {
#define VQ_EM(K)                                                                                   \
  hipLaunchKernelGGL(em_assign_kernel<K>, dim3(grid), dim3(256), 0, s, (const float*)W,            \
                     (const float*)hdiag, (const float*)cb, (uint8_t*)assign, n_cb, n_blocks, in_features)
    if (k == 16) VQ_EM(16);
    else if (k == 64) VQ_EM(64);
    else VQ_EM(256);
#undef VQ_EM
    return hipGetLastError();
  }
#define VQ_EM_ANY(K, D, NCB)                                                                             \
  hipLaunchKernelGGL((em_assign_any_kernel<K, D, NCB>), dim3(grid), dim3(256), 0, s, (const float*)W,     \
                     (const float*)hdiag, (const float*)cb, (uint8_t*)assign, n_cb, n_blocks, in_features, \
                     d.group_rows)
  if (d.group_rows == 1) {   // a codebook per row: k * d <= 64 (checked by the caller)
    if (d.d == 1) {
#define VQ_F(K) if constexpr (K <= 64) VQ_EM_ANY(K, 1, 8)
      VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
    } else if (d.d == 2) {
#define VQ_F(K) if constexpr (K <= 16) VQ_EM_ANY(K, 2, 8)
      VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
    } else {
#define VQ_F(K) if constexpr (K <= 16) VQ_EM_ANY(K, 4, 8)
      VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
    }
  } else if (d.group_rows == 4) {   // two codebooks per 8-row block (d = 1 or 2, checked by the caller)
    if (d.d == 1) {
#define VQ_F(K) VQ_EM_ANY(K, 1, 2)
      VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
    } else {
#define VQ_F(K) VQ_EM_ANY(K, 2, 2)
      VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
    }
  } else if (d.d == 1) {
#define VQ_F(K) VQ_EM_ANY(K, 1, 1)
    VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
  } else if (d.d == 2) {
#define VQ_F(K) VQ_EM_ANY(K, 2, 1)
    VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
  } else {
#define VQ_F(K) VQ_EM_ANY(K, 4, 1)
    VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
  }
#undef VQ_EM_ANY
  return hipGetLastError();
}

hipError_t launch_em_update(const vq_desc& d, const void* W, const void* hdiag, const void* assign,
                            void* cb_out, hipStream_t s) {
  const int k = d.k, out_features = d.out_features, in_features = d.in_features;
  const int n_cb = in_features / kGroupCols;
  const long long n_groups = (long long)(out_features / d.group_rows) * n_cb;
  const unsigned grid = (unsigned)((n_groups + 1) / 2);
  if (d.d == 2 && d.group_rows == kGroupRows && (k == 16 || k == 64 || k == 256)) {
#define VQ_EM(K)                                                                                   \
  hipLaunchKernelGGL(em_update_kernel<K>, dim3(grid), dim3(128), 0, s, (const float*)W,            \
                     (const float*)hdiag, (const uint8_t*)assign, (float*)cb_out, n_cb, n_groups, in_features)
    if (k == 16) VQ_EM(16);
    else if (k == 64) VQ_EM(64);
    else VQ_EM(256);
#undef VQ_EM
    return hipGetLastError();
  }
#define VQ_EM_ANY(K, D)                                                                                   \
  hipLaunchKernelGGL((em_update_any_kernel<K, D>), dim3(grid), dim3(128), 0, s, (const float*)W,          \
                     (const float*)hdiag, (const uint8_t*)assign, (float*)cb_out, n_cb, n_groups, in_features, \
                     d.group_rows)
  if (d.d == 1) {
#define VQ_F(K) VQ_EM_ANY(K, 1)
    VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
  } else if (d.d == 2) {
#define VQ_F(K) VQ_EM_ANY(K, 2)
    VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
  } else {
#define VQ_F(K) VQ_EM_ANY(K, 4)
    VQ_EM_K_SWITCH(k, VQ_F)
#undef VQ_F
  }
#undef VQ_EM_ANY
  return hipGetLastError();
}

}  // namespace vq
