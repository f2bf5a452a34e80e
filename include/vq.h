/*
 * vq.h -- C ABI of the MI355X (gfx950) vector-quantised matrix-vector library.
 *
 * The library implements the decode-time hot path of GPTVQ (arXiv 2402.15319):
 * y = W x where W[out,in] is never stored densely.  W is tiled into groups of
 * group_rows x group_cols weights (Sec. 4: e.g. 8 rows x 256 columns); each group
 * owns a codebook of k centroids of d fp16 values (Sec. 2.1) and stores one
 * index of index_bits = log2(k) bits for every run of d consecutive columns of
 * a row (Sec. 4: d columns are quantised at a time).  At inference a group is
 * decoded by table lookup to the native type and used in the matrix-vector
 * product (Sec. 3.2).
 *
 * Conventions common to every entry point
 *   - plain C, no C++/torch types; every pointer is a DEVICE pointer unless a
 *     comment says "host";
 *   - the caller owns all buffers; the library allocates nothing.  The only state it
 *     keeps between calls is a process-wide, thread-safe cache of launch parameters that
 *     depend on the device only (its number of compute units, how many workgroups of the
 *     streaming GEMV kernel fit on it, the address of the scratch array of
 *     vq_gemv_lora_multi_static), each asked of the HIP runtime the first time it is needed;
 *     those queries enqueue nothing, so a first call may be made while the stream is being
 *     captured into a HIP graph;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream); calls
 *     enqueue work and return without synchronising;
 *   - return value: VQ_OK (0) or a negative vq_status.  Arguments are validated
 *     on the host before anything is launched, so every error except VQ_ERR_HIP
 *     can be provoked without a GPU.  No exception crosses the boundary.
 *
 * Canonical (interchange) format, used only as the input of vq_pack_layout
 *   - groups are numbered row-block-major: g = (r / group_rows) * (in / group_cols) + c / group_cols;
 *   - inside a group vectors are row-major: v = (r % group_rows) * (group_cols / d) + (c % group_cols) / d;
 *   - indices: group g owns bytes [g*GB, (g+1)*GB), GB = group_rows*group_cols/d*index_bits/8,
 *     read as a little-endian bit stream: vector v is bits [v*index_bits, (v+1)*index_bits)
 *     (4-bit: even v in the low nibble; 8-bit: byte v);
 *   - codebooks (VQ_F16): fp16 cb[g][j][t], j < k, t < d, contiguous, same g order;
 *   - codebooks (VQ_I8; Sec. 3.1: a group is the tuple indices, lookup table, scale; the
 *     appendix on codebook compression makes 8-bit tables the default): int8 q[g][j][t],
 *     zero-padded to a multiple of 16 bytes, followed by one fp16 scale[g] per group.  The
 *     centroid value is scale[g] * q taken exactly and rounded once to fp16 (nearest even);
 *     that fp16 matrix is W for every entry point.
 *   - codebooks (VQ_I8_BN; appendix "Blockwise data normalization": every sub-row block of 32
 *     weights was divided by a scale that is quantised to 4 bits in the log domain, and the
 *     division is undone when a weight is decoded): q and scale as for VQ_I8, each padded to a
 *     multiple of 16 bytes, then fp16 level[g][16], the 16 block scales a code can select in
 *     group g (level j = 2^(a_g*j + s_0) in the appendix's parameterisation; stored explicitly
 *     so that the reconstruction is exact to state), then the 4-bit codes of the whole matrix,
 *     row-major code[r][c/32], two per byte, even block in the low nibble.  The decoded weight
 *     is fp16(scale*q) times level[g][code], the product of the two fp16 values rounded once.
 * The device layout written by vq_pack_layout is private to the library.
 *
 * Implemented representations (d = 2 unless stated): VQ_F16 with 8 x 256 groups and k = 16
 * or 256; VQ_I8 with k = 64 (6-bit indices) and groups of 8, 16 or 32 rows x 256 columns
 * (32 rows: the 8,192-weight groups and 3.125 bits per value of Sec. 5.1); VQ_I8 with k = 16
 * and 8 x 256 groups (2.125 bits per value) or 4 x 256 groups (1,024 weights: the 2.25-bit 2D row
 * of the appendix table; out_features a multiple of 8); VQ_I8 with k = 32 (5-bit indices, the
 * 2.5-bits-per-dimension row: 2.75 bits per value) and 8 x 256 groups; VQ_I8 with k = 256 and groups of 64, 128 or 256
 * rows x 256 columns (128 rows: the 32,768-weight groups and 4.125 bits per value of the 2D
 * 4-bits-per-dimension setting); and scalar codebooks, d = 1 (the 1D rows of the
 * appendix table of VQ configurations): VQ_F16, k = 16, 4-bit indices, 8 x 256 groups, 4.125
 * bits per value; VQ_I8, k = 8, 3-bit indices, groups of 8, 16 or 32 rows x 256 columns; and
 * VQ_I8, k = 4, 2-bit indices, groups of 1 x 256 (one codebook per row of a 256-column block,
 * the 2.125-bit 1D row; out_features a multiple of 8); VQ_I8_BN with k = 64 and groups of 8, 16
 * or 32 rows x 256 columns, with k = 16 and 8 x 256 groups, with d = 1, k = 8 and groups of
 * 8, 16 or 32 rows x 256 columns, or with k = 256 (d = 2 or 4) and groups of 64, 128 or 256 rows,
 * i.e. on every int8-table representation but the one-row groups of d = 1, k = 4; and
 * four-dimensional vectors, d = 4 (the 4D rows of that table): VQ_I8 or VQ_F16, k = 256 (one index
 * byte per 4 weights), groups of 64, 128 or 256 rows x 256 columns (256 rows: 2.125 bits per value
 * with int8 tables, 2.25 with fp16 tables).
 * Every entry point takes all of them.
 */
#ifndef VQ_H_
#define VQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VQ_API __attribute__((visibility("default")))

typedef enum vq_status {
  VQ_OK = 0,
  VQ_ERR_NULL = -1,        /* a required pointer is NULL                                  */
  VQ_ERR_BAD_DESC = -2,    /* descriptor is inconsistent (non-positive size, k != 2^bits) */
  VQ_ERR_UNSUPPORTED = -3, /* consistent but not implemented (shape not a multiple of the
                              group, or a d / k / group / dtype combination outside the
                              list above)                                                  */
  VQ_ERR_ALIGN = -4,       /* a device pointer is not 16-byte aligned / bad leading dim   */
  VQ_ERR_HIP = -5,         /* the HIP runtime refused the launch (see hipGetLastError)    */
  VQ_ERR_BAD_ARG = -6      /* a scalar argument is out of range (batch, count, dtype)     */
} vq_status;

/* VQ_I8 as codebook_dtype: int8 lookup tables with one fp16 scale per group (Sec. 3.1);
 * VQ_I8_BN: the same plus blockwise normalisation (see the canonical format above). */
typedef enum vq_dtype { VQ_F16 = 1, VQ_F32 = 2, VQ_I8 = 3, VQ_I8_BN = 4 } vq_dtype;

/* Shape of one vector-quantised matrix (Sec. 2.1, Sec. 3.1, Sec. 4). */
typedef struct vq_desc {
  int32_t out_features;   /* rows of W (length of y)                                */
  int32_t in_features;    /* columns of W (length of x)                             */
  int32_t group_rows;     /* rows sharing one codebook: 8 (VQ_F16); 8, 16 or 32 (k = 64, and
                             d = 1 with k = 8); 64, 128 or 256 (VQ_I8 with k = 256, d = 2 or 4);
                             8 or 4 (VQ_I8 with k = 16); 1 (d = 1 with k = 4)         */
  int32_t group_cols;     /* 256 (Sec. 4: at most 256 columns per group)            */
  int32_t d;              /* VQ dimensionality: 2, 1 (scalar codebooks) or 4        */
  int32_t k;              /* centroids.  d = 2: 16 or 256 (VQ_F16), 16, 32, 64 or 256 (VQ_I8),
                             16, 64 or 256 (VQ_I8_BN); d = 1: 16 (VQ_F16), 8 or 4 (VQ_I8), 8 (VQ_I8_BN);
                             d = 4: 256 (VQ_I8, VQ_I8_BN or VQ_F16) */
  int32_t index_bits;     /* log2(k): 2, 3, 4, 5, 6 or 8                            */
  int32_t codebook_dtype; /* VQ_F16, VQ_I8 or VQ_I8_BN (see the list above)         */
} vq_desc;

/* Human-readable name of a status code (host pointer to a static string). */
VQ_API const char* vq_status_string(int status);

/* Library version: increments when an entry point is added, a signature or the device layout
 * changes, or a kernel of the decode path is rewritten (measurements quote the version). */
VQ_API int vq_version(void);

/*
 * Sizes in bytes of the canonical arrays and of the device-layout arrays for
 * `desc` (host pointers; any output pointer may be NULL).  By Sec. 4's
 * bits-per-value formula the canonical pair obeys
 * (idx + cb) * 8 / (out*in) = log2(k)/d + k*d*16/(rows*cols).  The device layout
 * is as large, except that 4-bit row-blocks with an odd number of 256-column
 * blocks are padded to a whole pair of blocks (one zero group and one zero
 * codebook per row-block: +2.3 % for in = 11008).
 */
VQ_API int vq_canonical_bytes(const vq_desc* desc, size_t* idx_bytes, size_t* cb_bytes);
VQ_API int vq_layout_bytes(const vq_desc* desc, size_t* idx_bytes, size_t* cb_bytes);

/*
 * One-time re-layout (off the hot path): canonical indices/codebooks ->
 * device layout (Sec. 3.2: indices and tables are arranged for wide vector
 * accesses).  All four buffers are device memory, 16-byte
 * aligned, sized as reported above; input and output must not overlap.
 */
VQ_API int vq_pack_layout(const vq_desc* desc, const void* idx_canon, const void* cb_canon,
                   void* idx_dev, void* cb_dev, void* stream);

/*
 * y[out] = W x[in]  (Sec. 3.2: decode by lookup, then matrix-vector product;
 * batch 1).  x is fp16; products are accumulated in fp32; y is written as
 * y_dtype (VQ_F16 or VQ_F32).  idx_dev/cb_dev come from vq_pack_layout.  x and
 * y are 16-byte aligned and must not alias.  One kernel launch, deterministic
 * (no atomics).
 */
VQ_API int vq_gemv(const vq_desc* desc, const void* idx_dev, const void* cb_dev,
            const void* x_f16, void* y, int y_dtype, void* stream);

/*
 * `count` independent products y_i = W_i x_i enqueued as few launches as
 * possible (the q/k/v or gate/up projections of a decoder layer, or a whole
 * per-token weight pass replayed back to back; Sec. 1: every weight is loaded
 * once per generated token).  descs/idx_dev/cb_dev/x_f16/y are HOST arrays of
 * length `count` holding descriptors and device pointers; they are read
 * during the call and need not outlive it (the problem table travels in the
 * kernel arguments, up to 256 problems per launch).  All y_i share y_dtype and
 * all descriptors share one representation (d, k, codebook_dtype).  Each
 * product obeys the rules of vq_gemv.
 * count in [1, 65536].
 */
VQ_API int vq_gemv_multi(int count, const vq_desc* descs, const void* const* idx_dev,
                  const void* const* cb_dev, const void* const* x_f16, void* const* y,
                  int y_dtype, void* stream);

/*
 * y = W x + B (A x): the frozen vector-quantised matrix with a low-rank adapter next to it
 * (Sec. 5, "Combination of GPTVQ with LoRA adapters": adapters are trained on top of the
 * quantised base model and served with it; any scaling of the update is folded into B).
 *   A_f16  fp16 [rank, in]  row-major (device), 16-byte aligned
 *   B_f16  fp16 [out, rank] row-major (device), 16-byte aligned
 *   rank   0 (no adapter: plain y = W x) or a multiple of 8, at most 64
 * Two launches on `stream`: t = A x in fp32 into `workspace`, then the GEMV kernel, which
 * adds B[row, :] . t (fp32) to every row total before it is rounded and stored.
 * `workspace` is device memory owned by the caller, 16-byte aligned, of at least
 * vq_lora_workspace_bytes(count) bytes (256 bytes per product); its contents are overwritten
 * and mean nothing afterwards; calls that share a workspace must not overlap in time.
 * Everything else as for vq_gemv / vq_gemv_multi (`lora` is a HOST array of `count`
 * descriptors holding device pointers); every representation that vq_gemv takes.
 */
typedef struct vq_lora_desc {
  const void* A_f16;
  const void* B_f16;
  int32_t rank;
  int32_t reserved;     /* 0 */
} vq_lora_desc;

VQ_API int vq_lora_workspace_bytes(int count, size_t* bytes);
VQ_API int vq_gemv_lora(const vq_desc* desc, const void* idx_dev, const void* cb_dev,
                        const void* x_f16, const void* A_f16, const void* B_f16, int rank,
                        void* workspace, size_t workspace_bytes, void* y, int y_dtype,
                        void* stream);
VQ_API int vq_gemv_lora_multi(int count, const vq_desc* descs, const void* const* idx_dev,
                              const void* const* cb_dev, const void* const* x_f16,
                              const vq_lora_desc* lora, void* workspace, size_t workspace_bytes,
                              void* const* y, int y_dtype, void* stream);

/*
 * vq_gemv_lora_multi for callers that cannot allocate or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace; t = A x lives in a 64 KB array that is part of the library's code object on every
 * GPU it runs on (held until the process ends).  count <= 256, otherwise VQ_ERR_BAD_ARG.  The
 * call allocates nothing.  All calls on one GPU share that array: calls that overlap in time on
 * one GPU (different streams, or threads) race on it and must be serialised by the caller;
 * calls on one stream are ordered.  Nothing in the array needs clearing between calls (every
 * slot that is read has been written by the same call).  Results are bit-identical to
 * vq_gemv_lora_multi.
 */
VQ_API int vq_gemv_lora_multi_static(int count, const vq_desc* descs, const void* const* idx_dev,
                                     const void* const* cb_dev, const void* const* x_f16,
                                     const vq_lora_desc* lora, void* const* y, int y_dtype,
                                     void* stream);

/*
 * Y[out, B] = W X[in, B]  (the batched / prefill form of the same product; a
 * dense contraction, decoded tiles go through LDS to the matrix cores).
 * X is fp16 with row stride ldx >= B elements (batch index contiguous), Y has
 * row stride ldy >= B and dtype y_dtype; accumulation is fp32.  ldx and ldy
 * are multiples of 8 elements and the X buffer spans in*ldx elements (rows are
 * read in 8-element pieces up to the stride).  B in [1, 65536].
 */
VQ_API int vq_gemm_batched(const vq_desc* desc, const void* idx_dev, const void* cb_dev,
                    const void* X_f16, int B, int ldx, void* Y, int ldy, int y_dtype,
                    void* stream);

/*
 * Dense reconstruction W[out, in], fp16 row-major: W[r, c+t] = cb[g][I_g[v]][t]
 * copied bit for bit (Sec. 3.2 decode step on its own; the appendix "Further
 * on-device results" times exactly this transfer + decode on a 11008x4096 layer).
 */
VQ_API int vq_decode_dense(const vq_desc* desc, const void* idx_dev, const void* cb_dev,
                    void* W_f16, void* stream);

/*
 * Quantiser side (offline; paragraph "Codebook Initialization"): the two steps of the
 * Hessian-weighted EM that initialises the codebook of every group (desc->codebook_dtype is
 * ignored: weights and codebooks are fp32 here).  Implemented for d = 1, 2 or 4, k = 4, 8, 16,
 * 32, 64 or 256, and groups of 1, 4, 8, 16, 32, 64, 128 or 256 rows x 256 columns (one row: k * d <= 64;
 * 4 rows: d = 1 or 2),
 * which covers the group shapes of every representation the decode side takes; out_features is
 * a multiple of max(group_rows, 8).
 *
 *   W_f32      fp32 W[out, in], row-major, contiguous
 *   hdiag_f32  fp32 h[in], h[c] = 1 / [H^-1]_cc: the diagonal D of eq. "kmeans_objective"; the
 *              vector on columns c .. c+d-1 uses D_i = diag(h[c], ..., h[c+d-1])
 *   cb_f32     fp32 cb[g][m][t] in the canonical group order, t < d
 *   assign_u8  one byte per vector, assign[r][c/d], row-major (out x in/d bytes)
 *
 * vq_em_assign (E-step, eq. "hessian_e_step"; also the VQ_quant operation of Algorithm 2):
 *   assign[r][v] = argmin_m  sum_t h[c+t]*(W[r][c+t] - cb[g][m][t])^2,  c = d*v,
 *   evaluated in binary32 with every operation rounded separately in the order subtract, square,
 *   times weight, add (t ascending); the lowest m wins a tie.
 * vq_em_update (M-step, closed form below eq. "hessian_m_step"):
 *   cb_out[g][m][t] = sum h[c+t]*W[r][c+t] / sum h[c+t] over the vectors of group g with
 *   assign = m, and 0 where that sum of weights is 0 (the pseudoinverse of the text: an empty
 *   cluster becomes the zero vector).  binary32 sums in a fixed order: deterministic.
 *   Assignment bytes >= k are ignored.
 * All pointers are device memory, 16-byte aligned; cb_out must not alias the inputs.
 */
VQ_API int vq_em_assign(const vq_desc* desc, const void* W_f32, const void* hdiag_f32,
                        const void* cb_f32, void* assign_u8, void* stream);
VQ_API int vq_em_update(const vq_desc* desc, const void* W_f32, const void* hdiag_f32,
                        const void* assign_u8, void* cb_f32_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VQ_H_ */
