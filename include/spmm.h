/*
 * spmm.h - C ABI of the MI355X (gfx950) structured-sparse INT8 SpMM library.
 *
 * The library computes   out = postops( W_sparse . X )   where
 *   W  int8  [N][K]  weight matrix pruned in constant 4x1 blocks (paper Section 3.1,
 *                    Figure 1), handed over dense-with-zeros on the host and kept
 *                    compressed on the device,
 *   X  uint8 [K][M]  dense activations (tokens contiguous), device memory,
 *   accumulation is unsigned 8-bit x signed 8-bit into 32-bit integers (Section 3.2,
 *   Algorithm 1), followed by the fused post-operator chain of Section 3.3 / Figure 3
 *   (BiasAdd, GeLU, Quantize) and the lookup table of Algorithm 2 for the
 *   low-precision GELU chain.
 *
 * Axis names used throughout (the paper's own letters change between paragraphs):
 *   N = output channels = rows of W and of out,  K = reduction dimension,
 *   M = tokens = columns of X and of out.
 *
 * Conventions: C linkage, no exceptions cross the boundary, every call returns a
 * status and leaves its outputs untouched on error.  "host" / "device" is stated
 * for every pointer.  No call reads or writes memory it was not handed.
 */
#ifndef SPMM_H_
#define SPMM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spmm_handle spmm_handle_t; /* opaque; owns its host and device storage */

typedef enum {
    SPMM_OK = 0,
    SPMM_E_ARG = 1,         /* null pointer, non-positive size, ld < extent, bad enum, missing table */
    SPMM_E_UNSUPPORTED = 2, /* valid request outside the implemented range (e.g. K too large)      */
    SPMM_E_ALLOC = 3,       /* host or device allocation failed                                     */
    SPMM_E_DEVICE = 4       /* a HIP call or kernel launch failed                                   */
} spmm_status_t;

/* Orientation of the 4x1 block (Section 3.1).  The paper places the sparsity dimension
 * on the output channels: a block is 4 consecutive output rows at one k, so four rows
 * share their k indices (Algorithm 1 broadcasts four weight words against one gathered
 * input).  The transposed reading (one row, 4 consecutive k) is accepted as well; it only
 * changes how non-zero blocks are counted and how well the weight compresses. */
typedef enum {
    SPMM_BLOCK_N4K1 = 0, /* 4 consecutive output rows x 1 k */
    SPMM_BLOCK_N1K4 = 1  /* 1 output row x 4 consecutive k  */
} spmm_block_t;

typedef enum { SPMM_POST_NONE = 0, SPMM_POST_GELU = 1, SPMM_POST_TABLE = 2 } spmm_postop_t;

typedef enum {
    SPMM_OUT_S32 = 0, /* raw accumulator; scales, bias and post-op are ignored */
    SPMM_OUT_F32 = 1,
    SPMM_OUT_S8 = 2,
    SPMM_OUT_U8 = 3
} spmm_out_t;

/* Post-operator chain (Section 3.3).  Pointers are DEVICE pointers owned by the caller
 * and must stay valid until the launch that uses them has finished.
 *
 *   acc = sum_k W[n][k] * (X[k][m] - x_zero_point)                          (int32)
 *   y   = fmaf((float)acc, w_scale[n] * x_scale, bias ? bias[n] : 0)         (binary32)
 *   POST_NONE: z = y        POST_GELU, F32 out: z = y * Phi(y)  (erf form)
 *   Sum (Figure 3), when `sum` is given: z = z + sum[n][m], one binary32 add of a second
 *            tensor of the output's shape (the residual), after BiasAdd / GeLU and before
 *            Quantize.  Not available with S32 output, nor with the table chain
 *            (GELU + S8/U8), whose value is a function of one key: SPMM_E_UNSUPPORTED.
 *   S8/U8 out without GELU: q = sat(rint(z * (1/out_scale)) + out_zero_point)
 *   S8/U8 out with GELU   : t = sat_s8(rint(y * (1/mid_scale)));  q = lut[t + 128]
 *   POST_TABLE (S8/U8 out only): the same look-up with the caller's own 256-entry table of any
 *            element-wise chain (Algorithm 2 in general; other output types: SPMM_E_UNSUPPORTED)
 * rint is round-half-to-even; 1/scale is one binary32 division done on the host.
 */
typedef struct {
    const float *w_scale;   /* device [N]; required unless out_type is S32               */
    float x_scale;          /* scalar activation scale                                   */
    int32_t x_zero_point;   /* activation zero point in [0,255], normally 0              */
    const float *bias;      /* device [N] or NULL                                        */
    spmm_postop_t postop;
    spmm_out_t out_type;
    float out_scale;        /* S8/U8 without GELU: output quantisation scale (> 0)       */
    int32_t out_zero_point; /* S8/U8 without GELU                                        */
    float mid_scale;        /* GELU / TABLE + S8/U8: scale of the pre-activation code (> 0) */
    const int8_t *lut;      /* GELU / TABLE + S8/U8: device [256] table (spmm_make_gelu_lut
                               builds the GELU one)                                        */
    const float *sum;       /* device [N][ld_sum] binary32 or NULL: operand of Sum       */
    int64_t ld_sum;         /* >= M when sum is given (in elements)                       */
} spmm_epilogue_t;

/* Compress a weight matrix (Section 3.2: the kernel is specialised on the sparse weight
 * and its indices; padding of the block count as in the note after Algorithm 1).
 *   W_host  host, int8 [N][ldw], dense with zeros; ANY content is accepted and packed
 *           losslessly (a non-conforming matrix just compresses worse).
 *   N, K    > 0;  K <= 65536;  ldw >= K.
 *   block   orientation used for counting blocks (see spmm_block_t).
 *   out_handle  receives a new handle bound to the current HIP device; the caller
 *           releases it with spmm_destroy.  W_host is not referenced after return.
 * Errors: SPMM_E_ARG, SPMM_E_UNSUPPORTED, SPMM_E_ALLOC, SPMM_E_DEVICE. */
spmm_status_t spmm_pack(const int8_t *W_host, int64_t N, int64_t K, int64_t ldw,
                        spmm_block_t block, spmm_handle_t **out_handle);

/* Same compression as spmm_pack but HOST ONLY: no HIP call is made and the handle owns
 * no device memory, so it can be inspected (spmm_unpack, spmm_info, spmm_layout_*) on a
 * machine without a GPU.  spmm_run on such a handle returns SPMM_E_ARG. */
spmm_status_t spmm_pack_host(const int8_t *W_host, int64_t N, int64_t K, int64_t ldw,
                             spmm_block_t block, spmm_handle_t **out_handle);

/* spmm_pack with options (Section 3.2: the blocking is tunable offline for a given weight).
 *   flags   SPMM_PACK_HOST_ONLY     as spmm_pack_host
 *           SPMM_PACK_REORDER_ROWS  the library chooses the ORDER of the output rows: whole
 *                   block-rows (4 consecutive rows for N4K1, single rows for N1K4; a trailing
 *                   partial block-row stays last) are clustered by the overlap of their k
 *                   lists, so that a row tile multiplies a smaller union.  The handle then
 *                   stands for the weight with its rows in that order: row i of the output,
 *                   of w_scale, of bias and of the Sum operand in spmm_run is row
 *                   order[i] of the matrix given here (spmm_row_order).  A following layer
 *                   absorbs the order by the same permutation of its weight's columns, done
 *                   once offline.  spmm_unpack still returns the matrix as given.
 *   other bits: SPMM_E_ARG. */
#define SPMM_PACK_HOST_ONLY 1u
#define SPMM_PACK_REORDER_ROWS 2u
spmm_status_t spmm_pack_ex(const int8_t *W_host, int64_t N, int64_t K, int64_t ldw,
                           spmm_block_t block, uint32_t flags, spmm_handle_t **out_handle);

/* The row order of a packed weight: order_host (host, int32 [N]) receives, for every row i
 * the handle computes, the row of the caller's matrix it is (the identity unless the weight
 * was packed with SPMM_PACK_REORDER_ROWS; always a permutation of 0..N-1). */
spmm_status_t spmm_row_order(const spmm_handle_t *h, int32_t *order_host);

/* Exact inverse of spmm_pack (whatever the row order chosen): writes the dense-with-zeros
 * matrix into host memory W_host_out [N][ldw], ldw >= K (all N*K entries are written). */
spmm_status_t spmm_unpack(const spmm_handle_t *h, int8_t *W_host_out, int64_t ldw);

/* Sizes of a packed weight.  Any output pointer may be NULL.
 *   nnz_blocks     4x1 blocks with at least one non-zero element (orientation of pack)
 *   padded_blocks  block slots the device layout multiplies (>= nnz_blocks; padding and
 *                  zero fill are never counted in any reported rate)
 *   device_bytes   bytes of device memory the handle owns */
spmm_status_t spmm_info(const spmm_handle_t *h, int64_t *N, int64_t *K, int64_t *nnz_blocks,
                        int64_t *padded_blocks, int64_t *device_bytes);

/* Geometry of the compressed device layout (any output pointer may be NULL).  The weight
 * is cut into row tiles of `tile_rows` output rows; per row tile and per K segment of
 * `segment_rows` consecutive k, the k positions where any row of the tile is non-zero are
 * listed and cut into steps of `step_k` slots (the padding of the block count described
 * after Algorithm 1, in units of the matrix instruction's accumulation depth). */
spmm_status_t spmm_layout_dims(const spmm_handle_t *h, int32_t *tile_rows, int32_t *step_k,
                               int32_t *segment_rows, int64_t *n_tiles, int64_t *n_segments,
                               int64_t *n_steps);

/* Copy the compressed layout into HOST buffers sized from spmm_layout_dims (NULL = skip):
 *   vals    uint8 [n_steps][64 lanes][16]  weight of row (lane % 16) at list slot 16*(lane/16)+t
 *   idx     uint32 [n_steps][32]           entry 8g+t = k_local[16g+t] | k_local[16g+8+t] << 16,
 *                                           k_local relative to the segment start, in an
 *                                           order chosen for LDS banking; padding slots
 *                                           have zero weights and a valid row index
 *   seg_ptr int32 [n_tiles*n_segments + 1] first step of (tile, segment), CSR style
 *   rowsum  int32 [n_tiles*tile_rows]      sum over k of each (padded) row of W */
spmm_status_t spmm_layout_export(const spmm_handle_t *h, uint8_t *vals_host, uint32_t *idx_host,
                                 int32_t *seg_ptr_host, int32_t *rowsum_host);

/* out = postops(W . X), asynchronous on `hip_stream` (a hipStream_t, NULL = default
 * stream).  Performs no allocation and no synchronisation; reads no host memory after
 * it returns.  The handle is immutable: concurrent calls on different streams are fine.
 *   X_dev   device, uint8 [K][ldx], ldx >= M
 *   out_dev device, [N][ldo] of the element type of ep->out_type, ldo >= M (in elements)
 *   M > 0
 * Any alignment, any leading dimension >= M and any token count work.  The fast paths need X_dev
 * and out_dev (and sum) 16-byte aligned with row pitches that are multiples of 16 bytes; M itself
 * may be anything then (a ragged last token tile costs only that tile).  Unaligned operands are
 * read through aligned dwords and written in the widest aligned pieces, which is noticeably
 * slower for short batches and several times slower for long ones: pad the pitches.
 * The current HIP device must be the one the handle was packed on (SPMM_E_ARG otherwise).
 * Errors: SPMM_E_ARG (also: missing w_scale / lut, non-positive scales, zero point out
 * of range, ld_sum < M), SPMM_E_UNSUPPORTED (Sum with S32 output or with the table chain),
 * SPMM_E_DEVICE. */
spmm_status_t spmm_run(const spmm_handle_t *h, const uint8_t *X_dev, int64_t M, int64_t ldx,
                       const spmm_epilogue_t *ep, void *out_dev, int64_t ldo, void *hip_stream);

/* spmm_run with activations in TOKEN-TILE-MAJOR order (Section 3.2 re-structures the input for the
 * kernel's blocking; this is that layout for this kernel).  A tile-major matrix of R rows and M tokens is
 *     1-byte elements [ceil(M / SPMM_X_TILE)][R][SPMM_X_TILE],   T[t][r][j] = A[r][SPMM_X_TILE * t + j],
 * device memory, 16-byte aligned, the last tile padded to full width (the padding of an input is read
 * and never used; that of an output is not written).  A workgroup's token tile is then three or four
 * contiguous regions of memory instead of K pieces a row pitch apart, which is what HBM wants when X
 * does not come out of a cache.
 *   tiled   SPMM_TILED_X    X_dev is tile-major (R = K); ldx is ignored
 *           SPMM_TILED_OUT  the S8 / U8 output is written tile-major (R = N), i.e. as the next layer's
 *                           tile-major activations; ldo is ignored; with S32 / F32 output:
 *                           SPMM_E_UNSUPPORTED.  The Sum operand stays row-major.
 *           other bits: SPMM_E_ARG.
 * Everything else as in spmm_run; a tile-major operand must be smaller than 2 GiB
 * (SPMM_E_UNSUPPORTED otherwise). */
#define SPMM_X_TILE 32
#define SPMM_TILED_X 1u
#define SPMM_TILED_OUT 2u
spmm_status_t spmm_run_tiled(const spmm_handle_t *h, const uint8_t *X_dev, int64_t M, int64_t ldx,
                             const spmm_epilogue_t *ep, void *out_dev, int64_t ldo, uint32_t tiled,
                             void *hip_stream);

/* Algorithm 2: the 256-entry table of the chain dequantise(mid_scale) -> GELU ->
 * quantise(out_scale, out_zero_point), entry [i + 128] for key i in [-128, 127], computed
 * in double and rounded half to even.  lut_host is HOST memory; the caller copies it to
 * the device.  out_type must be S8 or U8 (U8 codes are stored as their byte). */
spmm_status_t spmm_make_gelu_lut(float mid_scale, float out_scale, int32_t out_zero_point,
                                 spmm_out_t out_type, int8_t lut_host[256]);

/* Kernel configuration chosen for a problem (reporting / tuning aid, Section 3.2 notes
 * that the tile size is tunable offline).  Writes the token-tile width, rows per
 * workgroup and the launch grid spmm_run would use for M tokens with 16-byte aligned operands
 * (unaligned operands may take a different kernel: their general paths need registers that the
 * widest configurations do not have). */
spmm_status_t spmm_plan(const spmm_handle_t *h, int64_t M, spmm_out_t out_type,
                        int32_t *token_tile, int32_t *rows_per_workgroup, int64_t *workgroups);

/* Override the automatic choice of kernel configuration for later spmm_run calls on this
 * handle; (0, 0) restores the automatic choice.
 *   token_tile 128: pipelined kernel, one workgroup per CU; variant 0 = automatic, 8 or 16 =
 *                   waves per workgroup (16 only holds weights with <= 6 steps per segment,
 *                   denser weights silently use 8).
 *   token_tile  96: the same kernel on 96-token tiles, variant 0 or 16 (16 waves; denser
 *                   weights silently use token tile 128 with 8 waves).
 *   token_tile  64: variant 101 / 102 = the simple, unpipelined kernel with 1 / 2 row tiles
 *                   per wave (an independent second implementation for cross-checks, and the
 *                   automatic choice for problems too small to fill the chip).
 *   token_tile 32, 16: variant 101 = the simple kernel on narrower token tiles (what the
 *                   automatic choice takes for short batches: more, smaller workgroups).
 *   token_tile 16, 32: variant 103 = the short-batch kernel, which keeps a workgroup's whole
 *                   [K x token_tile] slab of activations in LDS (K <= 4096 with 16-token tiles,
 *                   K <= 3072 with 32; a longer K silently runs variant 101).  The automatic
 *                   choice for short batches with 2048 < K <= 4096:
 *                   Section 4.3 measures the kernels at 32 tokens and the models at sequence
 *                   lengths of 16 to 384.
 *   token_tile 64, 32, 16: variant 104 = the streamed kernel: the simple kernel's segment by
 *                   segment staging with the weights arriving through rotating register sets
 *                   (the automatic choice for short batches from seven K segments on, K > 3072,
 *                   where the short-batch kernel does not apply).
 * Unsupported values return SPMM_E_UNSUPPORTED and change nothing.  Not thread-safe against
 * concurrent spmm_run on the same handle. */
spmm_status_t spmm_set_tuning(spmm_handle_t *h, int32_t token_tile, int32_t variant);

/* Base name of the device kernels spmm_run launches (for profilers). */
const char *spmm_kernel_name(void);

/* Full name, as a profiler prints it, of the kernel instantiation spmm_run would launch for
 * M tokens with this output type and post-operator, for 16-byte aligned operands and without
 * the Sum operand (see spmm_plan).  buf is HOST memory of buflen bytes; the name is
 * NUL-terminated and truncated if it does not fit. */
spmm_status_t spmm_kernel_variant(const spmm_handle_t *h, int64_t M, spmm_out_t out_type,
                                  spmm_postop_t postop, char *buf, int64_t buflen);
/* The same for spmm_run_tiled with these layout flags (for profilers; the callers are the
 * benchmark and the tests). */
spmm_status_t spmm_kernel_variant_tiled(const spmm_handle_t *h, int64_t M, spmm_out_t out_type,
                                        spmm_postop_t postop, uint32_t tiled, char *buf, int64_t buflen);

/* Measured ceiling of a candidate multiply instruction on the current device, registers only
 * (Section 3.2 builds the kernel around the widest integer multiply-accumulate the hardware has;
 * which one that is here is decided on measured rates):
 *   which 0: the int8 matrix instruction the kernels use (16x16x64), 1: the 4-wide int8 dot product.
 * Runs a short kernel on the default stream, synchronises, and writes 10^12 operations per second
 * (2 per multiply-accumulate) to *tera_ops_per_s (HOST).  Allocates a few bytes of device memory
 * for its own use and frees them.  Errors: SPMM_E_ARG, SPMM_E_ALLOC, SPMM_E_DEVICE. */
spmm_status_t spmm_measure_peak(int32_t which, double *tera_ops_per_s);

void spmm_destroy(spmm_handle_t *h); /* NULL is allowed */

const char *spmm_status_string(spmm_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* SPMM_H_ */
