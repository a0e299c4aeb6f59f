/*
 * mx.h -- C ABI of the MI355X (gfx950) microscaling library.
 *
 * The library implements, as hand-written HIP kernels, the data-parallel hot path of
 * multi-format QAT with anchor storage:
 *   - block-wise MX quantization of fp32 / bf16 tensors (Eq. (1), Eq. (2)),
 *   - Slice-and-Scale conversion of an 8-bit anchor (MXINT8 / MXFP8 E4M3) to a lower MXINT /
 *     MXFP format without going back to fp32 weights (Eq. (4), Eq. (6)),
 *   - the fused quantize-dequantize ("fake-quant") of the training forward pass (Sec. 3.2,
 *     Eq. (7)) and the reconstruction V^ = X * P (Sec. 3.3 notation).
 *
 * Conventions common to every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller (borrowed for the call); the
 *     descriptor structs themselves and the format structs are HOST memory.
 *   - Nothing is allocated, freed or synchronized by the library, on the device or on the host.
 *     Work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to void*; NULL =
 *     the default stream) and is complete when that stream reaches the end of the enqueued work.
 *   - The library keeps no state between calls apart from facts it memoizes per device on first
 *     use (its number of compute units; that a kernel has been granted its LDS size there; the
 *     device address of the descriptor array of mx_slice_and_scale_batched_noalloc); calls from
 *     several threads are safe (for that one entry point: as long as they do not overlap on a GPU).
 *   - All arguments are validated on the host before anything is launched: a call that returns
 *     an error has had no effect on device memory.  Errors are reported by return code only.
 *   - Dense tensors are row-major [rows, cols] with leading dimension `ld` (elements, >= cols).
 *   - Packed tensors are block-contiguous: codes[outer][nblocks][block * bits / 8] bytes and
 *     scales[outer][nblocks] bytes, the block axis innermost.  For axis = 1 (blocks run along a
 *     row) outer = rows, nblocks = cols / block.  For axis = 0 (blocks run down a column) the
 *     packed tensor is stored transposed: outer = cols, nblocks = rows / block.
 *   - Inside one block, element i occupies bits [i * w, (i + 1) * w) of the block's
 *     little-endian bit string (w = element width).  MXINT codes are two's complement in w bits,
 *     MXFP codes are sign | exponent | mantissa.
 *   - A scale is one E8M0 byte: X = 2^(byte - 127); byte 255 marks a block that held NaN / Inf.
 *   - MXINT uses the integer view of the paper's Eq. (4): e_max(b) = b - 2, symmetric clip
 *     +-(2^(b-1) - 1).  Rounding: MX_ROUND_DEFAULT is half-away-from-zero for MXINT and
 *     half-to-even for MXFP.
 *   - Pointers must be 16-byte aligned (MX_ERR_ALIGN otherwise), `ld` a multiple of 8 elements.
 */
#ifndef MX_H_
#define MX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MX_OK = 0,
  MX_ERR_NULL = 1,        /* a required pointer is NULL                                        */
  MX_ERR_FORMAT = 2,      /* unknown element / scale / rounding, or anchor -> target is not a  */
                          /* down-conversion inside one family                                 */
  MX_ERR_SHAPE = 3,       /* negative size, blocked extent not a multiple of block, ld < cols  */
  MX_ERR_ALIGN = 4,       /* pointer not 16-byte aligned, or ld not a multiple of 8            */
  MX_ERR_UNSUPPORTED = 5, /* valid request this build has no kernel for                        */
  MX_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch                                */
  MX_ERR_WORKSPACE = 7    /* workspace too small                                               */
} mx_status_t;

/* Element formats.  Sec. 3.2 "Evaluation" lists MXINT b = 2..8 and MXFP E2M1, E2M2, E3M2, E3M3,
 * E4M3; E2M3 is the OCP FP6 variant added by the benchmark definition. */
typedef enum {
  MX_INT8 = 0, MX_INT7, MX_INT6, MX_INT5, MX_INT4, MX_INT3, MX_INT2,
  MX_FP8_E4M3, MX_FP7_E3M3, MX_FP6_E3M2, MX_FP6_E2M3, MX_FP5_E2M2, MX_FP4_E2M1,
  MX_ELEM_COUNT
} mx_elem_t;

typedef enum { MX_SCALE_E8M0 = 0 } mx_scale_t;
typedef enum { MX_F32 = 0, MX_BF16 = 1 } mx_dtype_t;
typedef enum { MX_ROUND_DEFAULT = 0, MX_ROUND_HALF_AWAY = 1, MX_ROUND_HALF_EVEN = 2 } mx_round_t;

/* An MX format: element type, scale type, block size k and the axis the blocks run along
 * (Sec. 2 "Microscaling formats"; Sec. 3.3 notation). */
typedef struct {
  mx_elem_t elem;
  mx_scale_t scale;
  int32_t block;   /* k: 16, 32, 64 or 128 (down a column, axis 0: the row count must be a multiple of 32 also for
                      k = 16); 32 in the GEMM */
  int32_t axis;    /* 1: along rows (last axis); 0: down columns */
  mx_round_t round;
} mx_format_t;

/* Dense matrix in device memory. */
typedef struct {
  void* data;
  mx_dtype_t dtype;
  int64_t rows, cols, ld;
} mx_dense_t;

/* Packed MX tensor in device memory: outer * nblocks blocks. */
typedef struct {
  void* codes;
  uint8_t* scales;
  int64_t outer, nblocks;
} mx_packed_t;

/* Element width in bits, e_max (Sec. 3.3 notation), or -1 for an unknown element. */
int mx_elem_bits(mx_elem_t elem);
int mx_elem_emax(mx_elem_t elem);

/* Bytes needed for the codes and the scales of a [rows, cols] tensor in format f. */
mx_status_t mx_packed_bytes(const mx_format_t* f, int64_t rows, int64_t cols, size_t* code_bytes,
                            size_t* scale_bytes);

/* Q_f, Eq. (1) and Eq. (2): per block, shared_exp = floor(log2 max|V_i|) - e_max(f), clamped to
 * [-127, 127]; P_i = quantize_f(V_i / 2^shared_exp).  src: dense, read-only.  dst: packed with
 * outer / nblocks matching src and f->axis; dst must not overlap src.  An all-zero block gets
 * scale byte 0; a block holding NaN / Inf gets scale byte 255 and zero codes.
 * Codes are packed in runs of 32: with blocks of 16 and an odd number of blocks in the tensor,
 * element widths other than 8 and 4 bits are MX_ERR_UNSUPPORTED (here and in mx_dequant). */
mx_status_t mx_quantize(const mx_format_t* f, const mx_dense_t* src, const mx_packed_t* dst, void* stream);

/* Q_{A->t}, Eq. (4) (SSMXINT) and Eq. (6) (SSMXFP): P_l = quantize_t(P_h / 2^De),
 * X_l = X_h * 2^De, De = e_max(anchor) - e_max(target).  The anchor must be an 8-bit format
 * (MX_INT8 or MX_FP8_E4M3) and the target a narrower format of the same family with the same
 * block size; the axis is irrelevant (a flat run of blocks).  The scale byte saturates at 254;
 * 255 stays 255.  target->outer * target->nblocks must equal the anchor's block count.
 * The target must not overlap the anchor.  Targets of odd width are converted in runs of 32 codes:
 * MX_ERR_UNSUPPORTED if a tensor's code count is not a multiple of 32 (only possible with block 16). */
mx_status_t mx_slice_and_scale(const mx_format_t* fa, const mx_packed_t* anchor, const mx_format_t* ft,
                               const mx_packed_t* target, void* stream);

/* The same conversion for n tensors in ONE conversion launch (a whole checkpoint, Sec. 3.5
 * "Inference").  anchors / targets: host arrays of n descriptors, free to reuse when the call
 * returns.  workspace: device memory of at least
 * mx_slice_and_scale_batched_workspace(n, total number of blocks) bytes, 16-byte aligned; a few
 * tiny set-up kernels write the launch tables there on `stream` ahead of the conversion kernel
 * (nothing is copied from the host, so the call can be captured in a HIP graph).  The workspace
 * must stay untouched until the work has completed.  MX_ERR_WORKSPACE if it is too small. */
size_t mx_slice_and_scale_batched_workspace(int32_t n, int64_t total_blocks);
mx_status_t mx_slice_and_scale_batched(const mx_format_t* fa, const mx_format_t* ft, int32_t n,
                                       const mx_packed_t* anchors, const mx_packed_t* targets,
                                       void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid it): mx_slice_and_scale_batched with the launch tables in a fixed array inside the library instead of
 * a workspace.  It calls no allocator of any kind, on the host or on the device.  The array holds
 * MX_SS_NOALLOC_MAX_SEGMENTS descriptors of 64 bytes (1 MiB of device memory on every GPU the library runs on,
 * held until the process ends); one descriptor covers up to 2^16 pieces of 16 anchor codes (2^13 when the tensors
 * are small), and every tensor rounds up to whole descriptors for its codes and for its scale bytes: a whole
 * 8B-parameter checkpoint (224 tensors, 7 G elements) takes about 7 000.  MX_ERR_WORKSPACE, with nothing enqueued,
 * when a call needs more.  Results are those of mx_slice_and_scale_batched bit for bit.
 * All calls on one GPU share that GPU's array, which is rewritten by every call: two such calls must not overlap in
 * time on one GPU (same stream, or ordered by events); calls on different GPUs are independent. */
#define MX_SS_NOALLOC_MAX_SEGMENTS 16384
mx_status_t mx_slice_and_scale_batched_noalloc(const mx_format_t* fa, const mx_format_t* ft, int32_t n,
                                               const mx_packed_t* anchors, const mx_packed_t* targets, void* stream);

/* Several targets from one pass over the anchor (the "convert the anchor to every lower format" workload of
 * Sec. 3.5 "Inference"): the anchor codes and scales are read once and n_targets (1..3) packed tensors are written,
 * each exactly what mx_slice_and_scale gives for its format.  fts / targets: host arrays of n_targets entries, the
 * formats in increasing mx_elem_t order and with one rounding mode.  Sets with a kernel: any single target;
 * {INT6, INT4}; {E3M2, E2M3, E2M1} and its pairs.  MX_ERR_UNSUPPORTED for other sets.
 * The batched form takes targets[i * n_targets + q] = target q of tensor i; workspace as for
 * mx_slice_and_scale_batched. */
mx_status_t mx_slice_and_scale_multi(const mx_format_t* fa, const mx_packed_t* anchor, int32_t n_targets,
                                     const mx_format_t* fts, const mx_packed_t* targets, void* stream);
mx_status_t mx_slice_and_scale_multi_batched(const mx_format_t* fa, int32_t n_targets, const mx_format_t* fts, int32_t n,
                                             const mx_packed_t* anchors, const mx_packed_t* targets, void* workspace,
                                             size_t workspace_bytes, void* stream);

/* Fake-quant of the QAT forward pass.  anchor == NULL: dst = DQ(Q_target(src)) (Sec. 3.2).
 * anchor != NULL: dst = DQ(Q_{A->t}(Q_A(src))) (Eq. (7)).  src and dst have the same shape;
 * dst may be src itself (in place) but must not partially overlap it.  Nothing but dst is
 * written.  The backward pass of the straight-through estimator is the identity and needs no
 * kernel. */
mx_status_t mx_fake_quant(const mx_format_t* target, const mx_format_t* anchor, const mx_dense_t* src,
                          const mx_dense_t* dst, void* stream);

/* V^ = X * P (Sec. 3.3 notation) into a dense matrix; scale byte 255 gives NaN.  Results that
 * are not representable in dst->dtype round to nearest even (overflow gives +-Inf). */
mx_status_t mx_dequant(const mx_format_t* f, const mx_packed_t* src, const mx_dense_t* dst, void* stream);

/* Fused consumer of the anchor (Sec. 3.5 "Inference": the model runs with W_t = Q_{A->t}(W_A) generated on
 * demand):
 *     C[m, n] = sum_k DQ(A)[m, k] * DQ(Q_{A->t}(W_A))[n, k],   t = MXFP4 E2M1,
 * with the Slice-and-Scale conversion of Eq. (6) done in registers and the product taken by the CDNA4 scaled
 * MX matrix instruction with fp32 accumulation; W_t is never written to memory.
 *   a: MXFP8 E4M3 activations blocked along K: outer = M, nblocks = K / 32 (mx_quantize of a [M, K] tensor).
 *   w_anchor: MXFP8 E4M3 anchor of the weight, K-contiguous: outer = N, nblocks = K / 32 (mx_quantize of
 *             W[N, K] along axis 1, or of W[K, N] along axis 0).
 *   c: dense fp32 [M, N], written (not accumulated into).
 * K must be a multiple of 128.  MX_ERR_UNSUPPORTED for shapes this build has no kernel for (for M > 48: K >= 2^24
 * or a row stride of c of 2^22 elements or more).  Each output is an
 * fp32 sum over K in a fixed order (results are reproducible run to run). */
mx_status_t mx_gemm_ss_fp4(const mx_packed_t* a, const mx_packed_t* w_anchor, const mx_dense_t* c, void* stream);

/* The same product for callers that can lend a workspace of mx_gemm_ss_fp4_workspace(N, K) = N K / 2 + N K / 32 bytes
 * (device memory, 16-byte aligned, borrowed for the duration of the enqueued work; MX_ERR_ALIGN / MX_ERR_WORKSPACE when
 * it is misaligned or smaller).  Two things are done with it.
 *   From MX_GEMM_HOIST_MIN_ROWS rows of A on, and when C has enough tiles of 256 x 256 (from 1024 rows on: of 128 x 256)
 *   to fill the GPU, W_t (Eq. (6)) is generated once per call into the workspace -- MXFP4 codes and scale bytes -- and
 *   multiplied from there by a kernel that has the whole compute unit for the product (the on-the-fly kernels slice
 *   every tile of W once per 256 rows of A).  The results are those of mx_gemm_ss_fp4 bit for bit.
 *   Otherwise, from 49 rows on, when the tiles of C leave most compute units without one (a narrow N), K is split over
 *   2 to 8 workgroups per tile whose partial sums go through the workspace and are added in the order of the slices:
 *   still a fixed order (reproducible run to run), but not mx_gemm_ss_fp4's, so the two results differ by fp32 rounding.
 * In every other case, and with workspace == NULL, this is mx_gemm_ss_fp4. */
#define MX_GEMM_HOIST_MIN_ROWS 512
size_t mx_gemm_ss_fp4_workspace(int64_t n, int64_t k);
/* The number of K slices mx_gemm_ss_fp4_ws works with for an [m, k] x [n, k] product and a workspace of that size on the
 * current device: 1 when its result is mx_gemm_ss_fp4's bit for bit, 2 .. 8 when partial sums are added afterwards. */
int mx_gemm_ss_fp4_ws_slices(int64_t m, int64_t n, int64_t k, size_t workspace_bytes);
mx_status_t mx_gemm_ss_fp4_ws(const mx_packed_t* a, const mx_packed_t* w_anchor, const mx_dense_t* c, void* workspace,
                              size_t workspace_bytes, void* stream);

/* The same product for a W_t the caller keeps (Sec. 3.5 "Inference": a precision switch converts the anchor once,
 * W_t = Q_{A->t}(W_A), and every later call runs with that W_t):
 *     C[m, n] = sum_k DQ(A)[m, k] * DQ(W_t)[n, k].
 *   a: as for mx_gemm_ss_fp4.
 *   w_t: MXFP4 E2M1 weights, K-contiguous: outer = N, nblocks = K / 32, 16 bytes of codes per block (what
 *        mx_slice_and_scale writes for an E4M3 anchor and the target E2M1, or mx_quantize to E2M1).
 *   c: dense fp32 [M, N], written.
 * K must be a multiple of 128; MX_ERR_UNSUPPORTED for M > 48 and K >= 2^24 or a row stride of c of 2^22 elements or
 * more.  With w_t = the Slice-and-Scale of an anchor the results are those of mx_gemm_ss_fp4 on that anchor, bit for bit
 * (the same kernels without the slicing step; above 48 rows the kernel with tiles of 256 or 128 rows x 256 columns where
 * such tiles fill the GPU).  Up to 48 rows the call streams W_t once: half the anchor's bytes. */
mx_status_t mx_gemm_fp8_fp4(const mx_packed_t* a, const mx_packed_t* w_t, const mx_dense_t* c, void* stream);

/* The same for callers that can lend a workspace (device memory, 16-byte aligned, borrowed for the duration of the
 * enqueued work; MX_ERR_ALIGN when misaligned): from 49 rows of A on, when the tiles of C leave most compute units
 * without one, K is split over 2 to 8 workgroups per tile whose partial sums go through the workspace and are added in
 * the order of the slices -- a fixed order, but not mx_gemm_fp8_fp4's, so the two results differ by fp32 rounding.
 * mx_gemm_fp8_fp4_workspace(m, n, k) is what the split the library would choose on the current device needs (0: it
 * would not split); mx_gemm_fp8_fp4_ws_slices the number of slices for a workspace of a given size (1: the result is
 * mx_gemm_fp8_fp4's bit for bit).  With workspace == NULL, or one too small for any split, this is mx_gemm_fp8_fp4. */
size_t mx_gemm_fp8_fp4_workspace(int64_t m, int64_t n, int64_t k);
int mx_gemm_fp8_fp4_ws_slices(int64_t m, int64_t n, int64_t k, size_t workspace_bytes);
mx_status_t mx_gemm_fp8_fp4_ws(const mx_packed_t* a, const mx_packed_t* w_t, const mx_dense_t* c, void* workspace,
                               size_t workspace_bytes, void* stream);

const char* mx_status_str(mx_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* MX_H_ */
