/*
 * pdelta.h - C ABI of the 1-bit per-axis weight-delta library for AMD MI355X (gfx950).
 *
 * Notation follows the paper ("Per-Axis Weight Deltas for Frequent Model Updates", Section 2):
 *   W_b, W_f  base / fine-tuned weights of one linear layer, [d_out, d_in]
 *   B         = sign(W_f - W_b) in {-1,+1}^(d_out x d_in), stored one bit per entry
 *   v         per-axis FP16 scale: one entry per output feature ("row" mode, length d_out)
 *             or one per input feature ("col" mode, length d_in)
 *   W_hat     = v (.) B + W_b                                                    (Eq. 1)
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller; nothing is copied from or
 *     to the host.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on that stream and the call returns without synchronising; outputs are
 *     valid once the stream reaches that point.
 *   - The library allocates nothing and keeps no state between calls that affects a result
 *     (it remembers, per device, that a kernel has been granted its dynamic-LDS size).
 *   - Matrices are dense row-major: W[o, i] at W + o*d_in + i, X[m, i] at X + m*d_in + i,
 *     Y[m, o] at Y + m*d_out + o.
 *   - Bit layout: entry (o, i) is bit (i % 32) of the uint32 B_packed[o * (d_in/32) + i/32];
 *     bit 1 means B = +1, bit 0 means B = -1 (consecutive input indices share a word: the
 *     masks are packed along the input axis, Implementation remarks).  sign(0) is +1: the bit
 *     is !(W_f < W_b).
 *   - d_in must be a multiple of 32 (PDELTA_ESHAPE otherwise).  Every pointer must be 16-byte
 *     aligned (PDELTA_EALIGN).  v is always FP16 (Implementation remarks of the paper).
 *   - Return value: a pdelta_status.  All argument checks happen on the host before any HIP
 *     call, so they work without a GPU.  Nothing throws or aborts.  On an error return no
 *     kernel has been launched.  Inputs are never written.  Outputs must not alias inputs
 *     except where stated (pdelta_patch in place).
 *   - NaN / Inf inputs are outside the contract.
 *   - Developer knob: the environment variable PDELTA_TUNE="key=value,..." overrides the library's
 *     choice among its kernel variants (read once per call).  It changes no result beyond the
 *     order of floating-point summation; without it the built-in choices apply.
 */
#ifndef PDELTA_H
#define PDELTA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PDELTA_F16 = 0,  /* IEEE binary16 */
    PDELTA_BF16 = 1, /* bfloat16 */
    PDELTA_F32 = 2   /* IEEE binary32; accepted for Y only */
} pdelta_dtype;

typedef enum {
    PDELTA_ROW = 0,        /* v has d_out entries: W_hat[o,i] = W_b[o,i] + v[o] * B[o,i] */
    PDELTA_COL = 1,        /* v has d_in  entries: W_hat[o,i] = W_b[o,i] + v[i] * B[o,i] */
    PDELTA_PER_REQUEST = 2 /* pdelta_linear_variants only: each request names its own axis */
} pdelta_axis;

typedef enum {
    PDELTA_OK = 0,
    PDELTA_EINVAL = -1,     /* null pointer, non-positive dimension, bad axis, aliasing */
    PDELTA_ESHAPE = -2,     /* d_in is not a multiple of 32, or a dimension is too large */
    PDELTA_EALIGN = -3,     /* a pointer is not 16-byte aligned */
    PDELTA_EDTYPE = -4,     /* dtype code not accepted by this entry point */
    PDELTA_EWORKSPACE = -5, /* workspace missing or smaller than pdelta_pack_workspace_bytes */
    PDELTA_EHIP = -6        /* a kernel launch failed; hipGetLastError has been consumed */
} pdelta_status;

/* Bytes of device scratch pdelta_pack needs for these dimensions: fp64 partial sums of |dW|,
 * one per (row, tile of 1024 columns) and one per (tile of 64 rows, column), i.e.
 * 8 * (ceil(d_in / 1024) * d_out + ceil(d_out / 64) * d_in).  Returns 0 for non-positive
 * dimensions. */
size_t pdelta_pack_workspace_bytes(int64_t d_out, int64_t d_in);

/*
 * Offline companion: sign + bit-pack + per-axis scale initialisation.
 *   B      = sign(W_f - W_b)                            (Section 2, definition of B)
 *   Pack   : one bit per entry along the input axis     (per-layer compression algorithm,
 *                                                        packing step)
 *   v_row[o] = mean_i |W_f[o,i] - W_b[o,i]|,  v_col[i] = mean_o |W_f[o,i] - W_b[o,i]|
 *            (same algorithm, initial values of the Row and Col scale vectors), each the
 *            exact mean rounded once to FP16 (nearest-even).
 * Arguments
 *   W_f, W_b   in   [d_out, d_in], dtype w_dtype (PDELTA_F16 or PDELTA_BF16)
 *   B_packed   out  [d_out, d_in/32] uint32
 *   v_row      out  FP16 [d_out], may be NULL
 *   v_col      out  FP16 [d_in],  may be NULL
 *   workspace  scratch, >= pdelta_pack_workspace_bytes(d_out, d_in) bytes, 16-byte aligned;
 *              contents on entry are ignored, contents on exit are unspecified
 * Exactness: for FP16 inputs every difference is exact and the sums are formed without
 * rounding (fp64 inside a tile, 64-bit integers in units of 2^-24 across tiles), so the result
 * equals the fp64 reference bit for bit while each sum of |dW| stays below 2^29.  For BF16
 * inputs sums are accumulated in fp64 (exact whenever all |dW| are multiples of a common
 * 2^-q and the sum stays below 2^(53-q); otherwise within one FP16 ulp of the exact mean).
 * Partial sums are added in a fixed order: results are bit-reproducible for both dtypes.
 * d_out and d_in may each be at most 2^22.
 */
int pdelta_pack(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype,
                uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * pdelta_pack for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and error codes as pdelta_pack, minus the workspace: the partial sums go to an array
 * of pdelta_pack_noalloc_max_bytes() bytes (16 MiB) that the library owns, one copy per GPU,
 * resident until the process ends.  The call allocates and frees nothing.
 *   - Layers whose pdelta_pack_workspace_bytes(d_out, d_in) exceeds that size are rejected with
 *     PDELTA_EWORKSPACE when a scale vector is asked for (with v_row = v_col = NULL any size
 *     is accepted: the signs need no scratch).  16 MiB covers every projection of 7B / 8B-class
 *     models (14336 x 4096 needs 7.5 MiB).
 *   - All calls on one GPU share that GPU's array: two calls that may run at the same time on
 *     one GPU (different streams, different threads) race on it and give wrong scales.  Calls on
 *     one stream are ordered and safe; the contents left by one call are never read by the next.
 *   - PDELTA_EHIP when the runtime cannot give the array's device address.
 */
size_t pdelta_pack_noalloc_max_bytes(void);
int pdelta_pack_noalloc(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype,
                        uint32_t* B_packed, uint16_t* v_row, uint16_t* v_col, void* stream);

/*
 * Delta linear layer, row mode (Eq. 1 with v in R^(1 x d_out), then the layer forward
 * Y = X W_hat^T), evaluated without forming W_hat in memory:
 *   Y[m,o] = sum_i X[m,i] * W_b[o,i]  +  v_row[o] * sum_i X[m,i] * B[o,i]
 * Arguments
 *   X        in   [M, d_in],     dtype x_dtype (PDELTA_F16 or PDELTA_BF16)
 *   W_b      in   [d_out, d_in], same dtype as X
 *   B_packed in   [d_out, d_in/32] uint32
 *   v_row    in   FP16 [d_out]
 *   Y        out  [M, d_out], dtype y_dtype (PDELTA_F16, PDELTA_BF16 or PDELTA_F32)
 * Products of the 16-bit operands are accumulated in fp32; Y is rounded to y_dtype once
 * (nearest-even).  M = 0 is a no-op that returns PDELTA_OK (X and Y may then be NULL).  No
 * bias term (the paper leaves biases untouched, Limitations section).
 * Arithmetic and operand range, by batch size:
 *   M <= 64  the matrix cores multiply in the operands' own format (fp16 or bf16) with one
 *            accumulator for X W_b^T and one for X B^T; v_row multiplies the latter in fp32.
 *            Every finite input is in range.
 *   M > 64   one multiplication stream in fp16: the tile of W_hat = W_b +- v_row is formed as
 *            fp16(W_b + v B) with one rounding (relative error <= 2^-11 per weight, about 2e-4
 *            relative on Y for LLM-like weights), so a delta smaller than half an fp16 ulp of
 *            W_b (|v| < 2^-12 |W_b|) is partly rounded away.  bf16 X and W_b are converted to
 *            fp16 on the way, truncating toward zero: exact for magnitudes in [2^-14, 65504];
 *            smaller magnitudes lose their low bits (absolute error < 2^-24); magnitudes above
 *            65504 are OUTSIDE the contract for bf16 at M > 64 (they would become the largest
 *            fp16 value).  fp16 inputs are used as they are.
 * The results of both regimes satisfy the same tolerance against exact arithmetic
 * (max |err| <= 1e-2 RMS(Y), relative Frobenius error <= 1e-3) on inputs inside these ranges.
 */
int pdelta_linear_row(const void* X, const void* W_b, const uint32_t* B_packed,
                      const uint16_t* v_row, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                      int x_dtype, int y_dtype, void* stream);

/*
 * Delta linear layer, column mode (Eq. 1 with v in R^(d_in x 1)):
 *   Y[m,o] = sum_i X[m,i] * W_b[o,i]  +  sum_i (X[m,i] * v_col[i]) * B[o,i]
 * Arguments as pdelta_linear_row, with v_col FP16 [d_in].  Arithmetic as there, except that for
 * M <= 64 the sign part's operand is fp16(X[m,i] * v_col[i]) (one extra rounding of relative size
 * 2^-11 on the delta term; for bf16 X the product must stay below 65504 in magnitude), and for
 * M > 64 v_col[i] enters the fp16 tile of W_hat column by column.
 */
int pdelta_linear_col(const void* X, const void* W_b, const uint32_t* B_packed,
                      const uint16_t* v_col, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                      int x_dtype, int y_dtype, void* stream);

/*
 * Merge the delta into the weights (Eq. 1; the paper's deployed path adds all residual terms
 * once, Limitations section, and applies a saved delta module by module, algorithm "Model-wide
 * application from a saved delta file"):
 *   W_out[o,i] = round_to_w_dtype( W_b[o,i] + v[o or i] * B[o,i] )
 * The sum is formed exactly and rounded once (nearest-even).
 * Arguments
 *   W_b      in   [d_out, d_in], dtype w_dtype (PDELTA_F16 or PDELTA_BF16)
 *   B_packed in   [d_out, d_in/32] uint32
 *   v        in   FP16, [d_out] if axis == PDELTA_ROW, [d_in] if axis == PDELTA_COL
 *   W_out    out  [d_out, d_in], dtype w_dtype; may be the same pointer as W_b (in place),
 *                 must not overlap it otherwise
 * With W_b = 0 and v = 1 the result is exactly +-1: the unpacked B.
 */
int pdelta_patch(const void* W_b, const uint32_t* B_packed, const uint16_t* v, int axis,
                 void* W_out, int64_t d_out, int64_t d_in, int w_dtype, void* stream);

/*
 * Several delta linear layers in one launch, for layers that do not depend on each other (the
 * q/k/v or gate/up projections of one block, or many fine-tuned variants of one base served
 * together, the setting the paper's introduction motivates).  Every layer computes exactly what
 * pdelta_linear_row / pdelta_linear_col computes (Eq. 1 inside the layer forward); all layers
 * share the batch size M and the dtypes, each has its own X, W_b, B_packed, v, Y, shape and axis.
 *
 * pdelta_layer describes one layer; all pointers are device pointers as above.
 * pdelta_linear_batch_plan (host only, no HIP call) checks every descriptor of a HOST array as
 * the single-layer entry points would and fills `first_block`.  The caller then copies the array
 * to device memory and passes both copies: the host copy is read for validation and launch
 * geometry, the device copy by the kernel.  Editing pointers later needs no new plan as long
 * as shapes and axes stay the same (copy the array again).
 * When the layers do not fit the batched decode kernel (M > 16, a d_in that is not a multiple of
 * 128, or a sign slab too large for LDS) the call launches them one by one in order, with the
 * same results.  M = 0 or n_layers = 0 is a no-op.
 * Ownership and errors: layers_host is host memory, layers_device device memory holding the
 * same n_layers descriptors (16-byte aligned, PDELTA_EALIGN); both stay the caller's and must
 * stay valid until the stream has run the call.  Each layer is checked like a single-layer call
 * (same error codes); a descriptor whose first_block does not match the plan gives
 * PDELTA_EINVAL.  The Y of a layer must not overlap any buffer of another layer of the batch
 * (all layers run concurrently); this is the caller's obligation and is not checked.
 */
typedef struct pdelta_layer {
    const void* X;            /* [M, d_in] */
    const void* W_b;          /* [d_out, d_in] */
    const uint32_t* B_packed; /* [d_out, d_in/32] */
    const uint16_t* v;        /* FP16, [d_out] (row) or [d_in] (col) */
    void* Y;                  /* out [M, d_out] */
    int64_t d_out, d_in;
    int32_t axis;             /* PDELTA_ROW or PDELTA_COL */
    int32_t first_block;      /* filled by pdelta_linear_batch_plan */
} pdelta_layer;

int pdelta_linear_batch_plan(pdelta_layer* layers_host, int32_t n_layers);

int pdelta_linear_batch(const pdelta_layer* layers_host, const pdelta_layer* layers_device,
                        int32_t n_layers, int64_t M, int x_dtype, int y_dtype, void* stream);

/*
 * Merge the deltas of many layers in one launch: the paper's "Model-wide application from a
 * saved delta file" (every module of the model is patched; Eq. 1 per layer).  Each layer computes
 * exactly what pdelta_patch computes.  Descriptors are pdelta_layer records planned with
 * pdelta_linear_batch_plan: W_b, B_packed, v, d_out, d_in and axis as there, Y is W_out (same
 * dtype as W_b; may equal W_b for an in-place merge), X is ignored.  Host and device copies of
 * the array are passed as in pdelta_linear_batch; ownership and error rules are the same.  The
 * W_out of a layer must not overlap any buffer of another layer of the batch (not checked).
 */
int pdelta_patch_batch(const pdelta_layer* layers_host, const pdelta_layer* layers_device,
                       int32_t n_layers, int w_dtype, void* stream);

/*
 * pdelta_pack for many layers in two launches (all tiles, then all scale vectors): the paper's
 * compression of a whole model, module by module (per-layer compression algorithm applied to
 * every linear layer).  Each job computes exactly what pdelta_pack computes, with its own
 * workspace of at least pdelta_pack_workspace_bytes(d_out, d_in) bytes (workspaces of different
 * jobs must not overlap; outputs of a job must not overlap anything of another job: not checked).
 * pdelta_pack_batch_plan (host only) checks the shapes and fills first_tile, first_fin_block and
 * tile_blocks; the caller copies the planned array to the device and passes both copies, as in
 * pdelta_linear_batch.  n_jobs = 0 is a no-op.
 */
typedef struct pdelta_pack_job {
    const void* W_f;          /* [d_out, d_in] */
    const void* W_b;          /* [d_out, d_in] */
    uint32_t* B_packed;       /* out [d_out, d_in/32] */
    uint16_t* v_row;          /* out FP16 [d_out], may be NULL */
    uint16_t* v_col;          /* out FP16 [d_in],  may be NULL */
    void* workspace;          /* scratch of this job */
    size_t workspace_bytes;
    int64_t d_out, d_in;
    int32_t first_tile;       /* the next three are filled by pdelta_pack_batch_plan */
    int32_t first_fin_block;
    int32_t tile_blocks;
    int32_t reserved;
} pdelta_pack_job;

int pdelta_pack_batch_plan(pdelta_pack_job* jobs_host, int32_t n_jobs);

int pdelta_pack_batch(const pdelta_pack_job* jobs_host, const pdelta_pack_job* jobs_device,
                      int32_t n_jobs, int w_dtype, void* stream);

/*
 * Multi-variant decode: R requests of one token each share the base weights and each has its
 * own 1-bit delta - many fine-tuned variants of one base served together (the setting of the
 * paper's introduction).  Request r computes exactly what pdelta_linear_row / pdelta_linear_col
 * computes for M = 1 with (B_r, v_r) (Eq. 1 inside the layer forward):
 *   row:  Y[r,o] = sum_i X[r,i] W_b[o,i] + v_r[o] * sum_i X[r,i] B_r[o,i]
 *   col:  Y[r,o] = sum_i X[r,i] W_b[o,i] +          sum_i (X[r,i] v_r[i]) B_r[o,i]
 * but W_b is read once per group of up to 16 requests (2 + R/8 bytes per weight for R <= 16)
 * when d_in is a multiple of 128; otherwise the requests run one after the other with the
 * same results.
 * Arguments
 *   X         in   [R, d_in], dtype x_dtype; row r is the token of request r
 *   W_b       in   [d_out, d_in], same dtype
 *   variants  in   R records {B_packed [d_out, d_in/32], v FP16 [d_out] (row) or [d_in] (col),
 *                  axis}; a HOST copy (validated here) and a DEVICE copy (read by the kernel) of
 *                  the same array, both owned by the caller and valid until the stream has run
 *                  the call
 *   axis      PDELTA_ROW or PDELTA_COL: one mode for all requests of the call (the records' axis
 *             fields are ignored); PDELTA_PER_REQUEST: request r uses variants[r].axis - the
 *             per-layer Row/Col selection of the paper's compression algorithm may have chosen
 *             differently for different fine-tunes of the same base layer
 *   Y         out  [R, d_out], dtype y_dtype; must not overlap any input
 * When the requests of a PDELTA_PER_REQUEST call do not all share one axis, the sign part of
 * every request is evaluated in fp16: column-mode requests as in pdelta_linear_col, row-mode
 * requests with the operand fp16(X) (exact for fp16 X; for bf16 X exact for magnitudes in
 * [2^-14, 65504]).  R = 0 is a no-op.  Errors as for pdelta_linear_row, per variant; a record
 * axis other than PDELTA_ROW / PDELTA_COL gives PDELTA_EINVAL.
 */
typedef struct pdelta_variant {
    const uint32_t* B_packed;
    const uint16_t* v;
    int32_t axis;             /* PDELTA_ROW or PDELTA_COL; read when the call's axis is PDELTA_PER_REQUEST */
    int32_t reserved;         /* set to 0 */
} pdelta_variant;

int pdelta_linear_variants(const void* X, const void* W_b, const pdelta_variant* variants_host,
                           const pdelta_variant* variants_device, int32_t R, int axis, void* Y,
                           int64_t d_out, int64_t d_in, int x_dtype, int y_dtype, void* stream);

/*
 * Gradient of a loss with respect to the scale vector, given dY = dL/dY: the backward step of
 * the paper's algorithm "Train per-row/column scaling vectors via activation matching", which
 * backpropagates through v only.  From Eq. 1 inside the layer forward:
 *   row:  grad_v[o] = sum_m dY[m,o] * sum_i X[m,i] B[o,i]
 *   col:  grad_v[i] = sum_m X[m,i]  * sum_o dY[m,o] B[o,i]
 * Arguments
 *   X        in   [M, d_in],  dtype (PDELTA_F16 or PDELTA_BF16)
 *   dY       in   [M, d_out], same dtype
 *   B_packed in   [d_out, d_in/32] uint32
 *   grad_v   out  fp32, [d_out] (row) or [d_in] (col); overwritten, not accumulated
 *   workspace scratch of >= pdelta_grad_v_workspace_bytes(M, d_out, d_in, axis) bytes, 16-byte
 *             aligned (PDELTA_EWORKSPACE otherwise); contents on entry ignored
 * Products are exact, sums are accumulated in fp32 in a fixed order (reproducible).  Column mode
 * needs d_out to be a multiple of 32 (PDELTA_ESHAPE): it transposes the packed signs into the
 * workspace.  M = 0 writes zeros.
 */
size_t pdelta_grad_v_workspace_bytes(int64_t M, int64_t d_out, int64_t d_in, int axis);

int pdelta_grad_v(const void* X, const void* dY, const uint32_t* B_packed, int axis, float* grad_v,
                  int64_t M, int64_t d_out, int64_t d_in, int dtype, void* workspace,
                  size_t workspace_bytes, void* stream);

/*
 * Blockwise ("per-group") and scalar scales: Eq. 1 with v constant over blocks of the matrix
 * instead of along one whole axis.  The paper's conclusion names blockwise per-group scales as
 * its first extension, and its comparison baseline (Experiments section, the BitDelta rows of
 * the results tables) is the case of one scalar per matrix.
 *   scale(o, i) = v[ (shared_rows ? 0 : o) * (d_in / group) + i / group ]
 *   W_hat[o,i]  = W_b[o,i] + scale(o, i) * B[o,i]
 * v is FP16 [d_out or 1, d_in / group]: one scale per output row and group of `group` consecutive
 * inputs, or (shared_rows = 1) one per group for all rows.  shared_rows = 1 with group = d_in is
 * ONE scalar for the whole matrix; shared_rows = 0 with group = d_in is row mode.
 * `group` must be d_in itself, or a power of two >= 32 that divides d_in (PDELTA_ESHAPE
 * otherwise); shared_rows must be 0 or 1 (PDELTA_EINVAL).  Everything else (pointers, layouts,
 * dtypes, alignment, aliasing, error codes, arithmetic and operand ranges) is as for the
 * per-axis entry points: pdelta_linear_group as pdelta_linear_row except that for M <= 64 the
 * sign part is multiplied in fp16 with the exact operands fp16(X) and +-v (for bf16 X exact for
 * magnitudes in [2^-14, 65504]); pdelta_patch_group as pdelta_patch (exact sum, one rounding,
 * in place allowed); pdelta_pack_group as pdelta_pack with
 *   v[r, g] = mean |W_f - W_b| over the rows r covers and inputs g*group .. g*group + group - 1,
 * the exact mean rounded once to FP16 (bit-equal to the fp64 reference for FP16 inputs while a
 * block's sum of |dW| stays below 2^29).  Its workspace (pdelta_pack_group_workspace_bytes; 0
 * unless shared_rows) holds one fp64 partial sum per row and group; contents on entry ignored.
 */
size_t pdelta_pack_group_workspace_bytes(int64_t d_out, int64_t d_in, int64_t group, int shared_rows);

int pdelta_pack_group(const void* W_f, const void* W_b, int64_t d_out, int64_t d_in, int w_dtype,
                      int64_t group, int shared_rows, uint32_t* B_packed, uint16_t* v,
                      void* workspace, size_t workspace_bytes, void* stream);

int pdelta_linear_group(const void* X, const void* W_b, const uint32_t* B_packed, const uint16_t* v,
                        int64_t group, int shared_rows, void* Y, int64_t M, int64_t d_out,
                        int64_t d_in, int x_dtype, int y_dtype, void* stream);

int pdelta_patch_group(const void* W_b, const uint32_t* B_packed, const uint16_t* v, int64_t group,
                       int shared_rows, void* W_out, int64_t d_out, int64_t d_in, int w_dtype,
                       void* stream);

/* Static, human-readable name of a pdelta_status value. */
const char* pdelta_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* PDELTA_H */
