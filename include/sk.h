/*
 * libsk -- forward and backward pass of the sketched linear layer (SKLinear)
 * on AMD MI355X (gfx950).  Plain C ABI: device pointers, sizes, a stream.
 *
 * The layer (paper Sec. 3.1, "During Development use-case"): the output is the
 * average over num_terms (= l) sketched matrix products, each of rank low_rank
 * (= k), and the layer is a drop-in for a dense linear layer (hence a bias):
 *
 *     y = (1/l) * sum_i (x . S_i) . U_i + b
 *
 * S_i (in x k) are fixed random sketches, U_i (k x out) learned factors.  The
 * library takes the l terms concatenated:
 *
 *     S_cat [in, R]   column i*k + j  = column j of S_i         (R = l*k)
 *     U_cat [R, out]  rows   i*k .. i*k+k-1 = U_i
 *
 * so that  y = (1/l) * (x . S_cat) . U_cat + b.
 *
 * Common rules for the three compute entry points
 *   - Every pointer is a DEVICE pointer, 16-byte aligned, to a dense row-major
 *     array with no padding (leading dimension = last dimension).
 *   - `dtype` is the storage type of x, S_cat, U_cat, bias, y, dY and dX
 *     (SK_F32, or SK_BF16 with fp32 accumulation).  dU_cat and dbias are
 *     always fp32.
 *   - tokens >= 1 (any value); in, out and R = l*k must be positive multiples
 *     of 16, l >= 1, k >= 1.
 *   - The caller owns every buffer, the workspace included.  The library
 *     allocates nothing, keeps no state between calls, and never synchronises:
 *     all work is enqueued on `stream` (a hipStream_t; NULL = default stream).
 *     Outputs are overwritten, not accumulated into.  Inputs and outputs must
 *     not overlap.  `workspace` must hold at least
 *     sk_linear_workspace_bytes(op, ...) bytes (it may be NULL when that is 0)
 *     and its contents are undefined after the call.
 *   - The intermediate x . S_cat is never kept between calls: the backward
 *     pass for the factors recomputes it.
 *   - Return value: SK_OK, or an error code; nothing is thrown across the ABI.
 *     Arguments are validated before any HIP call is made, so a bad call
 *     returns SK_ERR_INVALID_ARG / SK_ERR_UNSUPPORTED / SK_ERR_WORKSPACE with
 *     no GPU work enqueued (and also on a machine with no GPU).
 */
#ifndef SK_H
#define SK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SK_OK = 0,
  SK_ERR_INVALID_ARG = 1, /* null required pointer, misaligned pointer, non-positive size */
  SK_ERR_UNSUPPORTED = 2, /* unknown dtype/op, or in/out/R not a multiple of 16 */
  SK_ERR_WORKSPACE = 3,   /* workspace missing or smaller than required */
  SK_ERR_HIP = 4          /* a HIP call failed; see sk_last_hip_error() */
} sk_status;

typedef enum { SK_F32 = 0, SK_BF16 = 1 } sk_dtype;

typedef enum {
  SK_OP_FWD = 0,
  SK_OP_BWD_INPUT = 1,
  SK_OP_BWD_WEIGHT = 2,
  SK_OP_BWD_WEIGHT_FIRST = 3, /* sized so that it serves any column range */
  SK_OP_BWD = 4               /* sk_linear_bwd: both gradients in one call */
} sk_op;

/*
 * Forward (Sec. 3.1):  y = (1/l) * (x . S_cat) . U_cat + bias.
 *   x [tokens, in], S_cat [in, R], U_cat [R, out], bias [out] or NULL (no bias),
 *   y [tokens, out] (output, storage type `dtype`).
 * In bf16 the R-wide intermediate is rounded to bf16 once, between the two
 * contractions; scaling and bias are applied in fp32 before y is rounded.
 */
sk_status sk_linear_fwd(const void* x, const void* S_cat, const void* U_cat, const void* bias,
                        void* y, int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                        sk_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Gradient with respect to the input (the exact derivative of the forward of
 * Sec. 3.1; the paper prints no formula):
 *     dX = (1/l) * (dY . U_cat^T) . S_cat^T
 *   dY [tokens, out], S_cat [in, R], U_cat [R, out], dX [tokens, in] (output).
 */
sk_status sk_linear_bwd_input(const void* dY, const void* S_cat, const void* U_cat, void* dX,
                              int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                              sk_dtype dtype, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Gradient with respect to the learned factors and the bias (exact derivative
 * of the forward of Sec. 3.1):
 *     dU_cat = (1/l) * (x . S_cat)^T . dY          (rows i*k.. are dU_i)
 *     dbias  = sum over tokens of dY
 *   x [tokens, in], S_cat [in, R], dY [tokens, out],
 *   dU_cat [R, out] fp32 (output), dbias [out] fp32 (output) or NULL (skipped).
 * x . S_cat is recomputed here (into the workspace), not read from a saved
 * copy.  The reduction over tokens uses a fixed order: results are
 * bit-reproducible from run to run for the same shapes.
 */
sk_status sk_linear_bwd_weight(const void* x, const void* S_cat, const void* dY, float* dU_cat,
                               float* dbias, int64_t tokens, int64_t in, int64_t out, int32_t l,
                               int32_t k, sk_dtype dtype, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * sk_linear_bwd_weight for callers that cannot allocate or supply a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs,
 * outputs, kernels and results (bit for bit) as sk_linear_bwd_weight, with the workspace
 * (the recomputed x . S_cat, the token-split slabs, the column-sum partials) in a fixed
 * array of SK_NOALLOC_SCRATCH_BYTES = 32 MiB of device memory that is part of the loaded
 * library: every GPU the library runs on holds one copy until the process ends.  The call
 * makes no hipMalloc / hipFree and no allocating library call; it looks the array's address
 * up once per device (hipGetSymbolAddress) on the first call there.
 *   - Shapes whose sk_linear_workspace_bytes(SK_OP_BWD_WEIGHT, ...) exceeds that size return
 *     SK_ERR_WORKSPACE with nothing enqueued (BERT-base and BERT-large layer sizes fit; a
 *     2048-wide sketch over 16384 tokens does not).
 *   - All calls on one GPU share the array: two calls that can overlap there (different
 *     streams, or two threads) race on it; serialise them.  Its contents after a call are
 *     undefined; nothing has to be cleared between calls.
 *   - The GPU used is the calling thread's current device, which must be the one `stream`
 *     and the pointers belong to.
 */
#define SK_NOALLOC_SCRATCH_BYTES (32u << 20)
sk_status sk_linear_bwd_weight_noalloc(const void* x, const void* S_cat, const void* dY,
                                       float* dU_cat, float* dbias, int64_t tokens, int64_t in,
                                       int64_t out, int32_t l, int32_t k, sk_dtype dtype,
                                       void* stream);

/*
 * Both gradients in one call: what sk_linear_bwd_input followed by sk_linear_bwd_weight
 * compute (same formulas, same outputs, same rounding points; the order of the fp32
 * partial sums inside dX may differ from the separate call's; dU_cat and dbias are
 * bit-identical to it except on the one-pass schedule below), scheduled together.
 *   - Narrow sketches (bf16, R <= 128): kernels of the two gradients that do not depend
 *     on each other share launches -- dY . U_cat^T runs beside the recomputation of
 *     x . S_cat, and the sum of the factor gradient's token splits rides on the kernel
 *     that expands dX -- three launches instead of five, which is most of the cost at
 *     BERT-base sizes.
 *   - Very narrow sketches (bf16, R <= 32, in <= 848, out <= 896) over up to 16384
 *     tokens: one kernel reads x and dY once, recomputes x . S_cat, and produces dX and
 *     a partial dU_cat and dbias per token tile, which a second kernel sums in tile
 *     order -- two launches, dY read once.  dU_cat and dbias then differ from the
 *     separate call's in the order of their fp32 partial sums (they remain
 *     bit-reproducible from run to run).
 *   - Other shapes run the two gradients one after the other.
 *   x [tokens, in], dY [tokens, out], S_cat [in, R], U_cat [R, out],
 *   dX [tokens, in] (output), dU_cat [R, out] fp32 (output), dbias [out] fp32 (output) or NULL.
 * Workspace: sk_linear_workspace_bytes(SK_OP_BWD, ...) (at least the two gradients'
 * workspaces side by side, since they are in use at the same time).
 */
sk_status sk_linear_bwd(const void* x, const void* dY, const void* S_cat, const void* U_cat,
                        void* dX, float* dU_cat, float* dbias, int64_t tokens, int64_t in,
                        int64_t out, int32_t l, int32_t k, sk_dtype dtype, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * Gradient of learned columns of the FIRST stage matrix (two-sided layers).
 *
 * The paper's size rule (Sec. 4.1) counts a sketched layer as 2 l k (in + out)
 * numbers, which fits a layer of 2 l terms: l that sketch the input side,
 * (x . S1_i) . U1_i, and l that sketch the output side, (x . U2_i) . S2_i^T with
 * U2_i (in x k) learned and S2_i (out x k) fixed, averaged over all 2 l.  That layer
 * is the same two-stage chain with 2 l terms,
 *     S_cat = [S1 | U2]  [in, 2lk],     U_cat = [U1 ; S2^T]  [2lk, out],
 * so sk_linear_fwd, sk_linear_bwd_input and sk_linear_bwd_weight serve it unchanged
 * with 2 l passed as `l` (the rows of dU_cat that belong to S2^T are gradients of
 * fixed numbers and are simply not used).  What the chain lacks is the gradient of
 * the learned first-stage columns, which this call computes for a column range:
 *     dA = (1/l) * x^T . (dY . U_cat[col_begin .. col_begin+col_count, :]^T)
 *   x [tokens, in], U_cat [R, out], dY [tokens, out],
 *   dA [in, col_count] fp32, dense (output): column j is the gradient of column
 *   col_begin + j of S_cat.  col_begin and col_count are multiples of 16,
 *   col_count >= 16, col_begin + col_count <= R (else SK_ERR_INVALID_ARG).
 * For the two-sided layer: l = 2 * (terms per side), col_begin = col_count = R / 2.
 * Fixed-order reduction over tokens (bit-reproducible), as in sk_linear_bwd_weight.
 */
sk_status sk_linear_bwd_weight_first(const void* x, const void* U_cat, const void* dY, float* dA,
                                     int64_t tokens, int64_t in, int64_t out, int32_t l, int32_t k,
                                     int64_t col_begin, int64_t col_count, sk_dtype dtype,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bytes of workspace that `op` needs for these sizes (0 when it needs none).
 * Returns (size_t)-1 for arguments the compute call would reject.
 */
size_t sk_linear_workspace_bytes(sk_op op, int64_t tokens, int64_t in, int64_t out, int32_t l,
                                 int32_t k, sk_dtype dtype);

/* Static, human-readable name of a status code. */
const char* sk_status_string(sk_status status);

/* Text of the HIP error behind the calling thread's last SK_ERR_HIP ("" if none). */
const char* sk_last_hip_error(void);

/*
 * Tuning/testing knob, process-wide (not part of the layer's definition):
 * which kernel plan the three entry points pick.
 *   0 = automatic (default): per-shape choice;
 *   1 = fused: one kernel per call, the R-wide intermediate of a token tile never
 *       leaves the chip (bf16 with R <= 256; wider R falls back to plan 3, then 2);
 *   2 = two general GEMMs with the intermediate in the workspace (any dtype);
 *   3 = split-K first contraction into fp32 slabs in the workspace, then a second
 *       kernel that sums the slabs into LDS and keeps the tile on chip (bf16, R <= 512;
 *       otherwise plan 2).
 * Only sk_linear_fwd and sk_linear_bwd_input have several plans.
 * sk_linear_workspace_bytes reports the maximum over the plans, so a workspace
 * sized by it serves whatever is selected.  Returns the previous value, or -1
 * (and changes nothing) for a value out of range.
 */
int sk_set_plan(int plan);

#ifdef __cplusplus
}
#endif
#endif /* SK_H */
