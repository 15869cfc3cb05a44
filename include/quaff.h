/*
 * quaff.h - C ABI of the MI355X (gfx950) implementation of the Quaff quantized linear layer
 * (arXiv 2505.14742, Sec. 3 "Methodology").
 *
 * One fine-tuning step of one linear layer Y = X W (X [t x c_in] tokens x input channels,
 * W [c_in x c_out], Sec. 2.2) runs as
 *
 *     quaff_scale_update   momentum scales on the fixed outlier channels O        (Eq. 7, Eq. 8)
 *                          and the dynamic outlier weights what = (s_O - 1) W_O   (Eq. 5, Eq. 9)
 *     quaff_quant_act      Xhat = X s^-1 on the O columns, per-token INT8 codes   (Eq. 5, Eq. 1)
 *     quaff_linear_fwd     Y = Dx (Xq Wq Dw + xq_O what_int Dwhat) + LoRA branch  (Eq. 9; App. "settings")
 *     quaff_linear_bwd_dx  dX = dY W^T through the same INT8 product + LoRA branch
 *
 * preceded once per layer by quaff_prepare_weight (Sec. 3.3: quantize the frozen W, keep W_O).
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller, valid on the device that is current when
 *    the call is made; the library never frees or keeps them.  The library allocates nothing and creates no
 *    streams or events (the quaff_microbench_* aids excepted): scratch comes from the caller's `workspace`
 *    (quaff_workspace_bytes tells how much).
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream) and the
 *    call returns without synchronizing.  Nothing is printed.
 *  - Matrices are row-major.  bf16 values are passed as uint16_t bit patterns.
 *  - c_in and c_out must be multiples of 16; t >= 1; n_outlier >= 0; lora_rank is 0 or a multiple of 16
 *    (at most 64).  Data pointers must be 16-byte aligned and leading dimensions multiples of 8 elements.
 *  - O must be sorted, unique and inside [0, c_in): a precondition of every per-step call, which use its entries
 *    as column indices without looking at them; quaff_check_outliers verifies a list on the device (O is fixed
 *    before fine-tuning starts, Sec. 3.3, so once per layer is enough).
 *    Non-finite inputs are outside the contract (no hang, no out-of-bounds access, values unspecified).
 *  - Return value: QUAFF_OK or a negative QUAFF_ERR_* code; nothing has been enqueued when an error is
 *    returned for an argument problem.
 *  - n_p ("padded outlier count") is n_outlier rounded up to a multiple of 64 (0 stays 0); see
 *    quaff_padded_outliers.
 *
 * Arithmetic contract.  Integer codes and int32 accumulators are exact.  Quantization decisions are taken
 * in IEEE fp32, one rounding per operation, ties to even: for a group (token row / output channel) with
 * absolute maximum m, the step is Delta = m / 127, codes are rne(x * (127 / m)) clamped to [-127, 127], and
 * a group with m = 0 gets Delta = 0 and all-zero codes.  Dequantised outputs are computed in fp32.
 */
#ifndef QUAFF_H_
#define QUAFF_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QUAFF_OK 0
#define QUAFF_ERR_NULL (-1)      /* a required pointer is NULL */
#define QUAFF_ERR_SHAPE (-2)     /* a size is out of the supported range */
#define QUAFF_ERR_WORKSPACE (-3) /* workspace missing or too small */
#define QUAFF_ERR_ALIGN (-4)     /* a pointer or leading dimension is misaligned */
#define QUAFF_ERR_HIP (-5)       /* a HIP call failed; see quaff_last_hip_error */

/* Human-readable name of a status code (static string, never NULL). */
const char* quaff_status_string(int status);

/* hipError_t value of the last failed HIP call made by this library on the calling thread (0 if none). */
int quaff_last_hip_error(void);

/* n_p: n_outlier rounded up to the INT8 MFMA contraction step (64). */
int32_t quaff_padded_outliers(int32_t n_outlier);

/* Bytes of the opaque packed INT8 weight produced by quaff_prepare_weight: one byte per weight (c_in rounded up to a
 * multiple of 64, c_out to a multiple of 2).  The one copy serves both products of the layer: element (j, k) of the
 * [c_out x c_in] code matrix sits at byte (j / 2) * 2 * cpad + (k / 64) * 128 + (j % 2) * 64 + k % 64, so that every
 * 128-byte line holds 64 consecutive input channels of two neighbouring output channels; the forward product reads
 * it contraction-contiguous, the input-gradient product transposes 8 x 8 byte blocks while reading them from LDS. */
size_t quaff_packed_weight_bytes(int64_t c_in, int64_t c_out);

/* Byte offset inside the packed weight of the code of W[k, j] (input channel k, output channel j), for tools that want
 * to read single codes back; -1 for indices outside [0, c_in) x [0, c_out). */
int64_t quaff_packed_weight_offset(int64_t c_in, int64_t c_out, int64_t k, int64_t j);

/* Bytes of scratch that the per-step calls below need for the given problem (the maximum over the calls). */
size_t quaff_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t n_outlier, int32_t lora_rank);

/*
 * Offline weight preprocessing (Sec. 3.3, "weights preprocessing"): per-output-channel Eq. 1 on the frozen
 * full-precision W, retaining the outlier rows W_O in full precision.
 *   in : W [c_in x c_out] fp32, leading dimension ldw;  O [n_outlier] int32 (may be NULL when n_outlier = 0)
 *   out: Wq_packed  opaque, quaff_packed_weight_bytes(c_in, c_out) bytes
 *        delta_w    [c_out] fp32 step sizes
 *        W_O        [n_outlier x c_out] fp32 copy of the O rows of W       (may be NULL when n_outlier = 0)
 *        wmax_O     [n_outlier] fp32, max_j |W_O[k, j]| (the max|W_i| of Eq. 8) (may be NULL when n_outlier = 0)
 *        Wq_plain   optional [c_in x c_out] int8 codes in the paper's layout (NULL to skip)
 * `workspace` holds partial column maxima; it must be at least quaff_prepare_workspace_bytes(c_in, c_out) bytes.
 */
size_t quaff_prepare_workspace_bytes(int64_t c_in, int64_t c_out);
int quaff_prepare_weight(const float* W, int64_t c_in, int64_t c_out, int64_t ldw, const int32_t* O,
                         int32_t n_outlier, void* Wq_packed, float* delta_w, float* W_O, float* wmax_O,
                         int8_t* Wq_plain, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Validity of an outlier channel set (Sec. 3.3: O is identified once on calibration data and stays fixed during
 * fine-tuning; Eq. 5 indexes the columns of X and the rows of W with it).  Scans O on the device.
 *   in : O [n_outlier] int32 (may be NULL when n_outlier = 0), c_in
 *   out: result, one DEVICE int32: 0 when O is strictly ascending (hence unique) with every entry in [0, c_in);
 *        otherwise 1 + k for the first position k whose entry is out of range or not above its predecessor.
 * An empty list is valid.  The call only enqueues the scan; read *result after synchronizing with `stream`.
 */
int quaff_check_outliers(const int32_t* O, int32_t n_outlier, int64_t c_in, int32_t* result, void* stream);

/*
 * Targeted momentum scaling (Eq. 7, Eq. 8) and the dynamic outlier weights (Eq. 5, quantized as in Eq. 9).
 *   cmax_k = max_i |X[i, O_k]| over all t tokens of the unscaled X
 *   beta_k = max(1, sqrt(cmax_k / wmax_k))   (1 when wmax_k = 0)
 *   s_k    = gamma * s_k + (1 - gamma) * beta_k
 *   what[k, j] = (s_k - 1) * W_O[k, j], quantized per output channel j -> what_int, delta_what
 *   in    : X [t x c_in] bf16 (ldx); O, W_O, wmax_O as produced by quaff_prepare_weight; gamma in [0, 1]
 *   in/out: s_O [n_outlier] fp32 - the only state carried from step to step
 *   out   : colscale [c_in] fp32: entries O_k are overwritten with 1 / s_k; all other entries are left
 *           untouched (the caller initialises the array to 1.0f once)
 *           what_int [c_out x n_p] int8, row j holds the codes of output channel j for k = 0..n_outlier-1,
 *           zero for k >= n_outlier;  delta_what [c_out] fp32
 *           cmax_out [n_outlier] fp32, optional (NULL to skip)
 * With n_outlier = 0 the call is a no-op that returns QUAFF_OK.
 */
int quaff_scale_update(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O,
                       int32_t n_outlier, const float* W_O, const float* wmax_O, int64_t c_out, float gamma,
                       float* s_O, float* colscale, int8_t* what_int, float* delta_what, float* cmax_out,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * quaff_scale_update for callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same results bit for
 * bit, with the scratch of that call (partial column maxima and a copy of the previous scales) in an array of
 * static device memory inside the library instead of `workspace`: 129 x 1024 floats (516 KiB) per device, held until
 * the process ends.  n_outlier may be at most quaff_scale_update_static_max_outliers() = 1024 (QUAFF_ERR_SHAPE
 * beyond).  The call allocates nothing; the array's device address is looked up once per device, at the first call
 * on that device.  All calls on one device share the array: calls that overlap on one device (different streams,
 * or different host threads) race on it; calls ordered on one stream do not.  Nothing needs clearing between calls:
 * every entry that a call reads it has written before.
 */
int32_t quaff_scale_update_static_max_outliers(void);
int quaff_scale_update_static(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O,
                              int32_t n_outlier, const float* W_O, const float* wmax_O, int64_t c_out, float gamma,
                              float* s_O, float* colscale, int8_t* what_int, float* delta_what, float* cmax_out,
                              void* stream);

/*
 * Column scaling and per-token quantization (Eq. 5 then Eq. 1 with one step size per token,
 * App. "Quantization Granularity").
 *   xhat[i, j] = X[i, j] * colscale[j]           (colscale NULL = all ones)
 *   delta[i]   = max_j |xhat[i, j]| / 127,  Xq[i, j] = rne(xhat[i, j] * (127 / max_j |xhat[i, j]|))
 *   xq_O[i, k] = Xq[i, O_k]  (the shared activation codes of Eq. 9's remark), zero for k >= n_outlier
 *   in : X [t x c] bf16 (ldx);  colscale [c] fp32 or NULL;  O [n_outlier] or NULL
 *   out: Xq [t x c] int8 (dense, leading dimension c);  delta [t] fp32;
 *        xq_O [t x n_p] int8 (NULL to skip; required layout for quaff_linear_fwd)
 * Used for X in the forward pass and, with colscale = delta_w, for dY in the backward pass.
 */
int quaff_quant_act(const uint16_t* X, int64_t t, int64_t c, int64_t ldx, const float* colscale,
                    const int32_t* O, int32_t n_outlier, int8_t* Xq, float* delta, int8_t* xq_O, void* stream);

/*
 * Integer forward with dequantising epilogue (Eq. 9) and the LoRA branch (rank r, App. "Model and
 * experimental settings"; no dropout):
 *   acc1 = Xq Wq,  acc2 = xq_O what_int                                   (int32, exact)
 *   Y[i, j] = delta_x[i] * (acc1[i, j] * delta_w[j] + acc2[i, j] * delta_what[j])
 *           + lora_scale * sum_p (sum_k X[i, k] A[k, p]) B[p, j]
 *   in : Xq [t x c_in], delta_x [t], xq_O [t x n_p] from quaff_quant_act; Wq_packed, delta_w from
 *        quaff_prepare_weight; what_int [c_out x n_p], delta_what [c_out] from quaff_scale_update
 *        (xq_O, what_int, delta_what may be NULL when n_outlier = 0);
 *        X [t x c_in] bf16 (ldx), lora_A [c_in x r] bf16, lora_B [r x c_out] bf16: read only when
 *        lora_rank > 0 (may be NULL otherwise)
 *   out: Y [t x c_out] fp32, leading dimension ldy (c_out <= ldy < 2^27, QUAFF_ERR_SHAPE otherwise)
 */
int quaff_linear_fwd(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const void* Wq_packed,
                     const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                     const float* delta_what, int32_t n_outlier, const uint16_t* X, int64_t ldx,
                     const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* Y,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/*
 * One call for the whole forward step of a layer: quaff_scale_update, quaff_quant_act and quaff_linear_fwd with the
 * same arguments, the same results bit for bit and the same side effects (s_O, colscale, what_int, delta_what,
 * cmax_out, Xq, delta_x, xq_O are all written as by the three calls).  Knowing the whole step lets the library
 * run it in fewer launches and fewer passes over X: up to 2048 tokens (at most 64 outlier channels, rank 0 or 16)
 * everything before the product is ONE launch that reads X once; other usual cases take two combined launches;
 * cases that gain nothing run the three calls one after the other.
 * The one-launch form contains the only grid-wide dependency of the path (the column maxima of Eq. 8 range over all
 * tokens): its workgroups announce themselves through a word of `workspace` and wait for each other.  That wait is
 * bounded (see quaff_debug_grid_wait_ticks); a workgroup that gives up recomputes the maxima from X itself, so the
 * results are the same whether or not all workgroups are resident at once.  `workspace` is read and written while
 * the call runs and must not be shared with work that may run at the same time (as for every call here); what an
 * earlier call left in it does not matter.
 * `workspace` must hold quaff_fwd_step_workspace_bytes(t, c_in, c_out, n_outlier, lora_rank) bytes.
 */
size_t quaff_fwd_step_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t n_outlier, int32_t lora_rank);
int quaff_linear_fwd_step(const uint16_t* X, int64_t t, int64_t c_in, int64_t ldx, const int32_t* O, int32_t n_outlier,
                          const float* W_O, const float* wmax_O, int64_t c_out, float gamma, float* s_O,
                          float* colscale, int8_t* what_int, float* delta_what, float* cmax_out, int8_t* Xq,
                          float* delta_x, int8_t* xq_O, const void* Wq_packed, const float* delta_w,
                          const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* Y,
                          int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* Test aid (not part of the method): bound of the grid-wide wait inside quaff_linear_fwd_step's one-launch form, in
 * ticks of the device's 100 MHz wall clock (default 5000 = 50 us; process-wide).  ticks >= 0 sets the bound and
 * returns the previous one, ticks < 0 only returns it.  0 makes every workgroup that is not the last to arrive give
 * up at once, which exercises the recomputing path with kernels that still finish normally. */
long long quaff_debug_grid_wait_ticks(long long ticks);

/* quaff_linear_fwd with the result rounded (to nearest even) to bf16 instead of stored as fp32: the output write,
 * which a launch cannot overlap with anything at a few thousand tokens, is halved.  Everything up to the final
 * rounding is the same arithmetic.  Restrictions: c_in a multiple of 64, n_outlier <= 128 (QUAFF_ERR_SHAPE
 * otherwise); Y 16-byte aligned, ldy a multiple of 8 (QUAFF_ERR_ALIGN otherwise). */
int quaff_linear_fwd_bf16(const int8_t* Xq, const float* delta_x, const int8_t* xq_O, int64_t t, const void* Wq_packed,
                          const float* delta_w, int64_t c_in, int64_t c_out, const int8_t* what_int,
                          const float* delta_what, int32_t n_outlier, const uint16_t* X, int64_t ldx,
                          const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale,
                          uint16_t* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* Same product as quaff_linear_fwd, but the exact int32 accumulators of Eq. 9 are written instead of Y
 * (acc1, acc2: [t x c_out] int32, dense; acc2 may be NULL).  For checking the integer path bit for bit. */
int quaff_linear_fwd_acc(const int8_t* Xq, const int8_t* xq_O, int64_t t, const void* Wq_packed, int64_t c_in,
                         int64_t c_out, const int8_t* what_int, int32_t n_outlier, int32_t* acc1, int32_t* acc2,
                         void* stream);

/*
 * Backward input gradient.  The paper does not describe the backward pass; since Xhat = X s^-1 and
 * What = s W, s cancels in the true gradient dX = dY W^T (Eq. 3), so no outlier data is needed.  delta_w lies
 * on the contraction axis and is folded into dY before per-token quantization (the reason App.
 * "Quantization Granularity" gives for rejecting per-input-channel steps):
 *   G = dY * delta_w (per column), Gq, delta_g = per-token Eq. 1 of G
 *   acc[i, k] = sum_j Gq[i, j] Wq[k, j]                                        (int32, exact)
 *   dX[i, k] = delta_g[i] * acc[i, k] + lora_scale * sum_p (sum_j dY[i, j] B[p, j]) A[k, p]
 *   in : dY [t x c_out] bf16 (lddy); Wq_packed, delta_w; lora_A [c_in x r], lora_B [r x c_out] bf16
 *   out: dX [t x c_in] fp32, leading dimension lddx (c_in <= lddx < 2^27, QUAFF_ERR_SHAPE otherwise)
 */
int quaff_linear_bwd_dx(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                        int64_t c_in, int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B,
                        int32_t lora_rank, float lora_scale, float* dX, int64_t lddx, void* workspace,
                        size_t workspace_bytes, void* stream);

/* quaff_linear_bwd_dx with dX rounded (to nearest even) to bf16.  Restrictions: c_out a multiple of 64; dX 16-byte
 * aligned, lddx a multiple of 8. */
int quaff_linear_bwd_dx_bf16(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                             int64_t c_in, int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B,
                             int32_t lora_rank, float lora_scale, uint16_t* dX, int64_t lddx, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Integer part of quaff_linear_bwd_dx with its intermediates exposed, for bit-exact checks:
 * Gq [t x c_out] int8, delta_g [t] fp32, acc [t x c_in] int32 (all dense, all required). */
int quaff_linear_bwd_dx_acc(const uint16_t* dY, int64_t t, int64_t lddy, const void* Wq_packed, const float* delta_w,
                            int64_t c_in, int64_t c_out, int8_t* Gq, float* delta_g, int32_t* acc, void* stream);

/*
 * LoRA weight gradients of the adapter branch lora_scale (X A) B (App. "Model and experimental settings": LoRA on
 * every linear layer; the frozen quantized weight gets no gradient, Sec. 2.1).  The paper does not describe its
 * backward pass; the adapter's gradients are taken on the unquantized bf16 X and dY, like its forward, no dropout:
 *   dA[k, p] = lora_scale * sum_i X[i, k] * (sum_j dY[i, j] B[p, j])
 *   dB[p, j] = lora_scale * sum_i (sum_k X[i, k] A[k, p]) * dY[i, j]
 *   in : X [t x c_in] bf16 (ldx), dY [t x c_out] bf16 (lddy), lora_A [c_in x r] bf16, lora_B [r x c_out] bf16,
 *        lora_rank a multiple of 16 in [16, 64]
 *   out: dA [c_in x r] fp32, dB [r x c_out] fp32 (dense; overwritten, not accumulated)
 * `workspace` must hold quaff_lora_bwd_workspace_bytes(t, c_in, c_out, lora_rank) bytes.  fp32 accumulation over
 * the tokens in a fixed order: results are reproducible from run to run.
 */
size_t quaff_lora_bwd_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t lora_rank);
int quaff_lora_bwd_weights(const uint16_t* X, int64_t ldx, const uint16_t* dY, int64_t lddy, int64_t t, int64_t c_in,
                           int64_t c_out, const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank,
                           float lora_scale, float* dA, float* dB, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * One call for the backward step of a layer: quaff_linear_bwd_dx followed by quaff_lora_bwd_weights, with the
 * down-projection dY B^T computed once for both (same arguments, same results up to the rounding of the fp32 sums of
 * that down-projection, whose order may differ between the launches).  Needs lora_rank > 0.
 * `workspace` must hold quaff_bwd_step_workspace_bytes(t, c_in, c_out, lora_rank) bytes.
 * The weight gradients do not depend on the input-gradient product.  When the caller passes a second stream
 * (`side_stream`, default priority, on the same device) and two events created with timing disabled (`fork_event`,
 * `join_event`; hipStream_t / hipEvent_t passed as void*), they are enqueued on that stream beside the product: forked
 * from `stream` after the shared down-projection and joined back into `stream` before the call returns, so that
 * towards the caller everything is ordered on `stream` as usual, also when a later launch of the call fails.  The
 * stream and the events belong to the caller (one set per concurrent caller; the library creates and keeps none)
 * and may be reused by the next call on the same `stream`.  With any of the three NULL everything runs on `stream`.
 */
size_t quaff_bwd_step_workspace_bytes(int64_t t, int64_t c_in, int64_t c_out, int32_t lora_rank);
int quaff_linear_bwd_step(const uint16_t* dY, int64_t t, int64_t lddy, const uint16_t* X, int64_t ldx,
                          const void* Wq_packed, const float* delta_w, int64_t c_in, int64_t c_out,
                          const uint16_t* lora_A, const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* dX,
                          int64_t lddx, float* dA, float* dB, void* workspace, size_t workspace_bytes, void* stream,
                          void* side_stream, void* fork_event, void* join_event);

/*
 * Variant of the input gradient on the outlier channels (to be called after quaff_linear_bwd_dx on the same dY and
 * dX).  The paper retains the outlier rows W_O of the frozen weight in full precision (Sec. 3.3) and s cancels in
 * the true gradient (Eq. 3); this call overwrites the O columns of dX, where the quantization error of the
 * activations concentrates, with the product on those retained rows:
 *   dX[i, O_k] = sum_j dY[i, j] W_O[k, j] + lora_scale * sum_p (sum_j dY[i, j] B[p, j]) A[O_k, p]
 * (bf16 MFMA on a 16-bit hi/lo split of the fp32 rows, fp32 accumulation).  All other columns are left untouched.
 *   in    : dY [t x c_out] bf16 (lddy); O, W_O as for quaff_scale_update; lora_A, lora_B as for quaff_linear_bwd_dx
 *   in/out: dX [t x c_in] fp32 (lddx)
 * `workspace` must hold quaff_bwd_dx_outlier_workspace_bytes(t, c_out) bytes.  n_outlier = 0 is a no-op.
 */
size_t quaff_bwd_dx_outlier_workspace_bytes(int64_t t, int64_t c_out);
int quaff_bwd_dx_outlier_exact(const uint16_t* dY, int64_t t, int64_t lddy, int64_t c_in, int64_t c_out,
                               const int32_t* O, int32_t n_outlier, const float* W_O, const uint16_t* lora_A,
                               const uint16_t* lora_B, int32_t lora_rank, float lora_scale, float* dX, int64_t lddx,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Outlier-channel identification on calibration data (Eq. 6, Sec. 3.3) and selection of O within a budget:
 *   xi[o] = number of samples i with  max_rows |X^i[:, o]| > ratio * mean(|X^i|)      (the paper uses ratio = 100)
 *   O     = the `budget` channels with the largest xi (ties to the lower channel index; channels with xi = 0 are
 *           never selected), in ascending channel order - the form every other call here expects
 *   in : X [t_total x c_in] bf16 (ldx): the calibration samples one after the other; sample_offsets
 *        [n_samples + 1] int64 DEVICE array, sample i = rows sample_offsets[i] .. sample_offsets[i + 1] - 1
 *        (values outside [0, t_total] are clamped; an empty sample flags nothing); 1 <= n_samples <= 65535
 *   out: xi [c_in] int32;  O [budget] int32 (the first *n_outlier entries are written), n_outlier device scalar
 *        (O and n_outlier may be NULL when budget = 0: only xi is computed)
 * The mean is over all elements of a sample; the comparison is strict and is made in fp64.
 * `workspace` must hold quaff_calibrate_workspace_bytes(c_in, n_samples) bytes.
 */
size_t quaff_calibrate_workspace_bytes(int64_t c_in, int32_t n_samples);
int quaff_calibrate_outliers(const uint16_t* X, int64_t t_total, int64_t c_in, int64_t ldx,
                             const int64_t* sample_offsets, int32_t n_samples, double ratio, int32_t budget,
                             int32_t* xi, int32_t* O, int32_t* n_outlier, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * Optional per-launch kernel timing for benchmarks (not part of the method).  While enabled, every kernel the
 * library launches is bracketed by a pair of HIP events on the caller's stream; this perturbs end-to-end time, so
 * whole-step timing is taken with profiling off.  State is process-wide and guarded by a mutex.
 *   quaff_profile_enable(on)    drop all records, then start (on != 0) or stop recording; returns QUAFF_OK
 *   quaff_profile_collect()     wait for the recorded events; returns the number of recorded launches, -1 on error
 *   quaff_profile_launch(i,..)  kind and duration (ms) of the i-th recorded launch, in launch order
 *   quaff_profile_kind_name(k)  static name of a kernel kind
 */
int quaff_profile_enable(int on);
int64_t quaff_profile_collect(void);
int quaff_profile_launch(int64_t index, int* kind, float* ms);
const char* quaff_profile_kind_name(int kind);

/*
 * Device micro-benchmarks for honest roofline denominators (not part of the method).  Unlike everything above
 * these calls allocate device memory, run on the default stream and synchronize.
 *   quaff_microbench_mfma_i8  sustained rate (TOP/s) and shader clock (MHz) of a register-only
 *                             v_mfma_i32_32x32x32_i8 loop, two wavefronts per SIMD on every compute unit, with
 *                             constant operands (random_operands = 0) or full-range random INT8 operands (1): the
 *                             clock the chip sustains, and so the attainable MFMA rate, depends on operand toggling
 *   quaff_microbench_copy     bandwidth (GB/s, bytes read + bytes written) of a streaming copy of `bytes` bytes
 */
int quaff_microbench_mfma_i8(int random_operands, double* tops, double* clock_mhz);
int quaff_microbench_copy(size_t bytes, double* gbs_read_plus_write);

#ifdef __cplusplus
}
#endif
#endif /* QUAFF_H_ */
