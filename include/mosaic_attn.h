/*
 * mosaic_attn.h -- C ABI of the MI355X (gfx950) unpad -> ALiBi varlen attention -> pad library.
 *
 * The calls follow the encoder layer of the MosaicBERT paper (arXiv 2312.17482), section
 * "MosaicBERT Architecture Modifications for Fast Pretraining":
 *   - "Unpadding" paragraph: the real tokens of a padded [B, L] batch are concatenated, in order,
 *     into one packed sequence of T tokens (mb_unpad_index, mb_unpad), and scattered back (mb_pad);
 *   - "FlashAttention" + "Attention with Linear Biases" paragraphs, Eq. 1: exact softmax attention,
 *     computed tile-wise without materialising the score matrix, with the bias  -m_h * |i - j|
 *     added to the scores, bidirectional (mb_alibi_attn_fwd / mb_alibi_attn_bwd), m_h geometric with
 *     ratio 2^(-8/H) (mb_alibi_slopes);
 *   - the two neighbouring sublayers of the same block, on the packed token rows: "Low Precision
 *     LayerNorm" paragraph with the residual add of Figure 1A (mb_add_layernorm_fwd / _bwd), and the
 *     "Gated Linear Units" paragraph, Eq. 2, with the arrangements of the appendix on GLU
 *     implementations (mb_geglu_fwd / mb_geglu_bwd, mb_linear_fwd, mb_gelu_gate).
 *
 * Conventions common to every call
 *   Pointers   "dev" = device (HBM) pointer, "host" = host pointer.  The caller allocates and owns
 *              every buffer; the library allocates nothing and never frees.  Device pointers must be
 *              16-byte aligned.  The only state kept between calls lives on the device: one sticky
 *              misuse word (see mb_device_status) and the fixed scratch array of mb_alibi_attn_bwd_static.
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device
 *              work is enqueued on it; no call synchronises with the host except mb_read_meta and
 *              mb_device_status.  Calls
 *              enqueue kernels only (no memsets, no allocations), so a sequence of them can be captured in
 *              a HIP graph.
 *   Errors     every call returns an mb_status and never throws or aborts.  Arguments are validated
 *              on the host before anything is launched, so error paths need no GPU.  A message for
 *              the last failing call on this thread is available from mb_last_error().
 *   Layouts    packed activations are [T, H, D] with D contiguous; consecutive tokens are
 *              `row_stride` ELEMENTS apart (H*D <= row_stride < 2^24, a multiple of 16 bytes), so q, k and v may
 *              point into one fused [T, 3, H, D] buffer.  The row log-sum-exp is [H, T] float,
 *              natural log.  Positions used by the bias are positions inside the packed sequence:
 *              token t of sequence b sits at position t - cu_seqlens[b].
 *   Precision  MB_BF16 with D = 64: bf16 operands on the matrix cores, fp32 accumulation and fp32
 *              softmax statistics; probabilities and score gradients are rounded to bf16 only as
 *              matrix operands; outputs are rounded to bf16 once.  MB_F32 (D <= 128, multiple of 4)
 *              and MB_BF16 with other D (<= 128, multiple of 8): plain fp32 arithmetic throughout.
 *   Degenerate B == 0, T == 0 and zero-length sequences are legal: MB_OK, nothing written for them.
 *   Threads    re-entrant; the only global state is the thread-local error string.
 */
#ifndef MOSAIC_ATTN_H
#define MOSAIC_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported from the shared library (everything else in it has hidden visibility). */
#define MB_API __attribute__((visibility("default")))

typedef enum {
  MB_OK = 0,
  MB_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, misaligned pointer, bad stride */
  MB_ERR_UNSUPPORTED = 2, /* dtype / head_dim / size combination with no kernel */
  MB_ERR_WORKSPACE = 3,   /* workspace NULL or smaller than mb_alibi_attn_bwd_workspace_bytes */
  MB_ERR_HIP = 4          /* the HIP runtime reported an error at launch */
} mb_status;

typedef enum { MB_F32 = 0, MB_BF16 = 1 } mb_dtype;

/* Message describing the last error returned on the calling thread ("" if none). */
MB_API const char* mb_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
MB_API int mb_version(void);

/*
 * Head slopes of the ALiBi bias ("Attention with Linear Biases" paragraph: geometric sequence with
 * ratio 2^(-8/H)); the first term is the ratio itself, so slopes_host[h-1] = 2^(-8h/H), h = 1..H,
 * for any H (no power-of-two special case).  Evaluated in double, rounded to float.
 *   slopes_host  host, [H] floats, written.
 * Errors: H <= 0 or NULL -> MB_ERR_INVALID_ARG.
 */
MB_API mb_status mb_alibi_slopes(int H, float* slopes_host);

/*
 * Index maps of the "Unpadding" paragraph.  mask[b, l] != 0 marks a real token; any 0/nonzero
 * pattern is accepted (holes allowed).
 *   mask        dev, [B, L] int32, read.
 *   seqlens     dev, [B] int32, written: number of real tokens of each row.
 *   cu_seqlens  dev, [B+1] int32, written: exclusive prefix sum of seqlens, cu[0]=0, cu[B]=T.
 *   indices     dev, capacity B*L int32; the first T entries are written with the flat positions
 *               b*L + l of the real tokens in ascending order; the rest is left untouched.
 *   meta_dev    dev, [2] int32, written: meta[0] = T, meta[1] = max_b seqlens[b].
 * B*L must be < 2^31.  B == 0: meta = {0, 0}, cu[0] = 0.
 */
MB_API mb_status mb_unpad_index(const int32_t* mask, int B, int L, int32_t* seqlens, int32_t* cu_seqlens,
                         int32_t* indices, int32_t* meta_dev, void* stream);

/* Blocking read-back of meta_dev ({T, max_seqlen}) for callers that size buffers on the host.
 *   meta_host  host, [2] int32, written.  Synchronises `stream`. */
MB_API mb_status mb_read_meta(const int32_t* meta_dev, int32_t* meta_host, void* stream);

/*
 * Gather of the "Unpadding" paragraph:  packed[t, :] = padded[indices[t], :]  for t < T.
 *   padded    dev, [rows_padded, W] elements, read (rows_padded = B*L of the mask).
 *   indices   dev, [>= T] int32 from mb_unpad_index, read.
 *   T_cap     upper bound of T used to size the launch (e.g. B*L); rows t >= T are not touched.
 *   meta_dev  dev, [2] int32 or NULL.  If given, T = min(meta_dev[0], T_cap) is read on the device
 *             (no host round trip); if NULL, T = T_cap.
 *   W         row width in elements; W * element_size must be a multiple of 16 bytes.
 *   packed    dev, [T_cap, W] capacity, rows [0, T) written.
 */
MB_API mb_status mb_unpad(const void* padded, const int32_t* indices, int T_cap, const int32_t* meta_dev,
                   int W, mb_dtype dt, void* packed, void* stream);

/*
 * Inverse scatter (Figure 1A of the paper, the step back to the padded batch):
 *   padded[indices[t], :] = packed[t, :] for t < T;  every other row of padded is set to zero bits.
 * `indices` must be strictly ascending (as mb_unpad_index writes them).  All B*L rows are written.
 *   packed    dev, [>= T, W], read.      padded  dev, [B*L, W], written in full.
 *   T_cap, meta_dev, W, dt as for mb_unpad.
 */
MB_API mb_status mb_pad(const void* packed, const int32_t* indices, int T_cap, const int32_t* meta_dev,
                 int B, int L, int W, mb_dtype dt, void* padded, void* stream);

/*
 * Companion of token_rows: sets to zero bits every row of `padded` that is NOT listed in `indices`
 * (the padding rows), leaving the listed rows alone.  After an attention call that wrote its output
 * straight into the padded layout this completes what mb_pad would have produced.
 *   indices, T_cap, meta_dev, B, L, W, dt as for mb_pad;  padded  dev, [B*L, W].
 */
MB_API mb_status mb_zero_padding(const int32_t* indices, int T_cap, const int32_t* meta_dev, int B, int L, int W,
                                 mb_dtype dt, void* padded, void* stream);

/*
 * Work plan of the any-length attention kernels (max_seqlen > 128 on the matrix cores): which workgroup computes
 * which (sequence, head, 128 tokens), dealt evenly to the chip's XCDs, longest sequences first.  It depends on
 * cu_seqlens, key_lens, B, max_seqlen and H only.  mb_alibi_attn_fwd and mb_alibi_attn_bwd build one themselves
 * on every call (the forward with a small launch of its own); a caller that runs several attention calls on the
 * same batch (every layer of an encoder, forward and backward) builds it once here and passes it as `plan`.
 *   cu_seqlens, key_lens, B, max_seqlen, H   exactly as they will be passed to the attention calls.
 *   plan   dev, at least mb_attn_plan_bytes(B, max_seqlen, H) bytes, 16-byte aligned, written.
 * Sequences longer than max_seqlen get no work (they are skipped) and raise the misuse word, see mb_device_status.
 */
MB_API size_t mb_attn_plan_bytes(int B, int max_seqlen, int H);
MB_API mb_status mb_attn_plan(const int32_t* cu_seqlens, const int32_t* key_lens, int B, int max_seqlen, int H,
                              void* plan, size_t plan_bytes, void* stream);

/*
 * Forward attention, Eq. 1:  for every sequence b, head h and tokens i, j of that sequence
 *   S_ij = softmax_scale * q_i . k_j - slopes[h] * |i - j|,   P = softmax_j(S),   O_i = sum_j P_ij v_j,
 *   lse_i = log sum_j exp(S_ij).
 *   q, k, v      dev, [T, H, D] with row strides q/k/v_row_stride (elements; >= H*D, rows a multiple of 16
 *                bytes, < 2^24), read.
 *   cu_seqlens   dev, [B+1] int32, read.
 *   T            number of token rows the packed buffers hold; T >= cu_seqlens[B].  It may be a capacity
 *                (e.g. B*L) known without reading anything back from the device: rows at or beyond
 *                cu_seqlens[B] are neither read nor written.  T is also the row pitch of lse.
 *   max_seqlen   any upper bound of the longest sequence (e.g. L); sizes the launch and picks the kernel.
 *                A sequence that turns out to be LONGER than max_seqlen is skipped as a whole, never truncated:
 *                its rows of o are left untouched, its rows of lse are set to NaN, and the device's sticky
 *                misuse word is raised (mb_device_status then reports MB_ERR_INVALID_ARG).  The lengths live
 *                on the device, so the call itself still returns MB_OK.
 *   slopes       dev, [H] float, read.
 *   o            dev, [T, H, D] with row stride o_row_stride, written.
 *   lse          dev, [H, T] float, written.
 *   workspace    dev, at least mb_alibi_attn_fwd_workspace_bytes(...) bytes, scratch (the work plan of the
 *                any-length kernels); may be NULL when that is 0 (max_seqlen <= 128, or a combination served by
 *                the generic kernels) or when `plan` is given.
 *   plan         dev, NULL or a plan built by mb_attn_plan for these very cu_seqlens, key_lens, B, max_seqlen, H
 *                (read only; ignored by kernels that need none).  With a plan of the caller's the log-sum-exp rows
 *                of a sequence longer than max_seqlen are left untouched instead of being set to NaN.
 *   key_lens     dev, [B] int32, or NULL.  NULL: every token of a sequence is a key for every query of that
 *                sequence (the packed computation).  Otherwise only the first min(key_lens[b], len_b) tokens of
 *                sequence b act as keys; the others are masked out of every softmax (S_ij = -inf) while all len_b
 *                tokens remain queries.  This is attention over a PADDED batch with a key-padding mask, what the
 *                paper's own code ran (appendix on sequence length): cu_seqlens = 0, L, 2L, ... and key_lens = the
 *                real lengths.  The backward gives masked tokens dK = dV = 0.  A sequence with key_lens[b] <= 0 is
 *                skipped.  Matrix-core kernels only (MB_ERR_UNSUPPORTED with a combination the generic kernels serve).
 *   token_rows   dev, [>= cu_seqlens[B]] int32, or NULL.  NULL: token t is row t of q, k, v and o (packed
 *                buffers).  Otherwise token t is row token_rows[t] of all four buffers: passing the
 *                `indices` of mb_unpad_index lets the call read a padded [B*L, ...] batch directly and
 *                write o into the padded layout, i.e. the gather of mb_unpad and the scatter of mb_pad
 *                happen inside the attention kernel's own row loads and stores (rows of o that belong to
 *                padding are not written: see mb_zero_padding).  lse stays packed, [H, T].  The rows of one
 *                sequence must be listed in strictly ascending order (as `indices` lists them): the kernels
 *                take a sequence whose first and last row are n - 1 apart as n consecutive rows.
 * Errors: head_dim > 128, a row stride of 2^24 elements or more, T*H >= 2^31, B*H >= 2^30, max_seqlen >= 2^22,
 * B > 65535 -> MB_ERR_UNSUPPORTED; workspace NULL or too small -> MB_ERR_WORKSPACE.
 * MB_BF16 with D = 64 and softmax_scale > 0 runs on the
 * matrix cores; every other supported combination runs the generic fp32-arithmetic kernels.
 */
MB_API mb_status mb_alibi_attn_fwd(const void* q, const void* k, const void* v, int64_t q_row_stride,
                            int64_t k_row_stride, int64_t v_row_stride, const int32_t* cu_seqlens,
                            int B, int T, int max_seqlen, int H, int D, const float* slopes,
                            float softmax_scale, mb_dtype dt, void* o, int64_t o_row_stride,
                            float* lse, void* workspace, size_t workspace_bytes, const int32_t* key_lens,
                            const int32_t* token_rows, const void* plan, void* stream);

/* Bytes of device workspace mb_alibi_attn_fwd / mb_alibi_attn_bwd need for these sizes (0 on invalid sizes; the
 * forward's is also 0 when it needs none). */
MB_API size_t mb_alibi_attn_fwd_workspace_bytes(int B, int T, int max_seqlen, int H, int D, mb_dtype dt);
MB_API size_t mb_alibi_attn_bwd_workspace_bytes(int B, int T, int max_seqlen, int H, int D, mb_dtype dt);

/*
 * Backward attention: gradients of  sum(O * dO)  for the forward above (the slopes are fixed
 * constants of the model, so they receive no gradient):
 *   Delta_i = dO_i . O_i;  dV_j = sum_i P_ij dO_i;  dP_ij = dO_i . v_j;  dS_ij = P_ij (dP_ij - Delta_i);
 *   dQ_i = softmax_scale * sum_j dS_ij k_j;   dK_j = softmax_scale * sum_i dS_ij q_i.
 * P is recomputed from q, k and lse; the score matrix is never stored.
 *   dout, o      dev, [T, H, D] with row strides do_row_stride / o_row_stride, read.
 *   lse          dev, [H, T] float from the forward, read.
 *   dq, dk, dv   dev, [T, H, D] with row strides dq/dk/dv_row_stride, written (rows [0, T)).
 *   workspace    dev, at least mb_alibi_attn_bwd_workspace_bytes(...) bytes, scratch.
 *   key_lens     as in the forward (NULL or [B]); tokens that are no keys get zero rows of dk and dv.
 *   plan         as in the forward (NULL or from mb_attn_plan); the workspace then only needs the [H, T] floats
 *                of Delta.
 *   token_rows   as in the forward; applies to dout, q, k, v, o, dq, dk and dv alike.
 * Deterministic: no atomics; two calls on the same inputs give identical bits.
 * A sequence longer than max_seqlen is skipped as in the forward (its rows of dq, dk, dv are left untouched, the
 * misuse word is raised).
 */
MB_API mb_status mb_alibi_attn_bwd(const void* dout, const void* q, const void* k, const void* v,
                            const void* o, const float* lse, int64_t do_row_stride,
                            int64_t q_row_stride, int64_t k_row_stride, int64_t v_row_stride,
                            int64_t o_row_stride, const int32_t* cu_seqlens, int B, int T,
                            int max_seqlen, int H, int D, const float* slopes, float softmax_scale,
                            mb_dtype dt, void* dq, void* dk, void* dv, int64_t dq_row_stride,
                            int64_t dk_row_stride, int64_t dv_row_stride, void* workspace,
                            size_t workspace_bytes, const int32_t* key_lens, const int32_t* token_rows,
                            const void* plan, void* stream);

/*
 * The backward attention for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, arguments, results
 * (bit for bit) and errors as mb_alibi_attn_bwd, minus `workspace` / `workspace_bytes`: the scratch lives in a
 * fixed array of MB_STATIC_SCRATCH_BYTES bytes inside the library's device image, one copy per GPU, held until
 * the process ends.  The call allocates and frees nothing.
 *   Limit    sizes whose mb_alibi_attn_bwd_workspace_bytes exceeds MB_STATIC_SCRATCH_BYTES are rejected with
 *            MB_ERR_WORKSPACE before anything is launched (about H * T <= 4 million (head, token-row) pairs).
 *   Sharing  every call on a GPU uses that GPU's one array, which keeps the previous call's contents; nothing
 *            in it needs clearing (each word is written before it is read within a call).  Two such calls that
 *            overlap in time on one GPU (different streams or threads) race on it: serialise them.
 */
#define MB_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
MB_API mb_status mb_alibi_attn_bwd_static(const void* dout, const void* q, const void* k, const void* v,
                            const void* o, const float* lse, int64_t do_row_stride,
                            int64_t q_row_stride, int64_t k_row_stride, int64_t v_row_stride,
                            int64_t o_row_stride, const int32_t* cu_seqlens, int B, int T,
                            int max_seqlen, int H, int D, const float* slopes, float softmax_scale,
                            mb_dtype dt, void* dq, void* dk, void* dv, int64_t dq_row_stride,
                            int64_t dk_row_stride, int64_t dv_row_stride, const int32_t* key_lens,
                            const int32_t* token_rows, const void* plan, void* stream);

/*
 * Reads and clears the current device's sticky misuse word.  Synchronises `stream`.
 *   MB_OK               no attention call since the last check met a sequence longer than its max_seqlen;
 *   MB_ERR_INVALID_ARG  one did (see max_seqlen of mb_alibi_attn_fwd for what happened to that sequence).
 * The word is per device and shared by all streams and threads: a check reports misuse by any of them.
 */
MB_API mb_status mb_device_status(void* stream);

/*
 * Add & LayerNorm over packed token rows with 2-byte storage ("Low Precision LayerNorm" paragraph of the
 * paper: LayerNorm is bandwidth-bound, so it reads and writes bfloat16; "Add & Norm" in Figure 1A):
 *   s = x + r  (stored, rounded once to the storage type),   mean, var over the W elements of a row,
 *   y = (s - mean) / sqrt(var + eps) * gamma + beta.         Statistics and normalisation are fp32.
 *   x, r      dev, [T_cap, W], read; r may be NULL (then s = x and `s` is not written and may be NULL).
 *   gamma, beta  dev, [W], same type as x, read.
 *   T_cap, meta_dev  rows [0, T) are processed, T = min(meta_dev[0], T_cap), or T_cap if meta_dev is NULL.
 *   W         row width; W * element_size a multiple of 16 bytes and at most 4096 bytes.
 *   y, s      dev, [T_cap, W], written.     mean, rstd  dev, [T_cap] float, written (needed by the backward).
 *   y_rows    dev, NULL or [T] int32 (the `indices` of mb_unpad_index): row t of the result is written to row
 *             y_rows[t] of y, which is then a padded batch [B*L, W]: the scatter of mb_pad happens in this
 *             call's own stores when the LayerNorm is the last operation on the packed tokens (the padding rows
 *             are not written: see mb_zero_padding).  s, mean and rstd stay packed.
 */
MB_API mb_status mb_add_layernorm_fwd(const void* x, const void* r, const void* gamma, const void* beta, int T_cap,
                                      const int32_t* meta_dev, int W, float eps, mb_dtype dt, void* y, void* s,
                                      float* mean, float* rstd, const int32_t* y_rows, void* stream);

/* Bytes of device workspace mb_add_layernorm_bwd needs for rows of W elements (0 on invalid W). */
MB_API size_t mb_add_layernorm_bwd_workspace_bytes(int W);

/*
 * Gradient of sum(y * dy) for the call above:  xhat = (s - mean) rstd,  g = dy * gamma,
 *   ds = rstd * (g - mean(g) - xhat * mean(g * xhat))   (the gradient of both x and r),
 *   dgamma = sum_t dy * xhat,   dbeta = sum_t dy         (fp32, summed in a fixed order: deterministic).
 *   dy, s  dev, [T_cap, W], read (s = the stored sum of the forward, or x when r was NULL).
 *   ds     dev, [T_cap, W], written.   dgamma, dbeta  dev, [W] float, written.
 *   workspace  dev, at least mb_add_layernorm_bwd_workspace_bytes(W) bytes, scratch.
 *   dy_rows    dev, NULL or [T] int32: row t of dy is read from row dy_rows[t] of a padded batch (the gather of
 *              mb_unpad in this call's own loads); everything else stays packed.
 */
MB_API mb_status mb_add_layernorm_bwd(const void* dy, const void* s, const void* gamma, const float* mean,
                                      const float* rstd, int T_cap, const int32_t* meta_dev, int W, mb_dtype dt,
                                      void* ds, float* dgamma, float* dbeta, void* workspace,
                                      size_t workspace_bytes, const int32_t* dy_rows, void* stream);

/*
 * GeGLU feed-forward sublayer, forward (Eq. 2 of the paper:  y = (GeLU(x W1) (*) x V) W2,  GeLU(h) = h Phi(h)
 * in its exact form, no bias terms), in the fused arrangement of the appendix on GLU implementations: the two
 * input projections are one matrix of twice the width whose product is sliced in two.
 *   x      dev, [T_cap, hidden], read.
 *   w1v    dev, [2*inter, hidden], read: rows 0..inter-1 hold W1 transposed, rows inter..2*inter-1 hold V
 *          transposed (the [out_features, in_features] storage of a linear layer, contiguous along hidden).
 *   w2     dev, [hidden, inter], read: W2 transposed, same convention.
 *   T_cap, meta_dev  rows [0, T) are processed, T = min(meta_dev[0], T_cap), or T_cap if meta_dev is NULL;
 *          rows at and beyond T are neither read nor written.
 *   act    dev, [T_cap, inter], written: GeLU(x W1) (*) x V rounded once to the storage type; it is the
 *          operand of the second projection and what a backward pass needs.
 *   y      dev, [T_cap, hidden], written.
 * Products accumulate in fp32.  Supported: MB_BF16 with hidden a multiple of 256 and inter a multiple of 128
 * (MB_ERR_UNSUPPORTED otherwise).  All pointers 16-byte aligned.  Nothing is allocated; work is enqueued on
 * `stream`.
 */
MB_API mb_status mb_geglu_fwd(const void* x, const void* w1v, const void* w2, int T_cap, const int32_t* meta_dev,
                              int hidden, int inter, mb_dtype dt, void* act, void* y, void* stream);

/* Bytes of device workspace mb_geglu_bwd needs (0 on arguments it would reject). */
MB_API size_t mb_geglu_bwd_workspace_bytes(int T_cap, int hidden, int inter, mb_dtype dt);

/*
 * Backward of mb_geglu_fwd for the scalar loss sum(y * dy) (the textbook derivative of Eq. 2; the paper prints
 * none).  With h = x W1, g = x V, a = GeLU(h) (*) g:
 *   dA = dy W2^T,   dh = dA (*) g (*) GeLU'(h),   dg = dA (*) GeLU(h),   GeLU'(h) = Phi(h) + h phi(h),
 *   dx = dh W1^T + dg V^T,   dW2 = a^T dy,   dW1 = x^T dh,   dV = x^T dg.
 *   dy   dev, [T_cap, hidden], read.        x, w1v, w2   as in mb_geglu_fwd, read.
 *   act  dev, [T_cap, inter], read: the activation the forward stored.
 *   hg   dev, [T_cap, 2*inter] or NULL, read: x W1 | x V as the unfused forward (mb_linear_fwd with w1v) stores
 *        them; NULL (the fused forward keeps neither) makes this call compute them again.
 *   dx   dev, [T_cap, hidden], written (rows [0, T) only).
 *   dw1v dev, [2*inter, hidden] float, written: gradient of w1v in its own (transposed) layout, dW1^T over dV^T.
 *   dw2  dev, [hidden, inter] float, written: gradient of w2 in its own layout (dW2^T).
 *   workspace  dev, 256-byte aligned, at least mb_geglu_bwd_workspace_bytes bytes, scratch.
 * Weight gradients are fp32 sums over the T token rows taken in a fixed order (deterministic); with T = 0 they
 * are zeros.  dh and dg pass through bf16 on their way into the products.  Supported: MB_BF16 with hidden and
 * inter multiples of 256.
 */
MB_API mb_status mb_geglu_bwd(const void* dy, const void* x, const void* w1v, const void* w2, const void* act,
                              const void* hg, int T_cap, const int32_t* meta_dev, int hidden, int inter, mb_dtype dt, void* dx,
                              float* dw1v, float* dw2, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The pieces of the UNFUSED arrangements of the same sublayer (appendix on GLU implementations: two separate
 * input projections, or one of twice the width whose product is stored and sliced), for comparison with
 * mb_geglu_fwd, which never stores the projections:
 *
 * mb_linear_fwd:  y = x W for a bias-free linear layer.
 *   x   dev, [T_cap, n_in], read.      wt  dev, [n_out, n_in], read: W transposed.      y  dev, [T_cap, n_out], written.
 *   Supported: MB_BF16, n_in a multiple of 128, n_out a multiple of 256 or of 192 (MB_ERR_UNSUPPORTED otherwise).
 * mb_gelu_gate:   act = GeLU(h) (*) gate, elementwise, exact-form GeLU.
 *   h, gate  dev, [T_cap, inter] blocks with a common row stride `row_stride` (elements): two separate buffers
 *            (row_stride = inter) or the two halves of one [T_cap, 2*inter] buffer (gate = h + inter, row_stride =
 *            2*inter).  act  dev, [T_cap, inter] contiguous, written.  inter and row_stride multiples of 8.
 * Rows [0, T), T = min(meta_dev[0], T_cap) or T_cap if meta_dev is NULL; pointers 16-byte aligned.
 */
MB_API mb_status mb_linear_fwd(const void* x, const void* wt, int T_cap, const int32_t* meta_dev, int n_in, int n_out,
                               mb_dtype dt, void* y, void* stream);
MB_API mb_status mb_gelu_gate(const void* h, const void* gate, int64_t row_stride, int T_cap, const int32_t* meta_dev,
                              int inter, mb_dtype dt, void* act, void* stream);

/*
 * Ceiling probe for callers that measure (bench.py): enqueues one launch of a kernel that saturates one unit
 * and does nothing else, and reports the work of that launch; the caller times it.  Not an operation of the
 * paper: it exists so that the roofs kernels are priced against are measured on the machine at hand.
 *   kind   0: v_mfma_f32_32x32x16_bf16, independent accumulators (work = flops)
 *          1: fp32 fused multiply-add on the vector unit (work = flops)
 *          2: fp32 exponential on the vector unit (work = exponentials)
 *          (the HBM ceiling is measured with mb_unpad as a plain row copy: identity indices)
 *   iters  rounds per lane (> 0).      out  dev, 4 floats of scratch (never written in practice).
 *   work_per_launch  host, written.
 */
MB_API mb_status mb_probe_ceiling(int kind, int iters, float* out, double* work_per_launch, void* stream);

/*
 * Ceiling probe for the memory traffic of the backward attention at sequence lengths <= 128 (the kernel the
 * benchmark's roofline is about): one launch that moves exactly that kernel's bytes in its access pattern and does
 * no arithmetic.  Per (sequence, head) a workgroup reads the Q, K, V rows of a fused [T, 3, H, 64] buffer and the
 * dO and O rows of [T, H, 64] buffers (128 bytes per row and tensor), passes them once through LDS, and writes the
 * three row sets of a fused [T, 3, H, 64] gradient buffer.  Eight concurrent row streams (5 in, 3 out) reach less
 * than a plain copy; the caller times the launch and prices the real kernel against it.
 *   qkv, dout, o  dev, bf16, read.    dqkv  dev, [T, 3, H, 64] bf16, OVERWRITTEN with meaningless values.
 *   cu_seqlens    dev, [B+1] int32 (sequences longer than 128 are cut at 128).
 */
MB_API mb_status mb_probe_bwd_traffic(const void* qkv, const void* dout, const void* o, void* dqkv,
                                      const int32_t* cu_seqlens, int B, int H, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOSAIC_ATTN_H */
