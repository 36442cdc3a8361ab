/*
 * turbo_reduce.h - C ABI of the MI355X (gfx950) batch-reduction library.
 *
 * The two operations are the "batch reduction" kernels of the
 * TurboTransformers paper, Section 4.1.2: on the low dimension of a 2-D view
 * of a tensor, Softmax needs a maximum and a sum per row, LayerNorm a mean
 * and a variance per row, for a whole batch of rows at once.
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device.  The
 *     caller owns every buffer; the library allocates nothing, keeps no
 *     workspace and never synchronises.  Work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the null stream) and the call
 *     returns immediately.
 *   - Tensors are dense, row-major, last index fastest.
 *   - The return value is a TURBO_* status.  Argument validation happens
 *     before the first HIP call, so every error except TURBO_ERR_LAUNCH is
 *     reported without touching the GPU and without enqueuing work.
 *   - A size of zero (or below) in any dimension is TURBO_ERR_SHAPE: an empty
 *     call is treated as a caller bug, not as a no-op.
 *   - Base pointers must be aligned to the element size (TURBO_ERR_ALIGN
 *     otherwise).  16-byte alignment together with a row length that is a
 *     multiple of 16 bytes selects the widest loads; nothing more is required.
 *   - Non-finite inputs are outside the contract.
 *   - The entry points may be called from several host threads.  The only state the library keeps is a per-device
 *     cache of two launch facts (the device's compute-unit count and, per looping kernel, how many of its workgroups
 *     a compute unit holds), filled on first use with relaxed atomic stores of values that are the same whoever
 *     writes them.  The testing hooks of turbo_reduce_testing.h are the exception: they are process-wide switches
 *     for tests and tuning runs and must not be flipped while another thread is inside the library.
 */
#ifndef TURBO_REDUCE_H
#define TURBO_REDUCE_H

#ifdef __cplusplus
extern "C" {
#endif

enum turbo_status {
    TURBO_OK = 0,
    TURBO_ERR_NULL = 1,   /* a required pointer is NULL */
    TURBO_ERR_SHAPE = 2,  /* a dimension is <= 0, the row count exceeds 2^31 - 2^16, or a mask stride is negative */
    TURBO_ERR_DTYPE = 3,  /* dtype is not TURBO_F32 / TURBO_F16 */
    TURBO_ERR_ALIGN = 4,  /* a pointer is not aligned to its element size */
    TURBO_ERR_LAUNCH = 5  /* HIP reported an error when the kernel was enqueued */
};

enum turbo_dtype {
    TURBO_F32 = 0, /* IEEE binary32 in memory, binary32 arithmetic */
    TURBO_F16 = 1  /* IEEE binary16 in memory, binary32 arithmetic; rounded to binary16 (nearest-even) only on the final store */
};

/*
 * Scaled, masked softmax over attention scores (Section 2.1: the scaled
 * dot-product attention applies a softmax to the query-key products;
 * Section 4.1.2: softmax reduces a maximum and a sum over the low dimension).
 *
 *   scores[b,h,q,k] <- exp(z[b,h,q,k] - m) / sum_k exp(z[b,h,q,k] - m),
 *   z = scale * scores + mask,   m = max_k z            (IN PLACE)
 *
 *   scores  device, [B,H,Sq,Sk] of `dtype`, read and overwritten.
 *   mask    device, additive mask of the same dtype, dense [B,Sq,Sk], shared
 *           by all heads (the padding mask of a zero-padded variable-length
 *           batch, Section 2.1, holds 0 for real keys and -10000 for padded
 *           ones).  NULL = no mask.  Must not overlap `scores`.
 *   scale   multiplies the scores only; the mask is added unscaled.
 *   dtype   TURBO_F32 or TURBO_F16.
 *
 * Masked entries come out as 0 because exp() underflows, not by a special
 * case: a row whose keys are all masked is the softmax of its scores.
 */
int turbo_masked_softmax(void *scores, const void *mask, int B, int H, int Sq, int Sk, float scale, int dtype,
                         void *stream);

/*
 * Same operation with explicit element strides for the mask, so compact
 * masks need no expansion: mask element (b,q,k) is read from
 * mask[b*mask_stride_b + q*mask_stride_q + k].
 *   per-request key mask [B,Sk] : mask_stride_b = Sk,    mask_stride_q = 0
 *   causal mask [Sq,Sk]         : mask_stride_b = 0,     mask_stride_q = Sk
 *   dense [B,Sq,Sk]             : mask_stride_b = Sq*Sk, mask_stride_q = Sk
 * Strides must be >= 0 (TURBO_ERR_SHAPE otherwise); they are ignored when
 * mask is NULL.
 */
int turbo_masked_softmax_ex(void *scores, const void *mask, long long mask_stride_b, long long mask_stride_q, int B,
                            int H, int Sq, int Sk, float scale, int dtype, void *stream);

/*
 * Length-aware variant for zero-padded variable-length batches (Section 2.1: short sequences are padded to the
 * longest one of the batch; the paper's kernels then work on the padding too).  Instead of an additive mask the
 * caller passes the request lengths, and the kernel neither reads nor normalises what lies beyond them:
 *
 *   for q < q_lengths[b]:  scores[b,h,q,k] <- softmax over k < k_lengths[b] of scale*scores[b,h,q,k],
 *                          scores[b,h,q,k] <- 0 for k >= k_lengths[b];
 *   rows q >= q_lengths[b] are left untouched.
 *
 * For real rows this equals turbo_masked_softmax_ex with a 0 / -10000 key mask (where exp() underflows to the
 * same exact zeros).  k_lengths, q_lengths: DEVICE int32 arrays [B]; q_lengths may be NULL (all Sq rows are
 * computed); for self-attention pass the same array twice.  Lengths are clamped to 0..Sk; a request with
 * k_lengths[b] = 0 is left untouched.
 */
int turbo_masked_softmax_varlen(void *scores, const int *q_lengths, const int *k_lengths, int B, int H, int Sq, int Sk,
                                float scale, int dtype, void *stream);

/*
 * Causal variant of the length-aware call (decoder self-attention, e.g. the GPT-2 configuration of the benchmark):
 * query q sees the keys k <= q + (Sk - Sq), so with Sq == Sk the usual lower triangle and with a key cache
 * (Sk > Sq) the last query sees every key.  The keys beyond the diagonal get weight exactly 0 WITHOUT BEING READ,
 * which halves the bytes read for a square score matrix; this equals turbo_masked_softmax_ex with a 0 / -10000
 * mask above the diagonal.  q_lengths and k_lengths (DEVICE int32 [B]) restrict rows and keys further as in
 * turbo_masked_softmax_varlen; either may be NULL.  Rows that see no key (Sq > Sk, or a zero length) are left
 * untouched.
 */
int turbo_masked_softmax_causal(void *scores, const int *q_lengths, const int *k_lengths, int B, int H, int Sq, int Sk,
                                float scale, int dtype, void *stream);

/*
 * Row-packed variant for variable-length batches that are not padded in memory at all (the paper pads, Sections
 * 2.1 and 5; this is the layout its discussion of wasted padding work points to).  Request b, of len_b tokens,
 * stores its self-attention scores as a dense [H][len_b][len_b] block; the blocks lie in `scores` at the element
 * offsets score_offsets[b] (normally one after the other: score_offsets[b] = H * sum_{i<b} len_i^2).  In place:
 *
 *   for every request b, head h, query q < len_b:   row <- softmax over k < len_b of scale * row.
 *
 * cu_seqlens:    DEVICE int32 [B+1], cumulative lengths: cu_seqlens[0] = 0, cu_seqlens[b+1] - cu_seqlens[b] = len_b >= 0.
 * score_offsets: DEVICE int64 [B+1] (entry B is not used).
 * total_tokens:  the caller's HOST copy of cu_seqlens[B] (sizes the launch);  max_len: HOST upper bound on len_b
 *                (sizes the registers per row); what happens to a request longer than max_len is unspecified (it is
 *                either computed like the others or left untouched; nothing outside it is touched).
 * Requests of up to 4096 (TURBO_F32) or 8192 (TURBO_F16) tokens keep a row in one wavefront's registers; when max_len
 * is larger, a second kernel launch gives every longer row a workgroup.  max_len is at most 32768 (TURBO_ERR_SHAPE beyond).
 * The LayerNorm of a packed batch needs no entry point of its own: its tokens are [total_tokens, hidden] rows of
 * turbo_add_bias_layernorm_dt.
 */
int turbo_masked_softmax_packed(void *scores, const int *cu_seqlens, const long long *score_offsets, int B, int H,
                                int total_tokens, int max_len, float scale, int dtype, void *stream);

/*
 * Fused bias add + residual add + LayerNorm (the "AddBiasLayerNorm" kernel of
 * Section 6.2.1; Section 4.1.2 and Equation 1: LayerNorm reduces a mean and a
 * population variance per row), binary32 tensors:
 *
 *   t[r,j]   = x[r,j] + bias[j] + residual[r,j]
 *   mu_r     = mean_j t[r,j],   var_r = mean_j (t[r,j] - mu_r)^2
 *   out[r,j] = (t[r,j] - mu_r) / sqrt(var_r + eps) * gamma[j] + beta[j]
 *
 *   x, residual, out   device, [rows, hidden]
 *   bias, gamma, beta  device, [hidden]
 *   residual and bias may be NULL (treated as zeros); x, gamma, beta, out
 *   are required.  `out` may be exactly `x` or exactly `residual` (each row
 *   is read completely before any of it is written); any other overlap is
 *   undefined.
 */
int turbo_add_bias_layernorm(const void *x, const void *residual, const void *bias, const void *gamma,
                             const void *beta, int rows, int hidden, float eps, void *out, void *stream);

/* The same operation with all six tensors stored in `dtype` (TURBO_F32 or TURBO_F16). */
int turbo_add_bias_layernorm_dt(const void *x, const void *residual, const void *bias, const void *gamma,
                                const void *beta, int rows, int hidden, float eps, void *out, int dtype, void *stream);

/*
 * Length-aware variant for zero-padded variable-length batches: x, residual, out are [B, S, hidden]; token rows
 * (b, s) with s >= lengths[b] are padding and are neither read nor written (out keeps whatever it held there);
 * all other rows are computed exactly as by turbo_add_bias_layernorm_dt.  lengths: DEVICE int32 array [B].
 */
int turbo_add_bias_layernorm_varlen(const void *x, const void *residual, const void *bias, const void *gamma,
                                    const void *beta, const int *lengths, int B, int S, int hidden, float eps,
                                    void *out, int dtype, void *stream);

/*
 * Element-wise fused kernels between two GEMMs (Section 4.1.1 names the fused activation and the fused
 * transposes as the purely element-wise kind of non-GEMM kernel, without printing a formula or a layout; the
 * definitions below are this library's reading).  Same conventions as above; `dtype` is TURBO_F32 or TURBO_F16 with binary32 arithmetic.
 *
 * turbo_add_bias_gelu:  out[r,j] = gelu(x[r,j] + bias[j]) on [rows, hidden], the feed-forward activation of
 *   the BERT family.  approximate = 0: gelu(t) = t * Phi(t), Phi the standard normal distribution function;
 *   approximate = 1: 0.5 t (1 + tanh(sqrt(2/pi) (t + 0.044715 t^3))).  bias may be NULL.  out may be exactly x.
 *   rows * hidden may be any positive count whose 16-byte vectors number below 2^31.
 *
 * turbo_add_bias_split_heads:  x is [B, S, n_split, H, D], the output of one fused projection (n_split = 3 for
 *   Q, K, V together, 1 for a single projection); bias is [n_split, H, D] or NULL; out is
 *   [n_split, B, H, S, D]:  out[k,b,h,s,d] = x[b,s,k,h,d] + bias[k,h,d].  out must not overlap x.
 *
 * turbo_merge_heads:  x is [B, H, S, D] (attention output per head), out is [B, S, H, D]:
 *   out[b,s,h,d] = x[b,h,s,d].  out must not overlap x.
 */
int turbo_add_bias_gelu(const void *x, const void *bias, int rows, int hidden, int approximate, void *out, int dtype,
                        void *stream);
int turbo_add_bias_split_heads(const void *x, const void *bias, int B, int S, int n_split, int H, int D, void *out,
                               int dtype, void *stream);
int turbo_merge_heads(const void *x, int B, int H, int S, int D, void *out, int dtype, void *stream);

/* Static, NUL-terminated description of a status code (host pointer, never NULL). */
const char *turbo_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TURBO_REDUCE_H */
