/* ffn24 -- Squared-ReLU feed-forward block with 2:4 activation sparsity, for AMD MI355X (gfx950).
 *
 * C ABI of libffn24.so.  The method is that of "Accelerating Transformer Inference and Training with 2:4
 * Activation Sparsity" (Haziza et al.): the hidden activation H = max(0, X W1)^2 of an FFN is mostly zero, so of
 * every 4 consecutive hidden features of a token only the 2 of largest magnitude are kept, and the second GEMM
 * (and, in training, three of the four backward GEMMs) run on sparse matrix cores.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, row-major and contiguous, 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue kernels and copies
 *     on that stream (no memset nodes, so a sequence can be recorded into a HIP graph); they never synchronise and
 *     allocate no device memory.  The exceptions are the set-up calls: ffn24_ctx_create allocates, and
 *     ffn24_set_token_permutation waits for the device.
 *   - A context belongs to the device that was current when it was created; calls that launch work with another
 *     device current return FFN24_ERR_STATE.  A context is not thread-safe: one thread at a time per context.
 *   - Return value: FFN24_OK (0) or a negative FFN24_ERR_* code; ffn24_strerror() names it.  Bad arguments are
 *     rejected before anything is launched; nothing aborts or throws across this boundary.
 *   - Element type: bf16 (FFN24_BF16) with fp32 accumulation; or fp8 (FFN24_FP8_E4M3, the OCP e4m3 format, per-tensor
 *     fp32 scales, fp32 accumulation, bf16 results; see ffn24_set_scales and ffn24_set_bwd_scales).
 *   - Outputs are overwritten, never accumulated into.
 *
 * Compressed 2:4 form used everywhere (the paper leaves the encoding open; this one equals the index operand of
 * the gfx950 sparse matrix instruction, so it is consumed without any shuffling):
 *   values [rows][cols/2]  the two kept entries of each group of 4, in position order;
 *   meta   [rows][cols/8]  one nibble per group, i0 | (i1 << 2) with i0 < i1 the kept positions; the even
 *                          group of a pair sits in the low nibble of the byte.
 * Pick rule: order the 4 entries by (magnitude descending, position ascending) and keep the first two; the
 * magnitude is the bf16 word with its sign bit cleared, compared as an integer.  Zeros compete like any value,
 * so an all-zero group keeps positions {0, 1}.
 */
#ifndef FFN24_H
#define FFN24_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define FFN24_API __attribute__((visibility("default")))
#else
#define FFN24_API
#endif

#define FFN24_OK 0
#define FFN24_ERR_NULL (-1)   /* a required pointer is NULL */
#define FFN24_ERR_SHAPE (-2)  /* a size violates the divisibility rules stated at the call */
#define FFN24_ERR_ALIGN (-3)  /* a pointer is not 16-byte aligned */
#define FFN24_ERR_DTYPE (-4)  /* element type not supported */
#define FFN24_ERR_STATE (-5)  /* call order: backward without the matching forward, missing context flag, wrong current device */
#define FFN24_ERR_HIP (-6)    /* the HIP runtime reported an error (allocation, launch) */
#define FFN24_ERR_NOTREADY (-7) /* ffn24_get_telemetry without waiting: no snapshot has completed yet */
#define FFN24_ERR_SCRATCH (-8)  /* ffn24_fwd_static: the intermediate tensors exceed FFN24_STATIC_SCRATCH_BYTES */

typedef enum { FFN24_BF16 = 0, FFN24_FP8_E4M3 = 1 } ffn24_dtype;

/* context flags */
#define FFN24_TRAINING 1     /* allocate what ffn24_bwd needs (dZ, transposed operands) */
#define FFN24_DENSE 2        /* allocate what the dense baseline ffn_fwd / ffn_bwd needs (H, dZ as [T][F]) */
#define FFN24_DEBUG_DUMP_H 4 /* ffn24_fwd also stores the rounded activation before pruning, [T][F] */
#define FFN24_SPLIT 8        /* allocate what the split weight-gradient GEMMs need (with FFN24_TRAINING; see ffn24_set_split) */
#define FFN24_ROWWISE 16     /* fp8 context with row-wise instead of per-tensor scales (see ffn24_set_row_scales) */
#define FFN24_PERMUTE 32     /* context that can run with a token permutation (bf16, or fp8 with FFN24_ROWWISE; see ffn24_set_token_permutation) */
#define FFN24_TELEMETRY 64   /* bf16 context whose forwards and backwards count sparsity and drops (see ffn24_get_telemetry) */

typedef struct ffn24_ctx ffn24_ctx; /* opaque; owns only its device workspace */

/* Create a context for token count T, model dimension D, hidden dimension F.
 * Requires T, D, F to be multiples of 256 (the GEMM tile) and at most 2^20.  Other token counts are the caller's to
 * pad: give X and dY zero rows up to the next multiple of 256.  A zero row of dY gives a zero row of dZ and a zero
 * row of X multiplies it, so the padding adds nothing to dW1 and dW2; Y and dX are computed per token, the padding's
 * rows of them are ignored; and if the real token count is a multiple of 4 no padded token shares a feature-wise
 * 2:4 group with a real one (without a bias -- the paper's FFN -- a padded token's activation is zero anyway).
 * Allocates the device workspace with
 * hipMalloc on the current device: about 1.13 T F + 4 D F bytes; plus 3.13 T F + 4 T D + 4 D F with FFN24_TRAINING
 * (T F + 2 D F more with FFN24_SPLIT); plus
 * 2 T F with FFN24_DENSE (6 T F more when FFN24_TRAINING is set too); plus 2 T F with FFN24_DEBUG_DUMP_H.
 * *out is untouched on error. */
FFN24_API int ffn24_ctx_create(ffn24_ctx** out, int64_t T, int64_t D, int64_t F, ffn24_dtype dtype, int flags);

/* Scales of an FFN24_FP8_E4M3 context (all 1 after creation), each > 0:  the caller hands in X8 = e4m3(X / sx),
 * W1_8 = e4m3(W1 / sw1), W2_8 = e4m3(W2 / sw2) as byte tensors of the usual shapes, and the kernels compute
 *   Z = sx sw1 (X8 W1_8) + b1;  H = bf16(max(0, Z)^2);  keep-2-of-4 on the bf16 words (as in the bf16 path);
 *   Hc8 = e4m3(kept / sh), saturating at +-448, round to nearest even;  Y = bf16(sh sw2 (Hc8 . W2_8))
 * (paper Sec. 2: activation, then sparsification, then FP8 quantisation; per-tensor scales instead of the paper's
 * row-wise ones).  Saved tensors 0 and 1 are then bytes: Hc8 [T][F/2], meta [T][F/8]; tensor 7 is H8 [T][F].
 * ffn_fwd is the dense fp8 baseline of the forward.  With FFN24_TRAINING (FFN24_SPLIT only together with FFN24_ROWWISE, else
 * FFN24_ERR_DTYPE) the context
 * also supports ffn24_bwd -- and, with FFN24_DENSE, ffn_bwd -- in fp8, see ffn24_set_bwd_scales; with FFN24_ROWWISE as well
 * the backwards are ffn24_bwd_rowwise and ffn_bwd_rowwise. */
FFN24_API int ffn24_set_scales(ffn24_ctx* ctx, float sx, float sw1, float sh, float sw2);

/* fp8 backward of an FFN24_FP8_E4M3 | FFN24_TRAINING context (paper abstract: FP8 in both the forwards and the
 * backwards pass; Sec. 2, the paragraph on the fused backward pointwise kernel: it includes the FP8 scaling).  Both
 * scales > 0 (1 after creation).  ffn24_bwd then takes dY8 = e4m3(dY / sdy) as bytes [T][D] and computes, with every
 * GEMM operand in e4m3 and fp32 accumulation,
 *   dH = sdy sw2 (dY8 . W2_8^T);  dZ = dH * 2 max(0, Z) on the kept positions, the derivative taken as 2 sqrt(h) of the
 *   bf16 kept activation the forward saved;  dZ8 = e4m3(dZ / sdz), saturating, compressed with the forward's metadata;
 *   dX = bf16(sdz sw1 (dZ8 . W1_8^T));  feature-wise 2:4 on top, ranked on the stored e4m3 codes of the activation;
 *   dW2 = bf16(sh sdy ((H24_8 * M_T)^T . dY8));  dW1 = bf16(sx sdz (X8^T . (dZ8 * M_T))).
 * dX [T][D], dW1 [D][F], dW2 [F][D] are bf16.  Saved tensors 2, 3, 5 are then e4m3 bytes; tensor 12 is the bf16 kept
 * activation [T][F/2].  ffn_bwd on such a context (FFN24_DENSE too) is the dense fp8 baseline: the same with no masks,
 * dZ8 = e4m3(dH * 2 sqrt(h) / sdz) at every position (saved tensor 8, bytes), h the bf16 activation its forward saved. */
FFN24_API int ffn24_set_bwd_scales(ffn24_ctx* ctx, float sdy, float sdz);

/* Row-wise scaling of an fp8 context created with FFN24_ROWWISE (paper Sec. 2: "FP8 rowwise scaling"): the activation
 * operand of each GEMM has one scale per token, the weight operand one per output channel.  The caller hands in
 * X8[t][k] = e4m3(X[t][k] / sx[t]), W1_8[k][f] = e4m3(W1[k][f] / sw1[f]), W2_8[f][d] = e4m3(W2[f][d] / sw2[d]) and the
 * three scale vectors sx [T], sw1 [F], sw2 [D] (fp32, device memory, 16-byte aligned, kept alive by the caller).
 * ffn24_fwd then computes  Z = sx[t] sw1[f] (X8 W1_8) + b1;  H = bf16(max(0, Z)^2);  keep-2-of-4 on the bf16 words;
 * sh[t] = (largest activation of token t) / 448, 1 for an all-zero row;  Hc8 = e4m3(kept / sh[t]);
 * Y = bf16(sh[t] sw2[d] (Hc8 . W2_8)).  Three kernels as in the paper: the up-projection (with activation and
 * sparsification fused in), a quantisation kernel (the row scale needs the whole row), the 2:4 GEMM.
 * Saved tensor 11 is sh [T] fp32.  With FFN24_DENSE the context also runs ffn_fwd with the same scales: the dense
 * baseline of the paper's forward benchmark, whose FP8 GEMMs use row-wise scaling on both sides -- up-projection,
 * row-wise quantisation of every activation with sh[t] = (largest activation of token t) / 448, dense GEMM; saved tensor
 * 7 is then H8 [T][F] and tensor 11 the sh of that forward. */
FFN24_API int ffn24_set_row_scales(ffn24_ctx* ctx, const float* sx, const float* sw1, const float* sw2);

/* Row-wise scaling of a GEMM operand (paper Sec. 2: "FP8 rowwise scaling"): X is a bf16 matrix [rows][cols], row-major, device
 * memory, cols a multiple of 8.  axis 1: one scale per row, scales[r] = max_c |X[r][c]| / 448 (1 if the row is all zero);
 * axis 0: one scale per column, scales[c] = max_r |X[r][c]| / 448.  codes[r][c] = e4m3(X[r][c] / scale), round to nearest even
 * (nothing saturates: the largest entry of every row / column maps to 448).  codes: rows x cols bytes, row-major; scales: fp32,
 * [rows] or [cols] (with axis 0 the buffer also holds intermediate values until the call's last kernel has run).  These are the
 * (codes, scales) pairs that ffn24_set_row_scales / ffn24_fwd and ffn24_bwd_rowwise take, made from the caller's bf16 tensors:
 * X per row, W1 and W2 per column for the forward; dY per row and per column, X per column, W2 and W1 per row for the backward.
 * Empty matrices are a no-op.  FFN24_ERR_SHAPE for another axis or cols % 8 != 0. */
FFN24_API int quantise_e4m3(const void* X, int64_t rows, int64_t cols, int axis, void* codes, float* scales, void* stream);

/* Backward of a row-wise-scaled forward: an FFN24_FP8_E4M3 | FFN24_ROWWISE | FFN24_TRAINING context, after ffn24_fwd.  Every GEMM of the backward is scaled row-wise, as the paper's precision recipe has it for all
 * of its FP8 matrix multiplications (caption of the forward-speed-up figure; Sec. 2, the paragraph on the fused backward pointwise
 * kernel: it includes the transposition and the FP8 scaling): each operand carries one scale per index of its NON-reduced
 * dimension.  A tensor that enters two GEMMs with different reduced dimensions is therefore quantised twice, by the caller,
 * from its higher-precision copy -- all pointers are device memory, 16-byte aligned, codes are e4m3 bytes, scales fp32 > 0:
 *   dY8r [T][D], sdy_t [T]: dY8r[t][d] = e4m3(dY[t][d] / sdy_t[t])      (dH GEMM, reduced over d)
 *   dY8c [T][D], sdy_d [D]: dY8c[t][d] = e4m3(dY[t][d] / sdy_d[d])      (dW2 GEMM, reduced over t)
 *   X8c  [T][D], sx_d  [D]: X8c[t][d]  = e4m3(X[t][d]  / sx_d[d])       (dW1 GEMM, reduced over t)
 *   W2_8r [F][D], sw2_f [F]: W2_8r[f][d] = e4m3(W2[f][d] / sw2_f[f])    (dH GEMM)
 *   W1_8c [D][F], sw1_d [D]: W1_8c[d][f] = e4m3(W1[d][f] / sw1_d[d])    (dX GEMM, reduced over f)
 * The tensors the backward makes itself are quantised where they are made, each scale = (largest magnitude) / 448, 1 if all zero:
 *   dH[t][f] = sdy_t[t] sw2_f[f] (dY8r . W2_8r^T);  dZ = bf16(dH * 2 max(0, Z)) on the kept positions (the derivative taken as
 *   2 sqrt(h) of the bf16 kept activation the forward saved), compressed with the forward's metadata;
 *   sdz_t[t] = max_f |dZ[t][f]| / 448;  dZ8r = e4m3(dZ / sdz_t[t]);  dX = bf16(sdz_t[t] sw1_d[d] (dZ8r . W1_8c^T));
 *   feature-wise 2:4 on top of the token-wise mask, ranked on the bf16 activation (as in the bf16 backward), one mask for H and dZ;
 *   sh_f[f] = max_t (kept H)[t][f] / 448, sdz_f[f] = max_t |kept dZ[t][f]| / 448 over what the second mask kept;
 *   dW2 = bf16(sh_f[f] sdy_d[d] (H8c^T . dY8c));  dW1 = bf16(sx_d[d] sdz_f[f] (X8c^T . dZ8c)).
 * Outputs dX [T][D], dW1 [D][F], dW2 [F][D] are bf16 and overwritten.  Saved tensors afterwards: 2 dZ8r compressed [T][F/2] bytes,
 * 3 / 4 / 5 the transposed compressed operands (bytes), 13 sdz_t [T], 14 sh_f [F], 15 sdz_f [F] (fp32), 16 the bf16 compressed dZ
 * [T][F/2] before quantisation.  FFN24_ERR_STATE on any other context or before a forward.  ffn24_bwd refuses a row-wise context.
 * With FFN24_SPLIT and ffn24_set_split(n_dense > 0) (paper Sec. 2, "Optimization 1"): the n_dense least sparse features keep the
 * token-wise mask only in the two weight gradients; every feature's row of the transposed operands still has its own scale, taken
 * over what of the row enters the GEMM; the sparse features' rows are quantised in compressed form, the dense ones as plain rows,
 * and each weight gradient is one launch of a sparse and a dense fp8 GEMM.  The saved tensors 3 / 4 / 5 then hold the F - n_dense
 * sparse features in the row order of saved tensor 10, 14 and 15 the scales of all F rows in that order (sparse rows first), and
 * 20 / 21 the codes of the dense features' rows of the activation / of dZ. */
typedef struct {
  const void* dY8r;  const float* sdy_t;
  const void* dY8c;  const float* sdy_d;
  const void* X8c;   const float* sx_d;
  const void* W2_8r; const float* sw2_f;
  const void* W1_8c; const float* sw1_d;
} ffn24_rowwise_bwd_operands;
FFN24_API int ffn24_bwd_rowwise(ffn24_ctx* ctx, const ffn24_rowwise_bwd_operands* operands, void* dX, void* dW1, void* dW2, void* stream);
/* The dense baseline of ffn24_bwd_rowwise: the backward of ffn_fwd on an FFN24_FP8_E4M3 | FFN24_ROWWISE | FFN24_TRAINING |
 * FFN24_DENSE context (the paper's baseline recipe scales every FP8 GEMM row-wise), same operands, no masks:
 *   dH = sdy_t[t] sw2_f[f] (dY8r . W2_8r^T);  dZ = bf16(dH * 2 sqrt(h)) at every position, h the bf16 activation the forward kept;
 *   sdz_t[t] = max_f |dZ| / 448;  dX = bf16(sdz_t[t] sw1_d[d] (e4m3(dZ / sdz_t) . W1_8c^T));
 *   sh_f[f] = max_t h / 448, sdz_f[f] = max_t |dZ| / 448;  dW2 = bf16(sh_f[f] sdy_d[d] (e4m3(H / sh_f)^T . dY8c));
 *   dW1 = bf16(sx_d[d] sdz_f[f] (X8c^T . e4m3(dZ / sdz_f))).
 * Saved tensors afterwards: 8 e4m3(dZ / sdz_t) [T][F] bytes, 13 sdz_t, 14 sh_f, 15 sdz_f, 17 the bf16 dZ [T][F], 18 / 19 the codes of
 * the transposed activation and of the transposed dZ [F][T].  ffn_bwd refuses a row-wise context. */
FFN24_API int ffn_bwd_rowwise(ffn24_ctx* ctx, const ffn24_rowwise_bwd_operands* operands, void* dX, void* dW1, void* dW2, void* stream);

/* Fixed token permutation around the FFN (paper Sec. 2, "Optimization 2": features are correlated among consecutive
 * tokens, so the tokens are permuted before entering the FFN and shuffled back after).  perm_host is a HOST array
 * [T]: position p inside the FFN holds token perm_host[p].  It is checked here (FFN24_ERR_SHAPE unless it is a
 * permutation of 0..T-1) and copied to the device synchronously (the call waits for the device); NULL switches the
 * permutation off.  Afterwards ffn24_fwd / ffn24_bwd still take and return X, Y, dY, dX in token order: the rows of X
 * and dY are gathered by the operand DMA of the GEMMs that read them and the rows of Y and dX are scattered by the
 * epilogues of the GEMMs that produce them, so no extra pass over any tensor is made.  Inside, every saved tensor is in
 * permuted token order, and the feature-wise 2:4 groups of the weight gradients are made of the tokens the permutation
 * puts side by side.  Needs FFN24_PERMUTE (bf16 contexts, T d_model < 2^31; row-wise fp8 contexts, T d_model < 2^32, where
 * ffn24_fwd / ffn24_bwd_rowwise also bring the caller's per-token scales sx and sdy_t into that order; a per-tensor fp8 context
 * has no permutation: FFN24_ERR_DTYPE at creation). */
FFN24_API int ffn24_set_token_permutation(ffn24_ctx* ctx, const int32_t* perm_host);

/* Split of the weight-gradient GEMMs (paper Sec. 2, "Optimization 1"): some hidden features are too dense to be
 * 2:4-sparsified along tokens, so the n_dense least sparse features are kept out of the feature-wise pruning.
 * With n_dense > 0, ffn24_fwd also counts, per feature, the non-zero activations before pruning (in the up-projection's
 * epilogue), and ffn24_bwd partitions the features (the n_dense largest counts, ties to the lower index, are "dense"),
 * computes the rows of dW2 and the columns of dW1 of the dense features with dense GEMMs over the token-wise-pruned
 * activation, and all others with the sparse GEMMs as before.  n_dense is a multiple of 256, 0 <= n_dense <= F / 4
 * (0 = no split, the default).  Needs FFN24_SPLIT | FFN24_TRAINING; call it before the forward it shall apply to.
 * Saved tensors 9 (the counts, [F] uint32) and 10 (feature of each operand row, [F] int32: sparse features first,
 * then the dense ones, each in ascending order) are valid after the backward.  bf16 contexts take it with ffn24_bwd, row-wise fp8
 * contexts with ffn24_bwd_rowwise (see there); a per-tensor fp8 context has no split. */
FFN24_API int ffn24_set_split(ffn24_ctx* ctx, int64_t n_dense);

/* Free the workspace.  The caller must have synchronised every stream that used the context.  NULL is allowed. */
FFN24_API int ffn24_ctx_destroy(ffn24_ctx* ctx);

/* Standalone 2:4 compression along the columns (paper Sec. 2, first paragraph: keep the 2 largest magnitudes of
 * each block of 4).   H [rows][cols] -> values [rows][cols/2], meta [rows][cols/8].
 * dtype is the element type of H and of values: FFN24_BF16 (cols a multiple of 8), or FFN24_FP8_E4M3 (bytes; the pick is
 * made on the codes with the sign bit cleared, as integers; cols a multiple of 16, meta 16-byte aligned too).
 * rows >= 0 (rows == 0 is a no-op).  Signed inputs are allowed. */
FFN24_API int sparsify24(const void* H, int64_t rows, int64_t cols, ffn24_dtype dtype, void* values, uint8_t* meta, void* stream);

/* Sparsification and FP8 quantisation in one pass (paper Sec. 2, the second of the forward's kernels: activation, then
 * sparsification, then FP8 quantisation; the activation is already applied to H here).  H [rows][cols] bf16; the pick
 * is made on the bf16 words as in sparsify24; values8 [rows][cols/2] receives e4m3(kept / scale), saturating at +-448,
 * round to nearest even; meta [rows][cols/8].  scale > 0; cols a multiple of 8.  Moves 2.625 bytes per element. */
FFN24_API int sparsify24_quantise(const void* H, int64_t rows, int64_t cols, float scale, void* values8, uint8_t* meta, void* stream);

/* Feature-wise 2:4 on top of the token-wise one (paper Sec. 2, last paragraph, and Fig. 2c): the operand of a
 * GEMM that reduces over tokens must be 2:4 along tokens.  From the token-wise compressed activation
 * Hc [T][F/2] + meta [T][F/8] build, for each feature and each 4 consecutive tokens, the top-2 of the already
 * pruned activation:  Hc_t [F][T/2], meta_t [F][T/8].  If dZc (same shape and metadata as Hc) is given, dZc_t
 * [F][T/2] receives dZ at the positions picked for H; dZc and dZc_t may both be NULL.
 * T must be a multiple of 128, F a multiple of 64. */
FFN24_API int sparsify24_featurewise(const void* Hc, const uint8_t* meta, const void* dZc, int64_t T, int64_t F,
                           void* Hc_t, uint8_t* meta_t, void* dZc_t, void* stream);

/* C [M][N] = A24 . B on the sparse matrix cores (paper Sec. 1: a 2:4 operand lets the hardware skip half the
 * multiplications; Fig. 2b).  A24 is given compressed along K: values [M][K/2], meta [M][K/8].
 * B is given transposed, Bt [N][K] (K contiguous, like A).  M, N multiples of 256, K a multiple of 64. */
FFN24_API int spmm24(const void* values, const uint8_t* meta, const void* Bt, int64_t M, int64_t N, int64_t K, void* C,
                     void* stream);

/* Weights that stay the same over many calls (inference; the micro-batches of one optimizer step): runs the weight
 * pass of the forward calls once -- W1 [D][F] and W2 [F][D] are re-arranged into the context's workspace -- after
 * which ffn24_fwd and ffn_fwd accept W1 == NULL and W2 == NULL, meaning "the prepared weights", and skip that pass.
 * A forward call that is given weights runs the pass itself and drops the prepared state.  The context holds its own
 * copies: W1 and W2 need not outlive the call's work on the stream. */
FFN24_API int ffn24_prepare_weights(ffn24_ctx* ctx, const void* W1, const void* W2, void* stream);

/* Forward of the 2:4 FFN (paper Sec. 2):  Z = X W1 + b1;  H = bf16(max(0, Z)^2);  H24 = keep-2-of-4 of H along
 * the hidden features of each token;  Y = H24 W2.
 *   X [T][D], W1 [D][F], b1 [F] fp32 or NULL (the paper's FFN has no bias; b1 only dials the sparsity of synthetic
 *   inputs), W2 [F][D], Y [T][D].  W1 and W2 both NULL: the weights of ffn24_prepare_weights (FFN24_ERR_STATE if none).
 * Kernels: two weight transposes (every GEMM operand is consumed K-contiguous), the dense-MFMA up-projection with
 * the activation and the pruning fused into its epilogue (H is never written densely), the sparse-MFMA
 * down-projection.  The context keeps (Hc, meta), its own re-arranged copies of W1 and W2 and the X pointer for
 * ffn24_bwd; the caller keeps X alive and unchanged until then. */
FFN24_API int ffn24_fwd(ffn24_ctx* ctx, const void* X, const void* W1, const float* b1, const void* W2, void* Y, void* stream);

/* ffn24_fwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same forward (bf16, same kernels, bit-identical Y) without a context.  The
 * intermediate tensors -- the compressed activation and the two re-arranged weights, T F + T F / 8 + 4 D F bytes, which
 * ffn24_ctx_create would allocate -- live in a static device array of FFN24_STATIC_SCRATCH_BYTES inside the library, of
 * which every GPU that loads the library holds one copy until the process ends.  The call allocates and frees nothing
 * and calls no allocating routine; it only enqueues four kernels on `stream`.
 *   X [T][D], W1 [D][F], b1 [F] fp32 or NULL, W2 [F][D], Y [T][D]: device pointers, bf16, caller-owned as everywhere.
 *   T, D, F multiples of 256.  FFN24_ERR_SCRATCH if ffn24_static_scratch_needed(T, D, F) exceeds the buffer (use a
 *   context then); the other error codes as for ffn24_fwd.
 * All calls on one GPU share that GPU's buffer: two calls whose work overlaps in time on one GPU (different streams,
 * or different threads) race on it.  Calls on one stream are ordered and safe.  Nothing in the buffer has to start at
 * zero -- each call writes every byte it later reads -- so it is never cleared.  Inference only: nothing is kept for
 * a backward pass.  The first call on a device looks up the buffer's address and sets kernel attributes: make one call
 * before recording calls into a graph. */
#define FFN24_STATIC_SCRATCH_BYTES (64u << 20)
FFN24_API int64_t ffn24_static_scratch_needed(int64_t T, int64_t D, int64_t F);   /* bytes, or -1 for sizes out of range */
FFN24_API int ffn24_fwd_static(const void* X, const void* W1, const float* b1, const void* W2, void* Y, int64_t T, int64_t D, int64_t F,
                               void* stream);

/* Backward of the last ffn24_fwd on this context, masks held fixed (paper Fig. 4 and Sec. 2, backward paragraphs):
 *   dZ  = (dY W2^T) * 2 max(0, Z) on the kept positions        dense GEMM, derivative taken as 2 sqrt(H)
 *   dX  = dZ24 W1^T                                            sparse GEMM (token-wise mask)
 *   dW2 = (H24 * M_T)^T dY,   dW1 = X^T (dZ24 * M_T)           sparse GEMMs; M_T = feature-wise mask on top
 *   dY [T][D] -> dX [T][D], dW1 [D][F], dW2 [F][D].
 * Needs FFN24_TRAINING.  Returns FFN24_ERR_STATE unless the last forward on this context was an ffn24_fwd (ffn24_fwd
 * and ffn_fwd share the context's weight workspace, so each invalidates what the other saved). */
FFN24_API int ffn24_bwd(ffn24_ctx* ctx, const void* dY, void* dX, void* dW1, void* dW2, void* stream);

/* Dense Squared-ReLU FFN on the same GEMM core (paper Sec. 1, "Squared ReLU"): the speed-up baseline.
 * Y = bf16(max(0, X W1 + b1)^2) W2.  Needs FFN24_DENSE. */
FFN24_API int ffn_fwd(ffn24_ctx* ctx, const void* X, const void* W1, const float* b1, const void* W2, void* Y, void* stream);

/* Backward of the last ffn_fwd: dZ = (dY W2^T) * 2 sqrt(H); dX = dZ W1^T; dW2 = H^T dY; dW1 = X^T dZ.
 * Needs FFN24_DENSE | FFN24_TRAINING.  Returns FFN24_ERR_STATE unless the last forward on this context was an ffn_fwd. */
FFN24_API int ffn_bwd(ffn24_ctx* ctx, const void* dY, void* dX, void* dW1, void* dW2, void* stream);

/* Sparsity telemetry of a context created with FFN24_TELEMETRY (bf16 only; paper Sec. 1: the sparsity level of the
 * activation over training, Sec. 2: the share of non-zero values that 2:4 drops).  The up-projection epilogues of
 * ffn24_fwd and ffn_fwd and the feature-wise re-compression of ffn24_bwd count while they work; each of these three
 * calls ends by enqueuing a snapshot (a 40-byte copy to pinned host memory plus an event record, so such calls
 * cannot be recorded into a HIP graph).  counts[0..4]:
 *   0  T F                                                 1  non-zero stored activations before pruning
 *   2  of those, kept by the token-wise 2:4                 3  of those, still seen by the weight-gradient GEMMs
 *   4  1 if the snapshot comes from the 2:4 path, 0 from ffn_fwd (then 2 and 3 are 0)
 * Entry 3 is 0 in the snapshot of a forward and filled in by the backward's.  With FFN24_SPLIT the dense features
 * count in full in entry 3.  wait != 0: blocks until the newest snapshot has landed.  wait == 0: never blocks; returns
 * the newest snapshot that has landed, or FFN24_ERR_NOTREADY if none has. */
FFN24_API int ffn24_get_telemetry(ffn24_ctx* ctx, int64_t* counts, int wait);

/* The dense <-> 2:4 switch behind the paper's dense warm-up (Sec. 2, last paragraph: the activation is only about
 * half zeros at initialisation and reaches 90 % and more after a short while).  *use_sparse = 1 iff the newest landed
 * snapshot shows a share of zeros, 1 - counts[1] / counts[0], of at least min_sparsity (0..1); 0 while nothing has
 * been measured.  Never blocks: the decision for a step rests on an earlier step's measurement.  The caller then
 * runs ffn24_fwd / ffn24_bwd or ffn_fwd / ffn_bwd (a context with FFN24_DENSE | FFN24_TRAINING has both). */
FFN24_API int ffn24_policy_use_sparse(ffn24_ctx* ctx, double min_sparsity, int* use_sparse);

/* Copies of the context's saved tensors, for parity checks.  `which`:
 *   0 Hc [T][F/2]   1 meta [T][F/8]   2 dZc [T][F/2]   3 Hc_t [F][T/2]   4 meta_t [F][T/8]   5 dZc_t [F][T/2]
 *   6 pre-prune H dump [T][F] (FFN24_DEBUG_DUMP_H)   7 dense H [T][F]   8 dense dZ [T][F]
 *   9 per-feature non-zero counts [F] uint32, 10 feature of each split-operand row [F] int32 (FFN24_SPLIT)
 *   11 per-token activation scale sh [T] fp32 (FFN24_ROWWISE)
 *   12 kept activation before quantisation [T][F/2] bf16 (fp8 contexts with FFN24_TRAINING or FFN24_ROWWISE)
 *   13 sdz_t [T], 14 sh_f [F], 15 sdz_f [F] fp32 and 16 the compressed dZ before quantisation [T][F/2] bf16 (after ffn24_bwd_rowwise)
 *   17 the dense dZ before quantisation [T][F] bf16, 18 / 19 the codes of the transposed dense activation / dZ [F][T] (after ffn_bwd_rowwise;
 *   18 / 19 also after ffn_bwd on an fp8 context)
 *   20 / 21 the rows of the split's dense features [F/4][T], activation / dZ, of which the first n_dense are valid (bf16, or e4m3
 *   codes after ffn24_bwd_rowwise; FFN24_SPLIT)
 * ffn24_saved_bytes gives the size of tensor `which`; ffn24_copy_saved enqueues a copy of it into dst (device memory
 * of exactly that size, 16-byte aligned) in the row-major compressed form described at the top -- inside the context
 * the compressed tensors are kept in a tiled order that the sparse GEMM streams faster.  Returns FFN24_ERR_STATE if
 * the context was created without the flag that owns the tensor, FFN24_ERR_SHAPE on a size mismatch. */
FFN24_API int ffn24_saved_bytes(ffn24_ctx* ctx, int which, int64_t* nbytes);
FFN24_API int ffn24_copy_saved(ffn24_ctx* ctx, int which, void* dst, int64_t dst_bytes, void* stream);

/* Per-kernel timing with HIP events recorded on the stream each kernel is launched on.
 * ffn24_set_profiling(ctx, 1) makes every later call bracket each of its kernels with an event pair;
 * ffn24_kernel_ms(ctx, k, &ms) waits for kernel k's events of the most recent call and returns its duration.
 * Kernel ids: 0 up-projection+prune, 1 sparse down-projection, 2 dH+derivative, 3 sparse dX, 4 feature-wise
 * re-compression, 5 sparse dW2, 6 sparse dW1, 7..12 the six dense-baseline GEMMs in the same order
 * (up, down, dH, dX, dW2, dW1), 13 the weight pass of a forward or of ffn24_prepare_weights (W1, W2 re-arranged), 14 the two
 * activation transposes of a backward (dY, X), 15 the feature partition of the split, 16 the transpose that brings
 * dW1 into [D][F] after a split (with a split, 5 and 6 are the combined sparse + dense launches of dW2 and dW1),
 * 17 the row-wise fp8 quantisation kernel of a forward, 18 the one of dZ in ffn24_bwd_rowwise, 19 its two quantisations of the
 * transposed operands, 20 its re-arrangement of the caller's W2_8r and dY8r (ffn_bwd_rowwise: also W1_8c) into the forms the GEMMs stream, 21 the same for
 * X8 in the forward of an fp8 context.  Returns FFN24_ERR_STATE if that kernel has not run
 * with profiling on. */
FFN24_API int ffn24_set_profiling(ffn24_ctx* ctx, int on);
FFN24_API int ffn24_kernel_ms(ffn24_ctx* ctx, int kernel, float* ms);
/* The shader clock (MHz) GEMM kernel `kernel` of the most recent profiled call really ran at: the first 64 workgroups
 * each sample the shader-clock counter against the constant 100 MHz counter over their lifetime.  Under matrix load the
 * chip settles far below its nominal 2.4 GHz, which every fraction of the published peak has to be read against.
 * FFN24_ERR_STATE for the streaming kernels (they take no sample) or if the kernel has not run with profiling on. */
FFN24_API int ffn24_kernel_mhz(ffn24_ctx* ctx, int kernel, float* mhz);

/* Measurement probes (no paper passage: they measure the machine, for the benchmark's report).  Each allocates its own
 * device buffers, runs on the default stream and waits for its own work; not for serving code.
 *   ffn24_probe_mfma_rate: a register-resident loop of matrix instructions with no memory traffic, one wave per SIMD on
 *     every CU, pseudo-random operands.  kind 0 dense bf16 32x32x16, 1 sparse bf16 32x32x32, 2 dense fp8 32x32x64,
 *     3 sparse fp8 32x32x64; iters x 16 ops per wave.  Returns shader-clock cycles per op and wave, the clock (MHz) the
 *     loop ran at, and the chip-wide rate in dense-equivalent TFLOP/s (a sparse op counts its dense equivalent).
 *   ffn24_probe_gemm: the library's GEMM core (dense bf16 if sparse == 0, else 2:4 bf16; plain row-major epilogue) on
 *     pseudo-random operands, M, N multiples of 256, K a multiple of 128 and >= 512, with ingredients of its main loop
 *     taken out: variant 0 all of it, 1 no global->LDS DMA, 4 no LDS fragment reads, 6 DMA only (no matrix ops, no fragment reads),
 *     5 matrix ops only, 8 every K stage re-reads the first 8 stages (all L2 hits), 14 = 8 + 6; or the whole loop with
 *     another tile walk: 16 bands of 8 tile-rows per XCD, 32 the 8 per-XCD patches of a round side by side along M,
 *     64 patches of 4 x 8 tiles, 128 patches of 16 x 2 tiles (the product: a 4 x 2 grid of 8 x 4 patches); or, 256, with a
 *     stage's DMA instructions on consecutive matrix-op slots (the product issues them on every other slot); or, 512 (sparse only),
 *     with a quarter of every stage's operand bytes not fetched; or, 1024, as 256 persistent workgroups that walk the tiles and ask
 *     for a tile's first stages before the epilogue of the tile before.  Returns the median
 *     kernel duration over `reps` launches and the clock it ran at.  Variants other than 0 compute nothing meaningful.
 *   ffn24_probe_copy: a plain device-to-device copy kernel of `bytes` bytes (a multiple of 4096): median duration. */
FFN24_API int ffn24_probe_mfma_rate(int kind, int iters, double* cycles_per_op, double* mhz, double* tflops_dense_equivalent);
FFN24_API int ffn24_probe_gemm(int sparse, int variant, int64_t M, int64_t N, int64_t K, int reps, double* ms_median, double* mhz);
FFN24_API int ffn24_probe_copy(int64_t bytes, int reps, double* ms_median);

FFN24_API const char* ffn24_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* FFN24_H */
