/*
 * megatrain_kernels.h - C ABI of the individual gfx950 kernels behind the training step.
 *
 * These are the operations that make up f_i, the loss and LocalBackward of Algorithm 1
 * (MegaTrain, Sections 3.1 and 3.4: "stateless templates" that take the streamed weight
 * buffer as plain pointers at launch).  They are exported so that each kernel can be checked
 * against the CPU oracle and timed on its own.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless its name starts with "host_".
 *   - bf16 tensors are raw uint16_t bit patterns; "ld*" are leading dimensions in ELEMENTS.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; the caller synchronises.
 *   - bf16 pointers must be 16-byte aligned and leading dimensions multiples of 8 unless
 *     stated otherwise; violations return MT_ERR_INVALID_ARG before anything is launched.
 *   - Return value: mt_status as in megatrain.h.
 */
#ifndef MEGATRAIN_KERNELS_H_
#define MEGATRAIN_KERNELS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] = A[M,K] . B[N,K]^T with fp32 accumulation on the matrix cores.
 * A [M,K] bf16 (lda), B [N,K] bf16 (ldb), K % 8 == 0.
 * out_fp32 == 0: C bf16 [M,N] (ldc); if R != NULL, R bf16 [M,N] (ldr) is added before rounding
 *                (the residual connection of the block).
 * out_fp32 == 1: C fp32 [M,N] (ldc); accumulate != 0 adds to the existing C (weight gradients
 *                of the LM head summed over token chunks).  R must be NULL. */
int32_t mt_k_gemm_nt(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, void *C, int64_t ldc,
                     const uint16_t *R, int64_t ldr, int32_t M, int32_t N, int32_t K, int32_t out_fp32,
                     int32_t accumulate, void *stream);

/* C[M,N] bf16 = A . B^T + bias (bias bf16 [N], 8-byte aligned, added to every row before rounding): the q, k, v
 * projections of layers with biases. */
int32_t mt_k_gemm_nt_bias(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, uint16_t *C, int64_t ldc,
                          const uint16_t *bias, int32_t M, int32_t N, int32_t K, void *stream);
/* The q, k, v projection of a block (Section 3.2, layer forward) with the rotary embedding applied in the store:
 * C[M,N] bf16 = A . B^T (+ bias if not NULL), then in columns [0, rope_cols) every head of 128 columns has its
 * pairs (j, j + 64) rotated by the angle of position (row % T); tables cos/sin [T, 64] fp32 from mt_k_rope_table,
 * 16-byte aligned.  Only for large grids (at least 192 tiles of 256 x 256), K % 64 == 0, N % 128 == 0,
 * rope_cols % 128 == 0: MT_ERR_UNSUPPORTED otherwise (use mt_k_gemm_nt_bias / mt_k_gemm_nt, then mt_k_rope). */
int32_t mt_k_gemm_nt_rope(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, uint16_t *C, int64_t ldc,
                          const uint16_t *bias, const float *cos_tab, const float *sin_tab, int32_t T,
                          int32_t rope_cols, int32_t M, int32_t N, int32_t K, void *stream);
/* The gate|up projection of a block's MLP with the activation computed in the store: W [2F, K] bf16 holds the gate
 * rows then the up rows; s [M, F] bf16 (lds) = silu(gate) * up from the bf16-rounded gate and up, exactly what
 * mt_k_gemm_nt into gu followed by mt_k_swiglu_fwd gives; gu [M, 2F] bf16 (ldgu) receives gate | up unless it is
 * NULL.  Only for large grids (at least 192 tiles of 256 x 256 over M x 2F), K % 64 == 0, F % 128 == 0:
 * MT_ERR_UNSUPPORTED otherwise. */
int32_t mt_k_gemm_nt_swiglu(const uint16_t *A, int64_t lda, const uint16_t *W, int64_t ldw, uint16_t *gu, int64_t ldgu,
                            uint16_t *s, int64_t lds, int32_t M, int32_t F, int32_t K, void *stream);
/* The input gradient of the MLP's down projection with the SwiGLU backward applied in the store: ds = A . B^T
 * ([M,F], rounded to bf16), then dgu [M, 2F] (lddgu) = dgate | dup from ds and the forward's gate | up in gu [M, 2F]
 * (ldgu): exactly what mt_k_gemm_nt into ds followed by mt_k_swiglu_bwd gives.  Only for large grids (at least 192
 * tiles of 256 x 256), K % 64 == 0, F % 8 == 0, 16-byte aligned gu and dgu: MT_ERR_UNSUPPORTED otherwise. */
int32_t mt_k_gemm_nt_swiglu_bwd(const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb, uint16_t *dgu, int64_t lddgu,
                                const uint16_t *gu, int64_t ldgu, int32_t M, int32_t F, int32_t K, void *stream);
/* Weight-gradient form: C[M,N] fp32 = At^T . Bt with At [K, M] bf16 (lda) and Bt [K, N] bf16 (ldb), both
 * token-major as the other kernels leave them (dW = dY^T X); accumulate != 0 adds to the existing C.
 * Requires K % 64 == 0, M % 8 == 0, N % 8 == 0: MT_ERR_UNSUPPORTED otherwise (transpose and use mt_k_gemm_nt). */
int32_t mt_k_gemm_tn(const uint16_t *At, int64_t lda, const uint16_t *Bt, int64_t ldb, float *C, int64_t ldc, int32_t M,
                     int32_t N, int32_t K, int32_t accumulate, void *stream);
/* The same product with the reduction over K cut into split_k chunks that run as separate workgroups, for outputs
 * whose tile count fills the last round of workgroups badly: chunk 0 writes C, chunk s > 0 a slice of ws (device,
 * at least (split_k - 1) * M * N floats, 16-byte aligned), and a second kernel adds the slices to C in order, so the
 * result is deterministic.  1 <= split_k <= K / 64; split_k > 1 needs N % 4 == 0, ldc % 4 == 0 and a 16-byte aligned C.
 * mt_k_gemm_tn_pick_split returns the split the training step would choose on n_cu compute units. */
int32_t mt_k_gemm_tn_split(const uint16_t *At, int64_t lda, const uint16_t *Bt, int64_t ldb, float *C, int64_t ldc, int32_t M,
                           int32_t N, int32_t K, int32_t accumulate, int32_t split_k, float *ws, void *stream);
int32_t mt_k_gemm_tn_pick_split(int64_t M, int64_t N, int64_t K, int32_t n_cu);
/* db[cols] fp32 (written) = sum over the n rows of x [n, ld] bf16 (the gradient of such a bias); cols % 8 == 0;
 * ws: device scratch of at least mt_k_bias_grad_ws_bytes(cols) bytes.  Fixed summation order. */
size_t mt_k_bias_grad_ws_bytes(int32_t cols);
int32_t mt_k_bias_grad(float *db, const uint16_t *x, int64_t ld, int64_t n, int32_t cols, void *ws, void *stream);

/* out[b0][b1][c][r] = in[b0][b1][r][c], bf16; rows, cols multiples of 8; batch strides in elements. */
int32_t mt_k_transpose(const uint16_t *in, uint16_t *out, int32_t rows, int32_t cols, int64_t ld_in, int64_t ld_out,
                       int32_t nb0, int32_t nb1, int64_t in_s0, int64_t in_s1, int64_t out_s0, int64_t out_s1,
                       void *stream);

/* y = x / sqrt(mean(x^2) + eps) * gain, rows of length d (d % 8 == 0, d <= 8192), contiguous. */
int32_t mt_k_rmsnorm_fwd(uint16_t *y, const uint16_t *x, const uint16_t *gain, int64_t n, int32_t d, float eps,
                         void *stream);

/* dx = dres + dRMSNorm(dy; x, gain) (dres may be NULL), dgain[d] fp32 = sum over rows (written).
 * ws: device scratch of at least mt_k_rmsnorm_bwd_ws_bytes(d) bytes. */
size_t mt_k_rmsnorm_bwd_ws_bytes(int32_t d);
int32_t mt_k_rmsnorm_bwd(uint16_t *dx, float *dgain, const uint16_t *dy, const uint16_t *x, const uint16_t *gain,
                         const uint16_t *dres, void *ws, int64_t n, int32_t d, float eps, void *stream);

/* mt_k_rmsnorm_bwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments without ws, same results bit for bit.  The per-block
 * partial gain gradients go to a device array that is part of the library image (512 * 8192 floats = 16 MiB on
 * every device the library runs on, held until the process ends); its address is looked up once per device at the
 * first call there.  The call allocates nothing.  d <= MT_K_RMSNORM_BWD_NOALLOC_MAX_D, otherwise MT_ERR_UNSUPPORTED
 * and nothing is launched.  All calls on one device share the array: calls that overlap on one device (different
 * streams or threads) race; calls on one stream are ordered and safe.  Nothing in it needs to start at zero. */
#define MT_K_RMSNORM_BWD_NOALLOC_MAX_D 8192
int32_t mt_k_rmsnorm_bwd_noalloc(uint16_t *dx, float *dgain, const uint16_t *dy, const uint16_t *x, const uint16_t *gain,
                                 const uint16_t *dres, int64_t n, int32_t d, float eps, void *stream);

/* Fill cos/sin tables [T, hd/2] fp32 on the HOST: angle = t * base^(-2j/hd), computed in double. */
int32_t mt_k_rope_table(float *host_cos, float *host_sin, int32_t T, int32_t hd, double base);
/* Rotate in place the first n_heads heads (hd wide, hd % 16 == 0) of every row of x [n, ld];
 * the position of row r is r % T; sign = +1 forward, -1 inverse (the backward map). */
int32_t mt_k_rope(uint16_t *x, int64_t ld, int64_t n, int32_t T, int32_t n_heads, int32_t hd, const float *cos_tab,
                  const float *sin_tab, int32_t sign, void *stream);

/* gu [n, 2F] holds gate in columns [0,F) and up in [F,2F).  s = silu(gate) * up, [n,F]. */
int32_t mt_k_swiglu_fwd(uint16_t *s, const uint16_t *gu, int64_t n, int32_t F, void *stream);
/* dgu [n,2F] = (dgate | dup) from ds [n,F] and gu. */
int32_t mt_k_swiglu_bwd(uint16_t *dgu, const uint16_t *ds, const uint16_t *gu, int64_t n, int32_t F, void *stream);

/* h[r,:] = table[tokens[r],:] */
int32_t mt_k_embed_gather(uint16_t *h, const uint16_t *table, const int32_t *tokens, int64_t n, int32_t d,
                          void *stream);
/* dtable [V,d] fp32, every row written: row v = sum of dh[order[i],:] for i in [row_start[v], row_start[v+1]),
 * added in that order (deterministic).  row_start has V+1 entries. */
int32_t mt_k_embed_scatter(float *dtable, const uint16_t *dh, const int32_t *row_start, const int32_t *order,
                           int32_t V, int32_t d, void *stream);

/* Per row r of logits fp32 [n,V] (V % 4 == 0): loss_rows[r] = logsumexp(z_r) - z_r[label_r];
 * dlogits bf16 [n,V] = (softmax(z_r) - onehot(label_r)) * inv_n.  A negative label gives a zero
 * loss and a zero gradient row. */
int32_t mt_k_cross_entropy(float *loss_rows, uint16_t *dlogits, const float *logits, const int32_t *labels, int64_t n,
                           int32_t V, float inv_n, void *stream);
/* out[0] = (accumulate ? out[0] : 0) + scale * sum(in[0..n)), fixed summation order. */
int32_t mt_k_reduce_sum(float *out, const float *in, int64_t n, float scale, int32_t accumulate, void *stream);

/* Causal attention forward.  Rows of q/k/v/o are tokens (b*T + t); head h occupies columns
 * [h*hd, (h+1)*hd) after the given pointer.  hd in {64, 128}, T % 8 == 0, Hq % Hkv == 0; query head h
 * reads KV head h / (Hq/Hkv).  o bf16, lse fp32 [B, Hq, T] = log sum_u exp(q_t.k_u * scale). */
int32_t mt_k_flash_fwd(uint16_t *o, int64_t ldo, float *lse, const uint16_t *q, int64_t ldq, const uint16_t *k,
                       int64_t ldk, const uint16_t *v, int64_t ldv, int32_t B, int32_t T, int32_t Hq, int32_t Hkv,
                       int32_t hd, float scale, void *stream);
/* Causal attention backward: dq, dk, dv from dout, the forward's inputs, o and lse.  dk, dv of a KV head are
 * summed over the query heads of its group.  delta [B,Hq,T] fp32 is scratch written by this call
 * (delta = rowsum(dout * o)).  Deterministic: no atomics. */
int32_t mt_k_flash_bwd(uint16_t *dq, int64_t lddq, uint16_t *dk, int64_t lddk, uint16_t *dv, int64_t lddv,
                       const uint16_t *dout, int64_t lddo, const uint16_t *q, int64_t ldq, const uint16_t *k,
                       int64_t ldk, const uint16_t *v, int64_t ldv, const uint16_t *o, int64_t ldo, const float *lse,
                       float *delta, int32_t B, int32_t T, int32_t Hq, int32_t Hkv, int32_t hd, float scale,
                       void *stream);

/* The same with the backward of a rotary embedding folded into the stores: q and k are the rotated tensors the
 * forward attended with, and dq, dk come out as gradients of the unrotated ones (rotated back by the angle of
 * position t; pairs (j, j + hd/2)); tables cos/sin [T, hd/2] fp32, 16-byte aligned.  Equal to mt_k_flash_bwd
 * followed by mt_k_rope(sign = -1) on dq and dk, without the extra rounding to bf16 in between. */
int32_t mt_k_flash_bwd_rope(uint16_t *dq, int64_t lddq, uint16_t *dk, int64_t lddk, uint16_t *dv, int64_t lddv,
                            const uint16_t *dout, int64_t lddo, const uint16_t *q, int64_t ldq, const uint16_t *k,
                            int64_t ldk, const uint16_t *v, int64_t ldv, const uint16_t *o, int64_t ldo,
                            const float *lse, float *delta, const float *cos_tab, const float *sin_tab, int32_t B,
                            int32_t T, int32_t Hq, int32_t Hkv, int32_t hd, float scale, void *stream);

/* Host Adam on one array (the arithmetic of mt_adam_step; all HOST pointers).  shadow may be
 * NULL, otherwise it receives the updated parameters rounded to bf16 (nearest even). */
int32_t mt_k_host_adam(float *host_p, const float *host_g, float *host_m, float *host_v, uint16_t *host_shadow,
                       size_t n, float lr, float beta1, float beta2, float eps, float wd, int64_t step);
/* fp32 -> bf16 round-to-nearest-even on the host (the conversion applied to streamed weights). */
int32_t mt_k_host_f32_to_bf16(uint16_t *host_out, const float *host_in, size_t n);

#ifdef __cplusplus
}
#endif
#endif /* MEGATRAIN_KERNELS_H_ */
