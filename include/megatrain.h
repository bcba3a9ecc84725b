/*
 * megatrain.h - C ABI of the MI355X (gfx950) streamed training step.
 *
 * One handle owns one decoder-only transformer whose persistent training state lives in
 * HOST memory (MegaTrain, Section 3.1: parameters, gradients and Adam moments stay on the
 * host; the device is a transient execution cache).  A training step follows the paper's
 * Algorithm 1 "MegaTrain Training Step" with one transformer block per recomputation block
 * (checkpoint interval K = 1):
 *
 *   Phase 1  streaming forward:  for each unit (embedding, block 1..L) StreamIn its bf16
 *            weights into one of two device buffers, compute, keep only h_0..h_L in HBM.
 *   Phase 2  loss anchoring:     final norm + LM head + mean cross-entropy, head gradients.
 *   Phase 3  block-wise backward: for i = L..1 StreamIn theta_i again, recompute block i
 *            from h_{i-1} (except the last checkpoint block, whose internals the forward has
 *            just left in the work buffers), LocalBackward, Offload the fp32 gradients to the host while the
 *            next block's weights stream in (Section 3.2: three streams, double buffering,
 *            Weights-Ready / Backward-Done / Buffer-Free events).
 *   last     AdamUpdate on the host CPU (Section 3.1, optimizer update phase).
 *
 * Conventions
 *   - Every pointer in this header is a HOST pointer.  Device memory, streams and events
 *     are created and owned by the library.
 *   - All functions return mt_status (0 = MT_OK, negative = error) and never abort or
 *     throw.  After an error the handle can still be destroyed; outputs are unspecified.
 *     mt_last_error() gives a human-readable message for the calling thread.
 *   - One handle must be used by one thread at a time.
 *   - Environment (read once): MT_HOST_THREADS = threads of the host Adam / conversion loops (default: all
 *     cores); MT_PINNED_BUDGET_GB = pinned host memory the library may take before it switches to the
 *     gradient slab pool (default 56); MT_PROGRESS=1 prints one line to stderr whenever the GPU finishes a
 *     unit of a step (for steps that run for minutes); MT_GEMM_VARIANT forces one GEMM kernel, MT_GROUP_M the
 *     tile-row group of the large-grid GEMM kernels' tile order (diagnostics);
 *     MT_SUBPIECE_ELEMS (read at every step) = elements per sub-range in which mt_train_step_adam copies and
 *     updates a large gradient piece (default 16 Mi; tests use small values to cut through tensors).
 *
 * Canonical tensor order (index -> tensor), all fp32, row-major, matrices stored
 * [out_features, in_features] like a linear layer's weight:
 *     0                 embed      [vocab, hidden]
 *     1 + 9 l + 0       attn_norm  [hidden]                    (l = 0 .. n_layers-1)
 *     1 + 9 l + 1       wq         [n_q_heads*head_dim, hidden]
 *     1 + 9 l + 2       wk         [n_kv_heads*head_dim, hidden]
 *     1 + 9 l + 3       wv         [n_kv_heads*head_dim, hidden]
 *     1 + 9 l + 4       wo         [hidden, n_q_heads*head_dim]
 *     1 + 9 l + 5       mlp_norm   [hidden]
 *     1 + 9 l + 6       w_gate     [ffn, hidden]
 *     1 + 9 l + 7       w_up       [ffn, hidden]
 *     1 + 9 l + 8       w_down     [hidden, ffn]
 *     1 + 9 L           final_norm [hidden]
 *     2 + 9 L           lm_head    [vocab, hidden]
 * With cfg.tie_embeddings = 1 the list ends with final_norm (index 1 + 9 L) and tensor 0 is also the head.
 * With cfg.qkv_bias = 1 a layer has 12 tensors (replace 9 by 12 above) and
 *     1 + 12 l + 9      bq         [n_q_heads*head_dim]
 *     1 + 12 l + 10     bk         [n_kv_heads*head_dim]
 *     1 + 12 l + 11     bv         [n_kv_heads*head_dim]
 * The block is pre-norm: RMSNorm -> q,k,v projections -> rotary embedding (pairs
 * (j, j + head_dim/2), angle t * rope_base^(-2j/head_dim)) -> causal softmax attention with
 * scale 1/sqrt(head_dim), query head h reading KV head h / (n_q_heads/n_kv_heads) ->
 * output projection + residual -> RMSNorm -> SwiGLU MLP + residual.  No biases, except the optional
 * q, k, v biases (added before the rotary embedding).
 */
#ifndef MEGATRAIN_H_
#define MEGATRAIN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mt_handle mt_handle; /* opaque */
typedef int32_t mt_status;

#define MT_OK 0
#define MT_ERR_INVALID_ARG (-1) /* null pointer, bad struct size, non-positive dimension        */
#define MT_ERR_UNSUPPORTED (-2) /* valid request this build does not implement                   */
#define MT_ERR_HOST_OOM (-3)    /* a host allocation (pinned or pageable) failed                 */
#define MT_ERR_DEVICE_OOM (-4)  /* the device arena does not fit (HBM or max_device_bytes)       */
#define MT_ERR_HIP (-5)         /* a HIP runtime call or kernel launch failed                    */
#define MT_ERR_SHAPE (-6)       /* batch/seq outside what the handle was created for             */
#define MT_ERR_TOKEN_RANGE (-7) /* token < 0 or >= vocab, or label >= vocab                      */
#define MT_ERR_STATE (-8)       /* call out of order (e.g. Adam before any training step)        */

#define MT_ABI_VERSION 2

/* diagnostic flags (mt_model_cfg.flags) */
#define MT_FLAG_SERIAL 1u       /* no overlap: every copy and every unit is followed by a device sync.
                                   The "without double buffering" point of the paper's ablation (Table 4). */
#define MT_FLAG_COMPUTE_ONLY 2u /* weights are streamed once at create-time granularity: per-unit H2D and
                                   D2H copies are skipped inside the step (gradients stay on the device).
                                   For timing the compute stream alone; results on the host are stale. */
#define MT_FLAG_COPY_ONLY 4u    /* only the copies of a step are issued, no kernels. For timing the link. */
#define MT_FLAG_GRAD_SLABS 16u   /* force the gradient slab pool (Section 3.3): gradient blocks in pageable memory, device-to-host
                                   copies through 4 recycled pinned slabs folded in by a host thread.  Chosen automatically
                                   when pinning every gradient block would exceed the pinned-memory budget (56 GiB, or
                                   MT_PINNED_BUDGET_GB in the environment). */
#define MT_FLAG_STAGED_WEIGHTS 32u /* no persistent pinned bf16 copy of the weights (Section 3.3, pinned slab recycling): a host
                                  * thread converts the fp32 master tensors of the unit to be streamed next into one of three
                                  * pinned slabs of the largest unit's size, just in time; pinned host memory no longer grows
                                  * with the model.  Results are bit-identical to the default mode. */
#define MT_FLAG_KERNEL_TIMING 8u /* bracket every GEMM and attention launch with HIP events on the compute
                                   stream and report per-class time, FLOPs and launch counts in mt_stats */

typedef struct {
    uint32_t struct_size; /* sizeof(mt_model_cfg), checked */
    uint32_t abi_version; /* MT_ABI_VERSION, checked */
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t max_batch, max_seq; /* the device arena is sized once for max_batch*max_seq tokens */
    float rope_base, rms_eps;
    int32_t ckpt_interval; /* checkpoint interval K >= 1 of Algorithm 1 (values above n_layers act as n_layers):
                            * only h_0, h_K, h_2K, ... stay in device memory; the backward recomputes one block
                            * of K layers at a time (K activation sets) and streams its weights a third time */
    int32_t device_id;
    uint32_t flags;
    uint32_t qkv_bias; /* 1: every layer has bias vectors for the q, k and v projections (12 tensors per layer: the 9
                        * below, then bq, bk, bv); 0: none */
    uint64_t max_device_bytes; /* 0 = no cap; otherwise mt_create fails with MT_ERR_DEVICE_OOM above it */
    uint32_t tie_embeddings;   /* 1: the output projection reuses the embedding table (Appendix A.1, tied weights):
                                * the tensor list ends with final_norm (no lm_head); the table is streamed again for
                                * the loss, and its gradient is the head's weight gradient plus the embedding's
                                * scatter-add, summed on the host */
    uint32_t mlp_chunk;        /* 0: the MLP of a block runs on all tokens at once.  m > 0 (multiple of 8): it runs in chunks of m
                                * tokens (chunked MLP of the long-context runs, Section 4.6): gate/up/activation buffers are chunk-sized, nothing of
                                * the MLP is saved, and the backward recomputes each chunk right before differentiating it
                                * (same FLOPs: the block recomputation then skips the MLP) */
} mt_model_cfg;

typedef struct {
    /* wall-clock of the last mt_train_step and mt_adam_step, milliseconds */
    double step_ms, adam_ms;
    /* device-side busy time of the last step from HIP event timestamps, milliseconds */
    double compute_busy_ms, h2d_busy_ms, d2h_busy_ms;
    /* link-busy time that overlapped compute-busy time (Section 3.2: transfers hidden behind compute) */
    double h2d_hidden_ms, d2h_hidden_ms;
    /* bytes moved over the host link in the last step */
    uint64_t h2d_bytes, d2h_bytes;
    /* sizes fixed at create */
    uint64_t device_arena_bytes, host_pinned_bytes, host_pageable_bytes;
    uint64_t n_params;
    uint64_t steps_done;
    /* With MT_FLAG_KERNEL_TIMING, for the last step, per kernel class
     *   0 = matrix-core GEMM (all projections, their input/weight gradients, LM head)
     *   1 = flash-attention forward (including recompute)   2 = flash-attention backward (dK/dV + dQ kernels)
     * class_ms: summed launch durations from HIP events on the compute stream; class_flops: executed
     * FLOPs (2MNK per GEMM; causal tile products for attention); class_launches: bracketed launches;
     * class_bytes: algorithmic HBM bytes (every operand and result once). */
    double class_ms[3];
    double class_flops[3];
    uint64_t class_launches[3];
    double class_bytes[3];
} mt_stats;

/* Number of parameter tensors (9 n_layers + 3) for this configuration. */
mt_status mt_tensor_count(const mt_model_cfg *cfg, int32_t *n);

/* Shape and name of tensor idx in canonical order; cols == 1 for vectors. name points to
 * thread-local storage valid until the next call on the same thread. */
mt_status mt_tensor_info(const mt_model_cfg *cfg, int32_t idx, int64_t *rows, int64_t *cols, const char **name);

/* Create a handle.  host_param_ptrs[9L+3] (12L+3 with qkv_bias; one fewer with tie_embeddings) are the caller's fp32 master parameters in
 * canonical order (Section 3.1: the host copy is authoritative).  They stay owned by the
 * caller, must outlive the handle, may be pageable memory and are modified only by
 * mt_adam_step.  The library allocates: a pinned bf16 copy of every unit's weights laid out
 * as one contiguous 4 KiB-aligned block per unit (Section 3.3 layer-contiguous tiling: one DMA
 * per unit), fp32 gradient blocks (pinned, or pageable behind a pool of pinned slabs, see
 * MT_FLAG_GRAD_SLABS), Adam moments (zero), the device arena, three streams and the events.  Fails with MT_ERR_DEVICE_OOM / MT_ERR_HOST_OOM without leaking. */
mt_status mt_create(const mt_model_cfg *cfg, float *const *host_param_ptrs, mt_handle **out);

/* One training step without the optimizer (Algorithm 1, phases 1-3).
 * tokens, labels: int32 [batch, seq] row-major, borrowed for the call, pageable is fine.
 * The loss is the mean over the positions with label >= 0 of -log softmax(logits)[label];
 * the caller shifts labels.  On MT_OK *loss is set and every host gradient tensor holds this
 * step's fp32 gradient (overwritten, not accumulated).  Parameters are not modified.
 * Synchronous: returns after the last gradient byte has landed on the host.
 * Errors: MT_ERR_SHAPE (batch*seq > max_batch*max_seq, seq > max_seq, seq % 8 != 0),
 *         MT_ERR_TOKEN_RANGE, MT_ERR_HIP. */
mt_status mt_train_step(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch, int32_t seq,
                        float *loss);

/* One more micro-batch of the same optimizer step: same as mt_train_step, but every host gradient
 * tensor ends up holding (previous content + this micro-batch's gradient), one fp32 addition per element
 * on the host (Section 3.1 keeps "accumulated gradients" in host memory; Appendix A.3: a background
 * thread folds each returned gradient slab into the master gradient store).  The device-to-host copies
 * of such a step land in a pool of 4 pinned slabs of the largest unit's size (allocated at the first
 * call; MT_ERR_HOST_OOM if that fails) and a host thread adds each slab to its gradient block while the
 * GPU continues.  *loss is this micro-batch's mean loss; no rescaling is applied to either side.
 * Errors: MT_ERR_STATE before the first mt_train_step; otherwise as mt_train_step. */
mt_status mt_train_step_accumulate(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch,
                                   int32_t seq, float *loss);

/* Host Adam with decoupled weight decay on every parameter (Algorithm 1, last line), t = step >= 1:
 *   p <- p (1 - lr wd);  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   p <- p - lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)
 * Also refreshes the pinned bf16 copy (round to nearest even) that the next step streams.
 * Multi-threaded on the host CPU; no GPU work.  Errors: MT_ERR_STATE before the first
 * successful mt_train_step, MT_ERR_INVALID_ARG for step < 1. */
mt_status mt_adam_step(mt_handle *h, float lr, float beta1, float beta2, float eps, float wd, int64_t step);

/* mt_train_step and mt_adam_step in one call, with the optimizer overlapped: the Adam update of each
 * unit (same arithmetic as mt_adam_step, same arguments) runs on host threads as soon as that unit's
 * gradient block has landed, while the GPU continues with the remaining blocks (Algorithm 1,
 * optimizer phase; Section 3.3).  Returns after both the step and every
 * update have finished.  On MT_OK the gradient tensors hold this step's gradients and the parameters,
 * moments and bf16 copy are updated.  With MT_FLAG_COMPUTE_ONLY / MT_FLAG_COPY_ONLY no update is applied.
 * Failure: argument, shape and token-range errors are found before anything runs and leave every state untouched.
 * An error after that (MT_ERR_HIP) can leave the update applied to the units whose gradients had already landed
 * (the head and the later blocks) and not to the others; nothing is rolled back.  The handle then refuses
 * mt_train_step_adam and mt_adam_step with MT_ERR_STATE, so that a retry cannot apply the same step twice to some
 * units, until the caller has restored the parameters (its own arrays) and the moments (through mt_get_tensor)
 * from a copy of its own and called mt_refresh_shadow, which acknowledges the state.  mt_train_step alone stays
 * usable. */
mt_status mt_train_step_adam(mt_handle *h, const int32_t *tokens, const int32_t *labels, int32_t batch, int32_t seq,
                             float *loss, float lr, float beta1, float beta2, float eps, float wd, int64_t step);

/* Rebuild the bf16 copy from the caller's fp32 parameters (after the caller edited them).  Also acknowledges a
 * partially applied optimizer step (see mt_train_step_adam). */
mt_status mt_refresh_shadow(mt_handle *h);

#define MT_KIND_GRAD 0
#define MT_KIND_ADAM_M 1
#define MT_KIND_ADAM_V 2
/* Borrowed pointer to the library-owned host array of tensor idx; valid until mt_destroy. */
mt_status mt_get_tensor(mt_handle *h, int32_t idx, int32_t kind, float **p, size_t *numel);

mt_status mt_get_stats(mt_handle *h, mt_stats *out);

/* Synchronise, free every device and host resource of the handle.  NULL is allowed. */
mt_status mt_destroy(mt_handle *h);

/* Pinned, 4 KiB-aligned host memory from the HIP runtime (for callers that want their master
 * parameters page-locked).  mt_host_alloc returns NULL on failure. */
void *mt_host_alloc(size_t bytes);
void mt_host_free(void *p);

/* Number of visible HIP devices (0 if none or the runtime cannot initialise). */
int32_t mt_device_count(void);
/* Block until all work on the device has finished (hipDeviceSynchronize). */
mt_status mt_device_synchronize(int32_t device_id);

/* Message of the last error raised on the calling thread ("" if none). */
const char *mt_last_error(void);

/* Pinned-buffer copy-bandwidth probe over the same path the step uses (hipMemcpyAsync on a
 * non-blocking stream from/to pinned memory): GB/s for H2D alone, D2H alone and both at once
 * (sum of both directions).  bytes per transfer, repeated reps times. */
mt_status mt_link_probe(int32_t device_id, size_t bytes, int32_t reps, double *h2d_gbs, double *d2h_gbs,
                        double *bidir_gbs);

#ifdef __cplusplus
}
#endif
#endif /* MEGATRAIN_H_ */
