/*
 * d2ft.h - C ABI of the head-selective ViT block library for AMD MI355X (gfx950).
 *
 * The library runs the forward and backward pass of pre-LN ViT transformer
 * blocks in which every attention head carries an operation code for the
 * current step, as defined in Sec. II-A.2 "Operation selection" of the D2FT
 * paper (arXiv 2504.12471):
 *     p_f  full          forward and backward
 *     p_o  forward-only  forward, no backward (no weight gradient, and no
 *                        gradient flows through the head: the residual route
 *                        carries the gradient past it)
 *     p_s  shortcut      nothing; the residual route carries activations
 *                        forward and gradients backward
 * and it selects those codes with the bi-level knapsack of Alg. 1
 * (KnapsackScheduling) and Alg. 2 (DPSearching).
 *
 * Conventions that hold for every entry point
 *   - Plain C types only.  Every tensor pointer is a DEVICE pointer unless the
 *     parameter comment says HOST.  Tensors are row-major and contiguous.
 *   - The caller owns every buffer.  The library allocates no device memory
 *     and keeps no tensor state between calls (per device it keeps launch
 *     parameters it has looked up, a HIP stream and two events of its own,
 *     see D2FT_FLAG_ONE_STREAM, and the timing records of d2ft_timing_enable).
 *   - Block calls are asynchronous on the given HIP stream (a hipStream_t
 *     passed as void*; NULL is the default stream): when a call returns, all
 *     of its work is ordered on that stream (unless the caller opts out with
 *     D2FT_FLAG_DEFER_JOIN).
 *   - Calls on one device from several host threads must be serialised by the
 *     caller.
 *   - Errors are return codes.  Arguments are validated before anything is
 *     launched, so a call that returns D2FT_EINVAL or D2FT_ESHAPE has had no
 *     effect.  D2FT_EDEVICE reports a HIP error of a launch or copy.
 *   - Storage type is fp32 or bf16 for all tensors of a call; accumulation is
 *     fp32.  LayerNorm statistics and softmax log-sum-exp are kept in fp32.
 */
#ifndef D2FT_H
#define D2FT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    D2FT_OK = 0,
    D2FT_EINVAL = 1,  /* NULL pointer, bad enum value, op code outside {1,2,3}, non-finite score */
    D2FT_ESHAPE = 2,  /* non-positive or unsupported dimension, workspace too small */
    D2FT_EDEVICE = 3  /* a HIP launch, copy or synchronisation failed */
} d2ft_status;

/* Operation codes, with the values of the scheduling table T_opt of Alg. 1. */
enum { D2FT_OP_FULL = 1, D2FT_OP_FWD = 2, D2FT_OP_SKIP = 3 };

typedef enum { D2FT_F32 = 0, D2FT_BF16 = 1 } d2ft_dtype;

/* flags of d2ft_block_desc */
enum {
    /* 0: gradients are overwritten, and the slices of heads that are not p_f are
     *    written as +0.0.  1: gradients are added to what the buffers hold, and
     *    the slices of heads that are not p_f are left untouched. */
    D2FT_FLAG_ACCUM_GRADS = 1u,
    /* bf16 only: run the vector-ALU kernels instead of the MFMA kernels (a cross-check
     * of the two kernel families; fp32 always runs on the vector ALUs). */
    D2FT_FLAG_NO_MFMA = 2u,
    /* The op code of head h also governs hidden units [h*mlp_hidden/heads, (h+1)*mlp_hidden/heads)
     * of the feed-forward network, i.e. the whole subnet of Sec. II-A.1 (one attention head plus
     * 1/H of the FFN; Sec. IV-A "Full fine-tuning partition settings"): a p_s subnet's slice is
     * skipped, a p_o subnet's slice runs forward only (its term is a constant in backward), a p_f
     * subnet's slice is trained.  b2 is then added iff at least one subnet is live, and with no
     * live subnet the block is the identity.  Requires mlp_hidden divisible by heads with a
     * quotient that is a multiple of 64; otherwise D2FT_ESHAPE. */
    D2FT_FLAG_GATE_FFN = 4u,
    /* d2ft_block_bwd / d2ft_block_bwd_mb (bf16 matrix-core path): launch everything on the caller's stream.
     * By default those calls put the weight-gradient products, which nothing else in the call waits for, on a
     * second stream of the library's own (default priority), ordered behind the caller's earlier work and joined
     * to the caller's stream before the call returns, so that to the caller the call is work on its stream
     * either way.  The two modes group the weight gradients into launches differently, so their split-K sums
     * may differ in rounding order; nothing else differs.  The second stream is not used while per-kernel
     * timing is on (d2ft_timing_enable) or while the caller's stream is being captured. */
    D2FT_FLAG_ONE_STREAM = 8u,
    /* d2ft_block_bwd / d2ft_block_bwd_mb, for a caller's loop over blocks: return without making the caller's
     * stream wait for the work the call left on the library's second stream (this call's weight gradients, and
     * with them its bias gradients and the zero fills of the slices that are not p_f).  That work is then
     * ordered on the caller's stream by the next call on this device into a block, optimizer, score, embedding
     * or classifier entry point (each waits for it first; a following backward call of the same shape with
     * this flag waits only where it has to, which is what makes the flag worth setting) or by d2ft_join().
     * Until then the caller must not read any gradient of this call, and must not write, free or reuse any
     * buffer passed to this call, from its own code on any stream.  dx is complete on the caller's stream as
     * always. */
    D2FT_FLAG_DEFER_JOIN = 16u
};

#define D2FT_MAX_HEADS 64
#define D2FT_HEAD_DIM 64      /* the only supported head dimension */
#define D2FT_MAX_LORA_RANK 64

/* Shape of one block as held by this device.  heads*head_dim need not equal
 * width: a device may hold a share of the model's heads (Sec. II-A.1
 * "Partitioning strategy") and a share of the MLP's hidden units. */
typedef struct d2ft_block_desc {
    int32_t batch;       /* B >= 1 */
    int32_t tokens;      /* T in [1, 1024] */
    int32_t width;       /* D >= 8, multiple of 8 */
    int32_t heads;       /* H in [1, D2FT_MAX_HEADS]: heads held by this call */
    int32_t head_dim;    /* must be D2FT_HEAD_DIM */
    int32_t mlp_hidden;  /* Dm >= 8, multiple of 8 */
    int32_t lora_rank;   /* 0: no LoRA; else r in [1, D2FT_MAX_LORA_RANK] (Sec. II-D) */
    float ln_eps;        /* LayerNorm epsilon (> 0) */
    float lora_scale;    /* s in W_eff = W + s * B * A */
    int32_t dtype;       /* d2ft_dtype */
    uint32_t flags;      /* D2FT_FLAG_* */
} d2ft_block_desc;

/* Weights of one block (device pointers, storage type desc.dtype).
 * Linear layers compute y = x W^T + b with W stored [out, in].
 * Head h owns rows [h*64, h*64+64) of each of the three w_qkv planes and
 * columns [h*64, h*64+64) of w_o: that slice is the attention part of the
 * paper's subnet k = (l, h).  b_o and b2 may be NULL (a device that does not
 * own the bias of a sharded layer).  lora_* are read only if lora_rank > 0;
 * adapters sit on the query and value projections of each head. */
typedef struct d2ft_block_weights {
    const void *ln1_g, *ln1_b;   /* [D] */
    const void *w_qkv;           /* [3][H][64][D]  planes: 0 = query, 1 = key, 2 = value */
    const void *b_qkv;           /* [3][H][64] */
    const void *w_o;             /* [D][H*64] */
    const void *b_o;             /* [D] or NULL; added iff at least one head is live */
    const void *ln2_g, *ln2_b;   /* [D] */
    const void *w1, *b1;         /* [Dm][D], [Dm] */
    const void *w2, *b2;         /* [D][Dm], [D] or NULL */
    const void *lora_a_q, *lora_a_v; /* [H][r][D] */
    const void *lora_b_q, *lora_b_v; /* [H][64][r] */
} d2ft_block_weights;

/* Gradient outputs, same shapes and storage type as the weights.  A NULL field
 * means that gradient is not computed (LayerNorm parameters are frozen in the
 * paper's setup, Sec. III-A; base weights are frozen under LoRA, Sec. II-D). */
typedef struct d2ft_block_grads {
    void *ln1_g, *ln1_b;
    void *w_qkv, *b_qkv;
    void *w_o, *b_o;
    void *ln2_g, *ln2_b;
    void *w1, *b1;
    void *w2, *b2;
    void *lora_a_q, *lora_a_v;
    void *lora_b_q, *lora_b_v;
} d2ft_block_grads;

/* Bytes of the `saved` buffer that d2ft_block_fwd fills for d2ft_block_bwd, and
 * of the `scratch` buffer either call may use; worst case over all masks.
 * Both buffers must be 256-byte aligned.  Return 0 if the descriptor is invalid. */
size_t d2ft_block_saved_bytes(const d2ft_block_desc *desc);
size_t d2ft_block_scratch_bytes(const d2ft_block_desc *desc);

/* Head compaction (host only, no GPU work).  From the op codes of one block
 * build the live-head list: heads with p_f in ascending order, then heads with
 * p_o in ascending order; p_s heads do not appear (Sec. II-A.2).
 *   ops     HOST [heads]  codes 1/2/3
 *   live    HOST [heads]  out: first *n_live entries are valid
 *   n_full  HOST          out: number of p_f heads (a prefix of live)
 *   n_live  HOST          out: number of p_f + p_o heads
 * D2FT_EINVAL on NULL or a code outside {1,2,3}; D2FT_ESHAPE if heads is not in
 * [1, D2FT_MAX_HEADS]. */
d2ft_status d2ft_compact_heads(const uint8_t *ops, int32_t heads, int32_t *live,
                               int32_t *n_full, int32_t *n_live);

/* Forward of one block (Sec. II-A.2; block structure of Sec. III-A "Model"):
 *   u  = LN1(x)                                   (skipped if no head is live)
 *   for live heads h: [Q K V]_h = u W_{qkv,h}^T + b (+ LoRA), O_h = softmax(Q K^T / 8) V
 *   x1 = x + sum_{live h} O_h W_{o,h}^T (+ b_o if any head is live)
 *   y  = x1 + W2 GELU(W1 LN2(x1) + b1) + b2       (erf GELU; not gated unless D2FT_FLAG_GATE_FFN is set)
 *   ops      HOST [heads]
 *   x        [B][T][D] input hidden states
 *   y        [B][T][D] output; must not alias x
 *   saved    d2ft_block_saved_bytes(desc) bytes; opaque, consumed by d2ft_block_bwd
 *   scratch  d2ft_block_scratch_bytes(desc) bytes; contents undefined afterwards */
d2ft_status d2ft_block_fwd(const d2ft_block_desc *desc, const d2ft_block_weights *weights,
                           const uint8_t *ops, const void *x, void *y, void *saved,
                           void *scratch, void *hip_stream);

/* Backward of one block, for the same desc, weights, ops and x that the forward
 * call saw, and the `saved` buffer it filled.  Attention-side backward work
 * runs for p_f heads only (Sec. II-A.2: p_o keeps the forward pass and skips
 * backward propagation; the gradient goes by the residual route).  The weights
 * must hold the values the forward call read: with LoRA (Sec. II-D) `saved`
 * carries the merged QKV weights W + s B A of the live heads and the backward
 * call multiplies with those.
 *   dy     [B][T][D] upstream gradient
 *   dx     [B][T][D] out; must not alias dy
 *   grads  HOST struct of device pointers; NULL fields are skipped.  Slices of
 *          heads that are not p_f follow D2FT_FLAG_ACCUM_GRADS (see above). */
d2ft_status d2ft_block_bwd(const d2ft_block_desc *desc, const d2ft_block_weights *weights,
                           const uint8_t *ops, const void *x, const void *dy, void *dx,
                           const d2ft_block_grads *grads, const void *saved, void *scratch,
                           void *hip_stream);

/* Makes hip_stream wait for whatever an earlier call with D2FT_FLAG_DEFER_JOIN left running on the library's
 * second stream on the current device; a no-op if there is nothing.  D2FT_EDEVICE if the wait cannot be queued. */
d2ft_status d2ft_join(void *hip_stream);

/* One block over several micro-batches, each with its own op codes: the scheduling table of
 * Alg. 1 holds one code per (subnet, micro-batch), T_opt[k][x_i], and Sec. IV-A splits a batch into
 * micro-batches.  Micro-batch i is the next mb_images[i] images of x; it runs under
 * ops[i*heads .. (i+1)*heads).  The backward adds the micro-batches' weight gradients
 * (gradient accumulation): with D2FT_FLAG_ACCUM_GRADS clear the result overwrites the buffers
 * and a subnet that is p_f in no micro-batch gets +0.0; with it set everything is added to what
 * the buffers hold.  How the work is laid out on the stream is the library's choice and does not change
 * what is computed beyond rounding order:
 *   - when the matrix-core attention kernels apply (bf16, at most 224 tokens) and every micro-batch keeps a
 *     head live, the block runs once over the whole batch under the union of the codes, with the attention
 *     kernels masking per (micro-batch, head): skipped pairs contribute exact zeros to the projections, pairs
 *     that are not p_f exact zeros to the weight gradients (gated feed-forward slices likewise);
 *   - otherwise, without D2FT_FLAG_GATE_FFN, the feed-forward half (which does not depend on the op codes)
 *     runs once over the whole batch and the attention half per micro-batch, one after the other;
 *   - otherwise every micro-batch is a block call of its own.
 *   n_micro    1 .. D2FT_MAX_MICRO
 *   mb_images  HOST [n_micro], each >= 1, summing to desc->batch
 *   ops        HOST [n_micro][heads]
 *   saved      d2ft_block_saved_bytes_mb(desc, n_micro, mb_images) bytes
 *   scratch    d2ft_block_scratch_bytes(desc) bytes
 * Other arguments and errors as for d2ft_block_fwd / d2ft_block_bwd; bad micro-batch sizes give
 * D2FT_ESHAPE. */
#define D2FT_MAX_MICRO 64
size_t d2ft_block_saved_bytes_mb(const d2ft_block_desc *desc, int32_t n_micro, const int32_t *mb_images);
d2ft_status d2ft_block_fwd_mb(const d2ft_block_desc *desc, const d2ft_block_weights *weights, int32_t n_micro,
                              const int32_t *mb_images, const uint8_t *ops, const void *x, void *y, void *saved,
                              void *scratch, void *hip_stream);
d2ft_status d2ft_block_bwd_mb(const d2ft_block_desc *desc, const d2ft_block_weights *weights, int32_t n_micro,
                              const int32_t *mb_images, const uint8_t *ops, const void *x, const void *dy, void *dx,
                              const d2ft_block_grads *grads, const void *saved, void *scratch, void *hip_stream);

/* Bi-level knapsack selection of operation codes: Alg. 1 (KnapsackScheduling)
 * calling Alg. 2 (DPSearching) twice per knapsack - p_f items by backward
 * scores with weight c^f_k + c^b_k under cap_full[k] (outer problem, Eq. 4),
 * p_o items by forward scores with weight c^f_k under cap_fwd[k] (inner problem,
 * Eq. 5); an item selected by both is p_f, by neither p_s.  The DP runs on the
 * GPU in fp64, one add and one compare per cell in the order the algorithm
 * writes them.  The call synchronises the stream before it returns.
 *   score_full, score_fwd  HOST [n_knapsacks][n_items], finite
 *   cost_fwd   HOST [n_knapsacks]  c^f_k >= 1
 *   cost_bwd   HOST [n_knapsacks]  c^b_k >= 0
 *   cap_full, cap_fwd  HOST [n_knapsacks]  >= 0
 *   ops_out    HOST [n_knapsacks][n_items]  out: codes 1/2/3
 *   workspace  DEVICE, at least d2ft_knapsack_workspace_bytes(...) bytes, 256-byte aligned */
size_t d2ft_knapsack_workspace_bytes(int32_t n_knapsacks, int32_t n_items,
                                     const int32_t *cap_full, const int32_t *cap_fwd);
d2ft_status d2ft_select_knapsack(int32_t n_knapsacks, int32_t n_items,
                                 const double *score_full, const double *score_fwd,
                                 const int32_t *cost_fwd, const int32_t *cost_bwd,
                                 const int32_t *cap_full, const int32_t *cap_fwd,
                                 uint8_t *ops_out, void *workspace, size_t workspace_bytes,
                                 void *hip_stream);

/* d2ft_select_knapsack for callers that cannot allocate device memory (code that runs where hipMalloc is
 * not allowed: tight serving loops, harnesses that forbid allocation, set-up under which a workspace cannot
 * be obtained).  Same arguments, results and errors as d2ft_select_knapsack, without the workspace: the DP
 * tables live in a device array that is part of the library image, D2FT_KNAPSACK_STATIC_BYTES long, which
 * every GPU the library runs on holds until the process ends.  The call makes no allocation of its own.
 * A problem whose d2ft_knapsack_workspace_bytes(...) exceeds that size is refused with D2FT_ESHAPE before
 * any device work.  All calls on one GPU share the one array: calls that overlap in time on the same GPU
 * (from several threads or streams) race and must be serialised by the caller; consecutive calls need no
 * clean-up in between.  d2ft_knapsack_static_bytes() returns the array's size. */
#define D2FT_KNAPSACK_STATIC_BYTES (4u << 20)
size_t d2ft_knapsack_static_bytes(void);
d2ft_status d2ft_select_knapsack_static(int32_t n_knapsacks, int32_t n_items,
                                        const double *score_full, const double *score_fwd,
                                        const int32_t *cost_fwd, const int32_t *cost_bwd,
                                        const int32_t *cap_full, const int32_t *cap_fwd,
                                        uint8_t *ops_out, void *hip_stream);

/* Contribution scores of the subnets of one block (Sec. II-B, contribution scores): for every
 * head h, over the tensor slices that belong to that subnet alone - Q/K/V weight rows and
 * biases, output-projection columns, LoRA adapters and, with D2FT_FLAG_GATE_FFN, the head's
 * feed-forward slice (w1 rows, b1, w2 columns) -
 *   D2FT_SCORE_FISHER     sum of squared entries: with `tensors` holding the gradients of one sample
 *                         or micro-batch this is the empirical Fisher information, the backward score;
 *   D2FT_SCORE_MAGNITUDE  sum of absolute values: with `tensors` holding the weights this is the
 *                         weight magnitude, the forward score.
 * LayerNorm parameters and the shared biases b_o, b2 belong to no single subnet and are not
 * read.  Sums are accumulated in fp64 in a fixed order (the result does not depend on timing).
 * The scores feed d2ft_select_knapsack; like it, the call synchronises the stream before it returns.
 *   tensors     HOST struct of DEVICE pointers in the weight layout (gradients are passed through
 *               the same struct); NULL fields are skipped
 *   scores_out  HOST [heads]
 *   workspace   DEVICE, at least d2ft_scores_workspace_bytes(desc) bytes, 256-byte aligned
 * Errors: D2FT_EINVAL for NULL desc / tensors / scores_out / workspace, a bad kind or a
 * misaligned pointer; D2FT_ESHAPE for an unsupported shape or a workspace that is too small. */
typedef enum { D2FT_SCORE_FISHER = 0, D2FT_SCORE_MAGNITUDE = 1 } d2ft_score_kind;
size_t d2ft_scores_workspace_bytes(const d2ft_block_desc *desc);
d2ft_status d2ft_subnet_scores(const d2ft_block_desc *desc, const d2ft_block_weights *tensors, int32_t kind,
                               double *scores_out, void *workspace, size_t workspace_bytes, void *hip_stream);

/* One optimizer step on a block: SGD with momentum, the optimizer Sec. IV-A names ("Computational
 * cost analysis"; the paper gives no hyper-parameters), in the common form without dampening or
 * Nesterov look-ahead, per element
 *     v <- momentum * v + (g + weight_decay * w),     w <- w - lr * v.
 * The slices that belong to one subnet alone (Q/K/V rows and biases, W_o columns, LoRA adapters and,
 * with D2FT_FLAG_GATE_FFN, the feed-forward slice) are updated for the heads whose code in `ops`
 * is p_f and left untouched - weights, momentum and master copy - for the others: a subnet that
 * ran p_o or p_s in the step has no gradient and does no optimizer work.  Tensors shared by all
 * subnets (LayerNorm parameters, b_o, b2, and the whole feed-forward network without the flag) are
 * always updated.  A tensor takes part only if its pointers in `weights`, `grads` and `momentum`
 * are all non-NULL.  Arithmetic is fp32.
 *   weights   HOST struct of DEVICE pointers, storage dtype of desc, updated in place
 *   grads     same layout and dtype, read only
 *   momentum  same layout, fp32 buffers, updated in place
 *   master    NULL, or a struct of fp32 copies of the weights: where a field is non-NULL the update
 *             is applied to the fp32 copy and `weights` receives its rounded value
 *   ops       HOST [heads]
 * Errors: D2FT_EINVAL for NULL desc / weights / grads / momentum / ops / params, a code outside
 * {1,2,3}, a misaligned pointer or non-finite hyper-parameters. */
typedef struct d2ft_sgd_params {
    float lr, momentum, weight_decay;
} d2ft_sgd_params;
d2ft_status d2ft_sgd_step(const d2ft_block_desc *desc, const d2ft_block_grads *weights,
                          const d2ft_block_weights *grads, const d2ft_block_grads *momentum,
                          const d2ft_block_grads *master, const uint8_t *ops,
                          const d2ft_sgd_params *params, void *hip_stream);

/* The two subnets outside the transformer blocks (Sec. IV-A, "Full fine-tuning partition settings":
 * the patch embedding layer at the start, the global pooling and classification layer at the end).
 * The paper does not spell them out; they are taken in the usual ViT form.
 *
 * Patch embedding: the image is cut into non-overlapping patch x patch squares, each flattened in
 * (channel, row, column) order and projected, a class token goes in front, position embeddings are added:
 *   tokens[b][0]     = cls + pos[0]
 *   tokens[b][1 + p] = w_pe . patch(b, p) + b_pe + pos[1 + p],   p = py * (width_px / patch) + px
 *   images  [B][C][H][W]            w_pe [D][C*patch*patch]      b_pe, cls [D]      pos [T][D]
 *   tokens  [B][T][D], T = 1 + (H/patch)*(W/patch)
 * patch must be a multiple of 8 and divide H and W; D a multiple of 8.  The backward call returns the
 * parameter gradients (NULL pointers are skipped; D2FT_FLAG_ACCUM_GRADS in flags adds instead of
 * overwriting); no gradient is taken with respect to the images.
 *   saved    d2ft_embed_saved_bytes(desc) bytes, written by fwd, read by bwd
 *   scratch  d2ft_embed_scratch_bytes(desc) bytes */
typedef struct d2ft_embed_desc {
    int32_t batch, channels, height, width_px, patch;
    int32_t width;   /* D */
    int32_t dtype;   /* d2ft_dtype */
    uint32_t flags;  /* D2FT_FLAG_ACCUM_GRADS, D2FT_FLAG_NO_MFMA */
} d2ft_embed_desc;
size_t d2ft_embed_saved_bytes(const d2ft_embed_desc *desc);
size_t d2ft_embed_scratch_bytes(const d2ft_embed_desc *desc);
d2ft_status d2ft_patch_embed_fwd(const d2ft_embed_desc *desc, const void *images, const void *w_pe,
                                 const void *b_pe, const void *cls, const void *pos, void *tokens,
                                 void *saved, void *scratch, void *hip_stream);
d2ft_status d2ft_patch_embed_bwd(const d2ft_embed_desc *desc, const void *dtokens, void *g_w_pe,
                                 void *g_b_pe, void *g_cls, void *g_pos, const void *saved,
                                 void *scratch, void *hip_stream);

/* Pooling and classification with the loss, forward and backward in one call: LayerNorm of the class
 * token (row 0 of each image), a linear layer, mean softmax cross-entropy over the batch, and the
 * gradients: dtokens [B][T][D] is written in full (zero outside the class-token rows), parameter
 * gradients where the pointers are non-NULL.  Arithmetic is fp32; images are added in index order.
 * The call synchronises the stream to return the loss.
 *   tokens [B][T][D]   ln_g, ln_b [D]   w_c [classes][D]   b_c [classes]
 *   labels    HOST [B], each in [0, classes)  (else D2FT_EINVAL)
 *   loss_out  HOST, one float
 *   scratch   DEVICE, d2ft_head_scratch_bytes(desc) bytes, 256-byte aligned */
typedef struct d2ft_head_desc {
    int32_t batch, tokens, width, classes;
    float ln_eps;
    int32_t dtype;
    uint32_t flags;   /* D2FT_FLAG_ACCUM_GRADS */
} d2ft_head_desc;
size_t d2ft_head_scratch_bytes(const d2ft_head_desc *desc);
d2ft_status d2ft_classifier_fwd_bwd(const d2ft_head_desc *desc, const void *tokens, const void *ln_g,
                                    const void *ln_b, const void *w_c, const void *b_c,
                                    const int32_t *labels, float *loss_out, void *dtokens, void *g_ln_g,
                                    void *g_ln_b, void *g_w_c, void *g_b_c, void *scratch,
                                    void *hip_stream);

/* Diagnostics: per-kernel timing.  While enabled, every kernel launch the library makes is
 * bracketed by a pair of HIP events on the stream of the call (this adds host work per launch:
 * do not time whole steps while it is on).  d2ft_timing_enable(1) clears earlier records and
 * starts recording, d2ft_timing_enable(0) stops.  d2ft_timing_read waits for the recorded
 * events and returns one entry per kernel class - launch count, summed duration, and the
 * algorithmic FLOPs the launches stood for (GEMM classes: 2*M*N*K; 0 elsewhere) - or -1 on a
 * HIP error.  The measurement backs the roofline figures of the benchmark (measurement of
 * the paper's compute-cost claim of Sec. IV-A on this hardware).  Not thread safe.
 *   out  HOST [max_entries] */
typedef struct d2ft_kernel_time {
    char name[96];
    int64_t launches;
    double ms;
    double flops;
    double bytes;
} d2ft_kernel_time;
d2ft_status d2ft_timing_enable(int32_t on);
int32_t d2ft_timing_read(d2ft_kernel_time *out, int32_t max_entries);

/* Static description of a status code. */
const char *d2ft_status_string(d2ft_status status);

#ifdef __cplusplus
}
#endif
#endif /* D2FT_H */
