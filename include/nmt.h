/*
 * nmt.h — C ABI of the MI355X (gfx950) reduced-precision NMT training-step library.
 *
 * The library runs the data-parallel hot path of "Scaling Neural Machine Translation" on one
 * GPU: Transformer encoder-decoder forward and backward in fp16 with fp32 accumulation,
 * label-smoothed cross-entropy, loss scaling with overflow detection, fp32 master weights and
 * Adam, and gradient accumulation over several sub-batches.
 *
 * Conventions
 *  - Every function returns int: NMT_OK (0) or a negative NMT_E* code; nmt_last_error() gives
 *    the message of the last failure on the calling thread.  No C++ exception crosses the ABI.
 *  - Pointers named d_* (and all buffers handed to nmt_bind) are DEVICE pointers owned by the
 *    caller; they must stay valid until the work enqueued on them has finished.  The library
 *    never allocates or frees device memory (nmt_backward creates one extra stream and four
 *    events per context on first use).  Host pointers are marked "host".
 *  - `stream` is a hipStream_t passed as void*; all kernels are enqueued on it and no function
 *    synchronises unless it says so.
 *  - fp16 buffers are IEEE binary16 (passed as void*).  Matrices are row-major.
 *  - Linear weights are stored [out, in]; y = x W^T + b.
 */
#ifndef NMT_H_
#define NMT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NMT_OK 0
#define NMT_EINVAL (-1) /* bad argument or unsupported shape */
#define NMT_ESTATE (-2) /* call out of order (e.g. backward before forward) */
#define NMT_ENOMEM (-3) /* caller's workspace too small */
#define NMT_EHIP (-4)   /* HIP runtime error */

typedef struct nmt_ctx nmt_ctx;

/* Model and regularisation hyper-parameters (section "Models and Hyperparameters"). */
typedef struct {
  int32_t enc_layers, dec_layers; /* blocks in the encoder / decoder                     */
  int32_t d_model, n_heads, d_ff; /* d_model % n_heads == 0, head size in {16,32,64,128}  */
  int32_t vocab;                  /* shared vocabulary, multiple of 8, <= 65536           */
  int32_t pad_id;                 /* id of the padding symbol                              */
  float dropout;                  /* on each sub-layer output before the residual add, and
                                     on the embedding + position sum                       */
  float attn_dropout;             /* on the attention probabilities: not built, must be 0
                                     (nmt_create returns NMT_EINVAL otherwise)             */
  float act_dropout;              /* after the ReLU of the feed-forward layer              */
  float label_smoothing;          /* weight of the uniform prior over the vocabulary       */
  float ln_eps;                   /* variance floor of layer normalisation                 */
  uint64_t seed;                  /* Philox key of the dropout streams                     */
  int32_t max_sentences, max_len; /* limits for B (<= 2^20) and for S, T (<= 1024)        */
} nmt_config;

const char* nmt_last_error(void);

/* Host only.  Validates the configuration and builds the parameter layout. */
int nmt_create(const nmt_config* cfg, nmt_ctx** out);
void nmt_destroy(nmt_ctx* ctx);

/* Flat parameter layout: P scalars; tensor idx occupies [offset, offset + rows*cols).
 * Biases and LayerNorm vectors have rows == 1.  idx past the end returns NMT_EINVAL.
 * *name points into storage owned by ctx.  Every tensor offset is a multiple of 8. */
int64_t nmt_param_count(const nmt_ctx* ctx);
int32_t nmt_param_tensors(const nmt_ctx* ctx);
int nmt_param_info(const nmt_ctx* ctx, int32_t idx, const char** name, int64_t* offset,
                   int32_t* rows, int32_t* cols);

/* Bytes of workspace nmt_forward_loss / nmt_backward need for a batch of B sentences padded to
 * S source and T target positions (negative on invalid shapes). */
int64_t nmt_workspace_bytes(const nmt_ctx* ctx, int32_t B, int32_t S, int32_t T);

/* Attach the caller's device buffers.  w16, g16: fp16[P] weights and per-sub-batch gradients;
 * master32, acc32, adam_m, adam_v: fp32[P]; workspace: ws_bytes bytes, 256-byte aligned.
 * Any of master32/acc32/adam_m/adam_v may be NULL if the calls using them are not made. */
int nmt_bind(nmt_ctx* ctx, void* d_w16, void* d_g16, float* d_master32, float* d_acc32,
             float* d_adam_m, float* d_adam_v, void* d_workspace, int64_t ws_bytes);

/* Forward pass in fp16 and the label-smoothed loss in fp32 (sections "Models and
 * Hyperparameters", "Half-Precision Training").  d_src [B,S], d_tgt_in [B,T], d_tgt_out [B,T]:
 * int32 ids right-padded with pad_id; every sentence has at least one token.
 * The gradient of loss_scale * (sum of token losses) with respect to the logits is left in
 * the workspace for nmt_backward: the loss is scaled at the end of the forward pass, before any
 * fp16 gradient exists ("Half-Precision Training").
 * step (< 2^24) and micro_idx (< 256) select the dropout streams; d_sent_uid [B] (uint32, may
 * be NULL = row index) names each sentence so its dropout mask does not depend on batching.
 * training == 0 disables dropout.
 * Outputs: *d_loss_sum = sum over non-pad target tokens of the UNSCALED loss in nats,
 * *d_ntok = number of non-pad target tokens. */
int nmt_forward_loss(nmt_ctx* ctx, const int32_t* d_src, const int32_t* d_tgt_in,
                     const int32_t* d_tgt_out, int32_t B, int32_t S, int32_t T, float loss_scale,
                     uint32_t step, uint32_t micro_idx, const uint32_t* d_sent_uid, int32_t training,
                     float* d_loss_sum, int32_t* d_ntok, void* stream);

/* The same for a group of n_seg (1 .. NMT_MAX_SEGMENTS) sub-batches of different padded shapes in
 * one pass ("Training with Larger Batches": the gradients of the sub-batches of one update are
 * summed; here the sum over the sub-batches of a group is already formed, in fp32, inside the
 * weight-gradient products of the one backward pass that follows, before the gradient is rounded
 * to fp16).  segs (host, read before the call returns) gives every sub-batch's B, S, T and micro
 * index; the id buffers hold the sub-batches one after another (d_src: sum of B*S ids, d_tgt_in /
 * d_tgt_out: sum of B*T ids) and d_sent_uid one entry per sentence in the same order (NULL: a
 * sentence's index within its sub-batch).  Dropout masks, loss and gradients are those of the
 * sub-batches processed one by one and accumulated.  *d_loss_sum and *d_ntok are totals over the
 * group.  A group may hold at most 2^20 source and 2^20 target positions.
 * The overflow decision of a pass over several sub-batches is that of ITS fp16 gradient, fp16(s * sum over the
 * sub-batches), s = nmt_grad_scale(): one sub-batch whose own gradient would leave the fp16 range can be hidden
 * by the others, and a sum of gradients that each fit can leave it.  Decisions equal to the method's order
 * (every sub-batch's gradient rounded to fp16 on its own, "Half-Precision Training" / "Training with Larger
 * Batches") are guaranteed for one sub-batch per pass only; a pass of several follows its own predicate
 * exactly, and the dynamic loss scale settles where that predicate puts it. */
#define NMT_MAX_SEGMENTS 64
typedef struct {
  int32_t B, S, T;    /* sentences, padded source and target length */
  uint32_t micro_idx; /* index of the sub-batch within its update (< 256): selects its dropout streams */
} nmt_segment;
int64_t nmt_workspace_bytes_group(const nmt_ctx* ctx, int32_t n_seg, const nmt_segment* segs /*host*/);
int nmt_forward_loss_group(nmt_ctx* ctx, int32_t n_seg, const nmt_segment* segs /*host*/, const int32_t* d_src,
                           const int32_t* d_tgt_in, const int32_t* d_tgt_out, float loss_scale, uint32_t step,
                           const uint32_t* d_sent_uid, int32_t training, float* d_loss_sum, int32_t* d_ntok,
                           void* stream);

/* The same for sentences PACKED back to back, without padding: d_sentences (device, n_sent entries,
 * read by the kernels of this call) gives every sentence's source and target length, its uid and
 * the micro index of the sub-batch it belongs to; d_src holds n_src_tokens ids (the source sentences
 * one after another), d_tgt_in / d_tgt_out n_tgt_tokens ids.  n_src_tokens, n_tgt_tokens (host) must
 * be the sums of the lengths and max_src_len, max_tgt_len (host) at least the longest ones: the
 * library sizes its launches from them and clamps what it reads from d_sentences to them, so
 * inconsistent values give undefined results but no access outside the caller's buffers.  Padding
 * positions carry no loss and no gradient, so loss, token count and gradients equal those of the
 * padded sub-batches; only the rows that do nothing are gone. */
typedef struct {
  int32_t src_len, tgt_len; /* >= 1 */
  uint32_t uid;             /* names the sentence's dropout streams */
  uint32_t micro_idx;       /* < 256 */
} nmt_sentence;
int64_t nmt_workspace_bytes_packed(const nmt_ctx* ctx, int32_t n_sent, int64_t n_src_tokens, int64_t n_tgt_tokens);
int nmt_forward_loss_packed(nmt_ctx* ctx, int32_t n_sent, const nmt_sentence* d_sentences, int64_t n_src_tokens,
                            int64_t n_tgt_tokens, int32_t max_src_len, int32_t max_tgt_len, const int32_t* d_src,
                            const int32_t* d_tgt_in, const int32_t* d_tgt_out, float loss_scale, uint32_t step,
                            int32_t training, float* d_loss_sum, int32_t* d_ntok, void* stream);

/* Backward pass in fp16 of the last nmt_forward_loss / nmt_forward_loss_group /
 * nmt_forward_loss_packed; writes every element of g16 with nmt_grad_scale(ctx) times the gradient
 * of loss_scale * loss_sum.  Nothing in it knows about the scale: it is an ordinary reverse pass over
 * fp16 tensors ("Half-Precision Training"). */
int nmt_backward(nmt_ctx* ctx, void* stream);

/* Gradient accumulation over sub-batches ("Training with Larger Batches"):
 * first != 0: acc32 = float(g16) / s; else acc32 += float(g16) / s, where s = nmt_grad_scale(ctx). */
int nmt_accumulate(nmt_ctx* ctx, int32_t first, void* stream);

/* Running totals over the sub-batches of one update, kept on the device so that the caller's loop needs no
 * host arithmetic: adds the loss sum and token count the last forward call wrote (its d_loss_sum / d_ntok)
 * to *d_loss_total / *d_ntok_total (first != 0: overwrites them).  Call after the forward call, on its stream. */
int nmt_accumulate_loss(nmt_ctx* ctx, int32_t first, float* d_loss_total, int32_t* d_ntok_total, void* stream);

/* The power-of-two factor s <= 1 by which the last forward call's pass scales what it writes to g16:
 * g16 = fp16(s * gradient of loss_scale * loss_sum).  s = 1 for passes of fewer than 8192 target
 * positions (any single sub-batch of the paper's size) and halves with every doubling beyond that, so
 * that the sum over a group of sub-batches reaches the fp16 range at the same loss scale as a single
 * sub-batch's gradient would.  nmt_accumulate divides it out again (exactly). */
float nmt_grad_scale(const nmt_ctx* ctx);

/* Overflow detection on the accumulated gradients and their conversion to the original scale ("Half-Precision
 * Training": after accumulation the fp16 gradients, by then fp32 sums, are brought back to the scale of the
 * loss before the weights are updated).  *d_flag = 1 iff any element of acc32 is inf or NaN, else 0, in one
 * read-only pass over acc32; inv_scale = 1 / (loss_scale * total n_tok) is remembered by the context and applied
 * by nmt_adam_step to every element as it reads it (acc32 itself keeps the scaled sums: the unscaled gradient is
 * never written out, which saves one 4-byte write and one 4-byte read per parameter). */
int nmt_check_overflow(nmt_ctx* ctx, float inv_scale, int32_t* d_flag, void* stream);

/* Adam ("Models and Hyperparameters": beta1 0.9, beta2 0.98, epsilon 1e-8) on the fp32 master weights
 * with gradient acc32 * inv_scale (the factor of the last nmt_check_overflow; 1 if none was made) -- the optimizer
 * runs in fp32 ("Half-Precision Training") -- then w16 =
 * round-to-nearest-even of the new master weights.  t is the 1-based update count.  If *d_flag != 0 the
 * call changes nothing (the update is skipped on overflow). */
int nmt_adam_step(nmt_ctx* ctx, float lr, float beta1, float beta2, float eps, int32_t t,
                  const int32_t* d_flag, void* stream);

/* Host helpers holding the scalar decision logic.
 * Dynamic loss scaling: overflow -> scale /= 2, clean = 0; otherwise clean += 1 and when clean
 * reaches `window` (2000 in the paper) scale *= 2, clean = 0.  Returns NMT_EINVAL if the scale
 * would fall below 2^-14. */
int nmt_scaler_update(float* scale /*host*/, int32_t* clean /*host*/, int32_t overflow, int32_t window);
/* Learning rate of update t (1-based) as in "Models and Hyperparameters": linear warm-up to `peak`
 * (5e-4, or 1e-3 with large batches) over `warmup` (4000) updates, then proportional to the inverse
 * square root of t. */
double nmt_lr_schedule(int64_t t, double peak, int64_t warmup);

/* Host only.  Debug export for the parity tests: the place, inside the caller's workspace, of an activation the
 * last forward call saved for its backward pass.  name: "enc<l>.ffn.h" / "dec<l>.ffn.h" (the feed-forward
 * hidden activation after ReLU and dropout, fp16 [rows, d_ff]; an element > 0 is an open ReLU gate) or
 * "enc<l>.out" / "dec<l>.out" (the block's output, fp16 [rows, d_model]); rows = source / target positions of
 * the pass, in its row order.  The memory stays the caller's; it is overwritten by the next forward call. */
int nmt_debug_activation(const nmt_ctx* ctx, const char* name, const void** d_ptr, int64_t* rows, int64_t* cols);

/* Host only.  Process-wide switches of launch forms, for tests and profiling; none of them changes a
 * result bit.  name: "gemm_group" (tile rows swept together, >= 1; default 4), "gemm_persist" (0: never the
 * persistent GEMM form / 1: for large products whose epilogue loads nothing per element; default 1),
 * "attn_persist" (0: one attention work item per work-group; default 1), "worklists" (0: attention
 * kernels enumerate every (sentence, tile); default 1), "one_stream" (1: nmt_backward enqueues the weight
 * gradients on the caller's stream; default 0), "gemm_share" (1..16, default 1: the number of products a
 * caller keeps running side by side on streams of its own; large tiles are then chosen as if each product had
 * that fraction of the compute units), "gemm_tile" (0: tile shape chosen per product, the default; 1..5: every
 * product that is not cut along k takes 256x256 / 128x128 / 128x64 / 64x128 / 64x64 tiles), "gemm_timing" (1: every GEMM product is bracketed by a pair of
 * HIP events on the stream it is launched on; default 0), "defaults" (value ignored: all of the above back to
 * default).  Unknown names and values out of range return NMT_EINVAL. */
int nmt_tuning(const char* name, int32_t value);
/* Host only; waits for the products concerned.  With "gemm_timing" on: the sum of the event-bracketed durations
 * (milliseconds) of the GEMM products launched since the last call, their number, and their algorithmic FLOPs
 * (2 M N K each); any of the three pointers may be NULL.  The measurement behind the benchmark's roofline figure. */
int nmt_gemm_timing(double* ms /*host*/, int64_t* products /*host*/, double* flops /*host*/);

/* ------------------------------------------------------------------------------------------
 * Kernel-level entry points (used by the per-kernel parity tests and by profiling).
 * ------------------------------------------------------------------------------------------ */

/* Dropout description for the kernels that draw masks.  Element (row r, column c) of a
 * [rows, n_cols] activation whose row r is position r % n_pos of sentence r / n_pos is kept iff
 * the 16-bit word  (Philox4x32-10(counter = (c >> 3, uid, site << 16 | pos, step << 8 | micro),
 * key = seed)[(c >> 1) & 3] >> 16 * (c & 1)) & 0xffff  is >= ceil(p * 2^16); kept values are
 * multiplied by 1 / (1 - p).  uid = d_sent_uid[sentence] or the sentence index if NULL. */
typedef struct {
  float p;
  uint32_t site, step, micro;
  uint64_t seed;
  int32_t n_pos;
  const uint32_t* d_sent_uid;
} nmt_dropout;

/* C[M,N] = epilogue(sum_k A(m,k) B(n,k)), fp16 operands, fp32 accumulation, fp16 result.
 * a_t == 0: A stored [M,K] (lda >= K); a_t != 0: stored [K,M] (lda >= M).
 * b_t == 0: B stored [N,K]; b_t != 0: stored [K,N].  The contiguous dimension of each operand,
 * N, and all leading dimensions must be multiples of 8; pointers 16-byte aligned.
 * Epilogue, in this order: + bias[n] (fp16, or NULL); ReLU if relu != 0; dropout if drop != NULL
 * and drop->p > 0; + add[m,n] (fp16 with leading dimension ldc, may alias C; or NULL);
 * if relu_src != NULL (fp16 [M,N], ld = ldc): result = relu_src > 0 ? result * mask_scale : 0. */
int nmt_op_gemm(const void* d_A, int32_t a_t, int32_t lda, const void* d_B, int32_t b_t, int32_t ldb,
                void* d_C, int32_t ldc, int32_t M, int32_t N, int32_t K, const void* d_bias,
                int32_t relu, const nmt_dropout* drop, const void* d_add, const void* d_relu_src,
                float mask_scale, void* stream);

/* The same product without epilogue, with the contraction cut into `splits` (1..64; 0 = chosen by
 * the library) equal pieces whose fp32 partial results go to d_partial (partial_floats >= splits *
 * M * N floats, 16-byte aligned) and are summed in increasing k order by a second kernel: the form
 * used for weight gradients, whose contraction runs over all positions of a pass. */
int nmt_op_gemm_splitk(const void* d_A, int32_t a_t, int32_t lda, const void* d_B, int32_t b_t, int32_t ldb,
                       void* d_C, int32_t ldc, int32_t M, int32_t N, int32_t K, float* d_partial,
                       int64_t partial_floats, int32_t splits, void* stream);

/* The same product with fp32 operands and an fp32 result, no epilogue: C[M,N] = sum_k A(m,k) B(n,k) on the fp32
 * matrix instructions.  Benchmark only -- the training step never calls it: it times what the step's products cost
 * without half precision ("Half-Precision Training" compares fp32 and fp16 training at equal settings; Table 1,
 * rows "Our reimplementation" and "16-bit").  Operands 16-byte aligned, leading dimensions multiples of 4.
 * splits (1..64) > 1 cuts the contraction into that many pieces (the form a weight gradient over many positions
 * needs to fill the chip): piece z writes its partial product to rows [z*M, (z+1)*M) of d_C, which then holds
 * splits * M rows; the caller sums them. */
int nmt_op_gemm_f32(const float* d_A, int32_t a_t, int32_t lda, const float* d_B, int32_t b_t, int32_t ldb,
                    float* d_C, int32_t ldc, int32_t M, int32_t N, int32_t K, int32_t splits, void* stream);

/* Masked multi-head attention forward.  Q [B*Tq, *] with row stride ldq (head h at columns
 * h*dh..), K, V [B*Tk, *]; O [B*Tq, *]; d_lse fp32 = log-sum-exp of the scaled
 * scores, stored [H, B*Tq] (head-major).  Key j of sentence b is hidden iff d_key_ids[b*Tk + j] == pad_id, or causal != 0 and
 * j > query index.  Scores are scaled by 1/sqrt(dh). */
int nmt_op_attention_fwd(const void* d_Q, int32_t ldq, const void* d_K, int32_t ldk, const void* d_V,
                         int32_t ldv, void* d_O, int32_t ldo, float* d_lse, const int32_t* d_key_ids,
                         int32_t pad_id, int32_t causal, int32_t B, int32_t H, int32_t dh, int32_t Tq,
                         int32_t Tk, void* stream);
/* Backward of the above: dQ, dK, dV from dO (and the forward's Q, K, V, O, lse). */
int nmt_op_attention_bwd(const void* d_Q, int32_t ldq, const void* d_K, int32_t ldk, const void* d_V,
                         int32_t ldv, const void* d_O, int32_t ldo, const void* d_dO, int32_t lddo,
                         const float* d_lse, void* d_dQ, int32_t lddq, void* d_dK, int32_t lddk,
                         void* d_dV, int32_t lddv, const int32_t* d_key_ids, int32_t pad_id,
                         int32_t causal, int32_t B, int32_t H, int32_t dh, int32_t Tq, int32_t Tk,
                         void* stream);

/* out = LayerNorm(resid + dropout(sub)) * gamma + beta per row of [rows, d] (fp16 in/out, fp32
 * math); d_stats fp32 [rows, 2] receives (mean, 1/sqrt(var + eps)). */
int nmt_op_residual_layernorm_fwd(const void* d_sub, const void* d_resid, const void* d_gamma,
                                  const void* d_beta, void* d_out, float* d_stats, int32_t rows,
                                  int32_t d, float eps, const nmt_dropout* drop, void* stream);
/* Backward: from d_dout (gradient at the LayerNorm output) computes d_dy (gradient at the
 * pre-normalisation sum), d_dym = dropout-masked d_dy (gradient at the sub-layer output),
 * and the fp16 vectors dgamma, dbeta and dbias = column sums of d_dym.  d_partial: fp32 scratch
 * of nmt_op_layernorm_bwd_scratch(d) floats. */
int64_t nmt_op_layernorm_bwd_scratch(int32_t d);
int nmt_op_residual_layernorm_bwd(const void* d_dout, const void* d_sub, const void* d_resid,
                                  const void* d_gamma, const float* d_stats, void* d_dy, void* d_dym,
                                  void* d_dgamma, void* d_dbeta, void* d_dbias, float* d_partial,
                                  int32_t rows, int32_t d, const nmt_dropout* drop, void* stream);

/* x[r, :] = dropout(sqrt(d) * E[ids[r], :] + PE(r % n_pos, :)), sinusoidal positions. */
int nmt_op_embed_fwd(const int32_t* d_ids, const void* d_E, void* d_x, int32_t rows, int32_t d,
                     int32_t vocab, const nmt_dropout* drop, void* stream);

/* Per row of fp16 logits [rows, V]: label-smoothed loss against d_targets (pad_id rows count
 * nothing), written to d_row_loss (fp32 [rows]); logits are overwritten in place by
 * loss_scale * (softmax - smoothed target) (zeros on pad rows).  Then *d_loss_sum, *d_ntok are
 * reduced deterministically. */
int nmt_op_softmax_xent(void* d_logits, const int32_t* d_targets, float* d_row_loss, int32_t rows,
                        int32_t V, int32_t pad_id, float label_smoothing, float loss_scale,
                        float* d_loss_sum, int32_t* d_ntok, void* stream);

/* dst[c] = fp16(sum_r src[r, c]) for fp16 src [rows, cols] (ld); d_partial: fp32 scratch of
 * nmt_op_colsum_scratch(cols) floats. */
int64_t nmt_op_colsum_scratch(int32_t cols);
int nmt_op_colsum(const void* d_src, int32_t ld, void* d_dst, float* d_partial, int32_t rows,
                  int32_t cols, void* stream);

/* nmt_op_colsum for callers that cannot allocate device memory and have no scratch buffer to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and same
 * result bits; the partial sums live in a fixed device array of the library (8 MiB per GPU, held until the
 * process ends) instead of d_partial, so cols is limited to 4096 (NMT_EINVAL beyond that, before anything
 * is launched).  The call allocates and frees nothing.  All calls on one GPU share the array: calls that
 * overlap on one GPU (different streams) race; calls on one stream are ordered and need no clearing in
 * between (every partial sum read is written by the same call first). */
int nmt_op_colsum_static(const void* d_src, int32_t ld, void* d_dst, int32_t rows, int32_t cols, void* stream);

/* Embedding backward: d_gE[v, :] = fp16(float(d_gE[v, :]) + sqrt(d) * sum over positions r with
 * ids[r] == v of dropout-masked d_dx[r, :]), for two id streams (source then target) at once.
 * Deterministic: every sum is formed in a fixed order (increasing position within blocks of 64
 * positions of an id, then block after block).  d_scratch: 16-byte aligned int32 scratch of
 * nmt_op_embed_bwd_scratch(vocab, rows_a + rows_b, d) int32 elements.  vocab <= 65536. */
int64_t nmt_op_embed_bwd_scratch(int32_t vocab, int32_t rows_total, int32_t d);
int nmt_op_embed_bwd(const int32_t* d_ids_a, const void* d_dx_a, int32_t rows_a, const nmt_dropout* drop_a,
                     const int32_t* d_ids_b, const void* d_dx_b, int32_t rows_b, const nmt_dropout* drop_b,
                     void* d_gE, int32_t d, int32_t vocab, int32_t* d_scratch, void* stream);

/* Element-wise update kernels on n scalars (the bodies of nmt_accumulate, nmt_check_overflow
 * and nmt_adam_step). */
int nmt_op_accumulate(const void* d_g16, float* d_acc32, int64_t n, int32_t first, void* stream);
/* nmt_op_check_overflow is the single-pass form that also unscales in place: *d_flag as above and
 * d_acc32 *= inv_scale.  nmt_op_adam updates with d_g32 * grad_scale. */
int nmt_op_check_overflow(float* d_acc32, int64_t n, float inv_scale, int32_t* d_flag, void* stream);
int nmt_op_adam(float* d_master32, float* d_m, float* d_v, const float* d_g32, float grad_scale, void* d_w16, int64_t n,
                float lr, float beta1, float beta2, float eps, int32_t t, const int32_t* d_flag,
                void* stream);

/* Writes the dropout keep decisions (1 / 0 bytes) of a [rows, n_cols] activation. */
int nmt_op_dropout_mask(uint8_t* d_keep, int32_t rows, int32_t n_cols, const nmt_dropout* drop,
                        void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NMT_H_ */
