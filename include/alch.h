/*
 * alch.h -- C ABI of the activation-reuse training hot path for AMD MI355X (gfx950).
 *
 * Method (Alchemist, arXiv 2503.01066): the activations a model produces while it
 * serves a prompt are the ones a training forward pass over the same prompt would
 * produce, so online continual training can skip that forward pass and start
 * back-propagation from them (Section 1; Section 2.5.1; requirement R1 in
 * Section 3).  Two kernel families implement the device side of that statement:
 *
 *   1. capture/pack  -- while the prompt is prefilled, the per-layer activations of
 *      the tokens that are to be trained on are gathered into dense per-layer
 *      records (Section 4.1: record only in the prefill phase; Section 5: every saved
 *      tensor is tagged with the layer that owns it).
 *   2. backward from the saved record -- the decoder-layer backward pass, one layer
 *      at a time from the output layer to the input layer (Section 4.2: the trainer
 *      can be pre-empted at the start of each layer's backward; Section 4.3.2: layers
 *      are consumed in reverse order), topped by the cross-entropy loss on the saved
 *      prefill output (Section 5, Section 6 "Training").
 *
 * The paper trains Llama-3.1-8B, Mistral and Phi-4 (Section 6): pre-norm decoder
 * layers with RMSNorm, rotary position embedding, grouped-query causal attention and
 * a SwiGLU MLP.  The paper prints no formulas; the layer function is
 *
 *   h1 = x * rsqrt(mean(x^2) + eps) * g1
 *   q = RoPE(h1 Wq^T)   k = RoPE(h1 Wk^T)   v = h1 Wv^T
 *   o = softmax_causal(q k^T / sqrt(D)) v          (query head h reads kv head h / (Hq/Hkv))
 *   x2 = x + o Wo^T      h2 = x2 * rsqrt(mean(x2^2) + eps) * g2
 *   y = x2 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T
 *
 * with RoPE pairing element i with i + D/2 at angle position * base^(-2i/D).
 * The saved record of a layer is { X, X2, Q, K, V, O, LSE, G, U }: layer input, the
 * post-attention residual stream, Q and K after RoPE (what a KV cache holds, Section
 * 4.1), V, the attention output, the natural-log softmax normaliser per (token, query
 * head), and the gate / up projections before the activation.
 *
 * General conventions
 *   - Every pointer is DEVICE memory unless marked "host".  The caller owns every
 *     buffer, including the workspace; the library allocates no device memory.  It keeps
 *     no state between calls with two exceptions, both opt-in: the launch trace
 *     (alch_trace_enable / alch_trace_collect: a process-wide list of HIP events, guarded by
 *     a mutex) and the built-in scratch of alch_capture_pack_static (one 64 KiB device
 *     array per GPU).  Neither changes any result.
 *   - Every call validates its arguments on the host first, then enqueues kernels on
 *     `hip_stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *     returns without synchronising.  ALCH_OK means "enqueued".
 *   - Activations are packed row-major [tokens, width], heads contiguous inside a row
 *     ([T, heads, D]).  Weights are row-major [out, in] (y = x W^T).  Base pointers must
 *     be 16-byte aligned.
 *   - Errors: negative alch_status; a human-readable message for the calling thread is
 *     returned by alch_last_error().  No C++ exception crosses this boundary.
 */
#ifndef ALCH_H
#define ALCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ALCH_OK = 0,
    ALCH_ERR_INVALID_ARG = -1, /* NULL / misaligned pointer, negative size, bad enum */
    ALCH_ERR_SHAPE = -2,       /* inconsistent or unsupported dimensions */
    ALCH_ERR_WORKSPACE = -3,   /* workspace missing or smaller than the *_workspace_bytes query */
    ALCH_ERR_STALE = -4,       /* record captured under other weights than the ones passed */
    ALCH_ERR_UNSUPPORTED = -5, /* valid request that this build does not implement */
    ALCH_ERR_HIP = -6,         /* a HIP runtime call failed (message has the HIP error string) */
    ALCH_ERR_ABORTED = -7      /* the preempt hook asked to stop */
} alch_status;

typedef enum { ALCH_F32 = 0, ALCH_BF16 = 1 } alch_dtype;

/* Decoder-layer dimensions.  n_q_heads must be a multiple of n_kv_heads, head_dim even.
 * dtype is the storage type of every activation, weight and gradient (LSE is always
 * fp32); arithmetic accumulates in fp32. */
typedef struct {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn;
    float rms_eps, rope_base;
    alch_dtype dtype;
} alch_layer_shape;

/* A ragged batch of prompts laid end to end (Section 4.1: the prefill batch).
 *
 * Shared prefixes (Section 4.1, preference alignment: the responses attend to the saved KV cache of their
 * prompt, and the chosen and the rejected response share it).  With seq_prefix given, sequence s with
 * p = seq_prefix[s] >= 0 attends to every token of sequence p and causally to its own tokens; sequence p
 * must come earlier in the batch and have no prefix itself (seq_prefix[p] = -1).  Everything else of a
 * layer is row-local and unchanged.  The keys and values of p then receive gradient from the sequences
 * that attend to them.  positions must be given with seq_prefix (a response token i sits at position
 * len(p) + i); at most 4096 sequences.  seq_prefix == NULL: every sequence stands alone. */
typedef struct {
    int32_t n_seqs, total_tokens, max_seqlen;
    const int32_t* cu_seqlens; /* device [n_seqs+1]: cu[0]=0, non-decreasing, cu[n_seqs]=total_tokens */
    const int32_t* positions;  /* device [total_tokens] RoPE positions, or NULL => index inside the sequence */
    const int32_t* cu_seqlens_host; /* host copy of cu_seqlens (same values); used for validation and
                                       launch planning so that no call has to read device memory */
    const int32_t* seq_prefix;      /* device [n_seqs] or NULL */
    const int32_t* seq_prefix_host; /* host copy of seq_prefix (NULL exactly when seq_prefix is NULL) */
} alch_batch;

/* ------------------------------------------------------------------------------------
 * Family 1: capture/pack (Section 4.1 "Record and cache activation"; Section 5).
 *
 * One source/destination pair of the gather.  `src` has one row per token of the batch,
 * rows `src_row_stride_bytes` apart (so a stream may be a column slice of a fused
 * buffer, e.g. Q inside [T, (Hq+2Hkv) D]); `dst` is dense, rows `row_bytes` apart.
 * row_bytes must be a multiple of 4; row_bytes, the stride and both pointers multiples of
 * 16 take the fast path.
 */
typedef struct {
    const void* src;
    void* dst;
    size_t row_bytes;
    size_t src_row_stride_bytes;
} alch_stream; /* the array of these lives in HOST memory */

/*
 * alch_capture_pack: kept = ascending list of tokens t with keep_mask[t] != 0;
 *   kept_index[r] = kept[r];  cu_kept[s] = #{t in kept : t < cu_seqlens[s]};
 *   for every stream k and r < n_kept: dst_k[r, :] = src_k[kept[r], :]  (bit-for-bit).
 * The result is unique, so it is deterministic and bit-exact.
 *
 *   keep_mask          device uint8 [total_tokens]; any nonzero byte keeps the token
 *   n_streams, streams host array of n_streams descriptors (may be 0 streams: index only)
 *   dst_capacity_rows  rows every dst (and kept_index) can hold.  If n_kept exceeds it,
 *                      nothing beyond the capacity is written and n_kept_and_status[1] = 1.
 *   kept_index         device out int32 [dst_capacity_rows]
 *   cu_kept            device out int32 [n_seqs+1]
 *   n_kept_and_status  device out int32 [2]: { n_kept, overflow flag }
 *   workspace          device scratch of at least alch_capture_pack_workspace_bytes(T) bytes
 * Empty batches, empty sequences, all-zero and all-one masks are legal.
 */
int alch_capture_pack(const alch_batch* batch, const uint8_t* keep_mask, int32_t n_streams,
                      const alch_stream* streams, int64_t dst_capacity_rows, int32_t* kept_index,
                      int32_t* cu_kept, int32_t* n_kept_and_status, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

size_t alch_capture_pack_workspace_bytes(int32_t total_tokens);

/*
 * alch_capture_gather: the gather of alch_capture_pack alone, for further streams of the same batch and
 * mask (Section 4.1: one prefill batch is recorded layer after layer; which tokens are kept does not change
 * from layer to layer, so the mask is scanned once).  kept_index and n_kept_and_status are the device
 * outputs of an earlier alch_capture_pack on this batch, complete in stream order before this call; for every
 * stream k and r < min(n_kept, dst_capacity_rows): dst_k[r, :] = src_k[kept_index[r], :]  (bit-for-bit).
 * dst_capacity_rows must not exceed the capacity that earlier call was given.
 */
int alch_capture_gather(const alch_batch* batch, int32_t n_streams, const alch_stream* streams,
                        int64_t dst_capacity_rows, const int32_t* kept_index,
                        const int32_t* n_kept_and_status, void* hip_stream);

/*
 * alch_capture_pack_static: alch_capture_pack for callers that cannot allocate or hand over device
 * scratch: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error behaviour, minus the workspace: the scan's block counters live in a
 * 64 KiB array inside the library's device image (one copy per GPU, held until the process ends).
 * The call allocates nothing and frees nothing.
 *   - total_tokens above alch_capture_pack_static_max_tokens() (about 66.8 million) is rejected with
 *     ALCH_ERR_UNSUPPORTED before anything is enqueued; use alch_capture_pack with a workspace then.
 *   - every call on a GPU shares that GPU's array, on whatever stream: calls that overlap in time on
 *     one GPU race on it.  Calls in stream order on one stream are safe, and nothing has to be cleared
 *     between them (each call overwrites every counter it later reads).
 *   - the device that is current at the call is the one whose array is used; it must be the device of
 *     the buffers and of hip_stream.
 */
int alch_capture_pack_static(const alch_batch* batch, const uint8_t* keep_mask, int32_t n_streams,
                             const alch_stream* streams, int64_t dst_capacity_rows, int32_t* kept_index,
                             int32_t* cu_kept, int32_t* n_kept_and_status, void* hip_stream);
size_t alch_capture_pack_static_max_tokens(void);

/* ------------------------------------------------------------------------------------
 * Family 2: backward from saved activations (Section 1; Section 4.2; Section 4.3.2).
 */

/* The saved record of one layer (all [total_tokens, width], dtype of the shape):
 * X, X2 [T,hidden]; Q, O [T,n_q_heads*head_dim]; K, V [T,n_kv_heads*head_dim];
 * G, U [T,ffn]; LSE fp32 [T,n_q_heads].  weights_version tags the weights the record
 * was produced under: gradients from a record are only valid at those weights.
 * X2, O and LSE may be NULL (a record of the six streams X, Q, K, V, G, U): the backward calls then
 * recompute O and LSE by an attention forward on the saved Q, K, V and X2 = X + O Wo^T, the
 * recompute-instead-of-load choice of Section 4.3.2.  G and U may be NULL as well (a record of the
 * layer input, the query and the KV cache alone): they are recomputed as H2 Wg^T and H2 Wu^T from
 * the normalised X2, on the kept rows only under a loss mask.  Not supported for a projection that
 * carries an adapter (ALCH_ERR_UNSUPPORTED). */
typedef struct {
    const void *X, *X2, *Q, *K, *V, *O, *G, *U;
    const float* LSE;
    uint64_t weights_version;
} alch_saved;

/* Wq [Hq*D,hidden], Wk,Wv [Hkv*D,hidden], Wo [hidden,Hq*D], Wg,Wu [ffn,hidden],
 * Wd [hidden,ffn], g1,g2 [hidden]. */
typedef struct {
    const void *Wq, *Wk, *Wv, *Wo, *Wg, *Wu, *Wd, *g1, *g2;
    uint64_t weights_version;
} alch_weights;

/* Gradient outputs, same shapes and dtype as the weights.  A NULL member is skipped
 * (frozen parameter; Section 3 assumption A1 trains adapters on a frozen base).
 * accumulate != 0 adds to what the buffer holds (sum in fp32, one rounding). */
typedef struct {
    void *dWq, *dWk, *dWv, *dWo, *dWg, *dWu, *dWd, *dg1, *dg2;
    int32_t accumulate;
} alch_wgrads;

/*
 * alch_layer_backward: gradients of one decoder layer from its saved record.
 *   dY        [T,hidden] gradient w.r.t. the layer output
 *   loss_mask device uint8 [T] or NULL; where 0 the dY row is treated as zero
 *   dX        [T,hidden] out: gradient w.r.t. the layer input (may alias dY)
 *   wgrads    may be NULL (no weight gradients at all)
 * Every record tensor is consumed as given: probabilities are exp(q.k/sqrt(D) - LSE)
 * from the saved Q, K, LSE; nothing is recomputed from X and the weights except the
 * cheap row-wise normalisations and the MLP activation.  saved->weights_version must
 * equal weights->weights_version, else ALCH_ERR_STALE.
 * Results match the fp64 definition to max|err| / max|ref| <= 2e-2 (bf16) or 1e-4 (f32)
 * per output tensor.
 */
int alch_layer_backward(const alch_layer_shape* shape, const alch_batch* batch,
                        const alch_saved* saved, const alch_weights* weights, const void* dY,
                        const uint8_t* loss_mask, void* dX, const alch_wgrads* wgrads,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

size_t alch_layer_backward_workspace_bytes(const alch_layer_shape* shape, int32_t total_tokens,
                                           int32_t max_seqlen);

/* ------------------------------------------------------------------------------------
 * Low-rank adapters on the projections (Section 3, assumption A1: the system trains with
 * parameter-efficient fine-tuning such as LoRA on a frozen base; Section 6, "Training": the
 * evaluated models carry an adapter of rank 8).
 *
 * Projection p (order q, k, v, o, g, u, d) computes y = x W_p^T + scale * (x A_p^T) B_p^T with
 * A_p [rank, in_p] and B_p [out_p, rank], row-major, dtype of the shape.  A NULL pair means the
 * projection carries no adapter.  The saved record is the one the serving forward produced with
 * the adapters attached (Q, K, V, O, G, U contain the low-rank terms).
 * rank: multiple of 8, 8..64; every projection width must be a multiple of 8. */
enum { ALCH_PROJ_Q = 0, ALCH_PROJ_K, ALCH_PROJ_V, ALCH_PROJ_O, ALCH_PROJ_G, ALCH_PROJ_U, ALCH_PROJ_D, ALCH_N_PROJ };
typedef struct {
    int32_t rank;
    float scale;               /* alpha / rank of the LoRA formulation */
    const void* A[ALCH_N_PROJ];
    const void* B[ALCH_N_PROJ];
} alch_lora;

/* Adapter gradients, same shapes as A and B; a NULL member is skipped; accumulate as in alch_wgrads. */
typedef struct {
    void* dA[ALCH_N_PROJ];
    void* dB[ALCH_N_PROJ];
    int32_t accumulate;
} alch_lora_grads;

/*
 * alch_layer_backward_lora: alch_layer_backward for a layer with adapters.
 *   dX includes the low-rank paths (dx = dy W + scale (dy B) A for every adapted projection);
 *   wgrads may be NULL or hold NULL members: the frozen base of Section 3 A1 (then only the
 *   data-gradient products run: 2 flops per parameter and token instead of 4);
 *   lora_grads->dA[p] = scale * (dy_p B_p)^T x_p, dB[p] = scale * dy_p^T (x_p A_p^T).
 * The rank-r intermediates x A^T and dy B are rounded to the storage dtype once.
 * Same parity bar as alch_layer_backward.  Workspace: alch_layer_backward_lora_workspace_bytes.
 */
int alch_layer_backward_lora(const alch_layer_shape* shape, const alch_batch* batch,
                             const alch_saved* saved, const alch_weights* weights, const alch_lora* lora,
                             const void* dY, const uint8_t* loss_mask, void* dX, const alch_wgrads* wgrads,
                             const alch_lora_grads* lora_grads, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

size_t alch_layer_backward_lora_workspace_bytes(const alch_layer_shape* shape, int32_t total_tokens,
                                                int32_t max_seqlen, int32_t rank);


/* Host callbacks of the stack walk (Section 4.2: a hook at the start of each layer's
 * backward lets serving pre-empt training; Section 4.3.2: a layer's activations may
 * still be on their way back to the GPU).  layer_ready(user, l) is called before layer
 * l's kernels are enqueued and may block; it returns 0 to go on.  preempt(user, l)
 * returning nonzero stops the walk before layer l: the call returns ALCH_ERR_ABORTED
 * with layers above l already enqueued. */
typedef struct {
    int (*layer_ready)(void* user, int layer);
    int (*preempt)(void* user, int layer);
    void* user;
} alch_hooks;

/*
 * alch_stack_backward: cross-entropy loss on the saved stack output and the backward
 * walk over all layers (Section 5: loss from the prefill output and the prompt text).
 *   saved, weights, wgrads  HOST arrays of n_layers structs (wgrads may be NULL)
 *   X_final   [T,hidden] output of the last layer (the saved prefill output)
 *   g_final   [hidden] gain of the final RMSNorm;  W_lm [vocab,hidden]
 *   labels    device int32 [T]; a position counts if 0 <= label < vocab (and loss_mask != 0); any other label,
 *             negative or beyond the vocabulary, marks a position that is ignored
 *   loss = -(1/N) sum_counted log softmax(RMSNorm(X_final) W_lm^T)[label]; N = 0 gives
 *          loss 0 and zero gradients.  Logits are produced and consumed in row chunks and
 *          never stored whole.
 *   dg_final, dW_lm  out (NULL => skipped; `accumulate` of wgrads[0] applies, 0 if wgrads NULL)
 *   dX_embed  [T,hidden] out: gradient w.r.t. the input of layer 0
 *   loss_out  device float [1] out
 */
int alch_stack_backward(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab,
                        const alch_batch* batch, const alch_saved* saved, const alch_weights* weights,
                        const void* X_final, const void* g_final, const void* W_lm,
                        const int32_t* labels, const uint8_t* loss_mask, const alch_wgrads* wgrads,
                        void* dg_final, void* dW_lm, void* dX_embed, float* loss_out,
                        const alch_hooks* hooks, void* workspace, size_t workspace_bytes,
                        void* hip_stream);

size_t alch_stack_backward_workspace_bytes(const alch_layer_shape* shape, int32_t n_layers,
                                           int32_t vocab, int32_t total_tokens, int32_t max_seqlen);

/*
 * alch_stack_backward_lora: alch_stack_backward for a stack whose layers carry low-rank adapters
 * (Section 3 assumption A1, Section 6).  lora, lora_grads: HOST arrays of n_layers entries, the same
 * rank in every layer; lora_grads may be NULL.  The head carries no adapter.  With wgrads == NULL,
 * dg_final == NULL and dW_lm == NULL this is the paper's training setting: frozen base, adapter
 * gradients only.
 */
int alch_stack_backward_lora(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab,
                             const alch_batch* batch, const alch_saved* saved, const alch_weights* weights,
                             const alch_lora* lora, const void* X_final, const void* g_final, const void* W_lm,
                             const int32_t* labels, const uint8_t* loss_mask, const alch_wgrads* wgrads,
                             const alch_lora_grads* lora_grads, void* dg_final, void* dW_lm, void* dX_embed,
                             float* loss_out, const alch_hooks* hooks, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

size_t alch_stack_backward_lora_workspace_bytes(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab,
                                                int32_t total_tokens, int32_t max_seqlen, int32_t rank);

/*
 * alch_stack_backward_dpo: alch_stack_backward[_lora] with the DPO loss (Section 6: the example loss of
 * preference alignment) in place of cross-entropy, for batches whose responses share the saved prefill of
 * their prompt (batch->seq_prefix, Section 4.1).
 *
 * A scored token is an item m: the log-probability of item_label[m] under the LM-head row computed from
 * stack-output row item_row[m] adds to pi[item_slot[m]]; slots 2p and 2p+1 are the chosen and the rejected
 * response of pair p.  The first token of a response is scored from the last row of its prompt, so that
 * row carries one item per response.  With
 *     z_p = beta * [(pi[2p] - ref_logp[2p]) - (pi[2p+1] - ref_logp[2p+1])]
 * the loss is the mean over pairs of -log sigmoid(z_p); ref_logp are the same sums under the frozen
 * reference model (an input).  Items with a label outside 0..vocab-1 or a slot outside 0..2*n_pairs-1
 * score nothing.  item_row must be ascending (equal rows adjacent); item_row_host is its host copy, used
 * for validation.  n_items <= total_tokens.  z_out (device [n_pairs]) may be NULL.
 * lora / lora_grads may be NULL (no adapters); every other argument and the workspace size are those of
 * alch_stack_backward_lora (alch_stack_backward when lora == NULL).
 */
typedef struct {
    int32_t n_items, n_pairs;
    const int32_t *item_row, *item_label, *item_slot; /* device [n_items] */
    const int32_t* item_row_host;                      /* host [n_items] */
    const float* ref_logp;                             /* device [2*n_pairs] */
    float beta;
    float* z_out;                                      /* device [n_pairs] or NULL */
} alch_dpo;

int alch_stack_backward_dpo(const alch_layer_shape* shape, int32_t n_layers, int32_t vocab,
                            const alch_batch* batch, const alch_saved* saved, const alch_weights* weights,
                            const alch_lora* lora, const void* X_final, const void* g_final, const void* W_lm,
                            const alch_dpo* dpo, const alch_wgrads* wgrads, const alch_lora_grads* lora_grads,
                            void* dg_final, void* dW_lm, void* dX_embed, float* loss_out, const alch_hooks* hooks,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * alch_layer_forward: the forward pass of one layer, writing Y and the full record.
 * It is the producer side of the record (what serving prefill computes, Section 4.1) and
 * the "recompute" leg of the comparison in Section 6; record_out members are written,
 * X is copied from the input pointer only if record_out->X differs from it.
 */
typedef struct {
    void *X, *X2, *Q, *K, *V, *O, *G, *U;
    float* LSE;
} alch_record_out;

int alch_layer_forward(const alch_layer_shape* shape, const alch_batch* batch, const void* X,
                       const alch_weights* weights, void* Y, const alch_record_out* record_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

size_t alch_layer_forward_workspace_bytes(const alch_layer_shape* shape, int32_t total_tokens,
                                          int32_t max_seqlen);

/*
 * alch_layer_forward_from: alch_layer_forward for the sequences seq_begin .. n_seqs-1 only, i.e. rows
 * cu_seqlens[seq_begin] .. total_tokens-1 of X, Y and every record_out member (all of them
 * [total_tokens, width]; earlier rows are neither read nor written, except that the attention reads
 * record_out->K and record_out->V of the prefix sequences named by batch->seq_prefix).  This is the
 * forward over the response tokens alone on the saved KV cache of their prompts (Section 4.1,
 * preference alignment): the prompts' rows of the record come from serving, the responses' rows from
 * this call.  batch->positions must be given when seq_begin > 0.  The workspace is that of
 * alch_layer_forward for the rows computed (the bound for total_tokens always suffices).
 */
int alch_layer_forward_from(const alch_layer_shape* shape, const alch_batch* batch, int32_t seq_begin,
                            const void* X, const alch_weights* weights, void* Y,
                            const alch_record_out* record_out, void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/*
 * alch_gemm: the dense contraction every projection gradient of the per-layer backward
 * (Section 4.2 / 4.3.2) is made of, exposed for tests and for timing single launches:
 *   C[M,N] (+)= sum_i A_i(M,K_i) B_i(K_i,N),  fp32 accumulation, C row-major with stride ldc.
 *   a_kmajor != 0: A_i(m,k) = A_i[m*lda + k], else A_i(m,k) = A_i[k*lda + m]
 *   b_kmajor != 0: B_i(k,n) = B_i[n*ldb + k], else B_i(k,n) = B_i[k*ldb + n]
 * (data gradient: a_kmajor=1, b_kmajor=0; weight gradient: both 0; forward projection: both 1).
 * terms is a HOST array of 1..4 operand pairs.  bf16 problems with 16-byte aligned operands and
 * leading dimensions that are multiples of 8 run on the matrix cores; anything else takes a plain
 * fp32 kernel.
 */
typedef struct {
    const void* A;
    const void* B;
    int32_t K;
    int64_t lda, ldb;
} alch_gemm_term;

int alch_gemm(alch_dtype dtype, int32_t M, int32_t N, int32_t a_kmajor, int32_t b_kmajor, int32_t n_terms,
              const alch_gemm_term* terms, void* C, int64_t ldc, int32_t accumulate, void* hip_stream);

/*
 * alch_gemm_ws: alch_gemm with device scratch of alch_gemm_workspace_bytes() bytes (16-byte aligned; NULL
 * gives alch_gemm).  The matrix-core kernel walks the 256x256 output tiles in rounds of one tile per compute
 * unit; with scratch, a single-term product whose last round holds tiles for at most half of the compute
 * units splits each of those tiles along the contraction over several work-groups (fp32 partial tiles in the
 * scratch, added in a fixed order by a second kernel), as the weight-gradient products of the backward entry
 * points do.  The result is deterministic; it differs from alch_gemm's only in fp32 summation order.
 */
int alch_gemm_ws(alch_dtype dtype, int32_t M, int32_t N, int32_t a_kmajor, int32_t b_kmajor, int32_t n_terms,
                 const alch_gemm_term* terms, void* C, int64_t ldc, int32_t accumulate, void* workspace,
                 size_t workspace_bytes, void* hip_stream);
size_t alch_gemm_workspace_bytes(void);

/*
 * alch_attention_forward: causal grouped-query attention over saved (post-RoPE) Q, K and V,
 * writing O [T,Hq*D] and LSE fp32 [T,Hq].  It is the step of the prefill that defines the LSE
 * and O members of the record (Section 4.1); exposed so that a record can be completed from
 * its Q, K, V alone.
 */
int alch_attention_forward(const alch_layer_shape* shape, const alch_batch* batch, const void* Q,
                           const void* K, const void* V, void* O, float* LSE, void* hip_stream);

/*
 * Launch timing for benchmarks.  While enabled, the library brackets its main kernels with two
 * HIP events on the caller's stream; alch_trace_collect waits for them, writes up to max_records
 * records (HOST array) in launch order, and forgets them.  flops / bytes are the algorithmic
 * work of the launch (2*M*N*K for a contraction; rows read once + written once for the gather).
 * The trace is process-wide state of the library (the only state besides the scratch of
 * alch_capture_pack_static); the switch is atomic and the record list is guarded by a mutex, so
 * calls from several threads are safe, but their records interleave.  Each traced launch creates
 * and records two HIP events, so timings taken with the trace on include that host-side cost.
 */
typedef enum {
    ALCH_TRACE_GEMM_MFMA = 0, ALCH_TRACE_GEMM_GENERIC = 1, ALCH_TRACE_PACK_SCAN = 2,
    ALCH_TRACE_PACK_GATHER = 3, ALCH_TRACE_ATTN_BWD = 4, ALCH_TRACE_ATTN_FWD = 5,
    ALCH_TRACE_ROW_OPS = 6, ALCH_TRACE_CROSS_ENTROPY = 7, ALCH_TRACE_LORA = 8
} alch_trace_kind;
typedef struct {
    int32_t kind; /* alch_trace_kind */
    double flops, bytes;
    float ms;
} alch_trace_record;
int alch_trace_enable(int32_t enable);
int alch_trace_collect(alch_trace_record* out, int32_t max_records, int32_t* n_out);

/* Message describing the last error on the calling thread ("" if none). */
const char* alch_last_error(void);

/* Library version string (static storage). */
const char* alch_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ALCH_H */
