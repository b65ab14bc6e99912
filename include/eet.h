/*
 * eet.h -- C ABI of the MI355X-native decoder-layer hot path of EET (arXiv 2104.12470).
 *
 * The library implements one pre-LN GPT-2 style decoder layer with mask fusion (Section 2.1,
 * Algorithm 1): no attention-mask or padding-mask tensor is ever built; causality is an index
 * comparison between query and key position, and padding tokens are skipped, not masked.
 * Prompts are processed whole (Section 4.1: every sequence at its own length, the batch at the
 * maximum length); generation is incremental over a K/V cache that is sized once for the
 * maximum batch and sequence length (Section 3.1).  Row-wise kernels (softmax, LayerNorm,
 * add-bias/GELU/residual) handle rows of any width (the goal of Section 2.2).
 * Around the layer: a stack of layers driven by one call per step, the model around the stack
 * (token ids in, logits and the greedy next token out), the operators one by one, and the buffer
 * manager of Section 3.2.
 *
 * Conventions
 *   - All tensors are fp16 (IEEE binary16) in DEVICE memory unless a parameter says HOST.
 *     Accumulation and statistics are fp32.  Row-major, innermost dimension contiguous,
 *     base pointers 16-byte aligned.
 *   - Sequences are right-padded: sequence b has q_lens[b] valid rows [0, q_lens[b]) out of
 *     padded_len; the paper's per-sequence padding length is padded_len - q_lens[b].  The entry
 *     points named *_left_padded take the layout Algorithm 1 is printed for instead (valid rows
 *     padded_len - q_lens[b] .. padded_len - 1).
 *   - The library never allocates, frees or synchronises device memory: workspace, K/V cache,
 *     weights, inputs and outputs are the caller's.  Every call only enqueues work on the
 *     given hipStream_t (passed as void*; NULL = default stream), except eet_cache_lens (and
 *     eet_model_create, which clears a few KB of its workspace with a blocking memset).
 *   - Return value: EET_OK or a negative error code.  On error nothing has been enqueued and
 *     no state has changed; eet_last_error() describes the failure (thread-local storage).
 *   - Calls on one layer handle must not overlap in time (one stream at a time).
 */
#ifndef EET_H
#define EET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EET_OK                      0
#define EET_ERR_INVALID_ARG        (-1)  /* null pointer, non-positive size, length out of range   */
#define EET_ERR_UNSUPPORTED_SHAPE  (-2)  /* head size not 64/128, width not a multiple of 64, ...   */
#define EET_ERR_CAPACITY           (-3)  /* batch/prompt/sequence exceeds what the layer was sized for */
#define EET_ERR_STATE              (-4)  /* decode before prefill, batch mismatch                  */
#define EET_ERR_HIP                (-5)  /* a HIP runtime call failed                              */

#define EET_MAX_BATCH 128                /* per-sequence lengths travel as kernel arguments        */

typedef struct eet_layer eet_layer_t;    /* opaque, host memory owned by the library               */
typedef struct eet_bufmgr eet_bufmgr_t;  /* buffer manager of Section 3.2 (declared at the end of this header) */

/* Layer shape and capacity: the paper's h, n, and maximum b, p, s (Section 3.1 notation). */
typedef struct {
    int32_t hidden;       /* h: model width; hidden = heads * d with d in {64, 128}              */
    int32_t heads;        /* n                                                                    */
    int32_t ffn;          /* feed-forward width, multiple of 64                                   */
    int32_t max_batch;    /* b, 1..EET_MAX_BATCH                                                  */
    int32_t max_prompt;   /* p: largest padded prompt length                                      */
    int32_t max_seq;      /* s: K/V cache capacity per sequence (prompt + generated), >= max_prompt */
    float   ln_eps;       /* LayerNorm epsilon (1e-5 for GPT-2)                                   */
} eet_layer_config;

/* DEVICE fp16 parameters, BORROWED for the life of the layer.  Linear weights are row-major
 * [out, in].  w_qkv is [3*hidden, hidden]: rows [0,h) produce Q, [h,2h) K, [2h,3h) V; head g
 * owns rows g*d .. (g+1)*d-1 of each block. */
typedef struct {
    const void *ln1_g, *ln1_b;      /* [hidden]                 */
    const void *w_qkv, *b_qkv;      /* [3*hidden, hidden], [3*hidden] */
    const void *w_o,   *b_o;        /* [hidden, hidden], [hidden]     */
    const void *ln2_g, *ln2_b;      /* [hidden]                 */
    const void *w_fc1, *b_fc1;      /* [ffn, hidden], [ffn]     */
    const void *w_fc2, *b_fc2;      /* [hidden, ffn], [hidden]  */
} eet_layer_weights;

/* Bytes of one layer's K/V cache: 2 * max_batch * hidden * max_seq fp16 elements (Section 3.1,
 * the K/V cache size formula with l = 1).  Layout: [2 (K,V)][max_batch][heads][max_seq][d];
 * slot t of sequence b holds token t of that sequence.  Returns 0 on a bad config. */
size_t eet_kv_cache_bytes(const eet_layer_config *cfg);

/* Bytes of caller-provided workspace a layer needs (activation buffers for max_batch*max_prompt
 * packed tokens, split-attention partials, per-sequence lengths; the pre-sized buffers of
 * Section 3).  Returns 0 on a bad config. */
size_t eet_workspace_bytes(const eet_layer_config *cfg);

/* Create a layer (Section 3.1: everything a pass needs is sized once, for the maximum batch, prompt and
 * sequence length, before the first call, so that no call allocates).  `workspace` is DEVICE memory of
 * eet_workspace_bytes(cfg), 256-byte aligned, owned by the caller and used exclusively by this layer until
 * eet_layer_destroy; weights are borrowed.  All of it must be ready (filled, uploaded) on the stream a later
 * call is given: the library orders nothing against other streams.  Nothing is enqueued.
 * Errors: INVALID_ARG (null, misaligned), UNSUPPORTED_SHAPE. */
int eet_layer_create(const eet_layer_config *cfg, const eet_layer_weights *weights,
                     void *workspace, eet_layer_t **out_layer);

/* Prefill (whole-prompt pass; Sections 2.1 and 4.1).
 *   q_lens     HOST int32[batch], 1 <= q_lens[b] <= padded_len (read before the call returns)
 *   tokens     DEVICE fp16 [batch, padded_len, hidden] input hidden states; pad rows are never read
 *   out        DEVICE fp16 [batch, padded_len, hidden]; valid rows = layer output, pad rows = 0
 *   kv_cache   DEVICE, eet_kv_cache_bytes(cfg); slots [0, q_lens[b]) of sequence b are written,
 *              all other bytes are left untouched
 * Afterwards the cache length of sequence b is q_lens[b].
 * Errors: INVALID_ARG, CAPACITY (batch > max_batch or padded_len > max_prompt). */
int eet_prefill(eet_layer_t *layer, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                const void *tokens, void *out, void *kv_cache, void *hip_stream);

/* eet_prefill for LEFT-padded prompts, the layout Algorithm 1 is printed for: the valid rows of sequence b are
 * rows padded_len - q_lens[b] .. padded_len - 1 of `tokens` and of `out` (Algorithm 1's padLen = padded_len -
 * q_lens[b] pad rows come first; they are never read and are written as 0).  Cache slots and lengths stay
 * sequence-relative: slot t holds the t-th valid token, so the cache, the lengths and every following
 * eet_decode_step are exactly those of eet_prefill on the same prompts right-padded.  Errors as eet_prefill. */
int eet_prefill_left_padded(eet_layer_t *layer, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                            const void *tokens, void *out, void *kv_cache, void *hip_stream);

/* The layer as a bidirectional encoder (Section 4, "Speedup for Bert Layer": padding tokens are
 * skipped, there is no sequence mask): the same pass as eet_prefill with the window of a valid
 * row i of sequence b widened from slots 0..i to all q_lens[b] valid slots.
 * Arguments as eet_prefill; kv_scratch is DEVICE memory of eet_kv_cache_bytes(cfg) that holds the
 * keys and values of this pass only (slots [0, q_lens[b]) are written).  The layer's workspace is
 * reused, so any prefill / decode state of the layer is dropped: a following eet_decode_step
 * returns STATE until the next eet_prefill.  Errors as eet_prefill. */
int eet_layer_encode(eet_layer_t *layer, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                     const void *tokens, void *out, void *kv_scratch, void *hip_stream);

/* One incremental decoding step for every sequence of the last prefill (Section 3.1: keys and
 * values of each step are kept for the next).
 *   tokens     DEVICE fp16 [batch, hidden]; out DEVICE fp16 [batch, hidden]
 * The token of sequence b is written to cache slot n_b, attends to slots 0..n_b, and n_b
 * becomes n_b + 1 (the lengths live in device memory and are advanced on the stream, so a
 * step has no host-varying argument).
 * Errors: STATE (no prefill yet), CAPACITY (some n_b + 1 > max_seq).
 * The capacity check uses a host-side count of the calls.  A caller that captures this call into
 * a HIP graph of its own and replays it advances the device-side lengths once per replay without
 * the host seeing it, and must keep count itself; the kernels never touch memory outside a
 * sequence's max_seq slots whatever the device-side length says (a token past the capacity is
 * not stored and the attention stops at max_seq keys: that sequence's results are then
 * meaningless, nothing else is affected).  The same holds for the stack and model entry points. */
int eet_decode_step(eet_layer_t *layer, const void *tokens, void *out, void *kv_cache,
                    void *hip_stream);

/* Copy the device-side cache lengths n_b of the current batch to HOST int32[batch] (Section 3.1: the
 * number of keys and values kept per sequence; with the padding offsets of Section 2.1 these are the
 * integers that must match exactly).  Synchronises the stream.  Errors: STATE, HIP. */
int eet_cache_lens(eet_layer_t *layer, int32_t *out_host, void *hip_stream);

/* Resume from a saved state.  The resumable state of a layer is its K/V cache (the caller's memory) and the
 * lengths n_b (eet_cache_lens): with a cache that holds tokens [0, cache_lens[b]) of sequence b in its slots, this
 * call sets the lengths (device side, by a small kernel on the stream, and the host-side count) and the batch, after
 * which eet_decode_step continues exactly where the saved run stopped -- on this layer or on another one created
 * with the same configuration and weights.  cache_lens: HOST int32[batch], 1 <= cache_lens[b] <= max_seq.
 * Errors: INVALID_ARG, CAPACITY (batch > max_batch). */
int eet_restore(eet_layer_t *layer, const int32_t *cache_lens, int32_t batch, void *hip_stream);

/* Release the handle: host memory only; workspace, cache and weights stay the caller's (Section 3.1's
 * buffers live as long as the caller keeps them).  NULL is accepted. */
int eet_layer_destroy(eet_layer_t *layer);

/* Message for the last error on this thread ("" if none); static thread-local storage, valid until the
 * next failing call on the thread.  Not from the paper: part of the C-ABI conventions above. */
const char *eet_last_error(void);

/* ---------------------------------------------------------------------------------------------
 * A stack of identical-shape layers driven by one call per phase (the paper's model-level API,
 * Section 5).  The layers share one scratch workspace and two ping-pong activation buffers of
 * max_batch*max_prompt*hidden elements each -- the activation caches of Section 3.1, reused
 * across layers -- and one set of device-side cache lengths.  The K/V cache is
 * 2*b*h*s*l elements (Section 3.1): layer l uses bytes [l, l+1) * eet_kv_cache_bytes(cfg).
 * ------------------------------------------------------------------------------------------- */
typedef struct eet_stack eet_stack_t;

size_t eet_stack_kv_cache_bytes(const eet_layer_config *cfg, int32_t n_layers);
size_t eet_stack_workspace_bytes(const eet_layer_config *cfg, int32_t n_layers);

/* weights: HOST array of n_layers structs of DEVICE pointers (borrowed).  workspace: DEVICE,
 * eet_stack_workspace_bytes, 256-byte aligned.  use_graph != 0: eet_stack_decode_step records its
 * launches into a HIP graph the first time it sees a (tokens, out, kv_cache) triple and replays
 * it afterwards (the graph is instantiated inside that call; it is skipped on the null stream
 * and while the caller is capturing the stream itself).  Errors as eet_layer_create. */
int eet_stack_create(const eet_layer_config *cfg, int32_t n_layers, const eet_layer_weights *weights,
                     void *workspace, int32_t use_graph, eet_stack_t **out_stack);

/* As eet_prefill / eet_decode_step / eet_cache_lens, through all layers: the output of layer l is
 * the input of layer l+1; `out` receives the last layer's output. */
int eet_stack_prefill(eet_stack_t *stack, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                      const void *tokens, void *out, void *kv_cache, void *hip_stream);
/* As eet_prefill_left_padded through all layers: tokens and out hold sequence b at rows
 * padded_len - q_lens[b] .. padded_len - 1 of its block (the layout Algorithm 1 is printed for);
 * cache, lengths and every following decode step are those of eet_stack_prefill. */
int eet_stack_prefill_left_padded(eet_stack_t *stack, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                                  const void *tokens, void *out, void *kv_cache, void *hip_stream);
/* As eet_layer_encode through all layers (the encoder use of Section 4's Bert experiment: padding
 * skipped, no sequence mask, no decode afterwards).  kv_scratch: DEVICE memory of ONE layer's
 * eet_kv_cache_bytes(cfg), reused by every layer in turn for the keys and values of its pass.
 * Any prefill / decode state of the stack is dropped.  Errors as eet_prefill. */
int eet_stack_encode(eet_stack_t *stack, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                     const void *tokens, void *out, void *kv_scratch, void *hip_stream);
int eet_stack_decode_step(eet_stack_t *stack, const void *tokens, void *out, void *kv_cache,
                          void *hip_stream);
int eet_stack_cache_lens(eet_stack_t *stack, int32_t *out_host, void *hip_stream);
/* As eet_restore for all layers (they share the lengths): kv_cache holds every layer's saved region. */
int eet_stack_restore(eet_stack_t *stack, const int32_t *cache_lens, int32_t batch, void *hip_stream);
int eet_stack_destroy(eet_stack_t *stack);

/* ---------------------------------------------------------------------------------------------
 * The model around a stack: token ids in, logits and the greedy next token out (the model-level
 * interface of Section 5 for the paper's GPT-2 workload; the paper prints none of this arithmetic,
 * the readings are GPT-2's).  Input of layer 0 = wte[id] + wpe[position], token t of a sequence at
 * position t whatever the padding; after the last layer one more LayerNorm (lnf_g, lnf_b, the
 * stack's ln_eps); logits = that row times wte^T, no bias; next token = first maximum over
 * columns [0, vocab).
 * Section 3.1's first rule for activation caches is followed literally: the embedding is written
 * into one of the stack's two activation buffers, the feed-forward outputs of the layers alternate
 * between the two, and the final output lands in the same pair -- the model adds no prompt-sized
 * buffer of its own.
 * ------------------------------------------------------------------------------------------- */
typedef struct eet_model eet_model_t;    /* opaque, host memory owned by the library */

typedef struct {
    int32_t vocab;         /* valid token ids are [0, vocab)                                                  */
    int32_t vocab_padded;  /* rows of wte that exist in memory and columns of a logits row: >= vocab, multiple */
                           /* of 64 (rows [vocab, vocab_padded) may hold anything finite; their logits are     */
                           /* written and never chosen)                                                        */
    int32_t max_pos;       /* rows of wpe; every position the model is asked for must be below it             */
} eet_model_config;

typedef struct {           /* DEVICE fp16, BORROWED for the life of the model, 16-byte aligned */
    const void *wte;       /* [vocab_padded, hidden] token embeddings = output projection (tied) */
    const void *wpe;       /* [max_pos, hidden] position embeddings                               */
    const void *lnf_g, *lnf_b; /* [hidden] final LayerNorm                                        */
} eet_model_weights;

/* Workspace of the model itself (a few [max_batch, hidden] rows and a zero bias of vocab_padded
 * elements); 0 for an invalid configuration. */
size_t eet_model_workspace_bytes(const eet_layer_config *cfg, const eet_model_config *mcfg);

/* `stack` is BORROWED and must outlive the model; `cfg` must be the configuration it was created
 * with.  workspace: DEVICE, eet_model_workspace_bytes, 256-byte aligned; its zero bias is cleared
 * here with a synchronous memset (the only blocking call besides eet_stack_cache_lens).
 * Errors: EET_ERR_INVALID_ARG (null, vocab < 1, vocab_padded < vocab, max_pos < max_seq of the
 * stack, misaligned pointers), EET_ERR_UNSUPPORTED_SHAPE (vocab_padded not a multiple of 64). */
int eet_model_create(eet_stack_t *stack, const eet_layer_config *cfg, const eet_model_config *mcfg,
                     const eet_model_weights *weights, void *workspace, eet_model_t **out_model);

/* Whole prompts.  ids: DEVICE int32 [batch, padded_len], right-padded, entries at i >= q_lens[b]
 * are never read; q_lens: HOST.  logits: DEVICE fp16 [batch, vocab_padded], row b = logits of the
 * LAST valid token of sequence b.  next_ids: DEVICE int32 [batch] or NULL, the greedy choice.
 * An id outside [0, vocab) poisons its sequence: its logits come out NaN (and its choice 0).
 * Arguments, errors and cache behaviour otherwise as eet_stack_prefill. */
int eet_model_prefill(eet_model_t *model, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                      const int32_t *ids, void *logits, int32_t *next_ids, void *kv_cache, void *hip_stream);

/* The same with the pads in front: the valid ids of sequence b are ids[b, padded_len - q_lens[b] ..
 * padded_len - 1]; token t of a sequence still has position t.  Logits, next_ids, cache and
 * lengths are those of eet_model_prefill on the same tokens. */
int eet_model_prefill_left_padded(eet_model_t *model, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                                  const int32_t *ids, void *logits, int32_t *next_ids, void *kv_cache,
                                  void *hip_stream);

/* One new token per sequence, at position n_b (read on the device).  ids: DEVICE int32 [batch];
 * it may be the next_ids buffer of the previous call, so generation needs no host round trip.
 * logits [batch, vocab_padded], next_ids as above.  EET_ERR_CAPACITY when a sequence is at the
 * cache capacity, EET_ERR_STATE before the first prefill; otherwise as eet_stack_decode_step
 * (the stack's recorded graph is replayed: the model feeds it from fixed buffers of its own). */
int eet_model_decode_step(eet_model_t *model, const int32_t *ids, void *logits, int32_t *next_ids,
                          void *kv_cache, void *hip_stream);

/* DEVICE pointers to what the latest call left in the activation caches, for per-part checks:
 * *hidden_in = input of layer 0, *hidden_out = output of the last layer; [batch, padded_len,
 * hidden] after a prefill, [batch, hidden] after a decode step.  Either argument may be NULL.
 * After a prefill through an EVEN number of layers *hidden_in is NULL: the two activation caches
 * alternate, so the final output has replaced the embedding. */
int eet_model_hidden_states(eet_model_t *model, const void **hidden_in, const void **hidden_out);

int eet_model_destroy(eet_model_t *model);   /* frees host memory only; the stack stays */

/* ---------------------------------------------------------------------------------------------
 * Operator-level entry points: the individual kernels of the layer, for parity tests and
 * profiling (the paper exposes an operator-level API as well, Section 5).
 * ------------------------------------------------------------------------------------------- */

/* LayerNorm over rows (Section 2.2 kernel family): y = (x-mean)/sqrt(var+eps)*gamma+beta,
 * biased variance, fp32 statistics.  x, y [rows, width]; any width >= 1. */
int eet_op_layernorm(const void *x, const void *gamma, const void *beta, void *y,
                     int64_t rows, int32_t width, float eps, void *hip_stream);

/* Mask-free softmax, Algorithm 1 as an operator, in place on scores [batch, heads, S, S] with
 * S = padded_len: for row i < q_lens[b], entries j <= i become softmax(scale * score) over that
 * window and entries j > i become 0; rows i >= q_lens[b] are not touched.  q_lens is HOST. */
int eet_op_softmax_maskfree(void *scores, const int32_t *q_lens, int32_t batch, int32_t heads,
                            int32_t padded_len, float scale, void *hip_stream);

/* Algorithm 1 in the layout it is printed for (pads first): with padLen = padded_len - q_lens[b], rows
 * padLen .. padded_len-1 are the valid queries, row i becomes softmax(scale * score) over keys padLen .. i and 0
 * elsewhere in the row; rows i < padLen are not touched.  Same errors. */
int eet_op_softmax_maskfree_left_padded(void *scores, const int32_t *q_lens, int32_t batch, int32_t heads,
                                        int32_t padded_len, float scale, void *hip_stream);

/* Add-bias + GELU as a kernel of its own, the form the paper's layer has between its library GEMM calls
 * (Section 3.2: fusion stops at the GEMMs), for rows of any width (Section 2.2's goal; the layer's own pass
 * runs it as the epilogue of the first feed-forward projection).  y = gelu_tanh(x + bias), fp32 arithmetic;
 * x, y [rows, width], bias [width]; y may be x.  Errors: INVALID_ARG (null, rows < 0, width < 1). */
int eet_op_bias_gelu(const void *x, const void *bias, void *y, int64_t rows, int32_t width,
                     void *hip_stream);

/* Add-bias + residual as a kernel of its own (Section 3.1 names the residual connection; Section 3.2 and 2.2
 * as above).  y = x + bias + residual, summed in fp32 and rounded once; x, residual, y [rows, width],
 * bias [width]; y may be x.  Errors as eet_op_bias_gelu. */
int eet_op_bias_residual(const void *x, const void *bias, const void *residual, void *y,
                         int64_t rows, int32_t width, void *hip_stream);

/* Dense projection with its epilogue, the four matrix products of a layer that the paper leaves to library
 * GEMM calls (Section 3.2): y = act(x W^T + bias) (+ residual), fp32 accumulation, one rounding.
 * x [rows, in], W [out, in], y [rows, out], bias [out], residual [rows, out] or NULL; in and out multiples of
 * 64; act: 0 = identity, 1 = gelu_tanh (not together with a residual).  rows <= 16 takes the weight-streaming
 * path of a decode step, more rows the MFMA tile path of a prefill (or row slices, by a cost estimate).
 * Errors: INVALID_ARG (null, bad size, misaligned), UNSUPPORTED_SHAPE. */
int eet_op_linear(const void *x, const void *w, const void *bias, const void *residual, void *y,
                  int64_t rows, int32_t in, int32_t out, int32_t act, void *hip_stream);

/* eet_op_linear on rows that are not dense: row r of x starts at x + r*ldx, row r of y at y + r*ldy (in halfs;
 * multiples of 8, ldx >= in, ldy >= out); the residual rows stay dense.  This is the form the layer's own prefill uses
 * between its two feed-forward projections (Section 3.1), whose intermediate rows it keeps 128 bytes further apart than
 * their length when they are 64 KB or longer: rows a multiple of 32 KB apart slow the projection that reads them down.
 * Only the MFMA tile path takes strides: with rows <= 16 (the weight-streaming path of a decode step) and ldx != in or
 * ldy != out the call returns EET_ERR_UNSUPPORTED_SHAPE.  Other errors as eet_op_linear. */
int eet_op_linear_strided(const void *x, int64_t ldx, const void *w, const void *bias, const void *residual, void *y,
                          int64_t ldy, int64_t rows, int32_t in, int32_t out, int32_t act, void *hip_stream);

/* Causal, padding-skipping attention over whole prompts (mask fusion inside the contraction).
 *   q, ctx     [batch, padded_len, heads*d]; only valid rows are read / written
 *   k_cache, v_cache   [batch, heads, capacity, d]
 * Row i of sequence b attends to slots 0..i.  q_lens is HOST int32[batch]. */
int eet_op_attention_prefill(const void *q, const void *k_cache, const void *v_cache, void *ctx,
                             const int32_t *q_lens, int32_t batch, int32_t padded_len,
                             int32_t heads, int32_t d, int32_t capacity, void *hip_stream);

/* Same layouts and errors; padding skip only, no sequence mask (Section 4, Bert layer): every
 * valid row of sequence b attends to slots 0..q_lens[b]-1. */
int eet_op_attention_encoder(const void *q, const void *k_cache, const void *v_cache, void *ctx,
                             const int32_t *q_lens, int32_t batch, int32_t padded_len,
                             int32_t heads, int32_t d, int32_t capacity, void *hip_stream);

/* The same attention in the unfused form Section 2.1 starts from: scores = Q K^T materialised as
 * [batch, heads, padded_len, padded_len] fp16, Algorithm 1 (eet_op_softmax_maskfree, scale 1/sqrt(d)) in place,
 * ctx = P V.  The score buffer is requested from `buffers` for `module` (Section 3.2) and marked idle again
 * before the call returns: its next user must run on the same stream.  Tiles of pad queries, of keys past a
 * sequence and of keys no query of the tile sees are neither computed nor read.  Layouts as above; padded_len
 * must be a multiple of 8.  Adds EET_ERR_CAPACITY when the manager's arena cannot hold the scores. */
int eet_op_attention_unfused(const void *q, const void *k_cache, const void *v_cache, void *ctx,
                             const int32_t *q_lens, int32_t batch, int32_t padded_len, int32_t heads,
                             int32_t d, int32_t capacity, eet_bufmgr_t *buffers, int32_t module,
                             void *hip_stream);

/* Embedding of whole prompts: out [batch, padded_len, hidden] fp16; row (b, i) = wte[ids[b, i]] +
 * wpe[i] (sum in fp32, rounded once) for i < q_lens[b], zeros for pad rows, whose ids are never
 * read.  ids: DEVICE int32; q_lens: HOST.  hidden must be a multiple of 8.  A row whose id is
 * outside [0, vocab) or whose position is >= max_pos becomes NaN (nothing is indexed). */
int eet_op_embedding(const int32_t *ids, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                     int32_t hidden, int32_t vocab, int32_t max_pos, const void *wte, const void *wpe,
                     void *out, void *hip_stream);
/* The same with the pads in front: row (b, i) = wte[ids[b, i]] + wpe[i - (padded_len - q_lens[b])]
 * for i >= padded_len - q_lens[b], zeros before. */
int eet_op_embedding_left_padded(const int32_t *ids, const int32_t *q_lens, int32_t batch, int32_t padded_len,
                                 int32_t hidden, int32_t vocab, int32_t max_pos, const void *wte,
                                 const void *wpe, void *out, void *hip_stream);
/* Embedding of one token per sequence: out[b] = wte[ids[b]] + wpe[positions[b]]; ids and positions
 * DEVICE int32 [batch]. */
int eet_op_embedding_decode(const int32_t *ids, const int32_t *positions, int32_t batch, int32_t hidden,
                            int32_t vocab, int32_t max_pos, const void *wte, const void *wpe, void *out,
                            void *hip_stream);
/* Greedy choice: out[r] (DEVICE int32 [rows]) = index of the first maximum of the fp16 row
 * logits[r*row_stride + 0 .. vocab); NaN never wins; a row with nothing above -inf gives 0.
 * row_stride >= vocab, a multiple of 8 elements; logits 16-byte aligned. */
int eet_op_argmax(const void *logits, int32_t rows, int32_t vocab, int32_t row_stride, int32_t *out,
                  void *hip_stream);

/* Incremental attention over the K/V cache (Section 3.1: the keys and values of every step are kept for the
 * next step's attention; the padding offset of Section 2.1 is the loop bound).  q, ctx [batch, heads*d];
 * k_cache, v_cache [batch, heads, capacity, d]; sequence b attends to slots 0..n_keys[b]-1.
 * n_keys is DEVICE int32[batch], each 1..capacity (a value above capacity is clamped to it; a sequence with
 * n_keys[b] < 1 sees no key and its ctx rows are written as 0).  scratch: DEVICE, 16-byte aligned, at least
 * eet_op_attention_decode_scratch_bytes(batch, heads, d, capacity) bytes, owned by the caller: partial results
 * of the key ranges when a (sequence, head) pair is split over several workgroups; contents on entry do not
 * matter, calls that share it must not overlap.  Errors: INVALID_ARG (null, size < 1, misaligned),
 * UNSUPPORTED_SHAPE (d not 64 or 128, batch or heads above 65535). */
size_t eet_op_attention_decode_scratch_bytes(int32_t batch, int32_t heads, int32_t d, int32_t capacity);
int eet_op_attention_decode(const void *q, const void *k_cache, const void *v_cache, void *ctx,
                            const int32_t *n_keys, int32_t batch, int32_t heads, int32_t d,
                            int32_t capacity, void *scratch, void *hip_stream);

/* eet_op_attention_decode for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * `scratch`, same kernels, same results bit for bit: the partial results of a split key range live in a
 * 512 KiB device array inside the library (EET_STATIC_SCRATCH_BYTES; one copy per GPU, held until the process
 * ends), whose address is looked up on the first call on each device -- make that first call outside a capture.
 * The call allocates nothing.  Every call on a GPU shares that GPU's array: calls that overlap in time on one
 * GPU (two streams, two threads) race; calls on one stream are ordered by the stream.  Nothing has to be
 * cleared between calls.  Adds EET_ERR_CAPACITY when eet_op_attention_decode_scratch_bytes(batch, heads, d,
 * capacity) exceeds the array (it never does for d <= 128: the split count keeps it below 300 KB). */
#define EET_STATIC_SCRATCH_BYTES (512 * 1024)
int eet_op_attention_decode_static(const void *q, const void *k_cache, const void *v_cache, void *ctx,
                                   const int32_t *n_keys, int32_t batch, int32_t heads, int32_t d,
                                   int32_t capacity, void *hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Dynamic buffer manager (Section 3.2): the result buffers of operators that are not fused are
 * requested by size and marked idle when no longer needed; the manager decides what to reuse.
 *   - a request of a module is served by an idle buffer of the SAME module only if the sizes are
 *     identical (no fragmentation), by an idle buffer of ANOTHER module if the buffer is at least
 *     as large (no duplicated allocation); the list is scanned in creation order and the first
 *     buffer that qualifies is taken; otherwise a new buffer is created;
 *   - a buffer belongs to the module that used it last; sizes are rounded up to 256 bytes;
 *   - buffers are carved, one after the other, out of `arena`: DEVICE memory of arena_bytes, 256-byte
 *     aligned, owned by the caller for the life of the manager and never dereferenced by it
 *     (Section 3.1: the maximum is allocated in advance).  The bytes carved so far are the section's
 *     "total buffer size"; for an unfused layer that is b*p*(6h + n*p) elements.
 * Host logic: no call touches the device or a stream.  A manager is not thread-safe.
 * Errors: EET_ERR_INVALID_ARG (null, zero bytes, pointer that is not a buffer of the manager),
 * EET_ERR_CAPACITY (the request does not fit in what is left of the arena), EET_ERR_STATE (release
 * of a buffer that is already idle).  On error nothing changes.
 * ------------------------------------------------------------------------------------------- */
/* eet_bufmgr_t: opaque, host memory owned by the library (typedef at the top of this header) */
typedef struct {
    uint64_t arena_bytes;        /* size of the arena                                        */
    uint64_t footprint_bytes;    /* bytes of all buffers created so far                      */
    int64_t buffers, idle;       /* buffers in the list, and how many of them are idle       */
    int64_t requests;            /* successful requests                                      */
    int64_t reused_same_size;    /* ... served by an idle buffer of identical size           */
    int64_t reused_larger;       /* ... served by a larger idle buffer of another module     */
    int64_t created;             /* ... that created a buffer                                */
} eet_bufmgr_stats;
int eet_bufmgr_create(void *arena, size_t arena_bytes, eet_bufmgr_t **out);
int eet_bufmgr_request(eet_bufmgr_t *mgr, size_t bytes, int32_t module, void **out /* DEVICE pointer into the arena */);
int eet_bufmgr_release(eet_bufmgr_t *mgr, void *buffer);
int eet_bufmgr_query(const eet_bufmgr_t *mgr, eet_bufmgr_stats *out);
int eet_bufmgr_destroy(eet_bufmgr_t *mgr);

#ifdef __cplusplus
}
#endif
#endif /* EET_H */
