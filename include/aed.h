/*
 * aed.h -- C ABI of the MI355X (gfx950) autoregressive AED decoder library.
 *
 * The library runs the part of an attention-encoder-decoder speech model that
 * the paper identifies as the inference bottleneck (abstract; Sec.
 * "Transferring model capacity from decoder to encoder"): the batched,
 * token-by-token transformer-decoder step with cross-attention to the encoder
 * output, started from a fixed-length prompt (Fig. 3 caption).  Encoder states
 * and per-sequence lengths go in, token ids come out.  Every sequence keeps
 * its own encoder length and its own decoded length, so no work is spent on
 * the padding that the paper's bucketing fights (Sec. 1; Fig. 1).
 *
 * Model (pre-LayerNorm transformer decoder), for the token y_s at position s:
 *     x = emb_scale * tok_emb[y_s] + pos_emb[s]
 *     per layer:  x += Wo  . SelfAttn (LN1(x))          keys: positions 0..s
 *                 x += Wco . CrossAttn(LN2(x), enc)     keys: this sequence's frames
 *                 x += W2  . relu(W1 . LN3(x))
 *     logits = Wout . LNf(x) + bout ; next token = argmax (lowest index on ties)
 *
 * Conventions
 *  - All weight matrices are row-major [out, in]; a NULL bias pointer = zero.
 *    norm_type 1 replaces every LayerNorm below by RMSNorm (aed_config).
 *  - dtype 0: weights / encoder states / KV caches are float32.
 *    dtype 1: they are bfloat16; the residual stream, LayerNorm statistics,
 *    scores, softmax, accumulators and logits are float32 in both modes.
 *  - Ownership: the caller owns weights, encoder states, outputs and the
 *    workspace, all of which must outlive the decoder (weights, workspace) or
 *    the call (everything else).  After aed_decoder_create the library makes
 *    no device allocation; everything it needs is carved from the workspace.
 *  - Streams: all work is enqueued on the stream given at create.  Calls
 *    return after enqueueing, except aed_greedy_decode (polls a
 *    finished-count and synchronises the stream before returning) and
 *    aed_greedy_decode_queue (blocks until the queue is empty).
 *    One decoder = one stream = one host thread.
 *  - Errors: every call returns an aed_status; argument errors are found on
 *    the host before any launch and leave the decoder unchanged.
 *    aed_last_error gives a message for the most recent failure.
 */
#ifndef AED_H
#define AED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aed_decoder aed_decoder; /* opaque */

typedef enum aed_status {
    AED_OK = 0,
    AED_EINVAL = -1,       /* bad argument */
    AED_ECAPACITY = -2,    /* exceeds a capacity fixed at create */
    AED_ESTATE = -3,       /* call made in the wrong state */
    AED_EHIP = -4,         /* a HIP runtime call failed */
    AED_EUNSUPPORTED = -5  /* a shape this build has no kernel for */
} aed_status;

typedef struct aed_config {
    uint32_t struct_size;  /* = sizeof(aed_config) */
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab, max_positions;
    int32_t dtype;         /* 0 float32, 1 bfloat16 */
    int32_t norm_type;     /* 0 LayerNorm: g (z - mean) / sqrt(biased variance + ln_eps) + b.
                              1 RMSNorm in its place everywhere (ln1, ln2, ln3, lnf): g z / sqrt(mean(z^2) + ln_eps) + b,
                              no mean subtraction; the shift vectors ln*_b may then be NULL (= zero) */
    int32_t page_size;     /* tokens per self-attention KV page (16) */
    int32_t max_batch;             /* capacity: sequences per batch */
    int32_t max_total_enc_frames;  /* capacity: sum of encoder lengths of a batch */
    int32_t max_dec_len;           /* capacity: prompt + generated tokens per sequence */
    int32_t kv_pages;      /* self-KV pages in the pool; 0 = max_batch * ceil(max_dec_len / page_size) */
    int32_t eos_id;        /* < 0: never stop on EOS */
    int32_t pad_id;        /* written to out_tokens after a sequence has finished */
    float ln_eps, emb_scale;
    int32_t prefill_rows;  /* capacity: rows of one prompt-prefill pass (see aed_greedy_decode); 0 = none */
    int32_t kv_fp8;        /* 1: the self- and cross-attention caches hold 8-bit floating point codes instead of
                              dtype elements, which halves the bytes the two attention steps stream (bfloat16
                              models only, else AED_EUNSUPPORTED).  Format: E4M3 of the OCP 8-bit floating point
                              specification (bias 7, subnormals, no infinities, largest magnitude 448); a key or
                              value element is rounded from float32 to the nearest code, ties to even, and
                              saturates at +-448, when it is written to the cache; no scale factor.  An option of
                              this library, not part of the paper's method; results differ from kv_fp8 = 0 by the
                              storage rounding.  0: caches in dtype. */
} aed_config;

/* DEVICE pointers, element type per aed_config.dtype. */
typedef struct aed_layer_weights {
    const void *ln1_g, *ln1_b, *w_qkv /*[3d,d] = [Wq;Wk;Wv]*/, *b_qkv, *w_o /*[d,d]*/, *b_o;
    const void *ln2_g, *ln2_b, *w_cq /*[d,d]*/, *b_cq, *w_ckv /*[2d,d] = [Wk;Wv]*/, *b_ckv, *w_co /*[d,d]*/, *b_co;
    const void *ln3_g, *ln3_b, *w_ff1 /*[F,d]*/, *b_ff1, *w_ff2 /*[d,F]*/, *b_ff2;
} aed_layer_weights;

typedef struct aed_weights {
    const void *tok_emb /*[V,d]*/, *pos_emb /*[max_positions,d]*/;
    const void *lnf_g, *lnf_b, *w_out /*[V,d], may alias tok_emb*/, *b_out;
    const aed_layer_weights *layers; /* HOST array of n_layers structs (copied at create) */
} aed_weights;

/* Bytes of device workspace a decoder with this configuration needs.
 * Errors: AED_EINVAL (NULL, struct_size mismatch, non-positive or inconsistent
 * dimensions, n_heads*head_dim != d_model), AED_EUNSUPPORTED (shape without a
 * kernel: head_dim not 64/128, d_model not a multiple of 256 or above 1024,
 * d_ffn not a multiple of 256, vocab not a multiple of 64, page_size != 16). */
aed_status aed_workspace_bytes(const aed_config *cfg, size_t *bytes);

/* Create a decoder.  workspace: DEVICE memory, 256-byte aligned, at least
 * aed_workspace_bytes(); hip_stream: a hipStream_t (NULL = the default
 * stream).  Must be called with the target device current.
 * Errors: as aed_workspace_bytes, plus AED_EINVAL for NULL required weights,
 * a misaligned or too-small workspace; AED_EHIP. */
aed_status aed_decoder_create(const aed_config *cfg, const aed_weights *weights,
                              void *workspace, size_t workspace_bytes,
                              void *hip_stream, aed_decoder **out);

/* Waits for the stream, releases host resources.  NULL is allowed. */
aed_status aed_decoder_destroy(aed_decoder *dec);

/* Start a batch: compute every layer's cross-attention keys and values
 * K = enc Wk^T + bk, V = enc Wv^T + bv once, and reset the decode state (empty
 * self-attention caches, nothing generated).
 * enc_states: DEVICE, packed [sum(enc_lens), d_model] in batch order, no
 * padding rows; enc_lens: HOST int32[batch], each >= 1.
 * Errors: AED_EINVAL (NULL, batch < 1, a length < 1), AED_ECAPACITY (batch >
 * max_batch or sum(enc_lens) > max_total_enc_frames), AED_EHIP. */
aed_status aed_cross_kv_precompute(aed_decoder *dec, const void *enc_states,
                                   const int32_t *enc_lens, int32_t batch);

/* The same for a padded tensor [batch, t_max, d_model] (row_stride elements
 * between consecutive frames' rows is d_model; frames >= enc_lens[b] are
 * padding and are never read). */
aed_status aed_cross_kv_precompute_padded(aed_decoder *dec, const void *enc_padded,
                                          int32_t t_max, const int32_t *enc_lens, int32_t batch);

/* One decoder step for the whole batch: feed tokens_in[b] at the next
 * position of sequence b, append its self-attention key/value to the paged
 * cache, and return the greedy next token.
 * tokens_in: DEVICE int32[batch] (ids must be in [0, vocab); not checked on
 * the host, out-of-range ids are clamped on the device); tokens_out: DEVICE
 * int32[batch] or NULL; logits_out: DEVICE float32 [batch, vocab] or NULL.
 * No EOS handling: every sequence advances by one position.
 * Errors: AED_ESTATE before a precompute, AED_ECAPACITY when a sequence would
 * exceed max_dec_len / max_positions or the page pool is exhausted, AED_EHIP. */
aed_status aed_decode_step(aed_decoder *dec, const int32_t *tokens_in,
                           int32_t *tokens_out, float *logits_out);

/* aed_decode_step for callers that cannot allocate device memory at this
 * point or hand the library memory it may keep writing to behind their back:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same results, same errors.  The step's
 * activations and attention partials live in a static device array of 8 MiB
 * inside the library (each GPU the library runs on holds its copy until the
 * process ends) instead of the workspace, the kernels are launched directly
 * (no launch graph is built), the page table is advanced by a kernel instead
 * of a host copy, and the call makes no allocation of any kind.
 * Additional error: AED_ECAPACITY when the decoder's step activations do not
 * fit the array (they grow with max_batch * (5 d_model + d_ffn + vocab);
 * max_batch 64 of the 1024-wide configurations fits).
 * Every decoder on a GPU shares that GPU's array, which keeps what the last
 * call left in it: calls that overlap on one GPU (two streams, two threads)
 * race.  Steps of this call and of aed_decode_step may be mixed. */
aed_status aed_decode_step_noalloc(aed_decoder *dec, const int32_t *tokens_in,
                                   int32_t *tokens_out, float *logits_out);

/* Greedy decoding of the whole batch from a fixed-length prompt.  Restarts
 * the decode state of the current batch (cross K/V are kept), feeds the
 * prompt, then emits up to max_new tokens per sequence.
 * prompt: DEVICE int32 [batch, prompt_len]; max_new_per_seq: HOST
 * int32[batch] or NULL -- if given (needs eos_id >= 0), the
 * max_new_per_seq[b]-th emitted token of sequence b is forced to eos_id.
 * A sequence finishes when it emits eos_id; finished sequences cost no
 * attention work and append nothing to the cache.
 * out_tokens: DEVICE int32 [batch, max_new], pad_id after the end;
 * out_lens: DEVICE int32[batch], emitted tokens including the EOS token.
 * Synchronises the stream before returning.
 * Errors: AED_ESTATE, AED_EINVAL (NULL, prompt_len < 1, max_new < 1,
 * max_new_per_seq with eos_id < 0 or an entry < 1), AED_ECAPACITY
 * (prompt_len + max_new > max_dec_len or max_positions, page pool), AED_EHIP. */
aed_status aed_greedy_decode(aed_decoder *dec, const int32_t *prompt, int32_t prompt_len,
                             int32_t max_new, const int32_t *max_new_per_seq,
                             int32_t *out_tokens, int32_t *out_lens);

/* Greedy decoding of a queue of requests through max_batch slots, with slot
 * refill: when a sequence finishes, its slot takes the next queued request
 * instead of idling until the slowest sequence of a fixed batch is done (the
 * decoded length varies per utterance and the decoder runs one step per
 * token for the whole batch: Sec. 1; Fig. 3 caption).  Each request's result
 * is what aed_greedy_decode gives for it in any batch.
 * A refill computes the new requests' cross-attention K/V (all layers) into
 * free frames of the cache, re-uses the slot's self-attention pages from
 * position 0, and hands the finished request's tokens to the caller's rows.
 * Requests are started in queue order; one that does not fit the free frames
 * waits for a running one to end.
 * enc_states: DEVICE [sum(enc_lens), d_model] (all requests, packed);
 * enc_lens: HOST int32[n_requests]; prompts: DEVICE int32 [n_requests,
 * prompt_len]; max_new_per_req: HOST int32[n_requests] or NULL (as
 * max_new_per_seq above); out_tokens: DEVICE int32 [n_requests, max_new],
 * pad_id after the end; out_lens: DEVICE int32[n_requests]; steps_run: HOST,
 * may be NULL: decoder steps executed.  Needs eos_id >= 0.  Ends the current
 * batch, if any (a new aed_cross_kv_precompute is needed for the per-batch
 * calls).  Blocks until every request is done.
 * Errors: AED_EINVAL (NULL, n_requests / prompt_len / max_new < 1, an
 * enc_lens or max_new_per_req entry < 1, eos_id < 0), AED_ECAPACITY
 * (prompt_len + max_new > max_dec_len or max_positions; a request longer than
 * max_total_enc_frames; fewer than min(max_batch, n_requests) *
 * ceil((prompt_len + max_new) / page_size) pages), AED_EUNSUPPORTED (a request
 * above 65535 frames), AED_EHIP. */
aed_status aed_greedy_decode_queue(aed_decoder *dec, const void *enc_states, const int32_t *enc_lens,
                                   int32_t n_requests, const int32_t *prompts, int32_t prompt_len,
                                   int32_t max_new, const int32_t *max_new_per_req,
                                   int32_t *out_tokens, int32_t *out_lens, int32_t *steps_run);

/* Message for the most recent error of this decoder (or of the last failed
 * create when dec is NULL).  Owned by the library. */
const char *aed_last_error(const aed_decoder *dec);

/* Weight-matrix parameters of the decoder layers (4d^2 self-attention + 4d^2
 * cross-attention + 2 d F per layer; biases, LayerNorm and embeddings
 * excluded) -- the quantity behind the paper's 1016M -> 680M when 20 layers
 * are removed. */
int64_t aed_layer_matrix_params(const aed_config *cfg);

/* ---- inspection and measurement (used by the tests and the benchmark) ---- */

/* Copy one sequence's cross-attention K and V of one layer to HOST float32
 * buffers [enc_len, d_model] (synchronises).  The values are what the cache
 * holds: rounded to dtype, or to E4M3 with kv_fp8 (every value returned is
 * then exactly the value of its code). */
aed_status aed_read_cross_kv(aed_decoder *dec, int32_t layer, int32_t seq,
                             float *k_out, float *v_out);

/* Copy one sequence's cached self-attention K and V of one layer to HOST
 * float32 buffers [n_positions, d_model]; *n_positions receives the count
 * (synchronises).  Buffers must hold max_dec_len rows. */
aed_status aed_read_self_kv(aed_decoder *dec, int32_t layer, int32_t seq,
                            float *k_out, float *v_out, int32_t *n_positions);

/* Copy the logits of the most recent decoder step (aed_decode_step, or the
 * last step aed_greedy_decode ran) to a HOST float32 buffer [batch, vocab]
 * (synchronises).  Rows of sequences that had finished before that step hold
 * unspecified values. */
aed_status aed_read_logits(aed_decoder *dec, float *logits_out);

/* Kernel classes of one decoder step, for aed_time_kernels. */
enum {
    AED_K_LN_QKV = 0, AED_K_SELF_ATTN, AED_K_SELF_OUT, AED_K_LN_CROSSQ, AED_K_CROSS_ATTN,
    AED_K_CROSS_OUT, AED_K_LN_FFN1, AED_K_FFN2, AED_K_LN_VOCAB, AED_K_SAMPLE, AED_K_EMBED,
    AED_K_CROSS_KV, AED_K_COUNT
};

/* Re-run the kernels of one class with the decoder's current state, `reps`
 * rounds over all layers, bracketed by HIP events on the decoder's stream.
 * ms_total: elapsed milliseconds; launches: kernel launches inside the
 * bracket.  The residual stream is changed by this; call
 * aed_cross_kv_precompute / aed_greedy_decode again before decoding further. */
aed_status aed_time_kernels(aed_decoder *dec, int32_t kernel_class, int32_t reps,
                            float *ms_total, int32_t *launches);

/* Algorithmic HBM bytes and flops of one launch of a kernel class in the
 * decoder's current state, averaged over layers (what the method itself must
 * move and compute: no padding, no re-reads). */
aed_status aed_kernel_work(aed_decoder *dec, int32_t kernel_class, double *bytes, double *flops);

#ifdef __cplusplus
}
#endif
#endif
