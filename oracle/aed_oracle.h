/*
 * CPU oracle for the autoregressive attention-encoder-decoder (AED) decoder.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain definition that the HIP
 * library is checked against; the product never calls it.  It shares no source
 * with the HIP path.
 *
 * What it computes: the decoder the paper names as the inference bottleneck
 * (abstract; Sec. "Transferring model capacity from decoder to encoder"): a
 * pre-LayerNorm transformer decoder with causal self-attention, cross-attention
 * over the encoder output, a ReLU feed-forward block, a final LayerNorm, the
 * vocabulary projection and greedy argmax, fed with a fixed-length prompt
 * (Fig. 3 caption).  Each sequence is processed alone, so no padding exists;
 * aedo_forward_full is a second, independent routine that does use padding and
 * masks (Sec. 1: padded examples plus padding masks) and exists only to test
 * the incremental one.
 *
 * Precision: inputs and weights are float32 arrays; every intermediate value,
 * every accumulation and the returned logits are double.
 *
 * Pinning: every routine here is pinned by the CPU tests (closed forms, brute
 * force, invariants, and agreement with torch.nn.TransformerDecoder on CPU).
 * The paper prints no worked numeric example of the decoder, so absolute
 * logit values are pinned by those definitions only.
 *
 * All pointers are host pointers.  Weight matrices are row-major [out, in].
 * A NULL bias means zero.  Return value 0 = ok, negative = bad argument.
 */
#ifndef AED_ORACLE_H
#define AED_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aedo_config {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab, max_positions;
    int32_t eos_id;   /* < 0: never stop on EOS */
    int32_t pad_id;   /* written after a sequence has finished */
    float ln_eps, emb_scale;
    int32_t kv_fp8;   /* nonzero: attention keys and values are stored as 8-bit E4M3 codes (see below) */
    int32_t norm_type; /* 0: LayerNorm in every place the model normalises; 1: RMSNorm (aedo_rmsnorm) instead */
} aedo_config;

typedef struct aedo_layer {
    const float *ln1_g, *ln1_b, *w_qkv /*[3d,d]*/, *b_qkv, *w_o /*[d,d]*/, *b_o;
    const float *ln2_g, *ln2_b, *w_cq /*[d,d]*/, *b_cq, *w_ckv /*[2d,d]*/, *b_ckv, *w_co, *b_co;
    const float *ln3_g, *ln3_b, *w_ff1 /*[F,d]*/, *b_ff1, *w_ff2 /*[d,F]*/, *b_ff2;
} aedo_layer;

typedef struct aedo_weights {
    const float *tok_emb /*[V,d]*/, *pos_emb /*[max_positions,d]*/;
    const float *lnf_g, *lnf_b, *w_out /*[V,d]*/, *b_out;
    const aedo_layer *layers; /* n_layers entries */
} aedo_weights;

/* ---- primitives (exported so that tests can pin them one by one) ---- */

/* y = g * (z - mean) / sqrt(biased_var + eps) + b over n elements. */
void aedo_layernorm(const double *z, const float *g, const float *b, int n, double eps, double *y);
/* Root-mean-square normalisation (Zhang and Sennrich, 2019: the mean is not subtracted):
 * y = g * z / sqrt(mean(z^2) + eps) + b over n elements; b may be NULL (no shift). */
void aedo_rmsnorm(const double *z, const float *g, const float *b, int n, double eps, double *y);
/* y[o] = bias[o] + sum_i W[o, i] * x[i]. */
void aedo_linear(const double *x, const float *W, const float *bias, int n_in, int n_out, double *y);
/* p = exp(a - max a) / sum. */
void aedo_softmax(const double *a, int n, double *p);
/* One head, one query: out = sum_j softmax_j(q.K_j / sqrt(dh)) V_j over n_keys rows
 * of K and V (row stride `stride` doubles).  probs (n_keys) may be NULL. */
void aedo_attend(const double *q, const double *K, const double *V, int n_keys, int dh,
                 int stride, double *out, double *probs);
/* Lowest index of the maximum. */
int32_t aedo_argmax(const double *a, int n);

/* 8-bit floating point storage of the attention keys and values (an option of
 * this implementation, not of the paper: it halves the bytes the attention
 * steps stream).  Format: E4M3 of the OCP 8-bit floating point specification
 * (OFP8): 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals at
 * exponent field 0, no infinities, S.1111.111 is NaN, largest magnitude 448.
 * Encoding first rounds the (double) value to float32, then rounds that to
 * the nearest code, ties to the even code, and saturates (the float32 step is
 * part of this definition; it differs from rounding the double directly only
 * for values within 2^-24 relative of the midpoint of two codes): anything
 * beyond 448 becomes +-448.  With cfg.kv_fp8 set, every key / value element is replaced by decode(encode(.)) at the moment it is
 * cached; nothing else changes. */
uint8_t aedo_fp8_e4m3_encode(float x);
double aedo_fp8_e4m3_decode(uint8_t code);
void aedo_fp8_e4m3_encode_array(const float *x, int64_t n, uint8_t *codes);

/* Cross-attention memory of one layer for one sequence: K = enc Wk^T + bk,
 * V = enc Wv^T + bv with [Wk; Wv] = w_ckv.  enc [T, d] -> K_out, V_out [T, d]. */
int aedo_cross_kv(const aedo_config *cfg, const aedo_weights *w, int layer,
                  const float *enc, int T, double *K_out, double *V_out);

/* Teacher-forced incremental decoding (KV cache, one position at a time).
 * enc: packed [sum(enc_lens), d]; tokens [B, S]; logits_out [B, S, V]:
 * logits after feeding tokens[b, 0..s]. */
int aedo_decode_forced(const aedo_config *cfg, const aedo_weights *w,
                       const float *enc, const int32_t *enc_lens, int B,
                       const int32_t *tokens, int S, double *logits_out);

/* The self-attention cache of one layer after one sequence (enc [T, d]) has
 * been fed tokens[0..S-1]: the keys and values of those positions, [S, d]. */
int aedo_self_kv(const aedo_config *cfg, const aedo_weights *w, const float *enc, int T,
                 const int32_t *tokens, int S, int layer, double *K_out, double *V_out);

/* Greedy decoding.  prompt [B, P]; emits at most max_new tokens per sequence.
 * max_new_per_seq (may be NULL; needs eos_id >= 0): sequence b's
 * max_new_per_seq[b]-th emitted token is forced to eos_id.  A sequence
 * finishes when it emits eos_id.  out_tokens [B, max_new] (pad_id after the
 * end), out_lens [B] (count including the EOS token), logits_out
 * [B, max_new, V] or NULL (rows past the end are left untouched). */
int aedo_greedy_decode(const aedo_config *cfg, const aedo_weights *w,
                       const float *enc, const int32_t *enc_lens, int B,
                       const int32_t *prompt, int P, int max_new,
                       const int32_t *max_new_per_seq,
                       int32_t *out_tokens, int32_t *out_lens, double *logits_out);

/* Whole-sequence forward over a PADDED batch with masks: enc_padded
 * [B, T_max, d] (rows >= enc_lens[b] are padding and may hold anything),
 * tokens [B, S_max] (positions >= tok_lens[b] are padding); dense score
 * matrices with a causal mask and key-padding masks.  logits_out
 * [B, S_max, V]; rows at padded positions are set to 0. */
int aedo_forward_full(const aedo_config *cfg, const aedo_weights *w,
                      const float *enc_padded, int T_max, const int32_t *enc_lens, int B,
                      const int32_t *tokens, int S_max, const int32_t *tok_lens,
                      double *logits_out);

/* Weights per decoder layer excluding biases and LayerNorm (4d^2 self + 4d^2
 * cross + 2dF), times n_layers. */
int64_t aedo_layer_matrix_params(const aedo_config *cfg);

/* Threads the batch routines spread sequences over. */
int aedo_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
