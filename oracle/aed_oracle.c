/*
 * CPU oracle for the AED decoder step -- see aed_oracle.h.  TEST INFRASTRUCTURE
 * ONLY: plain loops, double arithmetic, one sequence at a time.
 *
 * Model (paper, Sec. "Transferring model capacity from decoder to encoder":
 * an autoregressive cross-attention transformer decoder of 24 or 4 layers;
 * Fig. 3 caption: fixed-length prompt; Sec. 1: padding must not contribute).
 * For position s with input token y_s:
 *     x = emb_scale * E[y_s] + Pos[s]
 *     for every layer:
 *         h = LN1(x); q,k,v = h Wqkv^T + b; cache k,v
 *         x += concat_h( softmax(q_h . K_h / sqrt(dh)) V_h ) Wo^T + bo      (keys 0..s)
 *         h = LN2(x); qc = h Wcq^T + b
 *         x += concat_h( softmax(qc_h . Kc_h / sqrt(dh)) Vc_h ) Wco^T + bco (keys 0..T-1)
 *         h = LN3(x); x += relu(h W1^T + b1) W2^T + b2
 *     logits = LNf(x) Wout^T + bout
 */
#include "aed_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* primitives                                                          */
/* ------------------------------------------------------------------ */
void aedo_layernorm(const double *z, const float *g, const float *b, int n, double eps, double *y)
{
    double mean = 0.0;
    for (int i = 0; i < n; ++i) mean += z[i];
    mean /= n;
    double var = 0.0;
    for (int i = 0; i < n; ++i) var += (z[i] - mean) * (z[i] - mean);
    var /= n; /* biased */
    double rstd = 1.0 / sqrt(var + eps);
    for (int i = 0; i < n; ++i) y[i] = (double)g[i] * ((z[i] - mean) * rstd) + (double)b[i];
}

void aedo_rmsnorm(const double *z, const float *g, const float *b, int n, double eps, double *y)
{
    double ms = 0.0;
    for (int i = 0; i < n; ++i) ms += z[i] * z[i];
    ms /= n;
    double r = 1.0 / sqrt(ms + eps);
    for (int i = 0; i < n; ++i) y[i] = (double)g[i] * (z[i] * r) + (b ? (double)b[i] : 0.0);
}

/* the normalisation the configuration names */
static void norm_rows(const aedo_config *cfg, const double *z, const float *g, const float *b, int n, double eps,
                      double *y)
{
    if (cfg->norm_type == 1) aedo_rmsnorm(z, g, b, n, eps, y);
    else aedo_layernorm(z, g, b, n, eps, y);
}

void aedo_linear(const double *x, const float *W, const float *bias, int n_in, int n_out, double *y)
{
    for (int o = 0; o < n_out; ++o) {
        const float *row = W + (size_t)o * n_in;
        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
        for (int i = 0; i < n_in; ++i) acc += (double)row[i] * x[i];
        y[o] = acc + (bias ? (double)bias[o] : 0.0);
    }
}

void aedo_softmax(const double *a, int n, double *p)
{
    double m = a[0];
    for (int i = 1; i < n; ++i)
        if (a[i] > m) m = a[i];
    double sum = 0.0;
    for (int i = 0; i < n; ++i) {
        p[i] = exp(a[i] - m);
        sum += p[i];
    }
    for (int i = 0; i < n; ++i) p[i] /= sum;
}

void aedo_attend(const double *q, const double *K, const double *V, int n_keys, int dh,
                 int stride, double *out, double *probs)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double *p = probs ? probs : (double *)malloc(sizeof(double) * (size_t)n_keys);
    double scale = 1.0 / sqrt((double)dh);
    for (int j = 0; j < n_keys; ++j) {
        double dot = 0.0;
        for (int c = 0; c < dh; ++c) dot += q[c] * K[(size_t)j * stride + c];
        a[j] = dot * scale;
    }
    aedo_softmax(a, n_keys, p);
    for (int c = 0; c < dh; ++c) {
        double acc = 0.0;
        for (int j = 0; j < n_keys; ++j) acc += p[j] * V[(size_t)j * stride + c];
        out[c] = acc;
    }
    free(a);
    if (!probs) free(p);
}

int32_t aedo_argmax(const double *a, int n)
{
    int32_t best = 0;
    for (int i = 1; i < n; ++i)
        if (a[i] > a[best]) best = i; /* strict: the lowest index wins ties */
    return best;
}

static int config_ok(const aedo_config *c)
{
    return c && c->n_layers > 0 && c->d_model > 0 && c->n_heads > 0 && c->head_dim > 0 &&
           c->n_heads * c->head_dim == c->d_model && c->d_ffn > 0 && c->vocab > 0 &&
           c->max_positions > 0;
}

int64_t aedo_layer_matrix_params(const aedo_config *cfg)
{
    int64_t d = cfg->d_model, F = cfg->d_ffn;
    int64_t self_attn = 3 * d * d + d * d;          /* Wqkv, Wo */
    int64_t cross_attn = d * d + 2 * d * d + d * d; /* Wcq, Wckv, Wco */
    int64_t ffn = 2 * d * F;
    return (self_attn + cross_attn + ffn) * cfg->n_layers;
}

int aedo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* 8-bit E4M3 storage of keys and values (OCP OFP8)                    */
/* ------------------------------------------------------------------ */
double aedo_fp8_e4m3_decode(uint8_t code)
{
    int sign = code >> 7, ef = (code >> 3) & 15, m = code & 7;
    double v;
    if (ef == 15 && m == 7) return NAN;
    if (ef == 0)
        v = ldexp((double)m / 8.0, -6); /* subnormal: 0.m * 2^(1 - bias) */
    else
        v = ldexp(1.0 + (double)m / 8.0, ef - 7);
    return sign ? -v : v;
}

uint8_t aedo_fp8_e4m3_encode(float x)
{
    uint8_t sign = signbit(x) ? 0x80 : 0;
    if (isnan(x)) return (uint8_t)(sign | 0x7f);
    double a = fabs((double)x);
    if (a >= 448.0) return (uint8_t)(sign | 0x7e); /* saturate */
    if (a == 0.0) return sign;
    int e = ilogb(a); /* a = f * 2^e, 1 <= f < 2 */
    if (e < -6) e = -6; /* below the smallest normal the spacing stays 2^-9 */
    /* a in units of the spacing 2^(e-3); rint rounds ties to even (default rounding mode), and an even
     * count is an even code because the mantissa field is the count's low bits */
    int q = (int)rint(ldexp(a, 3 - e));
    if (q < 8) return (uint8_t)(sign | q);          /* subnormal, or zero */
    if (q == 16) { q = 8; e += 1; }                 /* rounded up into the next binade */
    return (uint8_t)(sign | ((e + 7) << 3) | (q - 8));
}

void aedo_fp8_e4m3_encode_array(const float *x, int64_t n, uint8_t *codes)
{
    for (int64_t i = 0; i < n; ++i) codes[i] = aedo_fp8_e4m3_encode(x[i]);
}

/* v[i] <- the value its E4M3 code stands for */
static void store_as_fp8(double *v, int n)
{
    for (int i = 0; i < n; ++i) v[i] = aedo_fp8_e4m3_decode(aedo_fp8_e4m3_encode((float)v[i]));
}

/* ------------------------------------------------------------------ */
/* cross-attention memory                                              */
/* ------------------------------------------------------------------ */
int aedo_cross_kv(const aedo_config *cfg, const aedo_weights *w, int layer,
                  const float *enc, int T, double *K_out, double *V_out)
{
    if (!config_ok(cfg) || !w || !enc || T < 1 || layer < 0 || layer >= cfg->n_layers) return -1;
    int d = cfg->d_model;
    const aedo_layer *lw = &w->layers[layer];
    double *x = (double *)malloc(sizeof(double) * (size_t)d);
    double *kv = (double *)malloc(sizeof(double) * (size_t)(2 * d));
    for (int t = 0; t < T; ++t) {
        for (int i = 0; i < d; ++i) x[i] = (double)enc[(size_t)t * d + i];
        aedo_linear(x, lw->w_ckv, lw->b_ckv, d, 2 * d, kv);
        if (cfg->kv_fp8) store_as_fp8(kv, 2 * d);
        memcpy(K_out + (size_t)t * d, kv, sizeof(double) * (size_t)d);
        memcpy(V_out + (size_t)t * d, kv + d, sizeof(double) * (size_t)d);
    }
    free(x);
    free(kv);
    return 0;
}

/* ------------------------------------------------------------------ */
/* one sequence, one position at a time                                */
/* ------------------------------------------------------------------ */
typedef struct {
    int T, cap, len; /* encoder frames; self-cache capacity; positions cached */
    double **Kc, **Vc; /* per layer [T, d] */
    double **Ks, **Vs; /* per layer [cap, d] */
    double *x, *h, *qkv, *att, *proj, *ffn;
} seq_state;

static seq_state *seq_new(const aedo_config *cfg, const aedo_weights *w, const float *enc, int T, int cap)
{
    int L = cfg->n_layers, d = cfg->d_model;
    seq_state *s = (seq_state *)calloc(1, sizeof(seq_state));
    s->T = T;
    s->cap = cap;
    s->len = 0;
    s->Kc = (double **)calloc((size_t)L, sizeof(double *));
    s->Vc = (double **)calloc((size_t)L, sizeof(double *));
    s->Ks = (double **)calloc((size_t)L, sizeof(double *));
    s->Vs = (double **)calloc((size_t)L, sizeof(double *));
    for (int l = 0; l < L; ++l) {
        s->Kc[l] = (double *)malloc(sizeof(double) * (size_t)T * d);
        s->Vc[l] = (double *)malloc(sizeof(double) * (size_t)T * d);
        s->Ks[l] = (double *)malloc(sizeof(double) * (size_t)cap * d);
        s->Vs[l] = (double *)malloc(sizeof(double) * (size_t)cap * d);
        aedo_cross_kv(cfg, w, l, enc, T, s->Kc[l], s->Vc[l]);
    }
    s->x = (double *)malloc(sizeof(double) * (size_t)d);
    s->h = (double *)malloc(sizeof(double) * (size_t)d);
    s->qkv = (double *)malloc(sizeof(double) * (size_t)3 * d);
    s->att = (double *)malloc(sizeof(double) * (size_t)d);
    s->proj = (double *)malloc(sizeof(double) * (size_t)d);
    s->ffn = (double *)malloc(sizeof(double) * (size_t)cfg->d_ffn);
    return s;
}

static void seq_free(const aedo_config *cfg, seq_state *s)
{
    for (int l = 0; l < cfg->n_layers; ++l) {
        free(s->Kc[l]);
        free(s->Vc[l]);
        free(s->Ks[l]);
        free(s->Vs[l]);
    }
    free(s->Kc);
    free(s->Vc);
    free(s->Ks);
    free(s->Vs);
    free(s->x);
    free(s->h);
    free(s->qkv);
    free(s->att);
    free(s->proj);
    free(s->ffn);
    free(s);
}

/* Feed token `tok` at position s->len; logits [V] out. */
static void seq_step(const aedo_config *cfg, const aedo_weights *w, seq_state *s, int32_t tok, double *logits)
{
    int d = cfg->d_model, H = cfg->n_heads, dh = cfg->head_dim, F = cfg->d_ffn;
    int pos = s->len;
    double eps = (double)cfg->ln_eps;
    for (int i = 0; i < d; ++i)
        s->x[i] = (double)cfg->emb_scale * (double)w->tok_emb[(size_t)tok * d + i] +
                  (double)w->pos_emb[(size_t)pos * d + i];
    for (int l = 0; l < cfg->n_layers; ++l) {
        const aedo_layer *lw = &w->layers[l];
        /* causal self-attention: the cache holds positions 0..pos */
        norm_rows(cfg, s->x, lw->ln1_g, lw->ln1_b, d, eps, s->h);
        aedo_linear(s->h, lw->w_qkv, lw->b_qkv, d, 3 * d, s->qkv);
        if (cfg->kv_fp8) store_as_fp8(s->qkv + d, 2 * d);
        memcpy(s->Ks[l] + (size_t)pos * d, s->qkv + d, sizeof(double) * (size_t)d);
        memcpy(s->Vs[l] + (size_t)pos * d, s->qkv + 2 * d, sizeof(double) * (size_t)d);
        for (int hd = 0; hd < H; ++hd)
            aedo_attend(s->qkv + hd * dh, s->Ks[l] + hd * dh, s->Vs[l] + hd * dh, pos + 1, dh, d,
                        s->att + hd * dh, NULL);
        aedo_linear(s->att, lw->w_o, lw->b_o, d, d, s->proj);
        for (int i = 0; i < d; ++i) s->x[i] += s->proj[i];
        /* cross-attention over this sequence's own T encoder frames */
        norm_rows(cfg, s->x, lw->ln2_g, lw->ln2_b, d, eps, s->h);
        aedo_linear(s->h, lw->w_cq, lw->b_cq, d, d, s->qkv);
        for (int hd = 0; hd < H; ++hd)
            aedo_attend(s->qkv + hd * dh, s->Kc[l] + hd * dh, s->Vc[l] + hd * dh, s->T, dh, d,
                        s->att + hd * dh, NULL);
        aedo_linear(s->att, lw->w_co, lw->b_co, d, d, s->proj);
        for (int i = 0; i < d; ++i) s->x[i] += s->proj[i];
        /* feed-forward */
        norm_rows(cfg, s->x, lw->ln3_g, lw->ln3_b, d, eps, s->h);
        aedo_linear(s->h, lw->w_ff1, lw->b_ff1, d, F, s->ffn);
        for (int i = 0; i < F; ++i)
            if (s->ffn[i] < 0.0) s->ffn[i] = 0.0;
        aedo_linear(s->ffn, lw->w_ff2, lw->b_ff2, F, d, s->proj);
        for (int i = 0; i < d; ++i) s->x[i] += s->proj[i];
    }
    norm_rows(cfg, s->x, w->lnf_g, w->lnf_b, d, eps, s->h);
    aedo_linear(s->h, w->w_out, w->b_out, d, cfg->vocab, logits);
    s->len = pos + 1;
}

static int lens_ok(const int32_t *lens, int B)
{
    if (!lens || B < 1) return 0;
    for (int b = 0; b < B; ++b)
        if (lens[b] < 1) return 0;
    return 1;
}

int aedo_decode_forced(const aedo_config *cfg, const aedo_weights *w,
                       const float *enc, const int32_t *enc_lens, int B,
                       const int32_t *tokens, int S, double *logits_out)
{
    if (!config_ok(cfg) || !w || !enc || !tokens || !logits_out || !lens_ok(enc_lens, B)) return -1;
    if (S < 1 || S > cfg->max_positions) return -1;
    for (int i = 0; i < B * S; ++i)
        if (tokens[i] < 0 || tokens[i] >= cfg->vocab) return -1;
    int d = cfg->d_model, V = cfg->vocab;
    size_t *off = (size_t *)malloc(sizeof(size_t) * (size_t)(B + 1));
    off[0] = 0;
    for (int b = 0; b < B; ++b) off[b + 1] = off[b] + (size_t)enc_lens[b];
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        seq_state *s = seq_new(cfg, w, enc + off[b] * d, enc_lens[b], S);
        for (int t = 0; t < S; ++t)
            seq_step(cfg, w, s, tokens[(size_t)b * S + t], logits_out + ((size_t)b * S + t) * V);
        seq_free(cfg, s);
    }
    free(off);
    return 0;
}

int aedo_self_kv(const aedo_config *cfg, const aedo_weights *w, const float *enc, int T,
                 const int32_t *tokens, int S, int layer, double *K_out, double *V_out)
{
    if (!config_ok(cfg) || !w || !enc || !tokens || !K_out || !V_out || T < 1) return -1;
    if (S < 1 || S > cfg->max_positions || layer < 0 || layer >= cfg->n_layers) return -1;
    for (int i = 0; i < S; ++i)
        if (tokens[i] < 0 || tokens[i] >= cfg->vocab) return -1;
    int d = cfg->d_model;
    double *logits = (double *)malloc(sizeof(double) * (size_t)cfg->vocab);
    seq_state *s = seq_new(cfg, w, enc, T, S);
    for (int t = 0; t < S; ++t) seq_step(cfg, w, s, tokens[t], logits);
    memcpy(K_out, s->Ks[layer], sizeof(double) * (size_t)S * d);
    memcpy(V_out, s->Vs[layer], sizeof(double) * (size_t)S * d);
    seq_free(cfg, s);
    free(logits);
    return 0;
}

int aedo_greedy_decode(const aedo_config *cfg, const aedo_weights *w,
                       const float *enc, const int32_t *enc_lens, int B,
                       const int32_t *prompt, int P, int max_new,
                       const int32_t *max_new_per_seq,
                       int32_t *out_tokens, int32_t *out_lens, double *logits_out)
{
    if (!config_ok(cfg) || !w || !enc || !prompt || !out_tokens || !out_lens || !lens_ok(enc_lens, B))
        return -1;
    if (P < 1 || max_new < 1 || P + max_new > cfg->max_positions) return -1;
    if (max_new_per_seq && cfg->eos_id < 0) return -1;
    for (int i = 0; i < B * P; ++i)
        if (prompt[i] < 0 || prompt[i] >= cfg->vocab) return -1;
    if (max_new_per_seq)
        for (int b = 0; b < B; ++b)
            if (max_new_per_seq[b] < 1) return -1;
    int d = cfg->d_model, V = cfg->vocab;
    size_t *off = (size_t *)malloc(sizeof(size_t) * (size_t)(B + 1));
    off[0] = 0;
    for (int b = 0; b < B; ++b) off[b + 1] = off[b] + (size_t)enc_lens[b];
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        seq_state *s = seq_new(cfg, w, enc + off[b] * d, enc_lens[b], P + max_new);
        double *logits = (double *)malloc(sizeof(double) * (size_t)V);
        /* prompt positions 0..P-2: logits discarded */
        for (int p = 0; p + 1 < P; ++p) seq_step(cfg, w, s, prompt[(size_t)b * P + p], logits);
        int32_t tok = prompt[(size_t)b * P + P - 1];
        int n = 0, finished = 0;
        while (n < max_new && !finished) {
            seq_step(cfg, w, s, tok, logits);
            if (logits_out) memcpy(logits_out + ((size_t)b * max_new + n) * V, logits, sizeof(double) * (size_t)V);
            tok = aedo_argmax(logits, V);
            if (max_new_per_seq && n + 1 >= max_new_per_seq[b]) tok = cfg->eos_id; /* forced EOS */
            out_tokens[(size_t)b * max_new + n] = tok;
            ++n;
            if (cfg->eos_id >= 0 && tok == cfg->eos_id) finished = 1;
        }
        out_lens[b] = n;
        for (int t = n; t < max_new; ++t) out_tokens[(size_t)b * max_new + t] = cfg->pad_id;
        free(logits);
        seq_free(cfg, s);
    }
    free(off);
    return 0;
}

/* ------------------------------------------------------------------ */
/* independent second routine: padded batch, dense masked attention    */
/* ------------------------------------------------------------------ */
/* scores [n_q, n_k] with mask (0 = masked out) -> out [n_q, dh] for one head;
 * Q,K,V are [n, d]-strided. */
static void masked_attention_head(const double *Q, const double *K, const double *V,
                                  int n_q, int n_k, int dh, int stride,
                                  const unsigned char *mask /*[n_q, n_k]*/, double *out /*[n_q, stride]*/)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)n_k);
    double *p = (double *)malloc(sizeof(double) * (size_t)n_k);
    double scale = 1.0 / sqrt((double)dh);
    for (int i = 0; i < n_q; ++i) {
        for (int j = 0; j < n_k; ++j) {
            if (!mask[(size_t)i * n_k + j]) {
                a[j] = -INFINITY;
                continue;
            }
            double dot = 0.0;
            for (int c = 0; c < dh; ++c) dot += Q[(size_t)i * stride + c] * K[(size_t)j * stride + c];
            a[j] = dot * scale;
        }
        aedo_softmax(a, n_k, p); /* exp(-inf - m) = 0: masked keys get zero weight */
        for (int c = 0; c < dh; ++c) {
            double acc = 0.0;
            for (int j = 0; j < n_k; ++j)
                if (mask[(size_t)i * n_k + j]) acc += p[j] * V[(size_t)j * stride + c];
            out[(size_t)i * stride + c] = acc;
        }
    }
    free(a);
    free(p);
}

int aedo_forward_full(const aedo_config *cfg, const aedo_weights *w,
                      const float *enc_padded, int T_max, const int32_t *enc_lens, int B,
                      const int32_t *tokens, int S_max, const int32_t *tok_lens,
                      double *logits_out)
{
    if (!config_ok(cfg) || !w || !enc_padded || !tokens || !logits_out) return -1;
    if (!lens_ok(enc_lens, B) || !lens_ok(tok_lens, B)) return -1;
    if (S_max < 1 || S_max > cfg->max_positions || T_max < 1) return -1;
    for (int b = 0; b < B; ++b)
        if (enc_lens[b] > T_max || tok_lens[b] > S_max) return -1;
    int d = cfg->d_model, H = cfg->n_heads, dh = cfg->head_dim, F = cfg->d_ffn, V = cfg->vocab;
    double eps = (double)cfg->ln_eps;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int S = S_max, T = T_max; /* work on the PADDED shapes; masks remove the padding */
        double *X = (double *)calloc((size_t)S * d, sizeof(double));
        double *Hn = (double *)calloc((size_t)S * d, sizeof(double));
        double *Q = (double *)calloc((size_t)S * d, sizeof(double));
        double *K = (double *)calloc((size_t)S * d, sizeof(double));
        double *Vv = (double *)calloc((size_t)S * d, sizeof(double));
        double *A = (double *)calloc((size_t)S * d, sizeof(double));
        double *Kc = (double *)calloc((size_t)T * d, sizeof(double));
        double *Vc = (double *)calloc((size_t)T * d, sizeof(double));
        double *row3 = (double *)malloc(sizeof(double) * (size_t)3 * d);
        double *rowF = (double *)malloc(sizeof(double) * (size_t)F);
        double *rowd = (double *)malloc(sizeof(double) * (size_t)d);
        double *encrow = (double *)malloc(sizeof(double) * (size_t)d);
        unsigned char *self_mask = (unsigned char *)malloc((size_t)S * S);
        unsigned char *cross_mask = (unsigned char *)malloc((size_t)S * T);
        for (int i = 0; i < S; ++i) {
            for (int j = 0; j < S; ++j) self_mask[(size_t)i * S + j] = (j <= i) && (j < tok_lens[b]);
            for (int j = 0; j < T; ++j) cross_mask[(size_t)i * T + j] = (j < enc_lens[b]);
        }
        for (int s = 0; s < S; ++s) {
            int32_t tok = tokens[(size_t)b * S_max + s];
            if (s >= tok_lens[b] || tok < 0 || tok >= V) tok = 0; /* padded position: any valid id */
            for (int i = 0; i < d; ++i)
                X[(size_t)s * d + i] = (double)cfg->emb_scale * (double)w->tok_emb[(size_t)tok * d + i] +
                                       (double)w->pos_emb[(size_t)s * d + i];
        }
        for (int l = 0; l < cfg->n_layers; ++l) {
            const aedo_layer *lw = &w->layers[l];
            for (int s = 0; s < S; ++s) {
                norm_rows(cfg, X + (size_t)s * d, lw->ln1_g, lw->ln1_b, d, eps, Hn + (size_t)s * d);
                aedo_linear(Hn + (size_t)s * d, lw->w_qkv, lw->b_qkv, d, 3 * d, row3);
                if (cfg->kv_fp8) store_as_fp8(row3 + d, 2 * d);
                memcpy(Q + (size_t)s * d, row3, sizeof(double) * (size_t)d);
                memcpy(K + (size_t)s * d, row3 + d, sizeof(double) * (size_t)d);
                memcpy(Vv + (size_t)s * d, row3 + 2 * d, sizeof(double) * (size_t)d);
            }
            for (int hd = 0; hd < H; ++hd)
                masked_attention_head(Q + hd * dh, K + hd * dh, Vv + hd * dh, S, S, dh, d, self_mask, A + hd * dh);
            for (int s = 0; s < S; ++s) {
                aedo_linear(A + (size_t)s * d, lw->w_o, lw->b_o, d, d, rowd);
                for (int i = 0; i < d; ++i) X[(size_t)s * d + i] += rowd[i];
            }
            /* cross memory over ALL T_max rows, padding included; the mask removes it.
             * Padded rows may hold NaN/Inf: they are never multiplied into a result. */
            for (int t = 0; t < T; ++t) {
                if (t < enc_lens[b]) {
                    for (int i = 0; i < d; ++i)
                        encrow[i] = (double)enc_padded[((size_t)b * T_max + t) * d + i];
                    aedo_linear(encrow, lw->w_ckv, lw->b_ckv, d, 2 * d, row3);
                    if (cfg->kv_fp8) store_as_fp8(row3, 2 * d);
                    memcpy(Kc + (size_t)t * d, row3, sizeof(double) * (size_t)d);
                    memcpy(Vc + (size_t)t * d, row3 + d, sizeof(double) * (size_t)d);
                }
            }
            for (int s = 0; s < S; ++s) {
                norm_rows(cfg, X + (size_t)s * d, lw->ln2_g, lw->ln2_b, d, eps, Hn + (size_t)s * d);
                aedo_linear(Hn + (size_t)s * d, lw->w_cq, lw->b_cq, d, d, Q + (size_t)s * d);
            }
            for (int hd = 0; hd < H; ++hd)
                masked_attention_head(Q + hd * dh, Kc + hd * dh, Vc + hd * dh, S, T, dh, d, cross_mask, A + hd * dh);
            for (int s = 0; s < S; ++s) {
                aedo_linear(A + (size_t)s * d, lw->w_co, lw->b_co, d, d, rowd);
                for (int i = 0; i < d; ++i) X[(size_t)s * d + i] += rowd[i];
            }
            for (int s = 0; s < S; ++s) {
                norm_rows(cfg, X + (size_t)s * d, lw->ln3_g, lw->ln3_b, d, eps, Hn + (size_t)s * d);
                aedo_linear(Hn + (size_t)s * d, lw->w_ff1, lw->b_ff1, d, F, rowF);
                for (int i = 0; i < F; ++i)
                    if (rowF[i] < 0.0) rowF[i] = 0.0;
                aedo_linear(rowF, lw->w_ff2, lw->b_ff2, F, d, rowd);
                for (int i = 0; i < d; ++i) X[(size_t)s * d + i] += rowd[i];
            }
        }
        for (int s = 0; s < S; ++s) {
            double *out = logits_out + ((size_t)b * S_max + s) * V;
            if (s >= tok_lens[b]) {
                memset(out, 0, sizeof(double) * (size_t)V);
                continue;
            }
            norm_rows(cfg, X + (size_t)s * d, w->lnf_g, w->lnf_b, d, eps, rowd);
            aedo_linear(rowd, w->w_out, w->b_out, d, V, out);
        }
        free(X); free(Hn); free(Q); free(K); free(Vv); free(A); free(Kc); free(Vc);
        free(row3); free(rowF); free(rowd); free(encrow); free(self_mask); free(cross_mask);
    }
    return 0;
}
