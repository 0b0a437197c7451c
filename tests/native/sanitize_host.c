/* Host-code sanitizer run: a tiny decoder through the CPU oracle (incremental, greedy and padded
 * routines) built with -fsanitize=address,undefined.  Exit code 0 and no sanitizer report = clean. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/aed_oracle.h"

static float frand(unsigned *s) { *s = *s * 1664525u + 1013904223u; return ((*s >> 8) / 16777216.0f - 0.5f) * 0.6f; }

int main(void)
{
    aedo_config c = {2, 16, 2, 8, 24, 11, 12, 3, 0, 1e-5f, 1.0f};
    unsigned s = 7;
    int d = c.d_model, F = c.d_ffn, V = c.vocab;
    aedo_layer layers[2];
    float *pool = (float *)malloc(sizeof(float) * 200000);
    size_t used = 0;
#define TAKE(n) (pool + (used += (size_t)(n)) - (size_t)(n))
    for (size_t i = 0; i < 200000; ++i) pool[i] = frand(&s);
    for (int l = 0; l < 2; ++l) {
        aedo_layer *w = &layers[l];
        w->ln1_g = TAKE(d); w->ln1_b = TAKE(d); w->w_qkv = TAKE(3 * d * d); w->b_qkv = TAKE(3 * d);
        w->w_o = TAKE(d * d); w->b_o = NULL;
        w->ln2_g = TAKE(d); w->ln2_b = TAKE(d); w->w_cq = TAKE(d * d); w->b_cq = TAKE(d);
        w->w_ckv = TAKE(2 * d * d); w->b_ckv = TAKE(2 * d); w->w_co = TAKE(d * d); w->b_co = TAKE(d);
        w->ln3_g = TAKE(d); w->ln3_b = TAKE(d); w->w_ff1 = TAKE(F * d); w->b_ff1 = TAKE(F);
        w->w_ff2 = TAKE(d * F); w->b_ff2 = TAKE(d);
    }
    aedo_weights w = {TAKE(V * d), TAKE(c.max_positions * d), TAKE(d), TAKE(d), TAKE(V * d), TAKE(V), layers};
    int32_t enc_lens[3] = {5, 1, 9};
    float *enc = TAKE(15 * d);
    int32_t prompt[6] = {4, 5, 6, 7, 8, 9};
    int32_t out_tokens[3 * 8], out_lens[3], limits[3] = {2, 8, 1};
    double *logits = (double *)malloc(sizeof(double) * 3 * 8 * V);
    if (aedo_greedy_decode(&c, &w, enc, enc_lens, 3, prompt, 2, 8, limits, out_tokens, out_lens, logits) != 0) return 2;
    if (out_lens[2] != 1 || out_tokens[2 * 8] != 3 || out_lens[0] > 2) return 3;
    int32_t toks[3 * 5];
    for (int i = 0; i < 15; ++i) toks[i] = i % V;
    double *forced = (double *)malloc(sizeof(double) * 3 * 5 * V), *full = (double *)malloc(sizeof(double) * 3 * 5 * V);
    if (aedo_decode_forced(&c, &w, enc, enc_lens, 3, toks, 5, forced) != 0) return 4;
    float *padded = (float *)calloc((size_t)3 * 9 * d, sizeof(float));
    int off = 0;
    for (int b = 0; b < 3; ++b) { memcpy(padded + (size_t)b * 9 * d, enc + (size_t)off * d, sizeof(float) * enc_lens[b] * d); off += enc_lens[b]; }
    int32_t tok_lens[3] = {5, 5, 5};
    if (aedo_forward_full(&c, &w, padded, 9, enc_lens, 3, toks, 5, tok_lens, full) != 0) return 5;
    double worst = 0;
    for (int i = 0; i < 3 * 5 * V; ++i) worst = fmax(worst, fabs(forced[i] - full[i]));
    printf("incremental vs full: %.3e\n", worst);
    if (!(worst < 1e-9)) return 6;
    if (aedo_decode_forced(&c, &w, enc, enc_lens, 0, toks, 5, forced) == 0) return 7; /* bad batch is rejected */
    free(pool); free(logits); free(forced); free(full); free(padded);
    return 0;
}
