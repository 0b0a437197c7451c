// Host-side launch interface of the gfx950 kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aed {

enum Dtype { kF32 = 0, kBF16 = 1 };
constexpr int kPage = 16;  // tokens per self-attention KV page

// ---------------------------------------------------------------- decode GEMM
// C[M,N] = prologue(A)[M,K] . W[N,K]^T (+bias), then an epilogue.
// PRO_LNS (bfloat16 mode): the LayerNorm is folded around the product instead of being applied to the operand.
// Whoever writes the residual rows x (embedding, EPI_RESID_S) also writes their "shadow" x - mu_hat in the
// storage type and fragment order (mu_hat: the row mean before the update, so the shadow has no large common
// offset) and per-row statistics of x; the gain g of the LayerNorm is multiplied into the matrix once, when the
// decoder is created (Wg = W . diag(g), rounded to the storage type), and then
//   W . LN(x) + bias = rstd * (Wg . shadow - (mu - mu_hat) * c1) + c2,  c1 = Wg . 1,  c2 = W . b + bias,
// so the product streams half the bytes of the float32 rows and needs no pass over them first, and one shadow
// serves every product that reads the rows.
enum GemmPro { PRO_LN = 0, PRO_T = 1, PRO_LNS = 2 };
// EPI_RESID_S: EPI_RESID that also writes the shadow and the statistics of the updated rows.
enum GemmEpi { EPI_QKV = 0, EPI_RESID = 1, EPI_F32 = 2, EPI_RELU_T = 3, EPI_CROSSKV = 4, EPI_RESID_S = 5 };

struct GemmArgs {
    const void* A;        // PRO_LN: float [M,K] (residual stream); PRO_T: T [M,K]; both in fragment order
    int n_raw;            // PRO_LNS + EPI_QKV, streaming kernel: columns [n_raw, N) (n_raw = 3 d_model) are not normalised and not
    float* out2;          // part of q/k/v: their bare sums plus raw_bias go to out2, float [M, N - n_raw] row-major.  0: no such columns
    const float* raw_bias;  // [N - n_raw]
    const float* addend;  // PRO_T / PRO_LN + EPI_F32, streaming kernel, may be null: float [M,N] row-major added to the result
    const void* W;        // T [N,K] in fragment order (launch_reorder_weight)
    const void* bias;     // T [N] or null
    const void* ln_g;     // T [K]  (PRO_LN)
    const void* ln_b;     // T [K]
    float ln_eps;
    void* ln_scratch;     // T [M,K] fragment order: LN(x) when the LayerNorm runs as its own launch (M > 128)
    int M, N, K;
    void* out;            // EPI_RESID: float [M,N] fragment order, += ; EPI_F32: float [M,N] row-major;
                          // EPI_RELU_T: T [M,N] fragment order; EPI_QKV: float q [M,d_model] row-major
    // EPI_QKV: columns [d,2d) and [2d,3d) go to the paged self-attention cache of this layer
    void* k_pool;         // T (or E4M3 codes, kv_fp8) [pages][H][16][Dh]
    void* v_pool;
    const int* page_table;  // [batch][max_pages]
    int max_pages;
    const int* seq_len;     // position being written, per sequence
    const int* finished;    // nonzero: do not append
    int n_heads, head_dim, d_model;
    // EPI_CROSSKV: columns [0,d) -> kc, [d,2d) -> vc, layout [H][t_cap][Dh]
    void* kc;
    void* vc;
    long long t_cap;
    const int* out_row_map;  // EPI_CROSSKV, may be null: frame slot that GEMM row m is written to (default m)
    int a_rows;              // rows the A buffer holds (0: only the next multiple of 128 above M is promised)
    // Row statistics of the residual rows: for every row and every 16-column tile, the tile's mean and its sum
    // of squared deviations from that mean, [stat_tiles][m_stride] (stat_tiles = d_model / 16).
    const float2* stats_in;  // PRO_LNS: of A's rows
    const float* mu_hat_in;  // PRO_LNS: [M] the shift the shadow was written with;
                             // EPI_RESID_S: [M] row means before the update = the shift to write the shadow with
    const float* ln_c1;      // PRO_LNS: [N]
    const float* ln_c2;      // PRO_LNS: [N] (takes the place of bias)
    float* mu_hat_out;       // PRO_LNS, may be null: [M] row means of A's rows, for the residual updates that follow
    float2* stats_out;       // EPI_RESID_S: of the updated rows
    void* shadow_out;        // EPI_RESID_S: T [M,N] fragment order
    int stat_tiles, m_stride;
    int kv_fp8;              // EPI_QKV / EPI_CROSSKV: the caches hold 8-bit E4M3 codes instead of T
    int rms;                 // the normalisation is RMSNorm (no mean subtraction; ln_b may be null) instead of LayerNorm:
                             // PRO_LN normalises that way, PRO_LNS reads the statistics that way (see fold_norm)
    int w_nt;                // streaming kernel: load W with the non-temporal hint (weights that are not expected to
                             // survive in the caches until the next step anyway, and should not push other data out)
};

// Buffers in fragment order must hold a multiple of 128 rows (rows >= M are read, never written).
// Returns hipSuccess or the launch error.  Requirements (checked by the caller):
// K % 256 == 0, N % 64 == 0, PRO_LN: K <= 1024.
hipError_t launch_gemm(Dtype dt, GemmPro pro, GemmEpi epi, const GemmArgs& a, hipStream_t s);
// LDS-tiled MFMA GEMM for large M (bf16 only; fragment-order A padded to a multiple of 128 rows, N % 128 == 0)
hipError_t launch_gemm_tiled(GemmEpi epi, const GemmArgs& a, hipStream_t s);
// the same 128 x 128 tile fed by direct-to-LDS loads (bf16, K >= 512, not EPI_RESID); a.ln_c1 != null: PRO_LNS
hipError_t launch_gemm_dma128(GemmEpi epi, const GemmArgs& a, hipStream_t s);
// bf16 cross K/V product with 256 x 256 tiles fed by direct-to-LDS loads; A must hold whole 256-row tiles
hipError_t launch_gemm_dma_crosskv(const GemmArgs& a, hipStream_t s);
// dst (fragment order [M,K]) <- rows of a row-major source; row m comes from src row row_map[m] (or m); K % 64 == 0
hipError_t launch_reorder_rows(Dtype dt, const void* src, const int* row_map, void* dst, int M, int K, hipStream_t s);
// c1[n] = sum_k T(W[n,k] g[k]) (the column-scaled matrix as it is stored), c2[n] = sum_k W[n,k] b[k] + bias[n]
// (float32 sums; W row-major [N,K]; b and bias may be null)
hipError_t launch_fold_ln(Dtype dt, const void* W, const void* g, const void* b, const void* bias, float* c1, float* c2,
                          int N, int K, hipStream_t s);
// dst (fragment order) <- src (row-major [N,K]), each column k multiplied by gain[k] if gain is given (T [K];
// the product is rounded to T once); N % 16 == 0, K % 64 == 0.  With dst_K > 0 the destination is a fragment-order
// matrix of dst_K columns and src lands in its columns dst_k0 .. dst_k0 + K.
hipError_t launch_reorder_weight(Dtype dt, const void* src, const void* gain, void* dst, int N, int K, hipStream_t s,
                                 int dst_k0 = 0, int dst_K = 0);

// Merged products (bfloat16 mode, at most 256 rows).  A residual update x' = x + Wa . o + ba followed by a LayerNorm
// product Wb . LN(x') reads, in folded form, Wbg . (x' - mu_hat) = Wbg . (x - mu_hat) + (Wbg . Wa) . o + Wbg . ba.
// With the matrix product Wbg . Wa formed once at create, the second product no longer waits for the update:
//   P1 = Wbg . (x - mu_hat) + cb   needs only the shadow of x: computed by the launch that already reads that shadow
//                             (the QKV product, as extra columns: GemmArgs::n_raw, raw_bias),
//   P2 = (Wbg . Wa) . o       needs only o: computed in the same launch as the update (launch_gemm_pair), which
//                             adds P1 to it (GemmArgs::addend),
// and whoever reads P = P1 + P2 finishes it with the statistics of x' that the update's tiles wrote:
//   Wb . LN(x') + bb = rstd' * (P - (mu' - mu_hat) * c1) + c2,  cb = Wbg . ba, c1 = Wbg . 1, c2 = Wb . beta + bb.
// One launch per layer less (self-attention output projection + cross-attention query product).
// launch_gemm_pair: a0 = the update (EPI_RESID_S), a1 = the product P2 (PRO_T, epilogue epi1 = EPI_F32).
hipError_t launch_gemm_pair(Dtype dt, const GemmArgs& a0, GemmEpi epi1, const GemmArgs& a1, hipStream_t s);
// P[n,k] = sum_j T(W1[n,j] g[j]) W2[j,k] -> T, fragment order, columns dst_k0.. of a matrix with dst_K columns
// (W1 [N,J], W2 [J,K] row-major, g null or T [J]; N, K % 64 == 0, J % 16 == 0); bfloat16 only
hipError_t launch_weight_product(Dtype dt, const void* W1, const void* g, const void* W2, void* dst, int N, int J, int K,
                                 int dst_k0, int dst_K, hipStream_t s);
// out[n] = sum_j T(W[n,j] g[j]) v[j] (v null: zeros); bfloat16 only
hipError_t launch_fold_vec(Dtype dt, const void* W, const void* g, const void* v, float* out, int N, int J, hipStream_t s);

// ---------------------------------------------------------------- decode attention
struct AttnArgs {
    const float* q;       // [B, d_model]
    void* out;            // T [B, d_model] in fragment order
    const void* K;        // self: T [pages][H][16][Dh]; cross: T [H][t_cap][Dh]  (this layer)
    const void* V;
    int kv_fp8;           // K and V hold 8-bit E4M3 codes instead of T (bfloat16 mode only)
    const int* finished;  // [B]
    // self
    const int* page_table;
    int max_pages;
    const int* seq_len;   // keys = seq_len[b] + 1
    int chunk;            // keys per work item, multiple of 64 (self and cross)
    int n_chunks_max;     // grid.z
    int batch;
    // cross
    const int4* items;    // {b, key_start | chunk_idx << 16, n_keys | n_chunks << 16, first frame of b in the
                          // packed layout}, longest first
    int n_items;
    const int* enc_off;   // [B+1] frame offsets in the packed layout
    long long t_cap;
    // split-K merge
    float* part;          // [B*H][max_chunks][Dh+2]
    int* counters;        // [B*H] arrivals per (sequence, head); zero between launches
    int max_chunks;
    int n_heads, head_dim;
    float scale_log2e;    // log2(e) / sqrt(Dh)
    // cross-attention behind merged products (see "merged products" above): q holds P, and the kernel finishes it
    // with the statistics of the updated rows: q = rstd' (P - (mu' - mu_hat) c1) + c2.  q_stats null: q is final.
    const float2* q_stats;  // [q_stat_tiles][q_m_stride] tile statistics of the updated rows
    const float* q_mu_hat;  // [B] shift of the shadow that P was computed from
    const float* q_c1;      // [d_model]
    const float* q_c2;
    float q_eps;
    int q_stat_tiles, q_m_stride, q_rms;
};
hipError_t launch_attn_self(Dtype dt, const AttnArgs& a, hipStream_t s);
hipError_t launch_attn_cross(Dtype dt, const AttnArgs& a, hipStream_t s);

// ---------------------------------------------------------------- small kernels
struct StateArgs {
    int* seq_len; int* n_gen; int* finished; int* cur_tok; int* limit; int* n_finished;
    int* prompt;      // [B, prompt_stride]
    int* out_tokens;  // [B, out_stride]
    int prompt_len, prompt_stride, out_stride, max_new;
    int eos_id, pad_id, batch, vocab;
};
// What the folded LayerNorm of the first layer needs beside the rows themselves (bfloat16 mode; see PRO_LNS).
// shadow == null: not written.
struct ShadowArgs {
    void* shadow;       // T [B, d] fragment order: x - row mean
    float2* stats;      // [d / 16][m_stride]: mean and sum of squared deviations of every 16-column tile
    float* mu_hat;      // [B] row means (the shadow's shift)
    int m_stride;
    int rms;            // RMSNorm: the shift is 0 (the shadow is x itself in the storage type)
};
// x[b,:] = emb_scale * tok_emb[cur_tok[b]] + pos_emb[seq_len[b]]   (x in fragment order); d_model <= 1024
hipError_t launch_embed(Dtype dt, float* x, const void* tok_emb, const void* pos_emb, const StateArgs& st,
                        int d_model, int max_positions, float emb_scale, const ShadowArgs& sa, hipStream_t s);
// greedy = 1: prompt feeding, argmax, EOS rules, output writes; greedy = 0: argmax only -> step_out (may be null)
hipError_t launch_sample(const float* logits, const StateArgs& st, int greedy, int* step_out, hipStream_t s);
// seq_len = start_pos, cur_tok = prompt[b][start_pos], n_gen = finished = 0, n_finished = 0,
// limit = limits ? limits[b] : INT_MAX, out_tokens = pad (fill_out)
hipError_t launch_reset(const StateArgs& st, const int* limits_dev, int fill_out, int start_pos, hipStream_t s);
// cur_tok[b] = src[b * stride]
hipError_t launch_set_tokens(int* cur_tok, const int* src, int stride, int batch, hipStream_t s);
// out[b] = n_gen[b]; dst[b, t] = out_tokens[b, t]
hipError_t launch_copy_out(const StateArgs& st, int* dst_tokens, int* dst_lens, hipStream_t s);

// Slot turnover of the request queue, one workgroup per entry i: slot slots[i] hands its finished request
// old_reqs[i] over (tokens up to n_gen, then pad_id, and the length, into row old_reqs[i] of dst_tokens
// [n_requests, max_new] / dst_lens; -1: nothing to hand over) and starts request new_reqs[i] at position 0 with
// its prompt row of all_prompts [n_requests, prompt_len] and the limit limits[i] (-1: the slot is parked as
// finished).
hipError_t launch_turn_over_slots(const StateArgs& st, const int* slots, const int* old_reqs, const int* new_reqs,
                                  const int* limits, int n, const int* all_prompts, int* dst_tokens, int* dst_lens,
                                  hipStream_t s);

// page_table[b * max_pages + blk] = first_page + b for b < batch (the step API hands every sequence a new page at once)
hipError_t launch_assign_pages(int* page_table, int max_pages, int blk, int first_page, int batch, hipStream_t s);
// p[0 .. n) = 0
hipError_t launch_fill_zero(int* p, int n, hipStream_t s);

// finished[b] = 0, seq_len[b] = clamp(seq_len[b], 0, max_pos): a valid mid-decode state for timing runs
hipError_t launch_prepare_timing(const StateArgs& st, int max_pos, hipStream_t s);

}  // namespace aed
