// C ABI of the AED decoder library: argument checking, workspace carving, the
// decode state machine, launch-graph capture/replay and measurement helpers.
// All device work is in gemm_decode.hip, attn_decode.hip, step_kernels.hip.
#include <limits.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/aed.h"
#include "frame_space.h"
#include "kernels.h"

using namespace aed;

// Scratch memory of aed_decode_step_noalloc: the step's activations and attention partials, for callers that
// cannot hand over a workspace allocation of their own choosing at that point (see aed.h).  Every GPU the library
// runs on holds its own copy until the process ends.  In host code this name is only a handle: the array's device
// address comes from hipGetSymbolAddress, once per device (scratch_of_current_device).
constexpr size_t kStaticScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

// The static scratch array's address on the current device; resolved on first use per device.
hipError_t scratch_of_current_device(char** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static char* ptr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = static_cast<char*>(p);
    }
    *out = ptr[dev];
    return hipSuccess;
}

constexpr int kMaxChunks = 8;       // split-K chunks per (sequence, head)
constexpr int kTargetItems = 512;      // work items aimed at per attention launch when sequences are cut
constexpr int kMinItemsNoSplit = 128;  // batch * heads from which sequences are never cut
constexpr int kMaxPrefillPositions = 8;  // prompt positions per prefill pass

thread_local std::string g_create_error;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Offsets (bytes) of everything carved from the caller's workspace.
struct Layout {
    size_t x, q, q_aux, logits, attn_out, ffn_h, ln_h, x_shadow, ln_stats, mu_hat, ln_fold;
    size_t stats_elems;  // float2 per statistics buffer
    size_t shadow_bytes; // bytes per shadow buffer
    size_t act_bytes;    // [0, act_bytes): the step's activations and attention partials (x ... counters)
    size_t seq_len, n_gen, finished, cur_tok, limit, limits_in, n_finished, step_tok;
    size_t prompt_buf, out_buf, page_table, enc_off, row_map, frame_map, turn_buf, items, part, counters;
    size_t v_seq_len, v_finished, v_cur_tok, v_page_table, v_items;  // state of a prompt-prefill pass's rows
    int act_rows;  // rows the activation buffers hold: max(max_batch, prefill_rows)
    size_t k_pool, v_pool, kc, vc, w_frag, enc_frag;
    size_t w_merge, merge_vec;  // bfloat16 mode: the merged products' matrices and bias vectors (kernels.h)
    size_t total;
    int max_pages, n_pages, max_items;
    size_t pool_layer_elems, cross_layer_elems;
};

aed_status check_config(const aed_config* c, std::string& err) {
    auto bad = [&](const char* m) { err = m; return AED_EINVAL; };
    auto unsup = [&](const char* m) { err = m; return AED_EUNSUPPORTED; };
    if (!c) return bad("config is NULL");
    if (c->struct_size != sizeof(aed_config)) return bad("aed_config.struct_size does not match this library");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->head_dim < 1 || c->d_ffn < 1 || c->vocab < 1 ||
        c->max_positions < 1)
        return bad("model dimensions must be positive");
    if ((long long)c->n_heads * c->head_dim != c->d_model) return bad("n_heads * head_dim != d_model");
    if (c->dtype != 0 && c->dtype != 1) return bad("dtype must be 0 (float32) or 1 (bfloat16)");
    if (c->max_batch < 1 || c->max_total_enc_frames < 1 || c->max_dec_len < 1) return bad("capacities must be positive");
    if (c->max_total_enc_frames < c->max_batch) return bad("max_total_enc_frames < max_batch (every sequence has >= 1 frame)");
    if (c->kv_pages < 0) return bad("kv_pages < 0");
    if (!(c->ln_eps > 0.f)) return bad("ln_eps must be > 0");
    if (c->eos_id >= c->vocab || c->pad_id < 0) return bad("eos_id / pad_id out of range");
    if (c->norm_type != 0 && c->norm_type != 1) return bad("norm_type must be 0 (LayerNorm) or 1 (RMSNorm)");
    if (c->page_size != kPage) return unsup("page_size must be 16");
    if (c->head_dim != 64 && c->head_dim != 128) return unsup("head_dim must be 64 or 128");
    if (c->d_model % 256 != 0 || c->d_model > 1024) return unsup("d_model must be a multiple of 256, at most 1024");
    if (c->d_ffn % 256 != 0) return unsup("d_ffn must be a multiple of 256");
    if (c->vocab % 64 != 0) return unsup("vocab must be a multiple of 64");
    if (c->max_batch > 65535) return unsup("max_batch above 65535");
    if (c->prefill_rows < 0 || c->prefill_rows > 65535) return bad("prefill_rows must be in [0, 65535]");
    if (c->kv_fp8 != 0 && c->kv_fp8 != 1) return bad("kv_fp8 must be 0 or 1");
    if (c->kv_fp8 && c->dtype != 1) return unsup("8-bit key / value caches go with bfloat16 models only");
    return AED_OK;
}

void make_layout(const aed_config* c, Layout* L) {
    const size_t e = c->dtype == 1 ? 2 : 4;
    const size_t B = c->max_batch, d = c->d_model, H = c->n_heads, Dh = c->head_dim;
    // activations hold the rows of a decode step or of a prompt-prefill pass, whichever is more
    const size_t Ba = std::max<size_t>(B, (size_t)c->prefill_rows);
    L->act_rows = (int)Ba;
    const size_t Bp = align_up(Ba, 128);  // fragment-order activations are read in whole tiles of up to 128 rows
    L->max_pages = (c->max_dec_len + kPage - 1) / kPage;
    L->n_pages = c->kv_pages > 0 ? c->kv_pages : (int)(B * L->max_pages);
    L->max_items = c->max_total_enc_frames / 64 + c->max_batch;
    L->pool_layer_elems = (size_t)L->n_pages * H * kPage * Dh;
    L->cross_layer_elems = (size_t)c->max_total_enc_frames * d;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L->x = take(Bp * d * 4);
    L->q = take(Ba * d * 4);
    L->q_aux = take(c->dtype == 1 ? Ba * d * 4 : 0);  // merged products: the part of the cross-attention query that the QKV launch computes
    L->logits = take(B * (size_t)c->vocab * 4);
    L->attn_out = take(Bp * d * e);
    L->ffn_h = take(Bp * (size_t)c->d_ffn * e);
    L->ln_h = take(Bp * d * e);
    // bfloat16 mode: LayerNorm folded around the products (shadow of the residual rows, tile statistics in two
    // buffers that alternate from one residual update to the next, row shifts, folded gain/shift vectors)
    L->x_shadow = take(2 * Bp * d * e);  // two buffers, alternating like the statistics
    L->shadow_bytes = Bp * d * e;
    L->stats_elems = (d / 16) * Bp;
    L->ln_stats = take(2 * L->stats_elems * 8);
    L->mu_hat = take(2 * Bp * 4);  // two buffers, alternating like the statistics
    L->part = take(Ba * H * kMaxChunks * (Dh + 2) * 4);
    L->counters = take(Ba * H * 4);
    L->act_bytes = off;  // everything above is rewritten by every step before it is read (the counters: zero between launches)
    L->ln_fold = take(((size_t)c->n_layers * (4 * d + (size_t)c->d_ffn) + (size_t)c->vocab) * 2 * 4);
    L->seq_len = take(B * 4);
    L->n_gen = take(B * 4);
    L->finished = take(B * 4);
    L->cur_tok = take(B * 4);
    L->limit = take(B * 4);
    L->limits_in = take(B * 4);
    L->n_finished = take(256);
    L->step_tok = take(B * 4);
    L->prompt_buf = take(B * (size_t)c->max_dec_len * 4);
    L->out_buf = take(B * (size_t)c->max_dec_len * 4);
    L->page_table = take(B * (size_t)L->max_pages * 4);
    L->enc_off = take((B + 1) * 4);
    L->row_map = take((size_t)c->max_total_enc_frames * 4);
    L->frame_map = take((size_t)c->max_total_enc_frames * 4);  // request queue: where each new frame's K/V goes
    L->turn_buf = take(B * 4 * 4);                            // request queue: slot, old / new request, limit
    L->items = take((size_t)L->max_items * 16);
    L->v_seq_len = take(Ba * 4);
    L->v_finished = take(Ba * 4);
    L->v_cur_tok = take(Ba * 4);
    L->v_page_table = take(c->prefill_rows > 0 ? Ba * (size_t)L->max_pages * 4 : 0);
    L->v_items = take(c->prefill_rows > 0 ? (size_t)L->max_items * kMaxPrefillPositions * 16 : 0);
    const size_t ekv = c->kv_fp8 ? 1 : e;  // bytes per cached key / value element
    L->k_pool = take(L->pool_layer_elems * c->n_layers * ekv);
    L->v_pool = take(L->pool_layer_elems * c->n_layers * ekv);
    L->kc = take(L->cross_layer_elems * c->n_layers * ekv);
    L->vc = take(L->cross_layer_elems * c->n_layers * ekv);
    // every weight matrix once more, in MFMA fragment order
    L->w_frag = take(((size_t)c->n_layers * (8 * d * d + 2 * d * (size_t)c->d_ffn) + (size_t)c->vocab * d) * e);
    // merged products (bfloat16 mode): per layer Wcq.g . Wo and the vector Wcq.g . bo
    L->w_merge = take(c->dtype == 1 ? (size_t)c->n_layers * (d * d) * e : 0);
    L->merge_vec = take(c->dtype == 1 ? (size_t)c->n_layers * d * 4 : 0);
    // the batch's encoder states in fragment order (A operand of the cross K/V GEMMs), whole 256-row tiles
    L->enc_frag = take(align_up((size_t)c->max_total_enc_frames, 256) * d * e);
    L->total = off;
}

// The memory-side cache holds 256 MB; a decoder whose per-step weights stay well below that keeps them there from
// one step to the next (the keys and values are streamed around the caches), a larger one cannot.
constexpr double kCacheResidentWeightBytes = 192e6;
// Of a larger decoder, the first layers whose weights add up to this much are loaded the ordinary way and so stay
// cached from step to step; the rest is streamed with the non-temporal hint.  (24 layers of 29.4 MB: 7 or 8 resident
// layers are the optimum, 1.195 -> 1.160 ms per step; from 9 on the cache thrashes and the gain is gone.)
constexpr double kResidentLayerBytes = 220e6;

struct GraphKey {
    int batch = -1, n_items = 0, self_chunk = 0, self_nchunks = 0, prompt_len = 0, max_new = 0;
    long long total_enc = 0;
    bool operator==(const GraphKey& o) const {
        return batch == o.batch && n_items == o.n_items && total_enc == o.total_enc && self_chunk == o.self_chunk &&
               self_nchunks == o.self_nchunks && prompt_len == o.prompt_len && max_new == o.max_new;
    }
};

}  // namespace

struct aed_decoder {
    aed_config cfg;
    Dtype dt;
    size_t esz;
    size_t kv_esz;  // bytes per cached key / value element: esz, or 1 for E4M3 codes
    int w_nt = 0;   // the decode step's weights do not fit the memory-side cache: stream them with the non-temporal hint,
    int resident_layers = 0;  // except those of the first resident_layers layers
    Layout lay;
    std::vector<aed_layer_weights> layers;  // caller's pointers (biases, LayerNorm, embeddings are used in place)
    aed_weights w;
    struct FragWeights { const void *w_qkv, *w_o, *w_cq, *w_ckv, *w_co, *w_ff1, *w_ff2; };
    std::vector<FragWeights> fw;            // the matrices re-ordered into fragment order (workspace)
    struct LnFold { const float *qkv_c1, *qkv_c2, *cq_c1, *cq_c2, *ff1_c1, *ff1_c2; };
    std::vector<LnFold> fold;               // bfloat16 mode: W . g and W . b + bias of every LayerNorm product
    const float *out_c1 = nullptr, *out_c2 = nullptr;
    struct Merged { const void* w_p2; const float* cb_cq; };  // Wcq.g . Wo (fragment order), Wcq.g . bo
    std::vector<Merged> mw;
    int x_par = 0;                          // which statistics buffer describes the current residual rows
    const void* fw_out = nullptr;
    hipStream_t stream;
    char* ws;
    char* act;             // where the step's activations live: ws, or this device's static scratch array
    char* static_scratch = nullptr;  // this device's copy of the static scratch array
    // host-side state
    enum State { NO_BATCH, STEPPING, CONSUMED } state = NO_BATCH;
    int batch = 0;
    int host_pos = 0;     // positions fed so far (step API)
    int pages_used = 0;
    int n_items = 0;
    int self_chunk = 64, self_nchunks = 1, cross_chunk = 64;
    int last_prompt_len = 0, last_max_new = 0;
    long long total_enc = 0;
    const void* last_enc = nullptr;
    bool last_enc_padded = false;
    std::vector<int> enc_lens, enc_off, page_table;
    std::vector<int4> items_host;  // the cross-attention work list of the batch (a prefill pass repeats it per position)
    int* pin_poll = nullptr;  // pinned host memory for the finished-count poll
    hipEvent_t poll_event[2] = {nullptr, nullptr};
    hipEvent_t t0 = nullptr, t1 = nullptr;
    hipGraphExec_t gexec = nullptr;       // one greedy step (prompt feeding, EOS rules, output writes)
    GraphKey gkey;
    hipGraphExec_t step_gexec = nullptr;  // one aed_decode_step step (argmax only, ids into step_tok)
    GraphKey step_gkey;
    hipGraphExec_t pf_gexec = nullptr;    // one prompt-prefill pass
    GraphKey pf_gkey;
    std::string err;

    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
    template <typename T> T* act_at(size_t off) const { return reinterpret_cast<T*>(act + off); }
    StateArgs state_args(int prompt_len, int max_new) const {
        StateArgs st;
        st.seq_len = at<int>(lay.seq_len);
        st.n_gen = at<int>(lay.n_gen);
        st.finished = at<int>(lay.finished);
        st.cur_tok = at<int>(lay.cur_tok);
        st.limit = at<int>(lay.limit);
        st.n_finished = at<int>(lay.n_finished);
        st.prompt = prompt_len > 0 ? at<int>(lay.prompt_buf) : nullptr;
        st.out_tokens = at<int>(lay.out_buf);
        st.prompt_len = prompt_len;
        st.prompt_stride = prompt_len;
        st.out_stride = cfg.max_dec_len;
        st.max_new = max_new;
        st.eos_id = cfg.eos_id;
        st.pad_id = cfg.pad_id;
        st.batch = batch;
        st.vocab = cfg.vocab;
        return st;
    }
};

namespace {

aed_status fail(aed_decoder* d, aed_status st, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (d) d->err = buf; else g_create_error = buf;
    return st;
}

#define HIP_TRY(d, expr)                                                                          \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail(d, AED_EHIP, "%s: %s", #expr, hipGetErrorString(e_));  \
    } while (0)

// Keys per attention work item.  Whole sequences (one workgroup per sequence and
// head, no merge) whenever batch * heads gives the 256 CUs something to do:
// measured on MI355X, cutting the 24-layer batch-64 and the 4-layer batch-256
// workloads into 128-key chunks did not shorten the attention kernels (they are
// bound by the launch's total bytes at the achievable HBM rate plus fixed
// launch and first-access latency, not by the longest workgroup).  Only a batch
// too small to occupy the GPU (batch * heads < kMinItemsNoSplit) has its long
// sequences cut, aiming at kTargetItems items of at least 64 keys and at most
// kMaxChunks per sequence.
int pick_chunk(long long total_keys, int max_len, int batch, int n_heads) {
    const long long whole = std::max<long long>(64, ((long long)max_len + 63) / 64 * 64);
    if ((long long)batch * n_heads >= kMinItemsNoSplit) return (int)whole;
    long long c = (total_keys * n_heads + kTargetItems - 1) / kTargetItems;
    c = std::max(c, ((long long)max_len + kMaxChunks - 1) / kMaxChunks);
    c = std::max<long long>(64, (c + 63) / 64 * 64);
    return (int)std::min(c, whole);
}

// ---------------------------------------------------------------- kernel argument builders
// layer: whose weights the product reads (n_layers: the vocabulary matrix)
GemmArgs gemm_base(const aed_decoder* d, int layer) {
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.ln_eps = d->cfg.ln_eps;
    g.ln_scratch = d->act + d->lay.ln_h;
    g.M = d->batch;
    g.n_heads = d->cfg.n_heads;
    g.head_dim = d->cfg.head_dim;
    g.d_model = d->cfg.d_model;
    g.kv_fp8 = d->cfg.kv_fp8;
    g.rms = d->cfg.norm_type == 1;
    g.w_nt = d->w_nt && layer >= d->resident_layers;
    return g;
}

// bfloat16 mode: the LayerNorm products read the shadow of the residual rows and their statistics
bool folded_ln(const aed_decoder* d) { return d->dt == kBF16; }
float2* stats_buf(const aed_decoder* d, int par) {
    return reinterpret_cast<float2*>(d->act + d->lay.ln_stats) + (size_t)par * d->lay.stats_elems;
}
float* shift_buf(const aed_decoder* d, int par) {
    return d->act_at<float>(d->lay.mu_hat) + (size_t)par * (d->lay.stats_elems / (size_t)(d->cfg.d_model / 16));
}
char* shadow_buf(const aed_decoder* d, int par) { return d->act + d->lay.x_shadow + (size_t)par * d->lay.shadow_bytes; }
// Rows of version v (parity p = x_par): statistics in statistics buffer p, shadow in shadow buffer p.  The shift of a
// shadow is one value per row and layer: every shadow written inside layer l (by its three residual updates) is
// shifted by the mean the rows had when they entered the layer, which the layer's first product (QKV) leaves in
// shift buffer l & 1; the rows entering layer l carry the shift of layer l - 1 (buffer (l & 1) ^ 1; the embedding
// writes buffer 1 for layer 0).  first: this product is the one that reads the rows entering `layer` (QKV, or the
// vocabulary product with layer = n_layers).
void ln_consumer(const aed_decoder* d, GemmArgs& g, const float* c1, const float* c2, int layer, bool first) {
    g.A = shadow_buf(d, d->x_par);
    g.stats_in = stats_buf(d, d->x_par);
    g.mu_hat_in = shift_buf(d, first ? (layer & 1) ^ 1 : layer & 1);
    g.mu_hat_out = first && layer < d->cfg.n_layers ? shift_buf(d, layer & 1) : nullptr;
    g.ln_c1 = c1;
    g.ln_c2 = c2;
    g.stat_tiles = d->cfg.d_model / 16;
    g.m_stride = (int)(d->lay.stats_elems / (size_t)(d->cfg.d_model / 16));
}

// Small batches in bfloat16 mode: the cross-attention query product is split over the QKV launch and the launch of the
// self-attention output projection (kernels.h, "merged products"): one launch fewer per layer.
constexpr int kMergeMaxRows = 256;
bool merged_products(const aed_decoder* d) { return folded_ln(d) && d->batch <= kMergeMaxRows; }

hipError_t k_ln_qkv(aed_decoder* d, int l) {
    const aed_layer_weights& w = d->layers[l];
    GemmArgs g = gemm_base(d, l);
    g.A = d->act_at<float>(d->lay.x);
    g.W = d->fw[l].w_qkv; g.bias = w.b_qkv; g.ln_g = w.ln1_g; g.ln_b = w.ln1_b;
    g.N = 3 * d->cfg.d_model; g.K = d->cfg.d_model;
    g.out = d->act_at<float>(d->lay.q);
    g.k_pool = d->ws + d->lay.k_pool + (size_t)l * d->lay.pool_layer_elems * d->kv_esz;
    g.v_pool = d->ws + d->lay.v_pool + (size_t)l * d->lay.pool_layer_elems * d->kv_esz;
    g.page_table = d->at<int>(d->lay.page_table);
    g.max_pages = d->lay.max_pages;
    g.seq_len = d->at<int>(d->lay.seq_len);
    g.finished = d->at<int>(d->lay.finished);
    if (folded_ln(d)) {
        ln_consumer(d, g, d->fold[l].qkv_c1, d->fold[l].qkv_c2, l, true);
        if (merged_products(d)) {  // the stored matrix is [Wqkv.g1 ; Wcq.g2]: the last d columns are P1 of the merged products
            g.N = 4 * d->cfg.d_model;
            g.n_raw = 3 * d->cfg.d_model;
            g.out2 = d->act_at<float>(d->lay.q_aux);
            g.raw_bias = d->mw[l].cb_cq;
        }
        return launch_gemm(d->dt, PRO_LNS, EPI_QKV, g, d->stream);
    }
    return launch_gemm(d->dt, PRO_LN, EPI_QKV, g, d->stream);
}

AttnArgs attn_base(const aed_decoder* d) {
    AttnArgs a;
    memset(&a, 0, sizeof a);
    a.q = d->act_at<float>(d->lay.q);
    a.out = d->act + d->lay.attn_out;
    a.finished = d->at<int>(d->lay.finished);
    a.part = d->act_at<float>(d->lay.part);
    a.counters = d->act_at<int>(d->lay.counters);
    a.max_chunks = kMaxChunks;
    a.n_heads = d->cfg.n_heads;
    a.head_dim = d->cfg.head_dim;
    a.batch = d->batch;
    a.kv_fp8 = d->cfg.kv_fp8;
    a.scale_log2e = (float)(1.4426950408889634 / sqrt((double)d->cfg.head_dim));
    return a;
}

hipError_t k_self_attn(aed_decoder* d, int l) {
    AttnArgs a = attn_base(d);
    a.K = d->ws + d->lay.k_pool + (size_t)l * d->lay.pool_layer_elems * d->kv_esz;
    a.V = d->ws + d->lay.v_pool + (size_t)l * d->lay.pool_layer_elems * d->kv_esz;
    a.page_table = d->at<int>(d->lay.page_table);
    a.max_pages = d->lay.max_pages;
    a.seq_len = d->at<int>(d->lay.seq_len);
    a.chunk = d->self_chunk;
    a.n_chunks_max = d->self_nchunks;
    return launch_attn_self(d->dt, a, d->stream);
}

// x += A . W^T + bias
hipError_t k_resid(aed_decoder* d, int l, const void* A, const void* W, const void* bias, int K) {
    GemmArgs g = gemm_base(d, l);
    g.A = A; g.W = W; g.bias = bias;
    g.N = d->cfg.d_model; g.K = K;
    g.out = d->act_at<float>(d->lay.x);
    if (folded_ln(d)) {
        g.stats_out = stats_buf(d, d->x_par ^ 1);
        g.mu_hat_in = shift_buf(d, l & 1);  // the mean of the rows that entered the layer
        g.shadow_out = shadow_buf(d, d->x_par ^ 1);
        g.stat_tiles = d->cfg.d_model / 16;
        g.m_stride = (int)(d->lay.stats_elems / (size_t)(d->cfg.d_model / 16));
        d->x_par ^= 1;
        return launch_gemm(d->dt, PRO_T, EPI_RESID_S, g, d->stream);
    }
    return launch_gemm(d->dt, PRO_T, EPI_RESID, g, d->stream);
}

// x += Wo . o + bo and, in the same launch, P2 = (Wcq.g . Wo) . o -> q (finished by cross-attention)
hipError_t k_self_out_crossq(aed_decoder* d, int l) {
    const aed_layer_weights& w = d->layers[l];
    const int dm = d->cfg.d_model;
    GemmArgs a0 = gemm_base(d, l);
    a0.A = d->act + d->lay.attn_out; a0.W = d->fw[l].w_o; a0.bias = w.b_o;
    a0.N = dm; a0.K = dm;
    a0.out = d->act_at<float>(d->lay.x);
    a0.stats_out = stats_buf(d, d->x_par ^ 1);
    a0.mu_hat_in = shift_buf(d, l & 1);
    a0.shadow_out = shadow_buf(d, d->x_par ^ 1);
    a0.stat_tiles = dm / 16;
    a0.m_stride = (int)(d->lay.stats_elems / (size_t)(dm / 16));
    GemmArgs a1 = gemm_base(d, l);
    a1.A = d->act + d->lay.attn_out;
    a1.W = d->mw[l].w_p2;
    a1.N = dm; a1.K = dm;
    a1.out = d->act_at<float>(d->lay.q);
    a1.addend = d->act_at<float>(d->lay.q_aux);  // P1, left by the layer's QKV launch
    d->x_par ^= 1;
    return launch_gemm_pair(d->dt, a0, EPI_F32, a1, d->stream);
}

hipError_t k_ln_crossq(aed_decoder* d, int l) {
    const aed_layer_weights& w = d->layers[l];
    GemmArgs g = gemm_base(d, l);
    g.A = d->act_at<float>(d->lay.x);
    g.W = d->fw[l].w_cq; g.bias = w.b_cq; g.ln_g = w.ln2_g; g.ln_b = w.ln2_b;
    g.N = d->cfg.d_model; g.K = d->cfg.d_model;
    g.out = d->act_at<float>(d->lay.q);
    if (folded_ln(d)) {
        ln_consumer(d, g, d->fold[l].cq_c1, d->fold[l].cq_c2, l, false);
        return launch_gemm(d->dt, PRO_LNS, EPI_F32, g, d->stream);
    }
    return launch_gemm(d->dt, PRO_LN, EPI_F32, g, d->stream);
}

hipError_t k_cross_attn(aed_decoder* d, int l) {
    AttnArgs a = attn_base(d);
    a.K = d->ws + d->lay.kc + (size_t)l * d->lay.cross_layer_elems * d->kv_esz;
    a.V = d->ws + d->lay.vc + (size_t)l * d->lay.cross_layer_elems * d->kv_esz;
    a.items = d->at<int4>(d->lay.items);
    a.n_items = d->n_items;
    a.enc_off = d->at<int>(d->lay.enc_off);
    a.chunk = d->cross_chunk;
    a.t_cap = d->cfg.max_total_enc_frames;
    if (merged_products(d)) {  // q holds the merged product: the kernel finishes the normalisation
        a.q_stats = stats_buf(d, d->x_par);        // of the rows after the self-attention update
        a.q_mu_hat = shift_buf(d, (l & 1) ^ 1);    // shift of the shadow of the rows that entered the layer
        a.q_c1 = d->fold[l].cq_c1;
        a.q_c2 = d->fold[l].cq_c2;
        a.q_eps = d->cfg.ln_eps;
        a.q_stat_tiles = d->cfg.d_model / 16;
        a.q_m_stride = (int)(d->lay.stats_elems / (size_t)(d->cfg.d_model / 16));
        a.q_rms = d->cfg.norm_type == 1;
    }
    return launch_attn_cross(d->dt, a, d->stream);
}

hipError_t k_ln_ffn1(aed_decoder* d, int l) {
    const aed_layer_weights& w = d->layers[l];
    GemmArgs g = gemm_base(d, l);
    g.A = d->act_at<float>(d->lay.x);
    g.W = d->fw[l].w_ff1; g.bias = w.b_ff1; g.ln_g = w.ln3_g; g.ln_b = w.ln3_b;
    g.N = d->cfg.d_ffn; g.K = d->cfg.d_model;
    g.out = d->act + d->lay.ffn_h;
    if (folded_ln(d)) {
        ln_consumer(d, g, d->fold[l].ff1_c1, d->fold[l].ff1_c2, l, false);
        return launch_gemm(d->dt, PRO_LNS, EPI_RELU_T, g, d->stream);
    }
    return launch_gemm(d->dt, PRO_LN, EPI_RELU_T, g, d->stream);
}

hipError_t k_ln_vocab(aed_decoder* d) {
    GemmArgs g = gemm_base(d, d->cfg.n_layers);
    g.A = d->act_at<float>(d->lay.x);
    g.W = d->fw_out; g.bias = d->w.b_out; g.ln_g = d->w.lnf_g; g.ln_b = d->w.lnf_b;
    g.N = d->cfg.vocab; g.K = d->cfg.d_model;
    g.out = d->act_at<float>(d->lay.logits);
    if (folded_ln(d)) {
        ln_consumer(d, g, d->out_c1, d->out_c2, d->cfg.n_layers, true);
        return launch_gemm(d->dt, PRO_LNS, EPI_F32, g, d->stream);
    }
    return launch_gemm(d->dt, PRO_LN, EPI_F32, g, d->stream);
}

// K/V of rows [0, rows) of the fragment-ordered encoder frames; frame_map (may be null) names the frame slot of
// each row, else row m is frame m.
hipError_t k_cross_kv(aed_decoder* d, int l, long long rows, const int* frame_map) {
    const aed_layer_weights& w = d->layers[l];
    GemmArgs g = gemm_base(d, l);
    g.A = d->ws + d->lay.enc_frag;
    g.W = d->fw[l].w_ckv; g.bias = w.b_ckv;
    g.out_row_map = frame_map;
    g.a_rows = (int)align_up((size_t)d->cfg.max_total_enc_frames, 256);
    g.M = (int)rows; g.N = 2 * d->cfg.d_model; g.K = d->cfg.d_model;
    g.kc = d->ws + d->lay.kc + (size_t)l * d->lay.cross_layer_elems * d->kv_esz;
    g.vc = d->ws + d->lay.vc + (size_t)l * d->lay.cross_layer_elems * d->kv_esz;
    g.t_cap = d->cfg.max_total_enc_frames;
    return launch_gemm(d->dt, PRO_T, EPI_CROSSKV, g, d->stream);  // LDS-tiled kernel from 512 rows (bf16)
}

// launches of a kernel class per layer in the current mode
int class_launches(const aed_decoder* d, int cls) {
    if (merged_products(d) && cls == AED_K_LN_CROSSQ) return 0;  // part of AED_K_SELF_OUT's launch
    return 1;
}

hipError_t k_class(aed_decoder* d, int cls, int l) {
    const aed_layer_weights& w = d->layers[l];
    if (class_launches(d, cls) == 0) return hipSuccess;
    switch (cls) {
        case AED_K_LN_QKV: return k_ln_qkv(d, l);
        case AED_K_SELF_ATTN: return k_self_attn(d, l);
        case AED_K_SELF_OUT:
            if (merged_products(d)) return k_self_out_crossq(d, l);
            return k_resid(d, l, d->act + d->lay.attn_out, d->fw[l].w_o, w.b_o, d->cfg.d_model);
        case AED_K_LN_CROSSQ: return k_ln_crossq(d, l);
        case AED_K_CROSS_ATTN: return k_cross_attn(d, l);
        case AED_K_CROSS_OUT: return k_resid(d, l, d->act + d->lay.attn_out, d->fw[l].w_co, w.b_co, d->cfg.d_model);
        case AED_K_LN_FFN1: return k_ln_ffn1(d, l);
        case AED_K_FFN2:
            return k_resid(d, l, d->act + d->lay.ffn_h, d->fw[l].w_ff2, w.b_ff2, d->cfg.d_ffn);
        case AED_K_CROSS_KV: return k_cross_kv(d, l, d->total_enc, nullptr);
        default: return hipErrorInvalidValue;
    }
}

// One decoder step for the whole batch, enqueued on the stream.
hipError_t enqueue_step(aed_decoder* d, const StateArgs& st, int greedy, int* step_out) {
    hipError_t e;
    ShadowArgs sa;
    memset(&sa, 0, sizeof sa);
    if (folded_ln(d)) {
        d->x_par = 0;
        sa.shadow = shadow_buf(d, 0);
        sa.stats = stats_buf(d, 0);
        sa.mu_hat = shift_buf(d, 1);  // read as the shift of the rows entering layer 0
        sa.m_stride = (int)(d->lay.stats_elems / (size_t)(d->cfg.d_model / 16));
        sa.rms = d->cfg.norm_type == 1;
    }
    e = launch_embed(d->dt, d->act_at<float>(d->lay.x), d->w.tok_emb, d->w.pos_emb, st, d->cfg.d_model,
                     d->cfg.max_positions, d->cfg.emb_scale, sa, d->stream);
    if (e != hipSuccess) return e;
    for (int l = 0; l < d->cfg.n_layers; ++l)
        for (int cls = AED_K_LN_QKV; cls <= AED_K_FFN2; ++cls)
            if ((e = k_class(d, cls, l)) != hipSuccess) return e;
    if ((e = k_ln_vocab(d)) != hipSuccess) return e;
    return launch_sample(d->act_at<float>(d->lay.logits), st, greedy, step_out, d->stream);
}

aed_status check_weights(const aed_config* c, const aed_weights* w) {
    if (!w) return fail(nullptr, AED_EINVAL, "weights is NULL");
    const bool need_shift = c->norm_type == 0;  // RMSNorm: a missing shift vector is zero
    if (!w->tok_emb || !w->pos_emb || !w->lnf_g || (need_shift && !w->lnf_b) || !w->w_out || !w->layers)
        return fail(nullptr, AED_EINVAL, "a required top-level weight pointer is NULL");
    for (int l = 0; l < c->n_layers; ++l) {
        const aed_layer_weights& x = w->layers[l];
        if (!x.ln1_g || !x.w_qkv || !x.w_o || !x.ln2_g || !x.w_cq || !x.w_ckv || !x.w_co || !x.ln3_g || !x.w_ff1 ||
            !x.w_ff2 || (need_shift && (!x.ln1_b || !x.ln2_b || !x.ln3_b)))
            return fail(nullptr, AED_EINVAL, "layer %d: a required weight pointer is NULL", l);
    }
    return AED_OK;
}

aed_status start_batch(aed_decoder* d, const void* enc, bool padded, int t_max, const int32_t* enc_lens,
                       int32_t batch) {
    if (!d) return AED_EINVAL;
    if (!enc || !enc_lens) return fail(d, AED_EINVAL, "enc_states / enc_lens is NULL");
    if (batch < 1) return fail(d, AED_EINVAL, "batch must be >= 1");
    if (batch > d->cfg.max_batch) return fail(d, AED_ECAPACITY, "batch %d > max_batch %d", batch, d->cfg.max_batch);
    long long total = 0;
    int max_len = 0;
    for (int b = 0; b < batch; ++b) {
        if (enc_lens[b] < 1) return fail(d, AED_EINVAL, "enc_lens[%d] = %d (must be >= 1)", b, enc_lens[b]);
        if (enc_lens[b] > 65535) return fail(d, AED_EUNSUPPORTED, "enc_lens[%d] = %d: more than 65535 frames per sequence", b, enc_lens[b]);
        if (padded && enc_lens[b] > t_max) return fail(d, AED_EINVAL, "enc_lens[%d] = %d > t_max %d", b, enc_lens[b], t_max);
        total += enc_lens[b];
        max_len = std::max(max_len, enc_lens[b]);
    }
    if (total > d->cfg.max_total_enc_frames)
        return fail(d, AED_ECAPACITY, "sum(enc_lens) = %lld > max_total_enc_frames %d", total, d->cfg.max_total_enc_frames);

    // host tables: frame offsets, cross-attention work list, optional row map
    std::vector<int> off(batch + 1, 0);
    for (int b = 0; b < batch; ++b) off[b + 1] = off[b] + enc_lens[b];
    const int chunk = pick_chunk(total, max_len, batch, d->cfg.n_heads);
    std::vector<int4> items;
    for (int b = 0; b < batch; ++b) {
        const int nc = (enc_lens[b] + chunk - 1) / chunk;
        for (int c = 0; c < nc; ++c) {
            int4 it;
            it.x = b; it.y = (c * chunk) | (c << 16); it.z = std::min(chunk, enc_lens[b] - c * chunk) | (nc << 16);
            it.w = off[b];
            items.push_back(it);
        }
    }
    if ((int)items.size() > d->lay.max_items) return fail(d, AED_ECAPACITY, "cross-attention work list overflow");
    // longest first (stable: equal lengths stay in batch order, so the list is a function of the lengths alone)
    std::stable_sort(items.begin(), items.end(),
                     [](const int4& p, const int4& q) { return (p.z & 0xFFFF) > (q.z & 0xFFFF); });

    HIP_TRY(d, hipStreamSynchronize(d->stream));  // the previous batch's work is done with the old tables
    // the chunk merge's arrival counters return to zero by themselves after every launch; a batch still starts
    // from zero, whatever an earlier launch that ended abnormally may have left
    HIP_TRY(d, hipMemsetAsync(d->ws + d->lay.counters, 0, (size_t)d->lay.act_rows * d->cfg.n_heads * 4, d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.enc_off), off.data(), off.size() * 4, hipMemcpyHostToDevice, d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int4>(d->lay.items), items.data(), items.size() * 16, hipMemcpyHostToDevice, d->stream));
    if (padded) {
        std::vector<int> map((size_t)total);
        for (int b = 0; b < batch; ++b)
            for (int t = 0; t < enc_lens[b]; ++t) map[(size_t)off[b] + t] = b * t_max + t;
        HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.row_map), map.data(), map.size() * 4, hipMemcpyHostToDevice, d->stream));
    }
    d->batch = batch;
    d->n_items = (int)items.size();
    d->items_host = items;
    d->cross_chunk = chunk;
    d->total_enc = total;
    d->last_enc = enc;
    d->last_enc_padded = padded;
    d->enc_lens.assign(enc_lens, enc_lens + batch);
    d->enc_off = off;
    d->host_pos = 0;
    d->pages_used = 0;
    d->page_table.assign((size_t)batch * d->lay.max_pages, 0);
    d->self_chunk = pick_chunk((long long)batch * d->cfg.max_dec_len, d->cfg.max_dec_len, batch, d->cfg.n_heads);
    d->self_nchunks = (d->cfg.max_dec_len + d->self_chunk - 1) / d->self_chunk;
    d->state = aed_decoder::NO_BATCH;

    StateArgs st = d->state_args(0, 0);
    HIP_TRY(d, launch_reset(st, nullptr, 0, 0, d->stream));
    // encoder frames -> fragment order once (gathering the valid rows of a padded tensor), then one GEMM per layer
    HIP_TRY(d, launch_reorder_rows(d->dt, enc, padded ? d->at<int>(d->lay.row_map) : nullptr, d->ws + d->lay.enc_frag,
                                   (int)total, d->cfg.d_model, d->stream));
    for (int l = 0; l < d->cfg.n_layers; ++l) HIP_TRY(d, k_cross_kv(d, l, total, nullptr));
    HIP_TRY(d, hipStreamSynchronize(d->stream));  // host vectors above go out of scope
    d->state = aed_decoder::STEPPING;
    return AED_OK;
}

// Capture what enqueue launches into a launch graph; an existing graph of the same shape is kept.
template <typename F>
aed_status ensure_graph_of(aed_decoder* d, F enqueue, const GraphKey& key, hipGraphExec_t* exec, GraphKey* have) {
    if (*exec && key == *have) return AED_OK;
    if (*exec) { (void)hipGraphExecDestroy(*exec); *exec = nullptr; }
    hipGraph_t graph = nullptr;
    HIP_TRY(d, hipStreamBeginCapture(d->stream, hipStreamCaptureModeThreadLocal));
    hipError_t e = enqueue();
    hipError_t e2 = hipStreamEndCapture(d->stream, &graph);
    if (e != hipSuccess || e2 != hipSuccess) {
        if (graph) (void)hipGraphDestroy(graph);
        return fail(d, AED_EHIP, "graph capture: %s", hipGetErrorString(e != hipSuccess ? e : e2));
    }
    e = hipGraphInstantiate(exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) { *exec = nullptr; return fail(d, AED_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e)); }
    *have = key;
    return AED_OK;
}
// one step (greedy or plain)
aed_status ensure_graph(aed_decoder* d, const StateArgs& st, int greedy, int* step_out, const GraphKey& key,
                        hipGraphExec_t* exec, GraphKey* have) {
    return ensure_graph_of(d, [&]() { return enqueue_step(d, st, greedy, step_out); }, key, exec, have);
}

aed_status upload_page_table(aed_decoder* d) {
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.page_table), d->page_table.data(), d->page_table.size() * 4,
                              hipMemcpyHostToDevice, d->stream));
    return AED_OK;
}

// Prompt positions [p0, p1) of every sequence through the layers in one pass (greedy decoding only; see aed.h).
// Row r = (p - p0) * Bs + b (Bs = batch rounded up to 16, padding rows marked finished) is a sequence of its own
// for the kernels: position p, token prompt[b][p], sequence b's pages and encoder frames.  Only the self-attention
// keys and values matter afterwards, so the last layer stops after its QKV product.
aed_status prefill_pass(aed_decoder* d, const std::vector<int>& prompt_host, int prompt_len, int p0, int p1) {
    const int B = d->batch, Bs = (B + 15) / 16 * 16, np = p1 - p0, R = np * Bs, MP = d->lay.max_pages;
    std::vector<int> seq(R), fin(R), tok(R), pt((size_t)R * MP);
    std::vector<int4> items;
    items.reserve(d->items_host.size() * np);
    for (int q = 0; q < np; ++q) {
        for (int b = 0; b < Bs; ++b) {
            const int r = q * Bs + b;
            seq[r] = p0 + q;
            fin[r] = b >= B;
            tok[r] = b < B ? prompt_host[(size_t)b * prompt_len + p0 + q] : 0;
            for (int k = 0; k < MP; ++k) pt[(size_t)r * MP + k] = b < B ? d->page_table[(size_t)b * MP + k] : 0;
        }
    }
    for (const int4& it : d->items_host)  // longest first stays longest first
        for (int q = 0; q < np; ++q) {
            int4 v = it;
            v.x = q * Bs + it.x;
            items.push_back(v);
        }
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.v_seq_len), seq.data(), seq.size() * 4, hipMemcpyHostToDevice, d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.v_finished), fin.data(), fin.size() * 4, hipMemcpyHostToDevice, d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.v_cur_tok), tok.data(), tok.size() * 4, hipMemcpyHostToDevice, d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.v_page_table), pt.data(), pt.size() * 4, hipMemcpyHostToDevice, d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int4>(d->lay.v_items), items.data(), items.size() * 16, hipMemcpyHostToDevice, d->stream));
    // the kernels find their state through the layout: point it at the pass's rows for the duration
    const Layout saved = d->lay;
    const int saved_batch = d->batch, saved_items = d->n_items, saved_chunk = d->self_chunk, saved_nch = d->self_nchunks;
    d->lay.seq_len = saved.v_seq_len;
    d->lay.finished = saved.v_finished;
    d->lay.cur_tok = saved.v_cur_tok;
    d->lay.page_table = saved.v_page_table;
    d->lay.items = saved.v_items;
    d->batch = R;
    d->n_items = (int)items.size();
    d->self_chunk = std::max(64, (p1 + 63) / 64 * 64);  // a position sees at most p1 keys: one work item each
    d->self_nchunks = 1;
    const StateArgs st = d->state_args(0, 0);
    auto enqueue = [&]() -> hipError_t {
        ShadowArgs sa;
        memset(&sa, 0, sizeof sa);
        if (folded_ln(d)) {
            d->x_par = 0;
            sa.shadow = shadow_buf(d, 0);
                sa.stats = stats_buf(d, 0);
            sa.mu_hat = shift_buf(d, 1);
            sa.m_stride = (int)(d->lay.stats_elems / (size_t)(d->cfg.d_model / 16));
            sa.rms = d->cfg.norm_type == 1;
        }
        hipError_t e = launch_embed(d->dt, d->act_at<float>(d->lay.x), d->w.tok_emb, d->w.pos_emb, st, d->cfg.d_model,
                                    d->cfg.max_positions, d->cfg.emb_scale, sa, d->stream);
        for (int l = 0; l < d->cfg.n_layers && e == hipSuccess; ++l) {
            const int last_cls = l + 1 < d->cfg.n_layers ? AED_K_FFN2 : AED_K_LN_QKV;
            for (int cls = AED_K_LN_QKV; cls <= last_cls && e == hipSuccess; ++cls) e = k_class(d, cls, l);
        }
        return e;
    };
    // the pass's launches depend on its shape only (the tables above are read on the device): one graph per shape
    aed_status grc = AED_OK;
    hipError_t e = hipSuccess;
    if (d->stream != nullptr) {
        GraphKey key;
        key.batch = R; key.n_items = d->n_items; key.self_chunk = d->self_chunk; key.self_nchunks = 1;
        key.total_enc = d->total_enc;
        grc = ensure_graph_of(d, enqueue, key, &d->pf_gexec, &d->pf_gkey);
        if (grc == AED_OK) e = hipGraphLaunch(d->pf_gexec, d->stream);
    } else {
        e = enqueue();
    }
    d->lay = saved;
    d->batch = saved_batch;
    d->n_items = saved_items;
    d->self_chunk = saved_chunk;
    d->self_nchunks = saved_nch;
    if (grc != AED_OK) return grc;
    if (e != hipSuccess) return fail(d, AED_EHIP, "prompt prefill: %s", hipGetErrorString(e));
    HIP_TRY(d, hipStreamSynchronize(d->stream));  // the host tables above go out of scope
    return AED_OK;
}

}  // namespace

// ===================================================================== C ABI
extern "C" {

aed_status aed_workspace_bytes(const aed_config* cfg, size_t* bytes) {
    std::string err;
    aed_status st = check_config(cfg, err);
    if (st != AED_OK) { g_create_error = err; return st; }
    if (!bytes) return fail(nullptr, AED_EINVAL, "bytes is NULL");
    Layout L;
    make_layout(cfg, &L);
    *bytes = L.total;
    return AED_OK;
}

aed_status aed_decoder_create(const aed_config* cfg, const aed_weights* weights, void* workspace,
                              size_t workspace_bytes, void* hip_stream, aed_decoder** out) {
    std::string err;
    aed_status st = check_config(cfg, err);
    if (st != AED_OK) { g_create_error = err; return st; }
    if (!out) return fail(nullptr, AED_EINVAL, "out is NULL");
    *out = nullptr;
    if ((st = check_weights(cfg, weights)) != AED_OK) return st;
    Layout L;
    make_layout(cfg, &L);
    if (!workspace) return fail(nullptr, AED_EINVAL, "workspace is NULL");
    if ((uintptr_t)workspace % 256 != 0) return fail(nullptr, AED_EINVAL, "workspace must be 256-byte aligned");
    if (workspace_bytes < L.total)
        return fail(nullptr, AED_EINVAL, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);

    aed_decoder* d = new aed_decoder();
    d->cfg = *cfg;
    d->dt = cfg->dtype == 1 ? kBF16 : kF32;
    d->esz = cfg->dtype == 1 ? 2 : 4;
    d->kv_esz = cfg->kv_fp8 ? 1 : d->esz;
    {   // weights a decode step streams: 14 d^2 + ... per layer (all but the cross K/V matrices) and the vocabulary matrix
        const double dm = cfg->d_model, step_w = ((double)cfg->n_layers * (6 * dm * dm + 2 * dm * cfg->d_ffn) + dm * cfg->vocab) * d->esz;
        d->w_nt = step_w > kCacheResidentWeightBytes;
        const double layer_w = (6 * dm * dm + 2 * dm * cfg->d_ffn) * d->esz;
        d->resident_layers = d->w_nt ? std::min(cfg->n_layers, (int)(kResidentLayerBytes / layer_w)) : 0;
    }
    d->lay = L;
    d->layers.assign(weights->layers, weights->layers + cfg->n_layers);
    d->w = *weights;
    d->w.layers = d->layers.data();
    d->stream = static_cast<hipStream_t>(hip_stream);
    d->ws = static_cast<char*>(workspace);
    d->act = d->ws;
    auto cleanup = [&](hipError_t e, const char* what) {
        fail(nullptr, AED_EHIP, "%s: %s", what, hipGetErrorString(e));
        aed_decoder_destroy(d);
        return AED_EHIP;
    };
    hipError_t e;
    if ((e = scratch_of_current_device(&d->static_scratch)) != hipSuccess) return cleanup(e, "hipGetSymbolAddress(scratch)");
    // two poll words, then (from word 64) one finished flag per sequence for the request queue
    if ((e = hipHostMalloc(reinterpret_cast<void**>(&d->pin_poll), 256 + (size_t)cfg->max_batch * 4,
                           hipHostMallocDefault)) != hipSuccess)
        return cleanup(e, "hipHostMalloc");
    d->pin_poll[0] = d->pin_poll[1] = 0;
    for (int i = 0; i < 2; ++i)
        if ((e = hipEventCreateWithFlags(&d->poll_event[i], hipEventDisableTiming)) != hipSuccess)
            return cleanup(e, "hipEventCreate");
    if ((e = hipEventCreate(&d->t0)) != hipSuccess) return cleanup(e, "hipEventCreate");
    if ((e = hipEventCreate(&d->t1)) != hipSuccess) return cleanup(e, "hipEventCreate");

    // arrival counters of the chunk merge start at zero and return to zero after every launch
    if ((e = hipMemsetAsync(d->ws + L.counters, 0, (size_t)L.act_rows * cfg->n_heads * 4, d->stream)) != hipSuccess)
        return cleanup(e, "hipMemsetAsync");
    // re-order every weight matrix into fragment order, once
    {
        char* p = d->ws + L.w_frag;
        const int dm = cfg->d_model, F = cfg->d_ffn;
        // bfloat16 mode: a matrix that follows a LayerNorm is stored with that LayerNorm's gain multiplied into its
        // columns (the folded LayerNorm, kernels.h); float32 mode applies the gain to the rows instead
        auto put = [&](const void* src, int N, int K, const void* gain = nullptr) -> const void* {
            void* dst = p;
            if (e == hipSuccess) e = launch_reorder_weight(d->dt, src, folded_ln(d) ? gain : nullptr, dst, N, K, d->stream);
            p += (size_t)N * K * d->esz;
            return dst;
        };
        e = hipSuccess;
        d->fw.resize(cfg->n_layers);
        for (int l = 0; l < cfg->n_layers; ++l) {
            const aed_layer_weights& x = d->layers[l];
            aed_decoder::FragWeights& f = d->fw[l];
            f.w_qkv = put(x.w_qkv, 3 * dm, dm, x.ln1_g);
            f.w_cq = put(x.w_cq, dm, dm, x.ln2_g);  // directly behind w_qkv: together the [4 d, d] matrix of the merged QKV launch
            f.w_o = put(x.w_o, dm, dm);
            f.w_ckv = put(x.w_ckv, 2 * dm, dm);
            f.w_co = put(x.w_co, dm, dm);
            f.w_ff1 = put(x.w_ff1, F, dm, x.ln3_g);
            f.w_ff2 = put(x.w_ff2, dm, F);
        }
        d->fw_out = put(d->w.w_out, cfg->vocab, dm, d->w.lnf_g);
        if (e != hipSuccess) return cleanup(e, "weight re-ordering");
    }
    if (folded_ln(d)) {  // W . g and W . b + bias of every product that follows a LayerNorm
        float* p = reinterpret_cast<float*>(d->ws + L.ln_fold);
        const int dm = cfg->d_model, F = cfg->d_ffn;
        e = hipSuccess;
        auto fold = [&](const void* Wm, const void* gv, const void* bv, const void* bias, int N, const float** c1,
                        const float** c2) {
            *c1 = p; *c2 = p + N;
            if (e == hipSuccess) e = launch_fold_ln(d->dt, Wm, gv, bv, bias, p, p + N, N, dm, d->stream);
            p += 2 * (size_t)N;
        };
        d->fold.resize(cfg->n_layers);
        for (int l = 0; l < cfg->n_layers; ++l) {
            const aed_layer_weights& x = d->layers[l];
            aed_decoder::LnFold& f = d->fold[l];
            fold(x.w_qkv, x.ln1_g, x.ln1_b, x.b_qkv, 3 * dm, &f.qkv_c1, &f.qkv_c2);
            fold(x.w_cq, x.ln2_g, x.ln2_b, x.b_cq, dm, &f.cq_c1, &f.cq_c2);
            fold(x.w_ff1, x.ln3_g, x.ln3_b, x.b_ff1, F, &f.ff1_c1, &f.ff1_c2);
        }
        fold(d->w.w_out, d->w.lnf_g, d->w.lnf_b, d->w.b_out, cfg->vocab, &d->out_c1, &d->out_c2);
        if (e != hipSuccess) return cleanup(e, "folding LayerNorm gain and shift into the products");
    }
    if (folded_ln(d)) {  // merged products: Wcq.g . Wo and Wcq.g . bo per layer
        const int dm = cfg->d_model;
        char* p = d->ws + L.w_merge;
        float* v = reinterpret_cast<float*>(d->ws + L.merge_vec);
        e = hipSuccess;
        d->mw.resize(cfg->n_layers);
        for (int l = 0; l < cfg->n_layers && e == hipSuccess; ++l) {
            const aed_layer_weights& x = d->layers[l];
            e = launch_weight_product(d->dt, x.w_cq, x.ln2_g, x.w_o, p, dm, dm, dm, 0, dm, d->stream);
            if (e == hipSuccess) e = launch_fold_vec(d->dt, x.w_cq, x.ln2_g, x.b_o, v, dm, dm, d->stream);
            d->mw[l].w_p2 = p;
            d->mw[l].cb_cq = v;
            p += (size_t)dm * dm * d->esz;
            v += dm;
        }
        if (e != hipSuccess) return cleanup(e, "forming the merged products' matrices");
    }
    if ((e = hipStreamSynchronize(d->stream)) != hipSuccess) return cleanup(e, "hipStreamSynchronize");
    *out = d;
    return AED_OK;
}

aed_status aed_decoder_destroy(aed_decoder* d) {
    if (!d) return AED_OK;
    (void)hipStreamSynchronize(d->stream);
    if (d->gexec) (void)hipGraphExecDestroy(d->gexec);
    if (d->step_gexec) (void)hipGraphExecDestroy(d->step_gexec);
    if (d->pf_gexec) (void)hipGraphExecDestroy(d->pf_gexec);
    for (int i = 0; i < 2; ++i)
        if (d->poll_event[i]) (void)hipEventDestroy(d->poll_event[i]);
    if (d->t0) (void)hipEventDestroy(d->t0);
    if (d->t1) (void)hipEventDestroy(d->t1);
    if (d->pin_poll) (void)hipHostFree(d->pin_poll);
    delete d;
    return AED_OK;
}

aed_status aed_cross_kv_precompute(aed_decoder* d, const void* enc_states, const int32_t* enc_lens, int32_t batch) {
    return start_batch(d, enc_states, false, 0, enc_lens, batch);
}

aed_status aed_cross_kv_precompute_padded(aed_decoder* d, const void* enc_padded, int32_t t_max,
                                          const int32_t* enc_lens, int32_t batch) {
    if (d && t_max < 1) return fail(d, AED_EINVAL, "t_max must be >= 1");
    return start_batch(d, enc_padded, true, t_max, enc_lens, batch);
}

aed_status aed_decode_step(aed_decoder* d, const int32_t* tokens_in, int32_t* tokens_out, float* logits_out) {
    if (!d) return AED_EINVAL;
    if (d->state != aed_decoder::STEPPING)
        return fail(d, AED_ESTATE, "aed_decode_step needs a batch started by aed_cross_kv_precompute");
    if (!tokens_in) return fail(d, AED_EINVAL, "tokens_in is NULL");
    if (d->host_pos >= d->cfg.max_dec_len || d->host_pos >= d->cfg.max_positions)
        return fail(d, AED_ECAPACITY, "position %d exceeds max_dec_len %d / max_positions %d", d->host_pos,
                    d->cfg.max_dec_len, d->cfg.max_positions);
    d->act = d->ws;
    if (d->host_pos % kPage == 0) {  // every sequence enters a new page
        if (d->pages_used + d->batch > d->lay.n_pages)
            return fail(d, AED_ECAPACITY, "self-attention page pool exhausted (%d pages)", d->lay.n_pages);
        const int blk = d->host_pos / kPage;
        for (int b = 0; b < d->batch; ++b) d->page_table[(size_t)b * d->lay.max_pages + blk] = d->pages_used++;
        aed_status st = upload_page_table(d);
        if (st != AED_OK) return st;
    }
    StateArgs st = d->state_args(0, 0);
    HIP_TRY(d, launch_set_tokens(st.cur_tok, tokens_in, 1, d->batch, d->stream));
    if (d->stream != nullptr) {
        // the step itself is a replayed graph working on the library's own buffers; the caller's
        // pointers only appear in the small copies around it
        GraphKey key;
        key.batch = d->batch; key.n_items = d->n_items; key.self_chunk = d->self_chunk;
        key.self_nchunks = d->self_nchunks; key.total_enc = d->total_enc;
        aed_status grc = ensure_graph(d, st, 0, d->at<int>(d->lay.step_tok), key, &d->step_gexec, &d->step_gkey);
        if (grc != AED_OK) return grc;
        HIP_TRY(d, hipGraphLaunch(d->step_gexec, d->stream));
        if (tokens_out)
            HIP_TRY(d, hipMemcpyAsync(tokens_out, d->at<int>(d->lay.step_tok), (size_t)d->batch * 4,
                                      hipMemcpyDeviceToDevice, d->stream));
    } else {
        HIP_TRY(d, enqueue_step(d, st, 0, tokens_out));
    }
    if (logits_out)
        HIP_TRY(d, hipMemcpyAsync(logits_out, d->act_at<float>(d->lay.logits), (size_t)d->batch * d->cfg.vocab * 4,
                                  hipMemcpyDeviceToDevice, d->stream));
    d->host_pos += 1;
    return AED_OK;
}

aed_status aed_decode_step_noalloc(aed_decoder* d, const int32_t* tokens_in, int32_t* tokens_out, float* logits_out) {
    if (!d) return AED_EINVAL;
    if (d->state != aed_decoder::STEPPING)
        return fail(d, AED_ESTATE, "aed_decode_step_noalloc needs a batch started by aed_cross_kv_precompute");
    if (!tokens_in) return fail(d, AED_EINVAL, "tokens_in is NULL");
    if (d->lay.act_bytes > kStaticScratchBytes)
        return fail(d, AED_ECAPACITY,
                    "this decoder's step activations take %zu bytes (max_batch %d, d_model %d, d_ffn %d, vocab %d); "
                    "the static scratch array holds %zu",
                    d->lay.act_bytes, d->cfg.max_batch, d->cfg.d_model, d->cfg.d_ffn, d->cfg.vocab, kStaticScratchBytes);
    if (d->host_pos >= d->cfg.max_dec_len || d->host_pos >= d->cfg.max_positions)
        return fail(d, AED_ECAPACITY, "position %d exceeds max_dec_len %d / max_positions %d", d->host_pos,
                    d->cfg.max_dec_len, d->cfg.max_positions);
    if (d->host_pos % kPage == 0) {  // every sequence enters a new page: the table entries are written by a kernel
        if (d->pages_used + d->batch > d->lay.n_pages)
            return fail(d, AED_ECAPACITY, "self-attention page pool exhausted (%d pages)", d->lay.n_pages);
        const int blk = d->host_pos / kPage;
        HIP_TRY(d, launch_assign_pages(d->at<int>(d->lay.page_table), d->lay.max_pages, blk, d->pages_used, d->batch,
                                       d->stream));
        for (int b = 0; b < d->batch; ++b) d->page_table[(size_t)b * d->lay.max_pages + blk] = d->pages_used++;
    }
    d->act = d->static_scratch;
    // the array keeps what the last call on this GPU left: the merge's arrival counters must start at zero, all
    // other buffers are written by this step before they are read
    HIP_TRY(d, launch_fill_zero(d->act_at<int>(d->lay.counters), d->lay.act_rows * d->cfg.n_heads, d->stream));
    StateArgs st = d->state_args(0, 0);
    HIP_TRY(d, launch_set_tokens(st.cur_tok, tokens_in, 1, d->batch, d->stream));
    HIP_TRY(d, enqueue_step(d, st, 0, tokens_out));
    if (logits_out)
        HIP_TRY(d, hipMemcpyAsync(logits_out, d->act_at<float>(d->lay.logits), (size_t)d->batch * d->cfg.vocab * 4,
                                  hipMemcpyDeviceToDevice, d->stream));
    d->host_pos += 1;
    return AED_OK;
}

aed_status aed_greedy_decode(aed_decoder* d, const int32_t* prompt, int32_t prompt_len, int32_t max_new,
                             const int32_t* max_new_per_seq, int32_t* out_tokens, int32_t* out_lens) {
    if (!d) return AED_EINVAL;
    if (d->state == aed_decoder::NO_BATCH)
        return fail(d, AED_ESTATE, "aed_greedy_decode needs a batch started by aed_cross_kv_precompute");
    if (!prompt || !out_tokens || !out_lens) return fail(d, AED_EINVAL, "prompt / out_tokens / out_lens is NULL");
    if (prompt_len < 1 || max_new < 1) return fail(d, AED_EINVAL, "prompt_len and max_new must be >= 1");
    d->act = d->ws;
    if (max_new_per_seq) {
        if (d->cfg.eos_id < 0) return fail(d, AED_EINVAL, "max_new_per_seq needs eos_id >= 0");
        for (int b = 0; b < d->batch; ++b)
            if (max_new_per_seq[b] < 1) return fail(d, AED_EINVAL, "max_new_per_seq[%d] < 1", b);
    }
    const int total_len = prompt_len + max_new;
    if (total_len > d->cfg.max_dec_len || total_len > d->cfg.max_positions)
        return fail(d, AED_ECAPACITY, "prompt_len + max_new = %d exceeds max_dec_len %d / max_positions %d", total_len,
                    d->cfg.max_dec_len, d->cfg.max_positions);
    // pages: block-major, only the blocks a sequence can reach
    const int B = d->batch, MP = d->lay.max_pages;
    std::vector<int> need(B);
    int max_need = 0;
    long long pages = 0;
    for (int b = 0; b < B; ++b) {
        const int n = max_new_per_seq ? std::min(max_new, max_new_per_seq[b]) : max_new;
        need[b] = (prompt_len + n + kPage - 1) / kPage;
        max_need = std::max(max_need, need[b]);
        pages += need[b];
    }
    if (pages > d->lay.n_pages)
        return fail(d, AED_ECAPACITY, "self-attention page pool too small: %lld pages needed, %d available", pages,
                    d->lay.n_pages);
    std::fill(d->page_table.begin(), d->page_table.end(), 0);
    int next = 0;
    for (int blk = 0; blk < max_need; ++blk)
        for (int b = 0; b < B; ++b)
            if (blk < need[b]) d->page_table[(size_t)b * MP + blk] = next++;
    d->pages_used = next;
    aed_status rc = upload_page_table(d);
    if (rc != AED_OK) return rc;
    if (max_new_per_seq)
        HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.limits_in), max_new_per_seq, (size_t)B * 4, hipMemcpyHostToDevice,
                                  d->stream));
    HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.prompt_buf), prompt, (size_t)B * prompt_len * 4,
                              hipMemcpyDeviceToDevice, d->stream));
    d->self_chunk = pick_chunk((long long)B * total_len, total_len, B, d->cfg.n_heads);
    d->self_nchunks = (total_len + d->self_chunk - 1) / d->self_chunk;
    d->last_prompt_len = prompt_len;
    d->last_max_new = max_new;
    StateArgs st = d->state_args(prompt_len, max_new);
    // Prompt positions 0 .. prompt_len-2 emit nothing: with room for it they go through the layers several at a
    // time; the step loop then starts at the last prompt position.
    int start_pos = 0;
    {
        const int Bs = (B + 15) / 16 * 16;
        const int per_pass = std::min(kMaxPrefillPositions, d->cfg.prefill_rows / Bs);
        if (per_pass >= 1 && prompt_len >= 2) {
            std::vector<int> prompt_host((size_t)B * prompt_len);
            HIP_TRY(d, hipMemcpyAsync(prompt_host.data(), prompt, prompt_host.size() * 4, hipMemcpyDeviceToHost, d->stream));
            HIP_TRY(d, hipStreamSynchronize(d->stream));
            while (start_pos < prompt_len - 1) {
                const int p1 = std::min(prompt_len - 1, start_pos + per_pass);
                if ((rc = prefill_pass(d, prompt_host, prompt_len, start_pos, p1)) != AED_OK) return rc;
                start_pos = p1;
            }
        }
    }
    HIP_TRY(d, launch_reset(st, max_new_per_seq ? d->at<int>(d->lay.limits_in) : nullptr, 1, start_pos, d->stream));
    d->state = aed_decoder::CONSUMED;

    // one launch graph per shape; replayed for every step
    const bool use_graph = d->stream != nullptr;
    if (use_graph) {
        GraphKey key;
        key.batch = B; key.n_items = d->n_items; key.self_chunk = d->self_chunk; key.self_nchunks = d->self_nchunks;
        key.prompt_len = prompt_len; key.max_new = max_new; key.total_enc = d->total_enc;
        aed_status grc = ensure_graph(d, st, 1, nullptr, key, &d->gexec, &d->gkey);
        if (grc != AED_OK) return grc;
    }
    // Early stop: every poll_every steps the finished count is copied to pinned
    // memory; completed polls are read without blocking, and the host runs at
    // most two polls ahead of the device.
    const int n_steps = prompt_len - 1 - start_pos + max_new;
    const bool can_stop_early = d->cfg.eos_id >= 0;
    const int poll_every = 8;
    int issued = 0, seen = 0;
    bool done = false;
    for (int s = 0; s < n_steps && !done; ++s) {
        if (use_graph) HIP_TRY(d, hipGraphLaunch(d->gexec, d->stream));
        else HIP_TRY(d, enqueue_step(d, st, 1, nullptr));
        if (!can_stop_early) continue;
        while (seen < issued && hipEventQuery(d->poll_event[seen & 1]) == hipSuccess) {
            done = done || d->pin_poll[seen & 1] >= B;
            ++seen;
        }
        if (done || (s + 1) % poll_every != 0) continue;
        if (issued - seen >= 2) {
            HIP_TRY(d, hipEventSynchronize(d->poll_event[seen & 1]));
            done = d->pin_poll[seen & 1] >= B;
            ++seen;
            if (done) break;
        }
        HIP_TRY(d, hipMemcpyAsync(&d->pin_poll[issued & 1], st.n_finished, 4, hipMemcpyDeviceToHost, d->stream));
        HIP_TRY(d, hipEventRecord(d->poll_event[issued & 1], d->stream));
        ++issued;
    }
    (void)hipGetLastError();  // hipEventQuery's "not ready" is not an error
    HIP_TRY(d, launch_copy_out(st, out_tokens, out_lens, d->stream));
    HIP_TRY(d, hipStreamSynchronize(d->stream));
    return AED_OK;
}

}  // extern "C"

// ------------------------------------------------------------------ request queue (slot refill)
extern "C" aed_status aed_greedy_decode_queue(aed_decoder* d, const void* enc_states, const int32_t* enc_lens,
                                              int32_t n_requests, const int32_t* prompts, int32_t prompt_len,
                                              int32_t max_new, const int32_t* max_new_per_req, int32_t* out_tokens,
                                              int32_t* out_lens, int32_t* steps_run) {
    if (!d) return AED_EINVAL;
    if (!enc_states || !enc_lens || !prompts || !out_tokens || !out_lens)
        return fail(d, AED_EINVAL, "enc_states / enc_lens / prompts / out_tokens / out_lens is NULL");
    if (n_requests < 1) return fail(d, AED_EINVAL, "n_requests must be >= 1");
    if (prompt_len < 1 || max_new < 1) return fail(d, AED_EINVAL, "prompt_len and max_new must be >= 1");
    if (d->cfg.eos_id < 0) return fail(d, AED_EINVAL, "the request queue needs eos_id >= 0");
    d->act = d->ws;
    const int total_len = prompt_len + max_new;
    if (total_len > d->cfg.max_dec_len || total_len > d->cfg.max_positions)
        return fail(d, AED_ECAPACITY, "prompt_len + max_new = %d exceeds max_dec_len %d / max_positions %d", total_len,
                    d->cfg.max_dec_len, d->cfg.max_positions);
    const int B = std::min(d->cfg.max_batch, n_requests), MP = d->lay.max_pages;
    const int need_pages = (total_len + kPage - 1) / kPage;
    if ((long long)B * need_pages > d->lay.n_pages)
        return fail(d, AED_ECAPACITY, "self-attention page pool too small: %lld pages needed, %d available",
                    (long long)B * need_pages, d->lay.n_pages);
    std::vector<long long> src_off((size_t)n_requests + 1, 0);
    int max_len = 0;
    for (int r = 0; r < n_requests; ++r) {
        if (enc_lens[r] < 1) return fail(d, AED_EINVAL, "enc_lens[%d] = %d (must be >= 1)", r, enc_lens[r]);
        if (enc_lens[r] > 65535)
            return fail(d, AED_EUNSUPPORTED, "enc_lens[%d] = %d: more than 65535 frames per sequence", r, enc_lens[r]);
        if (enc_lens[r] > d->cfg.max_total_enc_frames)
            return fail(d, AED_ECAPACITY, "enc_lens[%d] = %d > max_total_enc_frames %d", r, enc_lens[r],
                        d->cfg.max_total_enc_frames);
        if (max_new_per_req && max_new_per_req[r] < 1) return fail(d, AED_EINVAL, "max_new_per_req[%d] < 1", r);
        src_off[r + 1] = src_off[r] + enc_lens[r];
        max_len = std::max(max_len, enc_lens[r]);
    }
    if (src_off[n_requests] > INT_MAX) return fail(d, AED_EUNSUPPORTED, "more than 2^31 - 1 encoder frames in the queue");

    // Slot b owns pages [b * need_pages, (b + 1) * need_pages) for the whole run: a refilled slot starts again at
    // position 0 and overwrites them.  Frames of the cross K/V cache are handed out per request.
    HIP_TRY(d, hipStreamSynchronize(d->stream));
    HIP_TRY(d, hipMemsetAsync(d->ws + d->lay.counters, 0, (size_t)d->lay.act_rows * d->cfg.n_heads * 4, d->stream));
    d->state = aed_decoder::NO_BATCH;  // the per-batch inspection calls do not apply to a queue run
    d->batch = B;
    d->n_items = B;  // one work item per slot (whole sequences), so that the captured launch shape never changes
    d->cross_chunk = std::max(64, (max_len + 63) / 64 * 64);
    d->total_enc = -1;
    d->page_table.assign((size_t)B * MP, 0);
    for (int b = 0; b < B; ++b)
        for (int k = 0; k < need_pages; ++k) d->page_table[(size_t)b * MP + k] = b * need_pages + k;
    d->pages_used = B * need_pages;
    aed_status rc = upload_page_table(d);
    if (rc != AED_OK) return rc;
    d->self_chunk = pick_chunk((long long)B * total_len, total_len, B, d->cfg.n_heads);
    d->self_nchunks = (total_len + d->self_chunk - 1) / d->self_chunk;
    const StateArgs st = d->state_args(prompt_len, max_new);
    const bool use_graph = d->stream != nullptr;
    if (use_graph) {
        GraphKey key;
        key.batch = B; key.n_items = B; key.self_chunk = d->self_chunk; key.self_nchunks = d->self_nchunks;
        key.prompt_len = prompt_len; key.max_new = max_new; key.total_enc = -1;
        if ((rc = ensure_graph(d, st, 1, nullptr, key, &d->gexec, &d->gkey)) != AED_OK) return rc;
    }

    FrameSpace frames(d->cfg.max_total_enc_frames);
    std::vector<int> slot_req(B, -1), slot_at(B, 0);  // request in the slot (-1: none), its first frame
    std::vector<int> done_req(B, -1);                 // finished request whose tokens are still in the slot
    int next_req = 0, active = 0, n_steps = 0;
    bool first = true;
    int* turn = d->at<int>(d->lay.turn_buf);
    int* flags = d->pin_poll + 64;
    const int poll_every = 8;
    std::vector<int> h_turn, h_src, h_dst;
    std::vector<int4> items(B);

    for (;;) {
        // ---- turn slots over: hand finished requests out, start queued ones where frames are free (queue order)
        h_turn.assign((size_t)4 * B, -1);
        h_src.clear();
        h_dst.clear();
        int n_turn = 0;
        bool queue_blocked = false;
        for (int b = 0; b < B; ++b) {
            if (slot_req[b] >= 0) continue;
            int req = -1;
            if (next_req < n_requests && !queue_blocked) {
                const int at = frames.take(enc_lens[next_req]);
                if (at < 0) queue_blocked = true;  // wait for a running request to release its frames
                else {
                    req = next_req++;
                    slot_req[b] = req;
                    slot_at[b] = at;
                    ++active;
                    for (int t = 0; t < enc_lens[req]; ++t) {
                        h_src.push_back((int)(src_off[req] + t));
                        h_dst.push_back(at + t);
                    }
                }
            }
            if (req < 0 && done_req[b] < 0 && !first) continue;  // a parked slot stays as it is
            h_turn[n_turn] = b;
            h_turn[B + n_turn] = done_req[b];
            h_turn[2 * B + n_turn] = req;
            h_turn[3 * B + n_turn] = req >= 0 && max_new_per_req ? max_new_per_req[req] : INT_MAX;  // no forced end
            done_req[b] = -1;
            ++n_turn;
        }
        first = false;
        if (n_turn > 0) {
            for (int b = 0; b < B; ++b) {  // a parked slot keeps a valid one-frame item; its workgroups exit early
                const bool on = slot_req[b] >= 0;
                items[b].x = b; items[b].y = 0; items[b].z = (on ? enc_lens[slot_req[b]] : 1) | (1 << 16);
                items[b].w = on ? slot_at[b] : 0;
            }
            std::vector<int4> sorted(items);
            std::stable_sort(sorted.begin(), sorted.end(),
                             [](const int4& p, const int4& q) { return (p.z & 0xFFFF) > (q.z & 0xFFFF); });
            HIP_TRY(d, hipMemcpyAsync(turn, h_turn.data(), h_turn.size() * 4, hipMemcpyHostToDevice, d->stream));
            HIP_TRY(d, hipMemcpyAsync(d->at<int4>(d->lay.items), sorted.data(), sorted.size() * 16, hipMemcpyHostToDevice,
                                      d->stream));
            HIP_TRY(d, launch_turn_over_slots(st, turn, turn + B, turn + 2 * B, turn + 3 * B, n_turn, prompts, out_tokens,
                                              out_lens, d->stream));
            if (!h_src.empty()) {
                const long long rows = (long long)h_src.size();
                HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.row_map), h_src.data(), h_src.size() * 4, hipMemcpyHostToDevice,
                                          d->stream));
                HIP_TRY(d, hipMemcpyAsync(d->at<int>(d->lay.frame_map), h_dst.data(), h_dst.size() * 4,
                                          hipMemcpyHostToDevice, d->stream));
                HIP_TRY(d, launch_reorder_rows(d->dt, enc_states, d->at<int>(d->lay.row_map), d->ws + d->lay.enc_frag,
                                               (int)rows, d->cfg.d_model, d->stream));
                for (int l = 0; l < d->cfg.n_layers; ++l)
                    HIP_TRY(d, k_cross_kv(d, l, rows, d->at<int>(d->lay.frame_map)));
            }
            HIP_TRY(d, hipStreamSynchronize(d->stream));  // the host vectors are re-used
        }
        if (active == 0) break;  // nothing running, and then nothing queued either (a free axis fits any request)

        // ---- run steps until a slot finishes; the flags are looked at every poll_every steps
        bool any = false;
        while (!any) {
            for (int s = 0; s < poll_every; ++s) {
                if (use_graph) HIP_TRY(d, hipGraphLaunch(d->gexec, d->stream));
                else HIP_TRY(d, enqueue_step(d, st, 1, nullptr));
            }
            n_steps += poll_every;
            HIP_TRY(d, hipMemcpyAsync(flags, st.finished, (size_t)B * 4, hipMemcpyDeviceToHost, d->stream));
            HIP_TRY(d, hipStreamSynchronize(d->stream));
            for (int b = 0; b < B; ++b)
                if (slot_req[b] >= 0 && flags[b]) {
                    frames.give(slot_at[b], enc_lens[slot_req[b]]);
                    done_req[b] = slot_req[b];
                    slot_req[b] = -1;
                    --active;
                    any = true;
                }
        }
    }
    if (steps_run) *steps_run = n_steps;
    return AED_OK;
}

extern "C" {

const char* aed_last_error(const aed_decoder* d) { return d ? d->err.c_str() : g_create_error.c_str(); }

int64_t aed_layer_matrix_params(const aed_config* c) {
    if (!c) return 0;
    const int64_t d = c->d_model, F = c->d_ffn;
    return ((3 * d * d + d * d) + (d * d + 2 * d * d + d * d) + 2 * d * F) * c->n_layers;
}

}  // extern "C"

// ---------------------------------------------------------------- inspection / measurement
namespace {
// Value of an E4M3 code (OCP 8-bit floating point: 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no
// infinities, S.1111.111 is NaN).
float e4m3_value(uint8_t c) {
    const int ef = (c >> 3) & 15, m = c & 7;
    float v;
    if (ef == 15 && m == 7) v = NAN;
    else if (ef == 0) v = ldexpf((float)m, -9);
    else v = ldexpf((float)(8 + m), ef - 10);
    return (c & 0x80) ? -v : v;
}
// esz: bytes per element (4: float, 2: bfloat16, 1: E4M3 code)
void to_f32_host(const void* src, size_t n, size_t esz, float* dst) {
    if (esz == 4) { memcpy(dst, src, n * 4); return; }
    if (esz == 1) {
        const uint8_t* p = static_cast<const uint8_t*>(src);
        for (size_t i = 0; i < n; ++i) dst[i] = e4m3_value(p[i]);
        return;
    }
    const uint16_t* p = static_cast<const uint16_t*>(src);
    for (size_t i = 0; i < n; ++i) {
        uint32_t u = (uint32_t)p[i] << 16;
        memcpy(dst + i, &u, 4);
    }
}
}  // namespace

extern "C" {

aed_status aed_read_cross_kv(aed_decoder* d, int32_t layer, int32_t seq, float* k_out, float* v_out) {
    if (!d) return AED_EINVAL;
    if (d->state == aed_decoder::NO_BATCH) return fail(d, AED_ESTATE, "no batch");
    if (layer < 0 || layer >= d->cfg.n_layers || seq < 0 || seq >= d->batch || !k_out || !v_out)
        return fail(d, AED_EINVAL, "bad layer / seq / buffer");
    HIP_TRY(d, hipStreamSynchronize(d->stream));
    const int T = d->enc_lens[seq], Dh = d->cfg.head_dim, H = d->cfg.n_heads, dm = d->cfg.d_model;
    std::vector<char> tmp((size_t)T * Dh * d->kv_esz);
    std::vector<float> f((size_t)T * Dh);
    for (int which = 0; which < 2; ++which) {
        const char* base = d->ws + (which ? d->lay.vc : d->lay.kc) + (size_t)layer * d->lay.cross_layer_elems * d->kv_esz;
        float* out = which ? v_out : k_out;
        for (int h = 0; h < H; ++h) {
            const char* src = base + ((size_t)h * d->cfg.max_total_enc_frames + d->enc_off[seq]) * Dh * d->kv_esz;
            HIP_TRY(d, hipMemcpy(tmp.data(), src, tmp.size(), hipMemcpyDeviceToHost));
            to_f32_host(tmp.data(), f.size(), d->kv_esz, f.data());
            for (int t = 0; t < T; ++t) memcpy(out + (size_t)t * dm + h * Dh, f.data() + (size_t)t * Dh, Dh * 4);
        }
    }
    return AED_OK;
}

aed_status aed_read_self_kv(aed_decoder* d, int32_t layer, int32_t seq, float* k_out, float* v_out,
                            int32_t* n_positions) {
    if (!d) return AED_EINVAL;
    if (d->state == aed_decoder::NO_BATCH) return fail(d, AED_ESTATE, "no batch");
    if (layer < 0 || layer >= d->cfg.n_layers || seq < 0 || seq >= d->batch || !k_out || !v_out || !n_positions)
        return fail(d, AED_EINVAL, "bad layer / seq / buffer");
    HIP_TRY(d, hipStreamSynchronize(d->stream));
    int n = 0;
    HIP_TRY(d, hipMemcpy(&n, d->at<int>(d->lay.seq_len) + seq, 4, hipMemcpyDeviceToHost));
    n = std::min(n, d->cfg.max_dec_len);
    *n_positions = n;
    const int Dh = d->cfg.head_dim, H = d->cfg.n_heads, dm = d->cfg.d_model;
    std::vector<char> tmp((size_t)kPage * Dh * d->kv_esz);
    std::vector<float> f((size_t)kPage * Dh);
    for (int which = 0; which < 2; ++which) {
        const char* base = d->ws + (which ? d->lay.v_pool : d->lay.k_pool) + (size_t)layer * d->lay.pool_layer_elems * d->kv_esz;
        float* out = which ? v_out : k_out;
        for (int blk = 0; blk * kPage < n; ++blk) {
            const int page = d->page_table[(size_t)seq * d->lay.max_pages + blk];
            for (int h = 0; h < H; ++h) {
                const char* src = base + ((size_t)page * H + h) * kPage * Dh * d->kv_esz;
                HIP_TRY(d, hipMemcpy(tmp.data(), src, tmp.size(), hipMemcpyDeviceToHost));
                to_f32_host(tmp.data(), f.size(), d->kv_esz, f.data());
                for (int s = 0; s < kPage && blk * kPage + s < n; ++s)
                    memcpy(out + (size_t)(blk * kPage + s) * dm + h * Dh, f.data() + (size_t)s * Dh, Dh * 4);
            }
        }
    }
    return AED_OK;
}

aed_status aed_read_logits(aed_decoder* d, float* logits_out) {
    if (!d) return AED_EINVAL;
    if (d->state == aed_decoder::NO_BATCH) return fail(d, AED_ESTATE, "no batch");
    if (!logits_out) return fail(d, AED_EINVAL, "logits_out is NULL");
    HIP_TRY(d, hipStreamSynchronize(d->stream));
    HIP_TRY(d, hipMemcpy(logits_out, d->act_at<float>(d->lay.logits), (size_t)d->batch * d->cfg.vocab * 4, hipMemcpyDeviceToHost));
    return AED_OK;
}

aed_status aed_time_kernels(aed_decoder* d, int32_t cls, int32_t reps, float* ms_total, int32_t* launches) {
    if (!d) return AED_EINVAL;
    if (d->state == aed_decoder::NO_BATCH) return fail(d, AED_ESTATE, "no batch");
    if (!ms_total || !launches || reps < 1) return fail(d, AED_EINVAL, "bad arguments");
    const bool per_layer = cls >= AED_K_LN_QKV && cls <= AED_K_FFN2;
    if (!per_layer && cls != AED_K_LN_VOCAB && cls != AED_K_CROSS_KV) return fail(d, AED_EINVAL, "kernel class cannot be timed alone");
    d->act = d->ws;
    const int cap = d->state == aed_decoder::CONSUMED ? d->last_prompt_len + d->last_max_new : d->host_pos;
    StateArgs st = d->state_args(0, 0);
    HIP_TRY(d, launch_prepare_timing(st, std::max(0, std::min(cap, d->cfg.max_dec_len) - 1), d->stream));
    int n = 0;
    HIP_TRY(d, hipEventRecord(d->t0, d->stream));
    for (int r = 0; r < reps; ++r) {
        if (cls == AED_K_LN_VOCAB) { HIP_TRY(d, k_ln_vocab(d)); ++n; continue; }
        for (int l = 0; l < d->cfg.n_layers; ++l) { HIP_TRY(d, k_class(d, cls, l)); n += class_launches(d, cls); }
    }
    HIP_TRY(d, hipEventRecord(d->t1, d->stream));
    HIP_TRY(d, hipEventSynchronize(d->t1));
    HIP_TRY(d, hipEventElapsedTime(ms_total, d->t0, d->t1));
    *launches = n;
    return AED_OK;
}

aed_status aed_kernel_work(aed_decoder* d, int32_t cls, double* bytes, double* flops) {
    if (!d) return AED_EINVAL;
    if (d->state == aed_decoder::NO_BATCH) return fail(d, AED_ESTATE, "no batch");
    if (!bytes || !flops) return fail(d, AED_EINVAL, "NULL output");
    HIP_TRY(d, hipStreamSynchronize(d->stream));
    const double e = (double)d->esz, ekv = (double)d->kv_esz, B = d->batch, dm = d->cfg.d_model, F = d->cfg.d_ffn, V = d->cfg.vocab;
    // ln: the product follows a LayerNorm.  float32 mode reads the float32 rows and the gain / shift vectors;
    // bfloat16 mode reads the rows' shadow, their tile statistics and shifts, and the folded vectors c1, c2.
    // resid: a residual update (float32 rows read and written); bfloat16 mode also writes shadow and statistics.
    const bool folded = folded_ln(d);
    const double stats = (dm / 16) * B * 8;
    auto gemm = [&](double M, double N, double K, double a_bytes, double out_bytes, bool ln, bool resid) {
        *bytes = N * K * e + M * N * out_bytes;
        if (!ln) *bytes += N * e + M * K * a_bytes;
        else if (folded) *bytes += M * K * e + stats + M * 4 + 2 * N * 4;
        else *bytes += N * e + M * K * 4 + 2 * K * e;
        if (resid && folded) *bytes += M * N * e + 2 * stats + M * 4 + N * e;
        *flops = 2 * M * N * K;
    };
    switch (cls) {
        case AED_K_LN_QKV:
            gemm(B, 3 * dm, dm, 4, 0, true, false);
            *bytes += B * dm * 4 + 2 * B * dm * ekv;
            if (merged_products(d)) {  // the part of the cross-attention query product that reads the same rows rides along
                *bytes += dm * dm * e + B * dm * 4;
                *flops += 2 * B * dm * dm;
            }
            break;
        case AED_K_SELF_OUT:
            gemm(B, dm, dm, e, 8, false, true);
            if (merged_products(d)) {  // the part of the cross-attention query product that reads o rides along
                *bytes += dm * dm * e + B * dm * 4;
                *flops += 2 * B * dm * dm;
            }
            break;
        case AED_K_CROSS_OUT: gemm(B, dm, dm, e, 8, false, true); break;
        case AED_K_LN_CROSSQ:
            if (merged_products(d)) { *bytes = 0; *flops = 0; break; }
            gemm(B, dm, dm, 4, 4, true, false);
            break;
        case AED_K_LN_FFN1: gemm(B, F, dm, 4, e, true, false); break;
        case AED_K_FFN2: gemm(B, dm, F, e, 8, false, true); break;
        case AED_K_LN_VOCAB: gemm(B, V, dm, 4, 4, true, false); break;
        case AED_K_CROSS_KV: gemm((double)d->total_enc, 2 * dm, dm, e, ekv, false, false); break;
        case AED_K_SELF_ATTN: case AED_K_CROSS_ATTN: {
            double keys = 0;
            if (cls == AED_K_CROSS_ATTN) keys = (double)d->total_enc;
            else {
                std::vector<int> len(d->batch);
                HIP_TRY(d, hipMemcpy(len.data(), d->at<int>(d->lay.seq_len), (size_t)d->batch * 4, hipMemcpyDeviceToHost));
                for (int b = 0; b < d->batch; ++b) keys += std::min(len[b], d->cfg.max_dec_len - 1) + 1;
            }
            *bytes = keys * 2 * dm * ekv + B * dm * 4 + B * dm * e;
            *flops = keys * 4 * dm;
            break;
        }
        default: return fail(d, AED_EINVAL, "unknown kernel class");
    }
    return AED_OK;
}

}  // extern "C"
