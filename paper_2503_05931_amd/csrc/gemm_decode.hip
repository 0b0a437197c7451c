// Weight-streaming MFMA GEMM for the decoder step's projections (QKV, attention
// output, cross-attention query, FFN, vocabulary) on gfx950.
//
// C[M,N] = prologue(A)[M,K] . W[N,K]^T: M is the decode batch (1..1024), the
// weights W are read exactly once per launch and dominate the traffic, so the
// kernel is organised around streaming W:
//   * a workgroup (4 wavefronts) owns a (16*MT) x (16*NT) output tile;
//   * the four wavefronts split K: wavefront w takes the 64-wide k blocks
//     w, w+4, w+8, ..., and the partial tiles are summed through LDS in a
//     fixed order (deterministic);
//   * lane (r, g) (r = lane % 16, g = lane / 16) holds, for row r of a 16-row
//     operand, the 16 consecutive k values k0 + 16 g .. +15 of a 64-wide block.
//     Both operands use the same k assignment, so the MFMA's internal k order
//     does not matter;
//   * both operands live in memory in fragment order (common.h): the weights
//     are re-ordered once when the decoder is created, the activations are
//     written in that order by the kernels that produce them.  Every operand
//     load is then one coalesced 1 KB instruction per wavefront straight into
//     MFMA registers -- no LDS staging, no transposes;
//   * the weight fragment is the first MFMA operand: lane (r, g) then holds
//     C[m = r][n = 4 g .. 4 g + 3], four consecutive outputs of one row, which
//     is one 16-byte (fp32) or 8-byte (bf16) store, also into fragment order.
// The LayerNorm prologue (batches up to 128 rows) keeps a wavefront's slice of
// the fp32 residual rows in registers, gets the row statistics with two LDS
// exchanges (mean, then centred sum of squares) and normalises in place, so the
// rows are read once per workgroup.  Larger batches normalise once in a
// separate small kernel (layernorm_frag_kernel) and stream the result.
#include "common.h"
#include "gemm_common.h"
#include "kernels.h"

namespace aed {

constexpr int kMaxLnBlocks = 4;  // PRO_LN: K <= 4 waves * 4 blocks * 64 = 1024
constexpr int kMaxStatTilesPerGroup = 16;  // folded LayerNorm: d_model <= 1024 = 4 groups * 16 tiles * 16 columns

// One output tile (column tile bx, row tile by) of the product described by a.
// WNT: W is loaded with the non-temporal hint (GemmArgs::w_nt)
template <typename T, int PRO, int EPI, int MT, int NT, bool WNT>
__device__ __forceinline__ void gemm_decode_body(const GemmArgs& a, const int bx, const int by) {
    constexpr int BM = 16 * MT, BN = 16 * NT;
    constexpr int EP = (MT * NT * 64 + 255) / 256;  // output 4-vectors per thread in the epilogue
    constexpr int ES = sizeof(T);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int m0 = by * BM, n0 = bx * BN;
    const int K = a.K, M = a.M;
    const int nblk = K >> 8;  // 64-wide k blocks per wavefront
    const char* __restrict__ W = static_cast<const char*>(a.W);

    __shared__ f32x4 part[4][MT * NT][64];
    __shared__ float red[2][4][BM];

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // block (n tile, k block i*4 + wave) of the re-ordered weights
    auto wblk = [&](int nt, int i) {
        return reinterpret_cast<const T*>(W + frag_block_off<ES>((n0 >> 4) + nt, i * 4 + wave, K));
    };

    // ---- the operand stream (everything but the float32-mode LayerNorm prologue)
    const char* __restrict__ A = static_cast<const char*>(a.A);
    // U blocks are fetched per group, two groups in flight (register double buffer)
    constexpr int U = (MT + NT) <= 2 ? 4 : ((MT + NT) <= 4 ? 2 : 1);
    Frag16<T> af[2][U][MT], wf[2][U][NT];
    auto fetch = [&](int buf, int blk0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = blk0 + u;
            if (i < nblk) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) wf[buf][u][nt] = WNT ? load_frag_nt(wblk(nt, i), lane) : load_frag(wblk(nt, i), lane);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    af[buf][u][mt] = load_frag(
                        reinterpret_cast<const T*>(A + frag_block_off<ES>((m0 >> 4) + mt, i * 4 + wave, K)), lane);
            }
        }
    };
    auto compute = [&](int buf, int blk0) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (blk0 + u < nblk)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) mma(acc[mt][nt], wf[buf][u][nt], af[buf][u][mt]);
    };
    // The stream's first requests go out before anything else: every request in front of them (the epilogue's
    // operands below are a dozen or two per wavefront) holds the whole stream back by its issue time.
    if constexpr (PRO != PRO_LN) fetch(0, 0);

    // Epilogue operands do not depend on the product: they are requested here, behind the stream's first group, and
    // have long arrived when the stream is through.
    constexpr bool LNS = PRO == PRO_LNS;         // LayerNorm folded around the product (see kernels.h)
    constexpr bool RS = EPI == EPI_RESID_S;      // residual update that also writes shadow and statistics
    constexpr bool RES = EPI == EPI_RESID || RS;
    const T* __restrict__ bias = static_cast<const T*>(a.bias);
    f32x4 e_bias[EP], e_res[EP], e_aux[EP];  // e_aux: c1 (LNS)
    float e_mu[EP];                          // LNS: the shift this row's shadow was written with; RS: the row's
                                             // mean before the update = the shift its new shadow is written with
#pragma unroll
    for (int j = 0; j < EP; ++j) {
        const int idx = tid + 256 * j;
        const int t = idx >> 6, l = idx & 63;
        const int m = m0 + (t / NT) * 16 + (l & 15);
        const int n = n0 + (t % NT) * 16 + (l >> 4) * 4;
        const bool live = idx < MT * NT * 64 && m < M;
        const f32x4 zero = f32x4{0.f, 0.f, 0.f, 0.f};
        if constexpr (LNS) {
            const bool raw = a.n_raw > 0 && n >= a.n_raw;  // columns from n_raw on are not normalised here
            e_bias[j] = !live ? zero : *reinterpret_cast<const f32x4*>(raw ? a.raw_bias + (n - a.n_raw) : a.ln_c2 + n);
            e_aux[j] = live && !raw ? *reinterpret_cast<const f32x4*>(a.ln_c1 + n) : zero;
        } else {
            e_bias[j] = (bias && live) ? load4(bias + n) : zero;
        }
        if constexpr (LNS || RS) e_mu[j] = live ? a.mu_hat_in[m] : 0.f;
        if constexpr (RES)
            e_res[j] = live ? *reinterpret_cast<const f32x4*>(static_cast<const char*>(a.out) + frag_elem_off<4>(m, n, a.N))
                            : zero;
        if constexpr (EPI == EPI_F32 && !LNS)  // optional addend, float [M,N] row-major like the output
            e_res[j] = (live && a.addend) ? *reinterpret_cast<const f32x4*>(a.addend + (size_t)m * a.N + n) : zero;
    }
    // EPI_QKV: where this thread's key / value columns go in the paged cache (element index, -1: nowhere).  The
    // sequence's state and its page-table entry are two dependent loads; fetched here, they are off the critical
    // path at the end.
    long long e_kv[EP];
    if constexpr (EPI == EPI_QKV) {
#pragma unroll
        for (int j = 0; j < EP; ++j) {
            const int idx = tid + 256 * j;
            const int t = idx >> 6, l = idx & 63;
            const int m = m0 + (t / NT) * 16 + (l & 15);
            const int n = n0 + (t % NT) * 16 + (l >> 4) * 4;
            e_kv[j] = -1;
            if (idx < MT * NT * 64 && m < M && n >= a.d_model && n < 3 * a.d_model && !a.finished[m]) {
                const int c = n - (n >= 2 * a.d_model ? 2 * a.d_model : a.d_model);
                const int h = c / a.head_dim, e = c % a.head_dim;
                const int pos = a.seq_len[m];
                const int page = a.page_table[(size_t)m * a.max_pages + (pos >> 4)];
                e_kv[j] = (((long long)page * a.n_heads + h) * kPage + (pos & 15)) * a.head_dim + e;
            }
        }
    }
    // the epilogue of EPI_QKV with the cache position already known
    auto store_qkv = [&](int m, int n, f32x4 s, long long at) {
        if (n < a.d_model) {
            store4(static_cast<float*>(a.out) + (size_t)m * a.d_model + n, s);
        } else if (at >= 0) {
            void* pool = n >= 2 * a.d_model ? a.v_pool : a.k_pool;
            if (a.kv_fp8) store4_fp8(static_cast<unsigned char*>(pool) + at, s);
            else store4(static_cast<T*>(pool) + at, s);
        }
    };
    float stat_n = 0.f;  // elements behind each of the four partial results of the row statistics
    // mean and sum of squared deviations of local row rl over all columns, from the four partial results
    auto row_stats = [&](int rl, float& mu, float& m2) {
        const float a0 = red[0][0][rl], a1 = red[0][1][rl], a2 = red[0][2][rl], a3 = red[0][3][rl];
        mu = 0.25f * (a0 + a1 + a2 + a3);
        const float d0 = a0 - mu, d1 = a1 - mu, d2 = a2 - mu, d3 = a3 - mu;
        m2 = red[1][0][rl] + red[1][1][rl] + red[1][2][rl] + red[1][3][rl] + stat_n * (d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3);
    };

    // LNS: statistics of the rows being multiplied: four groups of threads combine a quarter of the 16-column
    // tiles each; the epilogue combines the four.  The loads go out here, ahead of the operand stream; nothing
    // waits for them before the stream is through.
    float2 sv[kMaxStatTilesPerGroup];
    const int st_row = tid % BM, st_grp = tid / BM, st_per = a.stat_tiles >> 2;
    if constexpr (LNS) {
        stat_n = 16.f * (float)st_per;
        const float2* sp = a.stats_in + (size_t)((st_grp & 3) * st_per) * a.m_stride + (m0 + st_row);
#pragma unroll
        for (int t = 0; t < kMaxStatTilesPerGroup; ++t)
            sv[t] = (t < st_per && st_grp < 4) ? sp[(size_t)t * a.m_stride] : float2{0.f, 0.f};
    }
    auto combine_row_stats = [&]() {  // equal-sized parts: mean of the means, then the parts' own sums of squares
                                      // plus 16 x the squared distances of their means (fixed order, no long chain)
        float sm = 0.f, sq = 0.f;
#pragma unroll
        for (int t = 0; t < kMaxStatTilesPerGroup; ++t) {
            sm += sv[t].x;  // entries beyond st_per are zero
            sq += sv[t].y;
        }
        const float mean = sm / (float)st_per;
        float dev = 0.f;
#pragma unroll
        for (int t = 0; t < kMaxStatTilesPerGroup; ++t)
            if (t < st_per) dev += (sv[t].x - mean) * (sv[t].x - mean);
        if (st_grp < 4) {
            red[0][st_grp][st_row] = mean;
            red[1][st_grp][st_row] = sq + 16.f * dev;
        }
    };

    if constexpr (PRO == PRO_LN) {
        const char* __restrict__ X = static_cast<const char*>(a.A);
        Frag16<float> xs[MT][kMaxLnBlocks];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < kMaxLnBlocks; ++i)
                if (i < nblk)
                    xs[mt][i] = load_frag(
                        reinterpret_cast<const float*>(X + frag_block_off<4>((m0 >> 4) + mt, i * 4 + wave, K)), lane);
        // the weight stream starts before the statistics are known
        Frag16<T> wf[NT][kMaxLnBlocks];
#pragma unroll
        for (int i = 0; i < kMaxLnBlocks; ++i)
            if (i < nblk)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) wf[nt][i] = WNT ? load_frag_nt(wblk(nt, i), lane) : load_frag(wblk(nt, i), lane);
        // LayerNorm gain/shift for this lane's k values, fetched before the statistics are known
        const T* __restrict__ G = static_cast<const T*>(a.ln_g);
        const T* __restrict__ Bt = static_cast<const T*>(a.ln_b);
        Frag16<T> gam_f[kMaxLnBlocks], bet_f[kMaxLnBlocks];
#pragma unroll
        for (int i = 0; i < kMaxLnBlocks; ++i)
            if (i < nblk) {
                gam_f[i] = load_frag_rm(G + (i * 4 + wave) * 64 + g * 16);
                if (Bt) bet_f[i] = load_frag_rm(Bt + (i * 4 + wave) * 64 + g * 16);
                else zero_frag(bet_f[i]);
            }
        // row mean
        float mean[MT], rstd[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < kMaxLnBlocks; ++i)
                if (i < nblk)
#pragma unroll
                    for (int e = 0; e < 16; ++e) s += xs[mt][i].v[e];
            s = rows4_sum(s);
            if (g == 0) red[0][wave][mt * 16 + r] = s;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            int i = mt * 16 + r;
            mean[mt] = a.rms ? 0.f : (red[0][0][i] + red[0][1][i] + red[0][2][i] + red[0][3][i]) / (float)K;
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < kMaxLnBlocks; ++b)
                if (b < nblk)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        float c = xs[mt][b].v[e] - mean[mt];
                        s += c * c;
                    }
            s = rows4_sum(s);
            if (g == 0) red[1][wave][i] = s;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            int i = mt * 16 + r;
            float var = (red[1][0][i] + red[1][1][i] + red[1][2][i] + red[1][3][i]) / (float)K;
            rstd[mt] = 1.0f / sqrtf(var + a.ln_eps);
        }
#pragma unroll
        for (int i = 0; i < kMaxLnBlocks; ++i) {
            if (i < nblk) {
                float gam[16], bet[16];
                unpack_frag(gam_f[i], gam);
                unpack_frag(bet_f[i], bet);
                Frag16<T> af[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    float y[16];
#pragma unroll
                    for (int e = 0; e < 16; ++e) y[e] = (xs[mt][i].v[e] - mean[mt]) * rstd[mt] * gam[e] + bet[e];
                    pack_frag(y, af[mt]);
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) mma(acc[mt][nt], wf[nt][i], af[mt]);
            }
        }
    } else {
        for (int b0 = 0; b0 < nblk; b0 += 2 * U) {
            fetch(1, b0 + U);
            compute(0, b0);
            fetch(0, b0 + 2 * U);
            compute(1, b0 + U);
        }
    }

    if constexpr (LNS) combine_row_stats();
    // ---- sum the four wavefronts' partial tiles in a fixed order, then the epilogue ----
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) part[wave][mt * NT + nt][lane] = acc[mt][nt];
    __syncthreads();

#pragma unroll
    for (int j = 0; j < EP; ++j) {
        const int idx = tid + 256 * j;
        if (idx >= MT * NT * 64) continue;
        const int t = idx >> 6, l = idx & 63;
        f32x4 s = part[0][t][l];
        s += part[1][t][l];
        s += part[2][t][l];
        s += part[3][t][l];
        const int mt = t / NT, nt = t % NT;
        const int m = m0 + mt * 16 + (l & 15);
        const int n = n0 + nt * 16 + (l >> 4) * 4;
        if (m >= M) continue;
        if constexpr (LNS) {
            float mu, m2;
            row_stats(mt * 16 + (l & 15), mu, m2);
            const float rstd = fold_norm(a.rms, (float)K, a.ln_eps, m2, mu), shift = mu - e_mu[j];
            if (a.n_raw > 0 && n >= a.n_raw) {
                // a product that belongs to a later normalisation of these rows (kernels.h, "merged products"):
                // the bare sums (plus raw_bias) go to out2, whoever reads them finishes them
                store4(a.out2 + (size_t)m * (a.N - a.n_raw) + (n - a.n_raw), s + e_bias[j]);
                continue;
            }
            s = (s - shift * e_aux[j]) * rstd + e_bias[j];
            if constexpr (EPI == EPI_QKV) store_qkv(m, n, s, e_kv[j]);
            else gemm_epilogue<T, EPI>(a, m, n, s, e_res[j]);
            if (n == 0 && a.mu_hat_out) a.mu_hat_out[m] = mu;  // the layer's residual updates shift their shadows by this
        } else if constexpr (RS) {
            const float mu_old = e_mu[j];
            const f32x4 x = e_res[j] + s + e_bias[j];
            *reinterpret_cast<f32x4*>(static_cast<char*>(a.out) + frag_elem_off<4>(m, n, a.N)) = x;
            store4(reinterpret_cast<T*>(static_cast<char*>(a.shadow_out) + frag_elem_off<ES>(m, n, a.N)), x - mu_old);
            // this row's 16 columns of the tile sit in the four lanes l, l ^ 16, l ^ 32, l ^ 48
            float sum = (x[0] + x[1]) + (x[2] + x[3]);
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            const float tmean = sum * (1.f / 16.f);
            const f32x4 dv = x - tmean;
            float q = (dv[0] * dv[0] + dv[1] * dv[1]) + (dv[2] * dv[2] + dv[3] * dv[3]);
            q += __shfl_xor(q, 16);
            q += __shfl_xor(q, 32);
            if ((l >> 4) == 0) {
                a.stats_out[(size_t)(n >> 4) * a.m_stride + m] = float2{tmean, q};
            }
        } else {
            s += e_bias[j];
            if constexpr (EPI == EPI_F32) s += e_res[j];
            if constexpr (EPI == EPI_QKV) store_qkv(m, n, s, e_kv[j]);
            else gemm_epilogue<T, EPI>(a, m, n, s, e_res[j]);
        }
    }
}

template <typename T, int PRO, int EPI, int MT, int NT, bool WNT>
__global__ __launch_bounds__(256) void gemm_decode_kernel(GemmArgs a) {
    gemm_decode_body<T, PRO, EPI, MT, NT, WNT>(a, blockIdx.x, blockIdx.y);
}

// Two products of the same operand in one launch: the first n0 workgroups are the tiles of a0 (a residual update,
// EPI_RESID_S), the others the tiles of a1 (kernels.h, "merged products").  Neither reads what the other writes.
template <typename T, int MT0, int NT0, int EPI1, int MT1, int NT1, bool WNT>
__global__ __launch_bounds__(256) void gemm_decode_pair_kernel(GemmArgs a0, GemmArgs a1, int n0) {
    int b = blockIdx.x;
    if (b < n0) {
        const int nx = a0.N / (16 * NT0);
        gemm_decode_body<T, PRO_T, EPI_RESID_S, MT0, NT0, WNT>(a0, b % nx, b / nx);
    } else {
        b -= n0;
        const int nx = a1.N / (16 * NT1);
        gemm_decode_body<T, PRO_T, EPI1, MT1, NT1, WNT>(a1, b % nx, b / nx);
    }
}

// ---------------------------------------------------------------- LayerNorm to fragment order
// For larger batches the LayerNorm is not fused into the GEMM (every n-tile workgroup would re-read
// and re-normalise all fp32 rows, and the resident rows starve the big tiles of registers): this
// kernel writes h = LN(x) once, in the storage type and fragment order, and the GEMM streams it like
// any other activation.  One wavefront per row: lane l holds the 16 k values of k-group l (block
// l / 4, quarter l % 4), the statistics are two wavefront reductions -- no LDS, no barrier -- and
// M / 4 workgroups spread the rows over the GPU.
template <typename T>
__global__ __launch_bounds__(256) void layernorm_frag_kernel(const char* __restrict__ X, const T* __restrict__ G,
                                                             const T* __restrict__ Bt, char* __restrict__ Hout, int M,
                                                             int K, float eps, int rms) {
    constexpr int ES = sizeof(T);
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const int n_groups = K >> 4;  // 16-wide k groups in a row (K <= 1024: at most 64, one per lane)
    const bool live = lane < n_groups;
    const int kb = lane >> 2, q = lane & 3;
    const int frag_lane = q * 16 + (row & 15);
    float x[16];
    if (live) {
        const f32x4* p = reinterpret_cast<const f32x4*>(X + frag_block_off<4>(row >> 4, kb, K)) + frag_lane;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x4 v = p[64 * j];
            x[4 * j] = v[0]; x[4 * j + 1] = v[1]; x[4 * j + 2] = v[2]; x[4 * j + 3] = v[3];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) x[e] = 0.f;
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) s += x[e];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    const float mean = rms ? 0.f : s / (float)K;  // RMSNorm: no mean subtraction
    float m2 = 0.f;
    if (live) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float c = x[e] - mean;
            m2 += c * c;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m2 += __shfl_xor(m2, off);
    const float rstd = 1.0f / sqrtf(m2 / (float)K + eps);
    if (!live) return;
    const int k0 = lane * 16;
    float gam[16], bet[16], y[16];
    unpack_frag(load_frag_rm(G + k0), gam);
    if (Bt) {
        unpack_frag(load_frag_rm(Bt + k0), bet);
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) bet[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (x[e] - mean) * rstd * gam[e] + bet[e];
    Frag16<T> f;
    pack_frag(y, f);
    store_frag(reinterpret_cast<T*>(Hout + frag_block_off<ES>(row >> 4, kb, K)), frag_lane, f);
}

constexpr int kWntMaxM = 128;
template <typename T, int PRO, int EPI, int MT, int NT>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
    dim3 grid(a.N / (16 * NT), (a.M + 16 * MT - 1) / (16 * MT));
    // the hint only where few row tiles share W: with many (measured at M = 1024) they need it from the cache
    if (a.w_nt && a.M <= kWntMaxM) hipLaunchKernelGGL((gemm_decode_kernel<T, PRO, EPI, MT, NT, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gemm_decode_kernel<T, PRO, EPI, MT, NT, false>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

// Tile choice by a traffic model: each workgroup pulls (BM * bytes(A) + BN * bytes(W)) * K
// through its CU and the launch's workgroups are spread over the 256 CUs; pick the
// candidate with the least bytes per CU, then the fewest workgroups.
template <typename T, int PRO>
static int choose_tile(const GemmArgs& a) {
    struct Cand { int mt, nt; };
    static const Cand cands[] = {{1, 1}, {2, 2}, {2, 4}, {4, 2}, {4, 4}};
    const double a_bytes = PRO == PRO_LN ? 4.0 : sizeof(T), w_bytes = sizeof(T);
    int best = 0;
    double best_cost = 1e300;
    long best_wgs = 0;
    // float32 fragments are twice as wide, and the fused LayerNorm keeps its rows in registers: small tiles only
    const int n_cands = (sizeof(T) == 4 || PRO == PRO_LN) ? 2 : 5;
    static_assert(PRO != PRO_LNS || sizeof(T) == 2, "the folded LayerNorm is a bfloat16-mode path");
    for (int c = 0; c < n_cands; ++c) {
        const int bm = 16 * cands[c].mt, bn = 16 * cands[c].nt;
        if (a.N % bn != 0) continue;
        const long wgs = (long)((a.M + bm - 1) / bm) * (a.N / bn);
        // Workgroups of the smaller tiles share a CU (two or three fit by registers), so beyond 256 workgroups the
        // bytes through a CU grow in proportion, not in whole rounds.  The 64 x 64 tile runs one workgroup per CU
        // and its stream costs about half more than its bytes say when K is short (measured at M = 256, K = 1024:
        // 9.7 us against 8.2 us for the 32 x 64 tile on the QKV product); over K = 4096 the start-up is a smaller
        // part and the bytes decide (second FFN product at M = 1024: 18.1 us against 19.4 us for 32 x 64).
        const double rounds = wgs > 256 ? (double)wgs / 256.0 : 1.0;
        const double cost = rounds * (bm * a_bytes + bn * w_bytes) * (c == 4 && a.K < 4096 ? 1.6 : 1.0);
        if (cost < best_cost || (cost == best_cost && wgs < best_wgs)) { best = c; best_cost = cost; best_wgs = wgs; }
    }
    return best;
}

template <typename T, int PRO, int EPI>
static hipError_t launch_tiles(const GemmArgs& a, hipStream_t s) {
    const int best = choose_tile<T, PRO>(a);
    if (best == 0) return launch_one<T, PRO, EPI, 1, 1>(a, s);
    if (best == 1) return launch_one<T, PRO, EPI, 2, 2>(a, s);
    if constexpr (PRO != PRO_LN) {
        if (best == 2) return launch_one<T, PRO, EPI, 2, 4>(a, s);
        if (best == 3) return launch_one<T, PRO, EPI, 4, 2>(a, s);
        return launch_one<T, PRO, EPI, 4, 4>(a, s);
    }
    return hipErrorInvalidValue;
}

constexpr int kLnFusedMaxM = 128;
// The LDS-tiled kernel (bf16, 128 x 128 tiles) takes over once its tiles fill the GPU; below that
// the streaming kernel's 256+ small workgroups are faster (measured at M = 1024: N = 1024 gives 64
// tiles and 17.8 us against 7.6 us streamed; N = 4096 gives 256 tiles and 23.8 us against 28.4 us).
constexpr int kTiledMinTiles = 160;
template <typename T> static bool use_tiled(const GemmArgs& a) {
    return sizeof(T) == 2 && a.N % 128 == 0 && (long)((a.M + 127) / 128) * (a.N / 128) >= kTiledMinTiles;
}

// The 256 x 256 direct-to-LDS kernel (cross K/V product only) needs whole 256-row tiles in A and enough
// tiles to occupy most of the compute units with one workgroup each.
constexpr int kDmaMinTiles = 160;
template <typename T> static bool use_dma_crosskv(const GemmArgs& a) {
    return sizeof(T) == 2 && a.N % 256 == 0 && a.N == 2 * a.d_model && a.K >= 256 &&
           a.a_rows >= (a.M + 255) / 256 * 256 && (long)((a.M + 255) / 256) * (a.N / 256) >= kDmaMinTiles;
}

template <typename T>
static hipError_t launch_typed(GemmPro pro, GemmEpi epi, const GemmArgs& a0, hipStream_t s) {
    GemmArgs a = a0;
    // fused LayerNorm while one round of 32x32 tiles covers the product; else LayerNorm once, separately
    if (pro == PRO_LN && a.M > kLnFusedMaxM && (long)((a.M + 31) / 32) * (a.N / 32) > 256) {
        // two launches: h = LN(x) in fragment order, then the plain streaming GEMM on h
        if (!a.ln_scratch) return hipErrorInvalidValue;
        hipLaunchKernelGGL(layernorm_frag_kernel<T>, dim3((a.M + 3) / 4), dim3(256), 0, s,
                           static_cast<const char*>(a.A), static_cast<const T*>(a.ln_g), static_cast<const T*>(a.ln_b),
                           static_cast<char*>(a.ln_scratch), a.M, a.K, a.ln_eps, a.rms);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        a.A = a.ln_scratch;
        if (use_tiled<T>(a)) return launch_gemm_tiled(epi, a, s);
        if (epi == EPI_QKV) return launch_tiles<T, PRO_T, EPI_QKV>(a, s);
        if (epi == EPI_F32) return launch_tiles<T, PRO_T, EPI_F32>(a, s);
        if (epi == EPI_RELU_T) return launch_tiles<T, PRO_T, EPI_RELU_T>(a, s);
        return hipErrorInvalidValue;
    }
    if constexpr (sizeof(T) == 2) {
        if (pro == PRO_LNS) {
            if (!a.stats_in || !a.mu_hat_in || !a.ln_c1 || !a.ln_c2 || a.stat_tiles < 4 || a.stat_tiles % 4 != 0 ||
                a.stat_tiles > 4 * kMaxStatTilesPerGroup)
                return hipErrorInvalidValue;
            if (use_tiled<T>(a)) return launch_gemm_tiled(epi, a, s);
            if (epi == EPI_QKV) return launch_tiles<T, PRO_LNS, EPI_QKV>(a, s);
            if (epi == EPI_F32) return launch_tiles<T, PRO_LNS, EPI_F32>(a, s);
            if (epi == EPI_RELU_T) return launch_tiles<T, PRO_LNS, EPI_RELU_T>(a, s);
            return hipErrorInvalidValue;
        }
        if (pro == PRO_T && epi == EPI_RESID_S) {
            if (!a.stats_out || !a.mu_hat_in || !a.shadow_out || a.stat_tiles < 4 ||
                a.stat_tiles % 4 != 0 || a.stat_tiles * 16 != a.N || a.stat_tiles > 4 * kMaxStatTilesPerGroup)
                return hipErrorInvalidValue;
            return launch_tiles<T, PRO_T, EPI_RESID_S>(a, s);
        }
    }
    if (pro == PRO_LN && epi == EPI_QKV) return launch_tiles<T, PRO_LN, EPI_QKV>(a, s);
    if (pro == PRO_LN && epi == EPI_F32) return launch_tiles<T, PRO_LN, EPI_F32>(a, s);
    if (pro == PRO_LN && epi == EPI_RELU_T) return launch_tiles<T, PRO_LN, EPI_RELU_T>(a, s);
    if (pro == PRO_T && epi == EPI_CROSSKV && use_dma_crosskv<T>(a)) return launch_gemm_dma_crosskv(a, s);
    if (pro == PRO_T && use_tiled<T>(a)) return launch_gemm_tiled(epi, a, s);
    if (pro == PRO_T && epi == EPI_RESID) return launch_tiles<T, PRO_T, EPI_RESID>(a, s);
    if (pro == PRO_T && epi == EPI_CROSSKV) return launch_tiles<T, PRO_T, EPI_CROSSKV>(a, s);
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------- two products in one launch
template <typename T, int MT0, int NT0, int EPI1, int MT1, int NT1>
static hipError_t launch_pair_one(const GemmArgs& a0, const GemmArgs& a1, hipStream_t s) {
    const int n0 = (a0.N / (16 * NT0)) * ((a0.M + 16 * MT0 - 1) / (16 * MT0));
    const int n1 = (a1.N / (16 * NT1)) * ((a1.M + 16 * MT1 - 1) / (16 * MT1));
    if (a0.w_nt && a0.M <= kWntMaxM)
        hipLaunchKernelGGL((gemm_decode_pair_kernel<T, MT0, NT0, EPI1, MT1, NT1, true>), dim3(n0 + n1), dim3(256), 0, s, a0, a1, n0);
    else
        hipLaunchKernelGGL((gemm_decode_pair_kernel<T, MT0, NT0, EPI1, MT1, NT1, false>), dim3(n0 + n1), dim3(256), 0, s, a0, a1, n0);
    return hipGetLastError();
}
template <typename T, int EPI1>
static hipError_t launch_pair_epi(const GemmArgs& a0, const GemmArgs& a1, hipStream_t s) {
    // 16 x 16 or 32 x 32 tiles for each of the two (the batches this is used for have at most 256 rows)
    const int t0 = choose_tile<T, PRO_T>(a0) > 0, t1 = choose_tile<T, PRO_T>(a1) > 0;
    if (a0.N % 32 != 0 || a1.N % 32 != 0) return hipErrorInvalidValue;
    if (!t0 && !t1) return launch_pair_one<T, 1, 1, EPI1, 1, 1>(a0, a1, s);
    if (!t0 && t1) return launch_pair_one<T, 1, 1, EPI1, 2, 2>(a0, a1, s);
    if (t0 && !t1) return launch_pair_one<T, 2, 2, EPI1, 1, 1>(a0, a1, s);
    return launch_pair_one<T, 2, 2, EPI1, 2, 2>(a0, a1, s);
}

hipError_t launch_gemm_pair(Dtype dt, const GemmArgs& a0, GemmEpi epi1, const GemmArgs& a1, hipStream_t s) {
    if (dt != kBF16 || a0.M < 1 || a0.M != a1.M || a0.M > 256 || a0.K % 256 != 0 || a1.K % 256 != 0) return hipErrorInvalidValue;
    if (!a0.stats_out || !a0.mu_hat_in || !a0.shadow_out || a0.stat_tiles < 4 || a0.stat_tiles % 4 != 0 ||
        a0.stat_tiles * 16 != a0.N || a0.stat_tiles > 4 * kMaxStatTilesPerGroup)
        return hipErrorInvalidValue;
    if (epi1 == EPI_F32) return launch_pair_epi<bf16_t, EPI_F32>(a0, a1, s);
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(Dtype dt, GemmPro pro, GemmEpi epi, const GemmArgs& a, hipStream_t s) {
    if (a.M < 1 || a.K % 256 != 0 || a.N % 64 != 0) return hipErrorInvalidValue;
    if (pro == PRO_LN && a.K > 256 * kMaxLnBlocks) return hipErrorInvalidValue;
    return dt == kBF16 ? launch_typed<bf16_t>(pro, epi, a, s) : launch_typed<float>(pro, epi, a, s);
}

// ---------------------------------------------------------------- LayerNorm folding (once, at create)
// One wavefront per output column: c1[n] = sum_k W[n,k] g[k], c2[n] = sum_k W[n,k] b[k] + bias[n].
template <typename T>
__global__ __launch_bounds__(256) void fold_ln_kernel(const T* __restrict__ W, const T* __restrict__ g,
                                                      const T* __restrict__ b, const T* __restrict__ bias,
                                                      float* __restrict__ c1, float* __restrict__ c2, int N, int K) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    float s1 = 0.f, s2 = 0.f;
    for (int k = lane; k < K; k += 64) {
        const float w = (float)W[(size_t)n * K + k];
        s1 += to_f32(from_f32<T>(w * (float)g[k]));  // the column-scaled matrix as reorder_weight_kernel stores it
        if (b) s2 += w * (float)b[k];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        s1 += __shfl_xor(s1, off);
        s2 += __shfl_xor(s2, off);
    }
    if (lane == 0) {
        c1[n] = s1;
        c2[n] = s2 + (bias ? (float)bias[n] : 0.f);
    }
}

hipError_t launch_fold_ln(Dtype dt, const void* W, const void* g, const void* b, const void* bias, float* c1, float* c2,
                          int N, int K, hipStream_t s) {
    const dim3 grid((N + 3) / 4);
    if (dt == kBF16)
        hipLaunchKernelGGL(fold_ln_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(W),
                           static_cast<const bf16_t*>(g), static_cast<const bf16_t*>(b),
                           static_cast<const bf16_t*>(bias), c1, c2, N, K);
    else
        hipLaunchKernelGGL(fold_ln_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(W),
                           static_cast<const float*>(g), static_cast<const float*>(b), static_cast<const float*>(bias),
                           c1, c2, N, K);
    return hipGetLastError();
}

// ---------------------------------------------------------------- weight re-ordering
// dst (fragment order) <- src (row-major [N, K]), columns scaled by gain (may be null); one thread per 16-byte piece.
template <typename T>
__global__ __launch_bounds__(256) void reorder_weight_kernel(const T* __restrict__ src, const T* __restrict__ gain,
                                                             char* __restrict__ dst, int N, int K, int dst_k0, int dst_K) {
    constexpr int ES = sizeof(T), EPP = 16 / ES;
    const size_t piece = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t n_pieces = (size_t)N * K / EPP;
    if (piece >= n_pieces) return;
    const int n = (int)(piece / (K / EPP));
    const int k = (int)(piece % (K / EPP)) * EPP;
    T v[EPP];
    *reinterpret_cast<f32x4*>(v) = *reinterpret_cast<const f32x4*>(src + (size_t)n * K + k);  // 16 bytes, any type
    if (gain) {
#pragma unroll
        for (int e = 0; e < EPP; ++e) v[e] = from_f32<T>(to_f32(v[e]) * to_f32(gain[k + e]));
    }
    *reinterpret_cast<f32x4*>(dst + frag_elem_off<ES>(n, dst_k0 + k, dst_K)) = *reinterpret_cast<const f32x4*>(v);
}

// Product of two weight matrices for a merged product (kernels.h): P[n, k] = sum_j T(W1[n, j] g[j]) W2[j, k], float32 sums
// of the stored (rounded) factors, rounded to T once and written in fragment order into columns dst_k0 .. dst_k0 + K
// of a matrix with dst_K columns.  W1 [N, J], W2 [J, K] row-major; g may be null.  One 64 x 64 output tile per
// workgroup, 4 x 4 outputs per thread, 16-deep slices through LDS.  Runs once, when the decoder is created.
template <typename T>
__global__ __launch_bounds__(256) void weight_product_kernel(const T* __restrict__ W1, const T* __restrict__ g,
                                                             const T* __restrict__ W2, char* __restrict__ dst, int N, int J,
                                                             int K, int dst_k0, int dst_K) {
    __shared__ float sa[16][64 + 4], sb[16][64 + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int n0 = blockIdx.y * 64, k0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int j0 = 0; j0 < J; j0 += 16) {
        for (int i = tid; i < 64 * 16; i += 256) {
            const int n = i >> 4, j = i & 15;  // W1 tile: 64 rows x 16 j, read along j
            float w = to_f32(W1[(size_t)(n0 + n) * J + j0 + j]);
            if (g) w = to_f32(from_f32<T>(w * to_f32(g[j0 + j])));
            sa[j][n] = w;
            const int jj = i >> 6, k = i & 63;  // W2 tile: 16 j x 64 columns, read along k
            sb[jj][k] = to_f32(W2[(size_t)(j0 + jj) * K + k0 + k]);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float av[4], bv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { av[u] = sa[j][ty * 4 + u]; bv[u] = sb[j][tx * 4 + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(av[u], bv[v], acc[u][v]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int n = n0 + ty * 4 + u, k = k0 + tx * 4;
        store4(reinterpret_cast<T*>(dst + frag_elem_off<sizeof(T)>(n, dst_k0 + k, dst_K)),
               f32x4{acc[u][0], acc[u][1], acc[u][2], acc[u][3]});
    }
}

hipError_t launch_weight_product(Dtype dt, const void* W1, const void* g, const void* W2, void* dst, int N, int J, int K,
                                 int dst_k0, int dst_K, hipStream_t s) {
    if (dt != kBF16 || N % 64 != 0 || K % 64 != 0 || J % 16 != 0 || dst_k0 % 64 != 0 || dst_K % 64 != 0 || dst_k0 + K > dst_K)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(weight_product_kernel<bf16_t>, dim3(K / 64, N / 64), dim3(256), 0, s, static_cast<const bf16_t*>(W1),
                       static_cast<const bf16_t*>(g), static_cast<const bf16_t*>(W2), static_cast<char*>(dst), N, J, K, dst_k0, dst_K);
    return hipGetLastError();
}

// out[n] = sum_j T(W[n, j] g[j]) v[j] (float32; v null: zeros).  One wavefront per n.
template <typename T>
__global__ __launch_bounds__(256) void fold_vec_kernel(const T* __restrict__ W, const T* __restrict__ g, const T* __restrict__ v,
                                                       float* __restrict__ out, int N, int J) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    float sum = 0.f;
    if (v)
        for (int j = lane; j < J; j += 64) {
            float w = to_f32(W[(size_t)n * J + j]);
            if (g) w = to_f32(from_f32<T>(w * to_f32(g[j])));
            sum += w * to_f32(v[j]);
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) out[n] = sum;
}

hipError_t launch_fold_vec(Dtype dt, const void* W, const void* g, const void* v, float* out, int N, int J, hipStream_t s) {
    if (dt != kBF16) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fold_vec_kernel<bf16_t>, dim3((N + 3) / 4), dim3(256), 0, s, static_cast<const bf16_t*>(W),
                       static_cast<const bf16_t*>(g), static_cast<const bf16_t*>(v), out, N, J);
    return hipGetLastError();
}

// dst (fragment order, [M, K]) <- rows of a row-major source, row m taken from src row row_map[m] (or m)
template <typename T>
__global__ __launch_bounds__(256) void reorder_rows_kernel(const T* __restrict__ src, const int* __restrict__ row_map,
                                                           char* __restrict__ dst, int M, int K) {
    constexpr int ES = sizeof(T), EPP = 16 / ES;
    const int m = blockIdx.x;
    const size_t srow = row_map ? (size_t)row_map[m] : (size_t)m;
    for (int k = threadIdx.x * EPP; k < K; k += 256 * EPP) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(src + srow * K + k);
        *reinterpret_cast<f32x4*>(dst + frag_elem_off<ES>(m, k, K)) = v;
    }
}

hipError_t launch_reorder_rows(Dtype dt, const void* src, const int* row_map, void* dst, int M, int K, hipStream_t s) {
    if (M < 1 || K % 64 != 0) return hipErrorInvalidValue;
    if (dt == kBF16)
        hipLaunchKernelGGL(reorder_rows_kernel<bf16_t>, dim3(M), dim3(256), 0, s, static_cast<const bf16_t*>(src), row_map,
                           static_cast<char*>(dst), M, K);
    else
        hipLaunchKernelGGL(reorder_rows_kernel<float>, dim3(M), dim3(256), 0, s, static_cast<const float*>(src), row_map,
                           static_cast<char*>(dst), M, K);
    return hipGetLastError();
}

hipError_t launch_reorder_weight(Dtype dt, const void* src, const void* gain, void* dst, int N, int K, hipStream_t s,
                                 int dst_k0, int dst_K) {
    if (dst_K <= 0) dst_K = K;
    if (N % 16 != 0 || K % 64 != 0 || dst_k0 % 64 != 0 || dst_K % 64 != 0 || dst_k0 + K > dst_K) return hipErrorInvalidValue;
    const size_t pieces = (size_t)N * K / (dt == kBF16 ? 8 : 4);
    dim3 grid((unsigned)((pieces + 255) / 256));
    if (dt == kBF16)
        hipLaunchKernelGGL(reorder_weight_kernel<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(src),
                           static_cast<const bf16_t*>(gain), static_cast<char*>(dst), N, K, dst_k0, dst_K);
    else
        hipLaunchKernelGGL(reorder_weight_kernel<float>, grid, dim3(256), 0, s, static_cast<const float*>(src),
                           static_cast<const float*>(gain), static_cast<char*>(dst), N, K, dst_k0, dst_K);
    return hipGetLastError();
}

}  // namespace aed
