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
//   * operands go from global memory straight into MFMA register layout with
//     16-byte loads -- lane (r, g) (r = lane % 16, g = lane / 16) holds, for
//     row r of a 16-row operand, the 16 consecutive k values k0 + 16 g .. +15
//     of a 64-wide block.  Both operands use the same k assignment, so the
//     MFMA's internal k order does not matter;
//   * the weight fragment is the first MFMA operand: lane (r, g) then holds
//     C[m = r][n = 4 g .. 4 g + 3], four consecutive outputs of one row, which
//     stores as one 16-byte (fp32) or 8-byte (bf16) vector.
// The LayerNorm prologue keeps a wavefront's slice of the fp32 residual rows
// in registers, gets the row statistics with two LDS exchanges (mean, then
// centred sum of squares) and normalises in place, so the rows are read once.
#include "common.h"
#include "kernels.h"

namespace aed {

template <typename T> struct Frag16;
template <> struct Frag16<bf16_t> { bf16x8 lo, hi; };
template <> struct Frag16<float> { float v[16]; };

__device__ __forceinline__ Frag16<bf16_t> load_frag(const bf16_t* p) {
    Frag16<bf16_t> f;
    f.lo = reinterpret_cast<const bf16x8*>(p)[0];
    f.hi = reinterpret_cast<const bf16x8*>(p)[1];
    return f;
}
__device__ __forceinline__ Frag16<float> load_frag(const float* p) {
    Frag16<float> f;
    load_f32<16>(p, f.v);
    return f;
}
__device__ __forceinline__ void pack_frag(const float* y, Frag16<bf16_t>& f) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { f.lo[i] = (bf16_t)y[i]; f.hi[i] = (bf16_t)y[8 + i]; }
}
__device__ __forceinline__ void pack_frag(const float* y, Frag16<float>& f) {
#pragma unroll
    for (int i = 0; i < 16; ++i) f.v[i] = y[i];
}
// acc[n-major 16x16] += W-fragment x A-fragment over the 64-wide k block
__device__ __forceinline__ void mma(f32x4& acc, const Frag16<bf16_t>& w, const Frag16<bf16_t>& a) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.lo, a.lo, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.hi, a.hi, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma(f32x4& acc, const Frag16<float>& w, const Frag16<float>& a) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(w.v[i], a.v[i], acc, 0, 0, 0);
}

constexpr int kMaxLnBlocks = 4;  // PRO_LN: K <= 4 waves * 4 blocks * 64 = 1024

template <typename T, int PRO, int EPI, int MT, int NT>
__global__ __launch_bounds__(256) void gemm_decode_kernel(GemmArgs a) {
    constexpr int BM = 16 * MT, BN = 16 * NT;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int K = a.K, M = a.M;
    const int nblk = K >> 8;  // 64-wide k blocks per wavefront
    const T* __restrict__ W = static_cast<const T*>(a.W);

    __shared__ f32x4 part[4][MT * NT][64];
    __shared__ float red[2][4][BM];

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const T* wrow[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wrow[nt] = W + (size_t)(n0 + nt * 16 + r) * K + g * 16;

    if constexpr (PRO == PRO_LN) {
        const float* __restrict__ X = static_cast<const float*>(a.A);
        float xs[MT][kMaxLnBlocks][16];
        const float* xrow[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            int m = m0 + mt * 16 + r;
            m = m < M ? m : M - 1;
            xrow[mt] = X + (size_t)m * K + g * 16;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < kMaxLnBlocks; ++i)
                if (i < nblk) load_f32<16>(xrow[mt] + (i * 4 + wave) * 64, xs[mt][i]);
        // row mean
        float mean[MT], rstd[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < kMaxLnBlocks; ++i)
                if (i < nblk)
#pragma unroll
                    for (int e = 0; e < 16; ++e) s += xs[mt][i][e];
            s = rows4_sum(s);
            if (g == 0) red[0][wave][mt * 16 + r] = s;
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            int i = mt * 16 + r;
            mean[mt] = (red[0][0][i] + red[0][1][i] + red[0][2][i] + red[0][3][i]) / (float)K;
            float s = 0.f;
#pragma unroll
            for (int b = 0; b < kMaxLnBlocks; ++b)
                if (b < nblk)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        float c = xs[mt][b][e] - mean[mt];
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
        const T* __restrict__ G = static_cast<const T*>(a.ln_g);
        const T* __restrict__ Bt = static_cast<const T*>(a.ln_b);
#pragma unroll
        for (int i = 0; i < kMaxLnBlocks; ++i) {
            if (i < nblk) {
                const int k0 = (i * 4 + wave) * 64;
                float gam[16], bet[16];
                load_f32<16>(G + k0 + g * 16, gam);
                load_f32<16>(Bt + k0 + g * 16, bet);
                Frag16<T> af[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    float y[16];
#pragma unroll
                    for (int e = 0; e < 16; ++e) y[e] = (xs[mt][i][e] - mean[mt]) * rstd[mt] * gam[e] + bet[e];
                    pack_frag(y, af[mt]);
                }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    Frag16<T> wf = load_frag(wrow[nt] + k0);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) mma(acc[mt][nt], wf, af[mt]);
                }
            }
        }
    } else {
        const T* __restrict__ A = static_cast<const T*>(a.A);
        const T* arow[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            int m = m0 + mt * 16 + r;
            m = m < M ? m : M - 1;
            size_t src = a.a_row_map ? (size_t)a.a_row_map[m] : (size_t)m;
            arow[mt] = A + src * K + g * 16;
        }
#pragma unroll 2
        for (int i = 0; i < nblk; ++i) {
            const int k0 = (i * 4 + wave) * 64;
            Frag16<T> af[MT], wf[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wf[nt] = load_frag(wrow[nt] + k0);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) af[mt] = load_frag(arow[mt] + k0);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) mma(acc[mt][nt], wf[nt], af[mt]);
        }
    }

    // ---- sum the four wavefronts' partial tiles in a fixed order, then the epilogue ----
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) part[wave][mt * NT + nt][lane] = acc[mt][nt];
    __syncthreads();

    const T* __restrict__ bias = static_cast<const T*>(a.bias);
    for (int idx = tid; idx < MT * NT * 64; idx += 256) {
        const int t = idx >> 6, l = idx & 63;
        f32x4 s = part[0][t][l];
        s += part[1][t][l];
        s += part[2][t][l];
        s += part[3][t][l];
        const int mt = t / NT, nt = t % NT;
        const int m = m0 + mt * 16 + (l & 15);
        const int n = n0 + nt * 16 + (l >> 4) * 4;
        if (m >= M) continue;
        if (bias) s += load4(bias + n);
        if constexpr (EPI == EPI_RESID) {
            float* p = static_cast<float*>(a.out) + (size_t)m * a.N + n;
            f32x4 v = *reinterpret_cast<f32x4*>(p);
            v += s;
            *reinterpret_cast<f32x4*>(p) = v;
        } else if constexpr (EPI == EPI_F32) {
            store4(static_cast<float*>(a.out) + (size_t)m * a.N + n, s);
        } else if constexpr (EPI == EPI_RELU_T) {
            s[0] = fmaxf(s[0], 0.f); s[1] = fmaxf(s[1], 0.f); s[2] = fmaxf(s[2], 0.f); s[3] = fmaxf(s[3], 0.f);
            store4(static_cast<T*>(a.out) + (size_t)m * a.N + n, s);
        } else if constexpr (EPI == EPI_QKV) {
            const int d = a.d_model;
            if (n < d) {
                store4(static_cast<float*>(a.out) + (size_t)m * d + n, s);
            } else if (!a.finished[m]) {
                const int which = n >= 2 * d;
                const int c = n - (which ? 2 * d : d);
                const int h = c / a.head_dim, e = c % a.head_dim;
                const int pos = a.seq_len[m];
                const int page = a.page_table[(size_t)m * a.max_pages + (pos >> 4)];
                T* pool = static_cast<T*>(which ? a.v_pool : a.k_pool);
                store4(pool + (((size_t)page * a.n_heads + h) * kPage + (pos & 15)) * a.head_dim + e, s);
            }
        } else {  // EPI_CROSSKV
            const int d = a.d_model;
            const int which = n >= d;
            const int c = n - (which ? d : 0);
            const int h = c / a.head_dim, e = c % a.head_dim;
            T* dst = static_cast<T*>(which ? a.vc : a.kc);
            store4(dst + ((size_t)h * a.t_cap + m) * a.head_dim + e, s);
        }
    }
}

template <typename T, int PRO, int EPI, int MT, int NT>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
    dim3 grid(a.N / (16 * NT), (a.M + 16 * MT - 1) / (16 * MT));
    hipLaunchKernelGGL((gemm_decode_kernel<T, PRO, EPI, MT, NT>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

template <typename T, int PRO, int EPI>
static hipError_t launch_tiles(const GemmArgs& a, hipStream_t s) {
    // Tile choice: enough workgroups to cover the 256 CUs while keeping the
    // per-workgroup operand traffic (BM + BN) * K small.
    if (a.M <= 128) return launch_one<T, PRO, EPI, 1, 1>(a, s);
    if (a.M <= 512) return launch_one<T, PRO, EPI, 2, 2>(a, s);
    return launch_one<T, PRO, EPI, 2, 4>(a, s);
}

template <typename T>
static hipError_t launch_typed(GemmPro pro, GemmEpi epi, const GemmArgs& a, hipStream_t s) {
    if (pro == PRO_LN && epi == EPI_QKV) return launch_tiles<T, PRO_LN, EPI_QKV>(a, s);
    if (pro == PRO_LN && epi == EPI_F32) return launch_tiles<T, PRO_LN, EPI_F32>(a, s);
    if (pro == PRO_LN && epi == EPI_RELU_T) return launch_tiles<T, PRO_LN, EPI_RELU_T>(a, s);
    if (pro == PRO_T && epi == EPI_RESID) return launch_tiles<T, PRO_T, EPI_RESID>(a, s);
    if (pro == PRO_T && epi == EPI_CROSSKV) return launch_tiles<T, PRO_T, EPI_CROSSKV>(a, s);
    return hipErrorInvalidValue;
}

hipError_t launch_gemm(Dtype dt, GemmPro pro, GemmEpi epi, const GemmArgs& a, hipStream_t s) {
    if (a.M < 1 || a.K % 256 != 0 || a.N % 64 != 0) return hipErrorInvalidValue;
    if (pro == PRO_LN && a.K > 256 * kMaxLnBlocks) return hipErrorInvalidValue;
    return dt == kBF16 ? launch_typed<bf16_t>(pro, epi, a, s) : launch_typed<float>(pro, epi, a, s);
}

}  // namespace aed
