// LDS-tiled MFMA GEMM for large M on gfx950: the cross-attention K/V
// precompute (M = all encoder frames of the batch) and, at large decode batches,
// the projections.  bf16 only (float32 mode uses the streaming kernel).
//
// C[M,N] = A[M,K] . W[N,K]^T with both operands already in fragment order
// (16-row x 64-k blocks of 2 KB whose bytes are laid out lane by lane exactly as
// the 16x16x32 MFMA wants them).  That makes the staging trivial and
// conflict-free:
//   * global -> LDS: a block is 2 KB contiguous in memory and is copied as is,
//     128 lanes x 16 B per block, fully coalesced;
//   * LDS -> registers: lane l of a wavefront reads bytes [16 l, 16 l + 16) of
//     each of the block's two 1 KB pieces: consecutive lanes, consecutive
//     addresses, no bank conflicts, no swizzle.
// Workgroup = 4 wavefronts in a 2 x 2 arrangement over a (32 WM) x (32 WN) tile;
// each wavefront owns WM x WN MFMA tiles of 16 x 16, accumulated over K in
// registers.  K advances in 64-wide steps with a two-stage LDS ring fed from a
// deeper ring of registers: the global loads of step k+D are issued before the
// MFMAs of step k, and step k+1 goes from registers to the other LDS stage after
// them; one barrier per step.
// As in the streaming kernel the weight fragment is the first MFMA operand, so a
// lane ends up with four consecutive outputs of one row.
#include "common.h"
#include "gemm_common.h"
#include "kernels.h"
#include "device_once.h"

namespace aed {

template <int EPI, int WM, int WN, int D, bool LNS>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(GemmArgs a) {
    typedef bf16_t T;
    constexpr int BM = 32 * WM, BN = 32 * WN;
    constexpr int A_BLOCKS = BM / 16, W_BLOCKS = BN / 16, BLOCKS = A_BLOCKS + W_BLOCKS;  // 2 KB each
    constexpr int LOADS = BLOCKS / 2;  // 256 threads copy two blocks per instruction
    static_assert(BLOCKS % 2 == 0, "block count must be even");
    extern __shared__ __align__(16) char lds[];  // 2 stages x BLOCKS x 2 KB

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    // XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so XCD x gets the
    // contiguous run of tiles [x * per_xcd, (x + 1) * per_xcd).  Tiles are numbered n-fastest: a run
    // sweeps all n-tiles of one row panel before moving on, so the panel of A rows is fetched from HBM
    // once and re-used from that XCD's L2, while the (small) weight matrix stays cache-resident.
    const int n_mt = (a.M + BM - 1) / BM, n_nt = a.N / BN;
    const int total = n_mt * n_nt, per_xcd = (total + 7) / 8;
    const int wg = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (wg >= total) return;  // the grid is rounded up to whole rounds over the XCDs
    const int tile_m = wg / n_nt, tile_n = wg % n_nt;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // LNS (LayerNorm folded around the product, see kernels.h): statistics of this tile's rows, two groups of
    // threads combine half of the 16-column tiles each; read back after the k loop's last barrier
    __shared__ float row_stat[2][2][BM];
    float stat_n = 0.f;
    if constexpr (LNS) {
        static_assert(BM == 128, "one thread per row and half");
        const int row = tid & 127, grp = tid >> 7, per = a.stat_tiles >> 1;
        stat_n = 16.f * (float)per;
        const float2* sp = a.stats_in + (size_t)(grp * per) * a.m_stride + (m0 + row);
        float2 v[32];  // d_model <= 1024: at most 32 tiles per group; all loads first, one round trip
#pragma unroll
        for (int t = 0; t < 32; ++t) v[t] = t < per ? sp[(size_t)t * a.m_stride] : float2{0.f, 0.f};
        float sm = 0.f, m2 = 0.f;
#pragma unroll
        for (int t = 0; t < 32; ++t) {
            sm += v[t].x;  // entries beyond per are zero
            m2 += v[t].y;
        }
        const float mean = sm / (float)per;
        float dev = 0.f;
#pragma unroll
        for (int t = 0; t < 32; ++t)
            if (t < per) dev += (v[t].x - mean) * (v[t].x - mean);
        m2 += 16.f * dev;
        row_stat[0][grp][row] = mean;
        row_stat[1][grp][row] = m2;
    }
    const int K = a.K, nk = K >> 6;
    const char* __restrict__ A = static_cast<const char*>(a.A);
    const char* __restrict__ W = static_cast<const char*>(a.W);

    // this thread's share of a k-step: LOADS 16-byte pieces; piece i covers block 2 i + (tid >> 7)
    const int half = tid >> 7, in_blk = (tid & 127) * 16;
    auto src = [&](int i, int kb) -> const f32x4* {
        const int blk = 2 * i + half;
        const char* p = blk < A_BLOCKS ? A + frag_block_off<2>((m0 >> 4) + blk, kb, K)
                                       : W + frag_block_off<2>((n0 >> 4) + (blk - A_BLOCKS), kb, K);
        return reinterpret_cast<const f32x4*>(p + in_blk);
    };
    auto dst = [&](int stage, int i) -> f32x4* {
        return reinterpret_cast<f32x4*>(lds + ((size_t)stage * BLOCKS + 2 * i + half) * 2048 + in_blk);
    };

    f32x4 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // D k-steps of global loads are in flight in registers (HBM latency is several k-steps long);
    // the LDS ring has two stages.  The k loop is unrolled by D so that the register slots are static.
    f32x4 stage_regs[D][LOADS];
#pragma unroll
    for (int u = 0; u < D; ++u)
        if (u < nk)
#pragma unroll
            for (int i = 0; i < LOADS; ++i) stage_regs[u][i] = *src(i, u);
#pragma unroll
    for (int i = 0; i < LOADS; ++i) *dst(0, i) = stage_regs[0][i];
    __syncthreads();

    for (int kb0 = 0; kb0 < nk; kb0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int kb = kb0 + u;
            if (kb < nk) {
                const int cur = kb & 1;
                // slot u held k-step kb, which is already in LDS: refill it with k-step kb + D
                if (kb + D < nk) {
#pragma unroll
                    for (int i = 0; i < LOADS; ++i) stage_regs[u][i] = *src(i, kb + D);
                }
                const char* base = lds + (size_t)cur * BLOCKS * 2048;
                // all fragments of the step are read from LDS first, then the MFMAs run back to back
                Frag16<T> wf[WN], af[WM];
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    const bf16x8* p =
                        reinterpret_cast<const bf16x8*>(base + (size_t)(A_BLOCKS + wn * WN + j) * 2048) + lane;
                    wf[j].lo = p[0];
                    wf[j].hi = p[64];
                }
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    const bf16x8* p = reinterpret_cast<const bf16x8*>(base + (size_t)(wm * WM + i) * 2048) + lane;
                    af[i].lo = p[0];
                    af[i].hi = p[64];
                }
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j].lo, af[i].lo, acc[i][j], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j].hi, af[i].hi, acc[i][j], 0, 0, 0);
                if (kb + 1 < nk) {  // k-step kb + 1 sits in slot (u + 1) % D
#pragma unroll
                    for (int i = 0; i < LOADS; ++i) *dst(cur ^ 1, i) = stage_regs[(u + 1) % D][i];
                }
                __syncthreads();
            }
        }
    }

    // epilogue: lane (r, g) of tile (i, j) holds C[m][n .. n+3], m = row r of the tile, n = 4 g
    const int r = lane & 15, g = lane >> 4;
    const T* __restrict__ bias = static_cast<const T*>(a.bias);
    float rstd[WM], shift[WM];  // LNS: per row of this lane
    if constexpr (LNS) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int rl = (wm * WM + i) * 16 + r;
            const float a0 = row_stat[0][0][rl], a1 = row_stat[0][1][rl];
            float mu = 0.5f * (a0 + a1);
            const float d0 = a0 - mu, d1 = a1 - mu;
            const float m2 = row_stat[1][0][rl] + row_stat[1][1][rl] + stat_n * (d0 * d0 + d1 * d1);
            rstd[i] = fold_norm(a.rms, (float)K, a.ln_eps, m2, mu);
            shift[i] = m0 + rl < a.M ? mu - a.mu_hat_in[m0 + rl] : 0.f;
            if (n0 == 0 && wn == 0 && g == 0 && m0 + rl < a.M && a.mu_hat_out) a.mu_hat_out[m0 + rl] = mu;  // for the residual updates
        }
    }
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int n = n0 + (wn * WN + j) * 16 + g * 4;
        f32x4 bv, c1 = f32x4{0.f, 0.f, 0.f, 0.f};
        if constexpr (LNS) {
            bv = *reinterpret_cast<const f32x4*>(a.ln_c2 + n);
            c1 = *reinterpret_cast<const f32x4*>(a.ln_c1 + n);
        } else {
            bv = bias ? load4(bias + n) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int m = m0 + (wm * WM + i) * 16 + r;
            if (m >= a.M) continue;
            f32x4 res = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (EPI == EPI_RESID)
                res = *reinterpret_cast<const f32x4*>(static_cast<const char*>(a.out) + frag_elem_off<4>(m, n, a.N));
            if constexpr (LNS) gemm_epilogue<T, EPI>(a, m, n, (acc[i][j] - shift[i] * c1) * rstd[i] + bv, res);
            else gemm_epilogue<T, EPI>(a, m, n, acc[i][j] + bv, res);
        }
    }
}

template <int EPI, int WM, int WN, int D, bool LNS>
static hipError_t launch_tiled_one(const GemmArgs& a, hipStream_t s) {
    constexpr int BM = 32 * WM, BN = 32 * WN;
    constexpr size_t kLds = 2ull * (BM / 16 + BN / 16) * 2048;
    static DeviceOnce configured;
    hipError_t e = configured.run([&]() {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_tiled_kernel<EPI, WM, WN, D, LNS>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
    });
    if (e != hipSuccess) return e;
    const int tiles = ((a.M + BM - 1) / BM) * (a.N / BN);
    const int grid = (tiles + 7) / 8 * 8;  // whole rounds over the 8 XCDs (surplus ids exit at once)
    hipLaunchKernelGGL((gemm_tiled_kernel<EPI, WM, WN, D, LNS>), dim3(grid), dim3(256), kLds, s, a);
    return hipGetLastError();
}

// bf16 only; A (fragment order) padded to a multiple of 128 rows in memory; N % 128 == 0; K % 64 == 0.
hipError_t launch_gemm_tiled(GemmEpi epi, const GemmArgs& a, hipStream_t s) {
    if (a.M < 1 || a.N % 128 != 0 || a.K % 64 != 0) return hipErrorInvalidValue;
    // from 8 k-blocks on, the same tile fed by direct-to-LDS loads (several k-steps in flight) is used instead
    if (a.K >= 512 && epi != EPI_RESID) return launch_gemm_dma128(epi, a, s);
    // Measured on MI355X for the cross K/V GEMM (K = 1024, N = 2048, bf16), TFLOP/s at M = 7 217 / 512 000:
    //   128x128 tile, D = 1: 627 / 684      256x128, D = 1: 485 / 529      128x64, D = 1: 567 / 621
    //   128x128, D = 2: 410 / 419 (one workgroup per CU instead of two: registers)
    // Two co-resident workgroups matter more than tile size or prefetch depth: with 64x64 wavefront
    // tiles LDS reads alone need as many cycles as the MFMAs, so a second workgroup fills the gaps.
    if (a.ln_c1) {  // LayerNorm folded around the product
        if (!a.ln_c2 || !a.stats_in || !a.mu_hat_in || a.stat_tiles < 2 || a.stat_tiles % 2 != 0 || a.stat_tiles > 64)
            return hipErrorInvalidValue;
        switch (epi) {
            case EPI_QKV: return launch_tiled_one<EPI_QKV, 4, 4, 1, true>(a, s);
            case EPI_F32: return launch_tiled_one<EPI_F32, 4, 4, 1, true>(a, s);
            case EPI_RELU_T: return launch_tiled_one<EPI_RELU_T, 4, 4, 1, true>(a, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (epi) {
        case EPI_CROSSKV: return launch_tiled_one<EPI_CROSSKV, 4, 4, 1, false>(a, s);
        case EPI_QKV: return launch_tiled_one<EPI_QKV, 4, 4, 1, false>(a, s);
        case EPI_RESID: return launch_tiled_one<EPI_RESID, 4, 4, 1, false>(a, s);
        case EPI_F32: return launch_tiled_one<EPI_F32, 4, 4, 1, false>(a, s);
        case EPI_RELU_T: return launch_tiled_one<EPI_RELU_T, 4, 4, 1, false>(a, s);
        default: break;
    }
    return hipErrorInvalidValue;
}

}  // namespace aed
