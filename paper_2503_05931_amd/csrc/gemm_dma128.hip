// 128 x 128 bf16 MFMA GEMM fed by direct-to-LDS loads, for the products whose M is
// in the hundreds or low thousands: the projections of a large decode batch and
// cross K/V precomputes too small for the 256 x 256 kernel (gemm_dma.hip, which
// documents the technique: fragment-order pieces moved by global_load_lds_dwordx4,
// explicit vmcnt waits, one barrier per k-step, requests spread between the MFMAs,
// every step the same straight-line code, persistent workgroups).
//
// What differs here:
//  * workgroup = 4 wavefronts (2 x 2), wavefront tile 64 x 64 = 2 x 2 MFMA tiles of
//    32 x 32, 64 accumulator registers per lane;
//  * a k-step is 64 k = both 1 KB pieces of each of the tile's 16 block rows
//    = 32 KB, 8 requests per wavefront; ring of 4 stages (128 KB);
//  * fragments are double-buffered in registers per 16-k sub-step (4 per step);
//  * the epilogue is the common one (gemm_epilogue: a lane's 4 consecutive outputs
//    of a row), optionally with the folded-LayerNorm correction (kernels.h, PRO_LNS).
// One 128 x 128 tile takes in 64 KB per 1024 MFMA cycles, which is more than a CU's
// memory pipeline delivers (about 50 bytes per clock), so this kernel is ingest-bound
// near 40 % of the MFMA peak; it is used where the problem has too few 256 x 256
// tiles to fill the GPU, and there it replaces a kernel that waited a full memory
// round trip per k-step.
#include <type_traits>

#include "common.h"
#include "gemm_common.h"
#include "kernels.h"
#include "device_once.h"

namespace aed {

namespace {

constexpr int kBM = 128, kBN = 128, kStages = 4, kStageBytes = 32768;
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void load_to_lds16(const void* g, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n" ::"s"(lds_base), "v"(g) : "memory");
}
template <int N> __device__ __forceinline__ void wait_loads_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace

template <int EPI, bool LNS>
__global__ __launch_bounds__(256) void gemm_dma128_kernel(GemmArgs a) {
    typedef bf16_t T;
    constexpr int S = kStages;
    extern __shared__ __align__(16) char lds[];
    __shared__ float row_stat[2][2][kBM];  // LNS: per row, two partial (mean, sum of squared deviations)
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;  // wavefront tile: rows [64 wm, +64), columns [64 wn, +64)
    const int r32 = lane & 31, hh = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int K = a.K, nk = K >> 6;
    const int n_mt = (a.M + kBM - 1) / kBM, n_nt = a.N / kBN, total = n_mt * n_nt;
    const int xcd = blockIdx.x & 7, j_in = blockIdx.x >> 3, per_x = gridDim.x >> 3;
    const int per_xcd = (total + 7) / 8;
    const int t_begin = xcd * per_xcd, t_end = min(total, t_begin + per_xcd);
    const int my_tiles = t_begin + j_in < t_end ? (t_end - (t_begin + j_in) + per_x - 1) / per_x : 0;
    if (my_tiles == 0) return;
    // Tile numbering.  An XCD works on a contiguous run of per_xcd tiles and fetches, through its L2, every row panel
    // of A and every column panel of W that the run touches (panels of equal size).  Numbered column-fastest, a run
    // covers few row panels and many column panels; row-fastest, the other way round.  Whichever touches fewer panels
    // is used: for a decode step's projections (8 row panels, 24 or 32 column panels) that is row-fastest, 11 or 12
    // panels per XCD instead of 25 or 33, and the run's panels then fit the 4 MB of L2.
    const int run = min(per_xcd, total);
    const bool m_fast = min(run, n_mt) + (run + n_mt - 1) / n_mt < (run + n_nt - 1) / n_nt + min(run, n_nt);
    auto tile_pos = [&](int tile, int& tm, int& tn) {
        if (m_fast) { tn = tile / n_mt; tm = tile - tn * n_mt; }
        else { tm = tile / n_nt; tn = tile - tm * n_nt; }
    };
    const char* __restrict__ A = static_cast<const char*>(a.A);
    const char* __restrict__ W = static_cast<const char*>(a.W);

    // ---- requests: this wavefront moves block rows 4 wave .. 4 wave + 3 of the stage (0..7: A, 8..15: W)
    const char* gp[4];
    const size_t row_bytes = (size_t)nk * 2048;  // one row of 16-row blocks
    auto set_tile_ptrs = [&](int ti) {
        const int tile = t_begin + j_in + ti * per_x;
        int tm, tn;
        tile_pos(tile, tm, tn);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int q = wave * 4 + jj;
            gp[jj] = (q < 8 ? A + (size_t)(tm * (kBM / 16) + q) * row_bytes
                            : W + (size_t)(tn * (kBN / 16) + q - 8) * row_bytes) + lane * 16;
        }
    };
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds0 + wave * 8192);
    int ld_slot = 0;
    // request j of a step (0..7): piece (j & 1) of block row 4 wave + (j >> 1); a k-step is one 2 KB block per row
    auto request_one = [&](int j) {
        load_to_lds16(gp[j >> 1] + (j & 1) * 1024, lds_wave + ld_slot * kStageBytes + j * 1024);
    };
    auto request_done = [&]() {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) gp[jj] += 2048;
        ld_slot = ld_slot == S - 1 ? 0 : ld_slot + 1;
    };

    // ---- fragments of sub-step sub (0..3) = piece (sub >> 1), chunks 2 (sub & 1) + (lane >> 5)
    const int frag_lane = (hh * 16 + (r32 & 15)) * 16 + (r32 >> 4) * 2048;
    struct Frags { bf16x8 w[2], a[2]; };
    auto read_frags = [&](int slot, int sub, Frags& f) {
        const char* st = lds + (size_t)slot * kStageBytes + frag_lane + (sub >> 1) * 1024 + (sub & 1) * 512;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) f.w[nt] = *reinterpret_cast<const bf16x8*>(st + (8 + wn * 4 + nt * 2) * 2048);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) f.a[mt] = *reinterpret_cast<const bf16x8*>(st + (wm * 4 + mt * 2) * 2048);
    };

    // acc[mt][nt][4 q + e] = C[row 32 mt + r32][column 32 nt + 8 q + 4 hh + e] of the wavefront tile
    f32x16 acc[2][2];
    auto zero_acc = [&]() {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;
    };
    zero_acc();

    // LNS: statistics of the tile's rows (two groups of threads combine half of the 16-column tiles each)
    float stat_n = 0.f;
    auto load_row_stats = [&](int ti) {
        const int tile = t_begin + j_in + ti * per_x;
        int tm, tn_unused;
        tile_pos(tile, tm, tn_unused);
        const int row = tid & 127, grp = tid >> 7, per = a.stat_tiles >> 1;
        stat_n = 16.f * (float)per;
        const float2* sp = a.stats_in + (size_t)(grp * per) * a.m_stride + (tm * kBM + row);
        float2 v[32];  // d_model <= 1024: at most 32 tiles per group; all loads first, one round trip
#pragma unroll
        for (int t = 0; t < 32; ++t) v[t] = t < per ? sp[(size_t)t * a.m_stride] : float2{0.f, 0.f};
        float sm = 0.f, m2 = 0.f;
#pragma unroll
        for (int t = 0; t < 32; ++t) {
            sm += v[t].x;
            m2 += v[t].y;
        }
        const float mean = sm / (float)per;
        float dev = 0.f;
#pragma unroll
        for (int t = 0; t < 32; ++t)
            if (t < per) dev += (v[t].x - mean) * (v[t].x - mean);
        row_stat[0][grp][row] = mean;
        row_stat[1][grp][row] = m2 + 16.f * dev;
    };

    // EPI_QKV: where the cache slot of each of this lane's two rows starts (element index for head 0; -1: the row is
    // finished or beyond M).  Position and page are two dependent loads per row: fetched here, at the start of a
    // tile, they are long there when the epilogue stores the keys and values.
    long long kv_base[2] = {-1, -1};
    auto load_kv_rows = [&](int ti) {
        const int tile = t_begin + j_in + ti * per_x;
        int tm, tn_unused;
        tile_pos(tile, tm, tn_unused);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int m = tm * kBM + wm * 64 + mt * 32 + r32;
            kv_base[mt] = -1;
            if (m < a.M && !a.finished[m]) {
                const int pos = a.seq_len[m];
                const int page = a.page_table[(size_t)m * a.max_pages + (pos >> 4)];
                kv_base[mt] = ((long long)page * a.n_heads * kPage + (pos & 15)) * a.head_dim;
            }
        }
    };

    set_tile_ptrs(0);
    if constexpr (EPI == EPI_QKV) load_kv_rows(0);
    for (int s = 0; s < S - 1; ++s) {  // nk >= 8: all inside the first tile
#pragma unroll
        for (int j = 0; j < 8; ++j) request_one(j);
        request_done();
    }
    if constexpr (LNS) load_row_stats(0);
    wait_loads_barrier<0>();  // steps 0 .. S-2 have landed
    Frags f0, f1;
    int slot = 0;  // slot of the step being computed

    auto mfma4 = [&](const Frags& f) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[nt], f.a[mt], acc[mt][nt], 0, 0, 0);
    };
    // One k-step: after the barrier step t+1 is complete in LDS and nobody reads the slot of step t-1 any more.
    auto step = [&](auto waited_before) {
        __builtin_amdgcn_sched_barrier(0);
        if (decltype(waited_before)::value) wait_lds_barrier();
        else wait_loads_barrier<(S - 2) * 8>();  // the requests of the two steps after this one may be in flight
        const int cur = slot;
        slot = slot == S - 1 ? 0 : slot + 1;
        read_frags(cur, 0, f0);
        read_frags(cur, 1, f1);
        mfma4(f0);
        request_one(0); request_one(1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 2, f0);
        mfma4(f1);
        request_one(2); request_one(3);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(cur, 3, f1);
        mfma4(f0);
        request_one(4); request_one(5);
        __builtin_amdgcn_sched_barrier(0);
        mfma4(f1);
        request_one(6); request_one(7);
        request_done();
        __builtin_amdgcn_sched_barrier(0);
    };

    for (int ti = 0; ti < my_tiles; ++ti) {
        // The requests of a tile's last S-1 steps are for the first steps of the next tile; after the last tile
        // they fetch that tile's own first steps again (never used), which keeps every step alike.
        const int ti_next = ti + 1 < my_tiles ? ti + 1 : ti;
        if (LNS && ti > 0) {
            wait_lds_barrier();  // every wavefront is through the previous tile's epilogue
            load_row_stats(ti);
        }
        if (EPI == EPI_QKV && ti > 0) load_kv_rows(ti);
#pragma unroll 1
        for (int ks = 0; ks < S - 2; ++ks) step(std::true_type{});  // waited for at the end of the previous tile
#pragma unroll 1
        for (int ks = S - 2; ks < nk; ++ks) {
            if (ks == nk - (S - 1)) set_tile_ptrs(ti_next);
            step(std::false_type{});
        }

        // ---- the tile is complete: everything requested so far has landed, so that the stores below may stay
        // in flight over the next tile's first S-2 steps
        const int tile = t_begin + j_in + ti * per_x;
        int tm, tn;
        tile_pos(tile, tm, tn);
        wait_loads_barrier<0>();
        const int m_base = tm * kBM + wm * 64, n_base = tn * kBN + wn * 64;
        float rstd[2], shift[2];
        if constexpr (LNS) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int rl = wm * 64 + mt * 32 + r32, m = tm * kBM + rl;
                const float a0 = row_stat[0][0][rl], a1 = row_stat[0][1][rl];
                float mu = 0.5f * (a0 + a1);
                const float d0 = a0 - mu, d1 = a1 - mu;
                const float m2 = row_stat[1][0][rl] + row_stat[1][1][rl] + stat_n * (d0 * d0 + d1 * d1);
                rstd[mt] = fold_norm(a.rms, (float)K, a.ln_eps, m2, mu);
                shift[mt] = m < a.M ? mu - a.mu_hat_in[m] : 0.f;
                if (tn == 0 && wn == 0 && hh == 0 && m < a.M && a.mu_hat_out) a.mu_hat_out[m] = mu;  // for the residual updates
            }
        }
        const T* __restrict__ bias = static_cast<const T*>(a.bias);
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n_base + nt * 32 + 8 * q + 4 * hh;
                f32x4 bv, c1 = f32x4{0.f, 0.f, 0.f, 0.f};
                if constexpr (LNS) {
                    bv = *reinterpret_cast<const f32x4*>(a.ln_c2 + n);
                    c1 = *reinterpret_cast<const f32x4*>(a.ln_c1 + n);
                } else {
                    bv = bias ? load4(bias + n) : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    const int m = m_base + mt * 32 + r32;
                    f32x4 v = {acc[mt][nt][4 * q], acc[mt][nt][4 * q + 1], acc[mt][nt][4 * q + 2], acc[mt][nt][4 * q + 3]};
                    if (m >= a.M) continue;
                    if constexpr (LNS) v = (v - shift[mt] * c1) * rstd[mt] + bv;
                    else v += bv;
                    if constexpr (EPI == EPI_QKV) {
                        const int d = a.d_model;
                        if (n < d) {
                            store4(static_cast<float*>(a.out) + (size_t)m * d + n, v);
                        } else if (kv_base[mt] >= 0) {
                            const int which = n >= 2 * d;
                            const int c = n - (which ? 2 * d : d);
                            const long long at = kv_base[mt] + (long long)(c / a.head_dim) * kPage * a.head_dim + c % a.head_dim;
                            if (a.kv_fp8) store4_fp8(static_cast<unsigned char*>(which ? a.v_pool : a.k_pool) + at, v);
                            else store4(static_cast<T*>(which ? a.v_pool : a.k_pool) + at, v);
                        }
                    } else {
                        gemm_epilogue<T, EPI>(a, m, n, v, f32x4{0.f, 0.f, 0.f, 0.f});
                    }
                }
            }
        zero_acc();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may land in LDS after the workgroup has ended
}

template <int EPI, bool LNS>
static hipError_t launch_dma128_one(const GemmArgs& a, hipStream_t s) {
    constexpr int kLds = kStages * kStageBytes;
    static DeviceOnce configured;
    hipError_t e = configured.run([&]() {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma128_kernel<EPI, LNS>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    });
    if (e != hipSuccess) return e;
    const int tiles = ((a.M + kBM - 1) / kBM) * (a.N / kBN);
    const int grid = persistent_grid(tiles);  // at most one workgroup per CU, whole rounds over the XCDs
    if (grid <= 0) return hipErrorInvalidDevice;
    hipLaunchKernelGGL((gemm_dma128_kernel<EPI, LNS>), dim3(grid), dim3(256), kLds, s, a);
    return hipGetLastError();
}

// bf16 only.  A (fragment order) must hold whole 128-row tiles; N % 128 == 0; K % 64 == 0 and K >= 512.
// a.ln_c1 != null: the LayerNorm is folded around the product (PRO_LNS).
hipError_t launch_gemm_dma128(GemmEpi epi, const GemmArgs& a, hipStream_t s) {
    if (a.M < 1 || a.N % kBN != 0 || a.K % 64 != 0 || a.K < 512) return hipErrorInvalidValue;
    if (a.ln_c1) {
        if (!a.ln_c2 || !a.stats_in || !a.mu_hat_in || a.stat_tiles < 2 || a.stat_tiles % 2 != 0 ||
            a.stat_tiles > 64)
            return hipErrorInvalidValue;
        switch (epi) {
            case EPI_QKV: return launch_dma128_one<EPI_QKV, true>(a, s);
            case EPI_F32: return launch_dma128_one<EPI_F32, true>(a, s);
            case EPI_RELU_T: return launch_dma128_one<EPI_RELU_T, true>(a, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (epi) {
        case EPI_CROSSKV: return launch_dma128_one<EPI_CROSSKV, false>(a, s);
        case EPI_QKV: return launch_dma128_one<EPI_QKV, false>(a, s);
        case EPI_F32: return launch_dma128_one<EPI_F32, false>(a, s);
        case EPI_RELU_T: return launch_dma128_one<EPI_RELU_T, false>(a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace aed
