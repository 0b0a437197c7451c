// Persistent 256 x 256 bf16 MFMA GEMM whose operands go from memory straight
// into LDS (no registers in between), for the cross-attention K/V precompute
// over all encoder frames of a batch: C[M, 2 d] = A[M, d] . W[2 d, d]^T + b,
// written as per-head K and V rows.
//
// Why a second tiled kernel: with 128 x 128 tiles a compute unit has to take in
// 64 KB per 1024 MFMA cycles, more than its memory pipeline delivers (measured:
// about 50 bytes per clock and CU from L2); at 256 x 256 it is 32 KB.
//
//  * Both operands are in fragment order, so a 1 KB piece (16 rows x 32 k, one
//    16-byte fragment slice per lane) is what one wavefront-wide
//    global_load_lds_dwordx4 moves: lane l's 16 bytes land at LDS base + 16 l,
//    which is the layout the MFMA operands are read back in.  A k-step is 32 k
//    = one piece of each of the tile's 32 block rows = 32 KB; the 8 wavefronts
//    request 4 pieces each.
//  * Ring of 5 stages (160 KB).  The requests are not visible to the compiler,
//    so the waits are explicit: vmcnt counts a wavefront's requests in issue
//    order, each wavefront waits for its own part of step t+1, and the barrier
//    that follows makes the whole stage visible to everyone.  A wait never
//    counts on anything but loads issued after the ones it needs, so stores in
//    flight only make it longer.
//  * One barrier per k-step.  After it: LDS reads of the second half of step t,
//    MFMAs of the first half with this wavefront's four requests for step t+4
//    spread between them (a burst of requests right after the barrier fills the
//    memory pipeline's queue and stalls every wavefront at its next request),
//    LDS reads of the first half of step t+1, MFMAs of the second half.  Every
//    step is the same straight-line code: with all wavefronts at the same place
//    after a barrier, any chain of branches before the first MFMA idles the
//    matrix pipeline (measured: 1 279 -> 1 100 cycles per step of 1 024 MFMA cycles).
//  * 32x32x16 MFMAs (they reach the matrix pipeline's peak with one wavefront
//    per SIMD and four accumulators; the 16x16x32 shape needs four times that).
//    Wavefront tile 128 (m) x 64 (n); the weight fragment is the first operand,
//    so a lane holds 4 consecutive n of one output row.
//  * The workgroup is persistent: it walks its tiles as one stream of k-steps,
//    so the requests for the next tile are in flight during the epilogue.  The
//    accumulators of a tile start from the bias.  At the end of a tile each
//    wavefront turns its accumulators (lane = row) into 128-byte row segments
//    (lane = 16 bytes of a row) through 4 KB of the stage it has just finished,
//    so that a store instruction writes 8 full 128-byte lines.
//  * Tiles are numbered n-fastest and each XCD owns a contiguous run of them
//    (workgroup ids go round-robin over the 8 XCDs): the workgroups of an XCD
//    share A row panels and the weight tiles through that XCD's L2.
#include <type_traits>

#include "common.h"
#include "gemm_common.h"
#include "kernels.h"
#include "device_once.h"

namespace aed {

namespace {

constexpr int kBM = 256, kBN = 256, kStages = 5, kStageBytes = 32768;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));

// One request: every lane's 16 bytes at g go to LDS byte (lds_base + 16 * lane).  lds_base is wavefront-uniform.
__device__ __forceinline__ void load_to_lds16(const void* g, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n" ::"s"(lds_base), "v"(g) : "memory");
}
// At most N of this wavefront's memory operations still in flight, its LDS reads done, then the barrier.
template <int N> __device__ __forceinline__ void wait_loads_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

}  // namespace

// FP8: the caches take 8-bit E4M3 codes (see store4_fp8) instead of bfloat16
template <bool FP8>
__global__ __launch_bounds__(512) void gemm_dma_crosskv_kernel(GemmArgs a) {
    constexpr int S = kStages;
    extern __shared__ __align__(16) char lds[];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 2, wn = wave & 3;  // wavefront tile: rows [128 wm, +128), columns [64 wn, +64)
    const int r32 = lane & 31, hh = lane >> 5;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int K = a.K, nk = K >> 5;
    const int n_mt = (a.M + kBM - 1) / kBM, n_nt = a.N / kBN, total = n_mt * n_nt;
    const int xcd = blockIdx.x & 7, j_in = blockIdx.x >> 3, per_x = gridDim.x >> 3;
    const int per_xcd = (total + 7) / 8;
    const int t_begin = xcd * per_xcd, t_end = min(total, t_begin + per_xcd);
    const int my_tiles = t_begin + j_in < t_end ? (t_end - (t_begin + j_in) + per_x - 1) / per_x : 0;
    if (my_tiles == 0) return;
    const char* __restrict__ A = static_cast<const char*>(a.A);
    const char* __restrict__ W = static_cast<const char*>(a.W);

    // ---- requests: one pointer per piece this wavefront asks for, and the ring slot of the next request step
    const char* gp[4];
    const size_t row_bytes = (size_t)(K >> 6) * 2048;  // one row of 16-row blocks
    auto set_tile_ptrs = [&](int ti) {
        const int tile = t_begin + j_in + ti * per_x;
        const int tm = tile / n_nt, tn = tile - tm * n_nt;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = wave * 4 + j;  // piece of the stage: 0..15 A block rows, 16..31 W block rows
            gp[j] = (q < 16 ? A + (size_t)(tm * (kBM / 16) + q) * row_bytes
                            : W + (size_t)(tn * (kBN / 16) + q - 16) * row_bytes) + lane * 16;
        }
    };
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane(lds0 + wave * 4096);
    int ld_slot = 0;
    // k-step ks of a tile is the 1 KB piece at byte ks * 1024 of every block row
    auto request_one = [&](int j) {
        load_to_lds16(gp[j], lds_wave + ld_slot * kStageBytes + j * 1024);
        gp[j] += 1024;
    };
    auto request_done = [&]() { ld_slot = ld_slot == S - 1 ? 0 : ld_slot + 1; };

    // ---- fragments: 32x32x16 takes row (lane & 31) and the 8 k of chunk (2 j + (lane >> 5)) of the piece
    const int frag_lane = (hh * 16 + (r32 & 15)) * 16 + (r32 >> 4) * 1024;
    auto read_frags = [&](int slot, int j, bf16x8* wf, bf16x8* af) {
        const char* st = lds + (size_t)slot * kStageBytes + frag_lane + j * 512;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) wf[nt] = *reinterpret_cast<const bf16x8*>(st + (16 + wn * 4 + nt * 2) * 1024);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) af[mt] = *reinterpret_cast<const bf16x8*>(st + (wm * 8 + mt * 2) * 1024);
    };

    // ---- accumulators: acc[mt][nt][4 q + e] = C[row 32 mt + r32][column 32 nt + 8 q + 4 hh + e] of the wavefront tile
    f32x16 acc[4][2];
    bf16x4 braw[2][4];
    const bf16_t* __restrict__ bias = static_cast<const bf16_t*>(a.bias);
    auto load_bias = [&](int ti) {
        const int tile = t_begin + j_in + ti * per_x;
        const int tn = tile % n_nt;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                braw[nt][q] = bias ? *reinterpret_cast<const bf16x4*>(bias + tn * kBN + wn * 64 + nt * 32 + 8 * q + 4 * hh)
                                   : bf16x4{(bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f, (bf16_t)0.f};
    };
    auto init_acc = [&]() {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mt][nt][i] = (float)braw[nt][i >> 2][i & 3];
    };
    load_bias(0);
    init_acc();
    set_tile_ptrs(0);
    for (int s = 0; s < S - 1; ++s) {  // nk >= 8: all inside the first tile
#pragma unroll
        for (int j = 0; j < 4; ++j) request_one(j);
        request_done();
    }
    wait_loads_barrier<0>();  // steps 0 .. S-2 have landed
    bf16x8 wf0[2], af0[4], wf1[2], af1[4];
    read_frags(0, 0, wf0, af0);
    int slot = 0;  // slot of the step being computed

    // One k-step; every step of the kernel is this code.  After the barrier the next step is complete in LDS
    // and nobody reads the slot of the previous step any more, which the four requests then overwrite.
    // Nothing but the wait and the barrier stands between the last MFMA of a step and the first of the next:
    // a chain of branches there leaves the matrix pipeline idle, because all wavefronts are at the same place.
    auto step = [&](auto waited_before) {
        __builtin_amdgcn_sched_barrier(0);
        if (decltype(waited_before)::value) wait_lds_barrier();
        else wait_loads_barrier<(S - 3) * 4>();  // the requests of the two steps after the next may be in flight
        read_frags(slot, 1, wf1, af1);
        slot = slot == S - 1 ? 0 : slot + 1;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf0[nt], af0[mt], acc[mt][nt], 0, 0, 0);
            request_one(mt);
            __builtin_amdgcn_sched_barrier(0);
        }
        request_done();
        read_frags(slot, 0, wf0, af0);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf1[nt], af1[mt], acc[mt][nt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    for (int ti = 0; ti < my_tiles; ++ti) {
        // The requests of a tile's last S-1 steps are for the first steps of the next tile; after the last tile
        // they fetch that tile's own first steps again (never used), which keeps every step alike.
        const int ti_next = ti + 1 < my_tiles ? ti + 1 : ti;
        // the first S-2 steps were waited for at the end of the previous tile (or above)
#pragma unroll 1
        for (int ks = 0; ks < S - 2; ++ks) step(std::true_type{});
#pragma unroll 1
        for (int ks = S - 2; ks < nk; ++ks) {
            if (ks == nk - (S - 1)) set_tile_ptrs(ti_next);
            if (ks == nk - 1) load_bias(ti_next);  // long before the stores of the epilogue
            step(std::false_type{});
        }

        // ---- the tile is complete
        const int tile = t_begin + j_in + ti * per_x;
        const int tm = tile / n_nt, tn = tile - tm * n_nt;
        // Everything requested so far has landed (so the stores below may stay in flight over the next S-2
        // steps) and every wavefront is done with the slot of the last step, 4 KB of which each wavefront
        // now uses for the transpose.
        wait_loads_barrier<0>();
        // the next tile's bias has landed too: say so here, or the compiler waits for it after the stores
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int q = 0; q < 4; ++q) asm volatile("" : "+v"(braw[nt][q]));
        char* scr = lds + (size_t)(slot == 0 ? S - 1 : slot - 1) * kStageBytes + wave * 4096;
        // the wavefront's 64 columns are one K or V head (head_dim 64) or half of one (head_dim 128)
        const int n_wave = tn * kBN + wn * 64;
        const int which = n_wave >= a.d_model;
        const int col = n_wave - (which ? a.d_model : 0);
        const int h = col / a.head_dim, e0 = col % a.head_dim;
        const size_t dst_off = (size_t)h * a.t_cap * a.head_dim + e0;
        if constexpr (!FP8) {
            bf16_t* __restrict__ dst = static_cast<bf16_t*>(which ? a.vc : a.kc) + dst_off;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int c = 4 * nt + q;  // 16-byte chunk of the 128-byte row: columns 8 c + 4 hh .. + 3
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (bf16_t)acc[mt][nt][4 * q + e];
                        *reinterpret_cast<bf16x4*>(scr + r32 * 128 + ((c ^ (r32 & 7)) * 16) + hh * 8) = o;
                    }
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int row = p * 8 + (lane >> 3), c = lane & 7;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(scr + row * 128 + ((c ^ (row & 7)) * 16));
                    const int m = tm * kBM + wm * 128 + mt * 32 + row;
                    if (m < a.M) {
                        const size_t frame = a.out_row_map ? (size_t)a.out_row_map[m] : (size_t)m;
                        *reinterpret_cast<f32x4*>(dst + frame * a.head_dim + c * 8) = v;
                    }
                }
            }
        } else {
            // one byte per element: the wavefront's 32 x 64 block is 32 rows of 64 bytes = four 16-byte chunks
            unsigned char* __restrict__ dst = static_cast<unsigned char*>(which ? a.vc : a.kc) + dst_off;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        // columns 32 nt + 8 q + 4 hh .. + 3: chunk 2 nt + (q >> 1), byte 8 (q & 1) + 4 hh of it
                        const int c = 2 * nt + (q >> 1);
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = acc[mt][nt][4 * q + e];
                        store4_fp8(reinterpret_cast<unsigned char*>(scr) + r32 * 64 + ((c ^ (r32 & 3)) * 16) + (q & 1) * 8 + hh * 4, o);
                    }
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    const int row = p * 16 + (lane >> 2), c = lane & 3;
                    const f32x4 v = *reinterpret_cast<const f32x4*>(scr + row * 64 + ((c ^ (row & 3)) * 16));
                    const int m = tm * kBM + wm * 128 + mt * 32 + row;
                    if (m < a.M) {
                        const size_t frame = a.out_row_map ? (size_t)a.out_row_map[m] : (size_t)m;
                        *reinterpret_cast<f32x4*>(dst + frame * a.head_dim + c * 16) = v;
                    }
                }
            }
        }
        init_acc();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // nothing may land in LDS after the workgroup has ended
}

// bf16 operands, EPI_CROSSKV (caches in bf16 or E4M3 codes).  A (fragment order) must hold whole 256-row tiles; N % 256 == 0; K % 64 == 0, K >= 256;
// head_dim 64 or 128 and d_model a multiple of 64, so that a wavefront's 64 columns stay inside one head.
hipError_t launch_gemm_dma_crosskv(const GemmArgs& a, hipStream_t s) {
    if (a.M < 1 || a.N % kBN != 0 || a.K % 64 != 0 || a.K < 256 || a.d_model % 64 != 0 ||
        (a.head_dim != 64 && a.head_dim != 128) || a.N != 2 * a.d_model)
        return hipErrorInvalidValue;
    constexpr int kLds = kStages * kStageBytes;
    static DeviceOnce configured;
    hipError_t e = configured.run([&]() {
        hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_crosskv_kernel<false>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        if (e1 != hipSuccess) return e1;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_dma_crosskv_kernel<true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    });
    if (e != hipSuccess) return e;
    const int tiles = ((a.M + kBM - 1) / kBM) * (a.N / kBN);
    const int grid = persistent_grid(tiles);  // at most one workgroup per CU, whole rounds over the XCDs
    if (grid <= 0) return hipErrorInvalidDevice;
    if (a.kv_fp8) hipLaunchKernelGGL(gemm_dma_crosskv_kernel<true>, dim3(grid), dim3(512), kLds, s, a);
    else hipLaunchKernelGGL(gemm_dma_crosskv_kernel<false>, dim3(grid), dim3(512), kLds, s, a);
    return hipGetLastError();
}

}  // namespace aed
