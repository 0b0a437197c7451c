// MFMA fragments in fragment order and the GEMM epilogues, shared by the streaming
// (gemm_decode.hip) and the LDS-tiled (gemm_tiled.hip) kernels.
#pragma once

#include "common.h"
#include "kernels.h"

namespace aed {

template <typename T> struct Frag16;
template <> struct Frag16<bf16_t> { bf16x8 lo, hi; };
template <> struct Frag16<float> { float v[16]; };

// a lane's 16 k-values of one block in fragment order: pieces at stride 1 KB
__device__ __forceinline__ Frag16<bf16_t> load_frag(const bf16_t* blk, int lane) {
    Frag16<bf16_t> f;
    const bf16x8* p = reinterpret_cast<const bf16x8*>(blk) + lane;
    f.lo = p[0];
    f.hi = p[64];
    return f;
}
__device__ __forceinline__ Frag16<bf16_t> load_frag_nt(const bf16_t* blk, int lane) {
    Frag16<bf16_t> f;
    const bf16x8* p = reinterpret_cast<const bf16x8*>(blk) + lane;
    f.lo = __builtin_nontemporal_load(p);
    f.hi = __builtin_nontemporal_load(p + 64);
    return f;
}
__device__ __forceinline__ Frag16<float> load_frag(const float* blk, int lane) {
    Frag16<float> f;
    const f32x4* p = reinterpret_cast<const f32x4*>(blk) + lane;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x4 v = p[64 * j];
        f.v[4 * j + 0] = v[0]; f.v[4 * j + 1] = v[1]; f.v[4 * j + 2] = v[2]; f.v[4 * j + 3] = v[3];
    }
    return f;
}
__device__ __forceinline__ Frag16<float> load_frag_nt(const float* blk, int lane) { return load_frag(blk, lane); }
__device__ __forceinline__ void store_frag(bf16_t* blk, int lane, const Frag16<bf16_t>& f) {
    bf16x8* p = reinterpret_cast<bf16x8*>(blk) + lane;
    p[0] = f.lo;
    p[64] = f.hi;
}
__device__ __forceinline__ void store_frag(float* blk, int lane, const Frag16<float>& f) {
    f32x4* p = reinterpret_cast<f32x4*>(blk) + lane;
#pragma unroll
    for (int j = 0; j < 4; ++j) p[64 * j] = f32x4{f.v[4 * j], f.v[4 * j + 1], f.v[4 * j + 2], f.v[4 * j + 3]};
}
// row-major source (LayerNorm gain/shift vectors): 16 consecutive elements
__device__ __forceinline__ Frag16<bf16_t> load_frag_rm(const bf16_t* p) {
    Frag16<bf16_t> f;
    f.lo = reinterpret_cast<const bf16x8*>(p)[0];
    f.hi = reinterpret_cast<const bf16x8*>(p)[1];
    return f;
}
__device__ __forceinline__ Frag16<float> load_frag_rm(const float* p) {
    Frag16<float> f;
    load_f32<16>(p, f.v);
    return f;
}
__device__ __forceinline__ void zero_frag(Frag16<bf16_t>& f) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { f.lo[i] = (bf16_t)0.f; f.hi[i] = (bf16_t)0.f; }
}
__device__ __forceinline__ void zero_frag(Frag16<float>& f) {
#pragma unroll
    for (int i = 0; i < 16; ++i) f.v[i] = 0.f;
}
__device__ __forceinline__ void pack_frag(const float* y, Frag16<bf16_t>& f) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { f.lo[i] = (bf16_t)y[i]; f.hi[i] = (bf16_t)y[8 + i]; }
}
__device__ __forceinline__ void pack_frag(const float* y, Frag16<float>& f) {
#pragma unroll
    for (int i = 0; i < 16; ++i) f.v[i] = y[i];
}
__device__ __forceinline__ void unpack_frag(const Frag16<bf16_t>& f, float* y) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { y[i] = (float)f.lo[i]; y[8 + i] = (float)f.hi[i]; }
}
__device__ __forceinline__ void unpack_frag(const Frag16<float>& f, float* y) {
#pragma unroll
    for (int i = 0; i < 16; ++i) y[i] = f.v[i];
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

// Four consecutive cache elements as 8-bit E4M3 codes (OCP 8-bit floating point: bias 7, no infinities, largest
// magnitude 448): round to nearest even, done by the conversion instruction; saturation is done here.
__device__ __forceinline__ void store4_fp8(unsigned char* p, f32x4 s) {
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i] = fminf(fmaxf(s[i], -448.f), 448.f);
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(s[0], s[1], 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(s[2], s[3], w, true);
    *reinterpret_cast<int*>(p) = w;
}

// One lane's four consecutive outputs C[m][n .. n+3] (bias already added) go where the epilogue says.
// res: the residual read earlier from the same place (EPI_RESID only).
template <typename T, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, int m, int n, f32x4 s, f32x4 res) {
    constexpr int ES = sizeof(T);
    if constexpr (EPI == EPI_RESID) {
        *reinterpret_cast<f32x4*>(static_cast<char*>(a.out) + frag_elem_off<4>(m, n, a.N)) = res + s;
    } else if constexpr (EPI == EPI_F32) {
        store4(static_cast<float*>(a.out) + (size_t)m * a.N + n, s);
    } else if constexpr (EPI == EPI_RELU_T) {
        s[0] = fmaxf(s[0], 0.f); s[1] = fmaxf(s[1], 0.f); s[2] = fmaxf(s[2], 0.f); s[3] = fmaxf(s[3], 0.f);
        store4(reinterpret_cast<T*>(static_cast<char*>(a.out) + frag_elem_off<ES>(m, n, a.N)), s);
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
            const size_t at = (((size_t)page * a.n_heads + h) * kPage + (pos & 15)) * a.head_dim + e;
            if (a.kv_fp8) store4_fp8(static_cast<unsigned char*>(which ? a.v_pool : a.k_pool) + at, s);
            else store4(static_cast<T*>(which ? a.v_pool : a.k_pool) + at, s);
        }
    } else {  // EPI_CROSSKV
        const int d = a.d_model;
        const int which = n >= d;
        const int c = n - (which ? d : 0);
        const int h = c / a.head_dim, e = c % a.head_dim;
        const size_t frame = a.out_row_map ? (size_t)a.out_row_map[m] : (size_t)m;
        const size_t at = ((size_t)h * a.t_cap + frame) * a.head_dim + e;
        if (a.kv_fp8) store4_fp8(static_cast<unsigned char*>(which ? a.vc : a.kc) + at, s);
        else store4(static_cast<T*>(which ? a.vc : a.kc) + at, s);
    }
}

}  // namespace aed
