// Device-side helpers shared by the gfx950 kernels of the AED decoder library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace aed {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

// ---- N consecutive elements of T from a pointer aligned to N*sizeof(T) (max 16 B per load) ----
template <int N> __device__ __forceinline__ void load_f32(const float* p, float* out) {
    static_assert(N % 4 == 0, "float runs are multiples of 4");
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
        f32x4 v = reinterpret_cast<const f32x4*>(p)[i];
        out[4 * i + 0] = v[0]; out[4 * i + 1] = v[1]; out[4 * i + 2] = v[2]; out[4 * i + 3] = v[3];
    }
}
template <int N> __device__ __forceinline__ void load_f32(const bf16_t* p, float* out) {
    static_assert(N == 4 || N % 8 == 0, "bf16 runs are 4 or multiples of 8");
    if constexpr (N == 4) {
        bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = (float)v[i];
    } else {
#pragma unroll
        for (int j = 0; j < N / 8; ++j) {
            bf16x8 v = reinterpret_cast<const bf16x8*>(p)[j];
#pragma unroll
            for (int i = 0; i < 8; ++i) out[8 * j + i] = (float)v[i];
        }
    }
}

// ---- store 4 consecutive values as T ----
__device__ __forceinline__ void store4(float* p, f32x4 v) { *reinterpret_cast<f32x4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, f32x4 v) {
    bf16x4 o;
    o[0] = (bf16_t)v[0]; o[1] = (bf16_t)v[1]; o[2] = (bf16_t)v[2]; o[3] = (bf16_t)v[3];
    *reinterpret_cast<bf16x4*>(p) = o;
}
__device__ __forceinline__ f32x4 load4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ f32x4 load4(const bf16_t* p) {
    bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
    f32x4 o = {(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
    return o;
}

// ---- fragment layout ----
// A [rows, K] matrix whose rows feed 16x16 MFMA tiles is kept in "fragment
// order": 16-row x 64-k blocks, and inside a block the 16 consecutive k values
// that lane l = 16 * ((k % 64) / 16) + row % 16 holds for the MFMA, cut into
// 16-byte pieces, piece-major: block[(piece j)][lane l][16 bytes].  A wavefront
// then loads piece j of a block with one fully coalesced 1 KB instruction.
// ES = element size in bytes (2: bf16, 4: fp32); a lane's 16 elements are ES pieces.
template <int ES> __host__ __device__ __forceinline__ size_t frag_block_bytes() { return (size_t)ES * 1024; }
// byte offset of block (row tile rt, k block kb)
template <int ES> __host__ __device__ __forceinline__ size_t frag_block_off(int rt, int kb, int K) {
    return ((size_t)rt * (K >> 6) + kb) * ES * 1024;
}
// byte offset of element (row, k)
template <int ES> __host__ __device__ __forceinline__ size_t frag_elem_off(int row, int k, int K) {
    constexpr int EPP = 16 / ES;  // elements per 16-byte piece
    const int e = k & 15, lane = ((k & 63) >> 4) * 16 + (row & 15);
    return frag_block_off<ES>(row >> 4, k >> 6, K) + ((size_t)(e / EPP) * 64 + lane) * 16 + (size_t)(e % EPP) * ES;
}

// ---- sum over the 16 lanes of a DPP row (lanes 16k..16k+15); every lane gets the total ----
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    v += dpp_mov<0x140>(v);  // row_mirror
    return v;
}
// ---- sum / max over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48) ----
__device__ __forceinline__ float rows4_sum(float v) {
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}
__device__ __forceinline__ float rows4_max(float v) {
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

// Folded normalisation (kernels.h, PRO_LNS): from a row's mean mu and its sum of squared deviations m2 over K
// elements, the factor the product is scaled with and the mean that counts.  LayerNorm: 1 / sqrt(m2 / K + eps) and mu.
// RMSNorm: the mean is not subtracted, so the factor is 1 / sqrt(sum of squares / K + eps) with
// sum of squares = m2 + K mu^2, and the row counts as having mean 0 (its shadow was written with shift 0).
__device__ __forceinline__ float fold_norm(int rms, float K, float eps, float m2, float& mu) {
    if (rms) {
        const float r = 1.0f / sqrtf((m2 + K * mu * mu) / K + eps);
        mu = 0.f;
        return r;
    }
    return 1.0f / sqrtf(m2 / K + eps);
}

// sum over the 64 lanes of a wavefront; every lane gets the total
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

}  // namespace aed
