// Decode attention for one query row per (sequence, head) on gfx950:
// causal self-attention over the paged KV cache and cross-attention over the
// ragged (unpadded) encoder keys/values.  One query row means ~1 flop per byte,
// so the kernel is a pure HBM stream: the dot products and the softmax run on
// the vector ALUs, no MFMA.
//
// Work item = (head, sequence, chunk of keys).  Self-attention: the grid's z
// axis counts chunks and items beyond a sequence's current length exit at
// once.  Cross-attention: items come from a list built on the host from the
// true encoder lengths, so neither padding frames nor empty chunks exist.
//
// Inside a workgroup (4 wavefronts) the chunk is cut into 16-key blocks
// (= one page of the self-attention cache), wavefront w takes blocks w, w+4,..
// A wavefront reads a block as 4 keys per load instruction: lane (r, g) loads
// 16 bytes (or 8) -- the slice r of head_dim -- of key 4 i + g, i = 0..3, so
// each instruction covers 4 whole rows (1 KB for bf16 head_dim 128).  The dot
// products are reduced over the 16 lanes of a DPP row, the running softmax
// (max, sum, weighted values) is kept per wavefront in base-2 exponent form,
// the four wavefronts are merged through LDS.  Sequences of this workload are
// short (at most 500 encoder frames, a few hundred decoded tokens), so one
// workgroup per (sequence, head) is the normal case; only when the batch is too
// small to occupy the GPU are long sequences cut into chunks, whose partial
// (max, sum, values) go to a scratch buffer and are combined in chunk order by
// a small second kernel (a kernel boundary is far cheaper here than
// device-scope fences inside the kernel, which write back and invalidate L2).
#include "common.h"
#include "kernels.h"

namespace aed {

template <typename T, int N> __device__ __forceinline__ void load_row(const T* p, float* out) {
    load_f32<N>(p, out);
}

template <typename T, int DH, bool SELF>
__global__ __launch_bounds__(256) void attn_decode_kernel(AttnArgs a) {
    constexpr int EPL = DH / 16;  // head_dim elements per lane
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int h = blockIdx.x, H = a.n_heads;

    int b, start, n, chunk_idx, n_chunks;
    if constexpr (SELF) {
        b = blockIdx.y;
        if (a.finished[b]) return;
        const int total = a.seq_len[b] + 1;
        n_chunks = (total + a.chunk - 1) / a.chunk;
        chunk_idx = blockIdx.z;
        if (chunk_idx >= n_chunks) return;
        start = chunk_idx * a.chunk;
        n = min(a.chunk, total - start);
    } else {
        const int4 it = a.items[blockIdx.y];
        b = it.x;
        if (a.finished[b]) return;
        start = it.y;
        n = it.z;
        chunk_idx = it.w & 0xFFFF;
        n_chunks = it.w >> 16;
    }

    const T* __restrict__ Kb = static_cast<const T*>(a.K);
    const T* __restrict__ Vb = static_cast<const T*>(a.V);
    size_t cross_base = 0;
    if constexpr (!SELF) cross_base = ((size_t)h * a.t_cap + a.enc_off[b] + start) * DH;

    float q[EPL];
    {
        const float* qp = a.q + (size_t)b * H * DH + h * DH + r * EPL;
        load_f32<EPL>(qp, q);
#pragma unroll
        for (int e = 0; e < EPL; ++e) q[e] *= a.scale_log2e;
    }

    float m_run = -INFINITY, l_run = 0.f;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    for (int kb = wave; kb * 16 < n; kb += 4) {
        size_t blk_base;
        if constexpr (SELF) {
            const int page = a.page_table[(size_t)b * a.max_pages + (start >> 4) + kb];
            blk_base = ((size_t)page * H + h) * kPage * DH;
        } else {
            blk_base = cross_base + (size_t)kb * 16 * DH;
        }
        const int last = n - 1 - kb * 16;  // last valid key of this block (>= 0)
        float kf[4][EPL], vf[4][EPL];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = i * 4 + g;
            const int jc = j < last ? j : last;  // clamp: never read past the valid keys
            load_row<T, EPL>(Kb + blk_base + (size_t)jc * DH + r * EPL, kf[i]);
            load_row<T, EPL>(Vb + blk_base + (size_t)jc * DH + r * EPL, vf[i]);
        }
        float s[4];
        float m_blk = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(q[e], kf[i][e], d);
            d = row16_sum(d);
            s[i] = (i * 4 + g <= last) ? d : -INFINITY;
            m_blk = fmaxf(m_blk, s[i]);
        }
        m_blk = rows4_max(m_blk);
        const float m_new = fmaxf(m_run, m_blk);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // first block: exp2(-inf) = 0
        l_run *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float p = __builtin_amdgcn_exp2f(s[i] - m_new);
            l_run += p;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[i][e], acc[e]);
        }
        m_run = m_new;
    }
    // lanes of different rows g hold different keys: add them up
    l_run = rows4_sum(l_run);
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = rows4_sum(acc[e]);

    __shared__ float sm_acc[4][DH];
    __shared__ float sm_m[4], sm_l[4];
    if (g == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm_acc[wave][r * EPL + e] = acc[e];
    }
    if (lane == 0) { sm_m[wave] = m_run; sm_l[wave] = l_run; }
    __syncthreads();

    // merge the four wavefronts (a wavefront without keys has m = -inf, l = 0, acc = 0)
    float m_tot = fmaxf(fmaxf(sm_m[0], sm_m[1]), fmaxf(sm_m[2], sm_m[3]));
    float l_tot = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float f = __builtin_amdgcn_exp2f(sm_m[w] - m_tot);
        l_tot += sm_l[w] * f;
        if (tid < DH) o += sm_acc[w][tid] * f;
    }
    if (n_chunks == 1) {  // the output feeds the next GEMM: fragment order
        if (tid < DH)
            *reinterpret_cast<T*>(static_cast<char*>(a.out) + frag_elem_off<sizeof(T)>(b, h * DH + tid, H * DH)) =
                from_f32<T>(o / l_tot);
        return;
    }

    // ---- several chunks: publish the partial; attn_merge_kernel combines them in chunk order ----
    float* __restrict__ my = a.part + ((size_t)(b * H + h) * a.max_chunks + chunk_idx) * (DH + 2);
    if (tid < DH) my[tid] = o;
    if (tid == 0) { my[DH] = m_tot; my[DH + 1] = l_tot; }
}

// Combines the partial results of the chunks of one (sequence, head) in chunk
// order (so the result does not depend on scheduling) -- launched only when a
// launch shape cuts some sequence into more than one chunk.
template <typename T, int DH, bool SELF>
__global__ __launch_bounds__(DH) void attn_merge_kernel(AttnArgs a) {
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, H = a.n_heads;
    if (a.finished[b]) return;
    int total;
    if constexpr (SELF) total = a.seq_len[b] + 1;
    else total = a.enc_off[b + 1] - a.enc_off[b];
    const int n_chunks = (total + a.chunk - 1) / a.chunk;
    if (n_chunks <= 1) return;  // the attention kernel wrote the final result itself
    const float* __restrict__ base = a.part + (size_t)(b * H + h) * a.max_chunks * (DH + 2);
    float M = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, base[(size_t)c * (DH + 2) + DH]);
    float L = 0.f, O = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float* pc = base + (size_t)c * (DH + 2);
        const float f = __builtin_amdgcn_exp2f(pc[DH] - M);
        L += pc[DH + 1] * f;
        O += pc[tid] * f;
    }
    *reinterpret_cast<T*>(static_cast<char*>(a.out) + frag_elem_off<sizeof(T)>(b, h * DH + tid, H * DH)) =
        from_f32<T>(O / L);
}

template <typename T, bool SELF>
static hipError_t launch_dh(const AttnArgs& a, dim3 grid, bool merge, hipStream_t s) {
    dim3 mgrid(a.n_heads, a.batch);
    if (a.head_dim == 128) {
        hipLaunchKernelGGL((attn_decode_kernel<T, 128, SELF>), grid, dim3(256), 0, s, a);
        if (merge) hipLaunchKernelGGL((attn_merge_kernel<T, 128, SELF>), mgrid, dim3(128), 0, s, a);
    } else if (a.head_dim == 64) {
        hipLaunchKernelGGL((attn_decode_kernel<T, 64, SELF>), grid, dim3(256), 0, s, a);
        if (merge) hipLaunchKernelGGL((attn_merge_kernel<T, 64, SELF>), mgrid, dim3(64), 0, s, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_attn_self(Dtype dt, const AttnArgs& a, hipStream_t s) {
    if (a.chunk < 64 || a.chunk % 64 != 0 || a.n_chunks_max < 1 || a.n_chunks_max > a.max_chunks)
        return hipErrorInvalidValue;
    dim3 grid(a.n_heads, a.batch, a.n_chunks_max);
    const bool merge = a.n_chunks_max > 1;
    return dt == kBF16 ? launch_dh<bf16_t, true>(a, grid, merge, s) : launch_dh<float, true>(a, grid, merge, s);
}

hipError_t launch_attn_cross(Dtype dt, const AttnArgs& a, hipStream_t s) {
    if (a.n_items < 1 || a.chunk < 64 || a.chunk % 64 != 0) return hipErrorInvalidValue;
    dim3 grid(a.n_heads, a.n_items);
    const bool merge = a.n_items > a.batch;
    return dt == kBF16 ? launch_dh<bf16_t, false>(a, grid, merge, s) : launch_dh<float, false>(a, grid, merge, s);
}

}  // namespace aed
