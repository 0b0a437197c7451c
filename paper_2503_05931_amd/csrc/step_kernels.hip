// Small kernels of the decoder step: token + position embedding, the greedy
// sampler with its device-side sequence state, and state bookkeeping.
//
// All per-sequence state that changes from step to step (position, number of
// generated tokens, finished flag, next input token) lives in device memory and
// is advanced by the sampler, so one captured launch graph can be replayed for
// every step without touching its arguments.
#include <limits.h>

#include "common.h"
#include "kernels.h"

namespace aed {

template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(float* __restrict__ x, const T* __restrict__ tok_emb,
                                                    const T* __restrict__ pos_emb, StateArgs st, int d,
                                                    int max_positions, float emb_scale, ShadowArgs sh) {
    const int b = blockIdx.x, tid = threadIdx.x;
    int tok = st.cur_tok[b];
    tok = tok < 0 ? 0 : (tok >= st.vocab ? st.vocab - 1 : tok);
    int pos = st.seq_len[b];
    pos = pos < max_positions ? pos : max_positions - 1;
    const T* e = tok_emb + (size_t)tok * d;
    const T* p = pos_emb + (size_t)pos * d;
    const int i = tid * 4;  // d <= 1024: one 4-vector per thread
    const bool live = i < d;
    f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
    if (live) {
        const f32x4 ev = load4(e + i), pv = load4(p + i);
        o[0] = emb_scale * ev[0] + pv[0];
        o[1] = emb_scale * ev[1] + pv[1];
        o[2] = emb_scale * ev[2] + pv[2];
        o[3] = emb_scale * ev[3] + pv[3];
        store4(reinterpret_cast<float*>(reinterpret_cast<char*>(x) + frag_elem_off<4>(b, i, d)), o);
    }
    if (!sh.shadow) return;
    // row mean over the workgroup, then the shadow; tile statistics over the 4 threads of a 16-column tile
    __shared__ float wsum[4];
    float s = (o[0] + o[1]) + (o[2] + o[3]);
    const float t4 = s;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
    if ((tid & 63) == 0) wsum[tid >> 6] = s;
    __syncthreads();
    const float mean = sh.rms ? 0.f : (wsum[0] + wsum[1] + wsum[2] + wsum[3]) / (float)d;  // RMSNorm: no shift
    float ts = t4;
    ts += __shfl_xor(ts, 1);
    ts += __shfl_xor(ts, 2);
    const float tmean = ts * (1.f / 16.f);
    float q = (o[0] - tmean) * (o[0] - tmean) + (o[1] - tmean) * (o[1] - tmean) + (o[2] - tmean) * (o[2] - tmean) +
              (o[3] - tmean) * (o[3] - tmean);
    q += __shfl_xor(q, 1);
    q += __shfl_xor(q, 2);
    if (!live) return;
    store4(reinterpret_cast<T*>(static_cast<char*>(sh.shadow) + frag_elem_off<sizeof(T)>(b, i, d)), o - mean);
    if ((tid & 3) == 0) sh.stats[(size_t)(i >> 4) * sh.m_stride + b] = float2{tmean, q};
    if (tid == 0) sh.mu_hat[b] = mean;
}

hipError_t launch_embed(Dtype dt, float* x, const void* tok_emb, const void* pos_emb, const StateArgs& st,
                        int d_model, int max_positions, float emb_scale, const ShadowArgs& sa, hipStream_t s) {
    if (d_model > 1024 || d_model % 64 != 0) return hipErrorInvalidValue;
    if (dt == kBF16)
        hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(st.batch), dim3(256), 0, s, x,
                           static_cast<const bf16_t*>(tok_emb), static_cast<const bf16_t*>(pos_emb), st, d_model,
                           max_positions, emb_scale, sa);
    else
        hipLaunchKernelGGL(embed_kernel<float>, dim3(st.batch), dim3(256), 0, s, x,
                           static_cast<const float*>(tok_emb), static_cast<const float*>(pos_emb), st, d_model,
                           max_positions, emb_scale, sa);
    return hipGetLastError();
}

// argmax with the lowest index on ties: (value, index) pairs ordered by value
// descending, then index ascending.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ __launch_bounds__(256) void sample_kernel(const float* __restrict__ logits, StateArgs st, int greedy,
                                                     int* __restrict__ step_out) {
    const int b = blockIdx.x, tid = threadIdx.x;
    // everything the decision needs is requested at once: the state words and this thread's share of the row
    // (vocab is a multiple of 64: 4-vectors; up to four per thread in flight, then the rest of a long row)
    const int fin = greedy ? st.finished[b] : 0;
    const int pos = st.seq_len[b];
    const int n = greedy ? st.n_gen[b] : 0;
    const int lim = greedy ? st.limit[b] : INT_MAX;
    const float* row = logits + (size_t)b * st.vocab;
    f32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = tid * 4 + u * 1024;
        v[u] = i < st.vocab ? *reinterpret_cast<const f32x4*>(row + i) : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    }
    if (fin) return;
    if (greedy && pos + 1 < st.prompt_len) {  // still feeding the prompt: no token is emitted
        if (tid == 0) {
            st.cur_tok[b] = st.prompt[(size_t)b * st.prompt_stride + pos + 1];
            st.seq_len[b] = pos + 1;
        }
        return;
    }
    float bv = -INFINITY;
    int bi = INT_MAX;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = tid * 4 + u * 1024 + e;
            if (i < st.vocab && better(v[u][e], i, bv, bi)) { bv = v[u][e]; bi = i; }
        }
    for (int base = tid * 4 + 4096; base < st.vocab; base += 1024) {
        const f32x4 w = *reinterpret_cast<const f32x4*>(row + base);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (better(w[e], base + e, bv, bi)) { bv = w[e]; bi = base + e; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    __shared__ float sv[4];
    __shared__ int si[4];
    if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
    __syncthreads();
    if (tid != 0) return;
    for (int w = 1; w < 4; ++w)
        if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    int tok = bi == INT_MAX ? 0 : bi;
    if (!greedy) {
        if (step_out) step_out[b] = tok;
        st.cur_tok[b] = tok;
        st.seq_len[b] = pos + 1;
        return;
    }
    if (n + 1 >= lim) tok = st.eos_id;  // forced end at the per-sequence target length
    st.out_tokens[(size_t)b * st.out_stride + n] = tok;
    st.n_gen[b] = n + 1;
    st.cur_tok[b] = tok;
    st.seq_len[b] = pos + 1;
    if ((st.eos_id >= 0 && tok == st.eos_id) || n + 1 >= st.max_new) {
        st.finished[b] = 1;
        atomicAdd(st.n_finished, 1);
    }
}

hipError_t launch_sample(const float* logits, const StateArgs& st, int greedy, int* step_out, hipStream_t s) {
    hipLaunchKernelGGL(sample_kernel, dim3(st.batch), dim3(256), 0, s, logits, st, greedy, step_out);
    return hipGetLastError();
}

__global__ void reset_kernel(StateArgs st, const int* __restrict__ limits, int fill_out, int start_pos) {
    const int b = blockIdx.x;
    if (threadIdx.x == 0) {
        st.seq_len[b] = start_pos;
        st.n_gen[b] = 0;
        st.finished[b] = 0;
        st.cur_tok[b] = st.prompt ? st.prompt[(size_t)b * st.prompt_stride + start_pos] : 0;
        st.limit[b] = limits ? limits[b] : INT_MAX;
        if (b == 0) *st.n_finished = 0;
    }
    if (fill_out)
        for (int t = threadIdx.x; t < st.max_new; t += blockDim.x) st.out_tokens[(size_t)b * st.out_stride + t] = st.pad_id;
}

hipError_t launch_reset(const StateArgs& st, const int* limits_dev, int fill_out, int start_pos, hipStream_t s) {
    hipLaunchKernelGGL(reset_kernel, dim3(st.batch), dim3(64), 0, s, st, limits_dev, fill_out, start_pos);
    return hipGetLastError();
}

__global__ void set_tokens_kernel(int* __restrict__ cur_tok, const int* __restrict__ src, int stride, int batch) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) cur_tok[b] = src[(size_t)b * stride];
}

hipError_t launch_set_tokens(int* cur_tok, const int* src, int stride, int batch, hipStream_t s) {
    hipLaunchKernelGGL(set_tokens_kernel, dim3((batch + 255) / 256), dim3(256), 0, s, cur_tok, src, stride, batch);
    return hipGetLastError();
}

__global__ void copy_out_kernel(StateArgs st, int* __restrict__ dst_tokens, int* __restrict__ dst_lens) {
    const int b = blockIdx.x;
    for (int t = threadIdx.x; t < st.max_new; t += blockDim.x)
        dst_tokens[(size_t)b * st.max_new + t] = st.out_tokens[(size_t)b * st.out_stride + t];
    if (threadIdx.x == 0) dst_lens[b] = st.n_gen[b];
}

hipError_t launch_copy_out(const StateArgs& st, int* dst_tokens, int* dst_lens, hipStream_t s) {
    hipLaunchKernelGGL(copy_out_kernel, dim3(st.batch), dim3(64), 0, s, st, dst_tokens, dst_lens);
    return hipGetLastError();
}

__global__ void turn_over_slots_kernel(StateArgs st, const int* __restrict__ slots, const int* __restrict__ old_reqs,
                                       const int* __restrict__ new_reqs, const int* __restrict__ limits,
                                       const int* __restrict__ all_prompts, int* __restrict__ dst_tokens,
                                       int* __restrict__ dst_lens) {
    const int i = blockIdx.x, tid = threadIdx.x;
    const int b = slots[i], old = old_reqs[i], req = new_reqs[i];
    if (old >= 0) {
        const int n = st.n_gen[b];
        for (int t = tid; t < st.max_new; t += blockDim.x)
            dst_tokens[(size_t)old * st.max_new + t] = t < n ? st.out_tokens[(size_t)b * st.out_stride + t] : st.pad_id;
        if (tid == 0) dst_lens[old] = n;
    }
    __syncthreads();  // n_gen is read above and cleared below
    if (req >= 0)
        for (int p = tid; p < st.prompt_len; p += blockDim.x)
            st.prompt[(size_t)b * st.prompt_stride + p] = all_prompts[(size_t)req * st.prompt_len + p];
    if (tid == 0) {
        st.seq_len[b] = 0;
        st.n_gen[b] = 0;
        st.finished[b] = req < 0;
        st.cur_tok[b] = req >= 0 ? all_prompts[(size_t)req * st.prompt_len] : 0;
        st.limit[b] = req >= 0 ? limits[i] : INT_MAX;
    }
}

hipError_t launch_turn_over_slots(const StateArgs& st, const int* slots, const int* old_reqs, const int* new_reqs,
                                  const int* limits, int n, const int* all_prompts, int* dst_tokens, int* dst_lens,
                                  hipStream_t s) {
    if (n < 1) return hipSuccess;
    hipLaunchKernelGGL(turn_over_slots_kernel, dim3(n), dim3(64), 0, s, st, slots, old_reqs, new_reqs, limits,
                       all_prompts, dst_tokens, dst_lens);
    return hipGetLastError();
}

__global__ void assign_pages_kernel(int* __restrict__ page_table, int max_pages, int blk, int first_page, int batch) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) page_table[(size_t)b * max_pages + blk] = first_page + b;
}

hipError_t launch_assign_pages(int* page_table, int max_pages, int blk, int first_page, int batch, hipStream_t s) {
    if (batch < 1 || blk < 0 || blk >= max_pages) return hipErrorInvalidValue;
    hipLaunchKernelGGL(assign_pages_kernel, dim3((batch + 255) / 256), dim3(256), 0, s, page_table, max_pages, blk,
                       first_page, batch);
    return hipGetLastError();
}

__global__ void fill_zero_kernel(int* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_fill_zero(int* p, int n, hipStream_t s) {
    if (n < 1) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

__global__ void prepare_timing_kernel(StateArgs st, int max_pos) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= st.batch) return;
    st.finished[b] = 0;
    const int p = st.seq_len[b];
    st.seq_len[b] = p < 0 ? 0 : (p > max_pos ? max_pos : p);
}

hipError_t launch_prepare_timing(const StateArgs& st, int max_pos, hipStream_t s) {
    hipLaunchKernelGGL(prepare_timing_kernel, dim3((st.batch + 255) / 256), dim3(256), 0, s, st, max_pos);
    return hipGetLastError();
}

}  // namespace aed
