// Decode attention for one query row per (sequence, head) on gfx950:
// causal self-attention over the paged KV cache and cross-attention over the
// ragged (unpadded) encoder keys/values.  One query row means ~1 flop per byte,
// so the kernel is a pure HBM stream: the dot products and the softmax run on
// the vector ALUs, no MFMA.
//
// Work item = (head, sequence, chunk of keys).  Self-attention: the grid's z
// axis counts chunks and items beyond a sequence's current length exit at
// once.  Cross-attention: items come from a list built on the host from the
// true encoder lengths, longest first, so neither padding frames nor empty
// chunks exist and the longest sequences are scheduled first.
//
// Inside a workgroup (NW = 4 or 8 wavefronts) the chunk is cut into 16-key blocks
// (= one page of the self-attention cache), wavefront w takes blocks w, w+NW,..
// and keeps two blocks in flight (the next block is fetched while the current
// one is consumed).
// A wavefront reads a block as 4 keys per load instruction: lane (r, g) loads
// 16 bytes (or 8) -- the slice r of head_dim -- of key 4 i + g, i = 0..3, so
// each instruction covers 4 whole rows (1 KB for bf16 head_dim 128).  When the
// caches hold 8-bit E4M3 codes a key row is half as long: 8 lanes share a key
// and an instruction covers 8 keys, so the loads keep their 16 bytes per lane.
// The dot products are reduced over the lanes of a key, the running softmax
// (max, sum, weighted values) is kept per wavefront in base-2 exponent form,
// the wavefronts are merged through LDS.  Sequences of this workload are short
// (at most 500 encoder frames, a few hundred decoded tokens), so one workgroup
// per (sequence, head) is the normal case.  When the batch is too small to
// occupy the GPU, long sequences are cut into chunks of keys handled by
// different workgroups, and the last workgroup of a (sequence, head) to finish
// combines the partial (max, sum, values) triples in chunk order.
#include "common.h"
#include "kernels.h"

namespace aed {

// One key row slice as it sits in memory (EPL elements of T), kept raw in
// registers until it is used so that two blocks can be in flight per wavefront.
// Keys and values are read once per launch and not again before everything else
// of the step has gone by, so they are loaded with the non-temporal hint: they
// then do not push the weights and activations out of the caches (measured: the
// 4-layer decoder at batch 256, whose weights fit the memory-side cache, decodes
// 15 % more tokens per second; cross-attention at batch 1024 streams 6.5 TB/s
// instead of 6.0).
template <typename T, int EPL> struct RawRow;
template <> struct RawRow<bf16_t, 8> { bf16x8 v; };
template <> struct RawRow<bf16_t, 4> { bf16x4 v; };
template <> struct RawRow<float, 8> { f32x4 v[2]; };
template <> struct RawRow<float, 4> { f32x4 v[1]; };
typedef unsigned char fp8_t;  // one E4M3 code (OCP 8-bit floating point; the conversion instructions' format)
template <> struct RawRow<fp8_t, 16> { u32x4 v; };
template <> struct RawRow<fp8_t, 8> { u32x2 v; };

template <int EPL> __device__ __forceinline__ RawRow<bf16_t, EPL> load_raw(const bf16_t* p) {
    RawRow<bf16_t, EPL> r;
    r.v = __builtin_nontemporal_load(reinterpret_cast<const decltype(r.v)*>(p));
    return r;
}
template <int EPL> __device__ __forceinline__ RawRow<float, EPL> load_raw(const float* p) {
    RawRow<float, EPL> r;
#pragma unroll
    for (int i = 0; i < EPL / 4; ++i) r.v[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p) + i);
    return r;
}
template <int EPL> __device__ __forceinline__ RawRow<fp8_t, EPL> load_raw(const fp8_t* p) {
    RawRow<fp8_t, EPL> r;
    r.v = __builtin_nontemporal_load(reinterpret_cast<const decltype(r.v)*>(p));
    return r;
}
// The row slice as floats.  bf16 / float rows are converted element by element where they are used (the
// compiler keeps them packed until then); E4M3 codes come out of the conversion instruction two at a time.
template <int EPL> struct Unpacked { float y[EPL]; __device__ __forceinline__ float operator[](int e) const { return y[e]; } };
template <int EPL> __device__ __forceinline__ const RawRow<bf16_t, EPL>& unpack(const RawRow<bf16_t, EPL>& r) { return r; }
template <int EPL> __device__ __forceinline__ const RawRow<float, EPL>& unpack(const RawRow<float, EPL>& r) { return r; }
template <int EPL> __device__ __forceinline__ Unpacked<EPL> unpack(const RawRow<fp8_t, EPL>& r) {
    Unpacked<EPL> u;
#pragma unroll
    for (int w = 0; w < EPL / 4; ++w) {  // bytes 0,1 of a word, then bytes 2,3
        const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.v[w], false);
        const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.v[w], true);
        u.y[4 * w] = lo[0]; u.y[4 * w + 1] = lo[1]; u.y[4 * w + 2] = hi[0]; u.y[4 * w + 3] = hi[1];
    }
    return u;
}
template <int EPL> __device__ __forceinline__ float raw_at(const RawRow<bf16_t, EPL>& r, int e) { return (float)r.v[e]; }
template <int EPL> __device__ __forceinline__ float raw_at(const RawRow<float, EPL>& r, int e) { return r.v[e >> 2][e & 3]; }
template <int EPL> __device__ __forceinline__ float raw_at(const Unpacked<EPL>& u, int e) { return u.y[e]; }

// sum over the LPK lanes that share a key (LPK consecutive lanes of a DPP row)
template <int LPK> __device__ __forceinline__ float key_sum(float v) {
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    if constexpr (LPK == 16) v += dpp_mov<0x140>(v);  // row_mirror
    return v;
}
// sum / max over the 64 / LPK keys that the lanes of a wavefront hold side by side
template <int LPK> __device__ __forceinline__ float keys_sum(float v) {
    if constexpr (LPK == 8) v += dpp_mov<0x128>(v);  // row_ror 8: lane l ^ 8
    return rows4_sum(v);
}
template <int LPK> __device__ __forceinline__ float keys_max(float v) {
    if constexpr (LPK == 8) v = fmaxf(v, dpp_mov<0x128>(v));
    return rows4_max(v);
}

// T: type of the output rows (and of the caches unless KV says otherwise); KV: what the caches hold;
// LPK: lanes that share a key row.
// (bfloat16 and 8-bit caches: at least four wavefronts per SIMD, i.e. at most 128 registers, so that two workgroups of
// eight wavefronts share a CU -- with one, half as many bytes are in flight and the launch takes a quarter longer)
template <typename T, typename KV, int LPK, int DH, bool SELF, int NW>
__global__ __launch_bounds__(64 * NW, sizeof(KV) <= 2 ? 4 : 1) void attn_decode_kernel(AttnArgs a) {
    constexpr int EPL = DH / LPK;   // head_dim elements per lane
    constexpr int KPI = 64 / LPK;   // keys per load instruction
    constexpr int NI = 16 / KPI;    // load instructions per 16-key block
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane % LPK, g = lane / LPK;
    const int h = blockIdx.x, H = a.n_heads;

    // Work item.  Cross-attention: from the host-built list (longest first, so the long sequences
    // start early and the short ones fill the tail); the item carries everything needed to address
    // the keys, so the finished flag, the query and the first key blocks are all fetched in the same
    // round trip.  Self-attention: blockIdx.y is the sequence, blockIdx.z the chunk.
    int b, start, n, chunk_idx, n_chunks, row0 = 0, fin;
    int first_page = 0;  // self-attention: page of this wavefront's first block, fetched with the scalars
    if constexpr (SELF) {
        b = blockIdx.y;
        fin = a.finished[b];
        const int total = a.seq_len[b] + 1;
        {
            const int blk = min((int)(blockIdx.z * a.chunk >> 4) + wave, a.max_pages - 1);
            first_page = a.page_table[(size_t)b * a.max_pages + blk];
        }
        if (fin) return;
        n_chunks = (total + a.chunk - 1) / a.chunk;
        chunk_idx = blockIdx.z;
        if (chunk_idx >= n_chunks) return;
        start = chunk_idx * a.chunk;
        n = min(a.chunk, total - start);
    } else {
        const int4 it = a.items[blockIdx.y];
        b = it.x;
        start = it.y & 0xFFFF;
        chunk_idx = it.y >> 16;
        n = it.z & 0xFFFF;
        n_chunks = it.z >> 16;
        row0 = it.w + start;  // first frame of this chunk in the packed layout
        fin = a.finished[b];  // tested after the first loads have been issued
    }

    const KV* __restrict__ Kb = static_cast<const KV*>(a.K);
    const KV* __restrict__ Vb = static_cast<const KV*>(a.V);
    size_t cross_base = 0;
    if constexpr (!SELF) cross_base = ((size_t)h * a.t_cap + row0) * DH;
    const int n_blocks = (n + 15) >> 4;
    const int* __restrict__ pages = SELF ? a.page_table + (size_t)b * a.max_pages + (start >> 4) : nullptr;

    // the query row slice and, behind merged products, what finishes it: requested here, before the first key
    // blocks, and used after them, so that the keys and values do not wait for this round trip
    float q[EPL];
    float qc1[EPL], qc2[EPL];
    float2 q_st = float2{0.f, 0.f};
    float q_muh = 0.f;
    bool q_fix = false;
    {
        const size_t qo = (size_t)b * H * DH + h * DH + r * EPL;
        load_f32<EPL>(a.q + qo, q);
        if constexpr (!SELF) {
            q_fix = a.q_stats != nullptr;
            // Only the first wavefront fetches what finishes the query (the row's tile statistics -- at most 64, one
            // lane each, 64 separate lines -- and the two vectors); it hands the others rstd' and the vector
            // c2 - rstd' (mu' - mu_hat) c1 through LDS.  Eight wavefronts fetching the same things cost 0.8 us of
            // load issue in front of the first key blocks.
            if (q_fix && wave == 0) {
                const int n0 = h * DH + r * EPL;
                load_f32<EPL>(a.q_c1 + n0, qc1);
                load_f32<EPL>(a.q_c2 + n0, qc2);
                if (lane < a.q_stat_tiles) q_st = a.q_stats[(size_t)lane * a.q_m_stride + b];
                q_muh = a.q_mu_hat[b];
            }
        }
    }
    typedef RawRow<KV, EPL> Raw;
    // element offset of this lane's slice of key (KPI i + g) of block kb (clamped to the valid keys)
    auto fetch = [&](int kb, Raw* kf, Raw* vf) {
        size_t blk_base;
        if constexpr (SELF) blk_base = ((size_t)(kb == wave ? first_page : pages[kb]) * H + h) * kPage * DH;
        else blk_base = cross_base + (size_t)kb * 16 * DH;
        const int last = n - 1 - kb * 16;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int j = i * KPI + g;
            const int jc = j < last ? j : last;  // never read past the valid keys
            const size_t off = blk_base + (size_t)jc * DH + r * EPL;
            kf[i] = load_raw<EPL>(Kb + off);
            vf[i] = load_raw<EPL>(Vb + off);
        }
    };
    // two blocks in flight per wavefront: fetch block i+1 while block i is consumed
    Raw k0[NI], v0[NI], k1[NI], v1[NI];
    int kb = wave;
    if (kb < n_blocks) fetch(kb, k0, v0);
    if constexpr (!SELF) {
        if (fin) return;
        if (q_fix) {  // q = rstd' (P - (mu' - mu_hat) c1) + c2 with this row's statistics
            __shared__ float sm_fix[DH + 1];
            if (wave == 0) {
                const int tiles = a.q_stat_tiles;
                float mu = wave_sum(q_st.x) / (float)tiles;
                const float dev = lane < tiles ? (q_st.x - mu) * (q_st.x - mu) : 0.f;
                const float m2 = wave_sum(q_st.y) + 16.f * wave_sum(dev);
                const float r0 = fold_norm(a.q_rms, 16.f * (float)tiles, a.q_eps, m2, mu);
                const float sh = r0 * (mu - q_muh);
                if (g == 0) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) sm_fix[r * EPL + e] = qc2[e] - sh * qc1[e];
                }
                if (lane == 0) sm_fix[DH] = r0;
            }
            // LDS only: the key / value loads in flight are not waited for here
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            const float rstd = sm_fix[DH];
#pragma unroll
            for (int e = 0; e < EPL; ++e) q[e] = rstd * q[e] + sm_fix[r * EPL + e];
        }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) q[e] *= a.scale_log2e;

    float m_run = -INFINITY, l_run = 0.f;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    auto consume = [&](int kb, const Raw* kf, const Raw* vf) {
        const int last = n - 1 - kb * 16;
        float s[NI];
        float m_blk = -INFINITY;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const auto& kx = unpack<EPL>(kf[i]);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(q[e], raw_at<EPL>(kx, e), d);
            d = key_sum<LPK>(d);
            s[i] = (i * KPI + g <= last) ? d : -INFINITY;
            m_blk = fmaxf(m_blk, s[i]);
        }
        m_blk = keys_max<LPK>(m_blk);
        const float m_new = fmaxf(m_run, m_blk);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // first block: exp2(-inf) = 0
        l_run *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const float p = __builtin_amdgcn_exp2f(s[i] - m_new);
            l_run += p;
            const auto& vx = unpack<EPL>(vf[i]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, raw_at<EPL>(vx, e), acc[e]);
        }
        m_run = m_new;
    };

    while (kb < n_blocks) {
        if (kb + NW < n_blocks) fetch(kb + NW, k1, v1);
        consume(kb, k0, v0);
        kb += NW;
        if (kb >= n_blocks) break;
        if (kb + NW < n_blocks) fetch(kb + NW, k0, v0);
        consume(kb, k1, v1);
        kb += NW;
    }
    // lanes of different groups g hold different keys: add them up
    l_run = keys_sum<LPK>(l_run);
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = keys_sum<LPK>(acc[e]);

    __shared__ float sm_acc[NW][DH];
    __shared__ float sm_m[NW], sm_l[NW];
    if (g == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sm_acc[wave][r * EPL + e] = acc[e];
    }
    if (lane == 0) { sm_m[wave] = m_run; sm_l[wave] = l_run; }
    __syncthreads();
    const bool owner = tid < DH;  // thread tid owns output element tid of this head

    // merge the wavefronts in order (a wavefront without keys has m = -inf, l = 0, acc = 0)
    float m_tot = sm_m[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m_tot = fmaxf(m_tot, sm_m[w]);
    float l_tot = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const float f = __builtin_amdgcn_exp2f(sm_m[w] - m_tot);
        l_tot += sm_l[w] * f;
        if (owner) o += sm_acc[w][tid] * f;
    }
    T* out = reinterpret_cast<T*>(static_cast<char*>(a.out) + frag_elem_off<sizeof(T)>(b, h * DH + (owner ? tid : 0), H * DH));
    if (n_chunks == 1) {  // the output feeds the next GEMM: fragment order
        if (owner) *out = from_f32<T>(o / l_tot);
        return;
    }

    // ---- several chunks: publish the partial; the last workgroup of this (sequence, head) to arrive
    // combines all of them in chunk order, so the result does not depend on scheduling.
    // Partials and the arrival counter are exchanged with relaxed device-scope atomic accesses, which
    // are performed at the device's coherence point rather than in this XCD's write-back L2.  Every
    // thread waits for its own stores to complete before the workgroup's arrival is counted, and the
    // last arriver issues its loads only after it has seen the full count.  (Device-scope fences would
    // do the same job, but each costs tens of nanoseconds serialised over all workgroups of the
    // launch: ~60 us per launch measured here.)
    const int bh = b * H + h;
    float* my = a.part + ((size_t)bh * a.max_chunks + chunk_idx) * (DH + 2);
    if (owner) __hip_atomic_store(&my[tid], o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) {
        __hip_atomic_store(&my[DH], m_tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&my[DH + 1], l_tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __shared__ int sm_last;
    __syncthreads();
    if (tid == 0) {
        const int old = __hip_atomic_fetch_add(&a.counters[bh], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm_last = (old == n_chunks - 1);
    }
    __syncthreads();
    if (!sm_last) return;
    float* base = a.part + (size_t)bh * a.max_chunks * (DH + 2);
    if (owner) {
        float M = -INFINITY;
        for (int c = 0; c < n_chunks; ++c)
            M = fmaxf(M, __hip_atomic_load(&base[(size_t)c * (DH + 2) + DH], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        float L = 0.f, O = 0.f;
        for (int c = 0; c < n_chunks; ++c) {
            float* pc = base + (size_t)c * (DH + 2);
            const float f = __builtin_amdgcn_exp2f(
                __hip_atomic_load(&pc[DH], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - M);
            L += __hip_atomic_load(&pc[DH + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * f;
            O += __hip_atomic_load(&pc[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * f;
        }
        *out = from_f32<T>(O / L);
    }
    if (tid == 0) __hip_atomic_store(&a.counters[bh], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next launch
}

// Wavefronts per workgroup: 8 when the launch has few workgroups (the longest
// sequence sets the kernel's duration), 4 when there are plenty.
template <typename T, typename KV, int LPK, bool SELF>
static hipError_t launch_kv(const AttnArgs& a, dim3 grid, hipStream_t s) {
    const bool wide = (size_t)grid.x * grid.y * grid.z <= 1024;
    if (a.head_dim == 128) {
        if (wide) hipLaunchKernelGGL((attn_decode_kernel<T, KV, LPK, 128, SELF, 8>), grid, dim3(512), 0, s, a);
        else hipLaunchKernelGGL((attn_decode_kernel<T, KV, LPK, 128, SELF, 4>), grid, dim3(256), 0, s, a);
    } else if (a.head_dim == 64) {
        if (wide) hipLaunchKernelGGL((attn_decode_kernel<T, KV, LPK, 64, SELF, 8>), grid, dim3(512), 0, s, a);
        else hipLaunchKernelGGL((attn_decode_kernel<T, KV, LPK, 64, SELF, 4>), grid, dim3(256), 0, s, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
template <typename T, bool SELF>
static hipError_t launch_dh(const AttnArgs& a, dim3 grid, hipStream_t s) {
    if (a.kv_fp8) {
        if constexpr (sizeof(T) == 2) return launch_kv<T, fp8_t, 8, SELF>(a, grid, s);
        else return hipErrorInvalidValue;  // 8-bit caches go with bfloat16 models only
    }
    return launch_kv<T, T, 16, SELF>(a, grid, s);
}

hipError_t launch_attn_self(Dtype dt, const AttnArgs& a, hipStream_t s) {
    if (a.chunk < 64 || a.chunk % 64 != 0 || a.n_chunks_max < 1 || a.n_chunks_max > a.max_chunks)
        return hipErrorInvalidValue;
    dim3 grid(a.n_heads, a.batch, a.n_chunks_max);
    return dt == kBF16 ? launch_dh<bf16_t, true>(a, grid, s) : launch_dh<float, true>(a, grid, s);
}

hipError_t launch_attn_cross(Dtype dt, const AttnArgs& a, hipStream_t s) {
    if (a.chunk < 64 || a.chunk % 64 != 0 || !a.items || a.n_items < 1) return hipErrorInvalidValue;
    dim3 grid(a.n_heads, a.n_items);
    return dt == kBF16 ? launch_dh<bf16_t, false>(a, grid, s) : launch_dh<float, false>(a, grid, s);
}

}  // namespace aed
