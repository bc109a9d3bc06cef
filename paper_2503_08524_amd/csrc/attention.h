// Device-side body of the decode attention (see attention.hip): one (column, head, context split)
// per call by a workgroup of NW waves, plus the merge of the splits by whichever split arrives last.
#pragma once
#include "d3_common.h"

namespace d3 {

template <typename T> struct KvVec;
template <> struct KvVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ float round(float v) { return v; }
};
template <> struct KvVec<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    }
    static __device__ __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};
template <> struct KvVec<f16_t> {
    static constexpr int N = 8;
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
        const half8 h = __builtin_bit_cast(half8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (float)h[e];
    }
    static __device__ __forceinline__ float round(float v) { return (float)(f16_t)fminf(fmaxf(v, -65504.f), 65504.f); }
};

template <int HD, int NW>
struct AttnShared {
    float red_m[NW], red_s[NW];
    float osum[NW][HD];
    int is_last;
};

// FUSED: the call runs inside a kernel that also produced q and the newest K/V row in this launch:
// q and that row are read from the fp32 projection buffer with agent-scope loads (the row rounded
// to the cache's element type, i.e. exactly what later steps will read back), and the merged
// output is published with agent-scope stores.
template <typename T, int HD, bool FUSED, int NW>
__device__ __forceinline__ void attn_split(const AttnArgs& a, int split, int h, int c, float* sc, AttnShared<HD, NW>& sh) {
    constexpr int EPL = KvVec<T>::N;       // elements per lane per 16-byte load
    constexpr int LPR = HD / EPL;          // lanes that share one cache row
    constexpr int RPW = 64 / LPR;          // rows per wave per load
    constexpr int RPB = RPW * NW;          // rows per workgroup per load
    constexpr int U = 4;                   // loads in flight per lane

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = a.cm.seq(c), ctx = a.cm.pos(c) + 1;
    const int j0 = split * a.split_len;
    const int j1 = min(j0 + a.split_len, ctx);
    const size_t pidx = ((size_t)c * a.H + h) * a.n_splits + split;
    if (j0 >= j1) return;                  // nothing of this column's context falls in this split
    const int n_live = (ctx + a.split_len - 1) / a.split_len;   // splits of this column that hold rows
    const int n = j1 - j0;
    const int kvh = h / (a.H / a.H_kv);
    const size_t head_off = ((size_t)seq * a.H_kv + kvh) * a.max_seq * HD;
    const T* Kb = static_cast<const T*>(a.k_cache) + head_off;
    const T* Vb = static_cast<const T*>(a.v_cache) + head_off;
    const int sub = lane % LPR, rg = lane / LPR;
    // FUSED: the newest row (ctx - 1) of this column, k then v, inside the projection buffer
    const float* cur_k = a.q + (size_t)c * a.q_stride + (size_t)(a.H + kvh) * HD + sub * EPL;
    const float* cur_v = cur_k + (size_t)a.H_kv * HD;

    // q is loaded raw and first touched in the score loop, after the K/V loads have been issued
    // (scaling it here would make those loads wait for it); 1/sqrt(hd) is applied to the scores
    const float scale = 1.0f / sqrtf((float)HD);
    float qv[EPL];
    {
        const float* qp = a.q + (size_t)c * a.q_stride + (size_t)h * HD + sub * EPL;
        if (FUSED) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) qv[e] = ld_agent(qp + e);
        } else {
#pragma unroll
            for (int e = 0; e < EPL; e += 4) {
                const float4 t = *reinterpret_cast<const float4*>(qp + e);
                qv[e] = t.x; qv[e + 1] = t.y; qv[e + 2] = t.z; qv[e + 3] = t.w;
            }
        }
    }

    const int iters = (n + RPB - 1) / RPB;
    constexpr int ITMAX = 8;               // a split of up to ITMAX * RPB rows keeps all its K and V rows in registers
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    float m, lsum = 0.f;
    if (iters <= ITMAX) {
        // short split: K and V loads all go out together (V does not wait for the softmax)
        uint4 kv[ITMAX], vv[ITMAX];
#pragma unroll
        for (int u = 0; u < ITMAX; ++u) {
            const int j = j0 + (u * NW + wave) * RPW + rg;
            const int jc = j < j1 ? j : j1 - 1;
            if (u < iters) {
                kv[u] = *reinterpret_cast<const uint4*>(Kb + (size_t)jc * HD + sub * EPL);
                vv[u] = *reinterpret_cast<const uint4*>(Vb + (size_t)jc * HD + sub * EPL);
            }
        }
        float sv[ITMAX];
        float lmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < ITMAX; ++u) {
            sv[u] = -INFINITY;
            if (u < iters) {
                const int j = j0 + (u * NW + wave) * RPW + rg;
                float kf[EPL];
                KvVec<T>::unpack(kv[u], kf);
                if (FUSED && j == ctx - 1) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) kf[e] = KvVec<T>::round(ld_agent(cur_k + e));
                }
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) s = fmaf(qv[e], kf[e], s);
#pragma unroll
                for (int o = LPR / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
                s *= scale;
                if (j < j1) { sv[u] = s; lmax = fmaxf(lmax, s); }
            }
        }
        lmax = wave_max(lmax);
        if (lane == 0) sh.red_m[wave] = lmax;
        __syncthreads();
        m = sh.red_m[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) m = fmaxf(m, sh.red_m[w]);
#pragma unroll
        for (int u = 0; u < ITMAX; ++u) {
            if (u < iters) {
                const int j = j0 + (u * NW + wave) * RPW + rg;
                const float p = expf(sv[u] - m);                    // exp(-inf) = 0 for rows past the split
                if (sub == 0) lsum += p;
                float vf[EPL];
                KvVec<T>::unpack(vv[u], vf);
                if (FUSED && j == ctx - 1) {
#pragma unroll
                    for (int e = 0; e < EPL; ++e) vf[e] = KvVec<T>::round(ld_agent(cur_v + e));
                }
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
            }
        }
        lsum = wave_sum(lsum);
        if (lane == 0) sh.red_s[wave] = lsum;
    } else {
    // ---- scores ----
    float lmax = -INFINITY;
    for (int it = 0; it < iters; it += U) {
        uint4 kv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * NW + wave) * RPW + rg;
            const int jc = j < j1 ? j : j1 - 1;
            kv[u] = *reinterpret_cast<const uint4*>(Kb + (size_t)jc * HD + sub * EPL);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * NW + wave) * RPW + rg;
            float kf[EPL];
            KvVec<T>::unpack(kv[u], kf);
            if (FUSED && j == ctx - 1) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) kf[e] = KvVec<T>::round(ld_agent(cur_k + e));
            }
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) s = fmaf(qv[e], kf[e], s);
#pragma unroll
            for (int o = LPR / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
            s *= scale;
            if (j < j1) {
                if (sub == 0) sc[j - j0] = s;
                lmax = fmaxf(lmax, s);
            }
        }
    }
    lmax = wave_max(lmax);
    if (lane == 0) sh.red_m[wave] = lmax;
    __syncthreads();
    m = sh.red_m[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) m = fmaxf(m, sh.red_m[w]);

    // ---- probabilities (relative to this split's max) ----
    for (int t = tid; t < n; t += NW * 64) {
        const float p = expf(sc[t] - m);
        sc[t] = p;
        lsum += p;
    }
    lsum = wave_sum(lsum);
    if (lane == 0) sh.red_s[wave] = lsum;
    __syncthreads();

    // ---- weighted sum of V rows ----
    for (int it = 0; it < iters; it += U) {
        uint4 vv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * NW + wave) * RPW + rg;
            const int jc = j < j1 ? j : j1 - 1;
            vv[u] = *reinterpret_cast<const uint4*>(Vb + (size_t)jc * HD + sub * EPL);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * NW + wave) * RPW + rg;
            const float p = j < j1 ? sc[j - j0] : 0.f;
            float vf[EPL];
            KvVec<T>::unpack(vv[u], vf);
            if (FUSED && j == ctx - 1) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) vf[e] = KvVec<T>::round(ld_agent(cur_v + e));
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
        }
    }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) acc[e] += __shfl_xor(acc[e], o, 64);
    }
    if (rg == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sh.osum[wave][sub * EPL + e] = acc[e];
    }
    __syncthreads();
    if (tid < HD) {
        float o = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) o += sh.osum[w][tid];
        st_agent(&a.part_o[pidx * HD + tid], o);
    }
    if (tid == 0) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += sh.red_s[w];
        st_agent(&a.part_ml[pidx * 2], m);
        st_agent(&a.part_ml[pidx * 2 + 1], l);
    }

    // ---- the split that arrives last merges all splits of this (column, head) ----
    wait_stores();                                     // this split's partial has reached the coherence point
    __syncthreads();
    if (tid == 0) {
        const int done = atomicAdd(&a.tickets[c * a.H + h], 1);
        sh.is_last = done == n_live - 1;
        if (sh.is_last) __hip_atomic_store(&a.tickets[c * a.H + h], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // all arrived: leave it clean
    }
    __syncthreads();
    if (!sh.is_last) return;
    if (tid < HD) {
        // all partials are fetched in rounds of 8 splits (one round trip each), merged with a running max
        const size_t p0 = ((size_t)c * a.H + h) * a.n_splits;
        float gm = -INFINITY, l = 0.f, o = 0.f;
        for (int s0 = 0; s0 < n_live; s0 += 8) {
            float ms[8], ls[8], os[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int sidx = s0 + k < n_live ? s0 + k : n_live - 1;
                ms[k] = ld_agent(&a.part_ml[(p0 + sidx) * 2]);
                ls[k] = ld_agent(&a.part_ml[(p0 + sidx) * 2 + 1]);
                os[k] = ld_agent(&a.part_o[(p0 + sidx) * HD + tid]);
            }
            float rm = gm;
#pragma unroll
            for (int k = 0; k < 8; ++k) if (s0 + k < n_live) rm = fmaxf(rm, ms[k]);
            const float keep = expf(gm - rm);             // gm = -inf on the first round: exp(-inf) = 0
            l *= keep; o *= keep;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (s0 + k < n_live) {
                    const float w = expf(ms[k] - rm);
                    l += ls[k] * w;
                    o += os[k] * w;
                }
            }
            gm = rm;
        }
        const float r = o / l;
        const size_t oi = (size_t)c * a.H * HD + (size_t)h * HD + tid;
        if (FUSED) st_agent(&a.out[oi], r); else a.out[oi] = r;
        if (a.out_hi) {
            const uint32_t hb = f32_to_bf16(r);
            a.out_hi[oi] = (bf16_t)hb;
            a.out_lo[oi] = (bf16_t)f32_to_bf16(r - bf16_to_f32(hb));
        }
    }
}

}  // namespace d3
