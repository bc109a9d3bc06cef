// Decode attention over the KV cache: one query row per column, softmax(q.K^T/sqrt(hd)).V
// over cache rows [0, pos].  The context of a (column, head) is cut into splits handled
// by different workgroups (each keeps a running max / sum / unnormalised output), and a
// small second kernel merges the splits.  K and V rows are streamed straight from HBM,
// 16 bytes per lane, several rows per wave per load; the scores of a split live in LDS;
// all reductions are wave shuffles plus one LDS hop across the four waves.
#include "d3_common.h"

namespace d3 {

namespace {

template <typename T> struct KvVec;
template <> struct KvVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
};
template <> struct KvVec<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    }
};

template <> struct KvVec<f16_t> {
    static constexpr int N = 8;
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
        const half8 h = __builtin_bit_cast(half8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (float)h[e];
    }
};

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    constexpr int EPL = KvVec<T>::N;       // elements per lane per 16-byte load
    constexpr int LPR = HD / EPL;          // lanes that share one cache row
    constexpr int RPW = 64 / LPR;          // rows per wave per load
    constexpr int RPB = RPW * 4;           // rows per workgroup per load
    constexpr int U = 4;                   // loads in flight per lane
    extern __shared__ float sc[];          // scores, then probabilities, of this split
    __shared__ float red_m[4], red_s[4];
    __shared__ float osum[4][HD];

    const int split = blockIdx.x, h = blockIdx.y, c = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = a.cm.seq(c), ctx = a.cm.pos(c) + 1;
    const int j0 = split * a.split_len;
    const int j1 = min(j0 + a.split_len, ctx);
    const size_t pidx = ((size_t)c * a.H + h) * a.n_splits + split;
    if (j0 >= j1) {                        // nothing of this column's context falls in this split
        if (tid == 0) { a.part_ml[pidx * 2] = -INFINITY; a.part_ml[pidx * 2 + 1] = 0.f; }
        return;
    }
    const int n = j1 - j0;
    const int kvh = h / (a.H / a.H_kv);
    const size_t head_off = ((size_t)seq * a.H_kv + kvh) * a.max_seq * HD;
    const T* Kb = static_cast<const T*>(a.k_cache) + head_off;
    const T* Vb = static_cast<const T*>(a.v_cache) + head_off;
    const int sub = lane % LPR, rg = lane / LPR;

    float qv[EPL];
    {
        const float scale = 1.0f / sqrtf((float)HD);
        const float* qp = a.q + (size_t)c * a.q_stride + (size_t)h * HD + sub * EPL;
#pragma unroll
        for (int e = 0; e < EPL; ++e) qv[e] = qp[e] * scale;
    }

    // ---- scores ----
    const int iters = (n + RPB - 1) / RPB;
    float lmax = -INFINITY;
    for (int it = 0; it < iters; it += U) {
        uint4 kv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * 4 + wave) * RPW + rg;
            const int jc = j < j1 ? j : j1 - 1;
            kv[u] = *reinterpret_cast<const uint4*>(Kb + (size_t)jc * HD + sub * EPL);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * 4 + wave) * RPW + rg;
            float kf[EPL];
            KvVec<T>::unpack(kv[u], kf);
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) s = fmaf(qv[e], kf[e], s);
#pragma unroll
            for (int o = LPR / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
            if (j < j1) {
                if (sub == 0) sc[j - j0] = s;
                lmax = fmaxf(lmax, s);
            }
        }
    }
    lmax = wave_max(lmax);
    if (lane == 0) red_m[wave] = lmax;
    __syncthreads();
    const float m = fmaxf(fmaxf(red_m[0], red_m[1]), fmaxf(red_m[2], red_m[3]));

    // ---- probabilities (relative to this split's max) ----
    float lsum = 0.f;
    for (int t = tid; t < n; t += 256) {
        const float p = expf(sc[t] - m);
        sc[t] = p;
        lsum += p;
    }
    lsum = wave_sum(lsum);
    if (lane == 0) red_s[wave] = lsum;
    __syncthreads();

    // ---- weighted sum of V rows ----
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int it = 0; it < iters; it += U) {
        uint4 vv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * 4 + wave) * RPW + rg;
            const int jc = j < j1 ? j : j1 - 1;
            vv[u] = *reinterpret_cast<const uint4*>(Vb + (size_t)jc * HD + sub * EPL);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + ((it + u) * 4 + wave) * RPW + rg;
            const float p = j < j1 ? sc[j - j0] : 0.f;
            float vf[EPL];
            KvVec<T>::unpack(vv[u], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) acc[e] += __shfl_xor(acc[e], o, 64);
    }
    if (rg == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) osum[wave][sub * EPL + e] = acc[e];
    }
    __syncthreads();
    if (tid < HD) a.part_o[pidx * HD + tid] = osum[0][tid] + osum[1][tid] + osum[2][tid] + osum[3][tid];
    if (tid == 0) {
        a.part_ml[pidx * 2] = m;
        a.part_ml[pidx * 2 + 1] = red_s[0] + red_s[1] + red_s[2] + red_s[3];
    }
}

// Merge the splits of one (column, head): rescale each partial to the global max.
__global__ __launch_bounds__(128) void attn_combine_kernel(AttnArgs a) {
    const int h = blockIdx.x, c = blockIdx.y, t = threadIdx.x;
    if (t >= a.hd) return;
    const size_t p0 = ((size_t)c * a.H + h) * a.n_splits;
    float m = -INFINITY;
    for (int s = 0; s < a.n_splits; ++s) m = fmaxf(m, a.part_ml[(p0 + s) * 2]);
    float l = 0.f, o = 0.f;
    for (int s = 0; s < a.n_splits; ++s) {
        const float ms = a.part_ml[(p0 + s) * 2];
        if (ms == -INFINITY) continue;               // empty split: its output was never written
        const float w = expf(ms - m);
        l += a.part_ml[(p0 + s) * 2 + 1] * w;
        o += a.part_o[(p0 + s) * a.hd + t] * w;
    }
    const float r = o / l;
    const size_t oi = (size_t)c * a.H * a.hd + (size_t)h * a.hd + t;
    a.out[oi] = r;
    if (a.out_hi) {
        const uint32_t hb = f32_to_bf16(r);
        a.out_hi[oi] = (bf16_t)hb;
        a.out_lo[oi] = (bf16_t)f32_to_bf16(r - bf16_to_f32(hb));
    }
}

}  // namespace

// Requirements (checked by the caller): hd in {64, 128}; split_len * n_splits >= longest context;
// n_splits <= kMaxSplits; split_len * 4 bytes of LDS <= 48 KiB.
int launch_attention(const AttnArgs& a, int kv_dtype, hipStream_t s) {
    dim3 grid(a.n_splits, a.H, a.ncols);
    const size_t lds = (size_t)a.split_len * sizeof(float);
#define D3_ATTN(T)                                                                                      \
    do {                                                                                                \
        if (a.hd == 64) hipLaunchKernelGGL((attn_partial_kernel<T, 64>), grid, dim3(256), lds, s, a);   \
        else hipLaunchKernelGGL((attn_partial_kernel<T, 128>), grid, dim3(256), lds, s, a);             \
    } while (0)
    if (kv_dtype == 0) D3_ATTN(float);
    else if (kv_dtype == 1) D3_ATTN(bf16_t);
    else D3_ATTN(f16_t);
#undef D3_ATTN
    int rc = (int)hipGetLastError();
    if (rc != 0) return rc;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(a.H, a.ncols), dim3(128), 0, s, a);
    return (int)hipGetLastError();
}

}  // namespace d3
