// Small kernels around the projections: embedding gather, gain + bf16 split for
// the MFMA path, rotary embedding + KV append, greedy argmax, missing-state KV fill.
#include "d3_common.h"

namespace d3 {

namespace {

// ---------------- embedding gather: x[c][:] = E[token(c)][:] ----------------
template <typename W>
__global__ __launch_bounds__(256) void embed_kernel(const W* __restrict__ emb, const int32_t* __restrict__ tokens,
                                                    ColMap cm, int d, int vocab, float* __restrict__ x,
                                                    const double* __restrict__ inv_freq, int half_hd,
                                                    float2* __restrict__ rope_cs, const int* __restrict__ row0) {
    const int c = blockIdx.x;
    if ((int)threadIdx.x < half_hd) {       // the rotation angles depend on the position only, not on the block
        double sn, cs;
        const int pos = cm.pos(c) - (row0 ? row0[cm.seq(c)] : 0);      // a left-padded sequence counts from its first token
        sincos((double)pos * inv_freq[threadIdx.x], &sn, &cs);
        rope_cs[(size_t)c * half_hd + threadIdx.x] = make_float2((float)cs, (float)sn);
    }
    int tok = tokens[cm.tok_index(c)];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);   // stay inside the table whatever the caller fed
    const W* row = emb + (size_t)tok * d;
    float* xo = x + (size_t)c * d;
    if (sizeof(W) == 4) {
        for (int j = threadIdx.x * 4; j < d; j += blockDim.x * 4)
            *reinterpret_cast<float4*>(xo + j) = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(row) + j);
    } else {
        for (int j = threadIdx.x * 8; j < d; j += blockDim.x * 8) {       // d % 8 == 0: eight bf16 per load
            const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(row) + j);
            *reinterpret_cast<float4*>(xo + j) = make_float4(bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y));
            *reinterpret_cast<float4*>(xo + j + 4) = make_float4(bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w));
        }
    }
}

// ---------------- gain + split into bf16 hi/lo, sum of squares ----------------
// The matrix-core projections fold the RMSNorm scale 1/rms into their epilogue; what they need from the
// residual is hi + lo = x * gain and sum(x^2).  Inside a pass the residual projections produce both; this
// kernel does it for the embedding output.  One workgroup per column; a thread keeps up to 8 float4 of the
// column in registers (all loads issued together); wider columns fall back to a second read.
__global__ __launch_bounds__(256) void gain_split_kernel(const float* __restrict__ x, int x_stride,
                                                         const float* __restrict__ gain, int K,
                                                         bf16_t* __restrict__ hi, bf16_t* __restrict__ lo,
                                                         float* __restrict__ ssq) {
    constexpr int R = 8;
    __shared__ float red[4];
    const int c = blockIdx.x, tid = threadIdx.x;
    const float* xc = x + (size_t)c * x_stride;
    const int n4 = K / 4;
    float ss = 0.f;
    auto emit = [&](int i4, const float4& t, const float4& gg) {
        const float f[4] = {t.x * gg.x, t.y * gg.y, t.z * gg.z, t.w * gg.w};
        ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
        uint32_t h[4], l[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[e] = f32_to_bf16(f[e]);
            l[e] = f32_to_bf16(f[e] - bf16_to_f32(h[e]));
        }
        *reinterpret_cast<uint2*>(hi + (size_t)c * K + i4 * 4) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
        *reinterpret_cast<uint2*>(lo + (size_t)c * K + i4 * 4) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
    };
    float4 v[R], g[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i4 = tid + r * 256;
        if (i4 < n4) {
            v[r] = *reinterpret_cast<const float4*>(xc + i4 * 4);
            g[r] = *reinterpret_cast<const float4*>(gain + i4 * 4);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i4 = tid + r * 256;
        if (i4 < n4) emit(i4, v[r], g[r]);
    }
    for (int i4 = tid + R * 256; i4 < n4; i4 += 256)
        emit(i4, *reinterpret_cast<const float4*>(xc + i4 * 4), *reinterpret_cast<const float4*>(gain + i4 * 4));
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) ssq[(size_t)c * kSsqStride] = (red[0] + red[1]) + (red[2] + red[3]);
}

// ---------------- rotary embedding + KV append ----------------
// Half-split pairing: dims (j, j + hd/2) of a head turn by pos * inv_freq[j].
template <typename T>
__device__ __forceinline__ void store_kv(T* p, float v);
template <> __device__ __forceinline__ void store_kv<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_kv<f16_t>(f16_t* p, float v) { *p = (f16_t)fminf(fmaxf(v, -65504.f), 65504.f); }

template <typename T>
__global__ __launch_bounds__(64) void rope_append_kernel(RopeArgs a) {
    const int head = blockIdx.x, c = blockIdx.y, j = threadIdx.x;
    const int half = a.hd / 2;
    if (j >= half) return;
    const int seq = a.cm.seq(c), pos = a.cm.pos(c);
    float* row = a.qkv + (size_t)c * (a.H + 2 * a.H_kv) * a.hd + (size_t)head * a.hd;
    if (head < a.H + a.H_kv) {
        const float2 cs = a.rope_cs[(size_t)c * half + j];
        const float x0 = row[j], x1 = row[j + half];
        const float y0 = x0 * cs.x - x1 * cs.y;
        const float y1 = x0 * cs.y + x1 * cs.x;
        if (head < a.H) {
            row[j] = y0;
            row[j + half] = y1;
        } else {
            T* dst = static_cast<T*>(a.k_cache) + (((size_t)seq * a.H_kv + (head - a.H)) * a.max_seq + pos) * a.hd;
            store_kv<T>(dst + j, y0);
            store_kv<T>(dst + j + half, y1);
        }
    } else {
        T* dst = static_cast<T*>(a.v_cache) + (((size_t)seq * a.H_kv + (head - a.H - a.H_kv)) * a.max_seq + pos) * a.hd;
        store_kv<T>(dst + j, row[j]);
        store_kv<T>(dst + j + half, row[j + half]);
    }
}

// ---------------- greedy argmax, lowest index on ties ----------------
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int vocab, int32_t* __restrict__ out) {
    __shared__ float bv[16];
    __shared__ int bi[16];
    const int c = blockIdx.x, tid = threadIdx.x;
    const float* lg = logits + (size_t)c * vocab;
    float best = -INFINITY;
    int idx = 0x7fffffff;
    auto take = [&](float v, int j) { if (v > best || (v == best && j < idx)) { best = v; idx = j; } };
    // vocab % 2 == 0: pairs, eight pair-loads in flight per thread
    const int n2 = vocab / 2;
    for (int base = 0; base < n2; base += 1024 * 8) {
        float2 v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int p = base + r * 1024 + tid;
            v[r] = p < n2 ? *reinterpret_cast<const float2*>(lg + 2 * p) : make_float2(-INFINITY, -INFINITY);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int p = base + r * 1024 + tid;
            if (p < n2) { take(v[r].x, 2 * p); take(v[r].y, 2 * p + 1); }
        }
    }
    // NaN logits never win (comparisons false); an all-NaN row yields index clamp below
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(best, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    if ((tid & 63) == 0) { bv[tid >> 6] = best; bi[tid >> 6] = idx; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 16; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
        out[c] = idx >= vocab ? 0 : idx;
    }
}

// ---------------- missing-state fill (COPY) ----------------
// One workgroup per (row, sequence, KV head): read the source block's head vector once,
// write it into every dropped block.  16 bytes per lane.
__global__ __launch_bounds__(64) void fill_kernel(FillArgs a, int bytes_per_vec) {
    const int pos = a.pos_begin + blockIdx.x;
    const int seq = blockIdx.y / a.H_kv, h = blockIdx.y % a.H_kv;
    const int piece = threadIdx.x;
    if (piece * 16 >= bytes_per_vec) return;
    const size_t layer_stride = (size_t)a.max_batch * a.H_kv * a.max_seq * bytes_per_vec;
    const size_t off = (((size_t)seq * a.H_kv + h) * a.max_seq + pos) * bytes_per_vec + (size_t)piece * 16;
    char* kc = static_cast<char*>(a.k_cache);
    char* vc = static_cast<char*>(a.v_cache);
    uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
    if (a.src >= 0) {
        kv = *reinterpret_cast<const uint4*>(kc + (size_t)a.src * layer_stride + off);
        vv = *reinterpret_cast<const uint4*>(vc + (size_t)a.src * layer_stride + off);
    }
    for (int l = a.drop_begin; l < a.drop_begin + a.n_drop; ++l) {
        *reinterpret_cast<uint4*>(kc + (size_t)l * layer_stride + off) = kv;
        *reinterpret_cast<uint4*>(vc + (size_t)l * layer_stride + off) = vv;
    }
}

// ---------------- read-only streaming yardstick ----------------
// What the memory system gives a pure read stream issued the way the projections issue theirs (16 bytes per lane,
// streaming loads, eight in flight per lane, one contiguous band at a time): every workgroup XORs its share and
// one lane per wave stores the result so that the loads cannot be dropped.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = load_stream16(src + i + r * stride);
#pragma unroll
        for (int r = 0; r < 8; ++r) acc ^= v[r];
    }
    for (; i < n16; i += stride) acc ^= load_stream16(src + i);
    unsigned x = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x ^= __shfl_xor(x, o, 64);
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = x;
}

// ---------------- state words of a decode step that runs in the static scratch array ----------------
__global__ __launch_bounds__(256) void static_seed_kernel(StaticSeed seed, double* __restrict__ inv_freq, int half_hd, int* __restrict__ row0,
                                                          int* __restrict__ tickets, int n_tickets, int* __restrict__ gemm_tickets,
                                                          int n_gemm_tickets) {
    const int tid = blockIdx.x * blockDim.x + threadIdx.x, n = gridDim.x * blockDim.x;
    if (tid < half_hd) inv_freq[tid] = seed.inv_freq[tid];
    if (tid < kMaxCols) row0[tid] = seed.row0[tid];
    for (int i = tid; i < n_tickets; i += n) tickets[i] = 0;
    for (int i = tid; i < n_gemm_tickets; i += n) gemm_tickets[i] = 0;
}

}  // namespace

int launch_static_seed(const StaticSeed& seed, double* inv_freq, int half_hd, int* row0, int* tickets, int n_tickets,
                       int* gemm_tickets, int n_gemm_tickets, hipStream_t s) {
    hipLaunchKernelGGL(static_seed_kernel, dim3(8), dim3(256), 0, s, seed, inv_freq, half_hd, row0, tickets, n_tickets, gemm_tickets,
                       n_gemm_tickets);
    return (int)hipGetLastError();
}

int launch_stream_read(const void* src, size_t bytes, unsigned* sink, int n_wg, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_wg), dim3(256), 0, s, static_cast<const u32x4*>(src), bytes / 16, sink);
    return (int)hipGetLastError();
}

int launch_embed(const void* tok_emb, int weight_dtype, const int32_t* tokens, ColMap cm, int ncols, int d,
                 int vocab, float* x, const double* inv_freq, int half_hd, float2* rope_cs, const int* row0, hipStream_t s) {
    if (weight_dtype == 0)
        hipLaunchKernelGGL(embed_kernel<float>, dim3(ncols), dim3(256), 0, s, static_cast<const float*>(tok_emb), tokens, cm, d, vocab, x,
                           inv_freq, half_hd, rope_cs, row0);
    else
        hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(ncols), dim3(256), 0, s, static_cast<const bf16_t*>(tok_emb), tokens, cm, d, vocab, x,
                           inv_freq, half_hd, rope_cs, row0);
    return (int)hipGetLastError();
}

int launch_gain_split(const float* x, int x_stride, const float* gain, int K, int ncols,
                      bf16_t* hi, bf16_t* lo, float* ssq, hipStream_t s) {
    hipLaunchKernelGGL(gain_split_kernel, dim3(ncols), dim3(256), 0, s, x, x_stride, gain, K, hi, lo, ssq);
    return (int)hipGetLastError();
}

int launch_rope_append(const RopeArgs& a, int kv_dtype, hipStream_t s) {
    dim3 grid(a.H + 2 * a.H_kv, a.ncols);
    if (kv_dtype == 0) hipLaunchKernelGGL(rope_append_kernel<float>, grid, dim3(64), 0, s, a);
    else if (kv_dtype == 2) hipLaunchKernelGGL(rope_append_kernel<f16_t>, grid, dim3(64), 0, s, a);
    else return (int)hipErrorInvalidValue;
    return (int)hipGetLastError();
}

int launch_argmax(const float* logits, int vocab, int ncols, int32_t* out, hipStream_t s) {
    hipLaunchKernelGGL(argmax_kernel, dim3(ncols), dim3(1024), 0, s, logits, vocab, out);
    return (int)hipGetLastError();
}

int launch_fill(const FillArgs& a, int kv_dtype, hipStream_t s) {
    if (a.pos_end <= a.pos_begin || a.n_drop <= 0) return 0;
    const int bytes_per_vec = a.hd * kv_elem_bytes(kv_dtype);
    dim3 grid(a.pos_end - a.pos_begin, a.B * a.H_kv);
    hipLaunchKernelGGL(fill_kernel, grid, dim3(64), 0, s, a, bytes_per_vec);
    return (int)hipGetLastError();
}

}  // namespace d3
