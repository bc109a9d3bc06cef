// Weight-streaming GEMV for one (or a few) activation columns on the vector ALUs.
//
// This is the batch-1 decode projection: every weight byte is read from HBM
// exactly once, 16 bytes per lane per load, a whole wave reading 1 KiB of one
// weight row per instruction.  Activations sit in LDS as fp32 (laid out so that a
// wave's reads are conflict-free), accumulation is fp32, a row's dot product is
// finished with a wave reduction.  The RMSNorm of the input (fused QKV, gate/up
// and lm_head projections) is recomputed by every workgroup in its prologue: the
// input is a few KiB that stay in L2, which is cheaper than a separate launch.
#include "d3_common.h"

namespace d3 {

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerWg = kThreads / kWave;
constexpr int kLdsBudget = 60 * 1024;   // dynamic LDS per workgroup (static reductions come on top)

template <typename W> struct Chunk;                    // one 16-byte piece of a weight row
template <> struct Chunk<float> { static constexpr int N = 4; };
template <> struct Chunk<bf16_t> { static constexpr int N = 8; };

// Position (in float4 units) of activation element k inside one column's LDS image.
// bf16 weights: a lane consumes 8 consecutive activations per chunk; they are stored as
// two float4 planes so that lanes of a wave read consecutive 16-byte words.
template <typename W> __device__ __forceinline__ int lds_f4_index(int k);
template <> __device__ __forceinline__ int lds_f4_index<float>(int k) { return k >> 2; }
template <> __device__ __forceinline__ int lds_f4_index<bf16_t>(int k) {
    int q = k >> 3;
    return (((q >> 6) << 1) + ((k >> 2) & 1)) * 64 + (q & 63);
}
template <typename W> __host__ __device__ inline int lds_f4_per_col(int K) {
    if (sizeof(W) == 4) return K / 4;
    int chunks = K / 8;
    return ((chunks + 63) / 64) * 128;
}

template <int NC>
__device__ __forceinline__ void fma_chunk_f32(const u32x4& w, const float4* xs, int f4_per_col, int q, float (&acc)[NC]) {
    float w0 = __uint_as_float(w.x), w1 = __uint_as_float(w.y), w2 = __uint_as_float(w.z), w3 = __uint_as_float(w.w);
#pragma unroll
    for (int n = 0; n < NC; ++n) {
        float4 x = xs[n * f4_per_col + q];
        acc[n] = fmaf(w0, x.x, acc[n]); acc[n] = fmaf(w1, x.y, acc[n]);
        acc[n] = fmaf(w2, x.z, acc[n]); acc[n] = fmaf(w3, x.w, acc[n]);
    }
}

template <int NC>
__device__ __forceinline__ void fma_chunk_bf16(const u32x4& w, const float4* xs, int f4_per_col, int q, float (&acc)[NC]) {
    const int base = ((q >> 6) << 7) + (q & 63);
#pragma unroll
    for (int n = 0; n < NC; ++n) {
        float4 xa = xs[n * f4_per_col + base];
        float4 xb = xs[n * f4_per_col + base + 64];
        acc[n] = fmaf(bf16_lo(w.x), xa.x, acc[n]); acc[n] = fmaf(bf16_hi(w.x), xa.y, acc[n]);
        acc[n] = fmaf(bf16_lo(w.y), xa.z, acc[n]); acc[n] = fmaf(bf16_hi(w.y), xa.w, acc[n]);
        acc[n] = fmaf(bf16_lo(w.z), xb.x, acc[n]); acc[n] = fmaf(bf16_hi(w.z), xb.y, acc[n]);
        acc[n] = fmaf(bf16_lo(w.w), xb.z, acc[n]); acc[n] = fmaf(bf16_hi(w.w), xb.w, acc[n]);
    }
}

template <typename W, int NC, int MODE, bool NORM>
__global__ __launch_bounds__(kThreads) void gemv_alu_kernel(GemvArgs a) {
    extern __shared__ float4 xs[];                     // [NC][f4_per_col]
    __shared__ float red[NC][kWavesPerWg];
    constexpr int EPC = Chunk<W>::N;
    const int K = a.K;
    const int f4_per_col = lds_f4_per_col<W>(K);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- prologue: activations -> LDS (optionally RMS-normalised) ----
    float ss[NC];
#pragma unroll
    for (int n = 0; n < NC; ++n) ss[n] = 0.f;
    for (int i4 = tid; i4 < K / 4; i4 += kThreads) {
        const int dst = lds_f4_index<W>(i4 * 4);
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < a.ncols) v = *reinterpret_cast<const float4*>(a.x + (size_t)n * a.x_stride + i4 * 4);
            if (NORM) ss[n] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            xs[n * f4_per_col + dst] = v;
        }
    }
    if (NORM) {
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            float s = wave_sum(ss[n]);
            if (lane == 0) red[n][wave] = s;
        }
        __syncthreads();
        float rinv[NC];
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < kWavesPerWg; ++w) s += red[n][w];
            rinv[n] = 1.0f / sqrtf(s / (float)K + a.eps);
        }
        for (int i4 = tid; i4 < K / 4; i4 += kThreads) {   // each thread rescales what it wrote
            const int dst = lds_f4_index<W>(i4 * 4);
            const float4 g = *reinterpret_cast<const float4*>(a.gain + i4 * 4);
#pragma unroll
            for (int n = 0; n < NC; ++n) {
                float4 v = xs[n * f4_per_col + dst];
                v.x *= rinv[n] * g.x; v.y *= rinv[n] * g.y; v.z *= rinv[n] * g.z; v.w *= rinv[n] * g.w;
                xs[n * f4_per_col + dst] = v;
            }
        }
    }
    __syncthreads();

    // ---- main loop: one unit = two weight rows per wave ----
    const int nchunks = K / EPC;
    const int n_units = (MODE == MODE_SWIGLU) ? a.total_rows : a.total_rows / 2;
    const int gw = blockIdx.x * kWavesPerWg + wave, nw = gridDim.x * kWavesPerWg;
    constexpr int U = 4;                               // chunks in flight per row
    for (int u = gw; u < n_units; u += nw) {
        const W *r0, *r1;
        int row;
        if (MODE == MODE_SWIGLU) {
            row = u;
            r0 = static_cast<const W*>(a.w[0]) + (size_t)u * K;
            r1 = static_cast<const W*>(a.w[1]) + (size_t)u * K;
        } else {
            row = 2 * u;
            int m = 0, local = row;
            if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
            r0 = static_cast<const W*>(a.w[m]) + (size_t)local * K;
            r1 = r0 + K;
        }
        float acc0[NC], acc1[NC];
#pragma unroll
        for (int n = 0; n < NC; ++n) { acc0[n] = 0.f; acc1[n] = 0.f; }
        for (int q0 = lane; q0 < nchunks; q0 += 64 * U) {
            u32x4 w0[U], w1[U];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int q = q0 + 64 * j;
                if (q < nchunks) {
                    w0[j] = load_stream16(r0 + (size_t)q * EPC);
                    w1[j] = load_stream16(r1 + (size_t)q * EPC);
                }
            }
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int q = q0 + 64 * j;
                if (q < nchunks) {
                    if (sizeof(W) == 4) { fma_chunk_f32<NC>(w0[j], xs, f4_per_col, q, acc0); fma_chunk_f32<NC>(w1[j], xs, f4_per_col, q, acc1); }
                    else { fma_chunk_bf16<NC>(w0[j], xs, f4_per_col, q, acc0); fma_chunk_bf16<NC>(w1[j], xs, f4_per_col, q, acc1); }
                }
            }
        }
#pragma unroll
        for (int n = 0; n < NC; ++n) { acc0[n] = wave_sum(acc0[n]); acc1[n] = wave_sum(acc1[n]); }
        if (lane == 0) {
#pragma unroll
            for (int n = 0; n < NC; ++n) {
                if (n >= a.ncols) break;
                float* o = a.out + (size_t)n * a.out_stride + row;
                if (MODE == MODE_STORE) { o[0] = acc0[n]; o[1] = acc1[n]; }
                else if (MODE == MODE_RESID) { o[0] += acc0[n]; o[1] += acc1[n]; }
                else { const float g = acc0[n]; o[0] = g / (1.0f + expf(-g)) * acc1[n]; }
            }
        }
    }
}

template <typename W, int NC>
int launch_nc(const GemvArgs& a, int mode, bool norm, int n_wg, hipStream_t s) {
    const size_t lds = (size_t)NC * lds_f4_per_col<W>(a.K) * sizeof(float4);
    const int n_units = (mode == MODE_SWIGLU) ? a.total_rows : a.total_rows / 2;
    int grid = (n_units + kWavesPerWg - 1) / kWavesPerWg;
    if (grid > n_wg) grid = n_wg;
    if (grid < 1) grid = 1;
#define D3_LAUNCH(MODE, NORM) hipLaunchKernelGGL((gemv_alu_kernel<W, NC, MODE, NORM>), dim3(grid), dim3(kThreads), lds, s, a)
    if (mode == MODE_STORE) { if (norm) D3_LAUNCH(MODE_STORE, true); else D3_LAUNCH(MODE_STORE, false); }
    else if (mode == MODE_RESID) { D3_LAUNCH(MODE_RESID, false); }
    else { D3_LAUNCH(MODE_SWIGLU, true); }
#undef D3_LAUNCH
    return (int)hipGetLastError();
}

template <typename W>
int launch_w(const GemvArgs& a, int mode, bool norm, int n_wg, hipStream_t s) {
    switch (a.ncols) {
        case 1: return launch_nc<W, 1>(a, mode, norm, n_wg, s);
        case 2: return launch_nc<W, 2>(a, mode, norm, n_wg, s);
        case 3: case 4: return launch_nc<W, 4>(a, mode, norm, n_wg, s);
        default: return (int)hipErrorInvalidValue;
    }
}

}  // namespace

size_t gemv_alu_max_cols(int K, int weight_dtype) {
    const size_t per_col = (size_t)(weight_dtype == 0 ? lds_f4_per_col<float>(K) : lds_f4_per_col<bf16_t>(K)) * sizeof(float4);
    size_t n = kLdsBudget / per_col;
    return n >= 4 ? 4 : (n >= 2 ? 2 : (n >= 1 ? 1 : 0));
}

// Requirements (checked by the caller): K % 8 == 0, total_rows even, 1 <= ncols <= gemv_alu_max_cols,
// MODE_RESID without norm, MODE_SWIGLU with norm, x/out/weights 16-byte aligned.
int launch_gemv_alu(const GemvArgs& a, int weight_dtype, int mode, bool norm, int n_wg, hipStream_t s) {
    return weight_dtype == 0 ? launch_w<float>(a, mode, norm, n_wg, s) : launch_w<bf16_t>(a, mode, norm, n_wg, s);
}

}  // namespace d3
