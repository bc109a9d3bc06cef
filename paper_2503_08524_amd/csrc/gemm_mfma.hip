// Skinny GEMM on the matrix cores for 2..32 activation columns (batched decode and the
// chunked prompt pass): out[col][row] = sum_k W[row][k] * x[col][k], bf16 weights.
//
// The weight matrix is the MFMA "A" operand (16 rows per tile), the activation columns the
// "B" operand (16 columns per tile, one or two tiles).  Weights are read from HBM exactly
// once, 16 bytes per lane; a workgroup owns one 16-row tile (a gate tile and its up tile
// for SwiGLU) and its waves split K between them, 128 consecutive k per wave per turn, so
// that a narrow matrix still puts thousands of waves on the memory system.  Partial tiles
// are summed through LDS.  Activations arrive pre-split as x = hi + lo (two bf16 halves,
// ~16 mantissa bits): two MFMAs per weight tile keep fp32-like accuracy, and the matrix
// cores have an order of magnitude of headroom on this HBM-bound contraction.
//
// v_mfma_f32_16x16x32_bf16 operand layout (lane l, i = l % 16, g = l / 16): A holds row i,
// k = 8g..8g+7; B holds column i, the same k; the result holds column i, rows 4g..4g+3.
#include "d3_common.h"

namespace d3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int U = 4;   // k-steps (of 32) a wave takes per turn: 256 contiguous bytes of each weight row

template <int NT, int MODE>
__global__ __launch_bounds__(1024) void gemm_mfma_kernel(GemvArgs a) {
    constexpr int RT = (MODE == MODE_SWIGLU) ? 2 : 1;
    constexpr int A = RT * NT * 4;                    // accumulator floats per lane
    extern __shared__ float red[];                    // [waves][A][64]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int K = a.K, row0 = blockIdx.x * 16;

    const bf16_t* wr[RT];
    if (MODE == MODE_SWIGLU) {
        wr[0] = static_cast<const bf16_t*>(a.w[0]) + (size_t)(row0 + i) * K + 8 * g;
        wr[RT - 1] = static_cast<const bf16_t*>(a.w[1]) + (size_t)(row0 + i) * K + 8 * g;
    } else {
        int m = 0, local = row0;
        if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
        wr[0] = static_cast<const bf16_t*>(a.w[m]) + (size_t)(local + i) * K + 8 * g;
    }
    const bf16_t* xh[NT];
    const bf16_t* xl[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        xh[t] = a.x_hi + (size_t)(t * 16 + i) * a.x_stride + 8 * g;
        xl[t] = a.x_lo + (size_t)(t * 16 + i) * a.x_stride + 8 * g;
    }

    f32x4 acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nks = K / 32;
    for (int ks0 = wave * U; ks0 < nks; ks0 += n_waves * U) {
        u32x4 wv[RT][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ks0 + u < nks) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    wv[r][u] = load_stream16(wr[r] + (size_t)(ks0 + u) * 32);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (ks0 + u < nks) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint4 bh = *reinterpret_cast<const uint4*>(xh[t] + (size_t)(ks0 + u) * 32);
                    const uint4 bl = *reinterpret_cast<const uint4*>(xl[t] + (size_t)(ks0 + u) * 32);
#pragma unroll
                    for (int r = 0; r < RT; ++r) {
                        const bf16x8 wa = __builtin_bit_cast(bf16x8, wv[r][u]);
                        acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bh), acc[r][t], 0, 0, 0);
                        acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bl), acc[r][t], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- sum the waves' partial tiles through LDS, then the epilogue ----
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[((size_t)wave * A + (r * NT + t) * 4 + e) * 64 + lane] = acc[r][t][e];
    __syncthreads();
    constexpr int A_OUT = NT * 4;                     // outputs per lane (gate/up pairs fold into one)
    for (int idx = tid; idx < A_OUT * 64; idx += blockDim.x) {
        const int ai = idx >> 6, l = idx & 63;
        float s0 = 0.f, s1 = 0.f;
        for (int w = 0; w < n_waves; ++w) {
            s0 += red[((size_t)w * A + ai) * 64 + l];
            if (MODE == MODE_SWIGLU) s1 += red[((size_t)w * A + A_OUT + ai) * 64 + l];
        }
        const int t = ai >> 2, e = ai & 3;
        const int row = row0 + 4 * (l >> 4) + e, col = t * 16 + (l & 15);
        if (col >= a.ncols) continue;
        const size_t oi = (size_t)col * a.out_stride + row;
        float v;
        if (MODE == MODE_STORE) v = s0;
        else if (MODE == MODE_RESID) v = a.out[oi] + s0;
        else v = s0 / (1.0f + expf(-s0)) * s1;
        if (a.out) a.out[oi] = v;
        if (a.out_hi) {
            const uint32_t hb = f32_to_bf16(v);
            a.out_hi[oi] = (bf16_t)hb;
            a.out_lo[oi] = (bf16_t)f32_to_bf16(v - bf16_to_f32(hb));
        }
    }
}

}  // namespace

// Requirements (checked by the caller): bf16 weights; K % 32 == 0; total_rows and every rows[m]
// multiples of 16; 1 <= ncols <= 32; x_hi/x_lo hold 32 rows of x_stride elements (rows beyond
// ncols may hold anything finite or not: their columns are never written).
int launch_gemm_mfma(const GemvArgs& a, int mode, int n_cu, hipStream_t s) {
    const int tiles = a.total_rows / 16;
    const int nt = a.ncols > 16 ? 2 : 1;
    const int rt = mode == MODE_SWIGLU ? 2 : 1;
    int waves = 4;
    while (waves < 16 && tiles * waves < 8 * n_cu) waves *= 2;
    while (waves > 4 && (a.K / 32) < waves * U) waves /= 2;                       // at least one turn per wave
    while (waves > 4 && (size_t)waves * rt * nt * 4 * 64 * sizeof(float) > 48 * 1024) waves /= 2;
    const size_t lds = (size_t)waves * rt * nt * 4 * 64 * sizeof(float);
#define D3_LAUNCH(NT, MODE) hipLaunchKernelGGL((gemm_mfma_kernel<NT, MODE>), dim3(tiles), dim3(64 * waves), lds, s, a)
    if (nt == 1) {
        if (mode == MODE_STORE) D3_LAUNCH(1, MODE_STORE); else if (mode == MODE_RESID) D3_LAUNCH(1, MODE_RESID); else D3_LAUNCH(1, MODE_SWIGLU);
    } else {
        if (mode == MODE_STORE) D3_LAUNCH(2, MODE_STORE); else if (mode == MODE_RESID) D3_LAUNCH(2, MODE_RESID); else D3_LAUNCH(2, MODE_SWIGLU);
    }
#undef D3_LAUNCH
    return (int)hipGetLastError();
}

}  // namespace d3
