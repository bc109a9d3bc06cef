// Skinny GEMM on the matrix cores for 2..32 activation columns (batched decode and the
// chunked prompt pass): out[col][row] = sum_k W[row][k] * x[col][k], bf16 weights.
//
// The weight matrix is the MFMA "A" operand (16 rows per tile), the activation columns the
// "B" operand (16 columns per tile, one or two tiles).  Weights are read from HBM exactly
// once, 16 bytes per lane.  A workgroup owns RT consecutive 16-row tiles (RT gate tiles and
// their up tiles for SwiGLU) and its waves split K between them, 128 consecutive k per wave
// per turn, so that a narrow matrix still puts thousands of waves on the memory system; a
// wave reuses each activation fragment for all its RT tiles, which keeps the L2 traffic of
// the activations below the HBM traffic of the weights.  Tiles are fetched with coalesced loads and
// re-shaped into MFMA fragments through a small per-wave LDS tile; the next turn's loads are in
// flight while the current turn's MFMAs run.  Partial tiles are summed
// through LDS.  Activations arrive pre-split as x = hi + lo (two bf16 halves, ~16 mantissa
// bits): two MFMAs per weight tile keep fp32-like accuracy, and the matrix cores have an
// order of magnitude of headroom on this HBM-bound contraction.  With at most 8 columns the two halves
// share ONE B tile (columns 0..7 hi, 8..15 lo) and their results are added in the epilogue: half the
// activation traffic, LDS re-shaping and MFMAs.
//
// v_mfma_f32_16x16x32_bf16 operand layout (lane l, i = l % 16, g = l / 16): A holds row i,
// k = 8g..8g+7; B holds column i, the same k; the result holds column i, rows 4g..4g+3.
#include <cstdlib>

#include "d3_common.h"

namespace d3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int U = 4;            // k-steps (of 32) a wave takes per turn: 256 contiguous bytes of each row
constexpr int kTileRowBytes = 272;   // LDS pitch of a staged 16 x 256 B tile (+16 B: conflict-free fragment reads)
constexpr int kTileBytes = 16 * kTileRowBytes;

// A 16-row x 128-k bf16 tile travels global -> registers (coalesced: 16 lanes read 256 contiguous bytes
// of one row, four rows per instruction) -> this wave's LDS tile -> MFMA fragments (lane (i, g) gets row i,
// k = 32u + 8g .. + 7 for the turn's k-step u).  Reading the fragments straight from global memory would
// make neighbouring lanes touch 16 different rows per instruction, which the memory pipeline punishes.
struct TileRegs { u32x4 q[4]; };

__device__ __forceinline__ void tile_load(TileRegs& r, const bf16_t* row0_k0, size_t row_stride, int k0, int K) {
    const int lane = threadIdx.x & 63;
    int k = k0 + (lane & 15) * 8;
    k = k <= K - 8 ? k : K - 8;                        // a ragged last turn re-reads valid bytes (those k-steps are skipped)
#pragma unroll
    for (int q = 0; q < 4; ++q) r.q[q] = load_stream16(row0_k0 + (size_t)(4 * q + (lane >> 4)) * row_stride + (k - k0));
}
__device__ __forceinline__ void tile_load_cached(TileRegs& r, const bf16_t* row0_k0, size_t row_stride, int k0, int K) {
    const int lane = threadIdx.x & 63;
    int k = k0 + (lane & 15) * 8;
    k = k <= K - 8 ? k : K - 8;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint4 v = *reinterpret_cast<const uint4*>(row0_k0 + (size_t)(4 * q + (lane >> 4)) * row_stride + (k - k0));
        r.q[q] = u32x4{v.x, v.y, v.z, v.w};
    }
}
// the packed B tile of up to 8 columns: tile rows 0..7 are the hi halves of columns 0..7, rows 8..15 their lo halves
__device__ __forceinline__ void tile_load_packed(TileRegs& r, const bf16_t* hi_k0, const bf16_t* lo_k0, size_t row_stride, int k0, int K) {
    const int lane = threadIdx.x & 63;
    int k = k0 + (lane & 15) * 8;
    k = k <= K - 8 ? k : K - 8;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bf16_t* base = q < 2 ? hi_k0 : lo_k0;
        const uint4 v = *reinterpret_cast<const uint4*>(base + (size_t)(4 * (q & 1) + (lane >> 4)) * row_stride + (k - k0));
        r.q[q] = u32x4{v.x, v.y, v.z, v.w};
    }
}
__device__ __forceinline__ void tile_to_frags(const TileRegs& r, char* tile, u32x4 (&frag)[U]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *reinterpret_cast<u32x4*>(tile + (4 * q + (lane >> 4)) * kTileRowBytes + (lane & 15) * 16) = r.q[q];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int u = 0; u < U; ++u)
        frag[u] = *reinterpret_cast<const u32x4*>(tile + (lane & 15) * kTileRowBytes + u * 64 + (lane >> 4) * 16);
    __builtin_amdgcn_wave_barrier();
}

template <int NT, int MODE, int RT, bool PACK>
__global__ __launch_bounds__(512) void gemm_mfma_kernel(GemvArgs a) {   // <= 8 waves
    constexpr int SW = (MODE == MODE_SWIGLU) ? 2 : 1;  // weight matrices per output tile
    constexpr int NA = RT * SW;                        // A tiles per wave
    constexpr int NB = PACK ? 1 : 2 * NT;              // B tiles per wave and turn (hi and lo of each column tile, or one packed tile)
    constexpr int ACC = NA * NT * 4;                   // accumulator floats per lane
    extern __shared__ float red[];                     // [waves][ACC][64] for the final sum; first, one staging tile per wave
    __shared__ float inv_rms[kMaxCols];                // RMSNorm scale of each column (input side)
    __shared__ float sq[MODE == MODE_RESID ? kMaxCols : 1][16 * RT];   // squares of the new residual (output side)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
    const int K = a.K, row0 = blockIdx.x * (16 * RT);
    char* tile = reinterpret_cast<char*>(red) + (size_t)wave * kTileBytes;

    const bf16_t* wrow[NA];                            // row 0 of each A tile
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        if (MODE == MODE_SWIGLU) {
            wrow[r * SW] = static_cast<const bf16_t*>(a.w[0]) + (size_t)(row0 + r * 16) * K;
            wrow[r * SW + SW - 1] = static_cast<const bf16_t*>(a.w[1]) + (size_t)(row0 + r * 16) * K;
        } else {
            int m = 0, local = row0 + r * 16;
            if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
            wrow[r] = static_cast<const bf16_t*>(a.w[m]) + (size_t)local * K;
        }
    }

    f32x4 acc[NA][NT];
#pragma unroll
    for (int r = 0; r < NA; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int nks = K / 32;
    const int stride = n_waves * U;
    TileRegs ga[NA], gb[NB];                           // the loads of one turn, in flight while the previous turn computes
    auto issue = [&](int ks0) {
        const int k0 = ks0 * 32;
        if constexpr (PACK) {
            tile_load_packed(gb[0], a.x_hi + k0, a.x_lo + k0, a.x_stride, k0, K);
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                tile_load_cached(gb[2 * t], a.x_hi + (size_t)(t * 16) * a.x_stride + k0, a.x_stride, k0, K);
                tile_load_cached(gb[2 * t + 1], a.x_lo + (size_t)(t * 16) * a.x_stride + k0, a.x_stride, k0, K);
            }
        }
#pragma unroll
        for (int r = 0; r < NA; ++r) tile_load(ga[r], wrow[r] + k0, K, k0, K);
    };
    // consume the turn held in ga/gb; when NEXT, re-issue each register set for turn ks_next as soon as it is in LDS
    auto turn = [&](int ks0, bool next, int ks_next) {
        u32x4 bf[NB][U];
        const int k1 = ks_next * 32;
        if constexpr (PACK) {
            tile_to_frags(gb[0], tile, bf[0]);
            if (next) tile_load_packed(gb[0], a.x_hi + k1, a.x_lo + k1, a.x_stride, k1, K);
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                tile_to_frags(gb[2 * t], tile, bf[2 * t]);
                if (next) tile_load_cached(gb[2 * t], a.x_hi + (size_t)(t * 16) * a.x_stride + k1, a.x_stride, k1, K);
                tile_to_frags(gb[2 * t + 1], tile, bf[2 * t + 1]);
                if (next) tile_load_cached(gb[2 * t + 1], a.x_lo + (size_t)(t * 16) * a.x_stride + k1, a.x_stride, k1, K);
            }
        }
#pragma unroll
        for (int r = 0; r < NA; ++r) {
            u32x4 af[U];
            tile_to_frags(ga[r], tile, af);
            if (next) tile_load(ga[r], wrow[r] + k1, K, k1, K);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (ks0 + u < nks) {
                    const bf16x8 wa = __builtin_bit_cast(bf16x8, af[u]);
                    if constexpr (PACK)
                        acc[r][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bf[0][u]), acc[r][0], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < (PACK ? 0 : NT); ++t) {
                        acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bf[2 * t][u]), acc[r][t], 0, 0, 0);
                        acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8, bf[2 * t + 1][u]), acc[r][t], 0, 0, 0);
                    }
                }
            }
        }
    };

    // 16 threads add up one column's partial sums of squares, in a fixed order; the loads queue behind the first
    // turn's weights and are consumed before it
    auto column_scales = [&]() {
        if (MODE == MODE_RESID || !a.ssq_in) return;
        for (int col = tid >> 4; col < a.ncols; col += blockDim.x >> 4) {
            const float* p = a.ssq_in + (size_t)col * kSsqStride;
            float ss = 0.f;
            for (int i0 = tid & 15; i0 < a.ssq_parts; i0 += 16 * 8) {
                float t[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) t[j] = i0 + 16 * j < a.ssq_parts ? p[i0 + 16 * j] : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) ss += t[j];
            }
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
            if ((tid & 15) == 0) inv_rms[col] = 1.0f / sqrtf(ss / (float)K + a.eps);
        }
    };

    int ks0 = wave * U;
    if (ks0 < nks) {
        issue(ks0);
        column_scales();
        while (ks0 + stride < nks) {                   // steady state: every register set is re-issued unconditionally
            turn(ks0, true, ks0 + stride);
            ks0 += stride;
        }
        turn(ks0, false, 0);
    } else {
        column_scales();
    }
    __syncthreads();                                   // the staging tiles give way to the partial sums

    // ---- sum the waves' partial tiles through LDS, then the epilogue ----
#pragma unroll
    for (int r = 0; r < NA; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[((size_t)wave * ACC + (r * NT + t) * 4 + e) * 64 + lane] = acc[r][t][e];
    __syncthreads();
    constexpr int OUT = RT * NT * 4;                   // outputs per lane (a gate/up pair folds into one)
    for (int idx = tid; idx < OUT * 64; idx += blockDim.x) {
        const int oi_ = idx >> 6, l = idx & 63;
        const int r = oi_ / (NT * 4), t = (oi_ >> 2) % NT, e = oi_ & 3;
        const int a0 = ((r * SW) * NT + t) * 4 + e;     // accumulator slot of the (gate) tile
        const int row = row0 + r * 16 + 4 * (l >> 4) + e, col = t * 16 + (l & 15);
        if (col >= a.ncols) continue;
        float s0 = 0.f, s1 = 0.f;
        for (int w = 0; w < n_waves; ++w) {
            s0 += red[((size_t)w * ACC + a0) * 64 + l];
            if (MODE == MODE_SWIGLU) s1 += red[((size_t)w * ACC + a0 + NT * 4) * 64 + l];
            if (PACK) {                                 // the lo halves sit eight columns further
                s0 += red[((size_t)w * ACC + a0) * 64 + l + 8];
                if (MODE == MODE_SWIGLU) s1 += red[((size_t)w * ACC + a0 + NT * 4) * 64 + l + 8];
            }
        }
        const size_t oi = (size_t)col * a.out_stride + row;
        if (MODE != MODE_RESID && a.ssq_in) { s0 *= inv_rms[col]; s1 *= inv_rms[col]; }
        float v;
        if (MODE == MODE_STORE) v = s0;
        else if (MODE == MODE_RESID) v = a.out[oi] + s0;
        else v = s0 / (1.0f + expf(-s0)) * s1;
        if (a.out) a.out[oi] = v;
        float split = v;
        if (MODE == MODE_RESID && a.ssq_out) {         // the consumer is a normalised projection: hand it x * gain and sum(x^2)
            sq[col][r * 16 + 4 * (l >> 4) + e] = v * v;
            split = v * a.gain_next[row];
        }
        if (a.out_hi) {
            const uint32_t hb = f32_to_bf16(split);
            a.out_hi[oi] = (bf16_t)hb;
            a.out_lo[oi] = (bf16_t)f32_to_bf16(split - bf16_to_f32(hb));
        }
    }
    if (MODE == MODE_RESID && a.ssq_out) {
        __syncthreads();
        if (tid < a.ncols) {
            float ss = 0.f;
#pragma unroll 4
            for (int i = 0; i < 16 * RT; ++i) ss += sq[tid][i];
            a.ssq_out[(size_t)tid * kSsqStride + blockIdx.x] = ss;
        }
    }
}

template <int NT, int MODE, bool PACK>
int launch_rt(const GemvArgs& a, int rt, int tiles, int waves, size_t lds, hipStream_t s) {
#define D3_LAUNCH(RT) hipLaunchKernelGGL((gemm_mfma_kernel<NT, MODE, RT, PACK>), dim3(tiles / RT), dim3(64 * waves), lds, s, a)
    if (rt == 4) { if (MODE == MODE_SWIGLU) return (int)hipErrorInvalidValue; D3_LAUNCH((MODE == MODE_SWIGLU ? 2 : 4)); }
    else if (rt == 2) D3_LAUNCH(2);
    else D3_LAUNCH(1);
#undef D3_LAUNCH
    return (int)hipGetLastError();
}

template <int NT, bool PACK>
int launch_mode(const GemvArgs& a, int mode, int rt, int tiles, int waves, size_t lds, hipStream_t s) {
    if (mode == MODE_STORE) return launch_rt<NT, MODE_STORE, PACK>(a, rt, tiles, waves, lds, s);
    if (mode == MODE_RESID) return launch_rt<NT, MODE_RESID, PACK>(a, rt, tiles, waves, lds, s);
    return launch_rt<NT, MODE_SWIGLU, PACK>(a, rt, tiles, waves, lds, s);
}

}  // namespace

// Requirements (checked by the caller): bf16 weights; K % 32 == 0; total_rows and every rows[m]
// multiples of 16; 1 <= ncols <= 32; x_hi/x_lo hold 32 rows of x_stride elements (rows beyond
// ncols may hold anything finite or not: their columns are never written); with ssq_out, total_rows / 16 <=
// kSsqStride (every workgroup owns a slot).
int launch_gemm_mfma(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups) {
    const int tiles = a.total_rows / 16;
    const int nt = a.ncols > 16 ? 2 : 1;
    if (a.ncols > 128 && a.part && tn.mfma_wide) return launch_gemm_prompt(a, mode, n_cu, tn, s, n_groups);
    if (nt == 2 && a.part && tn.mfma_wide) return launch_gemm_mfma_wide(a, mode, n_cu, tn, s, n_groups);
    if (a.ncols > kMaxCols) return (int)hipErrorInvalidValue;
    const int sw = mode == MODE_SWIGLU ? 2 : 1;
    const int turns = (a.K / 32 + U - 1) / U;                  // 128-k turns along K
    const bool pack = a.ncols <= 8;
    const int nb = pack ? 1 : 2 * nt;
    // Most tiles per workgroup (activation reuse) that still puts a workgroup on at least 0.6 of the compute units
    // (measured: fewer starve the memory system, more only add activation traffic) and >= 4 waves per CU on the
    // chip, within the register budget; stacked matrices must not share a workgroup
    // (rows[m] % (16 RT) == 0).
    int best_rt = 1, best_waves = 4;
    const int rt_max = (mode == MODE_SWIGLU ? 2 : 4) / nt;      // register budget: A tiles x column tiles per wave (more spills: measured 1.5-2.5x slower)
    const int rt_forced = tn.mfma_rt, waves_forced = tn.mfma_waves;
    for (int rt = rt_max; rt >= 1; rt /= 2) {
        if (tiles % rt != 0) continue;
        bool aligned = true;
        if (mode != MODE_SWIGLU)
            for (int m = 0; m < 3; ++m)
                if (a.rows[m] % (16 * rt) != 0) aligned = false;
        if (!aligned) continue;
        int waves = 32 / (rt * sw * (nb > 2 ? 2 : 1));
        if (waves > 8) waves = 8;
        while (waves > 4 && waves > turns) waves /= 2;         // at least one turn per wave
        if (waves < 4) continue;
        if (waves_forced) waves = waves_forced;
        best_rt = rt; best_waves = waves;
        // a gate/up pair doubles the bytes a wave keeps in flight: with workgroups to spare (>= 3 per CU at RT = 2)
        // one tile pair per wave ran faster (70B shape: 160 vs 176 us)
        if (!rt_forced && mode == MODE_SWIGLU && rt == 2 && tiles / 2 >= 3 * n_cu) continue;
        // ... and with too few of them (under 1.5 per CU) two pairs per wave starve the memory system
        // (7B shape, 4 columns: 344 workgroups 44.6 us, 688 of one pair 34.4 us; 13B shape: 432 of two pairs 50.1 us, 864 of one 52.8 us)
        if (!rt_forced && mode == MODE_SWIGLU && rt == 2 && 2 * (tiles / 2) < 3 * n_cu) continue;
        if (rt_forced ? rt <= rt_forced : (10 * (tiles / rt) >= 6 * n_cu && (long long)(tiles / rt) * waves >= 4LL * n_cu)) break;
    }
    if (n_groups) *n_groups = tiles / best_rt;
    if (a.ssq_out && tiles / best_rt > kSsqStride) return (int)hipErrorInvalidValue;
    size_t lds = (size_t)best_waves * best_rt * sw * nt * 4 * 64 * sizeof(float);   // cross-wave sum ...
    if (lds < (size_t)best_waves * kTileBytes) lds = (size_t)best_waves * kTileBytes;    // ... or one staging tile per wave
    if (nt == 2) return launch_mode<2, false>(a, mode, best_rt, tiles, best_waves, lds, s);
    if (pack) return launch_mode<1, true>(a, mode, best_rt, tiles, best_waves, lds, s);
    return launch_mode<1, false>(a, mode, best_rt, tiles, best_waves, lds, s);
}

}  // namespace d3
