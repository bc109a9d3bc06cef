// Skinny GEMM on the matrix cores for 17..128 activation columns (large decode batches: up to 32; the chunked
// prompt pass: up to 128): out[col][row] = sum_k W[row][k] * x[col][k], bf16 weights, activations x = hi + lo.
//
// With 32 columns the activations of one 128-k turn are four 16 x 128 tiles (hi and lo of two column
// tiles), twice the bytes of a weight tile pair: a kernel whose waves each fetch and re-shape their own
// copy spends most of its registers and LDS traffic on them and keeps only 8 KB of weights per wave in
// flight.  Here the four waves of a workgroup walk the SAME k range and share ONE activation panel per
// turn in LDS (double-buffered, one barrier per turn); every wave owns RT of the workgroup's 4 * RT row
// tiles, keeps its weight tiles of TWO turns in flight, re-shapes them through a private LDS tile and
// takes the activation fragments from the panel.  The k range of a workgroup is one of gridDim.y slices
// of K (a matrix has too few row groups to fill the chip otherwise); a slice publishes its accumulators,
// and the slice that arrives last at the row group's counter adds them up in slice order (independent of
// arrival order) and runs the epilogue straight from registers.
//
// Operand layouts and the RMSNorm folding are those of gemm_mfma.hip.
#include <cstdlib>
#include <type_traits>

#include "d3_common.h"

namespace d3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int U = 4;                 // k-steps (of 32) per turn
constexpr int kPitch = 272;          // LDS pitch of a staged 16 x 256 B tile (+16 B: conflict-free fragment reads)
constexpr int kTile = 16 * kPitch;

struct TileRegs { u32x4 q[4]; };

__device__ __forceinline__ void tile_load(TileRegs& r, const bf16_t* row0, size_t row_stride, int k0, int K) {
    const int lane = threadIdx.x & 63;
    int k = k0 + (lane & 15) * 8;
    k = k <= K - 8 ? k : K - 8;                        // a ragged last turn re-reads valid bytes (those k-steps are skipped)
#pragma unroll
    for (int q = 0; q < 4; ++q) r.q[q] = load_stream16(row0 + (size_t)(4 * q + (lane >> 4)) * row_stride + k);
}
__device__ __forceinline__ void tile_to_frags(const TileRegs& r, char* tile, u32x4 (&frag)[U]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *reinterpret_cast<u32x4*>(tile + (4 * q + (lane >> 4)) * kPitch + (lane & 15) * 16) = r.q[q];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int u = 0; u < U; ++u)
        frag[u] = *reinterpret_cast<const u32x4*>(tile + (lane & 15) * kPitch + u * 64 + (lane >> 4) * 16);
    __builtin_amdgcn_wave_barrier();
}

// grid: (row groups of W * RT tiles, K slices).  CT column tiles (2: up to 32 columns, 4 waves per workgroup; 4: up to
// 64 columns, 8 waves per workgroup, so that the bigger panel is shared by more row tiles; 8: up to 128 columns, 4 waves
// with up to 512 registers each, the two panels fill the LDS).
// A gate/up pair of tiles per wave wants 204 registers (two waves per SIMD); its launch has 2.7 workgroups per CU, so at that
// size the last quarter of them starts only when the first ones have finished (entry times up to 24 us into a 42 us
// launch).  Held to three waves per SIMD (168 registers, 33 spilled) every workgroup starts at once: 42 -> 38 us.
template <int MODE, int RT, int CT, int W>
__global__ __launch_bounds__(W * 64, (MODE == MODE_SWIGLU && CT == 2) ? 3 : 1) void gemm_wide_kernel(GemvArgs a) {
    constexpr int SW = (MODE == MODE_SWIGLU) ? 2 : 1;
    constexpr int NA = RT * SW;                        // A tiles per wave and turn
    constexpr int NB = 2 * CT;                         // panel tiles: hi, lo of every column tile
    constexpr int kPanel = NB * kTile;
    constexpr int PBT = NB * 256 / (W * 64);           // 16-byte panel pieces per thread and turn (= 4)
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [2][kPanel] panels, then [W][kTile] staging tiles
    char (*panel)[kPanel] = reinterpret_cast<char (*)[kPanel]>(lds);
    char (*stage)[kTile] = reinterpret_cast<char (*)[kTile]>(lds + 2 * kPanel);
    __shared__ float inv_rms[CT * 16];
    __shared__ float ssq_w[W][CT * 16];
    __shared__ int is_last;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int K = a.K, nks = K / 32, turns = (nks + U - 1) / U;
    const int KS = gridDim.y;
    const int t_begin = (int)((long long)turns * blockIdx.y / KS), t_end = (int)((long long)turns * (blockIdx.y + 1) / KS);
    const int n_turns = t_end - t_begin;
    const int tiles = a.total_rows / 16;
    const int tile0 = (blockIdx.x * W + wave) * RT;
    char* atile = stage[wave];

    const bf16_t* wrow[NA];                            // row 0 of each A tile; tiles past the matrix re-read the last tile (result dropped)
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const int tile = tile0 + r < tiles ? tile0 + r : tiles - 1;
        if (MODE == MODE_SWIGLU) {
            wrow[r * SW] = static_cast<const bf16_t*>(a.w[0]) + (size_t)tile * 16 * K;
            wrow[r * SW + SW - 1] = static_cast<const bf16_t*>(a.w[1]) + (size_t)tile * 16 * K;
        } else {
            int m = 0, local = tile * 16;
            if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
            wrow[r] = static_cast<const bf16_t*>(a.w[m]) + (size_t)local * K;
        }
    }

    // this thread's pieces of the panel: start of the activation row, k offset inside a turn, LDS offset
    const bf16_t* psrc[PBT];
    int pdst[PBT];
    const int pseg = tid & 15;
#pragma unroll
    for (int i = 0; i < PBT; ++i) {
        const int cidx = tid + i * (W * 64), tb = cidx >> 8, r = (cidx >> 4) & 15;
        psrc[i] = ((tb & 1) ? a.x_lo : a.x_hi) + (size_t)((tb >> 1) * 16 + r) * a.x_stride;
        pdst[i] = tb * kTile + r * kPitch + pseg * 16;
    }

    f32x4 acc[NA][CT];
#pragma unroll
    for (int r = 0; r < NA; ++r)
#pragma unroll
        for (int tt = 0; tt < CT; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 pb[PBT];
    TileRegs ga[2][NA];                                // weight tiles of two turns in flight
    auto panel_issue = [&](int t) {
        int k = t * (U * 32) + pseg * 8;
        k = k <= K - 8 ? k : K - 8;
#pragma unroll
        for (int i = 0; i < PBT; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(psrc[i] + k);
            pb[i] = u32x4{v.x, v.y, v.z, v.w};
        }
    };
    auto panel_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PBT; ++i) *reinterpret_cast<u32x4*>(panel[buf] + pdst[i]) = pb[i];
    };
    // One turn.  Slot SLOT of ga and panel (t - t_begin) & 1 hold turn t.  A_ISSUE: turn t + 2 exists (its weights take
    // over each register set as soon as it is in LDS); P_STORE: turn t + 1 exists (its panel, in pb, goes to the other
    // buffer); P_ISSUE: turn t + 2 exists (its panel is requested).  The flags are compile-time so that every load of
    // the steady state is unconditional and the wait counts exact.
    auto turn = [&](int t, auto slot_c, auto a_issue, auto p_store, auto p_issue) {
        constexpr int SLOT = decltype(slot_c)::value;
        const int buf = (t - t_begin) & 1;
        const char* pan = panel[buf];
        auto b_frag = [&](int tile, int u) {
            return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(pan + tile * kTile + (lane & 15) * kPitch + u * 64 + (lane >> 4) * 16));
        };
        if constexpr (NA > 1 && CT >= 4) {
            // every A tile of the turn becomes fragments first, so that a panel fragment is read from LDS once and used for
            // all of them: with four column tiles the panel reads are most of the LDS traffic, and the LDS pipe, not HBM,
            // sets the pace of a turn (gate/up at 64 columns: 58.8 -> 49.7 us).  With two column tiles the 16 extra
            // registers cost more than the reads (batch-32 gate/up: 42.5 -> 50 us), so that shape keeps the order below.
            u32x4 af[NA][U];
#pragma unroll
            for (int r = 0; r < NA; ++r) {
                tile_to_frags(ga[SLOT][r], atile, af[r]);
                if (decltype(a_issue)::value) tile_load(ga[SLOT][r], wrow[r], K, (t + 2) * (U * 32), K);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (t * U + u < nks) {
#pragma unroll
                    for (int tt = 0; tt < CT; ++tt) {
                        const bf16x8 bh = b_frag(2 * tt, u), bl = b_frag(2 * tt + 1, u);
#pragma unroll
                        for (int r = 0; r < NA; ++r) acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[r][u]), bh, acc[r][tt], 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < NA; ++r) acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[r][u]), bl, acc[r][tt], 0, 0, 0);
                    }
                }
            }
        } else {
#pragma unroll
            for (int r = 0; r < NA; ++r) {
                u32x4 af[U];
                tile_to_frags(ga[SLOT][r], atile, af);
                if (decltype(a_issue)::value) tile_load(ga[SLOT][r], wrow[r], K, (t + 2) * (U * 32), K);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (t * U + u < nks) {
                        const bf16x8 wa = __builtin_bit_cast(bf16x8, af[u]);
#pragma unroll
                        for (int tt = 0; tt < CT; ++tt) {
                            acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, b_frag(2 * tt, u), acc[r][tt], 0, 0, 0);
                            acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, b_frag(2 * tt + 1, u), acc[r][tt], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if (decltype(p_store)::value) panel_store(buf ^ 1);
        if (decltype(p_issue)::value) panel_issue(t + 2);
        __syncthreads();                               // panel t + 1 is complete; nobody still reads panel t
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;

    // 16 threads add up one column's partial sums of squares, in a fixed order
    auto column_scales = [&]() {
        if (MODE == MODE_RESID || !a.ssq_in) return;
        for (int col = tid >> 4; col < a.ncols; col += (W * 64) >> 4) {
            const float* p = a.ssq_in + (size_t)col * kSsqStride;
            float ss = 0.f;
            for (int i0 = tid & 15; i0 < a.ssq_parts; i0 += 16 * 8) {
                float tv[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) tv[j] = i0 + 16 * j < a.ssq_parts ? p[i0 + 16 * j] : 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) ss += tv[j];
            }
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
            if ((tid & 15) == 0) inv_rms[col] = 1.0f / sqrtf(ss / (float)K + a.eps);
        }
    };

    if (n_turns > 0) {
        int t = t_begin;
        panel_issue(t);
#pragma unroll
        for (int r = 0; r < NA; ++r) tile_load(ga[0][r], wrow[r], K, t * (U * 32), K);
        if (n_turns > 1) {
#pragma unroll
            for (int r = 0; r < NA; ++r) tile_load(ga[1][r], wrow[r], K, (t + 1) * (U * 32), K);
        }
        panel_store(0);
        if (n_turns > 1) panel_issue(t + 1);
        column_scales();
        __syncthreads();
        for (; t + 3 < t_end; t += 2) {                // steady state: every load is unconditional
            turn(t, S0{}, T_{}, T_{}, T_{});
            turn(t + 1, S1{}, T_{}, T_{}, T_{});
        }
        const int left = t_end - t;
        if (left == 3) { turn(t, S0{}, T_{}, T_{}, T_{}); turn(t + 1, S1{}, F_{}, T_{}, F_{}); turn(t + 2, S0{}, F_{}, F_{}, F_{}); }
        else if (left == 2) { turn(t, S0{}, F_{}, T_{}, F_{}); turn(t + 1, S1{}, F_{}, F_{}, F_{}); }
        else { turn(t, S0{}, F_{}, F_{}, F_{}); }
    } else {
        column_scales();
        __syncthreads();
    }

    // ---- K slices: publish, count arrivals, the last one adds the slices up in order ----
    constexpr int ACC = NA * CT * 4;
    if (KS > 1) {
        float* mine = a.part + (((size_t)blockIdx.x * KS + blockIdx.y) * W + wave) * (ACC * 64) + lane;
#pragma unroll
        for (int r = 0; r < NA; ++r)
#pragma unroll
            for (int tt = 0; tt < CT; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) st_agent(mine + ((r * CT + tt) * 4 + e) * 64, acc[r][tt][e]);
        wait_stores();                                 // this slice's partials have reached the coherence point
        __syncthreads();
        if (tid == 0) {
            int* ticket = &a.part_tickets[blockIdx.x];
            const int done = atomicAdd(ticket, 1);
            is_last = done == KS - 1;
            if (is_last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // all arrived: leave it clean
        }
        __syncthreads();
        if (!is_last) return;
#pragma unroll
        for (int r = 0; r < NA; ++r)
#pragma unroll
            for (int tt = 0; tt < CT; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
        // a few slices per round trip: all their loads are issued before the first is added (slice order is kept)
        constexpr int RND = ACC > 16 ? 2 : 4;          // slices per round trip (register budget)
        for (int ks0 = 0; ks0 < KS; ks0 += RND) {
            float v[RND][ACC];
#pragma unroll
            for (int q = 0; q < RND; ++q) {
                const int ks = ks0 + q < KS ? ks0 + q : KS - 1;
                const float* p = a.part + (((size_t)blockIdx.x * KS + ks) * W + wave) * (ACC * 64) + lane;
#pragma unroll
                for (int j = 0; j < ACC; ++j) v[q][j] = ld_agent(p + j * 64);
            }
#pragma unroll
            for (int q = 0; q < RND; ++q) {
                if (ks0 + q < KS) {
#pragma unroll
                    for (int r = 0; r < NA; ++r)
#pragma unroll
                        for (int tt = 0; tt < CT; ++tt)
#pragma unroll
                            for (int e = 0; e < 4; ++e) acc[r][tt][e] += v[q][(r * CT + tt) * 4 + e];
                }
            }
        }
    }

    // ---- epilogue from the accumulators: lane (i, g) holds column i of a column tile, rows 4g..4g+3 of each tile ----
    const int ci = lane & 15, g4 = lane >> 4;
    float sq[CT];                                      // this lane's share of sum(x_new^2) of columns ci, 16 + ci, ...
#pragma unroll
    for (int tt = 0; tt < CT; ++tt) sq[tt] = 0.f;
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        if (tile0 + r >= tiles) continue;
#pragma unroll
        for (int tt = 0; tt < CT; ++tt) {
            const int col = tt * 16 + ci;
            if (col >= a.ncols) continue;
            const int row = (tile0 + r) * 16 + 4 * g4;
            const size_t oi = (size_t)col * a.out_stride + row;
            f32x4 s0 = acc[r * SW][tt];
            float v[4], split[4];
            if (MODE == MODE_STORE) {
                const float sc = a.ssq_in ? inv_rms[col] : 1.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = s0[e] * sc;
            } else if (MODE == MODE_RESID) {
                const float4 o = *reinterpret_cast<const float4*>(a.out + oi);
                v[0] = o.x + s0[0]; v[1] = o.y + s0[1]; v[2] = o.z + s0[2]; v[3] = o.w + s0[3];
            } else {
                const f32x4 s1 = acc[r * SW + SW - 1][tt];
                const float sc = a.ssq_in ? inv_rms[col] : 1.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) { const float gt = s0[e] * sc; v[e] = gt / (1.0f + expf(-gt)) * (s1[e] * sc); }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) split[e] = v[e];
            if (MODE == MODE_RESID && a.ssq_out) {     // the consumer is a normalised projection: hand it x * gain and sum(x^2)
                const float4 gn = *reinterpret_cast<const float4*>(a.gain_next + row);
                sq[tt] += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
                split[0] = v[0] * gn.x; split[1] = v[1] * gn.y; split[2] = v[2] * gn.z; split[3] = v[3] * gn.w;
            }
            if (a.out) *reinterpret_cast<float4*>(a.out + oi) = make_float4(v[0], v[1], v[2], v[3]);
            if (a.out_hi) {
                uint32_t hb[4], lb[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    hb[e] = f32_to_bf16(split[e]);
                    lb[e] = f32_to_bf16(split[e] - bf16_to_f32(hb[e]));
                }
                *reinterpret_cast<uint2*>(a.out_hi + oi) = make_uint2(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16));
                *reinterpret_cast<uint2*>(a.out_lo + oi) = make_uint2(lb[0] | (lb[1] << 16), lb[2] | (lb[3] << 16));
            }
        }
    }
    if (MODE == MODE_RESID && a.ssq_out) {             // rows of a column: the 4 lane groups by butterfly, then the waves in order
#pragma unroll
        for (int tt = 0; tt < CT; ++tt) {
            sq[tt] += __shfl_xor(sq[tt], 16, 64);
            sq[tt] += __shfl_xor(sq[tt], 32, 64);
            if (g4 == 0) ssq_w[wave][tt * 16 + ci] = sq[tt];
        }
        __syncthreads();
        if (tid < a.ncols) {
            float ss = 0.f;
#pragma unroll
            for (int w = 0; w < W; ++w) ss += ssq_w[w][tid];
            a.ssq_out[(size_t)tid * kSsqStride + blockIdx.x] = ss;
        }
    }
}

template <int MODE, int RT, int CT, int W>
int launch_one(const GemvArgs& a, int groups, int ks, hipStream_t s) {
    constexpr size_t lds = (size_t)(2 * 2 * CT + W) * kTile;
    auto* k = gemm_wide_kernel<MODE, RT, CT, W>;
    if (lds > 48 * 1024) {
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (once != hipSuccess) return (int)once;
    }
    hipLaunchKernelGGL(k, dim3(groups, ks), dim3(W * 64), lds, s, a);
    return (int)hipGetLastError();
}

template <int MODE>
int launch_rt(const GemvArgs& a, int ct, int rt, int groups, int ks, hipStream_t s) {
    if (ct == 8) {
        if constexpr (MODE != MODE_SWIGLU) { if (rt == 2) return launch_one<MODE, 2, 8, 4>(a, groups, ks, s); }
        return launch_one<MODE, 1, 8, 4>(a, groups, ks, s);
    }
    if (ct == 4) {
        if constexpr (MODE != MODE_SWIGLU) { if (rt == 2) return launch_one<MODE, 2, 4, 8>(a, groups, ks, s); }
        return launch_one<MODE, 1, 4, 8>(a, groups, ks, s);
    }
    if (rt == 2) {
        if constexpr (MODE == MODE_SWIGLU) return (int)hipErrorInvalidValue;
        else return launch_one<MODE, 2, 2, 4>(a, groups, ks, s);
    }
    return launch_one<MODE, 1, 2, 4>(a, groups, ks, s);
}

}  // namespace

// Requirements: those of launch_gemm_mfma, 17 <= ncols <= kPassCols (x_hi / x_lo hold kPassCols rows); a.part holds kGemmPartBytes and a.part_tickets
// kGemmPartTickets zeroed counters (the kernel leaves them zero).
namespace {

int launch_config(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups, int force_ct);

// Column halves of a pass of more than 64 columns, both with the 64-column kernel (the same row groups, so the partial
// sums of squares of all columns have one layout).
int launch_halves(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups) {
    GemvArgs lo = a;
    lo.ncols = 64;
    int rc = launch_config(lo, mode, n_cu, tn, s, n_groups, 4);
    if (rc != 0) return rc;
    GemvArgs hi = a;
    hi.ncols = a.ncols - 64;
    hi.x_hi += (size_t)64 * a.x_stride; hi.x_lo += (size_t)64 * a.x_stride;
    if (hi.out) hi.out += (size_t)64 * a.out_stride;
    if (hi.out_hi) { hi.out_hi += (size_t)64 * a.out_stride; hi.out_lo += (size_t)64 * a.out_stride; }
    if (hi.ssq_in) hi.ssq_in += (size_t)64 * kSsqStride;
    if (hi.ssq_out) hi.ssq_out += (size_t)64 * kSsqStride;
    return launch_config(hi, mode, n_cu, tn, s, nullptr, 4);
}

}  // namespace

int launch_gemm_mfma_wide(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups) {
    // More than 64 columns: one launch of the 128-column kernel (four waves per workgroup) when the matrix is small enough
    // for its fixed costs to matter, else two of the 64-column kernel, whose eight-wave workgroups stream a large matrix
    // faster (70B shape, per 128 columns: gate/up 940 MB 396 against 330 us, down 470 MB 252 against 224 us; QKV 168 MB 85
    // against 95 us, O 134 MB 84 against 100 us)
    const size_t weight_bytes = (size_t)a.total_rows * a.K * 2 * (mode == MODE_SWIGLU ? 2 : 1);
    if (a.ncols > 64 && weight_bytes > (tn.wide_split_mb << 20)) return launch_halves(a, mode, n_cu, tn, s, n_groups);
    return launch_config(a, mode, n_cu, tn, s, n_groups, 0);
}

namespace {

int launch_config(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups, int force_ct) {
    const int tiles = a.total_rows / 16;
    const int sw = mode == MODE_SWIGLU ? 2 : 1;
    const int turns = (a.K / 32 + U - 1) / U;
    // Measured at the 7B shape with 32 columns: one tile (pair) per wave beats two, and the launch is fastest when
    // its workgroups number about three per CU (what fits at once): K slices make up for the few row groups,
    // at least four turns each and at most eight of them (the publish / arrive / merge of the slices is not free).
    const int ct = force_ct ? force_ct : a.ncols > 64 ? 8 : a.ncols > 32 ? 4 : 2;   // column tiles
    const int w = ct == 4 ? 8 : 4;                     // waves per workgroup
    int rt = 1;
    // 64 columns, one stacked matrix (QKV, lm_head): two row tiles per wave share the panel fragments and put the whole
    // launch on the chip at once (7B QKV: 240 workgroups, 37.8 -> 30.9 us); the residual projections have too few row
    // tiles for that (down-projection: 128 workgroups, 32.6 -> 44 us)
    if (ct == 4 && mode == MODE_STORE) rt = 2;
    if (ct == 8) rt = mode == MODE_STORE ? 2 : 1;
    if (const int v = tn.wide_rt) if (ct != 8 && (v == 1 || mode != MODE_SWIGLU)) rt = v;
    int groups = (tiles + w * rt - 1) / (w * rt);
    // up to 32 columns: three workgroups fit a CU; up to 64: one (its panels fill most of the LDS)
    int ks = (ct == 8 ? 1 : ct == 4 ? 2 : 3) * n_cu / groups;
    if (ks > 8) ks = 8;
    if (const int v = tn.wide_ks) ks = v;
    if (ks > turns / 4) ks = turns / 4;
    if (ks < 1) ks = 1;
    while (ks > 1 && (size_t)groups * ks * w * (rt * sw * ct * 4) * 64 * sizeof(float) > kGemmPartBytes) --ks;
    if (groups > kGemmPartTickets) return (int)hipErrorInvalidValue;
    if (a.ssq_out && groups > kSsqStride) return (int)hipErrorInvalidValue;
    if (n_groups) *n_groups = groups;
    if (mode == MODE_STORE) return launch_rt<MODE_STORE>(a, ct, rt, groups, ks, s);
    if (mode == MODE_RESID) return launch_rt<MODE_RESID>(a, ct, rt, groups, ks, s);
    return launch_rt<MODE_SWIGLU>(a, ct, rt, groups, ks, s);
}

}  // namespace

}  // namespace d3
