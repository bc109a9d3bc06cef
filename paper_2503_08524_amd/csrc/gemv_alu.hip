// Weight-streaming GEMV for one (or a few) activation columns on the vector ALUs.
//
// This is the batch-1 decode projection: every weight byte is read from HBM
// exactly once, 16 bytes per lane per load, a whole wave reading 1 KiB of one
// weight row per instruction.  Activations sit in LDS as fp32 (laid out so that a
// wave's reads are conflict-free), accumulation is fp32, a row's dot product is
// finished with a wave reduction.  The RMSNorm of the input (fused QKV, gate/up
// and lm_head projections) is recomputed by every workgroup in its prologue: the
// input is a few KiB that stay in L2, which is cheaper than a separate launch.
// Each wave issues its share of the activation loads first and the loads of its first
// weight rows right behind them, so the two latencies overlap and the activations, being
// first in the queue, arrive first.
//
// Epilogues: plain store; residual add; SiLU(gate)*up; and, for the fused QKV
// projection, the rotary embedding plus the append of the new K/V row to the
// cache (a wave owns the two rows (j, j + hd/2) of a head that one rotation pairs).
#include "gemv_alu.h"

namespace d3 {

namespace {

template <typename W, int NC, int MODE, bool NORM>
__global__ __launch_bounds__(kGemvThreads) void gemv_alu_kernel(GemvArgs a) {
    extern __shared__ float4 xs[];                     // [NC][f4_per_col]
    __shared__ float red[NC][kGemvWaves];
    __shared__ GemvEpBuf<NC> ep[kGemvWaves];
    constexpr int R = kGemvStageR / NC;
    const int tid = threadIdx.x, wave = tid >> 6;
    // Units go round-robin over the waves of the whole grid, so that at any moment the chip streams one contiguous
    // band of the matrix (spread over every memory channel); numbering the waves workgroup-fastest hands the units
    // that do not divide evenly to different workgroups, one each.
    const int gw = wave * gridDim.x + blockIdx.x, nw = gridDim.x * kGemvWaves;
    GemvStageRegs<NC, R> regs;
    GemvPipe<W, kGemvDepth> pipe;
    gemv_stage_issue<NC, NORM, kGemvThreads, R>(a, tid, regs);          // activations first ...
    gemv_preload<W, MODE, kGemvDepth>(a, gw, nw, pipe);                          // ... the weight stream right behind them
    gemv_stage_commit<W, NC, NORM, kGemvThreads, R>(a, tid, xs, regs, red);
    __syncthreads();
    float rinv[NC];
    gemv_inv_rms<NC, NORM, kGemvWaves>(a, red, rinv);
    gemv_run<W, NC, MODE, kGemvDepth>(a, xs, gw, nw, pipe, ep[wave], rinv);
}

template <typename W, int NC>
int launch_nc(const GemvArgs& a, int mode, bool norm, int n_wg, hipStream_t s) {
    const size_t lds = (size_t)NC * gemv_f4_per_col<W>(a.K) * sizeof(float4);
    const int n_units = gemv_n_units(a, mode);
    // n_wg workgroups, a multiple of the CU count (a compute unit is the unit of bandwidth: the same number of
    // workgroups on each makes them finish together); fewer when there are not four units for each
    int grid = (n_units + kGemvWaves - 1) / kGemvWaves;
    if (grid > n_wg) grid = n_wg;
    if ((long long)grid * kGemvWaves * kGemvEpCap < n_units) return (int)hipErrorInvalidValue;   // a wave parks at most kGemvEpCap (= 64 lanes) units
#define D3_LAUNCH(MODE, NORM) hipLaunchKernelGGL((gemv_alu_kernel<W, NC, MODE, NORM>), dim3(grid), dim3(kGemvThreads), lds, s, a)
    if (mode == MODE_STORE) { if (norm) D3_LAUNCH(MODE_STORE, true); else D3_LAUNCH(MODE_STORE, false); }
    else if (mode == MODE_RESID) { D3_LAUNCH(MODE_RESID, false); }
    else if (mode == MODE_SWIGLU) { D3_LAUNCH(MODE_SWIGLU, true); }
    else { D3_LAUNCH(MODE_QKV_ROPE, true); }
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
    const size_t per_col = (size_t)(weight_dtype == 0 ? gemv_f4_per_col<float>(K) : gemv_f4_per_col<bf16_t>(K)) * sizeof(float4);
    size_t n = kGemvLdsBudget / per_col;
    return n >= 4 ? 4 : (n >= 2 ? 2 : (n >= 1 ? 1 : 0));
}

// Requirements (checked by the caller): K % 8 == 0, total_rows even, 1 <= ncols <= gemv_alu_max_cols,
// MODE_RESID without norm, MODE_SWIGLU / MODE_QKV_ROPE with norm, x/out/weights 16-byte aligned.
int launch_gemv_alu(const GemvArgs& a, int weight_dtype, int mode, bool norm, int n_wg, hipStream_t s) {
    return weight_dtype == 0 ? launch_w<float>(a, mode, norm, n_wg, s) : launch_w<bf16_t>(a, mode, norm, n_wg, s);
}

}  // namespace d3
