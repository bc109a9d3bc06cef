// Device-side phases of the vector-ALU GEMV (see gemv_alu.hip).
//
// A wave walks its work as a sequence of "steps": one step = the two weight rows of a unit
// at one 64-lane stride (2 x 1 KiB per wave).  Loads run D steps ahead of the arithmetic in
// a ring of registers whose slots are compile-time indices, so the compiler's wait counts
// stay exact: in the steady state every lane always has 2*D sixteen-byte loads in flight.
#pragma once
#include "d3_common.h"

namespace d3 {

#ifndef D3_GEMV_WAVES
#define D3_GEMV_WAVES 4
#endif
constexpr int kGemvWaves = D3_GEMV_WAVES;   // waves per workgroup (they share the staged activations)
constexpr int kGemvThreads = kGemvWaves * kWave;
constexpr int kGemvStageR = 12;             // float4 activation loads a thread issues ahead of the weights (K <= 12288 in one round)
constexpr int kGemvLdsBudget = 60 * 1024;   // dynamic LDS per workgroup for the activations
#ifndef D3_GEMV_DEPTH
#define D3_GEMV_DEPTH 4
#endif
constexpr int kGemvDepth = D3_GEMV_DEPTH;   // steps in flight per wave (2 KiB each)
constexpr int kGemvEpCap = 64;              // finished units a wave can hold before writing them out

template <typename W> struct GemvChunk;                // one 16-byte piece of a weight row
template <> struct GemvChunk<float> { static constexpr int N = 4; };
template <> struct GemvChunk<bf16_t> { static constexpr int N = 8; };

// Position (in float4 units) of activation element k inside one column's LDS image.
// bf16 weights: a lane consumes 8 consecutive activations per chunk; they are stored as
// two float4 planes so that lanes of a wave read consecutive 16-byte words.
template <typename W> __device__ __forceinline__ int gemv_f4_index(int k);
template <> __device__ __forceinline__ int gemv_f4_index<float>(int k) { return k >> 2; }
template <> __device__ __forceinline__ int gemv_f4_index<bf16_t>(int k) {
    const int q = k >> 3;
    return (((q >> 6) << 1) + ((k >> 2) & 1)) * 64 + (q & 63);
}
// float4 slots of one column's image: whole 64-lane strides, the tail beyond K zero-filled
template <typename W> __host__ __device__ inline int gemv_f4_per_col(int K) {
    const int chunks = K / GemvChunk<W>::N;
    const int strides = (chunks + 63) / 64;
    return strides * 64 * (sizeof(W) == 4 ? 1 : 2);
}

// Work units: one output row of gate and up (SWIGLU), the rotation pair (j, j + hd/2) of one head
// (QKV_ROPE), else two consecutive output rows.
__host__ __device__ inline int gemv_n_units(const GemvArgs& a, int mode) {
    if (mode == MODE_SWIGLU) return a.total_rows;
    return a.total_rows / 2;
}

template <typename W, int MODE>
__device__ __forceinline__ void gemv_unit_rows(const GemvArgs& a, int u, const W*& r0, const W*& r1, int& row) {
    const int K = a.K;
    if (MODE == MODE_SWIGLU) {
        row = u;
        r0 = static_cast<const W*>(a.w[0]) + (size_t)u * K;
        r1 = static_cast<const W*>(a.w[1]) + (size_t)u * K;
    } else {
        int step;
        if (MODE == MODE_QKV_ROPE) {
            const int half = a.hd >> 1;
            row = (u / half) * a.hd + (u % half);
            step = half;
        } else {
            row = 2 * u;
            step = 1;
        }
        int m = 0, local = row;
        if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
        r0 = static_cast<const W*>(a.w[m]) + (size_t)local * K;
        r1 = r0 + (size_t)step * K;
    }
}

// The load side of a wave's pipeline.
template <typename W, int D>
struct GemvPipe {
    u32x4 b0[D], b1[D];   // ring of loaded chunks: slot j holds step (issued - D + j) mod D ...
    const W *r0, *r1;     // rows of the unit being loaded
    int lu, lit;          // unit and stride of the next step to load
    int issued, total;    // steps loaded so far / steps this wave owns in this phase
};

template <typename W, int MODE, int D>
__device__ __forceinline__ void gemv_issue(const GemvArgs& a, GemvPipe<W, D>& p, int slot, int nw, int n_units, int nchunks, int S) {
    constexpr int EPC = GemvChunk<W>::N;
    const int lane = threadIdx.x & 63;
    int q = lane + 64 * p.lit;
    q = q < nchunks ? q : nchunks - 1;                 // ragged last stride: reload a valid chunk (its activations are zero)
    p.b0[slot] = load_stream16(p.r0 + (size_t)q * EPC);
    p.b1[slot] = load_stream16(p.r1 + (size_t)q * EPC);
    p.issued += 1;
    if (++p.lit == S) {
        p.lit = 0;
        p.lu += nw;
        int row;
        gemv_unit_rows<W, MODE>(a, p.lu < n_units ? p.lu : n_units - 1, p.r0, p.r1, row);
    }
}

// Start a phase: fill the ring with the wave's first D steps.  All D loads are issued whatever the
// wave's share is (a wave with fewer steps re-reads valid rows), which keeps the wait counts exact.
template <typename W, int MODE, int D>
__device__ __forceinline__ void gemv_preload(const GemvArgs& a, int gw, int nw, GemvPipe<W, D>& p) {
    const int n_units = gemv_n_units(a, MODE);
    const int nchunks = a.K / GemvChunk<W>::N;
    const int S = (nchunks + 63) / 64;
    const int mine = gw < n_units ? (n_units - gw + nw - 1) / nw : 0;
    p.total = mine * S;
    p.issued = 0;
    p.lu = gw;
    p.lit = 0;
    int row;
    gemv_unit_rows<W, MODE>(a, gw < n_units ? gw : n_units - 1, p.r0, p.r1, row);
#pragma unroll
    for (int j = 0; j < D; ++j) gemv_issue<W, MODE, D>(a, p, j, nw, n_units, nchunks, S);
}

// Activations -> LDS (fp32), in two halves so that a kernel can put its weight preload in between:
// the activation loads are issued FIRST and therefore return first (vector memory returns in order
// within a wave, and the memory system is a queue: a load issued behind 16 KiB per wave of weight
// loads comes back several microseconds later).
//   gemv_stage_issue:  each of THREADS threads issues up to R float4 loads per column (+ gains);
//   gemv_stage_commit: writes them to LDS (x * gain when NORM), handles what exceeds R * THREADS
//                      float4s in further rounds, and leaves each wave's partial sum of squares in red.
// After the workgroup barrier that must follow, gemv_inv_rms gives 1/sqrt(mean(x^2) + eps) per column;
// it is applied to the finished dot products.
template <int NC, int R>
struct GemvStageRegs {
    float4 v[NC][R];
    float4 g[R];
};

template <int NC, bool NORM, int THREADS, int R>
__device__ __forceinline__ void gemv_stage_issue(const GemvArgs& a, int tid, GemvStageRegs<NC, R>& regs) {
    const int f4_used = a.K / 4;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i4 = tid + r * THREADS;
        regs.g[r] = make_float4(1.f, 1.f, 1.f, 1.f);
        if (NORM && i4 < f4_used) regs.g[r] = *reinterpret_cast<const float4*>(a.gain + i4 * 4);
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            regs.v[n][r] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < a.ncols && i4 < f4_used) regs.v[n][r] = *reinterpret_cast<const float4*>(a.x + (size_t)n * a.x_stride + i4 * 4);
        }
    }
}

template <typename W, int NC, bool NORM, int THREADS, int R>
__device__ __forceinline__ void gemv_stage_commit(const GemvArgs& a, int tid, float4* xs, GemvStageRegs<NC, R>& regs,
                                                  float (*red)[THREADS / 64]) {
    const int K = a.K;
    const int f4_per_col = gemv_f4_per_col<W>(K);     // slots of the image; those past K/4 are the zero tail
    const int f4_used = K / 4;
    float ss[NC];
#pragma unroll
    for (int n = 0; n < NC; ++n) ss[n] = 0.f;
    auto put = [&](int i4, int n, float4 t, const float4& g) {
        if (NORM) {
            ss[n] += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
            t.x *= g.x; t.y *= g.y; t.z *= g.z; t.w *= g.w;
        }
        xs[n * f4_per_col + gemv_f4_index<W>(i4 * 4)] = t;
    };
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i4 = tid + r * THREADS;
        if (i4 < f4_per_col) {
#pragma unroll
            for (int n = 0; n < NC; ++n) put(i4, n, regs.v[n][r], regs.g[r]);
        }
    }
    for (int i4 = tid + R * THREADS; i4 < f4_per_col; i4 += THREADS) {      // wide inputs: the rest, one at a time
        float4 g = make_float4(1.f, 1.f, 1.f, 1.f);
        if (NORM && i4 < f4_used) g = *reinterpret_cast<const float4*>(a.gain + i4 * 4);
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < a.ncols && i4 < f4_used) t = *reinterpret_cast<const float4*>(a.x + (size_t)n * a.x_stride + i4 * 4);
            put(i4, n, t, g);
        }
    }
    if (NORM) {
        const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            const float s = wave_sum(ss[n]);
            if (lane == 0) red[n][wave] = s;
        }
    }
}

template <int NC, bool NORM, int WAVES>
__device__ __forceinline__ void gemv_inv_rms(const GemvArgs& a, float (*red)[WAVES], float (&rinv)[NC]) {
#pragma unroll
    for (int n = 0; n < NC; ++n) {
        rinv[n] = 1.0f;
        if (NORM) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) s += red[n][w];
            rinv[n] = 1.0f / sqrtf(s / (float)a.K + a.eps);
        }
    }
}

// One step of both rows against the staged activations.
template <typename W, int NC>
__device__ __forceinline__ void gemv_fma_step(const u32x4& w0, const u32x4& w1, const float4* xs, int f4_per_col, int stride,
                                              float (&acc0)[NC], float (&acc1)[NC]) {
    const int lane = threadIdx.x & 63;
    if (sizeof(W) == 4) {
        const float a0 = __uint_as_float(w0.x), a1 = __uint_as_float(w0.y), a2 = __uint_as_float(w0.z), a3 = __uint_as_float(w0.w);
        const float b0 = __uint_as_float(w1.x), b1 = __uint_as_float(w1.y), b2 = __uint_as_float(w1.z), b3 = __uint_as_float(w1.w);
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            const float4 x = xs[n * f4_per_col + stride * 64 + lane];
            acc0[n] = fmaf(a0, x.x, acc0[n]); acc0[n] = fmaf(a1, x.y, acc0[n]); acc0[n] = fmaf(a2, x.z, acc0[n]); acc0[n] = fmaf(a3, x.w, acc0[n]);
            acc1[n] = fmaf(b0, x.x, acc1[n]); acc1[n] = fmaf(b1, x.y, acc1[n]); acc1[n] = fmaf(b2, x.z, acc1[n]); acc1[n] = fmaf(b3, x.w, acc1[n]);
        }
    } else {
        const int base = stride * 128 + lane;
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            const float4 xa = xs[n * f4_per_col + base];
            const float4 xb = xs[n * f4_per_col + base + 64];
            acc0[n] = fmaf(bf16_lo(w0.x), xa.x, acc0[n]); acc0[n] = fmaf(bf16_hi(w0.x), xa.y, acc0[n]);
            acc0[n] = fmaf(bf16_lo(w0.y), xa.z, acc0[n]); acc0[n] = fmaf(bf16_hi(w0.y), xa.w, acc0[n]);
            acc0[n] = fmaf(bf16_lo(w0.z), xb.x, acc0[n]); acc0[n] = fmaf(bf16_hi(w0.z), xb.y, acc0[n]);
            acc0[n] = fmaf(bf16_lo(w0.w), xb.z, acc0[n]); acc0[n] = fmaf(bf16_hi(w0.w), xb.w, acc0[n]);
            acc1[n] = fmaf(bf16_lo(w1.x), xa.x, acc1[n]); acc1[n] = fmaf(bf16_hi(w1.x), xa.y, acc1[n]);
            acc1[n] = fmaf(bf16_lo(w1.y), xa.z, acc1[n]); acc1[n] = fmaf(bf16_hi(w1.y), xa.w, acc1[n]);
            acc1[n] = fmaf(bf16_lo(w1.z), xb.x, acc1[n]); acc1[n] = fmaf(bf16_hi(w1.z), xb.y, acc1[n]);
            acc1[n] = fmaf(bf16_lo(w1.w), xb.z, acc1[n]); acc1[n] = fmaf(bf16_hi(w1.w), xb.w, acc1[n]);
        }
    }
}

// Store one element of a new cache row in the cache's element type.
__device__ __forceinline__ void kv_store(void* base, size_t idx, int kv_dtype, float v) {
    if (kv_dtype == 0) static_cast<float*>(base)[idx] = v;
    else static_cast<f16_t*>(base)[idx] = (f16_t)fminf(fmaxf(v, -65504.f), 65504.f);
}
// The value a later read of that cache element returns.
__device__ __forceinline__ float kv_round(int kv_dtype, float v) {
    if (kv_dtype == 0) return v;
    return (float)(f16_t)fminf(fmaxf(v, -65504.f), 65504.f);
}

// Finished units wait in LDS until the phase's loads have drained: their write-out needs loads of
// its own (residual, rotary table), which would otherwise stall the weight stream.
template <int NC>
struct GemvEpBuf {
    float s[kGemvEpCap][NC][2];
    int row[kGemvEpCap];
};

// Write-out of one finished unit for column n.
template <int MODE>
__device__ __forceinline__ void gemv_epilogue(const GemvArgs& a, int n, int row, float s0, float s1) {
    float* o = a.out + (size_t)n * a.out_stride + row;
    auto put = [](float* p, float v) { *p = v; };
    if (MODE == MODE_STORE) { put(o, s0); put(o + 1, s1); }
    else if (MODE == MODE_RESID) { }                   // handled in gemv_run with the prefetched residual
    else if (MODE == MODE_SWIGLU) { put(o, s0 / (1.0f + expf(-s0)) * s1); }
    else {
        // rows (j, j + hd/2) of one head: rotate q and k by the column's position, append k and v
        const int half = a.hd >> 1, head = row / a.hd, j = row % a.hd;
        const int c = a.col0 + n;
        if (head < a.H + a.H_kv) {
            const float2 cs = a.rope_cs[(size_t)c * half + j];
            const float y0 = s0 * cs.x - s1 * cs.y, y1 = s0 * cs.y + s1 * cs.x;
            s0 = y0; s1 = y1;
        }
        if (head >= a.H) {
            const bool is_k = head < a.H + a.H_kv;
            const int kvh = is_k ? head - a.H : head - a.H - a.H_kv;
            const size_t idx = (((size_t)a.cm.seq(c) * a.H_kv + kvh) * a.max_seq + a.cm.pos(c)) * a.hd + j;
            void* base = is_k ? a.k_cache : a.v_cache;
            kv_store(base, idx, a.kv_dtype, s0);
            kv_store(base, idx + half, a.kv_dtype, s1);
        }
        if (head < a.H) { put(o, s0); put(o + half, s1); }   // q
    }
}

template <int NC, int MODE>
__device__ __forceinline__ void gemv_flush(const GemvArgs& a, const GemvEpBuf<NC>& ep, int n_ep) {
    const int lane = threadIdx.x & 63;
    for (int e = lane; e < n_ep; e += 64) {
#pragma unroll
        for (int n = 0; n < NC; ++n)
            if (n < a.ncols) gemv_epilogue<MODE>(a, n, ep.row[e], ep.s[e][n][0], ep.s[e][n][1]);
    }
}

// Main loop of a phase: consume the wave's steps, keeping the ring full.  `ep` is this wave's buffer.
template <typename W, int NC, int MODE, int D>
__device__ __forceinline__ void gemv_run(const GemvArgs& a, const float4* xs, int gw, int nw, GemvPipe<W, D>& p, GemvEpBuf<NC>& ep,
                                         const float (&scale)[NC]) {
    const int lane = threadIdx.x & 63;
    const int f4_per_col = gemv_f4_per_col<W>(a.K);
    const int nchunks = a.K / GemvChunk<W>::N;
    const int S = (nchunks + 63) / 64;
    const int n_units = gemv_n_units(a, MODE);
    const int total = p.total;
    int cu = gw, cit = 0, n_ep = 0;
    // residual mode: lane e fetches the old values of the rows of this wave's e-th unit now, long before they are needed
    float res0[NC], res1[NC];
    if (MODE == MODE_RESID) {
        const int e_unit = gw + lane * nw;
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            res0[n] = 0.f; res1[n] = 0.f;
            if (e_unit < n_units && n < a.ncols) {
                const float* o = a.out + (size_t)n * a.out_stride + 2 * e_unit;
                const float2 v = *reinterpret_cast<const float2*>(o);
                res0[n] = v.x; res1[n] = v.y;
            }
        }
    }
    float acc0[NC], acc1[NC];
#pragma unroll
    for (int n = 0; n < NC; ++n) { acc0[n] = 0.f; acc1[n] = 0.f; }

    auto consume = [&](int slot) {
        gemv_fma_step<W, NC>(p.b0[slot], p.b1[slot], xs, f4_per_col, cit, acc0, acc1);
        if (++cit == S) {                               // unit finished: park its sums
            int row;
            const W *r0, *r1;
            gemv_unit_rows<W, MODE>(a, cu, r0, r1, row);
#pragma unroll
            for (int n = 0; n < NC; ++n) {
                const float s0 = wave_sum(acc0[n]) * scale[n], s1 = wave_sum(acc1[n]) * scale[n];
                if (lane == 0) { ep.s[n_ep][n][0] = s0; ep.s[n_ep][n][1] = s1; }
                acc0[n] = 0.f; acc1[n] = 0.f;
            }
            if (lane == 0) ep.row[n_ep] = row;
            n_ep += 1;
            cit = 0;
            cu += nw;
        }
    };

    int t = 0;
    while (p.issued + D <= total) {                     // steady state: every slot reloads unconditionally
#pragma unroll
        for (int j = 0; j < D; ++j) {
            consume(j);
            gemv_issue<W, MODE, D>(a, p, j, nw, n_units, nchunks, S);
        }
        t += D;
    }
    for (; t < total; t += D) {                         // tail: fewer than 2*D steps left
#pragma unroll
        for (int j = 0; j < D; ++j) {
            if (t + j < total) {
                consume(j);
                if (p.issued < total) gemv_issue<W, MODE, D>(a, p, j, nw, n_units, nchunks, S);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    if (MODE == MODE_RESID) {
        // lane e owns parked unit e (n_ep <= 64): add the prefetched residual and store, no load on the way out
        if (lane < n_ep) {
#pragma unroll
            for (int n = 0; n < NC; ++n) {
                if (n < a.ncols) {
                    float* o = a.out + (size_t)n * a.out_stride + ep.row[lane];
                    const float y0 = res0[n] + ep.s[lane][n][0], y1 = res1[n] + ep.s[lane][n][1];
                    o[0] = y0; o[1] = y1;
                }
            }
        }
    } else {
        gemv_flush<NC, MODE>(a, ep, n_ep);
    }
}

}  // namespace d3
