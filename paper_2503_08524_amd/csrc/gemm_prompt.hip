// Tiled GEMM on the matrix cores for the prompt pass, 129..2048 activation columns per launch:
// out[col][row] = sum_k W[row][k] * x[col][k], bf16 weights, activations x = hi + lo (two bf16 halves).
//
// With hundreds of columns the contraction is compute-bound (the prompt pass is the one part of the path that is),
// so the design is the opposite of the skinny kernels': operands are staged in LDS and re-used from there.  A
// workgroup of eight waves (4 x 2) owns a tile of 256 weight rows x 128 columns (gate/up: four waves, 128 x 128); each wave
// 64 x 64 of it, i.e. 4 x 4 MFMA tiles whose accumulators never leave registers.  K is walked in stages of 32: the stage's weight slab
// (128 rows) and activation slab (128 columns, hi and lo) travel global -> registers -> LDS with coalesced 16-byte
// pieces (rows of 64 bytes whose four segments are swizzled by the row number, which keeps both the stores and the fragment reads free of bank conflicts);
// a wave reads 4 weight fragments and 8 activation fragments per stage and issues 32 MFMAs with them.  Two LDS buffers
// and two or four register sets keep the loads of the next stages in flight while stage t is multiplied; one workgroup
// barrier per stage.
//
// Workgroup order: the column blocks of one row block are 8 apart in the launch order, which puts them on one XCD at the
// same time (workgroups go to the XCDs round-robin), so a weight slab pulled into that XCD's L2 serves all of them.  The
// activation slabs are shared by the few row blocks resident on an XCD only and are re-read through the fabric by every
// later one (they fit the 256 MB memory-side cache, not the 4 MB L2): the L2 misses of a 2048-column gate/up launch add up
// to 3.2 GB, 17 times the weight matrix.  A launch order in chunks of 8 row blocks x 4 column blocks per XCD cut that to
// 1.9 GB and was slower (its padded grid delays the residual projections: down 402 -> 731 us); not kept.
//
// SwiGLU: a workgroup's 128 slab rows are 64 gate rows and the 64 up rows of the same outputs, two tiles of each per
// wave, so a wave finishes silu(gate) * up from its own accumulators.  Operand layouts, RMSNorm folding (1/rms from the
// producer's partial sums of squares, x * gain and the sum of squares of the new residual handed to the consumer) and
// epilogues are those of the skinny matrix-core kernels.
#include <type_traits>

#include "d3_common.h"

namespace d3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 32;                        // k per stage = one MFMA k-step
constexpr int kPitch = 2 * kBK;                // bytes per staged row: four 16-byte segments, no padding
constexpr int kTileN = 128;                    // columns of a workgroup tile
constexpr int kBBytes = 2 * kTileN * kPitch;   // activation slab of a stage: hi plane, lo plane
// WY waves along the rows (x 2 along the columns).  4: eight waves, tile 256 rows x 128 columns, one workgroup per
// compute unit; 2: four waves, 128 x 128, two workgroups per compute unit.  The larger tile moves a quarter fewer bytes
// from L2 and through LDS per MFMA (7B shape, 2048 columns: QKV 458 -> 430 us, O 179 -> 165, down 469 -> 402); the gate/up
// launch has too few row blocks for it (5.4 rounds of workgroups: 820 -> 871 us) and keeps the smaller one.

// RW: 16-row weight tiles per wave.  4: workgroup tile 128 rows x 128 columns, two workgroups per compute unit.  (8, a tile
// of 256 rows with a third fewer LDS and L2 bytes per MFMA but one workgroup per compute unit, was measured 18 % slower:
// the kernel is bound by the latencies that a second resident workgroup hides, not by LDS bandwidth.)
template <int RW, int WY> struct PromptTile {
    static constexpr int kThreads = WY * 2 * 64;
    static constexpr int kBLoads = 2 * kTileN * 4 / kThreads;   // 16-byte pieces of the activation slab per thread and stage
    static constexpr int kTileM = 16 * RW * WY;             // slab rows
    static constexpr int kABytes = kTileM * kPitch;         // weight slab of a stage
    static constexpr int kStage = kABytes + kBBytes;        // 30720 or 40960 bytes
    static constexpr int kALoads = kTileM * 4 / kThreads;   // 16-byte pieces of the weight slab per thread and stage
    static constexpr int kLds = 2 * kStage;
};

extern __shared__ __attribute__((aligned(16))) char prompt_lds[];

template <int MODE, int RW, int WY>
__global__ __launch_bounds__(WY * 128, 2) void gemm_prompt_kernel(GemvArgs a, int n_rb, int n_cb) {
    typedef PromptTile<RW, WY> Tile;
    constexpr int SW = (MODE == MODE_SWIGLU) ? 2 : 1;
    constexpr int kWavesY = WY, kThreads = Tile::kThreads, kBLoads = Tile::kBLoads;
    constexpr int OT = kWavesY * RW / SW;              // output row tiles per workgroup (half as many gate/up pairs)
    constexpr int kABytes = Tile::kABytes, kStage = Tile::kStage, kALoads = Tile::kALoads;
    struct StageRegs { u32x4 a[kALoads], b[kBLoads]; };
    char* lds = prompt_lds;
    __shared__ float inv_rms[kTileN];
    __shared__ float ssq_w[kWavesY][kTileN];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const int li = lane & 15, lg = lane >> 4;
    // launch order -> (row block, column block): ids 8m .. 8m + 7 are eight row blocks of one column block, the next
    // eight ids the same row blocks of the next column block
    const int per_group = 8 * n_cb;
    const int rb = (blockIdx.x / per_group) * 8 + (blockIdx.x % per_group) % 8;
    const int cb = (blockIdx.x % per_group) / 8;
    if (rb >= n_rb) return;
    const int K = a.K, n_stages = K / kBK;
    const int tiles = a.total_rows / 16;               // output row tiles of the whole matrix

    // slab row -> weight row.  Slab tile st (0 .. 2 RW - 1): wave wy owns st = RW wy .. RW wy + RW - 1.  Plain modes:
    // output tile OT rb + st.  SwiGLU: the first RW / 2 tiles of a wave are gate rows, the others the up rows of the same
    // outputs OT rb + (RW / 2) wy + (st % (RW / 2)).
    auto slab_row = [&](int s) -> const bf16_t* {
        const int st = s >> 4, i = s & 15;
        if (MODE == MODE_SWIGLU) {
            const int t = st % RW;
            int otile = rb * OT + (st / RW) * (RW / 2) + t % (RW / 2);
            otile = otile < tiles ? otile : tiles - 1;  // past the matrix: re-read the last tile (result dropped)
            return static_cast<const bf16_t*>(a.w[t / (RW / 2)]) + (size_t)(otile * 16 + i) * K;
        }
        int otile = rb * OT + st;
        otile = otile < tiles ? otile : tiles - 1;
        int m = 0, local = otile * 16;
        if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
        return static_cast<const bf16_t*>(a.w[m]) + (size_t)(local + i) * K;
    };
    // this thread's pieces: slab row (tid / 4) + (kThreads / 4) j, 16-byte segment tid % 4 (four neighbouring lanes fetch 64 contiguous bytes)
    constexpr int kRowsPerPass = kThreads / 4;
    const int prow = tid >> 2, pseg = tid & 3;
    const bf16_t* asrc[kALoads];
    const bf16_t* bsrc[kBLoads];
#pragma unroll
    for (int j = 0; j < kALoads; ++j) asrc[j] = slab_row(prow + kRowsPerPass * j) + pseg * 8;
#pragma unroll
    for (int j = 0; j < kBLoads; ++j) {
        const int brow = prow + kRowsPerPass * j, plane = brow >> 7, col = cb * kTileN + (brow & 127);
        bsrc[j] = (plane ? a.x_lo : a.x_hi) + (size_t)col * a.x_stride + pseg * 8;
    }
    // Segment s of slab row r sits at slot s ^ ((r / 4) % 4) of the row.  A store instruction's sixteen-lane groups are
    // four consecutive rows x four segments, a fragment read's are sixteen consecutive rows x one segment: under this
    // swizzle both touch each of the sixteen 16-byte bank groups once (a padded pitch of 80 keeps the reads conflict-free
    // but puts rows 0 and 3 of a store group on the same banks: half of the LDS cycles were conflict cycles).
    const int pdst = prow * kPitch + ((pseg ^ ((prow >> 2) & 3)) << 4);

    auto issue = [&](StageRegs& r, int t) {
        const int k = t * kBK;
#pragma unroll
        for (int j = 0; j < kALoads; ++j) r.a[j] = *reinterpret_cast<const u32x4*>(asrc[j] + k);
#pragma unroll
        for (int j = 0; j < kBLoads; ++j) r.b[j] = *reinterpret_cast<const u32x4*>(bsrc[j] + k);
    };
    auto store = [&](const StageRegs& r, int buf) {
        char* base = lds + buf * kStage;
#pragma unroll
        for (int j = 0; j < kALoads; ++j) *reinterpret_cast<u32x4*>(base + pdst + kRowsPerPass * j * kPitch) = r.a[j];
#pragma unroll
        for (int j = 0; j < kBLoads; ++j) *reinterpret_cast<u32x4*>(base + kABytes + pdst + kRowsPerPass * j * kPitch) = r.b[j];
    };

    f32x4 acc[RW][4];                                  // [slab tile of the wave][column tile of the wave]
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto multiply = [&](int buf) {
        const int slot = (lg ^ ((li >> 2) & 3)) << 4;      // tile bases are multiples of 16 rows: the swizzle depends on li alone
        const char* A = lds + buf * kStage + (wy * 16 * RW + li) * kPitch + slot;
        const char* B = lds + buf * kStage + kABytes + (wx * 64 + li) * kPitch + slot;
        bf16x8 af[RW];
#pragma unroll
        for (int r = 0; r < RW; ++r) af[r] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(A + r * 16 * kPitch));
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(B + tt * 16 * kPitch));
            const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(B + (kTileN + tt * 16) * kPitch));
#pragma unroll
            for (int r = 0; r < RW; ++r) acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[r], bh, acc[r][tt], 0, 0, 0);
#pragma unroll
            for (int r = 0; r < RW; ++r) acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[r], bl, acc[r][tt], 0, 0, 0);
        }
    };

    // ---- the stages: LDS holds stages t and t + 1, registers the loads of the stages after them ----
    // A weight or activation row advances 64 bytes per stage, half a cache line: the loads of stages 2m and 2m + 1 are
    // issued together, so that the line is fetched into the compute unit's L1 once (issued a stage apart, the second half
    // found the line evicted and fetched it again: twice the L2 -> L1 traffic, which was what bounded the kernel).
    // Four register sets (stages t + 1 .. t + 4) for the projections that stream large matrices; two for the residual
    // projections, whose epilogue (old residual, next gains) leaves the register allocator no room for more.  Past the
    // last stage the loads re-read it and the store fills a buffer that nobody reads: the steady state has no branch.
    constexpr int NR = MODE == MODE_RESID ? 2 : 4;
    StageRegs ra, rb_, rc, rd;
    const int last = n_stages - 1;
    auto at = [&](int t) { return t < last ? t : last; };
    issue(ra, 0);
    issue(rb_, at(1));
    if (NR == 4) { issue(rc, at(2)); issue(rd, at(3)); }
    // 16 threads add up one column's partial sums of squares, in a fixed order
    if (MODE != MODE_RESID && a.ssq_in) {
        for (int c = tid >> 4; c < kTileN; c += kThreads / 16) {
            const int col = cb * kTileN + c;
            float ss = 0.f;
            if (col < a.ncols) {
                const float* p = a.ssq_in + (size_t)col * kSsqStride;
                for (int i0 = tid & 15; i0 < a.ssq_parts; i0 += 16) ss += p[i0];
            }
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
            if ((tid & 15) == 0) inv_rms[c] = 1.0f / sqrtf(ss / (float)K + a.eps);
        }
    }
    store(ra, 0);
    __syncthreads();
    // every __syncthreads below: the stage just stored is complete in LDS, and nobody still reads the one just multiplied
    if constexpr (NR == 4) {
        for (int t = 0; t < n_stages; t += 4) {
            multiply(0); store(rb_, 1); issue(ra, at(t + 4)); issue(rb_, at(t + 5)); __syncthreads();
            if (t + 1 >= n_stages) break;
            multiply(1); store(rc, 0); __syncthreads();
            if (t + 2 >= n_stages) break;
            multiply(0); store(rd, 1); issue(rc, at(t + 6)); issue(rd, at(t + 7)); __syncthreads();
            if (t + 3 >= n_stages) break;
            multiply(1); store(ra, 0); __syncthreads();
        }
    } else {
        for (int t = 0; t < n_stages; t += 2) {
            multiply(0); store(rb_, 1); issue(ra, at(t + 2)); issue(rb_, at(t + 3)); __syncthreads();
            if (t + 1 >= n_stages) break;
            multiply(1); store(ra, 0); __syncthreads();
        }
    }

    asm volatile("" ::: "memory");                     // the epilogue's loads stay behind the last stage
    // ---- epilogue from the accumulators: lane (i, g) holds column i of a column tile, rows 4g..4g+3 of each tile ----
    float sq[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) sq[tt] = 0.f;
#pragma unroll
    for (int r = 0; r < RW / SW; ++r) {
        // tiles and columns past the matrix compute on clamped addresses and store nothing (no divergent control flow around the loads)
        const int otile_raw = rb * OT + wy * (RW / SW) + r;
        const int otile = otile_raw < tiles ? otile_raw : tiles - 1;
        const int row = otile * 16 + 4 * lg;
        float4 gn = make_float4(1.f, 1.f, 1.f, 1.f);
        if (MODE == MODE_RESID && a.ssq_out) gn = *reinterpret_cast<const float4*>(a.gain_next + row);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const int cl = wx * 64 + tt * 16 + li, col_raw = cb * kTileN + cl;
            const bool live = otile_raw < tiles && col_raw < a.ncols;
            const int col = col_raw < a.ncols ? col_raw : a.ncols - 1;
            const size_t oi = (size_t)col * a.out_stride + row;
            const f32x4 s0 = acc[r][tt];
            float v[4], split[4];
            if (MODE == MODE_STORE) {
                const float sc = a.ssq_in ? inv_rms[cl] : 1.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = s0[e] * sc;
            } else if (MODE == MODE_RESID) {
                const float4 o = *reinterpret_cast<const float4*>(a.out + oi);
                v[0] = o.x + s0[0]; v[1] = o.y + s0[1]; v[2] = o.z + s0[2]; v[3] = o.w + s0[3];
            } else {
                const f32x4 s1 = acc[r + RW / 2][tt];
                const float sc = a.ssq_in ? inv_rms[cl] : 1.0f;
#pragma unroll
                for (int e = 0; e < 4; ++e) { const float gt = s0[e] * sc; v[e] = gt / (1.0f + expf(-gt)) * (s1[e] * sc); }
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) split[e] = v[e];
            if (MODE == MODE_RESID && a.ssq_out) {     // the consumer is a normalised projection: hand it x * gain and sum(x^2)
                if (live) sq[tt] += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
                split[0] = v[0] * gn.x; split[1] = v[1] * gn.y; split[2] = v[2] * gn.z; split[3] = v[3] * gn.w;
            }
            uint32_t hb[4], lb[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                hb[e] = f32_to_bf16(split[e]);
                lb[e] = f32_to_bf16(split[e] - bf16_to_f32(hb[e]));
            }
            if (live) {
                if (a.out) *reinterpret_cast<float4*>(a.out + oi) = make_float4(v[0], v[1], v[2], v[3]);
                if (a.out_hi) {
                    *reinterpret_cast<uint2*>(a.out_hi + oi) = make_uint2(hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16));
                    *reinterpret_cast<uint2*>(a.out_lo + oi) = make_uint2(lb[0] | (lb[1] << 16), lb[2] | (lb[3] << 16));
                }
            }
        }
    }
    if (MODE == MODE_RESID && a.ssq_out) {             // rows of a column: the 4 lane groups by butterfly, then the two row halves in order
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            sq[tt] += __shfl_xor(sq[tt], 16, 64);
            sq[tt] += __shfl_xor(sq[tt], 32, 64);
            if (lg == 0) ssq_w[wy][wx * 64 + tt * 16 + li] = sq[tt];
        }
        __syncthreads();
        if (tid < kTileN && cb * kTileN + tid < a.ncols) {
            float ss = 0.f;
#pragma unroll
            for (int w = 0; w < kWavesY; ++w) ss += ssq_w[w][tid];
            a.ssq_out[(size_t)(cb * kTileN + tid) * kSsqStride + rb] = ss;
        }
    }
}

template <int MODE, int RW, int WY>
int launch_tile(const GemvArgs& a, int n_rb, int n_cb, hipStream_t s) {
    auto* k = gemm_prompt_kernel<MODE, RW, WY>;
    constexpr int lds = PromptTile<RW, WY>::kLds;
    constexpr int kThreads = PromptTile<RW, WY>::kThreads;
    if (lds > 48 * 1024) {
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (once != hipSuccess) return (int)once;
    }
    hipLaunchKernelGGL(k, dim3((n_rb + 7) / 8 * 8 * n_cb), dim3(kThreads), lds, s, a, n_rb, n_cb);
    return (int)hipGetLastError();
}

}  // namespace

// Requirements: those of launch_gemm_mfma (bf16 weights, K % 32 == 0, row counts multiples of 16), 1 <= ncols <=
// kPassCols (x_hi / x_lo hold ncols rounded up to 128 rows); with ssq_out at most kSsqStride row blocks.
int launch_gemm_prompt(const GemvArgs& a, int mode, hipStream_t s, int* n_groups) {
    const int tiles = a.total_rows / 16;
    const int sw = mode == MODE_SWIGLU ? 2 : 1;
    const int n_cb = (a.ncols + kTileN - 1) / kTileN;
    if (a.ncols < 1 || a.ncols > kPassCols || a.K % kBK != 0) return (int)hipErrorInvalidValue;
    constexpr int rw = 4;
    const int wy = mode == MODE_SWIGLU ? 2 : 4;
    const int ot = wy * rw / sw;
    const int n_rb = (tiles + ot - 1) / ot;
    if (a.ssq_out && n_rb > kSsqStride) return (int)hipErrorInvalidValue;
    if (n_groups) *n_groups = n_rb;
    if (mode == MODE_STORE) return launch_tile<MODE_STORE, rw, 4>(a, n_rb, n_cb, s);
    if (mode == MODE_RESID) return launch_tile<MODE_RESID, rw, 4>(a, n_rb, n_cb, s);
    return launch_tile<MODE_SWIGLU, rw, 2>(a, n_rb, n_cb, s);
}

}  // namespace d3
