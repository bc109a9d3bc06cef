// Tiled GEMM on the matrix cores for the prompt pass, 129..2048 activation columns per launch:
// out[col][row] = sum_k W[row][k] * x[col][k], bf16 weights, activations x = hi + lo (two bf16 halves).
//
// With hundreds of columns the contraction is compute-bound (the prompt pass is the one part of the path that is), so
// the design is the opposite of the skinny kernels': operands are staged in LDS and re-used from there.  A workgroup
// owns a tile of 256 weight rows x 128 columns whose accumulators never leave registers, and walks K in stages of 32 (one
// MFMA k-step): the stage's weight slab (256 rows x 64 bytes) and activation slab (128 columns, hi plane and lo plane)
// go from global memory straight into LDS with global_load_lds_dwordx4 (16 bytes per lane, lane l of the wave lands at
// base + 16 l, so one instruction fills sixteen 64-byte slab rows; no staging registers, no ds_write instructions).
// The four 16-byte segments of a slab row are swizzled by the row number, which keeps the fragment reads free of bank
// conflicts (sixteen consecutive rows x one segment touch each of the sixteen 16-byte bank groups once); since the
// direct load fixes where a lane's bytes land, the swizzle is applied on the global side: lane l fetches segment
// (l % 4) ^ ((l / 16) % 4) of row l / 4 of its sixteen-row block.
//
// The LDS pipe delivers 128 bytes per cycle and a 16 x 16 x 32 MFMA takes 16 cycles, so with 64 x 64 per wave (12
// fragment reads for 32 MFMAs) the reads and writes of a stage occupy LDS for as many cycles as its MFMAs occupy the
// matrix cores, and any time the two do not overlap is lost.  Two kernels:
//  * gemm_prompt_w4_kernel (QKV, gate/up): four waves (2 x 2), 128 x 64 per wave = 8 x 4 MFMA tiles (16 fragment reads
//    for 64 MFMAs: a third fewer LDS bytes per MFMA), two LDS buffers of 32 KB, two workgroups per compute unit whose
//    stage barriers are independent: one multiplies while the other waits for its loads or reads its fragments.
//  * gemm_prompt_w8_kernel (the residual projections, whose 256 tiles are one per compute unit): eight waves (4 x 2), 64 x
//    64 per wave, four LDS buffers, and two sets of fragments in registers: while the MFMAs of stage t run from one set,
//    the LDS reads of stage t + 1 fill the other.
//    A long residual contraction is cut into K parts instead, one workgroup each on the four-wave kernel (see the launcher).
// The LDS reads are inline assembly: the compiler orders every LDS read it knows of behind ALL outstanding direct-to-LDS
// loads, which would drain the prefetch at every stage.  Here the vmcnt / lgkmcnt waits are written out (a wave's loads
// complete in issue order, NL per stage), and empty asm statements that name the fragments as operands keep the MFMAs
// behind the waits.  7B shape, 2048 columns: QKV 432 -> 350 us, gate/up 805 -> 660, O 167 -> 158, down 402 -> 382
// against the version that staged the slabs through registers (global -> VGPR -> ds_write, 64 x 64 per wave, fragments
// read and multiplied in turns).  Measured with the operands' loads taken out, the stage loop of the eight-wave kernel
// (LDS reads, MFMAs, barrier) takes 68 % of the full time; the matrix cores alone sustain 2.06-2.23 PFLOP/s on this chip
// (82-89 % of the nominal peak: the clock drops under MFMA load), 1.92-2.06 with the LDS reads of this loop beside them
// (mfma_yardstick_kernel below).
//
// Workgroup order: the column blocks of one row block are 8 apart in the launch order, which puts them on one XCD at the
// same time (workgroups go to the XCDs round-robin), so a weight slab pulled into that XCD's L2 serves all of them.  The
// activation slabs are shared by the few row blocks resident on an XCD only and are re-read through the fabric by every
// later one (they fit the 256 MB memory-side cache, not the 4 MB L2): the L2 misses of a 2048-column gate/up launch add up
// to 3.2 GB, 17 times the weight matrix.  A launch order in chunks of 8 row blocks x 4 column blocks per XCD cut that to
// 1.9 GB and was slower (its padded grid delays the residual projections); not kept.
//
// SwiGLU: a workgroup's 256 slab rows are 128 gate rows and the 128 up rows of the same outputs, four tiles of each per
// wave, so a wave finishes silu(gate) * up from its own accumulators.  Operand layouts, RMSNorm folding (1/rms from the
// producer's partial sums of squares, x * gain and the sum of squares of the new residual handed to the consumer) and
// epilogues are those of the skinny matrix-core kernels.
#include <type_traits>
#include <utility>

#include "d3_common.h"

namespace d3 {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;
typedef const __attribute__((address_space(1))) void global_cvoid;

constexpr int kBK = 32;                        // k per stage = one MFMA k-step
constexpr int kPitch = 2 * kBK;                // bytes per staged row: four 16-byte segments, no padding
constexpr int kTileN = 128;                    // columns of a workgroup tile
constexpr int kBBytes = 2 * kTileN * kPitch;   // activation slab of a stage: hi plane, lo plane
constexpr int kLo = kTileN * kPitch;           // the lo plane follows the hi plane

// RW: 16-row weight tiles per wave; WY waves along the rows (x 2 along the columns).
template <int RW, int WY> struct PromptTile {
    static constexpr int kThreads = WY * 2 * 64;
    static constexpr int kWaves = WY * 2;
    static constexpr int kTileM = 16 * RW * WY;             // slab rows (256 in both kernels)
    static constexpr int kABytes = kTileM * kPitch;         // weight slab of a stage
    static constexpr int kStage = kABytes + kBBytes;        // 32 KB
    static constexpr int kBlocks = kStage / 1024;           // sixteen-row blocks of a stage: weights first, then activations hi, lo
    static constexpr int NL = kBlocks / kWaves;             // direct loads per wave and stage
    static constexpr int kAJ = kTileM / 16 / kWaves;        // the first kAJ of them fetch weight rows
    static_assert(kBlocks % kWaves == 0 && (kTileM / 16) % kWaves == 0 && RW % 2 == 0, "slab blocks divide evenly over the waves");
};

// The epilogue of both kernels, from the accumulators: lane (i, g) holds column i of a column tile, rows 4g..4g+3 of each tile.
template <int MODE, int RW, int WY>
__device__ __forceinline__ void prompt_epilogue(const GemvArgs& a, f32x4 (&acc)[RW][4], int rb, int cb, int tiles,
                                                const float* inv_rms, float (*ssq_w)[kTileN]) {
    constexpr int SW = (MODE == MODE_SWIGLU) ? 2 : 1;
    constexpr int kWavesY = WY, OT = WY * RW / SW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1;
    const int li = lane & 15, lg = lane >> 4;
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

extern __shared__ __attribute__((aligned(16))) char prompt_lds[];

template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_frag(uint32_t addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return __builtin_bit_cast(bf16x8, v);
}
template <int N> __device__ __forceinline__ void vm_loads_left() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
template <int N> __device__ __forceinline__ void lds_reads_left() { asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(N) : "memory"); }
// Nothing that uses the fragment moves above this statement, and volatile statements keep their order: after a wait it
// keeps the MFMAs behind the wait; after the reads of the next stage it keeps this stage's MFMAs behind those reads.
__device__ __forceinline__ void pin_frag(bf16x8& v) { asm volatile("" : "+v"(v)); }

template <int RW> struct PromptFrags { bf16x8 a[RW], bh[4], bl[4]; };
template <int RW, int... R>
__device__ __forceinline__ void read_a_frags(PromptFrags<RW>& f, uint32_t A, std::integer_sequence<int, R...>) {
    ((f.a[R] = lds_read_frag<R * 1024>(A)), ...);
}
// all fragments of a stage: weight tiles 0 .. RW - 1, then hi and lo of column tile 0, of column tile 1, ...
template <int RW>
__device__ __forceinline__ void read_frags(PromptFrags<RW>& f, uint32_t A, uint32_t B) {
    read_a_frags<RW>(f, A, std::make_integer_sequence<int, RW>{});
    f.bh[0] = lds_read_frag<0>(B);      f.bl[0] = lds_read_frag<kLo>(B);
    f.bh[1] = lds_read_frag<1024>(B);   f.bl[1] = lds_read_frag<kLo + 1024>(B);
    f.bh[2] = lds_read_frag<2048>(B);   f.bl[2] = lds_read_frag<kLo + 2048>(B);
    f.bh[3] = lds_read_frag<3072>(B);   f.bl[3] = lds_read_frag<kLo + 3072>(B);
}
template <int RW>
__device__ __forceinline__ void pin_frags(PromptFrags<RW>& f) {
#pragma unroll
    for (int r = 0; r < RW; ++r) pin_frag(f.a[r]);
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) { pin_frag(f.bh[tt]); pin_frag(f.bl[tt]); }
}
template <int RW>
__device__ __forceinline__ void mma_column_tile(f32x4 (&acc)[RW][4], const PromptFrags<RW>& f, int tt) {
#pragma unroll
    for (int r = 0; r < RW; ++r) acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[r], f.bh[tt], acc[r][tt], 0, 0, 0);
#pragma unroll
    for (int r = 0; r < RW; ++r) acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.a[r], f.bl[tt], acc[r][tt], 0, 0, 0);
}

// What both kernels do before their stage loops.  Launch order -> (row block, column block): ids 8m .. 8m + 7 are eight
// row blocks of one column block, the next eight ids the same row blocks of the next column block.
template <int MODE, int RW, int WY>
struct PromptSetup {
    typedef PromptTile<RW, WY> Tile;
    static constexpr int SW = (MODE == MODE_SWIGLU) ? 2 : 1;
    static constexpr int OT = WY * RW / SW;            // output row tiles per workgroup (half as many gate/up pairs)
    int rb, cb, tiles, slice;                          // slice: which of the ks parts of K this workgroup walks
    const bf16_t* src[Tile::NL];                       // this lane's piece of each of the wave's sixteen-row blocks, at k = 0
    uint32_t a_off, b_off;                             // LDS addresses of this lane's first weight / activation fragment in buffer 0

    __device__ __forceinline__ bool init(const GemvArgs& a, int n_rb, int n_cb, int ks, int wave, int lane, float* inv_rms) {
        const int per_group = 8 * n_cb;
        const int v = (blockIdx.x / per_group) * 8 + (blockIdx.x % per_group) % 8;   // row block x K part
        cb = (blockIdx.x % per_group) / 8;
        rb = v / ks; slice = v - rb * ks;
        if (rb >= n_rb) return false;
        const int K = a.K;
        tiles = a.total_rows / 16;                     // output row tiles of the whole matrix
        // slab row -> weight row.  Slab tile st (0 .. WY RW - 1): wave row wy owns st = RW wy .. RW wy + RW - 1.  Plain modes:
        // output tile OT rb + st.  SwiGLU: the first RW / 2 tiles of a wave are gate rows, the others the up rows of the same
        // outputs OT rb + (RW / 2) wy + (st % (RW / 2)).  Tiles past the matrix re-read the last tile (result dropped).
        auto slab_row = [&](int s) -> const bf16_t* {
            const int st = s >> 4, i = s & 15;
            if (MODE == MODE_SWIGLU) {
                const int t = st % RW;
                int otile = rb * OT + (st / RW) * (RW / 2) + t % (RW / 2);
                otile = otile < tiles ? otile : tiles - 1;
                return static_cast<const bf16_t*>(a.w[t / (RW / 2)]) + (size_t)(otile * 16 + i) * K;
            }
            int otile = rb * OT + st;
            otile = otile < tiles ? otile : tiles - 1;
            int m = 0, local = otile * 16;
            if (local >= a.rows[0]) { local -= a.rows[0]; m = 1; if (local >= a.rows[1]) { local -= a.rows[1]; m = 2; } }
            return static_cast<const bf16_t*>(a.w[m]) + (size_t)(local + i) * K;
        };
        const int prow = lane >> 2, pseg = (lane & 3) ^ ((lane >> 4) & 3);
#pragma unroll
        for (int j = 0; j < Tile::NL; ++j) {
            const int s = 16 * (wave + Tile::kWaves * j) + prow;
            if (j < Tile::kAJ) src[j] = slab_row(s) + pseg * 8;
            else {
                const int b = s - Tile::kTileM, plane = b >> 7, col = cb * kTileN + (b & 127);
                src[j] = (plane ? a.x_lo : a.x_hi) + (size_t)col * a.x_stride + pseg * 8;
            }
        }
        // fragment reads: lane (i, g) takes segment g of row i of a tile, at slot g ^ ((i / 4) % 4) (tile bases are
        // multiples of 16 rows, so the swizzle depends on i alone)
        const int wy = wave >> 1, wx = wave & 1, li = lane & 15, lg = lane >> 4;
        const uint32_t slot = (uint32_t)((lg ^ ((li >> 2) & 3)) << 4);
        const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)prompt_lds;
        a_off = lds0 + (wy * 16 * RW + li) * kPitch + slot;
        b_off = lds0 + Tile::kABytes + (wx * 64 + li) * kPitch + slot;
        // 16 threads add up one column's partial sums of squares, in a fixed order (before the direct loads: vmcnt counts these loads too)
        if (MODE != MODE_RESID && a.ssq_in) {
            const int tid = threadIdx.x;
            for (int c = tid >> 4; c < kTileN; c += Tile::kThreads / 16) {
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
        vm_loads_left<0>();
        return true;
    }
    // stage t -> LDS buffer buf (its 1 KB blocks in slab order; this wave's are wave, wave + kWaves, ...)
    __device__ __forceinline__ void dma(int t, int buf, int wave) const {
        lds_char* dst = (lds_char*)prompt_lds + buf * Tile::kStage + wave * 1024;
#pragma unroll
        for (int j = 0; j < Tile::NL; ++j)
            __builtin_amdgcn_global_load_lds((global_cvoid*)(src[j] + (size_t)t * kBK),
                                             (__attribute__((address_space(3))) void*)(dst + j * Tile::kWaves * 1024), 16, 0, 0);
    }
};

// ---------------- four waves, 128 x 64 per wave, two workgroups per compute unit ----------------
// One set of fragments, two LDS buffers.  Stage t: wait for the wave's own loads of the stage, barrier (everybody's have
// landed, nobody still reads stage t - 1), request stage t + 1 into the other buffer, read the 16 fragments, and
// multiply column tile by column tile as its fragments arrive.
template <int MODE>
__global__ __launch_bounds__(256, 2) void gemm_prompt_w4_kernel(GemvArgs a, int n_rb, int n_cb, int ks) {
    constexpr int RW = 8, WY = 2;
    typedef PromptTile<RW, WY> Tile;
    __shared__ float inv_rms[kTileN];
    __shared__ float ssq_w[WY][kTileN];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __shared__ int is_last;
    PromptSetup<MODE, RW, WY> su;
    if (!su.init(a, n_rb, n_cb, ks, wave, lane, inv_rms)) return;
    const int all_stages = a.K / kBK;
    const int s0 = (int)((long long)all_stages * su.slice / ks), n_stages = (int)((long long)all_stages * (su.slice + 1) / ks) - s0;
    su.dma(s0, 0, wave);

    f32x4 acc[RW][4];                                  // [slab tile of the wave][column tile of the wave]
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
    PromptFrags<RW> f;
    for (int t = 0; t < n_stages; ++t) {
        vm_loads_left<0>();                            // this wave's part of stage t has landed ...
        __syncthreads();                               // ... and everybody's; nobody still reads stage t - 1 (and inv_rms is written)
        if (t + 1 < n_stages) su.dma(s0 + t + 1, (t + 1) & 1, wave);
        read_frags<RW>(f, su.a_off + (t & 1) * Tile::kStage, su.b_off + (t & 1) * Tile::kStage);
        lds_reads_left<6>();                           // the weight tiles and column tile 0
#pragma unroll
        for (int r = 0; r < RW; ++r) pin_frag(f.a[r]);
        pin_frag(f.bh[0]); pin_frag(f.bl[0]);
        mma_column_tile<RW>(acc, f, 0);
        __builtin_amdgcn_sched_barrier(0);             // the scheduler moves nothing across: the next wait stays behind these MFMAs
        lds_reads_left<4>();
        pin_frag(f.bh[1]); pin_frag(f.bl[1]);
        mma_column_tile<RW>(acc, f, 1);
        __builtin_amdgcn_sched_barrier(0);
        lds_reads_left<2>();
        pin_frag(f.bh[2]); pin_frag(f.bl[2]);
        mma_column_tile<RW>(acc, f, 2);
        __builtin_amdgcn_sched_barrier(0);
        lds_reads_left<0>();
        pin_frag(f.bh[3]); pin_frag(f.bl[3]);
        mma_column_tile<RW>(acc, f, 3);
        __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("" ::: "memory");                     // the epilogue's loads stay behind the last stage
    // ---- K parts: publish, count arrivals, the last one adds the parts up in order (independent of arrival order) ----
    if (ks > 1) {
        constexpr int ACC = RW * 4 * 4;
        const int tile_id = su.rb * n_cb + su.cb;
        float* mine = a.part + (((size_t)tile_id * ks + su.slice) * 4 + wave) * (ACC * 64) + lane;
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int e = 0; e < 4; ++e) st_agent(mine + ((r * 4 + tt) * 4 + e) * 64, acc[r][tt][e]);
        wait_stores();                                 // this part's partials have reached the coherence point
        __syncthreads();
        if (threadIdx.x == 0) {
            int* ticket = &a.part_tickets[tile_id];
            const int done = atomicAdd(ticket, 1);
            is_last = done == ks - 1;
            if (is_last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // all arrived: leave it clean
        }
        __syncthreads();
        if (!is_last) return;
#pragma unroll
        for (int r = 0; r < RW; ++r)
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int part = 0; part < ks; ++part) {
            const float* p = a.part + (((size_t)tile_id * ks + part) * 4 + wave) * (ACC * 64) + lane;
#pragma unroll
            for (int r = 0; r < RW; ++r)
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = ld_agent(p + ((r * 4 + tt) * 4 + e) * 64);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][tt][e] += v[e];
                }
        }
    }
    prompt_epilogue<MODE, RW, WY>(a, acc, su.rb, su.cb, su.tiles, inv_rms, ssq_w);
}

// ---------------- eight waves, 64 x 64 per wave, fragments double-buffered in registers ----------------
// Four LDS buffers: stage t + 1 is being read, t + 2 .. t + 4 are in flight or landed.  Stage t: the fragments of stage
// t are in registers (read during stage t - 1).  Loads are issued in the order 0 1 2 3 | 4 5 (at stage 1) | 6 7 (at stage
// 3) | ...: the two stages of a pair are the two halves of the rows' cache lines, requested together so that a line is
// fetched into the compute unit's L1 once.  When stage t + 1 must have landed, the stages issued after it are t + 2, t + 3
// (t even) or t + 2 (t odd).  The steady state has no branch; the last four stages issue nothing and wait for everything.
// Needs an even number of stages, at least four.
template <int MODE>
__global__ __launch_bounds__(512, 2) void gemm_prompt_w8_kernel(GemvArgs a, int n_rb, int n_cb) {
    constexpr int RW = 4, WY = 4, NB = 4;
    typedef PromptTile<RW, WY> Tile;
    constexpr int NL = Tile::NL, kStage = Tile::kStage;
    static_assert(3 * NL < 64, "vmcnt holds 6 bits");
    __shared__ float inv_rms[kTileN];
    __shared__ float ssq_w[WY][kTileN];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    PromptSetup<MODE, RW, WY> su;
    if (!su.init(a, n_rb, n_cb, 1, wave, lane, inv_rms)) return;
    const int n_stages = a.K / kBK;
    su.dma(0, 0, wave); su.dma(1, 1, wave); su.dma(2, 2, wave); su.dma(3, 3, wave);

    f32x4 acc[RW][4];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto read = [&](PromptFrags<RW>& f, int t) { read_frags<RW>(f, su.a_off + (t & (NB - 1)) * kStage, su.b_off + (t & (NB - 1)) * kStage); };
    // the reads of the next stage are in flight while this stage's MFMAs run, and the MFMAs stay above the next stage's waits
    auto mma = [&](PromptFrags<RW>& f) {
        pin_frags<RW>(f);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) mma_column_tile<RW>(acc, f, tt);
        __builtin_amdgcn_sched_barrier(0);
    };
    PromptFrags<RW> f0, f1;
    vm_loads_left<3 * NL>();
    __syncthreads();                                   // stage 0 is in LDS (and inv_rms is written)
    read(f0, 0);
    int t = 0;
    for (; t + 4 < n_stages; t += 2) {
        vm_loads_left<2 * NL>();
        lds_reads_left<0>();
        __syncthreads();                               // stage t + 1 is complete in LDS; nobody still reads stages <= t
        read(f1, t + 1);
        mma(f0);
        vm_loads_left<NL>();
        lds_reads_left<0>();
        __syncthreads();
        su.dma(t + 4, t & (NB - 1), wave); su.dma(t + 5, (t + 1) & (NB - 1), wave);
        read(f0, t + 2);
        mma(f1);
    }
    // t = n_stages - 4
    vm_loads_left<0>();
    lds_reads_left<0>();
    __syncthreads();
    read(f1, t + 1);
    mma(f0);
    lds_reads_left<0>();
    __syncthreads();
    read(f0, t + 2);
    mma(f1);
    lds_reads_left<0>();
    __syncthreads();
    read(f1, t + 3);
    mma(f0);
    lds_reads_left<0>();
    mma(f1);
    asm volatile("" ::: "memory");
    prompt_epilogue<MODE, RW, WY>(a, acc, su.rb, su.cb, su.tiles, inv_rms, ssq_w);
}

// ---------------- yardstick: what the matrix cores sustain with this file's stage loop ----------------
// The stage loop of the eight-wave kernel without its operands' loads: 32 MFMAs per wave and stage on fragments that
// (mode >= 1) are re-read from a fixed LDS buffer every stage as in the kernel, (mode 2) with the stage barrier.  One
// workgroup per launched block, no global memory traffic but one word per wave at the end.
template <int V>
__global__ __launch_bounds__(512, 2) void mfma_yardstick_kernel(float* __restrict__ sink, int stages) {
    constexpr int RW = 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, li = lane & 15, lg = lane >> 4;
    unsigned* words = reinterpret_cast<unsigned*>(prompt_lds);
    for (int i = tid; i < PromptTile<4, 4>::kStage / 4; i += 512) words[i] = 0x3c003c00u ^ ((unsigned)i * 2654435761u & 0x00ff00ffu);   // bf16 values near 1
    __syncthreads();
    const uint32_t slot = (uint32_t)((lg ^ ((li >> 2) & 3)) << 4);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)prompt_lds;
    const uint32_t A = lds0 + ((wave >> 1) * 16 * RW + li) * kPitch + slot, B = lds0 + PromptTile<4, 4>::kABytes + ((wave & 1) * 64 + li) * kPitch + slot;
    f32x4 acc[RW][4];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) acc[r][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
    PromptFrags<RW> f0, f1;
    read_frags<RW>(f0, A, B);
    lds_reads_left<0>();
    pin_frags<RW>(f0);
    f1 = f0;
    auto half = [&](PromptFrags<RW>& cur, PromptFrags<RW>& nxt) {
        if (V >= 1) lds_reads_left<0>();
        if (V >= 2) __syncthreads();
        if (V >= 1) read_frags<RW>(nxt, A, B);
        pin_frags<RW>(cur);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) mma_column_tile<RW>(acc, cur, tt);
        __builtin_amdgcn_sched_barrier(0);
    };
    for (int t = 0; t < stages; t += 2) { half(f0, f1); half(f1, f0); }
    lds_reads_left<0>();
    pin_frags<RW>(f0);
    float sum = (float)f0.a[0][0];
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) sum += acc[r][tt][0] + acc[r][tt][3];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (lane == 0) sink[blockIdx.x * 8 + wave] = sum;
}

template <int MODE>
int launch_w4(const GemvArgs& a, int n_rb, int n_cb, int ks, hipStream_t s) {
    constexpr int lds = 2 * PromptTile<8, 2>::kStage;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_prompt_w4_kernel<MODE>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return (int)attr;
    hipLaunchKernelGGL(gemm_prompt_w4_kernel<MODE>, dim3((n_rb * ks + 7) / 8 * 8 * n_cb), dim3(256), lds, s, a, n_rb, n_cb, ks);
    return (int)hipGetLastError();
}
int launch_w8_resid(const GemvArgs& a, int n_rb, int n_cb, hipStream_t s) {
    constexpr int lds = 4 * PromptTile<4, 4>::kStage;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_prompt_w8_kernel<MODE_RESID>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return (int)attr;
    hipLaunchKernelGGL(gemm_prompt_w8_kernel<MODE_RESID>, dim3((n_rb + 7) / 8 * 8 * n_cb), dim3(512), lds, s, a, n_rb, n_cb);
    return (int)hipGetLastError();
}

}  // namespace

// Requirements: those of launch_gemm_mfma (bf16 weights, K % 32 == 0, row counts multiples of 16), 1 <= ncols <=
// kPassCols (x_hi / x_lo hold ncols rounded up to 128 rows); with ssq_out at most kSsqStride row blocks.
int launch_gemm_prompt(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups) {
    const int tiles = a.total_rows / 16;
    const int n_cb = (a.ncols + kTileN - 1) / kTileN;
    if (a.ncols < 1 || a.ncols > kPassCols || a.K % kBK != 0 || a.K < kBK) return (int)hipErrorInvalidValue;
    const int ot = mode == MODE_SWIGLU ? 8 : 16;       // output row tiles per workgroup: 256 slab rows in both kernels
    const int n_rb = (tiles + ot - 1) / ot;
    if (a.ssq_out && n_rb > kSsqStride) return (int)hipErrorInvalidValue;
    if (n_groups) *n_groups = n_rb;
    const int n_stages = a.K / kBK;
    if (mode == MODE_STORE) return launch_w4<MODE_STORE>(a, n_rb, n_cb, 1, s);
    if (mode == MODE_SWIGLU) return launch_w4<MODE_SWIGLU>(a, n_rb, n_cb, 1, s);
    // A residual projection has few tiles (4096 rows x 2048 columns: 256, one per compute unit).  With room for a second
    // workgroup per compute unit K is cut into parts, one workgroup each on the four-wave kernel; the parts publish their
    // accumulators (128 KB) and the one that arrives last at the tile's counter adds them up in part order.  That costs
    // 40-65 us per launch (7B shape), so a part must keep enough stages: 96, or 48 when the tiles alone would leave a quarter
    // of the compute units idle (7B shape, 2048 columns: down 395 -> 362 us in two parts, O 166 -> 185 and left whole; 13B
    // shape, 1024 columns, 160 tiles: down 447 -> 314 in three parts, O 192 -> 173).
    const int tiles_wg = n_rb * n_cb;
    int ks = 2 * n_cu / tiles_wg;
    if (ks > 4) ks = 4;
    const int min_part = 4 * tiles_wg < 3 * n_cu ? 48 : 96;
    while (ks > 1 && n_stages / ks < min_part) --ks;
    if (tn.prompt_ks >= 1 && tn.prompt_ks <= n_stages) ks = tn.prompt_ks;
    if (ks < 1) ks = 1;
    if (ks > 1 && a.part && a.part_tickets && tiles_wg <= kGemmPartTickets && (size_t)tiles_wg * ks * 4 * 128 * 64 * sizeof(float) <= kPromptPartBytes)
        return launch_w4<MODE_RESID>(a, n_rb, n_cb, ks, s);
    if (n_stages >= 4 && n_stages % 2 == 0) return launch_w8_resid(a, n_rb, n_cb, s);
    return launch_w4<MODE_RESID>(a, n_rb, n_cb, 1, s);
}

// mode 0: MFMAs alone; 1: with the fragment reads of the stage loop; 2: with the stage barrier as well.  n_wg workgroups of
// eight waves; sink holds 8 floats per workgroup.  Flops issued: n_wg * 8 waves * stages * 32 MFMAs * 16384.
int launch_mfma_yardstick(int mode, int stages, int n_wg, float* sink, hipStream_t s) {
    constexpr int lds = PromptTile<4, 4>::kStage;
    if (mode < 0 || mode > 2 || stages < 2 || stages % 2 != 0) return (int)hipErrorInvalidValue;
    if (mode == 0) hipLaunchKernelGGL(mfma_yardstick_kernel<0>, dim3(n_wg), dim3(512), lds, s, sink, stages);
    else if (mode == 1) hipLaunchKernelGGL(mfma_yardstick_kernel<1>, dim3(n_wg), dim3(512), lds, s, sink, stages);
    else hipLaunchKernelGGL(mfma_yardstick_kernel<2>, dim3(n_wg), dim3(512), lds, s, sink, stages);
    return (int)hipGetLastError();
}

}  // namespace d3
