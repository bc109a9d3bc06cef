// Shared declarations of the D^3 HIP library (gfx950 only): kernel argument
// structs, launch wrappers, small device helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace d3 {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kMaxCols = 32;       // largest batch; columns of a decode pass
constexpr int kPassCols = 2048;    // most columns of a prompt chunk on the matrix-core path (a context holds min(this, max_seq rounded up to 128))
constexpr int kMaxSplits = 32;     // context splits of one attention head
constexpr size_t kGemmPartBytes = 16u << 20;   // partial accumulators of a K-sliced wide MFMA projection
constexpr size_t kPromptPartBytes = 64u << 20; // ... and of a K-sliced residual projection of the prompt pass (at most 512 workgroups of 128 KB)
constexpr int kGemmPartTickets = 2048;         // row groups such a projection may have
constexpr int kSsqStride = 512;    // partial sums of squares kept per column (one per workgroup of the producing projection)

typedef uint16_t bf16_t;           // bf16 bit pattern
typedef _Float16 f16_t;            // IEEE half (KV cache only)

// bytes per KV-cache element for a d3_dtype value (0 f32, 2 f16)
inline int kv_elem_bytes(int kv_dtype) { return kv_dtype == 0 ? 4 : 2; }

// Which (sequence, position, token) a column of the current pass stands for.
// Column c has global index g = base + c; sequence g % B, row pos_begin + g / B.
// Decode: base 0, P 1 (column b = sequence b).  Prompt pass: position-major
// enumeration of the [B][P] prompt, so the last B columns are the last positions.
struct ColMap {
    int base, B, P, pos_begin;
    int seq0 = 0;          // first sequence of the pass (a prompt chunk of one sequence: B = 1, seq0 = that sequence)
    __host__ __device__ int seq(int c) const { return seq0 + (base + c) % B; }
    __host__ __device__ int pos(int c) const { return pos_begin + (base + c) / B; }
    __host__ __device__ int tok_index(int c) const { return seq(c) * P + (base + c) / B; }
};

// 16-byte streaming load of weights that are read exactly once (non-temporal: do not
// displace the activations that live in L2)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4 load_stream16(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }
// round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Data handed from one workgroup to another inside a kernel is written and read with agent-scope
// accesses (coherent across the chip's eight L2s) instead of cache-wide fences, which cost tens of
// microseconds here.  Protocol: producer st_agent(...), wait_stores(), workgroup barrier, then one
// thread bumps an arrival counter; the consumer sees the counter and reads with ld_agent(...).
__device__ __forceinline__ void st_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---------------- projections ----------------
enum GemvMode { MODE_STORE = 0, MODE_RESID = 1, MODE_SWIGLU = 2, MODE_QKV_ROPE = 3 };

struct GemvArgs {
    // activations: fp32 [ncols][x_stride] (ALU path) or bf16 hi/lo halves [.][x_stride] (MFMA path)
    const float* x;
    const bf16_t* x_hi;
    const bf16_t* x_lo;
    int x_stride;
    const float* gain;   // RMSNorm gain [K] when the norm is fused (ALU path), else nullptr
    float eps;
    int K;
    // up to three row-stacked matrices [rows[m]][K] (STORE/RESID), or {gate, up} (SWIGLU)
    const void* w[3];
    int rows[3];
    int total_rows;      // output rows
    float* out;          // fp32 [ncols][out_stride]
    bf16_t* out_hi;      // optional split copy of the output for an MFMA consumer
    bf16_t* out_lo;
    int out_stride;
    int ncols;
    // MODE_QKV_ROPE only: rotate q and k, append k and v to this block's cache
    const float2* rope_cs;   // [columns of the pass][hd/2] (cos, sin) of pos * base^(-2j/hd)
    void* k_cache;           // this block's [max_batch][H_kv][max_seq][hd]
    void* v_cache;
    ColMap cm;
    int col0;                // pass column of this launch's column 0
    int H, H_kv, hd, max_seq, kv_dtype;
    // MFMA path, RMSNorm folded into the projections around it.  A projection whose input is a normalised
    // residual (STORE, SWIGLU) gets x * gain pre-split in x_hi/x_lo and scales its sums by
    // 1/sqrt(sum(ssq_in[col][0..ssq_parts)) / K + eps); a residual projection (RESID) with ssq_out set also
    // writes the split of (new x) * gain_next to out_hi/out_lo and its workgroup's sum of squares of the new x
    // to ssq_out[col][workgroup].
    const float* ssq_in;     // [ncols][kSsqStride]
    int ssq_parts;
    float* ssq_out;          // [ncols][kSsqStride]
    const float* gain_next;  // [total_rows]
    // wide MFMA kernel (17..32 columns), K cut into slices: partial accumulators and one arrival counter per row
    // group (zero between launches)
    float* part;
    int* part_tickets;
};

// Launch-shape overrides for measurements, read from the environment ONCE by d3_create (0 / default = the library's
// own choice).  D3_MFMA_RT, D3_MFMA_WAVES: row tiles per workgroup and waves of the narrow matrix-core projection;
// D3_MFMA_WIDE=0: no panel kernel (passes are limited to kMaxCols columns); D3_WIDE_RT, D3_WIDE_KS: row tiles per wave
// and K slices of the panel kernel; D3_WIDE_SPLIT_MB: matrix size above which a pass of more than 64 columns runs as
// two 64-column launches; D3_ATTN_MFMA=0: grouped-query and query-tile attention on the vector ALUs;
// D3_ATTN_MIN_SPLIT: shortest context split; D3_PREFILL_COLS: columns per prompt chunk (a multiple of 64, at most 2048); D3_PROMPT_KS: K parts of a residual projection of the prompt pass (1..4); D3_GEMV_WGS_PER_CU: workgroups
// per compute unit of the vector-ALU GEMV (default 3).
struct Tuning {
    int gemv_wgs_per_cu = 3;
    int mfma_rt = 0, mfma_waves = 0;
    bool mfma_wide = true;
    int wide_rt = 0, wide_ks = 0;
    size_t wide_split_mb = 300;
    bool attn_mfma = true;
    int attn_min_split = 128;
    int prefill_cols = 0;
    int prompt_ks = 0;
};
Tuning tuning_from_env();

// returns hipError_t as int
int launch_gemv_alu(const GemvArgs& a, int weight_dtype, int mode, bool norm, int n_wg, hipStream_t s);
// n_groups: workgroups launched (= parts written to ssq_out)
int launch_gemm_mfma(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups = nullptr);
int launch_gemm_mfma_wide(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups);   // 17..128 columns
int launch_gemm_prompt(const GemvArgs& a, int mode, int n_cu, const Tuning& tn, hipStream_t s, int* n_groups);   // 129..kPassCols columns: LDS-tiled, compute-bound
size_t gemv_alu_max_cols(int K, int weight_dtype);   // columns one ALU launch can take (LDS bound)

// first step of a pass on the MFMA path: hi + lo = x * gain (bf16 halves), ssq[col * kSsqStride] = sum(x^2)
int launch_gain_split(const float* x, int x_stride, const float* gain, int K, int ncols,
                      bf16_t* hi, bf16_t* lo, float* ssq, hipStream_t s);

// ---------------- the rest of a block ----------------
// x[c][:] = E[token(c)][:], and the pass's rotary table rope_cs[c][j] = (cos, sin)((pos(c) - row0[seq(c)]) * inv_freq[j])
// (row0 optional: the first cache row of each sequence of a left-padded batch)
int launch_embed(const void* tok_emb, int weight_dtype, const int32_t* tokens, ColMap cm, int ncols, int d,
                 int vocab, float* x, const double* inv_freq, int half_hd, float2* rope_cs, const int* row0, hipStream_t s);

struct RopeArgs {
    float* qkv;            // [ncols][(H + 2 H_kv) * hd] fp32: q rotated in place
    void* k_cache;         // this block's [max_batch][H_kv][max_seq][hd]
    void* v_cache;
    const float2* rope_cs;   // [ncols][hd/2] (cos, sin) of this pass
    ColMap cm;
    int ncols, H, H_kv, hd, max_seq;
};
int launch_rope_append(const RopeArgs& a, int kv_dtype, hipStream_t s);

struct AttnArgs {
    const float* q;        // [ncols][q_stride]: q heads, then (rope_cs set) the newest k and v rows; rotated unless rope_cs is set
    const float2* rope_cs; // optional [ncols][hd/2] (cos, sin): rotate q and k here and append the newest K/V row
    const int* row0;       // optional [B]: first cache row of each sequence (a left-padded batch); rows below it are never read
    int qtile;             // the columns are consecutive positions of one sequence (a prompt chunk): tiles of queries share the cache rows
    int q_stride;
    const void* k_cache;   // this block's cache
    const void* v_cache;
    ColMap cm;
    int ncols, H, H_kv, hd, max_seq;
    int split_len, n_splits;
    float* part_o;         // [ncols][H][n_splits][hd]
    float* part_ml;        // [ncols][H][n_splits][2]  (max, sum)
    int* tickets;          // [ncols][H] arrival counters, zero between launches
    float* out;            // [ncols][H*hd]
    bf16_t* out_hi;        // optional split copy
    bf16_t* out_lo;
};
int launch_attention(const AttnArgs& a, int kv_dtype, bool use_mfma, hipStream_t s);

int launch_argmax(const float* logits, int vocab, int ncols, int32_t* out, hipStream_t s);

struct FillArgs {
    void* k_cache;         // whole cache [L][max_batch][H_kv][max_seq][hd]
    void* v_cache;
    int max_batch, H_kv, max_seq, hd;
    int B, pos_begin, pos_end;
    int drop_begin, n_drop, src;   // src < 0: zero fill
};
int launch_fill(const FillArgs& a, int kv_dtype, hipStream_t s);

// read-only streaming yardstick: reads `bytes` (a multiple of 16) once; sink: n_wg * 4 words
int launch_stream_read(const void* src, size_t bytes, unsigned* sink, int n_wg, hipStream_t s);
int launch_mfma_yardstick(int mode, int stages, int n_wg, float* sink, hipStream_t s);   // gemm_prompt.hip

// The words of state a decode step expects in its scratch area, passed by value (no host buffer to copy from) and
// written by one small kernel, which also zeroes the arrival counters.
struct StaticSeed {
    double inv_freq[64];   // head_dim / 2 <= 64 rotary frequencies
    int row0[kMaxCols];    // first cache row of each sequence (all zero unless the batch is left-padded)
};
int launch_static_seed(const StaticSeed& seed, double* inv_freq, int half_hd, int* row0, int* tickets, int n_tickets,
                       int* gemm_tickets, int n_gemm_tickets, hipStream_t s);

}  // namespace d3
