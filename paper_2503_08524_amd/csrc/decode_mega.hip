// One decode step as ONE persistent kernel (batch 1, bf16 weights, head_dim 128).
//
// Launching each projection as its own kernel costs 7-9 us of fill, drain and cache
// write-back per launch, about as much as streaming the matrix itself at the 7B shape.  Here
// the whole step (embedding, every kept block, lm_head, argmax) is one cooperative launch
// of n_cu x {1,2} workgroups that stay resident; the phases of a block are separated by
// software grid barriers, and before a wave arrives at a barrier it has already issued the
// loads of its first weight rows of the next projection, so HBM keeps streaming while the
// barrier and the staging of the next activations are in flight.
//
// Data that crosses a barrier (residual stream, q/k/v, attention partials, activations) is
// written and read with agent-scope accesses; weights and older cache rows are read-only for
// the lifetime of the launch and use ordinary (streaming) loads.  Every wait is bounded: a wave
// that polls a barrier too long raises the abort flag and the whole grid drains.
#include "attention.h"
#include "decode_mega.h"
#include "gemv_alu.h"

namespace d3 {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ unsigned ld_agent_u(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

struct Barrier {
    unsigned* state;      // [8 groups x 32 words][global @ 256][abort @ 288]
    unsigned epoch;       // barriers completed so far (carried across launches by the host)
    int group, per_group, n_groups;
    int max_spins;
    bool dead;
};

// Tree barrier: workgroups arrive on their group's counter (group = blockIdx % 8, which is the XCD
// under round-robin dispatch), the last arriver of a group arrives on the global counter, everyone
// polls the global counter.  Returns false if the grid is being aborted.
// The caller has already waited for its own stores (wait_stores) before any prefetch it issued.
__device__ __forceinline__ bool grid_barrier(Barrier& b) {
    __syncthreads();
    b.epoch += 1;
    if (threadIdx.x == 0 && !b.dead) {
        const unsigned old = atomicAdd(&b.state[b.group * 32], 1u);
        if (old + 1u == b.epoch * (unsigned)b.per_group) atomicAdd(&b.state[256], 1u);
        const unsigned target = b.epoch * (unsigned)b.n_groups;
        int spins = 0;
        while ((int)(ld_agent_u(&b.state[256]) - target) < 0) {
            if (++spins > b.max_spins || ((spins & 63) == 0 && ld_agent_u(&b.state[288]) != 0u)) {
                __hip_atomic_store(&b.state[288], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                b.dead = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    }
    // thread 0's verdict reaches the workgroup through LDS
    __shared__ int alive;
    if (threadIdx.x == 0) alive = b.dead ? 0 : 1;
    __syncthreads();
    b.dead = alive == 0;
    return !b.dead;
}

struct Stamps {            // debug timeline, one row of `stride` marks per workgroup
    unsigned long long* ts;
    int n, stride;
    __device__ __forceinline__ void mark() {
        if (ts && threadIdx.x == 0 && n < stride) ts[(size_t)blockIdx.x * stride + n] = wall_clock64();
        n += 1;
    }
};

template <int MODE, bool NORM, int kD>
__device__ __forceinline__ void gemv_phase(const GemvArgs& a, float4* xs, float (*red)[kWaves], GemvEpBuf<1>& ep, GemvPipe<bf16_t, kD>& pipe,
                                           int gw, int nw, Stamps& st) {
    float ss[1];
    gemv_stage_load<bf16_t, 1, NORM, true, kThreads>(a, xs, ss);
    gemv_stage_norm<bf16_t, 1, NORM, kThreads>(a, xs, ss, red);
    __syncthreads();
    st.mark();
    gemv_run<bf16_t, 1, MODE, kD, true>(a, xs, gw, nw, pipe, ep);
    st.mark();
}

template <typename T, int kD>
__global__ __launch_bounds__(kThreads) void decode_mega_kernel(MegaArgs m) {
    typedef GemvPipe<bf16_t, kD> Pipe;
    extern __shared__ float4 lds[];                     // activations of the current projection / attention scores
    __shared__ float red[1][kWaves];
    __shared__ GemvEpBuf<1> ep[kWaves];
    __shared__ AttnShared<128> ash;
    constexpr int HD = 128;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n_wg = gridDim.x, wg = blockIdx.x;
    const int gw = wg * kWaves + wave, nw = n_wg * kWaves;
    const int dm = m.d_model, qdim = m.H * HD, kvdim = m.H_kv * HD, qkv_dim = qdim + 2 * kvdim, F = m.d_ffn;

    Barrier bar;
    bar.state = m.barrier_state; bar.epoch = m.barrier_epoch; bar.max_spins = m.max_spins; bar.dead = false;
    bar.n_groups = n_wg < 8 ? n_wg : 8;
    bar.group = wg % bar.n_groups;
    bar.per_group = (n_wg - bar.group + bar.n_groups - 1) / bar.n_groups;

    const ColMap cm{0, 1, 1, m.pos};
    Pipe pipe;
    Stamps st{m.debug_ts, 0, m.debug_stride};

    // ---- first projection's weights start streaming, then the embedding and the rotary table ----
    GemvArgs qkv{};
    auto make_qkv = [&](int l) {
        const d3_layer_weights& w = m.layers[l];
        qkv = GemvArgs{};
        qkv.x = m.x; qkv.x_stride = dm; qkv.gain = static_cast<const float*>(w.attn_norm); qkv.eps = m.eps; qkv.K = dm;
        qkv.w[0] = w.wq; qkv.w[1] = w.wk; qkv.w[2] = w.wv; qkv.rows[0] = qdim; qkv.rows[1] = kvdim; qkv.rows[2] = kvdim;
        qkv.total_rows = qkv_dim; qkv.out = m.qkv; qkv.out_stride = qkv_dim; qkv.ncols = 1;
        qkv.rope_cs = m.rope_cs; qkv.k_cache = m.k_cache + (size_t)l * m.kv_layer_bytes; qkv.v_cache = m.v_cache + (size_t)l * m.kv_layer_bytes;
        qkv.cm = cm; qkv.col0 = 0; qkv.H = m.H; qkv.H_kv = m.H_kv; qkv.hd = HD; qkv.max_seq = m.max_seq; qkv.kv_dtype = m.kv_dtype;
    };
    GemvArgs head{};
    head.x = m.x; head.x_stride = dm; head.gain = m.final_norm; head.eps = m.eps; head.K = dm;
    head.w[0] = m.lm_head; head.rows[0] = m.vocab; head.total_rows = m.vocab; head.out = m.logits; head.out_stride = m.vocab; head.ncols = 1;

    if (m.n_ids > 0) { make_qkv(m.layer_ids[0]); gemv_preload<bf16_t, MODE_QKV_ROPE, kD>(qkv, gw, nw, pipe); }
    else gemv_preload<bf16_t, MODE_STORE, kD>(head, gw, nw, pipe);

    {
        int tok = m.tok_in[0];
        tok = tok < 0 ? 0 : (tok >= m.vocab ? m.vocab - 1 : tok);
        const bf16_t* row = static_cast<const bf16_t*>(m.tok_emb) + (size_t)tok * dm;
        for (int j = wg * kThreads + tid; j < dm; j += n_wg * kThreads) st_agent(&m.x[j], bf16_to_f32(row[j]));
        if (wg == n_wg - 1 && tid < HD / 2) {
            double sn, cs;
            sincos((double)m.pos * m.inv_freq[tid], &sn, &cs);
            st_agent(reinterpret_cast<float*>(&m.rope_cs[tid]), (float)cs);
            st_agent(reinterpret_cast<float*>(&m.rope_cs[tid]) + 1, (float)sn);
        }
    }
    wait_stores();
    if (!grid_barrier(bar)) return;
    auto dump_x = [&](int slot) {            // debug tap: the residual stream as it stands
        if (m.hidden_dump && wg == 0)
            for (int j = tid; j < dm; j += kThreads) m.hidden_dump[(size_t)slot * dm + j] = ld_agent(&m.x[j]);
    };
    dump_x(0);

    AttnArgs at{};
    at.q = m.qkv; at.q_stride = qkv_dim; at.cm = cm; at.ncols = 1; at.H = m.H; at.H_kv = m.H_kv; at.hd = HD; at.max_seq = m.max_seq;
    at.split_len = m.split_len; at.n_splits = m.n_splits; at.part_o = m.part_o; at.part_ml = m.part_ml; at.tickets = m.tickets;
    at.out = m.attn_o; at.out_hi = nullptr; at.out_lo = nullptr;

    for (int e = 0; e < m.n_ids; ++e) {
        const int l = m.layer_ids[e];
        const d3_layer_weights& w = m.layers[l];

        // A: RMSNorm + QKV + rotary embedding + cache append
        st.mark();
        gemv_phase<MODE_QKV_ROPE, true, kD>(qkv, lds, red, ep[wave], pipe, gw, nw, st);
        wait_stores();                      // q, k, v are out before the next loads queue up behind them

        // the O-projection's first rows stream while attention runs
        GemvArgs o{};
        o.x = m.attn_o; o.x_stride = qdim; o.K = qdim; o.w[0] = w.wo; o.rows[0] = dm; o.total_rows = dm; o.out = m.x; o.out_stride = dm; o.ncols = 1;
        gemv_preload<bf16_t, MODE_RESID, kD>(o, gw, nw, pipe);
        if (!grid_barrier(bar)) return;

        // B: attention over the cache (the newest row comes from the projection buffer)
        at.k_cache = qkv.k_cache; at.v_cache = qkv.v_cache;
        st.mark();
        for (int item = wg; item < m.H * m.n_splits; item += n_wg) {
            attn_split<T, HD, true>(at, item % m.n_splits, item / m.n_splits, 0, reinterpret_cast<float*>(lds), ash);
            __syncthreads();
        }
        wait_stores();
        st.mark();
        if (!grid_barrier(bar)) return;

        // C: x += Wo . attention
        st.mark();
        gemv_phase<MODE_RESID, false, kD>(o, lds, red, ep[wave], pipe, gw, nw, st);
        wait_stores();
        GemvArgs u{};
        u.x = m.x; u.x_stride = dm; u.gain = static_cast<const float*>(w.mlp_norm); u.eps = m.eps; u.K = dm;
        u.w[0] = w.w_gate; u.w[1] = w.w_up; u.rows[0] = F; u.rows[1] = F; u.total_rows = F; u.out = m.act; u.out_stride = F; u.ncols = 1;
        gemv_preload<bf16_t, MODE_SWIGLU, kD>(u, gw, nw, pipe);
        if (!grid_barrier(bar)) return;

        // D: RMSNorm + gate/up + SiLU(gate) * up
        st.mark();
        gemv_phase<MODE_SWIGLU, true, kD>(u, lds, red, ep[wave], pipe, gw, nw, st);
        wait_stores();
        GemvArgs dn{};
        dn.x = m.act; dn.x_stride = F; dn.K = F; dn.w[0] = w.w_down; dn.rows[0] = dm; dn.total_rows = dm; dn.out = m.x; dn.out_stride = dm; dn.ncols = 1;
        gemv_preload<bf16_t, MODE_RESID, kD>(dn, gw, nw, pipe);
        if (!grid_barrier(bar)) return;

        // E: x += Wd . act
        st.mark();
        gemv_phase<MODE_RESID, false, kD>(dn, lds, red, ep[wave], pipe, gw, nw, st);
        wait_stores();
        if (e + 1 < m.n_ids) { make_qkv(m.layer_ids[e + 1]); gemv_preload<bf16_t, MODE_QKV_ROPE, kD>(qkv, gw, nw, pipe); }
        else gemv_preload<bf16_t, MODE_STORE, kD>(head, gw, nw, pipe);
        if (!grid_barrier(bar)) return;
        dump_x(e + 1);
    }

    // F: final RMSNorm + lm_head; every wave keeps the best of its own logits
    {
        float ss[1];
        gemv_stage_load<bf16_t, 1, true, true, kThreads>(head, lds, ss);
        gemv_stage_norm<bf16_t, 1, true, kThreads>(head, lds, ss, red);
        __syncthreads();
        gemv_run<bf16_t, 1, MODE_STORE, kD, true>(head, lds, gw, nw, pipe, ep[wave]);
        // the wave's parked units still sit in its LDS buffer: scan them for the argmax
        const int n_units = m.vocab / 2;
        const int mine = gw < n_units ? (n_units - gw + nw - 1) / nw : 0;
        float best = -INFINITY;
        int idx = 0x7fffffff;
        for (int t = lane; t < mine; t += 64) {
            const int row = ep[wave].row[t];
            const float v0 = ep[wave].s[t][0][0], v1 = ep[wave].s[t][0][1];
            if (v0 > best || (v0 == best && row < idx)) { best = v0; idx = row; }
            if (v1 > best || (v1 == best && row + 1 < idx)) { best = v1; idx = row + 1; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(best, off, 64);
            const int oi = __shfl_xor(idx, off, 64);
            if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
        }
        if (lane == 0) { st_agent(&m.cand_val[gw], best); st_agent(reinterpret_cast<float*>(&m.cand_idx[gw]), __int_as_float(idx)); }
    }
    wait_stores();
    if (!grid_barrier(bar)) return;

    // G: greedy argmax over the waves' candidates, lowest index on ties
    if (wg == 0) {
        __shared__ float bv[kWaves];
        __shared__ int bi[kWaves];
        float best = -INFINITY;
        int idx = 0x7fffffff;
        for (int t = tid; t < nw; t += kThreads) {
            const float v = ld_agent(&m.cand_val[t]);
            const int i = __float_as_int(ld_agent(reinterpret_cast<const float*>(&m.cand_idx[t])));
            if (v > best || (v == best && i < idx)) { best = v; idx = i; }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(best, off, 64);
            const int oi = __shfl_xor(idx, off, 64);
            if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
        }
        if (lane == 0) { bv[wave] = best; bi[wave] = idx; }
        __syncthreads();
        if (tid == 0) {
            for (int w2 = 1; w2 < kWaves; ++w2)
                if (bv[w2] > best || (bv[w2] == best && bi[w2] < idx)) { best = bv[w2]; idx = bi[w2]; }
            m.tok_out[0] = idx >= m.vocab ? 0 : idx;
        }
    }
}

}  // namespace

size_t mega_lds_bytes(const MegaArgs& m) {
    int widest = m.d_model > m.d_ffn ? m.d_model : m.d_ffn;
    if (m.H * 128 > widest) widest = m.H * 128;
    size_t xs = (size_t)gemv_f4_per_col<bf16_t>(widest) * sizeof(float4);
    const size_t sc = (size_t)m.split_len * sizeof(float);
    return xs > sc ? xs : sc;
}

namespace {
const void* mega_kernel(int kv_dtype, int depth) {
#define D3_PICK(T) (depth >= 16 ? (const void*)decode_mega_kernel<T, 16> : depth >= 12 ? (const void*)decode_mega_kernel<T, 12> : (const void*)decode_mega_kernel<T, 8>)
    return kv_dtype == 0 ? D3_PICK(float) : kv_dtype == 1 ? D3_PICK(bf16_t) : D3_PICK(f16_t);
#undef D3_PICK
}
}  // namespace

int mega_max_workgroups(int kv_dtype, int depth, size_t lds_bytes, int n_cu) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mega_kernel(kv_dtype, depth), kThreads, lds_bytes) != hipSuccess) return 0;
    return per_cu * n_cu;
}

// Requirements (checked by the caller): bf16 weights, head_dim 128, batch 1, a wave parks at most
// kGemvEpCap units per projection, n_wg <= mega_max_workgroups (the launch is cooperative, so the
// runtime refuses a grid that cannot be co-resident).  depth: weight-load steps in flight per wave (8, 12 or 16).
int launch_decode_mega(const MegaArgs& m, int kv_dtype, int depth, int n_wg, hipStream_t s) {
    const size_t lds = mega_lds_bytes(m);
    MegaArgs copy = m;
    void* args[] = {&copy};
    return (int)hipLaunchCooperativeKernel(mega_kernel(kv_dtype, depth), dim3(n_wg), dim3(kThreads), args, (unsigned)lds, s);
}

}  // namespace d3
