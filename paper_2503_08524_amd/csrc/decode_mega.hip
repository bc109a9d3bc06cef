// One decode step as ONE persistent kernel (batch 1, bf16 weights, head_dim 128).
//
// Launching each projection as its own kernel costs 7-9 us of fill, drain and cache
// write-back per launch, about as much as streaming the matrix itself at the 7B shape.  Here
// the whole step (embedding, every kept block, lm_head, argmax) is one cooperative launch
// of n_cu workgroups that stay resident; the phases of a block are separated by software grid
// barriers.  A workgroup has eight compute waves and one service wave:
//   * a compute wave, once its results are out, issues the loads of its first weight rows of the
//     NEXT projection and only then waits, so HBM keeps streaming through the barrier;
//   * the service wave owns the barrier (arrive, poll) and then stages the next projection's
//     activations into LDS.  It holds no weight loads: vector memory returns in order within a
//     wave, so an atomic or an activation load issued behind a ring of weight loads would only
//     come back after all of them.
//
// Data that crosses a barrier (residual stream, q/k/v, attention partials, activations) is
// written and read with agent-scope accesses; weights and older cache rows are read-only for
// the lifetime of the launch and use ordinary (streaming) loads.  Every wait is bounded: a
// service wave that polls too long raises the abort flag and the whole grid drains.
#include <type_traits>

#include "attention.h"
#include "decode_mega.h"
#include "gemv_alu.h"

namespace d3 {

namespace {

constexpr int kCW = 8;                       // compute waves per workgroup
constexpr int kWavesAll = kCW + 1;           // + the service wave
constexpr int kThreads = kWavesAll * 64;

__device__ __forceinline__ unsigned ld_agent_u(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

struct Barrier {
    unsigned* state;      // [8 groups x 32 words][global @ 256][abort @ 288]
    unsigned epoch;       // grid barriers completed so far (carried across launches by the host)
    unsigned local;       // boundaries passed in this launch (for the workgroup's own arrival counter)
    int group, per_group, n_groups;
    int max_spins;
};

struct WgSync {           // in LDS
    unsigned arrived;     // compute waves whose stores are out, monotonic over the launch
    int alive;
};

struct Stamps {            // debug timeline, one row of `stride` marks per workgroup
    unsigned long long* ts;
    int n, stride;
    __device__ __forceinline__ void mark() {
        if (ts && threadIdx.x == 0 && n < stride) ts[(size_t)blockIdx.x * stride + n] = wall_clock64();
        n += 1;
    }
};

// Service wave: wait until the workgroup's compute waves have their stores out (`lds_target` arrivals
// in total), then run the grid barrier.  Tree barrier: workgroups arrive on their group's counter
// (group = blockIdx % 8, the XCD under round-robin dispatch), the last arriver of a group arrives on
// the global counter, everyone polls the global counter.  Returns false if the grid is being aborted.
__device__ __forceinline__ bool barrier_service(Barrier& b, WgSync* ws, unsigned lds_target) {
    int ok = 1;
    if ((threadIdx.x & 63) == 0) {
        int spins = 0;
        while (__hip_atomic_load(&ws->arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < lds_target) {
            if (++spins > b.max_spins) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (ok) {
            const unsigned old = atomicAdd(&b.state[b.group * 32], 1u);
            if (old + 1u == b.epoch * (unsigned)b.per_group) atomicAdd(&b.state[256], 1u);
            const unsigned target = b.epoch * (unsigned)b.n_groups;
            spins = 0;
            while ((int)(ld_agent_u(&b.state[256]) - target) < 0) {
                if (++spins > b.max_spins || ((spins & 63) == 0 && ld_agent_u(&b.state[288]) != 0u)) { ok = 0; break; }
                __builtin_amdgcn_s_sleep(1);
            }
        }
        if (!ok) __hip_atomic_store(&b.state[288], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    ok = __shfl(ok, 0, 64);
    return ok != 0;
}

template <typename T, int kD>
__global__ __launch_bounds__(kThreads) void decode_mega_kernel(MegaArgs m) {
    typedef GemvPipe<bf16_t, kD> Pipe;
    extern __shared__ float4 lds[];                     // activations of the current projection / attention scores
    __shared__ float rinv_s[1];
    __shared__ GemvEpBuf<1> ep[kCW];
    __shared__ AttnShared<128, kWavesAll, 1> ash;
    __shared__ WgSync wsync;
    constexpr int HD = 128;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool svc = wave == kCW;
    const int n_wg = gridDim.x, wg = blockIdx.x;
    const int gw = wg * kCW + (svc ? 0 : wave), nw = n_wg * kCW;
    const int dm = m.d_model, qdim = m.H * HD, kvdim = m.H_kv * HD, qkv_dim = qdim + 2 * kvdim, F = m.d_ffn;

    Barrier bar;
    bar.state = m.barrier_state; bar.epoch = m.barrier_epoch; bar.local = 0; bar.max_spins = m.max_spins;
    bar.n_groups = n_wg < 8 ? n_wg : 8;
    bar.group = wg % bar.n_groups;
    bar.per_group = (n_wg - bar.group + bar.n_groups - 1) / bar.n_groups;
    if (tid == 0) { wsync.arrived = 0; wsync.alive = 1; }
    __syncthreads();

    // service-wave staging of one projection's input (one wave, agent-scope loads)
    __shared__ float red_s[1][1];
    auto stage = [&](const GemvArgs& a, auto norm_tag) {
        constexpr bool NORM = decltype(norm_tag)::value;
        GemvStageRegs<1, 8> regs;
        gemv_stage_issue<1, NORM, true, 64, 8>(a, lane, regs);
        gemv_stage_commit<bf16_t, 1, NORM, true, 64, 8>(a, lane, lds, regs, red_s);
        float r[1];
        __builtin_amdgcn_wave_barrier();
        gemv_inv_rms<1, NORM, 1>(a, red_s, r);
        if (lane == 0) rinv_s[0] = r[0];
    };
    typedef std::true_type TrueT;
    typedef std::false_type FalseT;

    const ColMap cm{0, 1, 1, m.pos};
    Pipe pipe;
    Stamps st{m.debug_ts, 0, m.debug_stride};
    GemvEpBuf<1>& my_ep = ep[svc ? 0 : wave];

    // A phase boundary.  Compute waves: results are out -> tell the service wave -> start the next
    // projection's weights.  Service wave: barrier, then stage the next projection's input.
#define D3_BOUNDARY(PRELOAD_STMT, STAGE_STMT)                                                     \
    do {                                                                                          \
        bar.epoch += 1; bar.local += 1;                                                           \
        wait_stores();                                                                            \
        if (!svc) {                                                                               \
            if (lane == 0) atomicAdd(&wsync.arrived, 1u);                                         \
            PRELOAD_STMT;                                                                         \
        } else {                                                                                  \
            const bool ok_ = barrier_service(bar, &wsync, bar.local * (unsigned)kCW);             \
            if (ok_) { STAGE_STMT; } else if (lane == 0) wsync.alive = 0;                         \
        }                                                                                         \
        __syncthreads();                                                                          \
        if (!wsync.alive) return;                                                                 \
    } while (0)

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
    if (m.n_ids > 0) make_qkv(m.layer_ids[0]);

    // ---- embedding + rotary table of this position (service waves), first weights already on their way ----
    if (!svc) {
        if (m.n_ids > 0) gemv_preload<bf16_t, MODE_QKV_ROPE, kD>(qkv, gw, nw, pipe);
        else gemv_preload<bf16_t, MODE_STORE, kD>(head, gw, nw, pipe);
    } else {
        int tok = m.tok_in[0];
        tok = tok < 0 ? 0 : (tok >= m.vocab ? m.vocab - 1 : tok);
        const bf16_t* row = static_cast<const bf16_t*>(m.tok_emb) + (size_t)tok * dm;
        for (int j = wg * 64 + lane; j < dm; j += n_wg * 64) st_agent(&m.x[j], bf16_to_f32(row[j]));
        if (wg == n_wg - 1) {
            double sn, cs;
            sincos((double)m.pos * m.inv_freq[lane], &sn, &cs);
            st_agent(reinterpret_cast<float*>(&m.rope_cs[lane]), (float)cs);
            st_agent(reinterpret_cast<float*>(&m.rope_cs[lane]) + 1, (float)sn);
        }
    }
    auto dump_x = [&](int slot) {            // debug tap: the residual stream as it stands (after a barrier)
        if (m.hidden_dump && wg == 0 && svc)
            for (int j = lane; j < dm; j += 64) m.hidden_dump[(size_t)slot * dm + j] = ld_agent(&m.x[j]);
    };
    float rinv[1];
    // the embedding's barrier passes without the compute waves' arrival: only service waves stored anything,
    // but the arrival counter is uniform, so they arrive all the same
    if (m.n_ids > 0) { D3_BOUNDARY((void)0, stage(qkv, TrueT{})); }
    else { D3_BOUNDARY((void)0, stage(head, TrueT{})); }
    dump_x(0);

    AttnArgs at{};
    at.q = m.qkv; at.q_stride = qkv_dim; at.cm = cm; at.ncols = 1; at.H = m.H; at.H_kv = m.H_kv; at.hd = HD; at.max_seq = m.max_seq;
    at.split_len = m.split_len; at.n_splits = m.n_splits; at.part_o = m.part_o; at.part_ml = m.part_ml; at.tickets = m.tickets;
    at.out = m.attn_o; at.out_hi = nullptr; at.out_lo = nullptr;

    for (int e = 0; e < m.n_ids; ++e) {
        const int l = m.layer_ids[e];
        const d3_layer_weights& w = m.layers[l];
        GemvArgs o{};
        o.x = m.attn_o; o.x_stride = qdim; o.K = qdim; o.w[0] = w.wo; o.rows[0] = dm; o.total_rows = dm; o.out = m.x; o.out_stride = dm; o.ncols = 1;
        GemvArgs u{};
        u.x = m.x; u.x_stride = dm; u.gain = static_cast<const float*>(w.mlp_norm); u.eps = m.eps; u.K = dm;
        u.w[0] = w.w_gate; u.w[1] = w.w_up; u.rows[0] = F; u.rows[1] = F; u.total_rows = F; u.out = m.act; u.out_stride = F; u.ncols = 1;
        GemvArgs dn{};
        dn.x = m.act; dn.x_stride = F; dn.K = F; dn.w[0] = w.w_down; dn.rows[0] = dm; dn.total_rows = dm; dn.out = m.x; dn.out_stride = dm; dn.ncols = 1;

        // A: RMSNorm + QKV + rotary embedding + cache append
        st.mark();
        rinv[0] = rinv_s[0];
        if (!svc) gemv_run<bf16_t, 1, MODE_QKV_ROPE, kD, true>(qkv, lds, gw, nw, pipe, my_ep, rinv);
        st.mark();
        // the O-projection's first rows stream while attention runs
        D3_BOUNDARY((gemv_preload<bf16_t, MODE_RESID, kD>(o, gw, nw, pipe)), (void)0);

        // B: attention over the cache (the newest row comes from the projection buffer); all nine waves
        at.k_cache = qkv.k_cache; at.v_cache = qkv.v_cache;
        st.mark();
        for (int item = wg; item < m.H * m.n_splits; item += n_wg) {
            attn_split<T, HD, true, kWavesAll, 1>(at, item % m.n_splits, item / m.n_splits, 0, ash);
            __syncthreads();
        }
        st.mark();
        D3_BOUNDARY((void)0, stage(o, FalseT{}));

        // C: x += Wo . attention
        st.mark();
        rinv[0] = 1.0f;
        if (!svc) gemv_run<bf16_t, 1, MODE_RESID, kD, true>(o, lds, gw, nw, pipe, my_ep, rinv);
        st.mark();
        D3_BOUNDARY((gemv_preload<bf16_t, MODE_SWIGLU, kD>(u, gw, nw, pipe)), stage(u, TrueT{}));

        // D: RMSNorm + gate/up + SiLU(gate) * up
        st.mark();
        rinv[0] = rinv_s[0];
        if (!svc) gemv_run<bf16_t, 1, MODE_SWIGLU, kD, true>(u, lds, gw, nw, pipe, my_ep, rinv);
        st.mark();
        D3_BOUNDARY((gemv_preload<bf16_t, MODE_RESID, kD>(dn, gw, nw, pipe)), stage(dn, FalseT{}));

        // E: x += Wd . act
        st.mark();
        rinv[0] = 1.0f;
        if (!svc) gemv_run<bf16_t, 1, MODE_RESID, kD, true>(dn, lds, gw, nw, pipe, my_ep, rinv);
        st.mark();
        if (e + 1 < m.n_ids) {
            make_qkv(m.layer_ids[e + 1]);
            D3_BOUNDARY((gemv_preload<bf16_t, MODE_QKV_ROPE, kD>(qkv, gw, nw, pipe)), stage(qkv, TrueT{}));
        } else {
            D3_BOUNDARY((gemv_preload<bf16_t, MODE_STORE, kD>(head, gw, nw, pipe)), stage(head, TrueT{}));
        }
        dump_x(e + 1);
    }

    // F: final RMSNorm + lm_head; every compute wave keeps the best of its own logits
    rinv[0] = rinv_s[0];
    if (!svc) {
        gemv_run<bf16_t, 1, MODE_STORE, kD, true>(head, lds, gw, nw, pipe, my_ep, rinv);
        // the wave's parked units still sit in its LDS buffer: scan them for the argmax
        const int n_units = m.vocab / 2;
        const int mine = gw < n_units ? (n_units - gw + nw - 1) / nw : 0;
        float best = -INFINITY;
        int idx = 0x7fffffff;
        for (int t = lane; t < mine; t += 64) {
            const int row = my_ep.row[t];
            const float v0 = my_ep.s[t][0][0], v1 = my_ep.s[t][0][1];
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
    D3_BOUNDARY((void)0, (void)0);

    // G: greedy argmax over the waves' candidates, lowest index on ties
    if (wg == 0 && svc) {
        float best = -INFINITY;
        int idx = 0x7fffffff;
        for (int t = lane; t < nw; t += 64) {
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
        if (lane == 0) m.tok_out[0] = idx >= m.vocab ? 0 : idx;
    }
#undef D3_BOUNDARY
}

const void* mega_kernel(int kv_dtype, int depth) {
#define D3_PICK(T) (depth >= 12 ? (const void*)decode_mega_kernel<T, 12> : (const void*)decode_mega_kernel<T, 8>)
    return kv_dtype == 0 ? D3_PICK(float) : kv_dtype == 1 ? D3_PICK(bf16_t) : D3_PICK(f16_t);
#undef D3_PICK
}

}  // namespace

size_t mega_lds_bytes(const MegaArgs& m) {
    int widest = m.d_model > m.d_ffn ? m.d_model : m.d_ffn;
    if (m.H * 128 > widest) widest = m.H * 128;
    size_t xs = (size_t)gemv_f4_per_col<bf16_t>(widest) * sizeof(float4);
    const size_t sc = (size_t)m.split_len * sizeof(float);
    return xs > sc ? xs : sc;
}

int mega_compute_waves() { return kCW; }

int mega_max_workgroups(int kv_dtype, int depth, size_t lds_bytes, int n_cu) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mega_kernel(kv_dtype, depth), kThreads, lds_bytes) != hipSuccess) return 0;
    return per_cu * n_cu;
}

// Requirements (checked by the caller): bf16 weights, head_dim 128, batch 1, a wave parks at most
// kGemvEpCap units per projection, n_wg <= mega_max_workgroups (the launch is cooperative, so the
// runtime refuses a grid that cannot be co-resident).  depth: weight-load steps in flight per wave (8 or 12).
int launch_decode_mega(const MegaArgs& m, int kv_dtype, int depth, int n_wg, hipStream_t s) {
    const size_t lds = mega_lds_bytes(m);
    MegaArgs copy = m;
    void* args[] = {&copy};
    return (int)hipLaunchCooperativeKernel(mega_kernel(kv_dtype, depth), dim3(n_wg), dim3(kThreads), args, (unsigned)lds, s);
}

}  // namespace d3
