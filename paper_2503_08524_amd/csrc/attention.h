// Device-side body of the decode attention (see attention.hip).
#pragma once
#include "d3_common.h"

namespace d3 {

template <typename T> struct KvVec;
template <> struct KvVec<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ float round(float v) { return v; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct KvVec<f16_t> {
    static constexpr int N = 8;
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
        const half8 h = __builtin_bit_cast(half8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (float)h[e];
    }
    static __device__ __forceinline__ float round(float v) { return (float)(f16_t)fminf(fmaxf(v, -65504.f), 65504.f); }
    static __device__ __forceinline__ void store(f16_t* p, float v) { *p = (f16_t)fminf(fmaxf(v, -65504.f), 65504.f); }
};

// Sum over each aligned group of LPR lanes, every lane of a group ending with the same bits.  Sixteen lanes
// are one DPP row: four rotate-and-add steps on the vector ALU instead of four trips through the LDS crossbar
// (after the step by 8 the values have period 8, after the step by 4 period 4, ..., so all lanes agree exactly).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
    if (LPR == 16) {
        v += dpp_move<0x128>(v);           // row_ror:8
        v += dpp_move<0x124>(v);           // row_ror:4
        v += dpp_move<0x122>(v);           // row_ror:2
        v += dpp_move<0x121>(v);           // row_ror:1
    } else {
#pragma unroll
        for (int o = LPR / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    }
    return v;
}

template <int HD, int NW, int G>
struct AttnShared {
    float m[G][NW], l[G][NW];              // per wave: running max and sum of each head's scores
    float o[G][NW][HD];                    // per wave: unnormalised output of each head
    int is_last;
};

// Second half of a split (all waves have put their running max, sum and unnormalised output of every head
// into `sh` and passed a barrier): merge the waves, publish the split's partial of every head, and let the
// split that arrives last at the (column, KV head) counter merge all splits and write the output.
//
// The G entries of `sh` are GH heads of each of G / GH consecutive columns: entry e is head h0 + e % GH of column
// c + e / GH (decode: GH = G, one column; a prompt chunk's query tile: several columns).  Entries whose column
// lies past the pass are dropped.
template <int HD, bool FUSED, int NW, int G, int GH = G>
__device__ __forceinline__ void attn_merge_publish(const AttnArgs& a, int split, int h0, int c, int n_live, AttnShared<HD, NW, G>& sh) {
    const int tid = threadIdx.x;
    constexpr int RND = (G * HD > 4 * NW * 64) ? 2 : 8;   // splits fetched per round of the final merge (register budget)
    // ---- merge the waves; publish this split's partial of every head ----
    for (int idx = tid; idx < G * HD; idx += NW * 64) {
        const int g = idx / HD, t = idx % HD;
        const int ce = c + g / GH, he = h0 + g % GH;
        if (ce >= a.ncols) continue;
        float M = sh.m[g][0];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sh.m[g][w]);
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float f = sh.m[g][w] > -INFINITY ? exp2f(sh.m[g][w] - M) : 0.f;
            L += sh.l[g][w] * f;
            o += sh.o[g][w][t] * f;
        }
        if (n_live == 1) {                             // the only split of this column: the result is final
            const float r = o / L;
            const size_t oi = (size_t)ce * a.H * HD + (size_t)he * HD + t;
            if (FUSED) st_agent(&a.out[oi], r); else a.out[oi] = r;
            if (a.out_hi) {
                const uint32_t hb = f32_to_bf16(r);
                a.out_hi[oi] = (bf16_t)hb;
                a.out_lo[oi] = (bf16_t)f32_to_bf16(r - bf16_to_f32(hb));
            }
            continue;
        }
        const size_t pidx = ((size_t)ce * a.H + he) * a.n_splits + split;
        st_agent(&a.part_o[pidx * HD + t], o);
        if (t == 0) { st_agent(&a.part_ml[pidx * 2], M); st_agent(&a.part_ml[pidx * 2 + 1], L); }
    }

    if (n_live == 1) return;
    // ---- the split that arrives last merges all splits of this (column, KV head) ----
    wait_stores();                                     // this split's partials have reached the coherence point
    __syncthreads();
    if (tid == 0) {
        int* ticket = &a.tickets[c * a.H + h0];          // one counter per head group, indexed by its first query head
        const int done = atomicAdd(ticket, 1);
        sh.is_last = done == n_live - 1;
        if (sh.is_last) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // all arrived: leave it clean
    }
    __syncthreads();
    if (!sh.is_last) return;
    // every thread owns ITEMS (head, element) outputs; the partials of all of them are fetched together, in rounds
    // of 8 splits (one round trip per round), and merged with a running max
    constexpr int ITEMS = (G * HD + NW * 64 - 1) / (NW * 64);
    float gm[ITEMS], L[ITEMS], o[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) { gm[i] = -INFINITY; L[i] = 0.f; o[i] = 0.f; }
    for (int s0 = 0; s0 < n_live; s0 += RND) {
        float ms[ITEMS][RND], ls[ITEMS][RND], os[ITEMS][RND];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            int idx = tid + i * (NW * 64);
            idx = idx < G * HD ? idx : G * HD - 1;
            int ge = idx / HD;
            if (c + ge / GH >= a.ncols) ge = 0;           // a dropped entry re-reads entry 0 (the result is not stored)
            const size_t p0 = ((size_t)(c + ge / GH) * a.H + h0 + ge % GH) * a.n_splits;
#pragma unroll
            for (int k = 0; k < RND; ++k) {
                const int sidx = s0 + k < n_live ? s0 + k : n_live - 1;
                ms[i][k] = ld_agent(&a.part_ml[(p0 + sidx) * 2]);
                ls[i][k] = ld_agent(&a.part_ml[(p0 + sidx) * 2 + 1]);
                os[i][k] = ld_agent(&a.part_o[(p0 + sidx) * HD + idx % HD]);
            }
        }
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            float rm = gm[i];
#pragma unroll
            for (int k = 0; k < RND; ++k) if (s0 + k < n_live) rm = fmaxf(rm, ms[i][k]);
            const float keep = exp2f(gm[i] - rm);         // -inf on the first round: exp2(-inf) = 0
            L[i] *= keep; o[i] *= keep;
#pragma unroll
            for (int k = 0; k < RND; ++k) {
                if (s0 + k < n_live) {
                    const float w = exp2f(ms[i][k] - rm);
                    L[i] += ls[i][k] * w;
                    o[i] += os[i][k] * w;
                }
            }
            gm[i] = rm;
        }
    }
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
        const int idx = tid + i * (NW * 64);
        if (idx >= G * HD) continue;
        const int ge = idx / HD, ce = c + ge / GH;
        if (ce >= a.ncols) continue;
        const float r = o[i] / L[i];
        const size_t oi = (size_t)ce * a.H * HD + (size_t)(h0 + ge % GH) * HD + idx % HD;
        if (FUSED) st_agent(&a.out[oi], r); else a.out[oi] = r;
        if (a.out_hi) {
            const uint32_t hb = f32_to_bf16(r);
            a.out_hi[oi] = (bf16_t)hb;
            a.out_lo[oi] = (bf16_t)f32_to_bf16(r - bf16_to_f32(hb));
        }
    }
}

// One (column, KV head, context split) per call by a workgroup of NW waves, for the G query heads
// h0 .. h0+G-1 that share that KV head (G = 1: plain multi-head attention, or a group size the
// kernel is not instantiated for, handled one query head at a time).  Every cache row of the split is
// loaded ONCE into registers, 16 bytes per lane, and used for all G heads; K and V loads go out
// together, in chunks of up to ITMAX * RPB rows.  Each wave keeps an online softmax per head (running
// max, sum, unnormalised output; reductions by wave shuffles), the waves are merged through LDS, and the
// split that arrives last (arrival counter per (column, KV head)) merges all splits.
//
// FUSED: the call runs inside a kernel that also produced q and the newest K/V row in this launch:
// q and that row are read from the fp32 projection buffer with agent-scope loads (the row rounded
// to the cache's element type, i.e. exactly what later steps will read back), and the merged
// output is published with agent-scope stores.
//
// ROPE: q and the newest K/V row of every column arrive unrotated in the projection buffer, and that row
// is not in the cache yet (every column of the pass is a different sequence).  The workgroup rotates q
// while loading it (half-split pairing: dims j and j + HD/2 turn by the column's angle j), and the split
// that holds the newest position rotates k, rounds k and v to the cache's element type, uses them and
// appends them to the cache.
template <typename T, int HD, bool FUSED, int NW, int G, bool ROPE = false>
__device__ __forceinline__ void attn_split(const AttnArgs& a, int split, int h0, int c, AttnShared<HD, NW, G>& sh) {
    constexpr int EPL = KvVec<T>::N;       // elements per lane per 16-byte load
    constexpr int LPR = HD / EPL;          // lanes that share one cache row
    constexpr int RPW = 64 / LPR;          // rows per wave per load
    constexpr int RPB = RPW * NW;          // rows per workgroup per load
    constexpr int ITMAX = 8;               // loads of K (and of V) in flight per lane

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = a.cm.seq(c);
    const int row0 = a.row0 ? a.row0[seq] : 0;         // left-padded batch: this sequence's rows begin here; rows are counted from it
    const int ctx = a.cm.pos(c) + 1 - row0;
    const int j0 = split * a.split_len;
    const int jend = min(j0 + a.split_len, ctx);
    if (j0 >= jend) return;                // nothing of this column's context falls in this split
    const bool has_new = ROPE && jend == ctx;          // ROPE: the newest position comes from the projection buffer ...
    const int j1 = has_new ? ctx - 1 : jend;           // ... and the cache rows of this split end before it
    const int n_live = (ctx + a.split_len - 1) / a.split_len;   // splits of this column that hold rows
    const int kvh = h0 / (a.H / a.H_kv);
    const size_t head_off = (((size_t)seq * a.H_kv + kvh) * a.max_seq + row0) * HD;
    const T* Kb = static_cast<const T*>(a.k_cache) + head_off;
    const T* Vb = static_cast<const T*>(a.v_cache) + head_off;
    const int sub = lane % LPR, rg = lane / LPR;
    // FUSED: the newest row (ctx - 1) of this column, k then v, inside the projection buffer
    const float* cur_k = a.q + (size_t)c * a.q_stride + (size_t)(a.H + kvh) * HD + sub * EPL;
    const float* cur_v = cur_k + (size_t)a.H_kv * HD;
    // scores are kept in units of log2(e) so that every exponential is one hardware exp2
    const float scale = 1.4426950408889634f / sqrtf((float)HD);

    float m[G], l[G], acc[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
    }

    const int iters = (j1 - j0 + RPB - 1) / RPB;
    uint4 kv[ITMAX], vv[ITMAX];
    auto issue = [&](int it0) {
#pragma unroll
        for (int u = 0; u < ITMAX; ++u) {
            const int j = j0 + ((it0 + u) * NW + wave) * RPW + rg;
            const int jc = j < j1 ? j : j1 - 1;
            if (it0 + u < iters) {
                kv[u] = __builtin_bit_cast(uint4, load_stream16(Kb + (size_t)jc * HD + sub * EPL));   // each row is read once per step
                vv[u] = __builtin_bit_cast(uint4, load_stream16(Vb + (size_t)jc * HD + sub * EPL));
            }
        }
    };
    issue(0);
    __builtin_amdgcn_sched_barrier(0);     // the first chunk's cache rows are requested before q
    // ROPE: this lane's elements sit in the lower (partner HD/2 above) or upper (partner HD/2 below) half of the head
    const bool upper = sub * EPL >= HD / 2;
    const int poff = upper ? -(HD / 2) : HD / 2;
    float cosv[EPL], sinv[EPL], newk[EPL], newv[EPL];
    auto rotate = [&](const float* own, const float* partner, float* y) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) y[e] = upper ? partner[e] * sinv[e] + own[e] * cosv[e] : own[e] * cosv[e] - partner[e] * sinv[e];
    };
    auto load_vec = [&](const float* p, float* y) {
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
            const float4 t = *reinterpret_cast<const float4*>(p + e);
            y[e] = t.x; y[e + 1] = t.y; y[e + 2] = t.z; y[e + 3] = t.w;
        }
    };
    if (ROPE) {
        const float2* cs = a.rope_cs + (size_t)c * (HD / 2) + (sub * EPL) % (HD / 2);
#pragma unroll
        for (int e = 0; e < EPL; e += 2) {
            const float4 t = *reinterpret_cast<const float4*>(cs + e);
            cosv[e] = t.x; sinv[e] = t.y; cosv[e + 1] = t.z; sinv[e + 1] = t.w;
        }
        if (has_new) {
            float own[EPL], partner[EPL];
            load_vec(cur_k, own);
            load_vec(cur_k + poff, partner);
            rotate(own, partner, newk);
            load_vec(cur_v, newv);
#pragma unroll
            for (int e = 0; e < EPL; ++e) { newk[e] = KvVec<T>::round(newk[e]); newv[e] = KvVec<T>::round(newv[e]); }
            if (wave == 0 && rg == 0) {    // one copy of the row goes to the cache (the caches are this launch's to extend)
                T* kd = const_cast<T*>(Kb) + (size_t)(ctx - 1) * HD + sub * EPL;
                T* vd = const_cast<T*>(Vb) + (size_t)(ctx - 1) * HD + sub * EPL;
#pragma unroll
                for (int e = 0; e < EPL; ++e) { KvVec<T>::store(kd + e, newk[e]); KvVec<T>::store(vd + e, newv[e]); }
            }
        }
    }
    float qv[G][EPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const float* qp = a.q + (size_t)c * a.q_stride + (size_t)(h0 + g) * HD + sub * EPL;
        if (FUSED) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) qv[g][e] = ld_agent(qp + e);
        } else {
#pragma unroll
            for (int e = 0; e < EPL; e += 4) {
                const float4 t = *reinterpret_cast<const float4*>(qp + e);
                qv[g][e] = t.x; qv[g][e + 1] = t.y; qv[g][e + 2] = t.z; qv[g][e + 3] = t.w;
            }
            if (ROPE) {
                float partner[EPL], y[EPL];
                load_vec(qp + poff, partner);
                rotate(qv[g], partner, y);
#pragma unroll
                for (int e = 0; e < EPL; ++e) qv[g][e] = y[e];
            }
        }
    }
    if (has_new && wave == 0) {            // the newest row opens wave 0's running softmax: weight 1 at its own score
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float sn = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) sn = fmaf(qv[g][e], newk[e], sn);
            m[g] = group_sum<LPR>(sn) * scale;         // every row group holds the same q and k: the same score in all lanes
            if (rg == 0) {
                if (sub == 0) l[g] = 1.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] = newv[e];
            }
        }
    }
    for (int it0 = 0; it0 < iters; it0 += ITMAX) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float sv[ITMAX];
            float cmax = -INFINITY;
#pragma unroll
            for (int u = 0; u < ITMAX; ++u) {
                sv[u] = -INFINITY;
                if (it0 + u < iters) {
                    const int j = j0 + ((it0 + u) * NW + wave) * RPW + rg;
                    float kf[EPL];
                    KvVec<T>::unpack(kv[u], kf);
                    if (FUSED && j == ctx - 1) {
#pragma unroll
                        for (int e = 0; e < EPL; ++e) kf[e] = KvVec<T>::round(ld_agent(cur_k + e));
                    }

                    float s = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) s = fmaf(qv[g][e], kf[e], s);
                    s = group_sum<LPR>(s) * scale;
                    if (j < j1) { sv[u] = s; cmax = fmaxf(cmax, s); }
                }
            }
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, o, 64));   // equal within a row group already
            const float m_new = fmaxf(m[g], cmax);          // a wave with no valid row in this chunk keeps -inf
            if (m_new > -INFINITY) {
                const float keep = exp2f(m[g] - m_new);       // exp2(-inf) = 0 the first time
                l[g] *= keep;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] *= keep;
#pragma unroll
                for (int u = 0; u < ITMAX; ++u) {
                    if (it0 + u < iters) {
                        const int j = j0 + ((it0 + u) * NW + wave) * RPW + rg;
                        const float p = exp2f(sv[u] - m_new); // 0 for rows past the split (score -inf)
                        if (sub == 0) l[g] += p;
                        float vf[EPL];
                        KvVec<T>::unpack(vv[u], vf);
                        if (FUSED && j == ctx - 1) {
#pragma unroll
                            for (int e = 0; e < EPL; ++e) vf[e] = KvVec<T>::round(ld_agent(cur_v + e));
                        }

#pragma unroll
                        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(p, vf[e], acc[g][e]);
                    }
                }
                m[g] = m_new;
            }
        }
        if (it0 + ITMAX < iters) issue(it0 + ITMAX);
    }

    // ---- waves -> LDS ----
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) acc[g][e] += __shfl_xor(acc[g][e], o, 64);
        }
        const float lw = wave_sum(l[g]);
        if (rg == 0) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) sh.o[g][wave][sub * EPL + e] = acc[g][e];
        }
        if (lane == 0) { sh.m[g][wave] = m[g]; sh.l[g][wave] = lw; }
    }
    __syncthreads();

    attn_merge_publish<HD, FUSED, NW, G>(a, split, h0, c, n_live, sh);
}

// ---------------- grouped-query decode attention on the matrix cores ----------------
// With G query heads per KV head the vector-ALU kernel above does G times the arithmetic per cache byte
// and is bound by it (G = 8: 33 us for 34 MB at the 70B shape).  Here both contractions run as
// v_mfma_f32_16x16x32_f16 with the heads of the group (padded to 16) as one matrix dimension; fp16 cache,
// head_dim 128.  A wave takes 32 cache rows at a time:
//   scores^T [row][head] = K [row][hd] . q^T [hd][head]: A = a 16-row K tile (coalesced load, re-shaped through
//     LDS into fragments), B = q (scaled, split hi + lo in fp16): the result leaves lane (i, g) with head i,
//     rows 4g..4g+3 of the tile; two tiles give each lane 8 of the 32 rows of its head;
//   online softmax per head in that layout (max / sum across the 4 lanes of a head by shuffles);
//   out [head][col] += P [head][row] . V [row][col]: A = P (hi + lo in fp16), whose 8 rows per lane are exactly an A
//     fragment under the row numbering k = 8g + j <-> row 4g + j (j < 4), 16 + 4g + j - 4 (j >= 4);
//     B = V read from its LDS tile in the same numbering (eight 2-byte reads per fragment: V's contraction
//     index is the row, which is the slow index of the cache).
// The waves' states go through the same LDS merge, split partials and arrival counter as above.
typedef _Float16 attn_half8 __attribute__((ext_vector_type(8)));
typedef float attn_f32x4 __attribute__((ext_vector_type(4)));
constexpr int kAttnPitch = 272;            // bytes per staged row of 128 halves (+16: conflict-free fragment reads)

// B fragment of P.V for head-dim columns 16 nt .. 16 nt + 15 from a staged 32-row V tile: lane (i, g) gets column
// 16 nt + i of rows 4g..4g+3 and 16+4g..16+4g+3 (the row numbering the score tiles leave P in).  The contraction index
// is the tile's slow index, so each half is one LDS transpose read: inside a group of 16 lanes, lane s points at four
// consecutive columns (4 (s % 4)) of row s / 4, and lane i receives column i of those four rows.
typedef short attn_short4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ attn_half8 attn_v_fragment(const char* vbuf, int nt, int lane) {
    const int s = lane & 15, g = lane >> 4;
    const char* p = vbuf + (4 * g + (s >> 2)) * kAttnPitch + (16 * nt + 4 * (s & 3)) * 2;
    typedef __attribute__((address_space(3))) attn_short4 lds_short4;
    const attn_short4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(p));
    const attn_short4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(p + 16 * kAttnPitch));
    typedef short attn_short8 __attribute__((ext_vector_type(8)));
    const attn_short8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(attn_half8, both);
}

// PL planes per staged tile: 1 for an fp16 cache (the rows as they are), 2 for an fp32 cache (each row split into
// fp16 hi + lo, so that both contractions keep the cache's precision: K.q = Khi.q + Klo.q, P.V = P.Vhi + P.Vlo).
template <int NW, int G, int PL = 1>
struct AttnMfmaShared {
    union {
        struct {
            char k[NW][PL][16 * kAttnPitch];   // one K tile per wave
            char v[NW][PL][32 * kAttnPitch];   // one 32-row V tile per wave
            float keep[NW][16];                // rescale factor of each head, from the score layout to the output layout
        } stage;
        AttnShared<128, NW, G> merge;
    };
};

// Cache rows -> staged fp16 tiles.  A wave loads 32 rows of 128 elements with coalesced 16-byte loads and writes them
// into LDS tiles of kAttnPitch bytes per row: fp16 rows as they are (8 loads of K and of V per lane; lane = (row % 4, 16-byte
// segment)), fp32 rows split hi + lo on the way (16 loads each; lane = (row % 2, segment of 4 floats)).
template <typename T> struct AttnStage;
template <> struct AttnStage<f16_t> {
    static constexpr int PL = 1, NLOAD = 8;
    template <bool STREAM>
    static __device__ __forceinline__ void load(const f16_t* base, int r0, int j1, int lane, u32x4 (&reg)[NLOAD]) {
        const int lrow = lane >> 4, lseg = lane & 15;
#pragma unroll
        for (int q = 0; q < NLOAD; ++q) {
            int row = r0 + 4 * q + lrow;
            row = row < j1 ? row : j1 - 1;
            const f16_t* p = base + (size_t)row * 128 + 8 * lseg;
            reg[q] = STREAM ? load_stream16(p) : *reinterpret_cast<const u32x4*>(p);
        }
    }
    // rows [16 t, 16 t + 16) of the 32 loaded rows -> tile rows 0..15 (n_tiles = 1), or all 32 rows (n_tiles = 2, t = 0)
    static __device__ __forceinline__ void put(char (*buf)[16 * kAttnPitch], const u32x4 (&reg)[NLOAD], int t, int lane) {
        const int lrow = lane >> 4, lseg = lane & 15;
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<u32x4*>(buf[0] + (4 * q + lrow) * kAttnPitch + lseg * 16) = reg[4 * t + q];
    }
    static __device__ __forceinline__ void put32(char (*buf)[32 * kAttnPitch], const u32x4 (&reg)[NLOAD], int lane) {
        const int lrow = lane >> 4, lseg = lane & 15;
#pragma unroll
        for (int q = 0; q < 8; ++q) *reinterpret_cast<u32x4*>(buf[0] + (4 * q + lrow) * kAttnPitch + lseg * 16) = reg[q];
    }
};
template <> struct AttnStage<float> {
    static constexpr int PL = 2, NLOAD = 16;
    template <bool STREAM>
    static __device__ __forceinline__ void load(const float* base, int r0, int j1, int lane, u32x4 (&reg)[NLOAD]) {
        const int lrow = lane >> 5, lseg = lane & 31;
#pragma unroll
        for (int q = 0; q < NLOAD; ++q) {
            int row = r0 + 2 * q + lrow;
            row = row < j1 ? row : j1 - 1;
            const float* p = base + (size_t)row * 128 + 4 * lseg;
            reg[q] = STREAM ? load_stream16(p) : *reinterpret_cast<const u32x4*>(p);
        }
    }
    static __device__ __forceinline__ void split(const u32x4& v, uint2& hi, uint2& lo) {
        typedef _Float16 half4 __attribute__((ext_vector_type(4)));
        half4 h, l;
        const float f[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[e] = (f16_t)fminf(fmaxf(f[e], -65504.f), 65504.f);
            l[e] = (f16_t)(f[e] - (float)h[e]);
        }
        hi = __builtin_bit_cast(uint2, h);
        lo = __builtin_bit_cast(uint2, l);
    }
    static __device__ __forceinline__ void put(char (*buf)[16 * kAttnPitch], const u32x4 (&reg)[NLOAD], int t, int lane) {
        const int lrow = lane >> 5, lseg = lane & 31;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint2 hi, lo;
            split(reg[8 * t + q], hi, lo);
            *reinterpret_cast<uint2*>(buf[0] + (2 * q + lrow) * kAttnPitch + lseg * 8) = hi;
            *reinterpret_cast<uint2*>(buf[1] + (2 * q + lrow) * kAttnPitch + lseg * 8) = lo;
        }
    }
    static __device__ __forceinline__ void put32(char (*buf)[32 * kAttnPitch], const u32x4 (&reg)[NLOAD], int lane) {
        const int lrow = lane >> 5, lseg = lane & 31;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            uint2 hi, lo;
            split(reg[q], hi, lo);
            *reinterpret_cast<uint2*>(buf[0] + (2 * q + lrow) * kAttnPitch + lseg * 8) = hi;
            *reinterpret_cast<uint2*>(buf[1] + (2 * q + lrow) * kAttnPitch + lseg * 8) = lo;
        }
    }
};

template <typename T, bool ROPE, int NW, int G>
__device__ __forceinline__ void attn_split_mfma(const AttnArgs& a, int split, int h0, int c, AttnMfmaShared<NW, G, AttnStage<T>::PL>& sh) {
    constexpr int HD = 128;
    constexpr int PL = AttnStage<T>::PL;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int seq = a.cm.seq(c);
    const int row0 = a.row0 ? a.row0[seq] : 0;         // left-padded batch: rows are counted from the sequence's first row
    const int ctx = a.cm.pos(c) + 1 - row0;
    const int j0 = split * a.split_len;
    const int j1 = min(j0 + a.split_len, ctx);
    if (j0 >= j1) return;
    const bool has_new = ROPE && j1 == ctx;            // the newest row is patched into the staged tiles, not read from the cache
    const int n_live = (ctx + a.split_len - 1) / a.split_len;
    const int kvh = h0 / (a.H / a.H_kv);
    const size_t head_off = (((size_t)seq * a.H_kv + kvh) * a.max_seq + row0) * HD;
    const T* Kb = static_cast<const T*>(a.k_cache) + head_off;
    const T* Vb = static_cast<const T*>(a.v_cache) + head_off;
    const float scale = 1.4426950408889634f / sqrtf((float)HD);      // scores in log2 units

    // ---- q as the B operand: lane (i, g) holds q[h0 + i][32 kk + 8 g .. + 8], kk = 0..3, scaled, hi + lo ----
    attn_half8 qhi[4], qlo[4];
    {
        float qf[4][8];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[kk][e] = 0.f;
        if (i < G) {
            const float* qp = a.q + (size_t)c * a.q_stride + (size_t)(h0 + i) * HD + 8 * g;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const float4 t0 = *reinterpret_cast<const float4*>(qp + 32 * kk), t1 = *reinterpret_cast<const float4*>(qp + 32 * kk + 4);
                qf[kk][0] = t0.x; qf[kk][1] = t0.y; qf[kk][2] = t0.z; qf[kk][3] = t0.w;
                qf[kk][4] = t1.x; qf[kk][5] = t1.y; qf[kk][6] = t1.z; qf[kk][7] = t1.w;
            }
            if (ROPE) {                                // dims d and d + 64 are the same (g, e) of fragments kk and kk + 2
                const float2* cs = a.rope_cs + (size_t)c * (HD / 2) + 8 * g;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float4 t = *reinterpret_cast<const float4*>(cs + 32 * kk + e);
                        const float x0 = qf[kk][e], x1 = qf[kk + 2][e], z0 = qf[kk][e + 1], z1 = qf[kk + 2][e + 1];
                        qf[kk][e] = x0 * t.x - x1 * t.y;         qf[kk + 2][e] = x0 * t.y + x1 * t.x;
                        qf[kk][e + 1] = z0 * t.z - z1 * t.w;     qf[kk + 2][e + 1] = z0 * t.w + z1 * t.z;
                    }
            }
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = qf[kk][e] * scale;
                const f16_t h = (f16_t)v;
                qhi[kk][e] = h;
                qlo[kk][e] = (f16_t)(v - (float)h);
            }
    }

    // ---- the newest row in the layout of the staged tiles: lane (.., seg = lane % 16) holds dims 8 seg .. + 8 ----
    attn_half8 nk[PL], nv[PL];
    if (has_new) {
        const int seg = lane & 15;
        const bool upper = seg >= 8;
        const float* kp = a.q + (size_t)c * a.q_stride + (size_t)(a.H + kvh) * HD + 8 * seg;
        const float* pp = kp + (upper ? -(HD / 2) : HD / 2);
        const float* vp = kp + (size_t)a.H_kv * HD;
        const float2* cs = a.rope_cs + (size_t)c * (HD / 2) + 8 * (seg & 7);
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float2 own = *reinterpret_cast<const float2*>(kp + e), par = *reinterpret_cast<const float2*>(pp + e);
            const float4 t = *reinterpret_cast<const float4*>(cs + e);
            const float y0 = upper ? par.x * t.y + own.x * t.x : own.x * t.x - par.x * t.y;
            const float y1 = upper ? par.y * t.w + own.y * t.z : own.y * t.z - par.y * t.w;
            const float2 vv = *reinterpret_cast<const float2*>(vp + e);
            const float val[4] = {y0, y1, vv.x, vv.y};
            f16_t h[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) h[u] = (f16_t)fminf(fmaxf(val[u], -65504.f), 65504.f);
            nk[0][e] = h[0]; nk[0][e + 1] = h[1]; nv[0][e] = h[2]; nv[0][e + 1] = h[3];
            if (PL == 2) {                             // an fp32 cache keeps the row as it is: staged as hi + lo
                nk[PL - 1][e] = (f16_t)(y0 - (float)h[0]);   nk[PL - 1][e + 1] = (f16_t)(y1 - (float)h[1]);
                nv[PL - 1][e] = (f16_t)(vv.x - (float)h[2]); nv[PL - 1][e + 1] = (f16_t)(vv.y - (float)h[3]);
                if (wave == 0 && lane < 16) {
                    float* kd = reinterpret_cast<float*>(const_cast<T*>(Kb)) + (size_t)(ctx - 1) * HD + 8 * seg + e;
                    float* vd = reinterpret_cast<float*>(const_cast<T*>(Vb)) + (size_t)(ctx - 1) * HD + 8 * seg + e;
                    *reinterpret_cast<float2*>(kd) = make_float2(y0, y1);
                    *reinterpret_cast<float2*>(vd) = vv;
                }
            }
        }
        if (PL == 1 && wave == 0 && lane < 16) {       // one copy of the row goes to the cache (the caches are this launch's to extend)
            *reinterpret_cast<attn_half8*>(reinterpret_cast<f16_t*>(const_cast<T*>(Kb)) + (size_t)(ctx - 1) * HD + 8 * seg) = nk[0];
            *reinterpret_cast<attn_half8*>(reinterpret_cast<f16_t*>(const_cast<T*>(Vb)) + (size_t)(ctx - 1) * HD + 8 * seg) = nv[0];
        }
    }

    // ---- running state: score layout (lane = head i; the four g lanes of a head agree on m) and output layout ----
    float m = -INFINITY, lsum = 0.f;
    attn_f32x4 acc[8];                                 // [column tile nt]: lane (i, g) holds column 16 nt + i, heads 4g..4g+3
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) acc[nt] = attn_f32x4{0.f, 0.f, 0.f, 0.f};
    char (*kbuf)[16 * kAttnPitch] = sh.stage.k[wave];
    char (*vbuf)[32 * kAttnPitch] = sh.stage.v[wave];
    float* keepbuf = sh.stage.keep[wave];
    const int lseg = lane & 15;

    for (int r0 = j0 + wave * 32; r0 < j1; r0 += NW * 32) {
        u32x4 kreg[AttnStage<T>::NLOAD], vreg[AttnStage<T>::NLOAD];
        AttnStage<T>::template load<true>(Kb, r0, j1, lane, kreg);      // each row is read once per step: streaming loads
        AttnStage<T>::template load<true>(Vb, r0, j1, lane, vreg);
        // ---- scores^T of the two K tiles ----
        attn_f32x4 S[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            AttnStage<T>::put(kbuf, kreg, t, lane);
            if (has_new && ctx - 1 >= r0 + 16 * t && ctx - 1 < r0 + 16 * t + 16 && lane < 16) {
#pragma unroll
                for (int pl = 0; pl < PL; ++pl)
                    *reinterpret_cast<attn_half8*>(kbuf[pl] + (ctx - 1 - r0 - 16 * t) * kAttnPitch + lseg * 16) = nk[pl];
            }
            __builtin_amdgcn_wave_barrier();
            S[t] = attn_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const attn_half8 af = *reinterpret_cast<const attn_half8*>(kbuf[0] + i * kAttnPitch + kk * 64 + g * 16);
                S[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, qhi[kk], S[t], 0, 0, 0);
                S[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, qlo[kk], S[t], 0, 0, 0);
                if (PL == 2) {
                    const attn_half8 al = *reinterpret_cast<const attn_half8*>(kbuf[PL - 1] + i * kAttnPitch + kk * 64 + g * 16);
                    S[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, qhi[kk], S[t], 0, 0, 0);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        // ---- online softmax of head i over this lane's 8 rows and the other three lanes of the head ----
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (r0 + 16 * t + 4 * g + e >= j1) S[t][e] = -INFINITY;
                mx = fmaxf(mx, S[t][e]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));        // finite: row r0 is valid
        const float m_new = fmaxf(m, mx);
        const float keep = exp2f(m - m_new);           // exp2(-inf) = 0 the first time
        attn_half8 phi, plo;
        float ps = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p = exp2f(S[t][e] - m_new);
                ps += p;
                const f16_t h = (f16_t)p;
                phi[4 * t + e] = h;
                plo[4 * t + e] = (f16_t)(p - (float)h);
            }
        lsum = lsum * keep + ps;
        m = m_new;
        // ---- the heads' rescale factors, from lane = head to lane (column, heads 4g..4g+3) ----
        if (g == 0) keepbuf[i] = keep;
        // ---- V tile ----
        AttnStage<T>::put32(vbuf, vreg, lane);
        if (has_new && ctx - 1 >= r0 && ctx - 1 < r0 + 32 && lane < 16) {
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
                *reinterpret_cast<attn_half8*>(vbuf[pl] + (ctx - 1 - r0) * kAttnPitch + lseg * 16) = nv[pl];
        }
        __builtin_amdgcn_wave_barrier();
        const float4 kf = *reinterpret_cast<const float4*>(keepbuf + 4 * g);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            acc[nt][0] *= kf.x; acc[nt][1] *= kf.y; acc[nt][2] *= kf.z; acc[nt][3] *= kf.w;
            const attn_half8 vb = attn_v_fragment(vbuf[0], nt, lane);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(phi, vb, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(plo, vb, acc[nt], 0, 0, 0);
            if (PL == 2) {
                const attn_half8 vl = attn_v_fragment(vbuf[PL - 1], nt, lane);
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(phi, vl, acc[nt], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();               // the tiles are free for the next 32 rows
    }

    // ---- waves -> LDS (the staging tiles give way to the merge area), then the common second half ----
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    __syncthreads();
#pragma unroll
    for (int nt = 0; nt < 8; ++nt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (4 * g + e < G) sh.merge.o[4 * g + e][wave][16 * nt + i] = acc[nt][e];
    if (g == 0 && i < G) { sh.merge.m[i][wave] = m; sh.merge.l[i][wave] = lsum; }
    __syncthreads();
    attn_merge_publish<128, false, NW, G>(a, split, h0, c, n_live, sh.merge);
}

// ---------------- prompt chunks: a tile of consecutive queries on the matrix cores ----------------
// A prompt chunk holds consecutive positions of ONE sequence.  The kernel above, given a column at a time, would
// read the whole context once per query; here the 16 entries of the matrix dimension are QT = 16 / GH consecutive
// queries (columns c0 .. c0 + QT - 1) times the GH query heads of one KV head, so a cache row is read once per QT
// queries.  Entry e = query e / GH, head h0 + e % GH; its context ends at its own position (causal mask per
// entry).  The K/V rows of the chunk are already in the cache (rope_append_kernel ran before), q is rotated.
template <typename T, int NW, int GH>
__device__ __forceinline__ void attn_qtile_mfma(const AttnArgs& a, int split, int h0, int c0, AttnMfmaShared<NW, 16, AttnStage<T>::PL>& sh) {
    constexpr int HD = 128;
    constexpr int PL = AttnStage<T>::PL;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, g = lane >> 4;
    const int c_last = min(c0 + 16 / GH, a.ncols) - 1;               // last column of the tile that exists
    const int seq = a.cm.seq(c0);
    const int row0 = a.row0 ? a.row0[seq] : 0;         // left-padded batch: rows are counted from the sequence's first row
    const int ctx_max = a.cm.pos(c_last) + 1 - row0;
    const int j0 = split * a.split_len;
    const int j1 = min(j0 + a.split_len, ctx_max);
    if (j0 >= j1) return;
    const int n_live = (ctx_max + a.split_len - 1) / a.split_len;
    const int kvh = h0 / (a.H / a.H_kv);
    const size_t head_off = (((size_t)seq * a.H_kv + kvh) * a.max_seq + row0) * HD;
    const T* Kb = static_cast<const T*>(a.k_cache) + head_off;
    const T* Vb = static_cast<const T*>(a.v_cache) + head_off;
    const float scale = 1.4426950408889634f / sqrtf((float)HD);
    const int ci = c0 + i / GH;                                      // this lane's entry: column, head, end of context
    const bool live = ci < a.ncols;
    const int ctx_i = live ? a.cm.pos(ci) + 1 - row0 : 0;

    attn_half8 qhi[4], qlo[4];
    {
        const float* qp = a.q + (size_t)(live ? ci : c0) * a.q_stride + (size_t)(h0 + i % GH) * HD + 8 * g;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const float4 t0 = *reinterpret_cast<const float4*>(qp + 32 * kk), t1 = *reinterpret_cast<const float4*>(qp + 32 * kk + 4);
            const float qf[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = live ? qf[e] * scale : 0.f;
                const f16_t h = (f16_t)v;
                qhi[kk][e] = h;
                qlo[kk][e] = (f16_t)(v - (float)h);
            }
        }
    }

    float m = -INFINITY, lsum = 0.f;
    attn_f32x4 acc[8];
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) acc[nt] = attn_f32x4{0.f, 0.f, 0.f, 0.f};
    char (*kbuf)[16 * kAttnPitch] = sh.stage.k[wave];
    char (*vbuf)[32 * kAttnPitch] = sh.stage.v[wave];
    float* keepbuf = sh.stage.keep[wave];

    for (int r0 = j0 + wave * 32; r0 < j1; r0 += NW * 32) {
        u32x4 kreg[AttnStage<T>::NLOAD], vreg[AttnStage<T>::NLOAD];
        AttnStage<T>::template load<false>(Kb, r0, j1, lane, kreg);     // re-read by the next tiles: cached
        AttnStage<T>::template load<false>(Vb, r0, j1, lane, vreg);
        attn_f32x4 S[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            AttnStage<T>::put(kbuf, kreg, t, lane);
            __builtin_amdgcn_wave_barrier();
            S[t] = attn_f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const attn_half8 af = *reinterpret_cast<const attn_half8*>(kbuf[0] + i * kAttnPitch + kk * 64 + g * 16);
                S[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, qhi[kk], S[t], 0, 0, 0);
                S[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af, qlo[kk], S[t], 0, 0, 0);
                if (PL == 2) {
                    const attn_half8 al = *reinterpret_cast<const attn_half8*>(kbuf[PL - 1] + i * kAttnPitch + kk * 64 + g * 16);
                    S[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, qhi[kk], S[t], 0, 0, 0);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = r0 + 16 * t + 4 * g + e;
                if (row >= j1 || row >= ctx_i) S[t][e] = -INFINITY;  // past the split, or after this entry's own position
                mx = fmaxf(mx, S[t][e]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const bool any = m_new > -INFINITY;                           // an entry may have no row yet (its context ends earlier)
        const float keep = any ? exp2f(m - m_new) : 1.f;
        attn_half8 phi, plo;
        float ps = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p = any ? exp2f(S[t][e] - m_new) : 0.f;
                ps += p;
                const f16_t h = (f16_t)p;
                phi[4 * t + e] = h;
                plo[4 * t + e] = (f16_t)(p - (float)h);
            }
        lsum = lsum * keep + ps;
        m = m_new;
        if (g == 0) keepbuf[i] = keep;
        AttnStage<T>::put32(vbuf, vreg, lane);
        __builtin_amdgcn_wave_barrier();
        const float4 kf = *reinterpret_cast<const float4*>(keepbuf + 4 * g);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            acc[nt][0] *= kf.x; acc[nt][1] *= kf.y; acc[nt][2] *= kf.z; acc[nt][3] *= kf.w;
            const attn_half8 vb = attn_v_fragment(vbuf[0], nt, lane);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(phi, vb, acc[nt], 0, 0, 0);
            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(plo, vb, acc[nt], 0, 0, 0);
            if (PL == 2) {
                const attn_half8 vl = attn_v_fragment(vbuf[PL - 1], nt, lane);
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(phi, vl, acc[nt], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }

    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);
    __syncthreads();
#pragma unroll
    for (int nt = 0; nt < 8; ++nt)
#pragma unroll
        for (int e = 0; e < 4; ++e) sh.merge.o[4 * g + e][wave][16 * nt + i] = acc[nt][e];
    if (g == 0) { sh.merge.m[i][wave] = m; sh.merge.l[i][wave] = lsum; }
    __syncthreads();
    attn_merge_publish<128, false, NW, 16, GH>(a, split, h0, c0, n_live, sh.merge);
}

}  // namespace d3
