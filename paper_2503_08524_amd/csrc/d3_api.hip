// C ABI of the D^3 decode path: context, argument checks, and the per-step orchestration
// that launches only the blocks the schedule keeps (Section 3.4).  All device memory is the
// caller's; this file owns host state only.
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/d3.h"
#include "d3_common.h"
#include "d3_error.h"

using namespace d3;

namespace {

constexpr int kMaxPlanSteps = 4096;
constexpr size_t kAlign = 256;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Layout {          // byte offsets into the workspace
    size_t x, qkv, attn_o, act, part_o, part_ml, tickets, logits, s_hi, s_lo, f_hi, f_lo, inv_freq, rope_cs, n_hi, n_lo, ssq, h_skip, gemm_part, gemm_tickets, row0, total;
};

// The vector-ALU GEMV stages one column of its input in LDS.
bool alu_fits(const d3_model_desc& d) {
    const int widest = d.d_model > d.d_ffn ? d.d_model : d.d_ffn;
    return gemv_alu_max_cols(widest, d.weight_dtype) >= 1 && gemv_alu_max_cols(d.n_heads * d.head_dim, d.weight_dtype) >= 1;
}
// The matrix-core path takes bf16 weights, K in steps of 32 and rows in tiles of 16.
bool mfma_fits(const d3_model_desc& d) {
    const int qdim = d.n_heads * d.head_dim;
    return d.weight_dtype == D3_BF16 && d.d_model % 32 == 0 && d.d_ffn % 32 == 0 && qdim % 32 == 0 && d.vocab % 16 == 0;
}

int check_desc(const d3_model_desc* d) {
    if (!d) return fail(D3_EINVAL, "model desc is NULL");
    if (d->n_layers < 1 || d->d_model < 1 || d->n_heads < 1 || d->n_kv_heads < 1 || d->d_ffn < 1 || d->vocab < 2)
        return fail(D3_ESHAPE, "model dimensions must be positive");
    if (d->head_dim != 64 && d->head_dim != 128) return fail(D3_ESHAPE, "head_dim must be 64 or 128 (got %d)", d->head_dim);
    if (d->n_heads % d->n_kv_heads != 0)
        return fail(D3_ESHAPE, "n_heads (%d) must be a multiple of n_kv_heads (%d)", d->n_heads, d->n_kv_heads);
    if (d->d_model % 8 != 0 || d->d_ffn % 8 != 0) return fail(D3_ESHAPE, "d_model and d_ffn must be multiples of 8");
    if (d->vocab % 2 != 0) return fail(D3_ESHAPE, "vocab must be even (got %d)", d->vocab);
    if (d->max_batch < 1 || d->max_batch > kMaxCols) return fail(D3_ESHAPE, "max_batch must be in [1, %d] (got %d)", kMaxCols, d->max_batch);
    if (d->max_seq < 1 || d->max_seq > kMaxSplits * 8192) return fail(D3_ESHAPE, "max_seq must be in [1, %d]", kMaxSplits * 8192);
    if (d->weight_dtype != D3_F32 && d->weight_dtype != D3_BF16) return fail(D3_EINVAL, "weight_dtype must be D3_F32 or D3_BF16");
    if (d->kv_dtype == D3_BF16)
        return fail(D3_EINVAL, "kv_dtype D3_BF16 is not offered: a cache with an 8-bit mantissa puts the hidden state 3.7e-3 (relative) off per "
                               "block at real widths, outside the logit tolerance after two blocks; use D3_F16 (same bytes) or D3_F32");
    if (d->kv_dtype != D3_F32 && d->kv_dtype != D3_F16) return fail(D3_EINVAL, "kv_dtype must be D3_F32 or D3_F16");
    if (!(d->rms_eps >= 0.f) || !(d->rope_base > 1.f)) return fail(D3_EINVAL, "rms_eps must be >= 0 and rope_base > 1");
    if (!alu_fits(*d) && !mfma_fits(*d))
        return fail(D3_ESHAPE, "d_model / d_ffn fit neither the LDS-staged GEMV nor the matrix-core path");
    return D3_OK;
}

// C columns of fp32 activations, CS columns of bf16 hi/lo splits (the matrix-core projections read whole column tiles:
// at least 32 of them must exist), the K-slice partials of the panel kernel only when a pass can have more than 16 columns.
Layout make_layout(const d3_model_desc& d, size_t C, size_t CS, bool with_gemm_part) {
    const size_t qdim = (size_t)d.n_heads * d.head_dim;
    const size_t qkv_dim = (size_t)(d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
    const size_t s_dim = qdim > (size_t)d.d_model ? qdim : (size_t)d.d_model;
    Layout l{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
    l.x = take(C * d.d_model * 4);
    l.qkv = take(C * qkv_dim * 4);
    l.attn_o = take(C * qdim * 4);
    l.act = take(C * (size_t)d.d_ffn * 4);
    const size_t PC = C < (size_t)kMaxCols ? C : (size_t)kMaxCols;   // a pass has at most kMaxCols * kMaxSplits (column, split) pairs
    l.part_o = take(PC * d.n_heads * kMaxSplits * (size_t)d.head_dim * 4);
    l.part_ml = take(PC * d.n_heads * kMaxSplits * 2 * 4);
    l.tickets = take(C * d.n_heads * 4);
    l.logits = take(PC * (size_t)d.vocab * 4);                        // one row per sequence
    l.s_hi = take(CS * s_dim * 2);
    l.s_lo = take(CS * s_dim * 2);
    l.f_hi = take(CS * (size_t)d.d_ffn * 2);
    l.f_lo = take(CS * (size_t)d.d_ffn * 2);
    l.inv_freq = take((size_t)d.head_dim / 2 * 8);
    l.rope_cs = take(C * (size_t)d.head_dim / 2 * 8);
    l.n_hi = take(CS * d.d_model * 2);
    l.n_lo = take(CS * d.d_model * 2);
    l.ssq = take(C * kSsqStride * 4);
    l.h_skip = take(PC * d.d_model * 4);                              // decode passes only
    l.gemm_part = take(with_gemm_part ? (C > 128 ? kPromptPartBytes : kGemmPartBytes) : 0);   // passes of more than 128 columns are prompt chunks
    l.gemm_tickets = take((size_t)kGemmPartTickets * 4);
    l.row0 = take(kMaxCols * 4);
    l.total = o;
    return l;
}
// Columns of a prompt chunk: a whole sequence if it fits kPassCols (one pass over the weights per sequence, and enough
// column blocks for the 4096-row projections to fill the chip), never more than the cache can hold.
int pass_cols(const d3_model_desc& d) {
    const int need = (d.max_seq + 127) / 128 * 128;
    return need < kPassCols ? need : kPassCols;
}
// The caller's workspace serves prompt chunks of up to pass_cols() columns.
Layout make_layout(const d3_model_desc& d) { return make_layout(d, pass_cols(d), pass_cols(d), true); }

}  // namespace

namespace {
int env_int(const char* name, long lo, long hi, long dflt) {
    const char* e = getenv(name);
    if (!e) return (int)dflt;
    const long v = atol(e);
    return (int)(v >= lo && v <= hi ? v : dflt);
}
}  // namespace

namespace d3 {
Tuning tuning_from_env() {
    Tuning t;
    t.gemv_wgs_per_cu = env_int("D3_GEMV_WGS_PER_CU", 1, 8, 3);
    t.mfma_rt = env_int("D3_MFMA_RT", 1, 4, 0);
    t.mfma_waves = env_int("D3_MFMA_WAVES", 1, 8, 0);
    t.mfma_wide = env_int("D3_MFMA_WIDE", 0, 1, 1) != 0;
    t.wide_rt = env_int("D3_WIDE_RT", 1, 2, 0);
    t.wide_ks = env_int("D3_WIDE_KS", 1, 64, 0);
    t.wide_split_mb = (size_t)env_int("D3_WIDE_SPLIT_MB", 0, 1 << 20, 300);
    t.attn_mfma = env_int("D3_ATTN_MFMA", 0, 1, 1) != 0;
    t.attn_min_split = env_int("D3_ATTN_MIN_SPLIT", 64, 65536, 128) / 64 * 64;
    const int pc = env_int("D3_PREFILL_COLS", 64, kPassCols, 0);
    t.prefill_cols = pc % 64 == 0 ? pc : 0;
    t.prompt_ks = env_int("D3_PROMPT_KS", 1, 4, 0);
    return t;
}
}  // namespace d3

// d3_decode_step_static: the step's intermediates live here instead of the context's workspace.  One array per GPU,
// held until the process ends; calls that overlap on one GPU share it (and race).
constexpr size_t kStaticScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up by d3_create on that GPU
}  // namespace

struct d3_ctx {
    d3_model_desc desc;
    std::vector<d3_layer_weights> layers;
    const void *tok_emb, *final_norm, *lm_head;
    char *k_cache, *v_cache, *ws;
    Layout lay;
    int n_cu;
    int dev;                      // HIP device the context was made on
    std::vector<double> inv_freq; // rotary frequencies base^(-2j/hd) (host copy of the workspace's table)
    Tuning tn;                    // launch-shape overrides, read from the environment once by d3_create
    bool prefill_by_seq;          // prompt pass one sequence at a time (D3_PREFILL_BY_SEQ, default on)
    int attn_wgs_per_cu;          // attention workgroups per CU that the context splits aim for (D3_ATTN_WGS_PER_CU; default 2, 1 for grouped-query models)
    bool mfma_ok, alu_ok;         // which projection paths the shapes fit
    // plan
    bool has_plan;
    int n_steps;
    std::vector<int32_t> keep, drop_begin, layer_ids;
    // request state
    bool prefilled;
    int B, n_ctx, last_step;
    std::vector<int32_t> row_drop_begin, row_n_drop;   // per cache row: what the step that wrote it dropped
    bool ragged;                  // left-padded batch: sequence b's rows begin at row0[b] (device copy in the workspace)
    std::vector<int32_t> row0;
    int fill_mode;                // D3_FILL_RECOMPUTE: decode steps keep the residual that enters their drop window
    int skip_row;                 // cache row whose residual h_skip holds (-1: none)

    // per-launch timing of one kernel class
    int prof_class;
    std::vector<hipEvent_t> prof_events;   // pairs (start, stop), created on first use
    size_t prof_used;                      // events recorded so far

    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
    size_t kv_layer_bytes() const {
        return (size_t)desc.max_batch * desc.n_kv_heads * desc.max_seq * desc.head_dim * kv_elem_bytes(desc.kv_dtype);
    }
};

#define D3_HIP(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (hipError_t)(expr);                                                       \
        if (e_ != hipSuccess) return fail(D3_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

extern "C" const char* d3_last_error(void) { return error_buffer(); }

extern "C" size_t d3_workspace_size(const d3_model_desc* desc) {
    if (check_desc(desc) != D3_OK) return 0;
    return make_layout(*desc).total;
}

extern "C" int d3_create(d3_ctx** out, const d3_model_desc* desc, const d3_weights* w, void* k_cache, void* v_cache,
                         void* workspace, size_t workspace_bytes) {
    if (!out) return fail(D3_EINVAL, "d3_create: out is NULL");
    *out = nullptr;
    int rc = check_desc(desc);
    if (rc != D3_OK) return rc;
    if (!w || !w->tok_emb || !w->layers || !w->final_norm || !w->lm_head) return fail(D3_EINVAL, "d3_create: weights has a NULL field");
    for (int l = 0; l < desc->n_layers; ++l) {
        const d3_layer_weights& lw = w->layers[l];
        if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.mlp_norm || !lw.w_gate || !lw.w_up || !lw.w_down)
            return fail(D3_EINVAL, "d3_create: block %d has a NULL weight pointer", l);
    }
    if (!k_cache || !v_cache || !workspace) return fail(D3_EINVAL, "d3_create: cache or workspace is NULL");
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return fail(D3_EINVAL, "d3_create: workspace must be %zu-byte aligned", kAlign);
    const Layout lay = make_layout(*desc);
    if (workspace_bytes < lay.total) return fail(D3_EINVAL, "d3_create: workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);

    int dev = 0;
    hipDeviceProp_t prop;
    D3_HIP(hipGetDevice(&dev));
    D3_HIP(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return fail(D3_EDEVICE, "d3_create: built for gfx950, device is %s", prop.gcnArchName);

    if (dev < 0 || dev >= kMaxDevices) return fail(D3_EDEVICE, "d3_create: device index %d is outside [0, %d)", dev, kMaxDevices);
    if (!g_scratch_ptr[dev].load(std::memory_order_acquire)) {   // this GPU's copy of the static scratch array (the device is current)
        void* p = nullptr;
        D3_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }

    d3_ctx* c = new (std::nothrow) d3_ctx();
    if (!c) return fail(D3_EINVAL, "d3_create: out of host memory");
    c->desc = *desc;
    c->layers.assign(w->layers, w->layers + desc->n_layers);
    c->tok_emb = w->tok_emb; c->final_norm = w->final_norm; c->lm_head = w->lm_head;
    c->k_cache = static_cast<char*>(k_cache); c->v_cache = static_cast<char*>(v_cache); c->ws = static_cast<char*>(workspace);
    c->lay = lay;
    c->n_cu = prop.multiProcessorCount;
    c->dev = dev;
    c->tn = tuning_from_env();
    // grouped-query models on the MFMA attention kernel (fp16 cache, head_dim 128, 4 or 8 heads per KV head) do better with
    // one workgroup per CU (70B shape, batch 8: 24.41 against 24.55 ms a step), the others with two (13B, batch 4: 5.71 against 5.78)
    c->attn_wgs_per_cu = (desc->head_dim == 128 && desc->n_kv_heads > 0 &&
                          (desc->n_heads / desc->n_kv_heads == 4 || desc->n_heads / desc->n_kv_heads == 8)) ? 1 : 2;
    c->prefill_by_seq = env_int("D3_PREFILL_BY_SEQ", 0, 1, 1) != 0;
    c->attn_wgs_per_cu = env_int("D3_ATTN_WGS_PER_CU", 1, 16, c->attn_wgs_per_cu);
    c->mfma_ok = mfma_fits(*desc);
    c->alu_ok = alu_fits(*desc);
    c->prof_class = D3_K_NONE; c->prof_used = 0;
    c->has_plan = false; c->n_steps = 0;
    c->ragged = false; c->row0.assign(kMaxCols, 0);
    c->prefilled = false; c->B = 0; c->n_ctx = 0; c->last_step = 0;
    c->fill_mode = D3_FILL_COPY;
    c->skip_row = -1;
    c->row_drop_begin.assign(desc->max_seq, 0);
    c->row_n_drop.assign(desc->max_seq, 0);

    // rotary frequencies base^(-2j/hd), in binary64
    std::vector<double>& inv = c->inv_freq;
    inv.resize(desc->head_dim / 2);
    for (int j = 0; j < desc->head_dim / 2; ++j) inv[j] = std::pow((double)desc->rope_base, -2.0 * j / desc->head_dim);
    hipError_t e = hipMemcpy(c->at<double>(lay.inv_freq), inv.data(), inv.size() * sizeof(double), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(c->at<int>(lay.tickets), 0, (size_t)pass_cols(*desc) * desc->n_heads * sizeof(int));   // arrival counters start at 0
    if (e == hipSuccess) e = hipMemset(c->at<int>(lay.gemm_tickets), 0, (size_t)kGemmPartTickets * sizeof(int));
    if (e != hipSuccess) { delete c; return fail(D3_EDEVICE, "d3_create: hipMemcpy/hipMemset failed: %s", hipGetErrorString(e)); }
    *out = c;
    return D3_OK;
}

extern "C" int d3_destroy(d3_ctx* ctx) {
    if (ctx)
        for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
    delete ctx;
    return D3_OK;
}

extern "C" int32_t d3_n_ctx(const d3_ctx* ctx) { return ctx ? ctx->n_ctx : 0; }

namespace {

int install_plan(d3_ctx* ctx, std::vector<int32_t>& keep, std::vector<int32_t>& drop, std::vector<int32_t>& ids) {
    ctx->n_steps = (int)keep.size();
    ctx->keep.swap(keep); ctx->drop_begin.swap(drop); ctx->layer_ids.swap(ids);
    ctx->has_plan = true;
    ctx->last_step = 0;
    return D3_OK;
}

}  // namespace

extern "C" int d3_set_plan(d3_ctx* ctx, double alpha, int32_t start_layer, int32_t min_keep, int32_t n_steps) {
    if (!ctx) return fail(D3_EINVAL, "d3_set_plan: ctx is NULL");
    if (n_steps < 1 || n_steps > kMaxPlanSteps) return fail(D3_EINVAL, "d3_set_plan: n_steps must be in [1, %d] (got %d)", kMaxPlanSteps, n_steps);
    const int L = ctx->desc.n_layers;
    std::vector<int32_t> keep(n_steps), drop(n_steps), ids((size_t)n_steps * L);
    int rc = d3_plan_depth(L, alpha, start_layer, min_keep, n_steps, keep.data(), drop.data(), ids.data());
    if (rc != D3_OK) return rc;
    return install_plan(ctx, keep, drop, ids);
}

extern "C" int d3_set_plan_table(d3_ctx* ctx, const int32_t* keep_in, const int32_t* drop_begin_in, int32_t n_steps) {
    if (!ctx) return fail(D3_EINVAL, "d3_set_plan_table: ctx is NULL");
    if (n_steps < 1 || n_steps > kMaxPlanSteps) return fail(D3_EINVAL, "d3_set_plan_table: n_steps must be in [1, %d] (got %d)", kMaxPlanSteps, n_steps);
    if (!keep_in || !drop_begin_in) return fail(D3_EINVAL, "d3_set_plan_table: keep and drop_begin must not be NULL");
    const int L = ctx->desc.n_layers;
    std::vector<int32_t> keep(keep_in, keep_in + n_steps), drop(drop_begin_in, drop_begin_in + n_steps), ids((size_t)n_steps * L);
    int rc = d3_plan_from_table(L, n_steps, keep.data(), drop.data(), ids.data());
    if (rc != D3_OK) return rc;
    return install_plan(ctx, keep, drop, ids);
}

namespace {

constexpr size_t kMaxProfEvents = 2 * 16384;

// Brackets the launches issued during its lifetime with two events when `cls` is the selected class.
struct Timed {
    d3_ctx* c; hipStream_t s; bool on;
    Timed(d3_ctx* ctx, int cls, hipStream_t stream) : c(ctx), s(stream), on(false) {
        if (c->prof_class != cls || c->prof_used + 2 > c->prof_events.size()) return;
        on = hipEventRecord(c->prof_events[c->prof_used], s) == hipSuccess;
    }
    ~Timed() {
        if (!on) return;
        (void)hipEventRecord(c->prof_events[c->prof_used + 1], s);
        c->prof_used += 2;
    }
};

struct HeadOut {       // what to do after the last block
    int first_col, n_cols;      // columns that get logits
    float* logits;              // dev [n_cols][V]
    int32_t* tok_out;           // dev [n_cols]
};

// Attention split geometry for a pass whose longest context is `ctx` rows.
void pick_splits(const d3_ctx* c, int ncols, int ctx, int target_wgs, int* split_len, int* n_splits, bool qtile = false) {
    // workgroups per split: one per (column, KV head) when the group size has a grouped kernel, else per query head;
    // a prompt chunk on the query-tile kernel: one per (tile of 16 / group queries, KV head)
    const int group = c->desc.n_heads / c->desc.n_kv_heads;
    int heads = ncols * ((group == 2 || group == 4 || group == 8) ? c->desc.n_kv_heads : c->desc.n_heads);
    if (qtile) heads = ((ncols * group + 15) / 16) * c->desc.n_kv_heads;
    int want = (target_wgs + heads - 1) / heads;
    if (want < 1) want = 1;
    if (want > kMaxSplits) want = kMaxSplits;
    // shortest split: 128 rows is what one workgroup of the vector-ALU kernel keeps in flight; shorter splits only add
    // partials to merge (batch 1, 640 rows: 10 splits of 64 rows 11.7 us a launch, 5 of 128 rows 10.2 us, 3 of 256 rows 12.4 us)
    const int min_len = c->tn.attn_min_split;
    int len = ((ctx + want - 1) / want + 63) / 64 * 64;
    if (len < min_len) len = min_len;
    int n = (ctx + len - 1) / len;
    int most = kMaxCols * kMaxSplits / ncols;           // the partials buffer holds kMaxCols * kMaxSplits (column, split) pairs
    if (most > kMaxSplits) most = kMaxSplits;
    if (most < 1) most = 1;                             // a single split writes its result directly, no partials
    if (n > most) { len = ((ctx + most - 1) / most + 63) / 64 * 64; n = (ctx + len - 1) / len; }
    *split_len = len;
    *n_splits = n;
}

// ALU path: a projection takes as many columns per launch as its input fits in LDS
int alu_projection(d3_ctx* c, GemvArgs g, int first, int count, int mode, bool norm, hipStream_t s) {
    const int per = (int)gemv_alu_max_cols(g.K, c->desc.weight_dtype);
    for (int c0 = 0; c0 < count; c0 += per) {
        GemvArgs h = g;
        h.x = g.x + (size_t)(first + c0) * g.x_stride;
        h.out = g.out + (size_t)(first + c0) * g.out_stride;
        h.ncols = count - c0 < per ? count - c0 : per;
        h.col0 = first + c0;
        int rc = launch_gemv_alu(h, c->desc.weight_dtype, mode, norm, c->n_cu * c->tn.gemv_wgs_per_cu, s);
        if (rc != 0) return rc;

    }
    return 0;
}

// One pass of `ncols` columns through the listed blocks.  hidden_dump (or NULL): dev
// [(n_ids+1)][dump_cols][d], fed from columns [dump_first, dump_first + dump_cols).
// save_before >= 0: the residual that enters the first listed block >= save_before (the one after the last, if none)
// is copied to the workspace's h_skip: it is what the blocks of the drop window would have seen.
int forward(d3_ctx* c, const int32_t* tokens, ColMap cm, int ncols, const int32_t* ids, int n_ids,
            float* hidden_dump, int dump_first, int dump_cols, const HeadOut* head, hipStream_t s, int save_before = -1,
            int dump_total = -1, int dump_dst = 0) {
    const d3_model_desc& d = c->desc;
    const int dm = d.d_model, hd = d.head_dim, qdim = d.n_heads * hd, kvdim = d.n_kv_heads * hd, qkv_dim = qdim + 2 * kvdim, F = d.d_ffn;
    float* x = c->at<float>(c->lay.x);
    float* qkv = c->at<float>(c->lay.qkv);
    float* attn_o = c->at<float>(c->lay.attn_o);
    float* act = c->at<float>(c->lay.act);
    bf16_t *s_hi = c->at<bf16_t>(c->lay.s_hi), *s_lo = c->at<bf16_t>(c->lay.s_lo);
    bf16_t *f_hi = c->at<bf16_t>(c->lay.f_hi), *f_lo = c->at<bf16_t>(c->lay.f_lo);
    const bool mfma = c->mfma_ok && (ncols >= 2 || !c->alu_ok);
    // a decode pass (every column a different sequence) leaves the rotary embedding and the cache append to the
    // attention kernel (batch 1, 7B shape: the projection's rotate-and-scatter epilogue cost it 1.5 us, the attention
    // kernel does the same for 0.5 us with whole-row stores); a prompt chunk holds several positions of one sequence
    // and needs the rows in the cache before attention starts
    const bool rope_in_attn = ncols <= cm.B;

    float2* rope_cs = c->at<float2>(c->lay.rope_cs);
    const int* row0 = c->ragged ? c->at<int>(c->lay.row0) : nullptr;
    bf16_t *n_hi = c->at<bf16_t>(c->lay.n_hi), *n_lo = c->at<bf16_t>(c->lay.n_lo);   // split of residual * next norm's gain
    float* ssq = c->at<float>(c->lay.ssq);
    int ssq_parts = 1;
    D3_HIP(launch_embed(c->tok_emb, d.weight_dtype, tokens, cm, ncols, dm, d.vocab, x, c->at<double>(c->lay.inv_freq), hd / 2, rope_cs, row0, s));
    auto dump = [&](int slot) -> int {
        if (!hidden_dump) return 0;
        // destination slot layout [dump_total columns][d]; this pass fills columns dump_dst .. dump_dst + dump_cols - 1
        return (int)hipMemcpyAsync(hidden_dump + ((size_t)slot * (dump_total < 0 ? dump_cols : dump_total) + dump_dst) * dm, x + (size_t)dump_first * dm,
                                   (size_t)dump_cols * dm * sizeof(float), hipMemcpyDeviceToDevice, s);
    };
    D3_HIP(dump(0));

    auto alu = [&](GemvArgs g, int first, int count, int mode, bool norm) -> int { return alu_projection(c, g, first, count, mode, norm, s); };

    // a prompt chunk of one sequence (consecutive positions): tiles of queries share the cache rows they read
    const int grp = d.n_heads / d.n_kv_heads;
    const bool qtile = c->prefill_by_seq && mfma && cm.B == 1 && ncols >= 2 && hd == 128 &&
                       (grp == 1 || grp == 2 || grp == 4 || grp == 8);
    int split_len, n_splits;
    pick_splits(c, ncols, cm.pos(ncols - 1) + 1, c->attn_wgs_per_cu * c->n_cu, &split_len, &n_splits, qtile);

    // Matrix-core path: RMSNorm lives inside the projections.  Whoever writes the residual also writes the split of
    // residual * (gain of the norm that reads it next) and partial sums of squares; the reading projection scales its
    // sums by 1/rms.  The norm after block e is the next executed block's, or the final one.
    auto gain_after = [&](int e) -> const float* {
        return static_cast<const float*>(e + 1 < n_ids ? c->layers[ids[e + 1]].attn_norm : c->final_norm);
    };
    if (mfma) D3_HIP(launch_gain_split(x, dm, gain_after(-1), dm, ncols, n_hi, n_lo, ssq, s));

    bool saved = save_before < 0;
    auto save_skip = [&]() -> int {
        saved = true;
        return (int)hipMemcpyAsync(c->at<float>(c->lay.h_skip), x, (size_t)ncols * dm * sizeof(float), hipMemcpyDeviceToDevice, s);
    };
    for (int e = 0; e < n_ids; ++e) {
        const int l = ids[e];
        const d3_layer_weights& w = c->layers[l];
        if (!saved && l >= save_before) D3_HIP(save_skip());
        // --- attention half: x += Wo . attention(RoPE(Wq a), cache) with a = RMSNorm(x) ---
        GemvArgs g{};
        g.part = c->at<float>(c->lay.gemm_part); g.part_tickets = c->at<int>(c->lay.gemm_tickets);
        g.K = dm; g.eps = d.rms_eps;
        g.w[0] = w.wq; g.w[1] = w.wk; g.w[2] = w.wv;
        g.rows[0] = qdim; g.rows[1] = kvdim; g.rows[2] = kvdim; g.total_rows = qkv_dim;
        g.out = qkv; g.out_stride = qkv_dim; g.ncols = ncols;
        void* k_layer = c->k_cache + (size_t)l * c->kv_layer_bytes();
        void* v_layer = c->v_cache + (size_t)l * c->kv_layer_bytes();
        if (mfma) {
            g.x_hi = n_hi; g.x_lo = n_lo; g.x_stride = dm; g.ssq_in = ssq; g.ssq_parts = ssq_parts;
            {
                Timed t(c, D3_K_QKV, s);
                D3_HIP(launch_gemm_mfma(g, MODE_STORE, c->n_cu, c->tn, s));
            }
            if (!rope_in_attn) {
                RopeArgs r{};
                r.qkv = qkv; r.k_cache = k_layer; r.v_cache = v_layer; r.rope_cs = rope_cs;
                r.cm = cm; r.ncols = ncols; r.H = d.n_heads; r.H_kv = d.n_kv_heads; r.hd = hd; r.max_seq = d.max_seq;
                D3_HIP(launch_rope_append(r, d.kv_dtype, s));
            }
        } else {
            // a prompt chunk on this path: the GEMV epilogue rotates q and k and appends the new K/V rows itself
            g.x = x; g.x_stride = dm; g.gain = static_cast<const float*>(w.attn_norm);
            g.rope_cs = rope_cs; g.k_cache = k_layer; g.v_cache = v_layer; g.cm = cm;
            g.H = d.n_heads; g.H_kv = d.n_kv_heads; g.hd = hd; g.max_seq = d.max_seq; g.kv_dtype = d.kv_dtype;
            Timed t(c, D3_K_QKV, s);
            D3_HIP(alu(g, 0, ncols, rope_in_attn ? MODE_STORE : MODE_QKV_ROPE, true));
        }
        AttnArgs at{};
        at.q = qkv; at.q_stride = qkv_dim; at.k_cache = k_layer; at.v_cache = v_layer; at.cm = cm;
        at.ncols = ncols; at.H = d.n_heads; at.H_kv = d.n_kv_heads; at.hd = hd; at.max_seq = d.max_seq;
        at.split_len = split_len; at.n_splits = n_splits;
        at.part_o = c->at<float>(c->lay.part_o); at.part_ml = c->at<float>(c->lay.part_ml); at.tickets = c->at<int>(c->lay.tickets);
        at.out = attn_o; at.out_hi = mfma ? s_hi : nullptr; at.out_lo = mfma ? s_lo : nullptr;
        at.rope_cs = rope_in_attn ? rope_cs : nullptr;
        at.qtile = qtile ? 1 : 0;
        at.row0 = row0;
        {
            Timed t(c, D3_K_ATTN, s);
            D3_HIP(launch_attention(at, d.kv_dtype, c->tn.attn_mfma, s));
        }

        GemvArgs o{};
        o.part = c->at<float>(c->lay.gemm_part); o.part_tickets = c->at<int>(c->lay.gemm_tickets);
        o.K = qdim; o.w[0] = w.wo; o.rows[0] = dm; o.total_rows = dm; o.out = x; o.out_stride = dm; o.ncols = ncols;
        {
            Timed t(c, D3_K_OPROJ, s);
            if (mfma) {
                o.x_hi = s_hi; o.x_lo = s_lo; o.x_stride = qdim;
                o.out_hi = n_hi; o.out_lo = n_lo; o.gain_next = static_cast<const float*>(w.mlp_norm); o.ssq_out = ssq;
                D3_HIP(launch_gemm_mfma(o, MODE_RESID, c->n_cu, c->tn, s, &ssq_parts));
            }
            else { o.x = attn_o; o.x_stride = qdim; D3_HIP(alu(o, 0, ncols, MODE_RESID, false)); }
        }

        // --- SwiGLU half: x += Wd (silu(Wg m) * (Wu m)) with m = RMSNorm(x) ---
        GemvArgs u{};
        u.part = c->at<float>(c->lay.gemm_part); u.part_tickets = c->at<int>(c->lay.gemm_tickets);
        u.K = dm; u.eps = d.rms_eps; u.w[0] = w.w_gate; u.w[1] = w.w_up; u.rows[0] = F; u.rows[1] = F; u.total_rows = F;
        u.out_stride = F; u.ncols = ncols;
        GemvArgs dn{};
        dn.part = c->at<float>(c->lay.gemm_part); dn.part_tickets = c->at<int>(c->lay.gemm_tickets);
        dn.K = F; dn.w[0] = w.w_down; dn.rows[0] = dm; dn.total_rows = dm; dn.out = x; dn.out_stride = dm; dn.ncols = ncols;
        if (mfma) {
            u.x_hi = n_hi; u.x_lo = n_lo; u.x_stride = dm; u.ssq_in = ssq; u.ssq_parts = ssq_parts;
            u.out = nullptr; u.out_hi = f_hi; u.out_lo = f_lo;
            { Timed t(c, D3_K_GATE_UP, s); D3_HIP(launch_gemm_mfma(u, MODE_SWIGLU, c->n_cu, c->tn, s)); }
            dn.x_hi = f_hi; dn.x_lo = f_lo; dn.x_stride = F;
            dn.out_hi = n_hi; dn.out_lo = n_lo; dn.gain_next = gain_after(e); dn.ssq_out = ssq;
            { Timed t(c, D3_K_EMPTY, s); }
            { Timed t(c, D3_K_DOWN, s); D3_HIP(launch_gemm_mfma(dn, MODE_RESID, c->n_cu, c->tn, s, &ssq_parts)); }
        } else {
            u.x = x; u.x_stride = dm; u.gain = static_cast<const float*>(w.mlp_norm); u.out = act;
            { Timed t(c, D3_K_GATE_UP, s); D3_HIP(alu(u, 0, ncols, MODE_SWIGLU, true)); }
            dn.x = act; dn.x_stride = F;
            { Timed t(c, D3_K_EMPTY, s); }
            { Timed t(c, D3_K_DOWN, s); D3_HIP(alu(dn, 0, ncols, MODE_RESID, false)); }
        }
        D3_HIP(dump(e + 1));
    }

    if (!saved) D3_HIP(save_skip());
    if (head) {
        GemvArgs g{};
        g.part = c->at<float>(c->lay.gemm_part); g.part_tickets = c->at<int>(c->lay.gemm_tickets);
        g.K = dm; g.eps = d.rms_eps; g.w[0] = c->lm_head; g.rows[0] = d.vocab; g.total_rows = d.vocab;
        g.out = head->logits; g.out_stride = d.vocab; g.ncols = head->n_cols;
        if (mfma) {
            g.x_hi = n_hi + (size_t)head->first_col * dm; g.x_lo = n_lo + (size_t)head->first_col * dm; g.x_stride = dm;
            g.ssq_in = ssq + (size_t)head->first_col * kSsqStride; g.ssq_parts = ssq_parts;
            Timed t(c, D3_K_LM_HEAD, s);
            D3_HIP(launch_gemm_mfma(g, MODE_STORE, c->n_cu, c->tn, s));
        } else {
            g.x = x + (size_t)head->first_col * dm; g.x_stride = dm; g.gain = static_cast<const float*>(c->final_norm);
            Timed t(c, D3_K_LM_HEAD, s);
            D3_HIP(alu(g, 0, head->n_cols, MODE_STORE, true));
        }
        D3_HIP(launch_argmax(head->logits, d.vocab, head->n_cols, head->tok_out, s));
    }
    return D3_OK;
}

}  // namespace

namespace {

// Prompt pass.  lengths (host, optional): a left-padded batch, sequence b holds lengths[b] tokens in columns
// [P - lengths[b], P) of its row of `tokens` and in the cache rows of the same numbers.
int prefill_impl(d3_ctx* ctx, const int32_t* tokens, int32_t B, int32_t P, int32_t pos_begin, const int32_t* lengths,
                 int32_t* next_tok, float* logits, float* hidden_dump, void* hip_stream) {
    if (!ctx || !tokens || !next_tok) return fail(D3_EINVAL, "d3_prefill: NULL argument");
    const d3_model_desc& d = ctx->desc;
    if (B < 1 || B > d.max_batch) return fail(D3_ESHAPE, "d3_prefill: B must be in [1, %d] (got %d)", d.max_batch, B);
    if (P < 1) return fail(D3_EINVAL, "d3_prefill: P must be >= 1 (got %d)", P);
    if (pos_begin != 0 && !(ctx->prefilled && pos_begin == ctx->n_ctx && B == ctx->B))
        return fail(D3_ESTATE, "d3_prefill: pos_begin must be 0 or the current row count %d with the same batch (got %d)", ctx->n_ctx, pos_begin);
    if ((int64_t)pos_begin + P > d.max_seq) return fail(D3_ERANGE, "d3_prefill: rows [%d, %d) exceed max_seq %d", pos_begin, pos_begin + P, d.max_seq);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (lengths) {
        int longest = 0;
        for (int b = 0; b < B; ++b) {
            if (lengths[b] < 1 || lengths[b] > P) return fail(D3_EINVAL, "d3_prefill_ragged: lengths[%d] = %d is outside [1, %d]", b, lengths[b], P);
            longest = lengths[b] > longest ? lengths[b] : longest;
        }
        if (longest != P) return fail(D3_EINVAL, "d3_prefill_ragged: the longest sequence has %d tokens, P is %d (pad to the longest)", longest, P);
    }
    if (pos_begin == 0) {                     // a fresh request decides whether the batch is ragged; a continuation keeps it
        bool ragged = false;
        for (int b = 0; b < B; ++b) {
            ctx->row0[b] = lengths ? P - lengths[b] : 0;
            ragged = ragged || ctx->row0[b] != 0;
        }
        ctx->ragged = ragged;
        if (ragged) D3_HIP(hipMemcpyAsync(ctx->at<int>(ctx->lay.row0), ctx->row0.data(), (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice, s));
    }

    std::vector<int32_t> all(d.n_layers);
    for (int l = 0; l < d.n_layers; ++l) all[l] = l;
    float* lg = logits ? logits : ctx->at<float>(ctx->lay.logits);
    if (ctx->prefill_by_seq || (ctx->ragged && pos_begin == 0)) {
        // one sequence at a time, 32 consecutive positions per pass: the attention of such a chunk reads every cache
        // row once per tile of queries instead of once per query
        // the matrix-core path takes 128 columns a pass (the weights are streamed once per pass); D3_PREFILL_COLS=64 halves that
        // (projections of large matrices split such a pass into two launches of 64 columns by themselves)
        const int fit = pass_cols(d);
        const int wide_cols = ctx->tn.prefill_cols && ctx->tn.prefill_cols < fit ? ctx->tn.prefill_cols : fit;
        const int chunk_cols = ctx->mfma_ok && ctx->tn.mfma_wide ? wide_cols : kMaxCols;
        for (int b = 0; b < B; ++b) {
            for (int base = pos_begin == 0 ? ctx->row0[b] : 0; base < P;) {     // padding columns are not computed
                const int ncols = P - base < chunk_cols ? P - base : chunk_cols;
                const bool last = base + ncols == P;
                ColMap cm{base, 1, P, pos_begin, b};
                HeadOut head{ncols - 1, 1, lg + (size_t)b * d.vocab, next_tok + b};
                int rc = forward(ctx, tokens, cm, ncols, all.data(), d.n_layers, last ? hidden_dump : nullptr, ncols - 1, 1,
                                 last ? &head : nullptr, s, -1, B, b);
                if (rc != D3_OK) return rc;
                base += ncols;
            }
        }
    } else {
        const int chunk = (kMaxCols / B) * B;
        const int total = B * P;
        // position-major columns in chunks that are multiples of B: the last B columns of the last
        // chunk are the last prompt position of every sequence
        for (int base = 0; base < total;) {
            const int ncols = total - base < chunk ? total - base : chunk;
            const bool last = base + ncols == total;
            ColMap cm{base, B, P, pos_begin};
            HeadOut head{ncols - B, B, lg, next_tok};
            int rc = forward(ctx, tokens, cm, ncols, all.data(), d.n_layers, last ? hidden_dump : nullptr, ncols - B, B,
                             last ? &head : nullptr, s);
            if (rc != D3_OK) return rc;
            base += ncols;
        }
    }
    for (int p = pos_begin; p < pos_begin + P; ++p) { ctx->row_drop_begin[p] = 0; ctx->row_n_drop[p] = 0; }
    ctx->prefilled = true;
    ctx->B = B;
    ctx->n_ctx = pos_begin + P;
    ctx->last_step = 0;
    return D3_OK;
}

}  // namespace

extern "C" int d3_prefill(d3_ctx* ctx, const int32_t* tokens, int32_t B, int32_t P, int32_t pos_begin, int32_t* next_tok,
                          float* logits, float* hidden_dump, void* hip_stream) {
    return prefill_impl(ctx, tokens, B, P, pos_begin, nullptr, next_tok, logits, hidden_dump, hip_stream);
}

extern "C" int d3_prefill_ragged(d3_ctx* ctx, const int32_t* tokens, const int32_t* lengths, int32_t B, int32_t P,
                                 int32_t* next_tok, float* logits, float* hidden_dump, void* hip_stream) {
    if (!lengths) return fail(D3_EINVAL, "d3_prefill_ragged: lengths is NULL");
    return prefill_impl(ctx, tokens, B, P, 0, lengths, next_tok, logits, hidden_dump, hip_stream);
}

namespace {

int decode_step_impl(d3_ctx* ctx, const int32_t* tok_in, int32_t step_i, int32_t* tok_out, float* logits, float* hidden_dump,
                     hipStream_t s, bool static_scratch) {
    if (!ctx || !tok_in || !tok_out) return fail(D3_EINVAL, "d3_decode_step: NULL argument");
    if (!ctx->has_plan) return fail(D3_ESTATE, "d3_decode_step: no plan set (call d3_set_plan)");
    if (!ctx->prefilled) return fail(D3_ESTATE, "d3_decode_step: no prompt pass yet (call d3_prefill)");
    if (step_i != ctx->last_step + 1) return fail(D3_ESTATE, "d3_decode_step: expected step %d, got %d", ctx->last_step + 1, step_i);
    if (step_i >= ctx->n_steps) return fail(D3_ERANGE, "d3_decode_step: step %d is outside the plan of %d steps", step_i, ctx->n_steps);
    if (ctx->n_ctx >= ctx->desc.max_seq) return fail(D3_ERANGE, "d3_decode_step: cache is full (%d rows)", ctx->n_ctx);
    const int L = ctx->desc.n_layers, B = ctx->B;
    const int kept = ctx->keep[step_i];
    char* const own_ws = ctx->ws;
    const Layout own_lay = ctx->lay;
    if (static_scratch) {
        // the step's buffers, laid out for max_batch columns, inside this GPU's static array; the few words of state the
        // workspace carries between calls (rotary frequencies, first rows of a ragged batch, zeroed arrival counters) are
        // written there by one small kernel first, because the array keeps whatever the last call on this GPU left
        if (ctx->fill_mode == D3_FILL_RECOMPUTE)
            return fail(D3_ESTATE, "d3_decode_step_static: the RECOMPUTE fill keeps a residual in the context's workspace; use d3_decode_step");
        const Layout sl = make_layout(ctx->desc, ctx->desc.max_batch, kMaxCols, ctx->desc.max_batch > 16);
        if (sl.total > kStaticScratchBytes)
            return fail(D3_ESHAPE, "d3_decode_step_static: a step of this model at max_batch %d needs %zu bytes of scratch, the static array holds %zu",
                        ctx->desc.max_batch, sl.total, kStaticScratchBytes);
        char* sp = static_cast<char*>(g_scratch_ptr[ctx->dev].load(std::memory_order_acquire));
        if (!sp) return fail(D3_ESTATE, "d3_decode_step_static: no static scratch on device %d", ctx->dev);
        StaticSeed seed{};
        for (size_t j = 0; j < ctx->inv_freq.size(); ++j) seed.inv_freq[j] = ctx->inv_freq[j];
        for (int b = 0; b < kMaxCols; ++b) seed.row0[b] = ctx->row0[b];
        D3_HIP(launch_static_seed(seed, reinterpret_cast<double*>(sp + sl.inv_freq), ctx->desc.head_dim / 2, reinterpret_cast<int*>(sp + sl.row0),
                                  reinterpret_cast<int*>(sp + sl.tickets), ctx->desc.max_batch * ctx->desc.n_heads,
                                  reinterpret_cast<int*>(sp + sl.gemm_tickets), kGemmPartTickets, s));
        ctx->ws = sp;
        ctx->lay = sl;
    }
    ColMap cm{0, B, 1, ctx->n_ctx};
    HeadOut head{0, B, logits ? logits : ctx->at<float>(ctx->lay.logits), tok_out};
    const bool keep_skip = ctx->fill_mode == D3_FILL_RECOMPUTE && kept < L;
    const int rc = forward(ctx, tok_in, cm, B, ctx->layer_ids.data() + (size_t)step_i * L, kept, hidden_dump, 0, B, &head, s,
                           keep_skip ? ctx->drop_begin[step_i] + (L - kept) : -1);
    ctx->ws = own_ws;
    ctx->lay = own_lay;
    ctx->skip_row = keep_skip && rc == D3_OK ? ctx->n_ctx : -1;
    if (rc != D3_OK) return rc;
    ctx->row_drop_begin[ctx->n_ctx] = ctx->drop_begin[step_i];
    ctx->row_n_drop[ctx->n_ctx] = L - kept;
    ctx->n_ctx += 1;
    ctx->last_step = step_i;
    return D3_OK;
}

}  // namespace

extern "C" int d3_decode_step(d3_ctx* ctx, const int32_t* tok_in, int32_t step_i, int32_t* tok_out, float* logits,
                              float* hidden_dump, void* hip_stream) {
    return decode_step_impl(ctx, tok_in, step_i, tok_out, logits, hidden_dump, static_cast<hipStream_t>(hip_stream), false);
}

extern "C" int d3_decode_step_static(d3_ctx* ctx, const int32_t* tok_in, int32_t step_i, int32_t* tok_out, float* logits,
                                     float* hidden_dump, void* hip_stream) {
    return decode_step_impl(ctx, tok_in, step_i, tok_out, logits, hidden_dump, static_cast<hipStream_t>(hip_stream), true);
}

extern "C" size_t d3_static_scratch_bytes(void) { return kStaticScratchBytes; }

// RECOMPUTE fill of the row the latest decode step wrote: every dropped block l gets
// K[l][p] = RoPE(W_k^l a), V[l][p] = W_v^l a with a = RMSNorm_l(h), h = the residual that entered the drop window
// (kept by that decode step).  One fused launch per dropped block at batch 1 (the QKV kernel without its q heads),
// three on the matrix-core path (gain split, projection, RoPE + append).
int fill_recompute(d3_ctx* c, int pos_begin, int pos_end, hipStream_t s) {
    if (c->fill_mode != D3_FILL_RECOMPUTE)
        return fail(D3_ESTATE, "d3_fill_missing_kv: RECOMPUTE needs d3_set_fill_mode(ctx, D3_FILL_RECOMPUTE) before the decode step");
    if (pos_end == pos_begin) return D3_OK;
    if (pos_end != pos_begin + 1 || pos_begin != c->n_ctx - 1)
        return fail(D3_ESTATE, "d3_fill_missing_kv: RECOMPUTE fills the row of the latest decode step only (row %d), got [%d, %d)",
                    c->n_ctx - 1, pos_begin, pos_end);
    const int p = pos_begin, first = c->row_drop_begin[p], n = c->row_n_drop[p];
    if (n == 0) return D3_OK;
    if (c->skip_row != p) return fail(D3_ESTATE, "d3_fill_missing_kv: no kept residual for row %d (written by the prompt pass)", p);
    const d3_model_desc& d = c->desc;
    const int dm = d.d_model, hd = d.head_dim, kvdim = d.n_kv_heads * hd, B = c->B;
    const ColMap cm{0, B, 1, p};
    const float* h = c->at<float>(c->lay.h_skip);
    float* kv = c->at<float>(c->lay.qkv);
    float2* rope_cs = c->at<float2>(c->lay.rope_cs);       // the table of that decode step: same columns, same positions
    const bool mfma = c->mfma_ok && (B >= 2 || !c->alu_ok);
    for (int l = first; l < first + n; ++l) {
        const d3_layer_weights& w = c->layers[l];
        void* k_layer = c->k_cache + (size_t)l * c->kv_layer_bytes();
        void* v_layer = c->v_cache + (size_t)l * c->kv_layer_bytes();
        GemvArgs g{};
        g.part = c->at<float>(c->lay.gemm_part); g.part_tickets = c->at<int>(c->lay.gemm_tickets);
        g.K = dm; g.eps = d.rms_eps; g.w[0] = w.wk; g.w[1] = w.wv; g.rows[0] = kvdim; g.rows[1] = kvdim; g.total_rows = 2 * kvdim;
        g.out = kv; g.out_stride = 2 * kvdim; g.ncols = B;
        if (mfma) {
            bf16_t *n_hi = c->at<bf16_t>(c->lay.n_hi), *n_lo = c->at<bf16_t>(c->lay.n_lo);
            float* ssq = c->at<float>(c->lay.ssq);
            D3_HIP(launch_gain_split(h, dm, static_cast<const float*>(w.attn_norm), dm, B, n_hi, n_lo, ssq, s));
            g.x_hi = n_hi; g.x_lo = n_lo; g.x_stride = dm; g.ssq_in = ssq; g.ssq_parts = 1;
            D3_HIP(launch_gemm_mfma(g, MODE_STORE, c->n_cu, c->tn, s));
            RopeArgs r{};
            r.qkv = kv; r.k_cache = k_layer; r.v_cache = v_layer; r.rope_cs = rope_cs;
            r.cm = cm; r.ncols = B; r.H = 0; r.H_kv = d.n_kv_heads; r.hd = hd; r.max_seq = d.max_seq;
            D3_HIP(launch_rope_append(r, d.kv_dtype, s));
        } else {
            g.x = h; g.x_stride = dm; g.gain = static_cast<const float*>(w.attn_norm);
            g.rope_cs = rope_cs; g.k_cache = k_layer; g.v_cache = v_layer; g.cm = cm;
            g.H = 0; g.H_kv = d.n_kv_heads; g.hd = hd; g.max_seq = d.max_seq; g.kv_dtype = d.kv_dtype;
            D3_HIP(alu_projection(c, g, 0, B, MODE_QKV_ROPE, true, s));
        }
    }
    return D3_OK;
}

extern "C" int d3_set_fill_mode(d3_ctx* ctx, int32_t mode) {
    if (!ctx) return fail(D3_EINVAL, "d3_set_fill_mode: ctx is NULL");
    if (mode != D3_FILL_COPY && mode != D3_FILL_RECOMPUTE) return fail(D3_EINVAL, "d3_set_fill_mode: unknown mode %d", mode);
    ctx->fill_mode = mode;
    ctx->skip_row = -1;
    return D3_OK;
}

extern "C" int d3_fill_missing_kv(d3_ctx* ctx, int32_t pos_begin, int32_t pos_end, int32_t mode, void* hip_stream) {
    if (!ctx) return fail(D3_EINVAL, "d3_fill_missing_kv: ctx is NULL");
    if (mode != D3_FILL_COPY && mode != D3_FILL_RECOMPUTE) return fail(D3_EINVAL, "d3_fill_missing_kv: unknown mode %d", mode);
    if (pos_begin < 0 || pos_end < pos_begin || pos_end > ctx->n_ctx)
        return fail(D3_ERANGE, "d3_fill_missing_kv: rows [%d, %d) are outside the %d rows written", pos_begin, pos_end, ctx->n_ctx);
    const d3_model_desc& d = ctx->desc;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (mode == D3_FILL_RECOMPUTE) return fill_recompute(ctx, pos_begin, pos_end, s);
    // consecutive rows whose steps dropped the same window share one launch
    for (int p = pos_begin; p < pos_end;) {
        int q = p + 1;
        while (q < pos_end && ctx->row_drop_begin[q] == ctx->row_drop_begin[p] && ctx->row_n_drop[q] == ctx->row_n_drop[p]) ++q;
        const int first = ctx->row_drop_begin[p], n = ctx->row_n_drop[p];
        if (n > 0) {
            FillArgs f{};
            f.k_cache = ctx->k_cache; f.v_cache = ctx->v_cache;
            f.max_batch = d.max_batch; f.H_kv = d.n_kv_heads; f.max_seq = d.max_seq; f.hd = d.head_dim;
            f.B = ctx->B; f.pos_begin = p; f.pos_end = q;
            f.drop_begin = first; f.n_drop = n;
            f.src = first > 0 ? first - 1 : (first + n < d.n_layers ? first + n : -1);
            D3_HIP(launch_fill(f, d.kv_dtype, s));
        }
        p = q;
    }
    return D3_OK;
}

extern "C" int d3_truncate(d3_ctx* ctx, int32_t n_rows) {
    if (!ctx) return fail(D3_EINVAL, "d3_truncate: ctx is NULL");
    if (!ctx->prefilled) return fail(D3_ESTATE, "d3_truncate: no prompt pass yet");
    if (n_rows < 1 || n_rows > ctx->n_ctx) return fail(D3_ERANGE, "d3_truncate: n_rows must be in [1, %d] (got %d)", ctx->n_ctx, n_rows);
    if (ctx->ragged)                           // every sequence of a left-padded batch keeps at least its first row
        for (int b = 0; b < ctx->B; ++b)
            if (n_rows <= ctx->row0[b]) return fail(D3_ERANGE, "d3_truncate: sequence %d of the ragged batch begins at row %d (got n_rows %d)", b, ctx->row0[b], n_rows);
    ctx->n_ctx = n_rows;
    ctx->last_step = 0;
    ctx->skip_row = -1;
    return D3_OK;
}

extern "C" int d3_stream_read(d3_ctx* ctx, const void* src, size_t bytes, void* hip_stream) {
    if (!ctx || !src) return fail(D3_EINVAL, "d3_stream_read: NULL argument");
    if (bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return fail(D3_EINVAL, "d3_stream_read: the buffer must be 16-byte aligned and a multiple of 16 bytes");
    // three workgroups of four waves per compute unit, like the projections; their checksums land in the attention partials
    const int n_wg = 3 * ctx->n_cu;
    D3_HIP(launch_stream_read(src, bytes, ctx->at<unsigned>(ctx->lay.part_o), n_wg, static_cast<hipStream_t>(hip_stream)));
    return D3_OK;
}

extern "C" int d3_mfma_yardstick(d3_ctx* ctx, int32_t mode, int32_t stages, void* hip_stream) {
    if (!ctx) return fail(D3_EINVAL, "d3_mfma_yardstick: ctx is NULL");
    if (mode < 0 || mode > 2 || stages < 2 || stages > (1 << 20) || stages % 2 != 0)
        return fail(D3_EINVAL, "d3_mfma_yardstick: mode must be 0, 1 or 2 and stages even, in [2, 2^20] (got %d, %d)", mode, stages);
    // one workgroup of eight waves per compute unit, like the residual projections of the prompt pass; a word per wave lands in the attention partials
    if ((size_t)ctx->n_cu * 8 * sizeof(float) > ctx->lay.part_ml - ctx->lay.part_o) return fail(D3_ESHAPE, "d3_mfma_yardstick: the workspace of this model is too small for the result words");
    D3_HIP(launch_mfma_yardstick(mode, stages, ctx->n_cu, ctx->at<float>(ctx->lay.part_o), static_cast<hipStream_t>(hip_stream)));
    return D3_OK;
}

extern "C" int d3_profile_select(d3_ctx* ctx, int32_t kernel_class) {
    if (!ctx) return fail(D3_EINVAL, "d3_profile_select: ctx is NULL");
    if (kernel_class < D3_K_NONE || kernel_class > D3_K_EMPTY) return fail(D3_EINVAL, "d3_profile_select: unknown class %d", kernel_class);
    if (kernel_class != D3_K_NONE && ctx->prof_events.empty()) {
        ctx->prof_events.reserve(kMaxProfEvents);
        for (size_t i = 0; i < kMaxProfEvents; ++i) {
            hipEvent_t e;
            D3_HIP(hipEventCreate(&e));
            ctx->prof_events.push_back(e);
        }
    }
    ctx->prof_class = kernel_class;
    ctx->prof_used = 0;
    return D3_OK;
}

extern "C" int d3_profile_read(d3_ctx* ctx, double* total_ms, int64_t* launches) {
    if (!ctx || !total_ms || !launches) return fail(D3_EINVAL, "d3_profile_read: NULL argument");
    double sum = 0.0;
    for (size_t i = 0; i + 1 < ctx->prof_used; i += 2) {
        float ms = 0.f;
        D3_HIP(hipEventSynchronize(ctx->prof_events[i + 1]));
        D3_HIP(hipEventElapsedTime(&ms, ctx->prof_events[i], ctx->prof_events[i + 1]));
        sum += ms;
    }
    *total_ms = sum;
    *launches = (int64_t)(ctx->prof_used / 2);
    ctx->prof_used = 0;
    return D3_OK;
}
