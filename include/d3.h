/* d3.h -- C ABI of the MI355X (gfx950) implementation of Position-Aware Depth
 * Decay Decoding (D^3): the autoregressive decode step of a Llama-style decoder
 * that runs only floor(L * alpha^i) of its L blocks when generating token T_i.
 *
 * Conventions
 *   - Every function returns D3_OK (0) or a negative d3_status.  Nothing throws
 *     or aborts.  d3_last_error() gives the message of the calling thread's last
 *     failure (library-owned, valid until that thread's next failing call).
 *   - "dev" pointers are HIP device pointers, "host" pointers are ordinary
 *     memory.  The library allocates NO device memory: weights, KV cache,
 *     workspace, token and logit buffers are caller-owned and must outlive the
 *     context.  Device work is enqueued on the HIP stream the caller passes
 *     (a hipStream_t cast to void*; NULL = the null stream) and is asynchronous;
 *     argument checks are synchronous.
 *   - Token time step i (Section 1, Section 3.4): T_0 is the token produced by
 *     the prompt pass, which runs all L blocks (Section 3.2); decode step i >= 1
 *     consumes T_{i-1}, writes cache row n_ctx = P + i - 1 and produces T_i with
 *     keep[i] = floor(L * alpha^i) blocks.  All sequences of a batch share i and
 *     therefore the executed blocks (Section 1, challenge (ii); Table 1).
 *   - Layouts: linear weights row-major [out][in], float32 or bf16; RMSNorm
 *     gains float32; KV cache [L][max_batch][H_kv][max_seq][head_dim] for K and
 *     for V (keys stored after the rotary embedding), float32 or fp16.
 */
#ifndef D3_H
#define D3_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    D3_OK = 0,
    D3_EINVAL = -1,  /* bad scalar argument or NULL pointer */
    D3_ESHAPE = -2,  /* model shape or batch outside what the kernels support */
    D3_ERANGE = -3,  /* position or step outside the cache / the plan */
    D3_ESTATE = -4,  /* call out of order (no plan, no prefill, wrong step) */
    D3_EDEVICE = -5  /* a HIP call failed */
} d3_status;

typedef enum { D3_F32 = 0, D3_BF16 = 1, D3_F16 = 2 } d3_dtype;
typedef enum { D3_FILL_COPY = 0, D3_FILL_RECOMPUTE = 1 } d3_fill_mode;

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_base;
    int32_t weight_dtype; /* D3_F32 or D3_BF16: every linear weight and the embedding table */
    int32_t kv_dtype;     /* the KV cache: D3_F16 (IEEE half, values clamped to +-65504) or D3_F32.  The rounding of
                           * the cache rows is what separates the result from full precision: about 4.5e-4 of the
                           * hidden state's norm per block with D3_F16, growing like sqrt(blocks run), against
                           * 5e-6 with D3_F32; models of more than about 48 blocks need D3_F32 to keep logits within
                           * 2e-2.  D3_BF16 (3.7e-3 per block) is refused. */
    int32_t max_batch, max_seq;
} d3_model_desc;

/* One decoder block (Llama-2 blocks, Section 4.1): dev pointers.
 * attn_norm/mlp_norm: float32 [d_model].  wq [n_heads*head_dim][d_model];
 * wk, wv [n_kv_heads*head_dim][d_model]; wo [d_model][n_heads*head_dim];
 * w_gate, w_up [d_ffn][d_model]; w_down [d_model][d_ffn]. */
typedef struct {
    const void *attn_norm, *wq, *wk, *wv, *wo, *mlp_norm, *w_gate, *w_up, *w_down;
} d3_layer_weights;

/* tok_emb, lm_head: dev [vocab][d_model] (weight_dtype); final_norm: dev float32 [d_model];
 * layers: HOST array of n_layers entries (copied by d3_create). */
typedef struct {
    const void *tok_emb;
    const d3_layer_weights *layers;
    const void *final_norm, *lm_head;
} d3_weights;

typedef struct d3_ctx d3_ctx;

const char *d3_last_error(void);

/* Depth schedule and layer-index table (Section 3.4: power-law decay
 * floor(L * alpha^i); Table 6: drop-layer set starting at `start`).  Pure host
 * code, needs no GPU.  For i in [0, n_steps):
 *   pow_0 = 1, pow_i = pow_{i-1} * alpha (binary64);
 *   keep[i] = max(min_keep, floor(L * pow_i));  n_i = L - keep[i];
 *   drop_begin[i] = min(start_layer, L - n_i);  dropped = [drop_begin[i], drop_begin[i] + n_i);
 *   layer_ids[i*L + j] = j-th executed block in increasing order, -1 for j >= keep[i].
 * Host arrays of n_steps (keep, drop_begin) and n_steps*L (layer_ids) int32,
 * caller-owned; any may be NULL.  D3_EINVAL unless L >= 1, 0 < alpha <= 1,
 * 0 <= start_layer < L, 0 <= min_keep <= L, n_steps >= 0. */
int d3_plan_depth(int32_t L, double alpha, int32_t start_layer, int32_t min_keep, int32_t n_steps,
                  int32_t *keep, int32_t *drop_begin, int32_t *layer_ids);

/* Linear decay between two bounds, the schedule of the batched comparison
 * method that Section 3.4 contrasts with the power law (Section 4.1 runs it
 * between an upper and a lower bound on the executed blocks; its constants are
 * not in the paper, so the bounds are arguments).  In integers, for i in
 * [0, n_steps):  keep[i] = keep_first - ceil((keep_first - keep_last) * i /
 * max(1, n_steps - 1)), i.e. floor of the straight line from keep_first at
 * i = 0 to keep_last at the last step.  The dropped window follows the rule of
 * d3_plan_depth, so start_layer = 0 drops shallow blocks first and start_layer
 * = L - 1 deep blocks first (the two skip directions of Section 1 / Figure 1);
 * anything between is the middle-first order of D^3.  Same outputs and
 * ownership as d3_plan_depth.  D3_EINVAL unless L >= 1, 0 <= keep_last <=
 * keep_first <= L, 0 <= start_layer < L, n_steps >= 0. */
int d3_plan_depth_linear(int32_t L, int32_t keep_first, int32_t keep_last, int32_t start_layer,
                         int32_t n_steps, int32_t *keep, int32_t *drop_begin, int32_t *layer_ids);

/* Executed-block lists of a caller-made schedule (same table rule, Table 6):
 * host int32 keep[n_steps], drop_begin[n_steps] in, layer_ids[n_steps*L] out
 * (may be NULL: validation only).  D3_EINVAL unless every step has
 * 0 <= keep[i] <= L and its window [drop_begin[i], drop_begin[i] + L - keep[i])
 * inside [0, L). */
int d3_plan_from_table(int32_t L, int32_t n_steps, const int32_t *keep, const int32_t *drop_begin,
                       int32_t *layer_ids);

/* Bytes of device workspace d3_create needs for this model (0 on a bad desc). */
size_t d3_workspace_size(const d3_model_desc *desc);

/* Build a context around caller-owned device buffers.  k_cache / v_cache: dev,
 * [L][max_batch][H_kv][max_seq][head_dim] of kv_dtype.  workspace: dev, at least
 * d3_workspace_size() bytes, 256-byte aligned; the library keeps the residual
 * stream, activations, attention partials and the layer-index table there.
 * D3_ESHAPE unless head_dim in {64,128}, n_heads % n_kv_heads == 0,
 * d_model % 8 == 0, d_ffn % 8 == 0, 1 <= max_batch <= 32. */
int d3_create(d3_ctx **out, const d3_model_desc *desc, const d3_weights *weights, void *k_cache,
              void *v_cache, void *workspace, size_t workspace_bytes);
int d3_destroy(d3_ctx *ctx);

/* Start a request's schedule: computes the plan with d3_plan_depth and keeps
 * the layer-index table (n_steps <= 4096; host only, no device work).  The next
 * d3_decode_step must be step 1.  Keeps the cache contents and row count. */
int d3_set_plan(d3_ctx *ctx, double alpha, int32_t start_layer, int32_t min_keep, int32_t n_steps);

/* Same, for a schedule the caller made (d3_plan_depth_linear, or any table
 * d3_plan_from_table accepts): host int32 keep[n_steps], drop_begin[n_steps],
 * copied.  Step i of d3_decode_step runs the blocks outside step i's window. */
int d3_set_plan_table(d3_ctx *ctx, const int32_t *keep, const int32_t *drop_begin, int32_t n_steps);

/* Prompt pass (Section 3.1 "initiation phase"; all L blocks, Section 3.2).
 * tokens: dev int32 [B][P].  Writes cache rows [pos_begin, pos_begin + P) of
 * every block for sequences 0..B-1, causal attention over rows [0, pos_begin+p].
 * pos_begin must be 0 (fresh request) or the current row count (continue on the
 * same cache, e.g. after d3_fill_missing_kv).  next_tok: dev int32 [B] = T_0
 * (argmax of the last position's logits, lowest index on ties); logits: dev
 * float32 [B][vocab] or NULL; hidden_dump: dev float32 [L+1][B][d_model] or
 * NULL (residual stream of the last prompt position after the embedding and
 * after each block).  Resets the step counter: the next decode step is 1. */
int d3_prefill(d3_ctx *ctx, const int32_t *tokens, int32_t B, int32_t P, int32_t pos_begin,
               int32_t *next_tok, float *logits, float *hidden_dump, void *hip_stream);

/* Prompt pass of a batch of unequal prompt lengths (Section 4.2 runs batches of
 * 4 and 8 few-shot prompts through a harness that pads them on the left to the
 * longest).  tokens: dev int32 [B][P], sequence b's lengths[b] tokens in columns
 * [P - lengths[b], P), anything before them (never read); lengths: HOST int32
 * [B].  Cache rows have the column's number, so every sequence's last prompt
 * token is row P - 1 and decode steps append one common row; rows below
 * P - lengths[b] of sequence b are never written nor read, and its rotary
 * positions count from its first token (position = row - (P - lengths[b])), as
 * if it had run alone.  The depth schedule stays that of the common step index i
 * (Section 3.4).  Outputs as d3_prefill; always a fresh request (pos_begin 0);
 * a later d3_prefill with pos_begin > 0 continues it with B equal tails.
 * D3_EINVAL unless 1 <= lengths[b] <= P and the longest equals P. */
int d3_prefill_ragged(d3_ctx *ctx, const int32_t *tokens, const int32_t *lengths, int32_t B,
                      int32_t P, int32_t *next_tok, float *logits, float *hidden_dump,
                      void *hip_stream);

/* One decode step (Section 3.1 "generation phase"; Section 3.4).  tok_in: dev
 * int32 [B] = T_{step_i - 1}; runs the keep[step_i] executed blocks of the plan,
 * appends one cache row per sequence in each of them, and writes tok_out: dev
 * int32 [B] = T_{step_i}; logits: dev float32 [B][vocab] or NULL; hidden_dump:
 * dev float32 [keep+1][B][d_model] or NULL.  Skipped blocks leave the hidden
 * state unchanged and their cache rows unwritten (see d3_fill_missing_kv).
 * D3_ESTATE unless step_i == previous step + 1; D3_ERANGE if step_i is outside
 * the plan or the cache is full. */
int d3_decode_step(d3_ctx *ctx, const int32_t *tok_in, int32_t step_i, int32_t *tok_out,
                   float *logits, float *hidden_dump, void *hip_stream);

/* d3_decode_step for callers that cannot allocate device memory and have none to lend: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, state changes, results and
 * errors as d3_decode_step, but every intermediate of the step (residual stream, activations, attention
 * partials, arrival counters, the rotary table) lives in a static device array inside the library,
 * d3_static_scratch_bytes() = 32 MiB per GPU, held from the first d3_create on that GPU until the process
 * ends, instead of the context's workspace (which is left untouched).  The call allocates nothing, on the host or on
 * the device, and enqueues kernels and device-to-device copies only (no memset nodes).  D3_ESHAPE if a step of
 * this model at desc.max_batch needs more than the array holds (the 7B, 13B and 70B shapes fit up to batch 16);
 * D3_ESTATE with D3_FILL_RECOMPUTE (that fill reads a residual kept in the workspace).  All contexts on a GPU
 * share the one array: calls of this function that overlap on one GPU (different streams or threads) race;
 * calls on one stream, also of different contexts, are safe, since the array carries nothing from one call to the
 * next.  Steps of one request may mix d3_decode_step and d3_decode_step_static freely. */
int d3_decode_step_static(d3_ctx *ctx, const int32_t *tok_in, int32_t step_i, int32_t *tok_out,
                          float *logits, float *hidden_dump, void *hip_stream);
size_t d3_static_scratch_bytes(void);

/* Missing-state fill (Section 1, challenge (i); Section 3.2): for every cache
 * row p in [pos_begin, pos_end) that a decode step wrote with a reduced depth,
 * and every block l that step dropped, K[l][.][p], V[l][.][p] <- K[src][.][p],
 * V[src][.][p], where src is the last executed block before the drop window
 * (the first one after it when the window starts at block 0; zeros when no
 * block ran).  Rows written by the prompt pass need nothing.  D3_FILL_COPY may be
 * called every step with a one-row range or once before the cache is reused;
 * the result is the same.
 * D3_FILL_RECOMPUTE (Section 3.2: hidden state copied, KV recomputed, as in
 * CALM): K[l][.][p] = RoPE(W_k^l a), V[l][.][p] = W_v^l a with a = RMSNorm_l(h),
 * h = the residual that entered the drop window of the step that wrote row p
 * (the embedding when the window starts at block 0).  Needs
 * d3_set_fill_mode(ctx, D3_FILL_RECOMPUTE) before that decode step, and fills
 * the row of the latest decode step only: [pos_begin, pos_end) must be
 * [n_ctx - 1, n_ctx), else D3_ESTATE.  Streams W_k, W_v of every dropped block. */
int d3_fill_missing_kv(d3_ctx *ctx, int32_t pos_begin, int32_t pos_end, int32_t mode, void *hip_stream);

/* Which fill the caller will use.  With D3_FILL_RECOMPUTE every decode step keeps the
 * residual that enters its drop window (one device copy of [B][d_model] floats per
 * step) for the d3_fill_missing_kv call that follows it.  Default D3_FILL_COPY. */
int d3_set_fill_mode(d3_ctx *ctx, int32_t mode);

/* Current number of cache rows per sequence. */
int32_t d3_n_ctx(const d3_ctx *ctx);

/* Forget cache rows [n_rows, n_ctx): the next decode step writes row n_rows.
 * Used to re-run the generation phase on the same prompt (Section 3.1) without a
 * new prompt pass.  Resets the step counter (next decode step is 1).  Host only.
 * D3_ERANGE unless 1 <= n_rows <= n_ctx (and, after d3_prefill_ragged, n_rows
 * lies above every sequence's first row). */
int d3_truncate(d3_ctx *ctx, int32_t n_rows);

/* Measurement aid: per-launch timing of one kernel class with HIP events recorded
 * on the caller's stream (the projections dominate the step: its cost is that of
 * the decoder blocks it runs, Section 1).  While a class is
 * selected, every launch of it is bracketed by two events (at most 16384 launches
 * are recorded; further ones run untimed).  d3_profile_read synchronises on the
 * recorded events, returns their summed duration and count, and clears them.
 * Selecting D3_K_NONE switches the bracketing off. */
typedef enum {
    D3_K_NONE = 0, D3_K_QKV = 1, D3_K_ATTN = 2, D3_K_OPROJ = 3, D3_K_GATE_UP = 4, D3_K_DOWN = 5, D3_K_LM_HEAD = 6,
    D3_K_EMPTY = 7 /* a bracket with no launch inside, recorded once per block between the gate/up and the down
                      projection: what the pair of events itself adds to every bracketed launch */
} d3_kernel_class;
int d3_profile_select(d3_ctx *ctx, int32_t kernel_class);
int d3_profile_read(d3_ctx *ctx, double *total_ms, int64_t *launches);

/* Measurement aid: one launch that reads `bytes` of device memory (16-byte aligned, a multiple of 16) exactly once
 * and writes nothing but a checksum, with the same load instructions and launch shape as the weight-streaming
 * projections (Section 4.2 measures wall-clock time; this is the read-only yardstick the achieved HBM rates are held
 * against).  Asynchronous on the given stream; the checksum lands in the context's workspace. */
int d3_stream_read(d3_ctx *ctx, const void *src, size_t bytes, void *hip_stream);

/* Measurement aid for the prompt pass (Section 3.2: the first token runs every block; the one compute-bound part of the
 * path): one launch of one workgroup per compute unit that runs the stage loop of the prompt-pass GEMM on fixed
 * operands, 8 waves x `stages` x 32 matrix-core instructions of 16384 flops per workgroup, and touches no global memory
 * but one word per wave.  mode 0: the matrix-core instructions alone; 1: with the loop's LDS fragment reads beside
 * them; 2: with its workgroup barrier per stage as well.  `stages` even, in [2, 2^20].  Asynchronous on the given
 * stream; what the matrix cores sustain on this chip is the flop count over the launch's duration. */
int d3_mfma_yardstick(d3_ctx *ctx, int32_t mode, int32_t stages, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
