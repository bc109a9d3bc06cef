/* CPU oracle for Position-Aware Depth Decay Decoding (D^3).
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, obviously-correct implementation of
 * what the HIP path computes.  It shares no code with the HIP library and must
 * never be linked, loaded or called from the product path; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg use it.
 *
 * The paper defines the policy (Abstract, Section 1, Section 3.4, Table 6):
 * when generating token T_i, keep floor(L * alpha^i) decoder blocks and drop a
 * contiguous window of middle ("flex") blocks beginning at `start`.  Skipped
 * blocks pass the hidden state through unchanged (Section 3.2).  The decoder
 * blocks themselves are the Llama-2 ones the paper runs on (Section 4.1):
 * RMSNorm, rotary embedding, (grouped-query) attention, SwiGLU MLP.
 *
 * Precision: compiled twice, with D3O_REAL=double (default; parity reference)
 * and D3O_REAL=float.  Weights are taken exactly as given (float32, or bf16 bit
 * patterns upcast exactly).  No blocking, fusion or reordering: every dot
 * product is a left-to-right sum.
 *
 * Pins (tests/test_oracle_*.py): closed-form schedule vs exact rationals and
 * the paper's Table 5 averages; NumPy no-cache brute force; torch CPU library
 * routines for one block; RoPE / softmax / RMSNorm invariants.
 * Unpinned by the paper: the actual token sequences and logits of a
 * random-init model (only oracle-vs-brute-force agreement pins them).
 */
#ifndef D3_ORACLE_H
#define D3_ORACLE_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t L, d, H, H_kv, hd, F, V;
    double eps, rope_base;
    int32_t weight_dtype; /* 0 = float32, 1 = bf16 bit patterns (uint16) */
} d3o_config;

/* One block's tensors, row-major [out][in]; gains are float32. */
typedef struct {
    const float *attn_norm;
    const void *wq, *wk, *wv, *wo;
    const float *mlp_norm;
    const void *w_gate, *w_up, *w_down;
} d3o_layer;

typedef struct d3o_model d3o_model;
typedef struct d3o_seq d3o_seq;

int d3o_real_size(void);         /* sizeof(D3O_REAL) this library was built with */
void d3o_set_threads(int n);     /* row-parallel matvec threads (results unchanged) */

/* Depth schedule (Section 3.4; Table 6).  pow_0 = 1, pow_i = pow_{i-1} * alpha in
 * binary64; keep[i] = max(min_keep, floor(L * pow_i)); n_i = L - keep[i];
 * drop_begin[i] = min(start, L - n_i); dropped blocks = [drop_begin, drop_begin + n_i);
 * layer_ids[i*L + j] = j-th executed block, -1 padded.  Any output may be NULL.
 * Returns 0, or -1 on invalid arguments. */
int d3o_plan_depth(int32_t L, double alpha, int32_t start, int32_t min_keep, int32_t n_steps,
                   int32_t *keep, int32_t *drop_begin, int32_t *layer_ids);
int d3o_plan_depth_linear(int32_t L, int32_t keep_first, int32_t keep_last, int32_t start, int32_t n_steps,
                          int32_t *keep, int32_t *drop_begin, int32_t *layer_ids);

/* The model borrows every pointer; they must outlive it. */
d3o_model *d3o_model_new(const d3o_config *cfg, const void *tok_emb, const d3o_layer *layers,
                         const float *final_norm, const void *lm_head);
void d3o_model_free(d3o_model *);

/* One sequence's KV cache: [L][max_seq][H_kv*hd] for K and for V. */
d3o_seq *d3o_seq_new(const d3o_model *, int32_t max_seq);
void d3o_seq_free(d3o_seq *);

/* Run one token at absolute position `pos` through the listed blocks (increasing
 * ids), writing their K/V row `pos`.  Attention sees rows 0..pos of each executed
 * block.  hidden_out (or NULL): [(n_ids+1)][d], the residual stream after the
 * embedding and after each executed block.  logits_out (or NULL): [V], from the
 * final RMSNorm + lm_head.  Returns 0, or -1 on invalid arguments. */
int d3o_forward_token(d3o_seq *, int32_t token, int32_t pos, const int32_t *layer_ids, int32_t n_ids,
                      double *hidden_out, double *logits_out);

/* Only the cache write of d3o_forward_token(token, pos, {layer}): K[layer][pos], V[layer][pos] of a token that
 * enters `layer` as its bare embedding (same steps, same order; the rest of the block is not run). */
int d3o_first_block_kv(d3o_seq *, int32_t token, int32_t pos, int32_t layer);

/* Lowest index of the maximum. */
int32_t d3o_argmax(const double *logits, int32_t n);

/* COPY fill (Section 3.2, SkipDecode-style): for every block l in
 * [drop_begin, drop_begin + n_drop): K[l][pos], V[l][pos] <- K[src][pos], V[src][pos],
 * src = drop_begin - 1, or drop_begin + n_drop if drop_begin == 0; zeros if no block ran. */
int d3o_fill_missing_kv(d3o_seq *, int32_t pos, int32_t drop_begin, int32_t n_drop);

/* RECOMPUTE fill (Section 3.2, CALM-style): h [d] is the hidden state copied through the skipped blocks
 * (the residual that entered the drop window); for every block l in [drop_begin, drop_begin + n_drop):
 * K[l][pos] = RoPE(W_k^l RMSNorm_l(h)), V[l][pos] = W_v^l RMSNorm_l(h). */
int d3o_fill_recompute(d3o_seq *, int32_t pos, int32_t drop_begin, int32_t n_drop, const double *h);

/* Read one cache row (K and V, each [H_kv*hd]) as doubles. */
int d3o_get_kv(const d3o_seq *, int32_t layer, int32_t pos, double *k_out, double *v_out);

/* Sub-functions, exported so the tests can pin them one by one. */
void d3o_rmsnorm(const double *x, const float *gain, int32_t n, double eps, double *out);
void d3o_rope(double *vec, int32_t hd, int32_t pos, double base);      /* in place, one head */
void d3o_softmax(double *v, int32_t n);                               /* in place */
double d3o_silu(double x);
void d3o_attention_head(const double *q, const double *K, const double *V, int32_t n_rows,
                        int32_t hd, int32_t row_stride, double *out);  /* one query head */

#ifdef __cplusplus
}
#endif
#endif
