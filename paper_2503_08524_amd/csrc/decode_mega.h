// Arguments of the persistent one-launch decode step (decode_mega.hip).
#pragma once
#include "../../include/d3.h"
#include "d3_common.h"

namespace d3 {

struct MegaArgs {
    // model
    int d_model, H, H_kv, d_ffn, vocab, max_seq, kv_dtype;
    float eps;
    const void* tok_emb;
    const float* final_norm;
    const void* lm_head;
    const d3_layer_weights* layers;   // DEVICE copy of the per-block pointer table
    char* k_cache;                    // whole cache; block l starts at l * kv_layer_bytes
    char* v_cache;
    size_t kv_layer_bytes;
    const double* inv_freq;           // [hd/2]
    // this step
    const int32_t* layer_ids;         // DEVICE: executed blocks of this step (row of the layer-index table)
    int n_ids;
    int pos;                          // cache row written by this step
    const int32_t* tok_in;            // [1]
    int32_t* tok_out;                 // [1]
    float* logits;                    // [vocab]
    float* hidden_dump;               // [(n_ids+1)][d_model] or nullptr
    int split_len, n_splits;          // attention context splits
    // workspace
    float *x, *qkv, *attn_o, *act, *part_o, *part_ml, *cand_val;
    int *tickets, *cand_idx;
    float2* rope_cs;
    // grid barrier
    unsigned* barrier_state;          // 512 words, zero before the first launch
    unsigned barrier_epoch;           // barriers completed by earlier launches
    int max_spins;
    unsigned long long* debug_ts;     // optional: every workgroup's 100 MHz timestamps at phase boundaries (14 per block)
    int debug_stride;                 // marks per workgroup row
};

size_t mega_lds_bytes(const MegaArgs& m);
int mega_max_workgroups(int kv_dtype, int depth, size_t lds_bytes, int n_cu);      // co-resident workgroups, 0 on error
int launch_decode_mega(const MegaArgs& m, int kv_dtype, int depth, int n_wg, hipStream_t s);   // hipError_t as int

}  // namespace d3
