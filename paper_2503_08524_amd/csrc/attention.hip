// Decode attention over the KV cache: one query row per column, softmax(q.K^T/sqrt(hd)).V
// over cache rows [0, pos].  The context of a (column, head) is cut into splits handled
// by different workgroups (each keeps a running max / sum / unnormalised output), and a
// split that finishes last merges them (an arrival counter per (column, head)).  K and V rows
// are streamed straight from HBM,
// 16 bytes per lane, several rows per wave per load; the scores of a split live in LDS;
// all reductions are wave shuffles plus one LDS hop across the four waves.
#include "attention.h"

namespace d3 {

namespace {

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    extern __shared__ float sc[];          // scores, then probabilities, of this split
    __shared__ AttnShared<HD, 4> sh;
    attn_split<T, HD, false, 4>(a, blockIdx.x, blockIdx.y, blockIdx.z, sc, sh);
}

}  // namespace

// Requirements (checked by the caller): hd in {64, 128}; split_len * n_splits >= longest context;
// n_splits <= kMaxSplits; split_len * 4 bytes of LDS <= 48 KiB.
int launch_attention(const AttnArgs& a, int kv_dtype, hipStream_t s) {
    dim3 grid(a.n_splits, a.H, a.ncols);
    const size_t lds = (size_t)a.split_len * sizeof(float);
#define D3_ATTN(T)                                                                                      \
    do {                                                                                                \
        if (a.hd == 64) hipLaunchKernelGGL((attn_partial_kernel<T, 64>), grid, dim3(256), lds, s, a);   \
        else hipLaunchKernelGGL((attn_partial_kernel<T, 128>), grid, dim3(256), lds, s, a);             \
    } while (0)
    if (kv_dtype == 0) D3_ATTN(float);
    else if (kv_dtype == 1) D3_ATTN(bf16_t);
    else D3_ATTN(f16_t);
#undef D3_ATTN
    return (int)hipGetLastError();
}

}  // namespace d3
