// Decode attention over the KV cache: one query row per column, softmax(q.K^T/sqrt(hd)).V
// over cache rows [0, pos].  The context of a (column, head) is cut into splits handled
// by different workgroups (each keeps a running max / sum / unnormalised output), and a
// split that finishes last merges them (an arrival counter per (column, head)).  K and V rows
// are streamed straight from HBM,
// 16 bytes per lane, several rows per wave per load, once for all query heads of a KV head;
// every wave keeps an online softmax per head in registers; reductions are wave shuffles plus
// one LDS hop across the four waves.
#include <cstdlib>
#include <type_traits>

#include "attention.h"

namespace d3 {

namespace {

// grid: (split, KV-head group, column); G query heads per group
template <typename T, int HD, int G, bool ROPE>
__global__ __launch_bounds__(256) void attn_kernel(AttnArgs a) {
    __shared__ AttnShared<HD, 4, G> sh;
    attn_split<T, HD, false, 4, G, ROPE>(a, blockIdx.x, blockIdx.y * G, blockIdx.z, sh);
}

// The staging tiles of an fp32 cache (hi + lo planes, 105 KB for four waves) exceed what a kernel may declare statically:
// that variant takes its LDS as dynamic shared memory.
extern __shared__ __align__(16) char attn_dyn_lds[];

template <typename T, int G, bool ROPE>
__global__ __launch_bounds__(256) void attn_mfma_kernel(AttnArgs a) {
    typedef AttnMfmaShared<4, G, AttnStage<T>::PL> Shared;
    if constexpr (AttnStage<T>::PL == 1) {
        __shared__ Shared sh;
        attn_split_mfma<T, ROPE, 4, G>(a, blockIdx.x, blockIdx.y * G, blockIdx.z, sh);
    } else {
        attn_split_mfma<T, ROPE, 4, G>(a, blockIdx.x, blockIdx.y * G, blockIdx.z, *reinterpret_cast<Shared*>(attn_dyn_lds));
    }
}

// grid: (split, KV-head group, tile of 16 / GH consecutive queries)
template <typename T, int GH>
__global__ __launch_bounds__(256) void attn_qtile_kernel(AttnArgs a) {
    typedef AttnMfmaShared<4, 16, AttnStage<T>::PL> Shared;
    if constexpr (AttnStage<T>::PL == 1) {
        __shared__ Shared sh;
        attn_qtile_mfma<T, 4, GH>(a, blockIdx.x, blockIdx.y * GH, blockIdx.z * (16 / GH), sh);
    } else {
        attn_qtile_mfma<T, 4, GH>(a, blockIdx.x, blockIdx.y * GH, blockIdx.z * (16 / GH), *reinterpret_cast<Shared*>(attn_dyn_lds));
    }
}

// launch with the LDS the element type needs (dynamic for the two-plane variant, whose size must be allowed once per kernel)
template <typename T, typename Shared, typename K>
int launch_mfma(K kernel, dim3 grid, const AttnArgs& a, hipStream_t s) {
    size_t dyn = 0;
    if constexpr (AttnStage<T>::PL == 2) {
        dyn = sizeof(Shared);
        static const hipError_t once = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Shared));
        if (once != hipSuccess) return (int)once;
    }
    hipLaunchKernelGGL(kernel, grid, dim3(256), dyn, s, a);
    return (int)hipGetLastError();
}

template <typename T, int HD, bool ROPE>
int launch_g(const AttnArgs& a, bool use_mfma, hipStream_t s) {
    const int group = a.H / a.H_kv;
    if constexpr (HD == 128 && !ROPE) {
        if (a.qtile && (group == 1 || group == 2 || group == 4 || group == 8) && use_mfma) {
            const int qt = 16 / group;
            dim3 grid(a.n_splits, a.H / group, (a.ncols + qt - 1) / qt);
            typedef AttnMfmaShared<4, 16, AttnStage<T>::PL> Shared;
            if (group == 8) return launch_mfma<T, Shared>(attn_qtile_kernel<T, 8>, grid, a, s);
            if (group == 4) return launch_mfma<T, Shared>(attn_qtile_kernel<T, 4>, grid, a, s);
            if (group == 2) return launch_mfma<T, Shared>(attn_qtile_kernel<T, 2>, grid, a, s);
            return launch_mfma<T, Shared>(attn_qtile_kernel<T, 1>, grid, a, s);
        }
    }
    if constexpr (HD == 128) {
        if ((group == 4 || group == 8) && use_mfma) {
            dim3 grid(a.n_splits, a.H / group, a.ncols);
            if (group == 8) return launch_mfma<T, AttnMfmaShared<4, 8, AttnStage<T>::PL>>(attn_mfma_kernel<T, 8, ROPE>, grid, a, s);
            return launch_mfma<T, AttnMfmaShared<4, 4, AttnStage<T>::PL>>(attn_mfma_kernel<T, 4, ROPE>, grid, a, s);
        }
    }
    const int g = (group == 2 || group == 4 || group == 8) ? group : 1;    // other group sizes: one query head per workgroup
    dim3 grid(a.n_splits, a.H / g, a.ncols);
    if (g == 8) hipLaunchKernelGGL((attn_kernel<T, HD, 8, ROPE>), grid, dim3(256), 0, s, a);
    else if (g == 4) hipLaunchKernelGGL((attn_kernel<T, HD, 4, ROPE>), grid, dim3(256), 0, s, a);
    else if (g == 2) hipLaunchKernelGGL((attn_kernel<T, HD, 2, ROPE>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_kernel<T, HD, 1, ROPE>), grid, dim3(256), 0, s, a);
    return (int)hipGetLastError();
}

}  // namespace

// Requirements (checked by the caller): hd in {64, 128}; split_len * n_splits >= longest context;
// n_splits <= kMaxSplits; tickets zero on entry (the kernel leaves them zero).
template <bool ROPE>
int launch_t(const AttnArgs& a, int kv_dtype, bool use_mfma, hipStream_t s) {
    if (kv_dtype == 0) return a.hd == 64 ? launch_g<float, 64, ROPE>(a, use_mfma, s) : launch_g<float, 128, ROPE>(a, use_mfma, s);
    if (kv_dtype == 2) return a.hd == 64 ? launch_g<f16_t, 64, ROPE>(a, use_mfma, s) : launch_g<f16_t, 128, ROPE>(a, use_mfma, s);
    return (int)hipErrorInvalidValue;
}

// With rope_cs set, q and the newest K/V row of each column are still unrotated in the projection buffer and
// the kernel rotates and appends them itself; the columns of such a pass must belong to different sequences.
// use_mfma = false keeps grouped-query and query-tile attention on the vector ALUs (for comparisons).
int launch_attention(const AttnArgs& a, int kv_dtype, bool use_mfma, hipStream_t s) {
    return a.rope_cs ? launch_t<true>(a, kv_dtype, use_mfma, s) : launch_t<false>(a, kv_dtype, use_mfma, s);
}

}  // namespace d3
