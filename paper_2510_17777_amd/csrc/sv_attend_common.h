// Pieces shared by the attention kernels: length clamps, the exponential of each cache
// dtype, and the mapping from a position in the token list T to a cache row.
#pragma once
#include <type_traits>

#include "sv_device.h"
#include "sv_kernels.h"

namespace sv {

constexpr int kAttnWaves = 4;
constexpr int kAttnThreads = kAttnWaves * kWave;
constexpr int kHeadBlock = 8;   // query heads per workgroup when a group has more than 8

template <typename T>
__device__ __forceinline__ float exp_for(float x) {
    // fp32 caches are held to 1e-5: use the accurate exponential there.
    return std::is_same<T, float>::value ? expf(x) : __expf(x);
}

__device__ __forceinline__ int clamp_len(const int32_t* p, int i, int hi) {
    if (!p) return hi;
    const int v = p[i];
    return v < 0 ? 0 : (v < hi ? v : hi);
}

// The token list of one (b, g): text rows 0..nt-1, then the visual rows named by idx.
struct TokenList {
    int nt;                  // live text tokens
    int len;                 // nt + kept visual tokens
    const int32_t* idx_row;  // kept visual indices of this (b, g), or nullptr
    int n_vis_max;
    int64_t txt_sn, vis_sn;

    // Element offset of token t's row inside its cache; is_txt says which cache.
    __device__ __forceinline__ int64_t offset(int t, bool& is_txt) const {
        is_txt = t < nt;
        if (is_txt) return (int64_t)t * txt_sn;
        int j = idx_row ? idx_row[t - nt] : t - nt;   // no idx: the visual segment is packed
        j = j < 0 ? 0 : (j < n_vis_max ? j : n_vis_max - 1);   // a faulty idx must not fault the GPU
        return (int64_t)j * vis_sn;
    }
};

__device__ __forceinline__ TokenList token_list(const AttnArgs& a, int b, int64_t unit) {
    TokenList t;
    t.nt = clamp_len(a.txt_len, b, a.n_txt_max);
    const int kc = (a.k > 0 && a.count) ? clamp_len(a.count, (int)unit, a.k) : 0;
    t.len = t.nt + kc;
    t.idx_row = a.idx ? a.idx + unit * a.k : nullptr;
    t.n_vis_max = a.n_vis_max;
    t.txt_sn = a.txt_sn;
    t.vis_sn = a.vis_sn;
    return t;
}

// fp16 caches: logits through the matrix cores (sv_attend_mfma.hip), and for head_dim 128 logits
// and p*V through the matrix cores with wavefronts streaming over batches (sv_attend_flash.hip).
hipError_t launch_attn_partial_mfma(const AttnArgs& a, hipStream_t stream);
hipError_t launch_attn_partial_flash(const AttnArgs& a, hipStream_t stream);

}  // namespace sv
