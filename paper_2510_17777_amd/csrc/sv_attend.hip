// Step 3 of the decode path: decode attention over all text tokens plus the kept
// visual tokens (paper section 3.2, first paragraph; section 4.5, "Decoding
// Attention Kernel Efficiency": the step is bound by KV-cache traffic).
//
// The token list T of a (batch, kv head) -- text rows, then the visual rows named by
// idx -- is cut into chunks; one workgroup (4 wavefronts) handles one chunk for all
// query heads of the group, so every K and V row is fetched once per group:
//   A. logits: a row is spread over 16-byte chunks, one per lane; each lane keeps the
//      matching slice of every head's (pre-scaled) query in registers, partial dots
//      are reduced with DPP inside the row's lanes; logits go to LDS;
//   B. per head: chunk maximum m, p = exp(logit - m) written back to LDS, l = sum p;
//   C. acc[h,:] += p[h,t] * V[t,:] with the same row-per-lane-group layout, reduced
//      across lane groups and wavefronts at the end.
// Chunks write (m, l, acc); a second kernel merges them with the usual
// log-sum-exp rule.  Everything accumulates in fp32 in a fixed order.
#include "sv_device.h"
#include "sv_kernels.h"

#include <type_traits>

namespace sv {
namespace {

constexpr int kAttnWaves = 4;
constexpr int kAttnThreads = kAttnWaves * kWave;
constexpr int kAttnUnroll = 4;    // row loads in flight per lane
constexpr int kHeadBlock = 8;     // query heads per workgroup when G > 8

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

template <typename T, int D, int GB>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_kernel(const AttnArgs a, const int hblk) {
    constexpr int EPL = Chunk<T>::kElems;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int U = kAttnUnroll;
    extern __shared__ float smem[];

    const int CH = a.chunk;
    const int s = blockIdx.x;
    const int g = blockIdx.y / hblk, hb = blockIdx.y % hblk;
    const int b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int c = lane % LPR, grp = lane / LPR;
    const int64_t unit = (int64_t)b * a.Hkv + g;

    const int nt = clamp_len(a.txt_len, b, a.n_txt_max);
    const int kc = (a.k > 0 && a.count) ? clamp_len(a.count, (int)unit, a.k) : 0;
    const int T_len = nt + kc;
    const int t0 = s * CH;
    if (t0 >= T_len) return;   // block-uniform

    float* s_logit = smem;                       // [GB][CH]
    float* s_acc = smem + GB * CH;               // [waves][GB][D]
    float* s_m = s_acc + kAttnWaves * GB * D;    // [GB]
    float* s_l = s_m + GB;                       // [GB]

    const int h_first = g * a.G + hb * (hblk > 1 ? kHeadBlock : 0);
    const int g_valid = min(GB, a.G - hb * (hblk > 1 ? kHeadBlock : 0));

    const T* ktxt = static_cast<const T*>(a.k_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh + c * EPL;
    const T* vtxt = static_cast<const T*>(a.v_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh + c * EPL;
    const T* kvis = static_cast<const T*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh + c * EPL;
    const T* vvis = static_cast<const T*>(a.v_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh + c * EPL;
    const int32_t* idx_row = a.idx ? a.idx + unit * a.k : nullptr;

    // Element offset of token t's row inside its cache (text or visual).
    auto token_offset = [&](int t, bool& is_txt) -> int64_t {
        is_txt = t < nt;
        if (is_txt) return (int64_t)t * a.txt_sn;
        int j = idx_row[t - nt];
        j = j < 0 ? 0 : (j < a.n_vis_max ? j : a.n_vis_max - 1);   // a faulty idx must not fault the GPU
        return (int64_t)j * a.vis_sn;
    };

    const int CW = CH / kAttnWaves;          // tokens per wavefront
    const int tw0 = t0 + wave * CW;

    // ---- A: logits ----
    {
        float qf[GB][EPL];
#pragma unroll
        for (int h = 0; h < GB; ++h) {
            Chunk<T> qc = zero_chunk<T>();
            if (h < g_valid)
                qc = load_chunk(static_cast<const T*>(a.q) + (int64_t)b * a.q_sb +
                                (int64_t)(h_first + h) * a.q_sh + c * EPL);
#pragma unroll
            for (int i = 0; i < EPL; ++i) qf[h][i] = qc.at(i) * a.scale;
        }
        for (int st = 0; st < CW; st += RPW * U) {
            Chunk<T> kc_[U];
            bool valid[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = tw0 + st + u * RPW + grp;
                valid[u] = (st + u * RPW + grp) < CW && t < T_len;
                kc_[u] = zero_chunk<T>();
                if (valid[u]) {
                    bool is_txt;
                    const int64_t off = token_offset(t, is_txt);
                    kc_[u] = load_chunk((is_txt ? ktxt : kvis) + off);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float mine = 0.f;
#pragma unroll
                for (int h = 0; h < GB; ++h) {
                    float d = 0.f;
#pragma unroll
                    for (int i = 0; i < EPL; ++i) d = fmaf(kc_[u].at(i), qf[h][i], d);
                    d = group_sum<LPR>(d);
                    mine = (c == h) ? d : mine;
                }
                const int tl = wave * CW + st + u * RPW + grp;   // token slot inside the chunk
                if (c < GB && (st + u * RPW + grp) < CW)
                    s_logit[c * CH + tl] = valid[u] ? mine : -INFINITY;
            }
        }
    }
    __syncthreads();

    // ---- B: chunk softmax statistics, one head per wavefront at a time ----
    for (int h = wave; h < GB; h += kAttnWaves) {
        float m = -INFINITY;
        for (int i = lane; i < CH; i += kWave) m = fmaxf(m, s_logit[h * CH + i]);
        m = wave_max(m);
        float l = 0.f;
        for (int i = lane; i < CH; i += kWave) {
            const float p = exp_for<T>(s_logit[h * CH + i] - m);
            s_logit[h * CH + i] = p;
            l += p;
        }
        l = wave_sum(l);
        if (lane == 0) { s_m[h] = m; s_l[h] = l; }
    }
    __syncthreads();

    // ---- C: weighted sum of value rows ----
    {
        float acc[GB][EPL];
#pragma unroll
        for (int h = 0; h < GB; ++h)
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[h][i] = 0.f;
        for (int st = 0; st < CW; st += RPW * U) {
            Chunk<T> vc[U];
            bool valid[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = tw0 + st + u * RPW + grp;
                valid[u] = (st + u * RPW + grp) < CW && t < T_len;
                vc[u] = zero_chunk<T>();
                if (valid[u]) {
                    bool is_txt;
                    const int64_t off = token_offset(t, is_txt);
                    vc[u] = load_chunk((is_txt ? vtxt : vvis) + off);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (!valid[u]) continue;
                const int tl = wave * CW + st + u * RPW + grp;
#pragma unroll
                for (int h = 0; h < GB; ++h) {
                    const float p = s_logit[h * CH + tl];
#pragma unroll
                    for (int i = 0; i < EPL; ++i) acc[h][i] = fmaf(p, vc[u].at(i), acc[h][i]);
                }
            }
        }
        // lane groups of a wavefront hold different tokens: add them up
#pragma unroll
        for (int h = 0; h < GB; ++h)
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                float x = acc[h][i];
#pragma unroll
                for (int off = LPR; off < kWave; off <<= 1) x += __shfl_xor(x, off, kWave);
                acc[h][i] = x;
            }
        if (grp == 0) {
#pragma unroll
            for (int h = 0; h < GB; ++h)
#pragma unroll
                for (int i = 0; i < EPL; ++i) s_acc[(wave * GB + h) * D + c * EPL + i] = acc[h][i];
        }
    }
    __syncthreads();

    const int S = a.n_chunks;
    for (int o = threadIdx.x; o < GB * D; o += kAttnThreads) {
        const int h = o / D, d = o % D;
        if (h >= g_valid) continue;
        float x = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) x += s_acc[(w * GB + h) * D + d];
        a.part_acc[(((int64_t)b * a.Hq + h_first + h) * S + s) * D + d] = x;
    }
    if ((int)threadIdx.x < g_valid) {
        const int h = threadIdx.x;
        float* ml = a.part_ml + (((int64_t)b * a.Hq + h_first + h) * S + s) * 2;
        ml[0] = s_m[h];
        ml[1] = s_l[h];
    }
}

// Merge of the chunk results of one query head: out = sum_s e^{m_s-m} acc_s / sum_s e^{m_s-m} l_s.
template <typename T, int D>
__global__ __launch_bounds__(D) void attn_combine_kernel(const AttnArgs a) {
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int g = h / a.G;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int nt = clamp_len(a.txt_len, b, a.n_txt_max);
    const int kc = (a.k > 0 && a.count) ? clamp_len(a.count, (int)unit, a.k) : 0;
    const int T_len = nt + kc;
    const int S = a.n_chunks;
    const int Sb = (T_len + a.chunk - 1) / a.chunk;
    const int64_t bh = (int64_t)b * a.Hq + h;
    if (Sb == 0) {
        a.out[bh * D + d] = 0.f;
        if (a.lse && d == 0) a.lse[bh] = -INFINITY;
        return;
    }
    const float* ml = a.part_ml + bh * S * 2;
    const float* acc = a.part_acc + bh * S * D;
    float m = -INFINITY;
    for (int s = 0; s < Sb; ++s) m = fmaxf(m, ml[2 * s]);
    float L = 0.f, o = 0.f;
    for (int s = 0; s < Sb; ++s) {
        const float w = exp_for<T>(ml[2 * s] - m);
        L = fmaf(w, ml[2 * s + 1], L);
        o = fmaf(w, acc[(int64_t)s * D + d], o);
    }
    a.out[bh * D + d] = o / L;
    if (a.lse && d == 0) a.lse[bh] = m + logf(L);
}

template <typename T, int D, int GB>
hipError_t launch_partial(const AttnArgs& a, int hblk, hipStream_t stream) {
    dim3 grid((unsigned)a.n_chunks, (unsigned)(a.Hkv * hblk), (unsigned)a.B), block(kAttnThreads);
    const size_t lds = sizeof(float) * ((size_t)GB * a.chunk + (size_t)kAttnWaves * GB * D + 2 * GB);
    hipLaunchKernelGGL((attn_partial_kernel<T, D, GB>), grid, block, lds, stream, a, hblk);
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_typed(const AttnArgs& a, hipStream_t stream) {
    hipError_t e = hipSuccess;
    if (a.n_chunks > 0) {
        const int G = a.G;
        if (G == 1) e = launch_partial<T, D, 1>(a, 1, stream);
        else if (G == 2) e = launch_partial<T, D, 2>(a, 1, stream);
        else if (G <= 4) e = launch_partial<T, D, 4>(a, 1, stream);
        else if (G == 7) e = launch_partial<T, D, 7>(a, 1, stream);
        else if (G <= 8) e = launch_partial<T, D, 8>(a, 1, stream);
        else e = launch_partial<T, D, 8>(a, (G + kHeadBlock - 1) / kHeadBlock, stream);
        if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)a.Hq, (unsigned)a.B), block(D);
    hipLaunchKernelGGL((attn_combine_kernel<T, D>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attend(const AttnArgs& a, hipStream_t stream) {
    if (a.B == 0) return hipSuccess;
    if (a.dtype == 0) {
        if (a.D == 128) return launch_typed<_Float16, 128>(a, stream);
        if (a.D == 64) return launch_typed<_Float16, 64>(a, stream);
    } else {
        if (a.D == 128) return launch_typed<float, 128>(a, stream);
        if (a.D == 64) return launch_typed<float, 64>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace sv
