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
#include "sv_attend_common.h"

namespace sv {
namespace {

constexpr int kAttnUnroll = 4;    // row loads in flight per lane

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

    const TokenList tokens = token_list(a, b, unit);
    const int T_len = tokens.len;
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
    auto token_offset = [&](int t, bool& is_txt) -> int64_t { return tokens.offset(t, is_txt); };

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
// One workgroup per (b, h).  Lane groups of D/4 lanes each take every NG-th chunk with
// 128-bit loads; all loads are issued before the maximum is known, so the kernel costs one
// round trip through memory.
template <typename T, int D>
__global__ __launch_bounds__(kAttnThreads) void attn_combine_kernel(const AttnArgs a) {
    constexpr int LPG = D / 4;                  // lanes per chunk row (float4 each)
    constexpr int NG = kAttnThreads / LPG;      // chunk rows in flight per pass
    constexpr int R = 4;                        // passes kept in registers
    __shared__ float s_red[kAttnWaves];
    __shared__ float s_part[NG][D + 1];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int g = h / a.G;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const TokenList tokens = token_list(a, b, unit);
    const int S = a.n_chunks;
    // live slots: joint list -> the first ceil(len / chunk); split list -> the first ceil(nt / chunk)
    // of the text range and the first ceil(kept / chunk_vis) of the visual range
    const bool split = a.split_base >= 0;
    const int Sb_txt = split ? (tokens.nt + a.chunk - 1) / a.chunk : 0;
    const int Sb = split ? Sb_txt + (tokens.len - tokens.nt + a.chunk_vis - 1) / a.chunk_vis
                         : (tokens.len + a.chunk - 1) / a.chunk;
    const int skip = split ? a.split_base - Sb_txt : 0;   // dead slots between the live text and visual ranges
    auto slot_of = [&](int i) -> int { return i < Sb_txt ? i : i + skip; };
    const int64_t bh = (int64_t)b * a.Hq + h;
    if (Sb == 0) {
        if (tid < D) a.out[bh * D + tid] = 0.f;
        if (a.lse && tid == 0) a.lse[bh] = -INFINITY;
        return;
    }
    const float* ml = a.part_ml + bh * S * 2;
    const float* acc = a.part_acc + bh * S * D;
    const int grp = tid / LPG, c4 = (tid % LPG) * 4;

    float4_t av[R];
    float mv[R], lv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int sidx = grp + r * NG;
        av[r] = 0;
        mv[r] = -INFINITY;
        lv[r] = 0.f;
        if (sidx < Sb) {
            const int sl = slot_of(sidx);
            av[r] = *reinterpret_cast<const float4_t*>(acc + (int64_t)sl * D + c4);
            mv[r] = ml[2 * sl];
            lv[r] = ml[2 * sl + 1];
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int r = 0; r < R; ++r) m = fmaxf(m, mv[r]);
    for (int sidx = grp + R * NG; sidx < Sb; sidx += NG) m = fmaxf(m, ml[2 * slot_of(sidx)]);
    m = wave_max(m);
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));

    float4_t o = {0.f, 0.f, 0.f, 0.f};
    float L = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float w = mv[r] == -INFINITY ? 0.f : exp_for<T>(mv[r] - m);
        o += w * av[r];
        L = fmaf(w, lv[r], L);
    }
    for (int sidx = grp + R * NG; sidx < Sb; sidx += NG) {
        const int sl = slot_of(sidx);
        const float ms = ml[2 * sl];
        const float w = ms == -INFINITY ? 0.f : exp_for<T>(ms - m);
        o += w * *reinterpret_cast<const float4_t*>(acc + (int64_t)sl * D + c4);
        L = fmaf(w, ml[2 * sl + 1], L);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) s_part[grp][c4 + i] = o[i];
    if (c4 == 0) s_part[grp][D] = L;
    __syncthreads();
    if (tid < D) {
        float x = 0.f, Lt = 0.f;
#pragma unroll
        for (int q = 0; q < NG; ++q) { x += s_part[q][tid]; Lt += s_part[q][D]; }
        a.out[bh * D + tid] = x / Lt;
        if (a.lse && tid == 0) a.lse[bh] = m + logf(Lt);
    }
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
        if (std::is_same<T, _Float16>::value && a.use_mfma) e = launch_attn_partial_mfma(a, stream);
        else if (G == 1) e = launch_partial<T, D, 1>(a, 1, stream);
        else if (G == 2) e = launch_partial<T, D, 2>(a, 1, stream);
        else if (G <= 4) e = launch_partial<T, D, 4>(a, 1, stream);
        else if (G == 7) e = launch_partial<T, D, 7>(a, 1, stream);
        else if (G <= 8) e = launch_partial<T, D, 8>(a, 1, stream);
        else e = launch_partial<T, D, 8>(a, (G + kHeadBlock - 1) / kHeadBlock, stream);
        if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)a.Hq, (unsigned)a.B), block(kAttnThreads);
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
