// Step 3 for fp16 caches: chunk attention with the logits on the matrix cores.
//
// The vector path spends 8 FMAs plus a lane reduction per (key chunk, head); with a GQA
// group of 7 heads that made the kernel ALU-bound (it ran at a third of the bandwidth it
// was given).  Here a 16x16x32 fp16 MFMA contracts 16 tokens against the (zero-padded)
// 16 head rows of the group: per 16 tokens the logits cost D/32 MFMAs instead of
// ~16 * G * (D/8 + 5) vector instructions.  Products of fp16 values are exact in fp32 and
// the accumulation is fp32, so the logits carry the same rounding as the FMA path.
//
// Operand mapping (wave64, v_mfma_f32_16x16x32_f16): lane l supplies 8 consecutive
// halfs of row (l % 16), taken from column block (l / 16); A rows are query heads, B rows
// are tokens, both read the same 8 dims [8*(l/16) + 32*kb, +8) of their row, so the
// pairing of contraction indices is the same on both sides whatever the hardware's
// internal order.  Result register r of lane l is (head 4*(l/16) + r, token l % 16).
//
// Each wavefront owns chunk/4 consecutive tokens and is independent until the end:
// logits -> LDS, per-wave softmax statistics (m_w, l_w), p -> LDS, acc_w = sum p*V with
// the row-per-16-lanes layout of the vector path (fp32 FMA: P*V needs the values
// transposed for an MFMA, which costs more than it saves at G <= 8).  One barrier, then
// the four (m_w, l_w, acc_w) are merged with the log-sum-exp rule and written as the
// chunk's partial result.
#include "sv_attend_common.h"

namespace sv {
namespace {

constexpr int kPvUnroll = 4;   // value-row loads in flight per lane

template <int D, int GB>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_mfma_kernel(const AttnArgs a, const int hblk) {
    using T = _Float16;
    constexpr int EPL = 8;
    constexpr int LPR = D / EPL;       // lanes per value row
    constexpr int RPW = kWave / LPR;   // value rows per wavefront load
    constexpr int KB = D / 32;         // MFMAs per 16-token tile
    constexpr int U = kPvUnroll;
    extern __shared__ float smem[];

    const int CH = a.chunk, CW = CH / kAttnWaves, n_tiles = CW / 16;
    const int s = blockIdx.x;
    const int g = blockIdx.y / hblk, hb = blockIdx.y % hblk;
    const int b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const TokenList tokens = token_list(a, b, unit);
    const int t0 = s * CH;
    if (t0 >= tokens.len) return;   // block-uniform

    float* s_p = smem;                          // [waves][GB][CW] logits, then softmax numerators
    float* s_acc = s_p + GB * CH;               // [waves][GB][D]
    float* s_m = s_acc + kAttnWaves * GB * D;   // [waves][GB]
    float* s_l = s_m + kAttnWaves * GB;         // [waves][GB]

    const int h_first = g * a.G + hb * (hblk > 1 ? kHeadBlock : 0);
    const int g_valid = min(GB, a.G - hb * (hblk > 1 ? kHeadBlock : 0));
    const T* ktxt = static_cast<const T*>(a.k_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh;
    const T* vtxt = static_cast<const T*>(a.v_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh;
    const T* kvis = static_cast<const T*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;
    const T* vvis = static_cast<const T*>(a.v_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;

    const int tw0 = t0 + wave * CW;             // first token of this wavefront
    float* my_p = s_p + wave * GB * CW;
    float* my_acc = s_acc + wave * GB * D;

    if (tw0 < tokens.len) {   // wave-uniform: this wavefront has at least one token
        // ---- logits: 16-token tiles on the matrix cores ----
        {
            const int row = lane & 15, kg = lane >> 4;
            half8_t qa[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                qa[kb] = 0;
                if (row < g_valid)
                    qa[kb] = *reinterpret_cast<const half8_t*>(static_cast<const T*>(a.q) + (int64_t)b * a.q_sb +
                                                               (int64_t)(h_first + row) * a.q_sh + kg * 8 + 32 * kb);
            }
            for (int tt = 0; tt < n_tiles; tt += 2) {
                half8_t kf[2][KB];
                bool valid[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int t = tw0 + (tt + j) * 16 + row;
                    valid[j] = (tt + j) < n_tiles && t < tokens.len;
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) kf[j][kb] = 0;
                    if (valid[j]) {
                        bool is_txt;
                        const int64_t off = tokens.offset(t, is_txt);
                        const T* p = (is_txt ? ktxt : kvis) + off + kg * 8;
#pragma unroll
                        for (int kb = 0; kb < KB; ++kb) kf[j][kb] = *reinterpret_cast<const half8_t*>(p + 32 * kb);
                    }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[kb], kf[j][kb], acc, 0, 0, 0);
                    if ((tt + j) < n_tiles) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int h = 4 * kg + r;
                            if (h < GB) my_p[h * CW + (tt + j) * 16 + row] = valid[j] ? acc[r] * a.scale : -INFINITY;
                        }
                    }
                }
            }
        }
        // ---- per-wave softmax statistics; LDS traffic of one wavefront stays in program order ----
        __builtin_amdgcn_wave_barrier();
        for (int h = 0; h < GB; ++h) {
            float m = -INFINITY;
            for (int i = lane; i < CW; i += kWave) m = fmaxf(m, my_p[h * CW + i]);
            m = wave_max(m);
            float l = 0.f;
            for (int i = lane; i < CW; i += kWave) {
                const float p = __expf(my_p[h * CW + i] - m);
                my_p[h * CW + i] = p;
                l += p;
            }
            l = wave_sum(l);
            if (lane == 0) { s_m[wave * GB + h] = m; s_l[wave * GB + h] = l; }
        }
        __builtin_amdgcn_wave_barrier();
        // ---- weighted sum of value rows ----
        {
            const int c = lane % LPR, grp = lane / LPR;
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
                    const int tl = st + u * RPW + grp;
                    const int t = tw0 + tl;
                    valid[u] = tl < CW && t < tokens.len;
                    vc[u] = zero_chunk<T>();
                    if (valid[u]) {
                        bool is_txt;
                        const int64_t off = tokens.offset(t, is_txt);
                        vc[u] = load_chunk((is_txt ? vtxt : vvis) + off + c * EPL);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!valid[u]) continue;
                    const int tl = st + u * RPW + grp;
#pragma unroll
                    for (int h = 0; h < GB; ++h) {
                        const float p = my_p[h * CW + tl];
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
                    for (int i = 0; i < EPL; ++i) my_acc[h * D + c * EPL + i] = acc[h][i];
            }
        }
    } else {
        for (int i = lane; i < GB * D; i += kWave) my_acc[i] = 0.f;
        if (lane < GB) { s_m[wave * GB + lane] = -INFINITY; s_l[wave * GB + lane] = 0.f; }
    }
    __syncthreads();

    // ---- merge the four wavefronts: one partial result per (head, chunk) ----
    const int S = a.n_chunks;
    for (int o = threadIdx.x; o < GB * D; o += kAttnThreads) {
        const int h = o / D, d = o % D;
        if (h >= g_valid) continue;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) m = fmaxf(m, s_m[w * GB + h]);
        float x = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            const float mw = s_m[w * GB + h];
            const float e = mw == -INFINITY ? 0.f : __expf(mw - m);
            x = fmaf(e, s_acc[(w * GB + h) * D + d], x);
            l = fmaf(e, s_l[w * GB + h], l);
        }
        const int64_t ph = ((int64_t)b * a.Hq + h_first + h) * S + s;
        a.part_acc[ph * D + d] = x;
        if (d == 0) { a.part_ml[ph * 2] = m; a.part_ml[ph * 2 + 1] = l; }
    }
}

template <int D, int GB>
hipError_t launch_one(const AttnArgs& a, int hblk, hipStream_t stream) {
    dim3 grid((unsigned)a.n_chunks, (unsigned)(a.Hkv * hblk), (unsigned)a.B), block(kAttnThreads);
    const size_t lds = sizeof(float) * ((size_t)GB * a.chunk + (size_t)kAttnWaves * GB * D + 2 * kAttnWaves * GB);
    hipLaunchKernelGGL((attn_partial_mfma_kernel<D, GB>), grid, block, lds, stream, a, hblk);
    return hipGetLastError();
}

template <int D>
hipError_t launch_dim(const AttnArgs& a, hipStream_t stream) {
    const int G = a.G;
    if (G == 1) return launch_one<D, 1>(a, 1, stream);
    if (G == 2) return launch_one<D, 2>(a, 1, stream);
    if (G <= 4) return launch_one<D, 4>(a, 1, stream);
    if (G == 7) return launch_one<D, 7>(a, 1, stream);
    if (G <= 8) return launch_one<D, 8>(a, 1, stream);
    return launch_one<D, 8>(a, (G + kHeadBlock - 1) / kHeadBlock, stream);
}

}  // namespace

hipError_t launch_attn_partial_mfma(const AttnArgs& a, hipStream_t stream) {
    if (a.D == 128) return launch_dim<128>(a, stream);
    if (a.D == 64) return launch_dim<64>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace sv
