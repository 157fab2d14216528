// Step 3 for fp16 caches: chunk attention with the logits on the matrix cores.
//
// Two measurements shaped this kernel.  (1) The vector path spends 8 FMAs plus a lane
// reduction per (16-byte key chunk, head); with a GQA group of 7 heads it was ALU-bound
// at a third of the bandwidth it was given.  A 16x16x32 fp16 MFMA contracts 16 tokens
// against the (zero-padded) 16 head rows of the group, D/32 instructions per 16 tokens.
// Products of fp16 values are exact in fp32 and the accumulation is fp32, so the logits
// carry the same rounding as the FMA path.  (2) A dependent trip through memory costs
// microseconds, far more than the arithmetic of a chunk, so a wavefront makes exactly two:
// one for the indices of its 64 tokens, one for ALL their K rows and V rows (32 KiB in
// flight per wavefront, held in registers), instead of idx -> K -> idx -> V per few rows.
//
// Operand mapping (wave64, v_mfma_f32_16x16x32_f16): lane l supplies 8 consecutive
// halfs of row (l % 16), taken from column block (l / 16); A rows are query heads, B rows
// are tokens, both read the same 8 dims [8*(l/16) + 32*kb, +8) of their row, so the
// pairing of contraction indices is the same on both sides whatever the hardware's
// internal order.  Result register r of lane l is (head 4*(l/16) + r, token l % 16).
//
// A wavefront owns 64 consecutive tokens of T and is independent until the end: logits
// stay in registers, the softmax statistics (m_w, l_w) come from DPP reductions inside
// the 16-lane rows, p goes through LDS to the row-per-lane-group layout in which
// acc_w = sum p*V is accumulated with fp32 FMAs (P*V on the matrix cores would need the
// values transposed, which costs more than it saves at G <= 8).  One barrier, then the
// four (m_w, l_w, acc_w) of a workgroup are merged with the log-sum-exp rule and written
// as the chunk's partial result.
#include "sv_attend_common.h"

namespace sv {
namespace {

#ifndef SV_ATTN_TOK
#define SV_ATTN_TOK 64
#endif
#ifndef SV_ATTN_NW
#define SV_ATTN_NW 4
#endif
constexpr int kWaveTokens = SV_ATTN_TOK;                 // tokens per wavefront
constexpr int kTiles = kWaveTokens / 16;                 // MFMA token tiles per wavefront
constexpr int kNW = SV_ATTN_NW;                          // wavefronts per workgroup
constexpr int kNT = kNW * kWave;

__device__ __forceinline__ float row16_max(float x) {
    x = fmaxf(x, dpp_move<kDppQuadXor1>(x));
    x = fmaxf(x, dpp_move<kDppQuadXor2>(x));
    x = fmaxf(x, dpp_move<kDppRowHalfMirror>(x));
    x = fmaxf(x, dpp_move<kDppRowMirror>(x));
    return x;
}

template <int D, int GB>
__global__ __launch_bounds__(kNT) void attn_partial_mfma_kernel(const AttnArgs a, const int hblk) {
    using T = _Float16;
    constexpr int EPL = 8;
    constexpr int LPR = D / EPL;                 // lanes per value row
    constexpr int RPW = kWave / LPR;             // value rows per wavefront load
    constexpr int VSTEPS = kWaveTokens / RPW;    // value loads per lane
    constexpr int KB = D / 32;                   // MFMAs per 16-token tile
    constexpr int CH = kNW * kWaveTokens;
    __shared__ float s_p[kNW][GB][kWaveTokens];
    __shared__ float s_acc[kNW][GB][D];
    __shared__ float s_m[kNW][GB], s_l[kNW][GB];

    const int s = blockIdx.x;
    const int g = blockIdx.y / hblk, hb = blockIdx.y % hblk;
    const int b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const TokenList tokens = token_list(a, b, unit);
    const int t0 = s * CH;
    if (t0 >= tokens.len) return;   // block-uniform

    const int h_first = g * a.G + hb * (hblk > 1 ? kHeadBlock : 0);
    const int g_valid = min(GB, a.G - hb * (hblk > 1 ? kHeadBlock : 0));
    const T* ktxt = static_cast<const T*>(a.k_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh;
    const T* vtxt = static_cast<const T*>(a.v_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh;
    const T* kvis = static_cast<const T*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;
    const T* vvis = static_cast<const T*>(a.v_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;
    const int tw0 = t0 + wave * kWaveTokens;   // first token of this wavefront

    if (tw0 < tokens.len) {   // wave-uniform: this wavefront has at least one token
        // ---- round trip 1: where does each of the 64 tokens live?  >= 0: text row, < 0: -(visual row) - 1
        int my_code = 0;
        {
            const int t = tw0 + lane;
            if (t < tokens.len) {
                if (t < tokens.nt) {
                    my_code = t;
                } else {
                    int j = tokens.idx_row ? tokens.idx_row[t - tokens.nt] : t - tokens.nt;
                    j = j < 0 ? 0 : (j < a.n_vis_max ? j : a.n_vis_max - 1);   // a faulty idx must not fault the GPU
                    my_code = -j - 1;
                }
            }
        }
        const int n_live = min(kWaveTokens, tokens.len - tw0);   // live tokens of this wavefront
        auto row_ptr = [&](int code, const T* txt, const T* vis) -> const T* {
            return code >= 0 ? txt + (int64_t)code * a.txt_sn : vis + (int64_t)(-code - 1) * a.vis_sn;
        };

        // ---- round trip 2: every K row and V row of the wavefront ----
        const int row = lane & 15, kg = lane >> 4;
        half8_t qa[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            qa[kb] = 0;
            if (row < g_valid)
                qa[kb] = *reinterpret_cast<const half8_t*>(static_cast<const T*>(a.q) + (int64_t)b * a.q_sb +
                                                           (int64_t)(h_first + row) * a.q_sh + kg * 8 + 32 * kb);
        }
        half8_t kf[kTiles][KB];
#pragma unroll
        for (int tt = 0; tt < kTiles; ++tt) {
            const int tl = tt * 16 + row;
            const int code = __shfl(my_code, tl, kWave);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) kf[tt][kb] = 0;
            if (tl < n_live) {
                const T* p = row_ptr(code, ktxt, kvis) + kg * 8;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) kf[tt][kb] = *reinterpret_cast<const half8_t*>(p + 32 * kb);
            }
        }
        const int c = lane % LPR, grp = lane / LPR;
        // the first half of the V rows rides along with the K rows; the second half is issued
        // once the MFMAs have released the K registers (keeps the kernel at 3 wavefronts per SIMD)
        constexpr int VH = VSTEPS / 2;
        Chunk<T> vc[VSTEPS];
#pragma unroll
        for (int u = 0; u < VH; ++u) {
            const int tl = u * RPW + grp;
            const int code = __shfl(my_code, tl, kWave);
            vc[u] = zero_chunk<T>();
            if (tl < n_live) vc[u] = load_chunk(row_ptr(code, vtxt, vvis) + c * EPL);
        }

        // ---- logits on the matrix cores; lane (row, kg) holds heads 4*kg..4*kg+3 of token tt*16+row ----
        float4_t lg[kTiles];
#pragma unroll
        for (int tt = 0; tt < kTiles; ++tt) {
            float4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[kb], kf[tt][kb], acc, 0, 0, 0);
            const bool live = (tt * 16 + row) < n_live;
#pragma unroll
            for (int r = 0; r < 4; ++r) lg[tt][r] = live ? acc[r] * a.scale : -INFINITY;
        }
#pragma unroll
        for (int u = VH; u < VSTEPS; ++u) {
            const int tl = u * RPW + grp;
            const int code = __shfl(my_code, tl, kWave);
            vc[u] = zero_chunk<T>();
            if (tl < n_live) vc[u] = load_chunk(row_ptr(code, vtxt, vvis) + c * EPL);
        }
        // ---- softmax statistics of the wavefront's 64 tokens, per head, inside the 16-lane rows ----
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float m = lg[0][r];
#pragma unroll
            for (int tt = 1; tt < kTiles; ++tt) m = fmaxf(m, lg[tt][r]);
            m = row16_max(m);
            float l = 0.f;
#pragma unroll
            for (int tt = 0; tt < kTiles; ++tt) {
                const float p = __expf(lg[tt][r] - m);
                lg[tt][r] = p;
                l += p;
            }
            l = group_sum<16>(l);
            const int h = 4 * kg + r;
            if (h < GB) {
#pragma unroll
                for (int tt = 0; tt < kTiles; ++tt) s_p[wave][h][tt * 16 + row] = lg[tt][r];
                if (row == 0) { s_m[wave][h] = m; s_l[wave][h] = l; }
            }
        }
        __builtin_amdgcn_wave_barrier();   // LDS traffic of one wavefront stays in program order

        // ---- weighted sum of value rows: lane group grp holds token u*RPW+grp, lane c its dims ----
        float acc[GB][EPL];
#pragma unroll
        for (int h = 0; h < GB; ++h)
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[h][i] = 0.f;
#pragma unroll
        for (int u = 0; u < VSTEPS; ++u) {
            const int tl = u * RPW + grp;
#pragma unroll
            for (int h = 0; h < GB; ++h) {
                const float p = s_p[wave][h][tl];   // 0 for tokens past the end
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc[h][i] = fmaf(p, vc[u].at(i), acc[h][i]);
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
                for (int i = 0; i < EPL; ++i) s_acc[wave][h][c * EPL + i] = acc[h][i];
        }
    } else {
        for (int i = lane; i < GB * D; i += kWave) (&s_acc[wave][0][0])[i] = 0.f;
        if (lane < GB) { s_m[wave][lane] = -INFINITY; s_l[wave][lane] = 0.f; }
    }
    __syncthreads();

    // ---- merge the four wavefronts: one partial result per (head, chunk) ----
    const int S = a.n_chunks;
    for (int o = threadIdx.x; o < GB * D; o += kNT) {
        const int h = o / D, d = o % D;
        if (h >= g_valid) continue;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < kNW; ++w) m = fmaxf(m, s_m[w][h]);
        float x = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kNW; ++w) {
            const float mw = s_m[w][h];
            const float e = mw == -INFINITY ? 0.f : __expf(mw - m);
            x = fmaf(e, s_acc[w][h][d], x);
            l = fmaf(e, s_l[w][h], l);
        }
        const int64_t ph = ((int64_t)b * a.Hq + h_first + h) * S + s;
        a.part_acc[ph * D + d] = x;
        if (d == 0) { a.part_ml[ph * 2] = m; a.part_ml[ph * 2 + 1] = l; }
    }
}

template <int D, int GB>
hipError_t launch_one(const AttnArgs& a, int hblk, hipStream_t stream) {
    dim3 grid((unsigned)a.n_chunks, (unsigned)(a.Hkv * hblk), (unsigned)a.B), block(kNT);
    hipLaunchKernelGGL((attn_partial_mfma_kernel<D, GB>), grid, block, 0, stream, a, hblk);
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

int attn_mfma_chunk() { return kNW * kWaveTokens; }

hipError_t launch_attn_partial_mfma(const AttnArgs& a, hipStream_t stream) {
    if (a.D == 128) return launch_attn_partial_flash(a, stream);
    if (a.chunk != kNW * kWaveTokens) return hipErrorInvalidValue;
    if (a.D == 64) return launch_dim<64>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace sv
