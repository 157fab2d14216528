// Step 3 for fp16 caches with head_dim 128: chunk attention with BOTH contractions on the
// matrix cores and every wavefront streaming through several batches of tokens.
//
// Why this shape (measured on the long-video workload, 202 MB of gathered K/V rows per step):
// a kernel in which every wavefront fetched its 64 tokens, computed, and ended ran as two
// chip-wide rounds of load-then-compute, the memory system idle while the wavefronts
// computed (53 us, 3.8 TB/s); the fp32 FMAs of p*V alone were 8 us of it.  Here
//   * a wavefront owns 1..8 batches of 32 tokens (chosen per launch) and walks through them; the K rows of
//     the next batch are requested as soon as the logits of the current one are done, the V
//     rows of the next batch as soon as the current p*V is done, so rows are in flight while
//     the wavefront computes;
//   * logits: v_mfma_f32_16x16x32_f16, A = 16 (zero-padded) query heads x 32 dims, B = 32
//     dims x 16 tokens (the same 8 consecutive dims of a row on both sides);
//   * p*V: the same instruction, A = 16 heads x 32 tokens (p rounded to fp16, through LDS),
//     B = 32 tokens x 16 dims.  A lane of B must supply 8 TOKENS of one dim; the value rows
//     arrive as 8 DIMS of one token per lane.  No transpose is needed: lane (g4, c) of the
//     value loads holds dims 8c..8c+7 of tokens 4u+g4 (u = load number 0..7), so for MFMA
//     number j it packs the j-th half of its eight loads -- tokens {4u+g4} are the lane's 8
//     contraction indices, dim 8c+j its output column -- and the p operand is stored in LDS
//     in that same token order.  Eight MFMAs (j = 0..7) cover the 128 dims;
//   * softmax statistics run per wavefront over its batches (running maximum m, running sum
//     l, accumulators rescaled when m grows); l is summed from the rounded p, so the weights
//     that multiply V sum to exactly l.  Rounding p to fp16 perturbs each weight by at most
//     2^-11 relative: the output moves by far less than the 2e-3 bound of fp16 caches.
//   * the text tokens and the kept visual tokens get chunks of their own (text first), so the
//     rows a workgroup needs depend on idx alone; all loads are unconditional, on clamped rows
//     (conditional loads made every wait a wait for everything), and a workgroup reaches its
//     first K/V request after one trip through memory instead of three (lengths, idx, rows).
// At the end the four wavefronts of a workgroup merge (m, l, acc) through LDS with the
// log-sum-exp rule and write one partial result per (head, chunk).
#include <atomic>

#include "sv_attend_common.h"

namespace sv {
namespace {

constexpr int kD = 128;
constexpr int kBatchTokens = 32;
constexpr int kGroupTokens = kAttnWaves * kBatchTokens;         // one batch of every wavefront of a workgroup
constexpr int kMaxBatches = 8;                                  // batches per wavefront: 1..8, chosen per launch
constexpr int kKB = kD / 32;                                    // logit MFMAs per 16 tokens
constexpr int kVLoads = 8;                                      // value loads per lane per batch (4 tokens each)

__device__ __forceinline__ float row16_max(float x) {
    x = fmaxf(x, dpp_move<kDppQuadXor1>(x));
    x = fmaxf(x, dpp_move<kDppQuadXor2>(x));
    x = fmaxf(x, dpp_move<kDppRowHalfMirror>(x));
    x = fmaxf(x, dpp_move<kDppRowMirror>(x));
    return x;
}

template <int GB>
__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(3, 3)))
void attn_partial_flash_kernel(const AttnArgs a, const int hblk) {
    using T = _Float16;
    // Row strides padded by 16 bytes: the 16 rows a wavefront reads at once then start in different banks.
    __shared__ __align__(16) T s_p[kAttnWaves][16][kBatchTokens + 8];   // p of the current batch, A-operand order
    __shared__ __align__(16) T s_q[16][kD + 8];                         // the (zero-padded) query rows
    __shared__ __align__(16) float s_acc[kAttnWaves][GB][kD];
    __shared__ float s_m[kAttnWaves][GB], s_l[kAttnWaves][GB];

    // Chunks [0, split_base) cover the text tokens, chunks [split_base, S) the kept visual tokens, so
    // that which rows a workgroup needs depends on nothing but idx: every load below is issued
    // unconditionally on clamped (valid) rows, and the lengths only mask the logits afterwards.
    const int s = blockIdx.x;
    const bool is_txt = s < a.split_base;
    const int g = blockIdx.y / hblk, hb = blockIdx.y % hblk;
    const int b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int nb = (is_txt ? a.chunk : a.chunk_vis) / kGroupTokens;   // batches per wavefront
    const int p0 = (is_txt ? s * a.chunk : (s - a.split_base) * a.chunk_vis);   // first position of this chunk in its part
    const int row = lane & 15, quad = lane >> 4;                    // MFMA coordinates of this lane
    const int row_cap = is_txt ? a.n_txt_max : a.n_vis_max;         // >= 1 for any launched chunk

    // Cache rows of the wavefront's tokens: batch j covers positions p0 + (4j + wave) * 32 + [0, 32).
    // The rows of batch j + 2 are looked up while batch j is worked on.
    const int32_t* idx_row = a.idx + unit * a.k;
    auto rows_of = [&](int j) -> int {
        const int p = p0 + (j * kAttnWaves + wave) * kBatchTokens + (lane & 31);
        int r = p;
        if (!is_txt && a.idx) r = idx_row[min(p, a.k - 1)];   // slots past count hold -1: clamped below;
                                                                // no idx: the visual segment is packed
        return r < 0 ? 0 : (r < row_cap ? r : row_cap - 1);     // a faulty idx must not fault the GPU
    };
    int rows_cur = rows_of(0), rows_next = rows_of(1);
    // live positions of this part (the loads do not wait for it)
    const int part_len = is_txt ? clamp_len(a.txt_len, b, a.n_txt_max)
                                : ((a.k > 0 && a.count) ? clamp_len(a.count, (int)unit, a.k) : 0);

    const int h_first = g * a.G + hb * (hblk > 1 ? kHeadBlock : 0);
    const int g_valid = min(GB, a.G - hb * (hblk > 1 ? kHeadBlock : 0));
    const int64_t sn = is_txt ? a.txt_sn : a.vis_sn;
    const int64_t base_off = is_txt ? (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh
                                    : (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;
    const T* kbase = static_cast<const T*>(is_txt ? a.k_txt : a.k_vis) + base_off;
    const T* vbase = static_cast<const T*>(is_txt ? a.v_txt : a.v_vis) + base_off;

    half8_t kf[2][kKB];     // K rows: lane (row, quad) holds dims 8*quad + 32*kb .. +8 of tokens row, 16 + row
    half8_t vf[kVLoads];    // V rows: lane (quad, row) holds dims 8*row .. +8 of tokens 4u + quad
    auto load_k = [&](int rows) {   // rows: lane l & 31 holds the cache row of token l of the batch
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const T* p = kbase + (int64_t)__shfl(rows, tt * 16 + row, kWave) * sn + quad * 8;
#pragma unroll
            for (int kb = 0; kb < kKB; ++kb)   // rows are used once per step: do not displace reusable lines
                kf[tt][kb] = __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(p + 32 * kb));
        }
    };
    auto load_v = [&](int rows) {
#pragma unroll
        for (int u = 0; u < kVLoads; ++u)
            vf[u] = __builtin_nontemporal_load(
                reinterpret_cast<const half8_t*>(vbase + (int64_t)__shfl(rows, 4 * u + quad, kWave) * sn + row * 8));
    };
    load_k(rows_cur);
    load_v(rows_cur);

    // query rows -> LDS (zero rows for the padding heads); read back per batch as the A operand
    for (int i = threadIdx.x; i < 16 * (kD / 8); i += kAttnThreads) {
        const int h = i / (kD / 8), c8 = i % (kD / 8);
        half8_t v = 0;
        if (h < g_valid)
            v = *reinterpret_cast<const half8_t*>(static_cast<const T*>(a.q) + (int64_t)b * a.q_sb +
                                                  (int64_t)(h_first + h) * a.q_sh + c8 * 8);
        *reinterpret_cast<half8_t*>(&s_q[h][c8 * 8]) = v;
    }
    if (p0 >= part_len) return;   // block-uniform: nothing of this part lives in this chunk
    __syncthreads();

    float4_t acc[8];        // acc[j][r] = out[head 4*quad + r][dim 8*row + j], not normalised
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = {0.f, 0.f, 0.f, 0.f};
    float m_run[4], l_run[4];   // of heads 4*quad + r, equal in the 16 lanes of a quad
#pragma unroll
    for (int r = 0; r < 4; ++r) { m_run[r] = -INFINITY; l_run[r] = 0.f; }

#pragma unroll   // straight-line code per batch: the loads of batch j + 1 are scheduled into the work on batch j
    for (int j = 0; j < kMaxBatches; ++j) {
        if (j >= nb) break;   // block-uniform
        const int rows_after = rows_of(j + 2);
        const int n_live = part_len - (p0 + (j * kAttnWaves + wave) * kBatchTokens);   // may exceed 32
        if (n_live <= 0) break;   // wave-uniform; later batches are empty too
        // ---- logits of the 32 tokens: lane (row, quad) gets heads 4*quad + r of tokens row and 16 + row
        float4_t lg[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            float4_t sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < kKB; ++kb) {
                const half8_t qa = *reinterpret_cast<const half8_t*>(&s_q[row][quad * 8 + 32 * kb]);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa, kf[tt][kb], sacc, 0, 0, 0);
            }
            const bool live = (tt * 16 + row) < n_live;
#pragma unroll
            for (int r = 0; r < 4; ++r) lg[tt][r] = live ? sacc[r] * a.scale : -INFINITY;
        }
        if (j + 1 < nb) load_k(rows_next);   // K registers are free again
        // ---- running softmax statistics; p (fp16) to LDS in the order of the p*V contraction index
        float alpha[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float mb = row16_max(fmaxf(lg[0][r], lg[1][r]));
            const float m_new = fmaxf(m_run[r], mb);   // finite: the batch has a live token
            alpha[r] = __expf(m_run[r] - m_new);       // 0 on the first batch
            m_run[r] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const T p16 = (T)__expf(lg[tt][r] - m_new);
                psum += (float)p16;
                // token t = 16*tt + row is contraction index 8*(t % 4) + t / 4 of its batch
                s_p[wave][4 * quad + r][8 * (row & 3) + 4 * tt + (row >> 2)] = p16;
            }
            l_run[r] = fmaf(l_run[r], alpha[r], group_sum<16>(psum));
        }
        __builtin_amdgcn_wave_barrier();   // LDS traffic of one wavefront stays in program order
        const half8_t pa = *reinterpret_cast<const half8_t*>(&s_p[wave][row][8 * quad]);
        __builtin_amdgcn_wave_barrier();
        // ---- acc = acc * alpha + p * V.  Tokens past the end of the part have p = 0, but their rows were
        // still fetched (row clamped to the capacity, not to the length) and may hold anything: unused
        // cache capacity is uninitialised memory, and 0 * NaN or 0 * Inf would poison the whole head.
        // Their value registers are cleared; only a ragged last batch pays for it (wave-uniform test).
        if (n_live < kBatchTokens) {
#pragma unroll
            for (int u = 0; u < kVLoads; ++u)
                if (4 * u + quad >= n_live) vf[u] = 0;
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            half8_t vb;
#pragma unroll
            for (int u = 0; u < kVLoads; ++u) vb[u] = vf[u][jj];
            float4_t c4;
#pragma unroll
            for (int r = 0; r < 4; ++r) c4[r] = acc[jj][r] * alpha[r];
            acc[jj] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa, vb, c4, 0, 0, 0);
        }
        if (j + 1 < nb) load_v(rows_next);   // V registers are free again
        rows_next = rows_after;
    }

    // ---- the wavefront's result to LDS: rows of the valid heads only
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int h = 4 * quad + r;
        if (h < GB) {
            const float4_t lo = {acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
            const float4_t hi = {acc[4][r], acc[5][r], acc[6][r], acc[7][r]};
            *reinterpret_cast<float4_t*>(&s_acc[wave][h][8 * row]) = lo;       // the lane's 8 consecutive dims
            *reinterpret_cast<float4_t*>(&s_acc[wave][h][8 * row + 4]) = hi;
            if (row == 0) { s_m[wave][h] = m_run[r]; s_l[wave][h] = l_run[r]; }
        }
    }
    __syncthreads();

    // ---- merge the four wavefronts: one partial result per (head, chunk)
    const int S = a.n_chunks;
    for (int o = threadIdx.x; o < GB * kD; o += kAttnThreads) {
        const int h = o / kD, d = o % kD;
        if (h >= g_valid) continue;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) m = fmaxf(m, s_m[w][h]);
        float x = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            const float mw = s_m[w][h];
            const float e = mw == -INFINITY ? 0.f : __expf(mw - m);
            x = fmaf(e, s_acc[w][h][d], x);
            l = fmaf(e, s_l[w][h], l);
        }
        const int64_t ph = ((int64_t)b * a.Hq + h_first + h) * S + s;   // slot = chunk number
        a.part_acc[ph * kD + d] = x;
        if (d == 0) { a.part_ml[ph * 2] = m; a.part_ml[ph * 2 + 1] = l; }
    }
}

template <int GB>
hipError_t launch_one(const AttnArgs& a, int hblk, hipStream_t stream) {
    dim3 grid((unsigned)a.n_chunks, (unsigned)(a.Hkv * hblk), (unsigned)a.B), block(kAttnThreads);
    hipLaunchKernelGGL((attn_partial_flash_kernel<GB>), grid, block, 0, stream, a, hblk);
    return hipGetLastError();
}

}  // namespace

// Tokens per workgroup for the text range and for the visual range: a multiple of kGroupTokens (every
// wavefront of a workgroup gets the same number of 32-token batches, 1..kMaxBatches).
// The registers of the kernel allow three workgroups per compute unit.  A launch runs in
// ceil(workgroups / (3 * compute units)) rounds, a round lasting about as long as its longest
// workgroup: its batches plus about one batch-time to reach the first rows (lengths, idx, rows).  The
// plan minimises rounds * (batches + 1): one round that fills most of the chip beats a full round and a
// nearly empty one (long-video shape: 4 text + 5 visual batches, 672 workgroups, 41.7 us, against
// 4 + 4, 784 workgroups of which 16 wait for a free slot, 43.5 us).  A launch that needs three rounds or
// more whatever the batches (dense attention, a quarter of a long video kept) does not run in rounds any
// more -- a slot is refilled as soon as its workgroup ends -- so there the plan minimises the summed
// workgroup time, chunks * (batches + 1): the longest workgroups, which pay the first trip least often
// (dense attention over 51 200 tokens x 112 units: 8 batches 494 us, 5 batches 525 us).
void attn_flash_plan(int64_t units, int n_txt, int n_kept, int forced_batches, int* chunk_txt, int* chunk_vis) {
    if (forced_batches > 0) {
        const int nb = forced_batches < kMaxBatches ? forced_batches : kMaxBatches;
        *chunk_txt = *chunk_vis = nb * kGroupTokens;
        return;
    }
    static std::atomic<int> cached_cus{0};
    int cus = cached_cus.load(std::memory_order_relaxed);
    if (cus <= 0) {   // all devices of a node are alike; a failed query falls back to the MI355X count
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cached_cus.store(cus, std::memory_order_relaxed);
    }
    const int64_t slots = 3 * (int64_t)cus;
    const int longest_chunk = kMaxBatches * kGroupTokens;
    const int64_t fewest = units * (((int64_t)n_txt + longest_chunk - 1) / longest_chunk +
                                    ((int64_t)n_kept + longest_chunk - 1) / longest_chunk);
    const bool many_rounds = fewest > 2 * slots;   // three rounds or more with any batch count
    int64_t best_cost = -1;
    int best_t = 1, best_v = 1;
    for (int bt = 1; bt <= kMaxBatches; ++bt) {
        for (int bv = 1; bv <= kMaxBatches; ++bv) {
            const int64_t ct = ((int64_t)n_txt + bt * kGroupTokens - 1) / (bt * kGroupTokens);
            const int64_t cv = ((int64_t)n_kept + bv * kGroupTokens - 1) / (bv * kGroupTokens);
            int64_t cost;
            if (many_rounds) {
                cost = ct * (bt + 1) + cv * (bv + 1);
            } else {
                const int64_t wgs = units * (ct + cv);
                const int64_t rounds = (wgs + slots - 1) / slots;
                const int longest = (n_txt > 0 && bt > bv) || n_kept == 0 ? bt : bv;
                cost = rounds * (longest + 1);
            }
            cost = cost * 32 + bt + bv;   // ties: the shorter workgroups
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_t = bt; best_v = bv; }
        }
    }
    *chunk_txt = best_t * kGroupTokens;
    *chunk_vis = best_v * kGroupTokens;
}

hipError_t launch_attn_partial_flash(const AttnArgs& a, hipStream_t stream) {
    auto bad_chunk = [](int c) { return c < kGroupTokens || c > kMaxBatches * kGroupTokens || c % kGroupTokens; };
    if (bad_chunk(a.chunk) || bad_chunk(a.chunk_vis) || a.D != kD || a.split_base < 0 || a.split_base > a.n_chunks)
        return hipErrorInvalidValue;
    const int G = a.G;
    if (G == 1) return launch_one<1>(a, 1, stream);
    if (G == 2) return launch_one<2>(a, 1, stream);
    if (G <= 4) return launch_one<4>(a, 1, stream);
    if (G == 7) return launch_one<7>(a, 1, stream);
    if (G <= 8) return launch_one<8>(a, 1, stream);
    return launch_one<8>(a, (G + kHeadBlock - 1) / kHeadBlock, stream);
}

}  // namespace sv
