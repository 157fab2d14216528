// Query-agnostic salience of the tokens of a vision-encoder layer (section 3.1, "Token Salience
// Estimation": for encoders without a summary token, importance is the intra-visual attention averaged
// over all tokens; "Efficient Implementation": softmax normalisation and salience accumulation are
// streamed, the attention matrix is never formed):
//
//   salience[b, j] = 1 / (H n_b) * sum_h sum_{i < n_b} softmax_row(i, h)[j],
//
// where row (i, h) is token i's query of head h and its softmax runs over the keys of all n_b live tokens.
//
// Two passes, both with the logits on the matrix cores (v_mfma_f32_16x16x32_f16) and the streamed
// operand staged through LDS 64 rows at a time (one barrier per stage, the next stage fetched into
// registers while the current one is used):
//   pass 1 (salience_rowstat_kernel)  a workgroup holds 256 query rows in registers and streams a block of
//          keys: per query row the sum of exponentials relative to a reference (one per wavefront on the fast
//          path, one per row on the exact path);
//          salience_lse_kernel merges the key blocks into lse[b, i, h];
//   pass 2 (salience_colsum_kernel)   the roles are swapped: a workgroup holds 256 KEYS in registers (as
//          the A operand) and streams a segment of the query tokens, each with its lse: the tile is
//          K Q^T, a lane adds 2^(logit - lse of its query column) into the accumulators of its key rows --
//          one multiply-add, one exponential and one add per (query, key) -- and the 16 lanes of a key
//          row are merged once at the end; salience_finish_kernel adds the query segments and the heads
//          in a fixed order and divides by H n_b.
// Both passes cost one contraction and one exponential per (query, key, head): bound by the
// exponential and matrix pipes; Q and K (N * H * D * 2 bytes each) are re-read N / 256 times, from
// the caches.
#include <type_traits>

#include "sv_kernels.h"
#include "sv_mass_device.h"

namespace sv {
namespace {

constexpr int kRowsPerGroup = kMaxRowTiles * 16;   // 256 rows held in registers by one workgroup

// A 16-row tile of the operand kept in registers: lane (row, quad) supplies dims 8*quad + 32*kb .. +8 of
// row `r`; plain (cached) loads, every row is read again by other workgroups.
template <int KB>
__device__ __forceinline__ void load_row(const _Float16* base, int64_t stride, int r, int quad, half8_t (&v)[KB]) {
    const _Float16* p = base + (int64_t)r * stride + quad * 8;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) v[kb] = *reinterpret_cast<const half8_t*>(p + 32 * kb);
}

// The 4 row tiles of this wavefront out of the 256 rows that start at row0; rows at or past n are zero.
template <int KB>
__device__ __forceinline__ void load_held_tiles(const _Float16* base, int64_t stride, int row0, int n, int wave, int rot,
                                                int lane, half8_t (&held)[kTilesPerWave][KB]) {
    const int row = lane & 15, quad = lane >> 4;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {   // unconditional loads on a clamped row: no load waits for a branch
        const int r = row0 + row_tile_of(wave, rot, t) * 16 + row;
        half8_t v[KB];
        load_row<KB>(base, stride, min(r, n - 1), quad, v);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) held[t][kb] = r < n ? v[kb] : half8_t(0);
    }
}

// ---- pass 1 ----
// Wavefronts per SIMD that the registers of a head dim allow without spilling: the held query tiles take D / 2
// registers, the sums of 16 rows 16, two key tiles in flight D / 4 + 32.
#define SV_ROWSTAT_W(D) ((D) <= 64 ? 4 : 3)
template <int D>
__global__ __launch_bounds__(kMassThreads) __attribute__((amdgpu_waves_per_eu(SV_ROWSTAT_W(D), SV_ROWSTAT_W(D)))) void salience_rowstat_kernel(const SalienceArgs a) {
    constexpr int KB = D / 32;
    __shared__ KeyStage<KB> stage[2];
    __shared__ int s_flag;   // zero whenever block_any is entered
    if (threadIdx.x == 0) s_flag = 0;   // the sweep below starts with a barrier
    const int blk = blockIdx.x, b = blockIdx.z;
    const int h = blockIdx.y / a.n_row_chunks, qc = blockIdx.y - h * a.n_row_chunks;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int rot = (blk + qc) & (kMassWaves - 1);
    const int n = live_len(a.vis_len, b, a.N);
    const int row0 = qc * kRowsPerGroup, key0 = blk * a.stat_block_keys;
    if (row0 >= n || key0 >= n) return;   // block-uniform; nothing downstream reads this workgroup's slots
    const int ntl = live_tiles_of(wave, rot, min(n - row0, kRowsPerGroup));   // wave-uniform
    const float c2 = a.scale * kLog2e;
    float* part = a.part + (((((int64_t)b * a.H + h) * a.n_row_chunks + qc) * a.n_stat_blocks + blk) * kRowsPerGroup) * 2;

    const _Float16* qrows = static_cast<const _Float16*>(a.q) + (int64_t)b * a.q_sb + (int64_t)h * a.q_sh;
    const _Float16* keys = static_cast<const _Float16*>(a.k) + (int64_t)b * a.k_sb + (int64_t)h * a.k_sh;
    half8_t qa[kTilesPerWave][KB];
    load_held_tiles<KB>(qrows, a.q_st, row0, n, wave, rot, lane, qa);
    float ref[kTilesPerWave][4], l[kTilesPerWave][4];
    const int k_end = min(key0 + a.stat_block_keys, n);
    half8_t kfetch[KB];
    auto fetch = [&](int s0) {   // this wavefront's key tile of the stage at s0; rows clamped, dead columns masked at use
        load_row<KB>(keys, a.k_sn, min(s0 + wave * 16 + row, n - 1), quad, kfetch);
    };
    auto put = [&](KeyStage<KB>& st) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) st.w[wave][kb][lane] = kfetch[kb];
    };
    // every tile of an exact sweep: a reference per row kept as the exact running maximum, dead columns masked
    auto masked_tile = [&](int k0, const KeyStage<KB>& st, int kt) {
        half8_t kf[KB];
        read_key_tile<KB>(st, kt, lane, kf);
        const bool seen = k0 + row < n;   // this lane's key column
#pragma unroll
        for (int t = 0; t < kTilesPerWave; ++t) {   // one row tile at a time: this path is rare and is kept light on registers
            float4_t sv = {0.f, 0.f, 0.f, 0.f};     // rows past n are zero rows: computed, never stored
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) sv = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[kb], sv, 0, 0, 0);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const float x = seen ? sv[rr] * c2 : -INFINITY;
                const float mn = fmaxf(ref[t][rr], x);
                if (mn > -INFINITY) {
                    l[t][rr] = l[t][rr] * __builtin_amdgcn_exp2f(ref[t][rr] - mn) + __builtin_amdgcn_exp2f(x - mn);
                    ref[t][rr] = mn;
                }
            }
        }
    };
    // One sweep over the key block.  On the fast path every stage, the ragged last one included, runs in one loop --
    // references from the first 16 keys, then multiply-add, exponential, add per element, dead columns masked through
    // the reference --; the exact sweep (blocks whose fast sums left the trusted range) takes the masked path for every
    // tile.  The loops are separate and instantiated once per count of live row tiles, chosen outside them:
    // a stage loop that can take either path, or a switch inside it, costs the registers that decide between two and
    // three wavefronts per SIMD.  No branch around the fetch and the store of the next stage: past the end they are
    // harmless (clamped rows, a buffer nobody reads), and conditional blocks in the body keep the scheduler from
    // placing the matrix and vector instructions of a stage together.
    auto masked_stage = [&](int s0, const KeyStage<KB>& st) {
#pragma unroll 1
        for (int kt = 0; kt < kMassWaves; ++kt)
            if (s0 + kt * 16 < k_end) masked_tile(s0 + kt * 16, st, kt);
    };
    auto start = [&]() {   // statistics cleared, the first stage in LDS
#pragma unroll
        for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                ref[t][rr] = -INFINITY;
                l[t][rr] = 0.f;
            }
        fetch(key0);
        wait_for_loads();
        put(stage[0]);
        __syncthreads();
    };
    auto run_exact = [&]() {   // one instance: the masked tiles do not depend on the count of live row tiles
        start();
        int cur = 0;
        for (int s0 = key0; s0 < k_end; s0 += kStageKeys) {
            masked_stage(s0, stage[cur]);
            fetch(s0 + kStageKeys);   // after the stage, not a stage ahead: this rare path gives the registers of
            put(stage[cur ^ 1]);      // the key tile in flight back (its spills would make the kernel use scratch)
            __syncthreads();
            cur ^= 1;
        }
    };
    auto run_fast = [&](auto ntl_c) __attribute__((always_inline)) {
        constexpr int NTL = decltype(ntl_c)::value;
        start();
        int cur = 0;
        const float ref_w = rowstat_init_ref<KB, NTL>(stage[0], lane, wave, rot, min(n - row0, kRowsPerGroup), qa, c2);   // wave-uniform
        for (int s0 = key0; s0 < k_end; s0 += kStageKeys) {   // the ragged last stage included: its dead columns add 0
            fetch(s0 + kStageKeys);
            rowstat_fast_stage<KB, NTL>(stage[cur], lane, qa, c2, ref_w, min(k_end - s0, kStageKeys), l);
            put(stage[cur ^ 1]);
            __syncthreads();
            cur ^= 1;
        }
#pragma unroll
        for (int t = 0; t < NTL; ++t)   // from here on every row carries its own reference
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) ref[t][rr] = ref_w;
    };
    auto sweep_fast = [&]() __attribute__((always_inline)) {
        switch (ntl) {   // wave-uniform
            case 4: run_fast(std::integral_constant<int, 4>{}); break;
            case 3: run_fast(std::integral_constant<int, 3>{}); break;
            case 2: run_fast(std::integral_constant<int, 2>{}); break;
            case 1: run_fast(std::integral_constant<int, 1>{}); break;
            default: run_fast(std::integral_constant<int, 0>{}); break;
        }
    };
    sweep_fast();
    // did the sum of a live row leave the range in which it is trusted (inf, NaN, huge or tiny: logits far from the
    // wavefront's reference)?
    const bool sees_a_key = row < k_end - key0;   // a block of fewer than 16 keys leaves lanes without a live column: sum 0
    bool bad = false;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const bool live_row = t < ntl && row0 + row_tile_of(wave, rot, t) * 16 + 4 * quad + rr < n;
            bad |= live_row && sees_a_key && !(l[t][rr] < kSumLimit && l[t][rr] >= 1.f / kSumLimit);
        }
    if (block_any(bad, &s_flag)) run_exact();   // block-uniform
    // merge the 16 key columns of a row, store per key block (natural-log units from here on)
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const int tile = row_tile_of(wave, rot, t);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float mine = t < ntl ? ref[t][rr] : -INFINITY;   // the fast stages leave dead tiles untouched,
            const float lmine = t < ntl ? l[t][rr] : 0.f;          // the masked ones compute them: drop both
            const float mx = row_max16(mine);
            const float e = mine > -INFINITY ? __builtin_amdgcn_exp2f(mine - mx) : 0.f;
            const float lt = group_sum<16>(lmine * e);
            if (row == 0) {
                const int r = tile * 16 + 4 * quad + rr;
                part[r * 2] = mx * kLn2;
                part[r * 2 + 1] = lt;
            }
        }
    }
}

// lse[b, i, h] = log sum over the key blocks; one thread per query token of a chunk; +inf past the live tokens.
__global__ __launch_bounds__(kRowsPerGroup) void salience_lse_kernel(const SalienceArgs a) {
    const int qc = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int r = threadIdx.x, i = qc * kRowsPerGroup + r;
    if (i >= a.N) return;
    const int n = live_len(a.vis_len, b, a.N);
    float* dst = a.lse + ((int64_t)b * a.N + i) * a.H + h;
    if (i >= n) {
        *dst = INFINITY;
        return;
    }
    const int live_blocks = (n + a.stat_block_keys - 1) / a.stat_block_keys;
    const float* part = a.part + (((((int64_t)b * a.H + h) * a.n_row_chunks + qc) * a.n_stat_blocks) * kRowsPerGroup) * 2;
    float mx = -INFINITY;
    for (int s = 0; s < live_blocks; ++s) mx = fmaxf(mx, part[((int64_t)s * kRowsPerGroup + r) * 2]);
    float sum = 0.f;
    for (int s = 0; s < live_blocks; ++s) {
        const float ms = part[((int64_t)s * kRowsPerGroup + r) * 2];
        if (ms > -INFINITY) sum += part[((int64_t)s * kRowsPerGroup + r) * 2 + 1] * expf(ms - mx);
    }
    *dst = mx + logf(sum);
}

// ---- pass 2 ----
// One stage of 64 query tokens against the key tiles this wavefront holds: lane (row, quad) gets keys
// 4*quad + rr of each key tile at query column `row`; lse2 holds the stage's 64 query normalisers in base 2
// (+inf for columns past the segment: p = 0).
template <int KB, int NTL>
__device__ __forceinline__ void colsum_swapped_stage(const KeyStage<KB>& st, const float* lse2, int lane,
                                                     const half8_t (&ka)[kTilesPerWave][KB], float c2,
                                                     float (&acc)[kTilesPerWave][4]) {
    const int row = lane & 15;
    half8_t qf[2][KB];
    float4_t sv[2][kTilesPerWave];
    read_key_tile<KB>(st, 0, lane, qf[0]);
    tile_logits<KB, NTL>(ka, qf[0], sv[0]);
    constexpr int n_m = KB * NTL, n_e = 4 * NTL;   // matrix instructions of a query tile, elements per lane of a query tile
    constexpr int NT1 = NTL > 0 ? NTL : 1, n_e1 = n_e > 0 ? n_e : 1;   // divisors that exist when a wavefront holds no live tile
    static_assert(KB <= 4, "at most one matrix instruction per element");
#pragma unroll
    for (int qt = 0; qt < kMassWaves; ++qt) {
        const int cur = qt & 1, nxt = cur ^ 1;
        const bool has_next = qt + 1 < kMassWaves;
        if (has_next) {
            read_key_tile<KB>(st, qt + 1, lane, qf[nxt]);
#pragma unroll
            for (int t = 0; t < NTL; ++t) sv[nxt][t] = {0.f, 0.f, 0.f, 0.f};
        }
        const float l2 = lse2[qt * 16 + row];
        // Instruction order: one matrix instruction of the next query tile, then the multiply-add of element e, the
        // exponential of element e - 1 and the add of element e - 2 of this tile -- a matrix instruction keeps its
        // pipe busy for as long as those vector instructions take to issue, and none of them waits for its
        // neighbour.  The fences keep the scheduler from gathering the matrix instructions in one place.
        float y[n_e1], pr[n_e1];
#pragma unroll
        for (int step = 0; step < n_e + 2; ++step) {
            if (has_next && step < n_e) {
#pragma unroll
                for (int m = step * n_m / n_e1; m < (step + 1) * n_m / n_e1; ++m) {
                    const int kb = m / NT1, t = m % NT1;
                    sv[nxt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][kb], qf[nxt][kb], sv[nxt][t], 0, 0, 0);
                }
            }
            if (step < n_e) y[step] = fmaf(sv[cur][step / 4][step % 4], c2, -l2);
            if (step >= 1 && step - 1 < n_e) pr[step - 1] = __builtin_amdgcn_exp2f(y[step - 1]);
            if (step >= 2) acc[(step - 2) / 4][(step - 2) % 4] += pr[step - 2];
            SV_STAGE_FENCE();
        }
    }
}

// Wavefronts per SIMD the register budget of a head dim allows without spilling (more of them: more chances that one
// issues vector instructions while another's matrix instruction runs).
#define SV_COLSUM_W(D) ((D) <= 64 ? 4 : 3)
template <int D>
__global__ __launch_bounds__(kMassThreads) __attribute__((amdgpu_waves_per_eu(SV_COLSUM_W(D), SV_COLSUM_W(D)))) void salience_colsum_kernel(const SalienceArgs a) {
    constexpr int KB = D / 32;
    __shared__ KeyStage<KB> stage[2];
    __shared__ float s_lse2[2][kStageKeys];
    const int kblk = blockIdx.x, b = blockIdx.z;
    const int h = blockIdx.y / a.n_seg, seg = blockIdx.y - h * a.n_seg;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int rot = (kblk + seg) & (kMassWaves - 1);
    const int n = live_len(a.vis_len, b, a.N);
    const int key0 = kblk * kRowsPerGroup, q0 = seg * a.seg_len;
    if (key0 >= n || q0 >= n) return;   // block-uniform; the finishing kernel reads neither these keys nor this segment
    const int q_end = min(q0 + a.seg_len, n);
    const int ntl = live_tiles_of(wave, rot, min(n - key0, kRowsPerGroup));   // wave-uniform
    const float c2 = a.scale * kLog2e;

    const _Float16* qrows = static_cast<const _Float16*>(a.q) + (int64_t)b * a.q_sb + (int64_t)h * a.q_sh;
    const _Float16* keys = static_cast<const _Float16*>(a.k) + (int64_t)b * a.k_sb + (int64_t)h * a.k_sh;
    const float* lse = a.lse + (int64_t)b * a.N * a.H + h;
    half8_t ka[kTilesPerWave][KB];
    load_held_tiles<KB>(keys, a.k_sn, key0, n, wave, rot, lane, ka);
    float acc[kTilesPerWave][4];
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) acc[t][rr] = 0.f;

    half8_t qfetch[KB];
    float lfetch;
    auto fetch = [&](int s0) {   // this wavefront's query tile of the stage at s0 and the normalisers of its 16 queries
        const int i = s0 + wave * 16 + row, ic = min(i, n - 1);
        load_row<KB>(qrows, a.q_st, ic, quad, qfetch);
        const float v = lse[(int64_t)ic * a.H];   // unconditional, clamped row
        lfetch = i < q_end ? v * kLog2e : INFINITY;
    };
    auto put = [&](int buf) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) stage[buf].w[wave][kb][lane] = qfetch[kb];
        s_lse2[buf][wave * 16 + row] = lfetch;   // the four quads store the same value: no divergent branch in the loop body
    };
    auto run = [&](auto ntl_c) __attribute__((always_inline)) {
        constexpr int NTL = decltype(ntl_c)::value;
        fetch(q0);
        wait_for_loads();
        put(0);
        __syncthreads();
        int cur = 0;
        for (int s0 = q0; s0 < q_end; s0 += kStageKeys) {
            // No branch inside the body: the fetch and the store of the stage after the last one are harmless (clamped
            // rows, a buffer nobody reads), and a conditional store in the middle made the compiler sink every
            // vector instruction of the stage below it, away from the matrix instructions they are to overlap with.
            fetch(s0 + kStageKeys);
            colsum_swapped_stage<KB, NTL>(stage[cur], s_lse2[cur], lane, ka, c2, acc);
            put(cur ^ 1);
            __syncthreads();
            cur ^= 1;
        }
    };
    switch (ntl) {   // wave-uniform
        case 4: run(std::integral_constant<int, 4>{}); break;
        case 3: run(std::integral_constant<int, 3>{}); break;
        case 2: run(std::integral_constant<int, 2>{}); break;
        case 1: run(std::integral_constant<int, 1>{}); break;
        default: run(std::integral_constant<int, 0>{}); break;
    }
    // the 16 lanes of a key row hold different query columns: add them, store the segment's share per key
    float* out = a.colpart + ((((int64_t)b * a.H + h) * a.n_seg + seg) * a.N);
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const int tile = row_tile_of(wave, rot, t);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float x = group_sum<16>(t < ntl ? acc[t][rr] : 0.f);
            const int key = key0 + tile * 16 + 4 * quad + rr;
            if (row == 0 && key < n) out[key] = x;
        }
    }
}

// salience[b, j] = (sum over heads and query segments, in that fixed order) / (H n_b); -inf past the live tokens.
__global__ __launch_bounds__(256) void salience_finish_kernel(const SalienceArgs a) {
    const int b = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= a.N) return;
    const int n = live_len(a.vis_len, b, a.N);
    float* dst = a.salience + (int64_t)b * a.N + j;
    if (j >= n) {
        *dst = -INFINITY;
        return;
    }
    const int live_segs = (n + a.seg_len - 1) / a.seg_len;
    float sum = 0.f;
    for (int h = 0; h < a.H; ++h)
        for (int s = 0; s < live_segs; ++s) sum += a.colpart[((((int64_t)b * a.H + h) * a.n_seg + s) * a.N) + j];
    *dst = sum / ((float)a.H * (float)n);
}

}  // namespace

SaliencePlan salience_plan(int B, int H, int N) {
    SaliencePlan p{};
    if (B < 1 || H < 1 || N < 1) return p;
    p.n_row_chunks = (N + kRowsPerGroup - 1) / kRowsPerGroup;
    // Both passes hold a group of 256 tokens in registers and stream the others in segments of one planned length.
    p.seg_len = planned_block_len((int64_t)B * H * p.n_row_chunks, N, 512);
    p.n_seg = (N + p.seg_len - 1) / p.seg_len;
    p.stat_block_keys = p.seg_len;
    p.n_stat_blocks = p.n_seg;
    p.part_bytes = (size_t)B * H * p.n_row_chunks * p.n_stat_blocks * kRowsPerGroup * 2 * sizeof(float);
    p.colpart_bytes = (size_t)B * H * p.n_seg * N * sizeof(float);
    return p;
}

hipError_t launch_salience(const SalienceArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.N == 0) return hipSuccess;
    const SaliencePlan p = salience_plan(a.B, a.H, a.N);
    SalienceArgs k = a;
    k.n_row_chunks = p.n_row_chunks; k.stat_block_keys = p.stat_block_keys; k.n_stat_blocks = p.n_stat_blocks;
    k.seg_len = p.seg_len; k.n_seg = p.n_seg;
    if ((int64_t)a.H * p.n_row_chunks > 65535 || (int64_t)a.H * p.n_seg > 65535 || a.B > 65535) return hipErrorInvalidValue;
    const dim3 block(kMassThreads);
    const dim3 grid1((unsigned)p.n_stat_blocks, (unsigned)(a.H * p.n_row_chunks), (unsigned)a.B);
    const dim3 grid2((unsigned)p.n_row_chunks, (unsigned)a.H, (unsigned)a.B);
    const dim3 grid3((unsigned)p.n_row_chunks, (unsigned)(a.H * p.n_seg), (unsigned)a.B);
    const dim3 grid4((unsigned)((a.N + 255) / 256), (unsigned)a.B);
    switch (a.D) {
        case 128:
            hipLaunchKernelGGL((salience_rowstat_kernel<128>), grid1, block, 0, stream, k);
            hipLaunchKernelGGL(salience_lse_kernel, grid2, dim3(kRowsPerGroup), 0, stream, k);
            hipLaunchKernelGGL((salience_colsum_kernel<128>), grid3, block, 0, stream, k);
            break;
        case 96:
            hipLaunchKernelGGL((salience_rowstat_kernel<96>), grid1, block, 0, stream, k);
            hipLaunchKernelGGL(salience_lse_kernel, grid2, dim3(kRowsPerGroup), 0, stream, k);
            hipLaunchKernelGGL((salience_colsum_kernel<96>), grid3, block, 0, stream, k);
            break;
        case 64:
            hipLaunchKernelGGL((salience_rowstat_kernel<64>), grid1, block, 0, stream, k);
            hipLaunchKernelGGL(salience_lse_kernel, grid2, dim3(kRowsPerGroup), 0, stream, k);
            hipLaunchKernelGGL((salience_colsum_kernel<64>), grid3, block, 0, stream, k);
            break;
        default:
            return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(salience_finish_kernel, grid4, dim3(256), 0, stream, k);
    return hipGetLastError();
}

}  // namespace sv
