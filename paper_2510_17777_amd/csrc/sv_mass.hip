// Retrieval as the paper runs it, once per conversation round (section 3.2, "Query-Aware Token
// Selection"; section 3.1, "Efficient Implementation": softmax normalisation and salience
// accumulation are streamed, the attention matrix is never formed): the relevance of visual
// token j to the user's question is the attention mass the question's tokens put on it,
//
//   mass[b,g,j] = sum_{i < Tq} sum_{h in group g} softmax_row(i,h)[j],
//
// where row (i,h) is query token i, head h, and its softmax runs over everything that row
// attends to in the model: the text rows up to and including its own position (the question's
// tokens are the last Tq rows of the text segment) and every visual row.
//
// Two streaming passes over the keys, both with the logits on the matrix cores
// (v_mfma_f32_16x16x32_f16: A = 16 query rows x 32 dims, B = 32 dims x 16 keys):
//   pass 1 (mass_rowstat_kernel)   per key block, a reference value and the sum of exponentials
//          relative to it for every query row -- each lane keeps them for the key columns it sees
//          and they are merged across lanes once per block -- then mass_lse_kernel merges the
//          blocks into lse[b,i,h] = log sum_keys exp(logit);
//   pass 2 (mass_colsum_kernel)    p = exp(logit - lse) for every (row, visual key), summed over
//          the rows: each lane sums the rows it holds, lanes and wavefronts are merged once per
//          stage of 64 keys.
// The R = Tq * G query rows of a (b, g) are cut into tiles of 16; a wavefront of a workgroup
// holds up to four of them in registers for the whole kernel (R <= 256), and all four wavefronts
// work on the same keys.  The keys come through LDS in stages of 64: wavefront w fetches key tile w
// of the next stage into registers while the current stage is used, and stores it to the other
// LDS buffer afterwards (one barrier per stage), so a key line crosses the memory system once per
// workgroup and a whole stage of compute hides its latency.  (Each wavefront fetching every key
// tile itself, one tile ahead, was bound by that latency: 2 us per 16 keys.)
// The work is a contraction plus one exponential per (row, key) and pass: bound by the vector and
// matrix pipes, not by HBM.  Everything runs in base 2 (scale * log2(e) folded into one multiply-add
// before v_exp_f32), and an element costs a multiply-add, an exponential and an add in both passes.
// Pass 1 takes one reference per wavefront from the first visual keys of the block and never raises it;
// row sums that leave the trusted range send the block through an exact sweep (a reference per row).  The matrix instructions of
// the next key tile are placed between the vector instructions of the current one.
#include <type_traits>

#include "sv_kernels.h"
#include "sv_mass_device.h"

namespace sv {
namespace {

constexpr int kMinBlockKeys = 1024;               // a workgroup streams at least this many visual keys (if the row has them)
constexpr int kTextBlockKeys = 256;               // text rows per workgroup: few rows, all on the slow masked path

// The A operands of this wavefront: a row tile holds rows 16*tile + (lane & 15); lane (row, quad) supplies
// dims 8*quad + 32*kb .. +8.  Row r is query token r / G, head g*G + r % G; rows >= R are zero.
template <int KB>
__device__ __forceinline__ void load_query_tiles(const MassArgs& a, int b, int g, int wave, int rot, int lane,
                                                 half8_t (&qa)[kTilesPerWave][KB]) {
    const int row = lane & 15, quad = lane >> 4;
    const int R = a.Tq * a.G;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {   // unconditional loads on a clamped row: no load waits for a branch
        const int r = row_tile_of(wave, rot, t) * 16 + row;
        const int rc = min(r, R - 1);
        const int i = rc / a.G, hh = rc - i * a.G;
        const _Float16* p = static_cast<const _Float16*>(a.q) + (int64_t)b * a.q_sb + (int64_t)i * a.q_st +
                            (int64_t)(g * a.G + hh) * a.q_sh + quad * 8;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const half8_t v = *reinterpret_cast<const half8_t*>(p + 32 * kb);
            qa[t][kb] = r < R ? v : half8_t(0);
        }
    }
}

// ---- pass 1: per key block, (reference, sum exp) of every query row over the block's keys ----
// Key list of a (b, g): text rows [0, nt), then visual rows [0, nv).  Query token i sits at text row
// nt - Tq + i and sees the text rows up to itself.
// kText: this workgroup streams text rows (blocks of txt_block_keys rows, the causal mask, every tile on the masked
// path); otherwise visual rows (blocks of stat_block_keys rows).  Two bodies, chosen per workgroup by the kernel below,
// rather than one body with a block-uniform flag: each then fits the 168 registers of three wavefronts per SIMD.
template <int D, bool kText>
__device__ __forceinline__ void rowstat_body(const MassArgs& a, const int blk, KeyStage<D / 32> (&stage)[2],
                                             int (&s_last_txt)[kMaxRowTiles * 16], int& s_flag) {
    constexpr int KB = D / 32;
    const int g = blockIdx.y, b = blockIdx.z;
    // the wavefront's index in a scalar register, the lane from the lane counter: nothing here keeps the thread-index
    // register alive, and what depends on the wavefront alone costs no vector register
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    const int lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int row = lane & 15, quad = lane >> 4;
    const int rot = blk & (kMassWaves - 1);
    const int nt = live_len(a.txt_len, b, a.n_txt_max), nv = live_len(a.vis_len, b, a.n_vis_max);
    constexpr bool is_txt = kText;
    const int block_keys = is_txt ? a.txt_block_keys : a.stat_block_keys;
    const int key0 = blk * block_keys;   // within the text or the visual rows
    const int n_keys = is_txt ? nt : nv;
    const int R = a.Tq * a.G;
    const int ntl = live_tiles_of(wave, rot, R);   // wave-uniform
    const float c2 = a.scale * kLog2e;
    if (key0 >= n_keys) return;   // block-uniform; the merge reads the live blocks only
    // last text row that query row r sees: its token i = r / G sits at text row nt - Tq + i (one division per
    // row here instead of one per logit in the masked tiles); read after the first barrier below
    static_assert(kMassThreads == kMaxRowTiles * 16, "one thread per query row");
    if (is_txt) s_last_txt[threadIdx.x] = nt - a.Tq + ((int)threadIdx.x < R ? (int)threadIdx.x / a.G : 0);

    half8_t qa[kTilesPerWave][KB];
    load_query_tiles<KB>(a, b, g, wave, rot, lane, qa);
    // per lane, for the 4 rows (4*quad + rr) of each of its tiles, over the key columns it sees, in base 2:
    // a reference value ref and l = sum 2^(logit - ref)
    float ref[kTilesPerWave][4], l[kTilesPerWave][4];
    const _Float16* keys = is_txt ? static_cast<const _Float16*>(a.k_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh
                                  : static_cast<const _Float16*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;
    const int64_t key_sn = is_txt ? a.txt_sn : a.vis_sn;

    const int k_end = min(key0 + block_keys, n_keys);
    half8_t kfetch[KB];
    auto fetch = [&](int s0) {   // this wavefront's key tile of the stage at s0; rows clamped, dead columns masked at use
        load_key_tile<KB>(keys, key_sn, min(s0 + wave * 16 + row, n_keys - 1), quad, kfetch);
    };
    auto put = [&](KeyStage<KB>& st) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) st.w[wave][kb][lane] = kfetch[kb];
    };
    // The same fetch for the slow loop, from lane coordinates computed on the spot: sharing them with the fast loop
    // keeps one more value alive across it than its register budget holds.
    auto fetch_again = [&](int s0) {
        int ln = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        asm volatile("" : "+v"(ln));
        load_key_tile<KB>(keys, key_sn, min(s0 + wave * 16 + (ln & 15), n_keys - 1), ln >> 4, kfetch);
    };
    // text tiles and every tile of an exact sweep: masked, a reference per row kept as the exact running maximum
    auto masked_tile = [&](int k0, const KeyStage<KB>& st, int kt) {
        half8_t kf[KB];
        read_key_tile<KB>(st, kt, lane, kf);
        const int key = k0 + row;   // this lane's key column
#pragma unroll
        for (int t = 0; t < kTilesPerWave; ++t) {   // one row tile at a time: this path is rare and is kept light on registers
            float4_t sv = {0.f, 0.f, 0.f, 0.f};     // rows past R are zero rows: computed, never stored
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) sv = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[kb], sv, 0, 0, 0);
            int4 last4 = {0, 0, 0, 0};
            if (is_txt) last4 = *reinterpret_cast<const int4*>(&s_last_txt[row_tile_of(wave, rot, t) * 16 + 4 * quad]);
            const int last_of[4] = {last4.x, last4.y, last4.z, last4.w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const bool seen = key < n_keys && (!is_txt || key <= last_of[rr]);
                const float x = seen ? sv[rr] * c2 : -INFINITY;
                const float mn = fmaxf(ref[t][rr], x);
                if (mn > -INFINITY) {   // something seen so far
                    l[t][rr] = l[t][rr] * __builtin_amdgcn_exp2f(ref[t][rr] - mn) + __builtin_amdgcn_exp2f(x - mn);
                    ref[t][rr] = mn;
                }
            }
        }
    };
    // One sweep over the key block.  On the fast path every stage, the ragged last one included, runs in one loop --
    // references from the first 16 keys, then multiply-add, exponential, add per element, dead columns masked through
    // the reference --; the exact sweep (text blocks; blocks whose fast sums left the trusted range) takes the masked path
    // for every tile.  The loops are separate and instantiated once per count of live row tiles, chosen outside them:
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
            fetch_again(s0 + kStageKeys);   // after the stage, not a stage ahead: this slow path (text rows, the rare redo of a
            put(stage[cur ^ 1]);      // visual block) gives the registers of the key tile in flight back -- their spills
            __syncthreads();          // would make the kernel use scratch
            cur ^= 1;
        }
    };
    auto run_fast = [&](auto ntl_c) __attribute__((always_inline)) {
        constexpr int NTL = decltype(ntl_c)::value;
        start();
        int cur = 0;
        const float ref_w = rowstat_init_ref<KB, NTL>(stage[0], lane, wave, rot, R, qa, c2);   // wave-uniform
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
    if (is_txt) run_exact();   // text rows: the causal mask, every tile on the masked path
    else sweep_fast();
    // What follows takes its lane coordinates from the lane counter: values computed before the sweep -- the thread
    // index register itself included -- would otherwise be kept alive across its loops, in registers that the
    // three-wavefront budget does not have.
    const int lane_m = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int quad_m = lane_m >> 4, row_m = lane_m & 15;
    // did the sum of a live row leave the range in which it is trusted (inf, NaN, huge or tiny: logits far from the
    // wavefront's reference)?
    const bool sees_a_key = row_m < k_end - key0;   // a block of fewer than 16 keys leaves lanes without a live column: sum 0
    bool bad = false;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const bool live_row = t < ntl && row_tile_of(wave, rot, t) * 16 + 4 * quad_m + rr < R;
            bad |= live_row && sees_a_key && !(l[t][rr] < kSumLimit && l[t][rr] >= 1.f / kSumLimit);
        }
    if (!is_txt && block_any(bad, &s_flag)) run_exact();   // block-uniform
    // merge the 16 key columns of a row (the lanes of a 16-lane row hold the same rows), store per block
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* part = a.part + ((unit * a.n_stat_blocks + (is_txt ? blk : a.n_txt_blocks + blk)) * (int64_t)(kMaxRowTiles * 16)) * 2;
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
            if (row_m == 0) {
                const int r = tile * 16 + 4 * quad_m + rr;
                part[r * 2] = mx * kLn2;   // natural-log units from here on
                part[r * 2 + 1] = lt;
            }
        }
    }
}

template <int D>
__global__ __launch_bounds__(kMassThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void mass_rowstat_kernel(const MassArgs a) {
    __shared__ KeyStage<D / 32> stage[2];
    __shared__ __align__(16) int s_last_txt[kMaxRowTiles * 16];
    __shared__ int s_flag;   // zero whenever block_any is entered
    if (threadIdx.x == 0) s_flag = 0;   // the sweeps below start with a barrier
    // the text blocks come first in the grid: they are few and slow (masked path) and run beside the visual ones
    if ((int)blockIdx.x < a.n_txt_blocks) rowstat_body<D, true>(a, blockIdx.x, stage, s_last_txt, s_flag);
    else rowstat_body<D, false>(a, (int)blockIdx.x - a.n_txt_blocks, stage, s_last_txt, s_flag);
}

// lse[b, i, h] = log sum over the live key blocks (text blocks first, then visual ones); one thread per query row.
__global__ __launch_bounds__(256) void mass_lse_kernel(const MassArgs a) {
    const int g = blockIdx.y, b = blockIdx.z;
    const int r = blockIdx.x * 256 + threadIdx.x;
    const int R = a.Tq * a.G;
    if (r >= R) return;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int nt = live_len(a.txt_len, b, a.n_txt_max), nv = live_len(a.vis_len, b, a.n_vis_max);
    const float* part = a.part + (unit * a.n_stat_blocks * (int64_t)(kMaxRowTiles * 16)) * 2;
    auto live = [&](int s) {   // did pass 1 run this block?
        return s < a.n_txt_blocks ? s * a.txt_block_keys < nt : (s - a.n_txt_blocks) * a.stat_block_keys < nv;
    };
    float mx = -INFINITY;
    for (int s = 0; s < a.n_stat_blocks; ++s)
        if (live(s)) mx = fmaxf(mx, part[((int64_t)s * kMaxRowTiles * 16 + r) * 2]);
    float sum = 0.f;
    for (int s = 0; s < a.n_stat_blocks; ++s) {
        if (!live(s)) continue;
        const float ms = part[((int64_t)s * kMaxRowTiles * 16 + r) * 2];
        if (ms > -INFINITY) sum += part[((int64_t)s * kMaxRowTiles * 16 + r) * 2 + 1] * expf(ms - mx);
    }
    const int i = r / a.G, hh = r - i * a.G;
    a.lse[((int64_t)b * a.Tq + i) * a.Hq + g * a.G + hh] = sum > 0.f ? mx + logf(sum) : INFINITY;
}

// ---- pass 2: mass of every visual key ----
// One stage: col[k] = sum over the wavefront's live rows of 2^(logit - lse) at key column 16k + row.  Key
// tiles past the live keys hold copies of the last live row: computed, dropped when the masses are stored.
template <int KB, int NTL>
__device__ __forceinline__ void colsum_stage(const KeyStage<KB>& st, int lane, const half8_t (&qa)[kTilesPerWave][KB],
                                             float c2, const float (&lse2)[kTilesPerWave][4], float* col) {
    half8_t kf[2][KB];
    float4_t sv[2][kTilesPerWave];
    read_key_tile<KB>(st, 0, lane, kf[0]);
    tile_logits<KB, NTL>(qa, kf[0], sv[0]);
    constexpr int n_m = KB * NTL, n_e = 4 * NTL;   // matrix instructions of a key tile, elements per lane of a key tile
    constexpr int NT1 = NTL > 0 ? NTL : 1, n_e1 = n_e > 0 ? n_e : 1;   // divisors that exist when a wavefront holds no live tile
    static_assert(KB <= 4, "at most one matrix instruction per element");
#pragma unroll
    for (int kt = 0; kt < kMassWaves; ++kt) {
        const int cur = kt & 1, nxt = cur ^ 1;
        const bool has_next = kt + 1 < kMassWaves;
        if (has_next) {
            read_key_tile<KB>(st, kt + 1, lane, kf[nxt]);
#pragma unroll
            for (int t = 0; t < NTL; ++t) sv[nxt][t] = {0.f, 0.f, 0.f, 0.f};
        }
        // Instruction order: one matrix instruction of the next key tile, then the multiply-add of element e, the
        // exponential of element e - 1 and the add of element e - 2 of this tile (two partial sums, so that no add
        // waits for the one before it), fenced so that the scheduler keeps it.
        float y[n_e1], pr[n_e1], part[2] = {0.f, 0.f};
#pragma unroll
        for (int step = 0; step < n_e + 2; ++step) {
            if (has_next && step < n_e) {
#pragma unroll
                for (int m = step * n_m / n_e1; m < (step + 1) * n_m / n_e1; ++m) {
                    const int kb = m / NT1, t = m % NT1;
                    sv[nxt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[nxt][kb], sv[nxt][t], 0, 0, 0);
                }
            }
            if (step < n_e) y[step] = fmaf(sv[cur][step / 4][step % 4], c2, -lse2[step / 4][step % 4]);
            if (step >= 1 && step - 1 < n_e) pr[step - 1] = __builtin_amdgcn_exp2f(y[step - 1]);
            if (step >= 2) part[(step - 2) & 1] += pr[step - 2];
            SV_STAGE_FENCE();
        }
        col[kt] = part[0] + part[1];
    }
}

template <int D>
// Three wavefronts per SIMD (168 registers): the more of them, the more often one issues vector instructions while
// another's matrix instruction runs.
__global__ __launch_bounds__(kMassThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void mass_colsum_kernel(const MassArgs a) {
    constexpr int KB = D / 32;
    __shared__ KeyStage<KB> stage[2];
    __shared__ float s_col[2][kMassWaves][kStageKeys];
    const int blk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int rot = blk & (kMassWaves - 1);
    const int nv = live_len(a.vis_len, b, a.n_vis_max);
    const int key0 = blk * a.stat_block_keys;
    const int blk_end = min(key0 + a.stat_block_keys, a.n_vis_max);   // keys this workgroup writes
    const int k_end = min(blk_end, nv);                                // live keys among them
    const int R = a.Tq * a.G;
    const int ntl = live_tiles_of(wave, rot, R);   // wave-uniform
    const float c2 = a.scale * kLog2e;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* out = a.scores + unit * a.n_vis_max;

    if (key0 < k_end) {   // block-uniform
        half8_t qa[kTilesPerWave][KB];
        load_query_tiles<KB>(a, b, g, wave, rot, lane, qa);
        float lse2[kTilesPerWave][4];   // base 2, of rows 4*quad + rr of each tile; +inf for the padding rows: p = 0
#pragma unroll
        for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = row_tile_of(wave, rot, t) * 16 + 4 * quad + rr;
                const int rc = min(r, R - 1);
                const int i = rc / a.G, hh = rc - i * a.G;
                const float v = a.lse[((int64_t)b * a.Tq + i) * a.Hq + g * a.G + hh];   // unconditional, clamped row
                lse2[t][rr] = r < R ? v * kLog2e : INFINITY;
            }
        const _Float16* kvis = static_cast<const _Float16*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;
        half8_t kfetch[KB];
        auto fetch = [&](int s0) {   // this wavefront's key tile of the stage at s0; rows clamped, dead columns dropped below
            load_key_tile<KB>(kvis, a.vis_sn, min(s0 + wave * 16 + row, nv - 1), quad, kfetch);
        };
        auto put = [&](KeyStage<KB>& st) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) st.w[wave][kb][lane] = kfetch[kb];
        };
        // Chosen outside the loop per count of live row tiles; the fetch and the store of the stage after the last
        // one are harmless (clamped rows, a buffer nobody reads) and so sit in no conditional block.
        auto run = [&](auto ntl_c) __attribute__((always_inline)) {
            constexpr int NTL = decltype(ntl_c)::value;
            fetch(key0);
            wait_for_loads();
            put(stage[0]);
            __syncthreads();
            int cur = 0;
            for (int s0 = key0; s0 < k_end; s0 += kStageKeys) {
                fetch(s0 + kStageKeys);
                float col[kMassWaves];   // per lane: mass of key column (16*kt + row) of this stage from the rows this lane holds
                colsum_stage<KB, NTL>(stage[cur], lane, qa, c2, lse2, col);
                // the four quads of a wavefront hold different rows of the same key columns: add them (every lane ends
                // up with the total, and the four quads store the same value: no divergent branch)
#pragma unroll
                for (int kt = 0; kt < kMassWaves; ++kt) {
                    float x = col[kt];
                    x += __shfl_xor(x, 16, kWave);
                    x += __shfl_xor(x, 32, kWave);
                    s_col[cur][wave][kt * 16 + row] = x;
                }
                put(stage[cur ^ 1]);
                __syncthreads();
                // then the wavefronts: wavefront w finishes keys 16w .. 16w + 15 of the stage; s_col[cur] is written
                // again two stages on, behind the next barrier
                if (lane < 16) {
                    const int j = wave * 16 + lane, key = s0 + j;
                    if (key < blk_end) {
                        const float x = (s_col[cur][0][j] + s_col[cur][1][j]) + (s_col[cur][2][j] + s_col[cur][3][j]);
                        out[key] = key < nv ? x : -INFINITY;
                    }
                }
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
    }
    // keys of the block past the stages above hold no live token
    const int done = key0 < k_end ? key0 + (k_end - key0 + kStageKeys - 1) / kStageKeys * kStageKeys : key0;
    for (int key = done + (int)threadIdx.x; key < blk_end; key += kMassThreads) out[key] = -INFINITY;
}

}  // namespace

namespace {
struct MassPlan { int stat_block_keys, txt_block_keys, n_txt_blocks, n_stat_blocks, n_col_blocks; };
MassPlan mass_plan(int B, int Hkv, int n_txt_max, int n_vis_max) {
    MassPlan p{};
    const int64_t units = (int64_t)B * Hkv;
    // one block length for both passes, planned on the visual rows (the text rows are few)
    p.stat_block_keys = planned_block_len(units, n_vis_max, kMinBlockKeys);
    p.txt_block_keys = kTextBlockKeys;
    p.n_txt_blocks = (n_txt_max + p.txt_block_keys - 1) / p.txt_block_keys;
    p.n_col_blocks = (n_vis_max + p.stat_block_keys - 1) / p.stat_block_keys;
    p.n_stat_blocks = p.n_txt_blocks + p.n_col_blocks;
    return p;
}
}  // namespace

int mass_max_rows() { return kMaxRowTiles * 16; }

size_t mass_workspace_bytes(int B, int Hkv, int n_txt_max, int n_vis_max) {
    return (size_t)B * Hkv * mass_plan(B, Hkv, n_txt_max, n_vis_max).n_stat_blocks * kMaxRowTiles * 16 * 2 * sizeof(float);
}

hipError_t launch_mass(const MassArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0 || a.n_vis_max == 0) return hipSuccess;
    if (a.Tq * a.G > kMaxRowTiles * 16 || a.Tq < 1) return hipErrorInvalidValue;
    const MassPlan p = mass_plan(a.B, a.Hkv, a.n_txt_max, a.n_vis_max);
    MassArgs k = a;
    k.stat_block_keys = p.stat_block_keys; k.txt_block_keys = p.txt_block_keys; k.n_txt_blocks = p.n_txt_blocks;
    k.n_stat_blocks = p.n_stat_blocks;
    const dim3 block(kMassThreads);
    const dim3 grid1((unsigned)p.n_stat_blocks, (unsigned)a.Hkv, (unsigned)a.B);
    const dim3 grid2((unsigned)((a.Tq * a.G + 255) / 256), (unsigned)a.Hkv, (unsigned)a.B);
    const dim3 grid3((unsigned)p.n_col_blocks, (unsigned)a.Hkv, (unsigned)a.B);
    if (a.D == 128) {
        hipLaunchKernelGGL((mass_rowstat_kernel<128>), grid1, block, 0, stream, k);
        hipLaunchKernelGGL(mass_lse_kernel, grid2, dim3(256), 0, stream, k);
        hipLaunchKernelGGL((mass_colsum_kernel<128>), grid3, block, 0, stream, k);
    } else if (a.D == 96) {
        hipLaunchKernelGGL((mass_rowstat_kernel<96>), grid1, block, 0, stream, k);
        hipLaunchKernelGGL(mass_lse_kernel, grid2, dim3(256), 0, stream, k);
        hipLaunchKernelGGL((mass_colsum_kernel<96>), grid3, block, 0, stream, k);
    } else if (a.D == 64) {
        hipLaunchKernelGGL((mass_rowstat_kernel<64>), grid1, block, 0, stream, k);
        hipLaunchKernelGGL(mass_lse_kernel, grid2, dim3(256), 0, stream, k);
        hipLaunchKernelGGL((mass_colsum_kernel<64>), grid3, block, 0, stream, k);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sv
