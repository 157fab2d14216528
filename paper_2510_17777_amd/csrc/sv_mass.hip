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
//          block of 256 keys.
// The R = Tq * G query rows of a (b, g) are cut into tiles of 16; a wavefront of a workgroup
// holds up to four of them in registers for the whole kernel (R <= 256), and all four wavefronts
// work on the same keys.  The keys come through LDS in stages of 64: wavefront w fetches key tile w
// of the next stage into registers while the current stage is used, and stores it to the other
// LDS buffer afterwards (one barrier per stage), so a key line crosses the memory system once per
// workgroup and a whole stage of compute hides its latency.  (Each wavefront fetching every key
// tile itself, one tile ahead, was bound by that latency: 2 us per 16 keys.)
// The work is a contraction plus one exponential per (row, key) and pass: bound by the
// exponential and matrix pipes, not by HBM.  Everything runs in base 2 (scale * log2(e) folded into
// one multiply-add before v_exp_f32).  Pass 1 keeps a reference per (lane, row) that is raised only
// when a logit exceeds it by more than 2^8: the usual case is one multiply-add, one exponential and
// one add per element, and the sums stay far from overflow.
#include <type_traits>

#include "sv_kernels.h"
#include "sv_mass_device.h"

namespace sv {
namespace {

constexpr int kStatBlockKeys = 1024;              // keys per workgroup in pass 1
constexpr int kColBlockKeys = 256;                // keys per sub-block in pass 2 (their masses sit in registers)
constexpr int kColSubBlocks = 4;                  // sub-blocks per workgroup: the query tiles are loaded once for 1024 keys

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
template <int D>
// Two wavefronts per SIMD (256 registers): one register more and the compiler settles for one.
__global__ __launch_bounds__(kMassThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void mass_rowstat_kernel(const MassArgs a) {
    constexpr int KB = D / 32;
    __shared__ KeyStage<KB> stage[2];
    __shared__ __align__(16) int s_last_txt[kMaxRowTiles * 16];
    const int blk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int rot = blk & (kMassWaves - 1);
    const int nt = live_len(a.txt_len, b, a.n_txt_max), nv = live_len(a.vis_len, b, a.n_vis_max);
    const int n_keys = nt + nv;
    const int key0 = blk * kStatBlockKeys;
    const int R = a.Tq * a.G;
    const int ntl = live_tiles_of(wave, rot, R);   // wave-uniform
    const float c2 = a.scale * kLog2e;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* part = a.part + ((unit * a.n_stat_blocks + blk) * (int64_t)(kMaxRowTiles * 16)) * 2;
    // last text row that query row r sees: its token i = r / G sits at text row nt - Tq + i (one division per
    // row here instead of one per logit in the masked tiles); read after the first barrier below
    static_assert(kMassThreads == kMaxRowTiles * 16, "one thread per query row");
    s_last_txt[threadIdx.x] = nt - a.Tq + ((int)threadIdx.x < R ? (int)threadIdx.x / a.G : 0);

    half8_t qa[kTilesPerWave][KB];
    load_query_tiles<KB>(a, b, g, wave, rot, lane, qa);
    // per lane, for the 4 rows (4*quad + rr) of each of its tiles, over the key columns it sees, in base 2:
    // a reference value ref (the largest logit met, or up to 8 below it) and l = sum 2^(logit - ref)
    float ref[kTilesPerWave][4], l[kTilesPerWave][4];
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            ref[t][rr] = -INFINITY;
            l[t][rr] = 0.f;
        }
    const _Float16* ktxt = static_cast<const _Float16*>(a.k_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh;
    const _Float16* kvis = static_cast<const _Float16*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;

    const int k_end = min(key0 + kStatBlockKeys, n_keys);
    half8_t kfetch[KB];
    auto fetch = [&](int s0) {   // this wavefront's key tile of the stage at s0; rows clamped, dead columns
        const int kc = min(s0 + wave * 16 + row, n_keys - 1);   // are masked at use
        if (kc < nt) load_key_tile<KB>(ktxt, a.txt_sn, kc, quad, kfetch);
        else load_key_tile<KB>(kvis, a.vis_sn, kc - nt, quad, kfetch);
    };
    auto put = [&](KeyStage<KB>& st) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) st.w[wave][kb][lane] = kfetch[kb];
    };
    // text tiles, ragged tiles, and visual tiles met before every reference is set: masked, exact running maximum
    auto masked_tile = [&](int k0, const KeyStage<KB>& st, int kt) {
        half8_t kf[KB];
        read_key_tile<KB>(st, kt, lane, kf);
        const int key = k0 + row;   // this lane's key column
        float4_t sv[kTilesPerWave];
        tile_logits<KB, kTilesPerWave>(qa, kf, sv);   // rows past R are zero rows: computed, never stored
#pragma unroll
        for (int t = 0; t < kTilesPerWave; ++t) {
            const int4 last4 = *reinterpret_cast<const int4*>(&s_last_txt[row_tile_of(wave, rot, t) * 16 + 4 * quad]);
            const int last_of[4] = {last4.x, last4.y, last4.z, last4.w};
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int last_txt = last_of[rr];
                const bool seen = key < n_keys && (key >= nt || key <= last_txt);
                const float x = seen ? sv[t][rr] * c2 : -INFINITY;
                const float mn = fmaxf(ref[t][rr], x);
                if (mn > -INFINITY) {   // something seen so far
                    l[t][rr] = l[t][rr] * __builtin_amdgcn_exp2f(ref[t][rr] - mn) + __builtin_amdgcn_exp2f(x - mn);
                    ref[t][rr] = mn;
                }
            }
        }
    };
    // The stage loop is instantiated once per count of live row tiles and chosen outside the loop: a switch
    // inside it made the compiler shuffle the 32 state registers between the arms at every stage (as many
    // moves and selects as useful instructions).
    auto run = [&](auto ntl_c) __attribute__((always_inline)) {
        constexpr int NTL = decltype(ntl_c)::value;
        fetch(key0);
        wait_for_loads();
        put(stage[0]);
        __syncthreads();
        int cur = 0;
        bool ref_ready = false;   // block-uniform: every reference is finite
        for (int s0 = key0; s0 < k_end; s0 += kStageKeys) {
            const bool more = s0 + kStageKeys < k_end;   // block-uniform
            if (more) fetch(s0 + kStageKeys);
            const bool plain = s0 >= nt && s0 + kStageKeys <= k_end;   // visual keys, all live, seen by every row
            if (plain && ref_ready) {
                rowstat_plain_stage<KB, NTL, false>(stage[cur], lane, qa, c2, ref, l);
            } else if (plain && s0 == key0) {   // first stage of the block: nothing seen so far
                rowstat_plain_stage<KB, NTL, true>(stage[cur], lane, qa, c2, ref, l);
                ref_ready = true;
            } else {
#pragma unroll 1
                for (int kt = 0; kt < kMassWaves; ++kt)
                    if (s0 + kt * 16 < k_end) masked_tile(s0 + kt * 16, stage[cur], kt);
                if (plain) ref_ready = true;   // every row saw these 64 keys
            }
            if (more) put(stage[cur ^ 1]);
            __syncthreads();
            cur ^= 1;
        }
    };
    if (key0 < k_end) {   // block-uniform
        switch (ntl) {    // wave-uniform
            case 4: run(std::integral_constant<int, 4>{}); break;
            case 3: run(std::integral_constant<int, 3>{}); break;
            case 2: run(std::integral_constant<int, 2>{}); break;
            case 1: run(std::integral_constant<int, 1>{}); break;
            default: run(std::integral_constant<int, 0>{}); break;
        }
    }
    // merge the 16 key columns of a row (the lanes of a 16-lane row hold the same rows), store per block
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const int tile = row_tile_of(wave, rot, t);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float mine = t < ntl ? ref[t][rr] : -INFINITY;   // the plain stages leave dead tiles untouched,
            const float lmine = t < ntl ? l[t][rr] : 0.f;          // the masked ones compute them: drop both
            const float mx = row_max16(mine);
            const float e = mine > -INFINITY ? __builtin_amdgcn_exp2f(mine - mx) : 0.f;
            const float lt = group_sum<16>(lmine * e);
            if (row == 0) {
                const int r = tile * 16 + 4 * quad + rr;
                part[r * 2] = mx * kLn2;   // natural-log units from here on
                part[r * 2 + 1] = lt;
            }
        }
    }
}

// lse[b, i, h] = log sum over the key blocks; one thread per query row.
__global__ __launch_bounds__(256) void mass_lse_kernel(const MassArgs a) {
    const int g = blockIdx.y, b = blockIdx.z;
    const int r = blockIdx.x * 256 + threadIdx.x;
    const int R = a.Tq * a.G;
    if (r >= R) return;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int nt = live_len(a.txt_len, b, a.n_txt_max), nv = live_len(a.vis_len, b, a.n_vis_max);
    const int live_blocks = (nt + nv + kStatBlockKeys - 1) / kStatBlockKeys;
    const float* part = a.part + (unit * a.n_stat_blocks * (int64_t)(kMaxRowTiles * 16)) * 2;
    float mx = -INFINITY;
    for (int s = 0; s < live_blocks; ++s) mx = fmaxf(mx, part[((int64_t)s * kMaxRowTiles * 16 + r) * 2]);
    float sum = 0.f;
    for (int s = 0; s < live_blocks; ++s) {
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
#pragma unroll
    for (int kt = 0; kt < kMassWaves; ++kt) {
        if (kt + 1 < kMassWaves) {
            read_key_tile<KB>(st, kt + 1, lane, kf[(kt + 1) & 1]);
            tile_logits<KB, NTL>(qa, kf[(kt + 1) & 1], sv[(kt + 1) & 1]);
        }
        float acc = 0.f;
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) acc += __builtin_amdgcn_exp2f(fmaf(sv[kt & 1][t][rr], c2, -lse2[t][rr]));
        col[kt] = acc;
    }
}

template <int D>
// Three wavefronts per SIMD: at 168 registers the compiler keeps the matrix results in VGPRs (no copies from
// accumulation registers) and still pipelines the key tiles; measured against two wavefronts per SIMD below.
__global__ __launch_bounds__(kMassThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void mass_colsum_kernel(const MassArgs a) {
    constexpr int KB = D / 32;
    constexpr int KT = kColBlockKeys / 16;   // key tiles per sub-block
    __shared__ KeyStage<KB> stage[2];
    __shared__ float s_col[kMassWaves][kColBlockKeys];
    const int blk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int rot = blk & (kMassWaves - 1);
    const int nv = live_len(a.vis_len, b, a.n_vis_max);
    const int key0 = blk * kColBlockKeys * kColSubBlocks;
    const int R = a.Tq * a.G;
    const int ntl = live_tiles_of(wave, rot, R);   // wave-uniform
    const float c2 = a.scale * kLog2e;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* out = a.scores + unit * a.n_vis_max;

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
    const int k_end = min(key0 + kColBlockKeys * kColSubBlocks, nv);   // live keys of this workgroup end here

    half8_t kfetch[KB];
    auto fetch = [&](int s0) {   // this wavefront's key tile of the stage at s0; rows clamped, dead columns dropped below
        load_key_tile<KB>(kvis, a.vis_sn, min(s0 + wave * 16 + row, nv - 1), quad, kfetch);
    };
    auto put = [&](KeyStage<KB>& st) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) st.w[wave][kb][lane] = kfetch[kb];
    };
    int cur = 0;
    if (key0 < k_end) fetch(key0);   // block-uniform
    wait_for_loads();
    if (key0 < k_end) put(stage[0]);
    __syncthreads();
    for (int sub = 0; sub < kColSubBlocks; ++sub) {
        const int sub0 = key0 + sub * kColBlockKeys;
        if (sub0 >= a.n_vis_max) break;   // block-uniform
        float col[KT];   // per lane: mass of key column (16*kt + row) from the rows this lane holds
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) col[kt] = 0.f;
        if (sub0 < k_end) {   // block-uniform
#pragma unroll
            for (int st = 0; st < kColBlockKeys / kStageKeys; ++st) {
                const int s0 = sub0 + st * kStageKeys;
                if (s0 >= k_end) break;   // block-uniform
                const bool more = s0 + kStageKeys < k_end;
                if (more) fetch(s0 + kStageKeys);
                switch (ntl) {
                    case 4: colsum_stage<KB, 4>(stage[cur], lane, qa, c2, lse2, &col[st * kMassWaves]); break;
                    case 3: colsum_stage<KB, 3>(stage[cur], lane, qa, c2, lse2, &col[st * kMassWaves]); break;
                    case 2: colsum_stage<KB, 2>(stage[cur], lane, qa, c2, lse2, &col[st * kMassWaves]); break;
                    case 1: colsum_stage<KB, 1>(stage[cur], lane, qa, c2, lse2, &col[st * kMassWaves]); break;
                    default: break;
                }
                if (more) put(stage[cur ^ 1]);
                __syncthreads();
                cur ^= 1;
            }
        }
        // the four quads of a wavefront hold different rows of the same key columns: add them, then the wavefronts
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            float x = col[kt];
            x += __shfl_xor(x, 16, kWave);
            x += __shfl_xor(x, 32, kWave);
            if (quad == 0) s_col[wave][kt * 16 + row] = x;
        }
        __syncthreads();
        for (int j = threadIdx.x; j < kColBlockKeys; j += kMassThreads) {
            const int key = sub0 + j;
            if (key < a.n_vis_max) {
                const float x = (s_col[0][j] + s_col[1][j]) + (s_col[2][j] + s_col[3][j]);
                out[key] = key < nv ? x : -INFINITY;
            }
        }
        __syncthreads();
    }
}

}  // namespace

int mass_stat_blocks(int n_txt_max, int n_vis_max) { return (n_txt_max + n_vis_max + kStatBlockKeys - 1) / kStatBlockKeys; }
int mass_max_rows() { return kMaxRowTiles * 16; }

size_t mass_workspace_bytes(int B, int Hkv, int n_txt_max, int n_vis_max) {
    return (size_t)B * Hkv * mass_stat_blocks(n_txt_max, n_vis_max) * kMaxRowTiles * 16 * 2 * sizeof(float);
}

hipError_t launch_mass(const MassArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0 || a.n_vis_max == 0) return hipSuccess;
    if (a.Tq * a.G > kMaxRowTiles * 16 || a.Tq < 1) return hipErrorInvalidValue;
    MassArgs k = a;
    k.n_stat_blocks = mass_stat_blocks(a.n_txt_max, a.n_vis_max);
    const dim3 block(kMassThreads);
    const dim3 grid1((unsigned)k.n_stat_blocks, (unsigned)a.Hkv, (unsigned)a.B);
    const dim3 grid2((unsigned)((a.Tq * a.G + 255) / 256), (unsigned)a.Hkv, (unsigned)a.B);
    const dim3 grid3((unsigned)((a.n_vis_max + kColBlockKeys * kColSubBlocks - 1) / (kColBlockKeys * kColSubBlocks)),
                     (unsigned)a.Hkv, (unsigned)a.B);
    if (a.D == 128) {
        hipLaunchKernelGGL((mass_rowstat_kernel<128>), grid1, block, 0, stream, k);
        hipLaunchKernelGGL(mass_lse_kernel, grid2, dim3(256), 0, stream, k);
        hipLaunchKernelGGL((mass_colsum_kernel<128>), grid3, block, 0, stream, k);
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
