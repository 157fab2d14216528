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
//   pass 1 (mass_rowstat_kernel)   per key block, the running maximum and sum of exponentials of
//          every query row -- each lane keeps them for the key columns it sees and they are
//          merged across lanes once per block -- then mass_lse_kernel merges the blocks into
//          lse[b,i,h] = log sum_keys exp(logit);
//   pass 2 (mass_colsum_kernel)    p = exp(logit - lse) for every (row, visual key), summed over
//          the rows: each lane sums the rows it holds, lanes and wavefronts are merged once per
//          block of 256 keys.
// The R = Tq * G query rows of a (b, g) are cut into tiles of 16; wavefront w of a workgroup
// holds tiles w, w+4, w+8, w+12 in registers for the whole kernel (R <= 256), all four
// wavefronts stream the same keys.  The work is a contraction plus one exponential per
// (row, key): bound by the exponential and matrix pipes, not by HBM (at Tq = 32, G = 7 the
// 1.44 GB of keys are re-read twice while 2.5e9 exponentials are taken).
#include "sv_device.h"
#include "sv_kernels.h"

namespace sv {
namespace {

constexpr int kMassWaves = 4;
constexpr int kMassThreads = kMassWaves * kWave;
constexpr int kMaxRowTiles = 16;                  // R <= 256
constexpr int kTilesPerWave = kMaxRowTiles / kMassWaves;
constexpr int kStatBlockKeys = 1024;              // keys per workgroup in pass 1
constexpr int kColBlockKeys = 256;                // keys per sub-block in pass 2 (their masses sit in registers)
constexpr int kColSubBlocks = 4;                  // sub-blocks per workgroup: the query tiles are loaded once for 1024 keys

__device__ __forceinline__ int live_len(const int32_t* p, int i, int cap) {
    if (!p) return cap;
    const int v = p[i];
    return v < 0 ? 0 : (v < cap ? v : cap);
}

// The A operands of this wavefront: row tile t holds rows 16t + (lane & 15); lane (row, quad) supplies
// dims 8*quad + 32*kb .. +8.  Row r is query token r / G, head g*G + r % G; rows >= R are zero.
template <int KB>
__device__ __forceinline__ void load_query_tiles(const MassArgs& a, int b, int g, int wave, int lane,
                                                 half8_t (&qa)[kTilesPerWave][KB]) {
    const int row = lane & 15, quad = lane >> 4;
    const int R = a.Tq * a.G;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const int r = (wave + t * kMassWaves) * 16 + row;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) qa[t][kb] = 0;
        if (r < R) {
            const int i = r / a.G, hh = r - i * a.G;
            const _Float16* p = static_cast<const _Float16*>(a.q) + (int64_t)b * a.q_sb + (int64_t)i * a.q_st +
                                (int64_t)(g * a.G + hh) * a.q_sh + quad * 8;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) qa[t][kb] = *reinterpret_cast<const half8_t*>(p + 32 * kb);
        }
    }
}

// B operand of one key tile: lane (row, quad) supplies dims 8*quad + 32*kb .. +8 of key `key_row`.
template <int KB>
__device__ __forceinline__ void load_key_tile(const _Float16* base, int64_t sn, int key_row, int quad,
                                              half8_t (&kf)[KB]) {
    const _Float16* p = base + (int64_t)key_row * sn + quad * 8;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) kf[kb] = __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(p + 32 * kb));
}

// ---- pass 1: per key block, (max, sum exp) of every query row over the block's keys ----
// Key list of a (b, g): text rows [0, nt), then visual rows [0, nv).  Query token i sits at text row
// nt - Tq + i and sees the text rows up to itself.
template <int D>
__global__ __launch_bounds__(kMassThreads) void mass_rowstat_kernel(const MassArgs a) {
    constexpr int KB = D / 32;
    const int blk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int nt = live_len(a.txt_len, b, a.n_txt_max), nv = live_len(a.vis_len, b, a.n_vis_max);
    const int n_keys = nt + nv;
    const int key0 = blk * kStatBlockKeys;
    const int R = a.Tq * a.G;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* part = a.part + ((unit * a.n_stat_blocks + blk) * (int64_t)(kMaxRowTiles * 16)) * 2;

    half8_t qa[kTilesPerWave][KB];
    load_query_tiles<KB>(a, b, g, wave, lane, qa);
    // per lane: running max and sum of the 4 rows (4*quad + rr) of each of its tiles over the key columns it sees
    float m[kTilesPerWave][4], l[kTilesPerWave][4];
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            m[t][rr] = -INFINITY;
            l[t][rr] = 0.f;
        }
    const _Float16* ktxt = static_cast<const _Float16*>(a.k_txt) + (int64_t)b * a.txt_sb + (int64_t)g * a.txt_sh;
    const _Float16* kvis = static_cast<const _Float16*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;

    const int k_end = min(key0 + kStatBlockKeys, n_keys);
    auto load_tile = [&](int k0, half8_t (&kf)[KB]) {   // clamped rows: dead columns are masked at use
        const int kc = min(k0 + row, n_keys - 1);
        if (kc < nt) load_key_tile<KB>(ktxt, a.txt_sn, kc, quad, kf);
        else load_key_tile<KB>(kvis, a.vis_sn, kc - nt, quad, kf);
    };
    auto consume_tile = [&](int k0, const half8_t (&kf)[KB]) {
        const int key = k0 + row;               // this lane's key column
        const bool plain = k0 >= nt && k0 + 16 <= n_keys;   // wave-uniform: visual keys, all live, seen by every row
#pragma unroll
        for (int t = 0; t < kTilesPerWave; ++t) {
            if ((wave + t * kMassWaves) * 16 >= R) break;   // wave-uniform
            float4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) s = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[kb], s, 0, 0, 0);
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                float x = s[rr] * a.scale;
                if (!plain) {   // text tiles and the ragged last tile: query token i sits at text row nt - Tq + i
                    const int r = (wave + t * kMassWaves) * 16 + 4 * quad + rr;
                    const int last_txt = nt - a.Tq + (r < R ? r / a.G : 0);
                    const bool seen = key < n_keys && (key >= nt || key <= last_txt);
                    x = seen ? x : -INFINITY;
                }
                const float mn = fmaxf(m[t][rr], x);
                if (mn > -INFINITY) {   // something seen so far
                    l[t][rr] = l[t][rr] * __expf(m[t][rr] - mn) + __expf(x - mn);
                    m[t][rr] = mn;
                }
            }
        }
    };
    if (key0 < k_end) {
        half8_t kf0[KB], kf1[KB];
        load_tile(key0, kf0);
        for (int k0 = key0; k0 < k_end; k0 += 32) {
            if (k0 + 16 < k_end) load_tile(k0 + 16, kf1);
            consume_tile(k0, kf0);
            if (k0 + 16 < k_end) {
                if (k0 + 32 < k_end) load_tile(k0 + 32, kf0);
                consume_tile(k0 + 16, kf1);
            }
        }
    }
    // merge the 16 key columns of a row (the lanes of a 16-lane row hold the same rows), store per block
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
        const int tile = wave + t * kMassWaves;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            float mx = m[t][rr];
            mx = fmaxf(mx, dpp_move<kDppQuadXor1>(mx));
            mx = fmaxf(mx, dpp_move<kDppQuadXor2>(mx));
            mx = fmaxf(mx, dpp_move<kDppRowHalfMirror>(mx));
            mx = fmaxf(mx, dpp_move<kDppRowMirror>(mx));
            const float e = m[t][rr] > -INFINITY ? __expf(m[t][rr] - mx) : 0.f;
            const float lt = group_sum<16>(l[t][rr] * e);
            if (row == 0) {
                const int r = tile * 16 + 4 * quad + rr;
                part[r * 2] = mx;
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
template <int D>
__global__ __launch_bounds__(kMassThreads) void mass_colsum_kernel(const MassArgs a) {
    constexpr int KB = D / 32;
    constexpr int KT = kColBlockKeys / 16;   // key tiles per block
    __shared__ float s_col[kMassWaves][kColBlockKeys];
    const int blk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int row = lane & 15, quad = lane >> 4;
    const int nv = live_len(a.vis_len, b, a.n_vis_max);
    const int key0 = blk * kColBlockKeys * kColSubBlocks;
    const int R = a.Tq * a.G;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* out = a.scores + unit * a.n_vis_max;

    half8_t qa[kTilesPerWave][KB];
    load_query_tiles<KB>(a, b, g, wave, lane, qa);
    float lse[kTilesPerWave][4];   // of rows 4*quad + rr of each tile; +inf for the padding rows: p = 0
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const int r = (wave + t * kMassWaves) * 16 + 4 * quad + rr;
            lse[t][rr] = INFINITY;
            if (r < R) {
                const int i = r / a.G, hh = r - i * a.G;
                lse[t][rr] = a.lse[((int64_t)b * a.Tq + i) * a.Hq + g * a.G + hh];
            }
        }
    const _Float16* kvis = static_cast<const _Float16*>(a.k_vis) + (int64_t)b * a.vis_sb + (int64_t)g * a.vis_sh;

    for (int sub = 0; sub < kColSubBlocks; ++sub) {
        const int sub0 = key0 + sub * kColBlockKeys;
        if (sub0 >= a.n_vis_max) break;   // block-uniform
        float col[KT];   // per lane: mass of key column (16*kt + row) from the rows this lane holds
        if (sub0 < nv) {   // block-uniform
            half8_t kf[2][KB];
            load_key_tile<KB>(kvis, a.vis_sn, min(sub0 + row, nv - 1), quad, kf[0]);
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                col[kt] = 0.f;
                if (kt + 1 < KT)   // next tile in flight while this one is used; rows clamped, dead columns dropped below
                    load_key_tile<KB>(kvis, a.vis_sn, min(sub0 + (kt + 1) * 16 + row, nv - 1), quad, kf[(kt + 1) & 1]);
                if (sub0 + kt * 16 >= nv) continue;   // wave-uniform: tile past the live keys
#pragma unroll
                for (int t = 0; t < kTilesPerWave; ++t) {
                    if ((wave + t * kMassWaves) * 16 >= R) break;   // wave-uniform
                    float4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb)
                        s = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[kt & 1][kb], s, 0, 0, 0);
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) col[kt] += __expf(s[rr] * a.scale - lse[t][rr]);
                }
            }
        } else {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) col[kt] = 0.f;
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
