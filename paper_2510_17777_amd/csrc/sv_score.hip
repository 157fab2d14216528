// Step 1 of the decode path: relevance of every cached visual key to the current
// query (paper section 3.2, "Query-Aware Token Selection").
//
//   scores[b,g,j] = sum_{h in group g} scale * <q[b,h,:], K_vis[b,g,j,:]>
//
// The sum over the group's heads commutes with the dot product, so each workgroup
// first adds the group's query rows in fp32 and then needs ONE dot product per key.
// The kernel is a pure stream over K_vis (1 flop per byte): a row is split over
// 16-byte chunks, one per lane, so a wavefront load instruction fetches 1 KiB of
// consecutive memory; eight such loads are issued before the first is consumed.
// Lanes of one row are reduced with DPP inside a 16-lane row.
//
// Inside sv_decode_step the kernel also feeds the selection: a presample kernel scores a
// jittered, stratified sample of each row and takes an order statistic of it as t_lo, a
// value that lies below the k-th largest score of the row except with negligible
// probability; the scoring kernel then stores every (score, row) >= t_lo in the slot of
// the wavefront pass that produced it (LDS); after its last pass the workgroup's first
// wavefront packs the tile's candidates, in row order, into the tile's record in memory
// with (usually) one store instruction.  No atomics.  The selection ranks those few
// candidates instead of re-reading every score.  Measured on the long-video shape: the
// emission inside the loop is free, the barrier and the record store cost about 5 % of
// the kernel; thousands of small scattered stores straight from the passes cost 8 %.
#include "sv_device.h"
#include "sv_kernels.h"

namespace sv {
namespace {

constexpr int kScoreUnroll = 8;   // independent row loads in flight per lane
constexpr int kScoreWaves = 4;    // wavefronts per workgroup
constexpr int kFilterMaxTileRows = 512;   // rows of one scoring workgroup when it emits candidates
constexpr int kFilterPrimary = kFilterRecordPairs;

template <typename T, int D, bool kStream, bool kFilter>
__global__ __launch_bounds__(kScoreWaves * kWave) void score_kernel(const ScoreArgs a) {
    constexpr int EPL = Chunk<T>::kElems;   // elements per lane
    constexpr int LPR = D / EPL;            // lanes per row
    constexpr int RPW = kWave / LPR;        // rows per wavefront load
    constexpr int U = kScoreUnroll;
    constexpr int WAVE_ROWS = RPW * U;
    constexpr int BLOCK_ROWS = kScoreWaves * WAVE_ROWS;
    static_assert(U <= LPR, "store lane selection needs U <= lanes per row");

    const int b = blockIdx.z, g = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int c = lane % LPR;     // chunk of the row this lane owns
    const int grp = lane / LPR;   // which of the RPW rows of a load

    int n = a.n_vis_max;
    if (a.vis_len) {
        const int v = a.vis_len[b];
        n = v < 0 ? 0 : (v < n ? v : n);
    }
    const int row_begin = blockIdx.x * a.rows_per_block;
    const int row_end = min(row_begin + a.rows_per_block, a.n_vis_max);
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* __restrict__ srow = a.scores + unit * a.n_vis_max;
    // Candidate filter: every wavefront pass owns a slot of WAVE_ROWS entries in LDS.
    __shared__ uint2 s_ent[kFilter ? kFilterMaxTileRows : 1];
    __shared__ uint32_t s_cnt[kFilter ? kFilterMaxTileRows / WAVE_ROWS : 1];
    float t_lo = INFINITY;
    uint64_t rows_before = 0;   // lanes whose stored row precedes this lane's: lane (grp, c) stores row c*RPW + grp
    if (kFilter) {
        t_lo = a.filt.t_lo[unit];
        for (int gp = 0; gp < RPW; ++gp) {
            rows_before |= ((1ull << c) - 1ull) << (gp * LPR);
            if (gp < grp) rows_before |= 1ull << (gp * LPR + c);
        }
        if (lane == 0)
            for (int sl = wave; sl < a.rows_per_block / WAVE_ROWS; sl += kScoreWaves) s_cnt[sl] = 0;
    }

    // Summed query of the group, this lane's EPL dims.
    float qs[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) qs[i] = 0.f;
    if (row_begin < n) {
        const T* qp = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)g * a.G * a.q_sh + c * EPL;
        for (int h = 0; h < a.G; ++h) {
            const Chunk<T> qc = load_chunk(qp + (int64_t)h * a.q_sh);
#pragma unroll
            for (int i = 0; i < EPL; ++i) qs[i] += qc.at(i);
        }
    }

    const T* kbase = static_cast<const T*>(a.k_vis) + (int64_t)b * a.k_sb + (int64_t)g * a.k_sh + c * EPL;

    for (int r0 = row_begin + wave * WAVE_ROWS; r0 < row_end; r0 += BLOCK_ROWS) {
        float acc[U];
        Chunk<T> kc[U];
        if (r0 + WAVE_ROWS <= n) {   // wave-uniform: every row of this pass is live
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const T* p = kbase + (int64_t)(r0 + u * RPW + grp) * a.k_sn;
                kc[u] = kStream ? load_chunk_stream(p) : load_chunk(p);
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int row = r0 + u * RPW + grp;
                kc[u] = row < n ? load_chunk(kbase + (int64_t)row * a.k_sn) : zero_chunk<T>();
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < EPL; ++i) s = fmaf(kc[u].at(i), qs[i], s);
            acc[u] = group_sum<LPR>(s);
        }
        // Lane c of row-group grp stores the row of load u == c: a wavefront writes
        // WAVE_ROWS consecutive floats with one instruction.
        float o = acc[0];
#pragma unroll
        for (int u = 1; u < U; ++u) o = (c == u) ? acc[u] : o;
        const int row = r0 + c * RPW + grp;
        const float val = o * a.scale;
        if (c < U && row < row_end) srow[row] = row < n ? val : -INFINITY;
        if (kFilter) {
            const bool is_cand = c < U && row < row_end && row < n && val >= t_lo;
            const uint64_t cand_lanes = __ballot(is_cand);
            const int slot = (r0 - row_begin) / WAVE_ROWS;
            if (is_cand)
                s_ent[slot * WAVE_ROWS + __popcll(cand_lanes & rows_before)] =
                    make_uint2(__float_as_uint(val), (uint32_t)row);
            if (lane == 0) s_cnt[slot] = (uint32_t)__popcll(cand_lanes);
        }
    }
    if (kFilter) {
        __syncthreads();
        if (wave != 0) return;
        // Record of this tile, 8-byte items: {count, 0}, {0, 0}, then the first kFilterPrimary entries;
        // records of consecutive tiles are adjacent.  Entries beyond that go to the tile's overflow rows.
        const int64_t tile = unit * a.filt.n_tiles + blockIdx.x;
        uint2* rec = reinterpret_cast<uint2*>(a.filt.tiles) + tile * (kFilterPrimary + 2);
        uint2* ovf = a.filt.overflow + tile * a.rows_per_block;
        const int n_slots = a.rows_per_block / WAVE_ROWS;
        uint32_t total = 0;
        for (int sl = 0; sl < n_slots; ++sl) total += s_cnt[sl];
        for (uint32_t item = lane; item < total + 2; item += kWave) {
            uint2 v = make_uint2(item == 0 ? total : 0u, 0u);
            if (item >= 2) {
                uint32_t f = item - 2, base = 0;   // the f-th candidate of the tile: find its slot
                int sl = 0;
                for (; sl < n_slots - 1; ++sl) {
                    const uint32_t cs = s_cnt[sl];
                    if (f < base + cs) break;
                    base += cs;
                }
                v = s_ent[sl * WAVE_ROWS + (f - base)];
            }
            if (item < kFilterPrimary + 2) rec[item] = v;
            else ovf[item - 2] = v;
        }
    }
}

// ---------------------------------------------------------------- presample: t_lo per (b, g)
constexpr int kSample = 512;          // sampled rows per (b, g)
constexpr int kSampleThreads = 1024;

__device__ __forceinline__ uint32_t mix32(uint32_t x) {   // integer finaliser, for the sample jitter
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// Sample rank whose score serves as t_lo: with p = kb/n the number of sampled rows among the
// row's true top kb is about Binomial(S, p) (less spread, since the sample is stratified);
// t_lo exceeds the kb-th largest score only if that number reaches the rank.
__device__ __forceinline__ int sample_rank(int n, int kb) {
    const float m = (float)kSample * (float)kb / (float)n;
    return (int)ceilf(m + 5.f * sqrtf(m) + 4.f);
}

template <typename T, int D>
__global__ __launch_bounds__(kSampleThreads) void presample_kernel(const ScoreArgs a) {
    constexpr int EPL = Chunk<T>::kElems;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int NW = kSampleThreads / kWave;
    constexpr int LOADS = kSample / (NW * RPW);
    static_assert(LOADS >= 1 && LOADS * NW * RPW == kSample, "sample must divide over the workgroup");
    __shared__ float samp[kSample];

    const int g = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int c = lane % LPR, grp = lane / LPR;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    int n = a.n_vis_max;
    if (a.vis_len) {
        const int v = a.vis_len[b];
        n = v < 0 ? 0 : (v < n ? v : n);
    }
    const int kb = a.filt.k < n ? a.filt.k : n;
    if (kb == 0 || kb == n) {   // the selection handles these without candidates
        if (tid == 0) a.filt.t_lo[unit] = INFINITY;
        return;
    }
    int rank = a.filt.rank_override > 0 ? a.filt.rank_override : sample_rank(n, kb);
    if (rank > kSample - kSample / 8) {   // the sample cannot separate the top kb: every row is a candidate
        if (tid == 0) a.filt.t_lo[unit] = -INFINITY;
        return;
    }

    const T* kbase = static_cast<const T*>(a.k_vis) + (int64_t)b * a.k_sb + (int64_t)g * a.k_sh + c * EPL;
    Chunk<T> kc[LOADS];
    const int stratum = n / kSample;   // >= 1 unless the row is shorter than the sample
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
        const int i = (wave * LOADS + u) * RPW + grp;   // sample number
        int row = (int)(((int64_t)i * n) / kSample);
        if (stratum > 1) row += (int)(mix32((uint32_t)unit * 0x9E3779B9u + (uint32_t)i) % (uint32_t)stratum);
        row = row < n ? row : n - 1;
        kc[u] = load_chunk(kbase + (int64_t)row * a.k_sn);
    }
    float qs[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) qs[i] = 0.f;
    {
        const T* qp = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)g * a.G * a.q_sh + c * EPL;
        for (int h = 0; h < a.G; ++h) {
            const Chunk<T> qc = load_chunk(qp + (int64_t)h * a.q_sh);
#pragma unroll
            for (int i = 0; i < EPL; ++i) qs[i] += qc.at(i);
        }
    }
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) s = fmaf(kc[u].at(i), qs[i], s);
        s = group_sum<LPR>(s) * a.scale;
        if (c == 0) samp[(wave * LOADS + u) * RPW + grp] = s;
    }
    __syncthreads();
    // The rank-th largest sample, four bits of its order-preserving key per round: every
    // wavefront holds all keys (kSample/64 per lane); wavefront w counts the keys >= the probe
    // with digit w+1, and the digit is the number of probes that still have `rank` keys.
    {
        constexpr int KPL = kSample / kWave;
        __shared__ uint32_t s_probe[2][NW];
        uint32_t keys[KPL];
#pragma unroll
        for (int i = 0; i < KPL; ++i) keys[i] = score_key(samp[lane + i * kWave]);
        uint32_t prefix = 0;
#pragma unroll
        for (int round = 0; round < 8; ++round) {
            const int shift = 28 - 4 * round;
            if (wave < 15) {
                const uint32_t probe = prefix | ((uint32_t)(wave + 1) << shift);
                int cnt = 0;
#pragma unroll
                for (int i = 0; i < KPL; ++i) cnt += __popcll(__ballot(keys[i] >= probe));
                if (lane == 0) s_probe[round & 1][wave] = (uint32_t)cnt;
            }
            __syncthreads();
            uint32_t digit = 0;
#pragma unroll
            for (int w = 0; w < 15; ++w) digit += s_probe[round & 1][w] >= (uint32_t)rank ? 1u : 0u;
            prefix |= digit << shift;
        }
        if (tid == 0) {
            const uint32_t u = (prefix & 0x80000000u) ? (prefix & 0x7fffffffu) : ~prefix;
            a.filt.t_lo[unit] = __uint_as_float(u);
        }
    }
}

template <typename T, int D>
hipError_t launch_typed(const ScoreArgs& a, hipStream_t stream) {
    const int granule = score_row_granule(a.dtype, D);
    ScoreArgs k = a;
    int rpb = a.rows_per_block < granule ? granule : a.rows_per_block;
    rpb = (rpb + granule - 1) / granule * granule;
    if (a.filt.tiles) rpb = a.filt.tile_rows;   // the candidate records were laid out for this tiling
    k.rows_per_block = rpb;
    const unsigned tiles = (unsigned)((a.n_vis_max + rpb - 1) / rpb);
    if (tiles == 0 || a.B == 0) return hipSuccess;
    dim3 grid(tiles, (unsigned)a.Hkv, (unsigned)a.B), block(kScoreWaves * kWave);
    if (a.filt.tiles) {
        if (a.stream_loads) hipLaunchKernelGGL((score_kernel<T, D, true, true>), grid, block, 0, stream, k);
        else hipLaunchKernelGGL((score_kernel<T, D, false, true>), grid, block, 0, stream, k);
    } else {
        if (a.stream_loads) hipLaunchKernelGGL((score_kernel<T, D, true, false>), grid, block, 0, stream, k);
        else hipLaunchKernelGGL((score_kernel<T, D, false, false>), grid, block, 0, stream, k);
    }
    return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_presample_typed(const ScoreArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0) return hipSuccess;
    dim3 grid((unsigned)a.Hkv, (unsigned)a.B), block(kSampleThreads);
    hipLaunchKernelGGL((presample_kernel<T, D>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace

int score_row_granule(int dtype, int D) {
    const int epl = dtype == 0 ? 8 : 4;
    const int lpr = D / epl;
    return kScoreWaves * (kWave / lpr) * kScoreUnroll;
}

int score_wave_rows(int dtype, int D) { return score_row_granule(dtype, D) / kScoreWaves; }

int presample_rows() { return kSample; }

int filter_tile_rows(int dtype, int D, int requested, int n_vis_max, int max_tiles) {
    const int granule = score_row_granule(dtype, D);
    int rpb = requested < granule ? granule : requested;
    rpb = (rpb + granule - 1) / granule * granule;
    if (rpb > kFilterMaxTileRows) rpb = kFilterMaxTileRows / granule * granule;
    while ((n_vis_max + rpb - 1) / rpb > max_tiles && rpb + granule <= kFilterMaxTileRows) rpb += granule;
    return (n_vis_max + rpb - 1) / rpb > max_tiles ? 0 : rpb;
}

hipError_t launch_presample(const ScoreArgs& a, hipStream_t stream) {
    if (a.dtype == 0) {
        if (a.D == 128) return launch_presample_typed<_Float16, 128>(a, stream);
        if (a.D == 64) return launch_presample_typed<_Float16, 64>(a, stream);
    } else {
        if (a.D == 128) return launch_presample_typed<float, 128>(a, stream);
        if (a.D == 64) return launch_presample_typed<float, 64>(a, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_score(const ScoreArgs& a, hipStream_t stream) {
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
