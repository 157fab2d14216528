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
// Inside sv_decode_step the same launch also feeds the selection (kFilter):
//   * the first `units` workgroups of the (linear) grid are SAMPLERS, one per (b, g): each
//     scores a jittered, stratified sample of 512 rows of its row and publishes an order
//     statistic of those scores as t_lo -- a value below the k-th largest score of the
//     row except with negligible probability -- as one 8-byte word {epoch, t_lo};
//   * every other workgroup scores one TILE of a row as usual, keeps the tile's scores
//     in LDS, and after its last pass its first wavefront reads t_lo and writes the
//     tile's (score, row) pairs >= t_lo, in row order, to the tile's record, together
//     with the t_lo it used, as one store of whole 128-byte lines.
// t_lo is a hint, not a dependency: whatever value a tile uses, the selection verifies
// on the device that the candidates it received determine the kept set, and otherwise
// selects from all scores of the row.  So a tile may read t_lo without any ordering
// guarantee; it polls the word a bounded number of times (samplers are dispatched first
// and a tile needs the value only after streaming its rows, so in practice the first
// read succeeds) and falls back to "every row is a candidate" if the word never shows
// the call's epoch.  A separate sampler launch in front of the scoring launch cost
// 13 us on the long-video shape, of which 4.5 us is the price of any kernel boundary.
// The record store by one wavefront after a barrier costs about 5 % of the kernel;
// small scattered stores straight from the passes cost 8 %.
#include "sv_score_device.h"

namespace sv {
namespace {

constexpr int kScoreWaves = 4;    // wavefronts per workgroup
constexpr int kScoreThreads = kScoreWaves * kWave;
constexpr int kFilterMaxTileRows = 512;   // rows of one scoring workgroup when it emits candidates
constexpr int kFilterPrimary = kFilterRecordPairs;
constexpr int kSample = 512;              // sampled rows per (b, g), at most (FilterArgs::n_samples: this or half of it)
constexpr int kHintPolls = 64;            // bounded wait for t_lo
constexpr int kFilterTilesPerWave = 4;    // scores_filter_kernel: tiles one wavefront turns into records

__device__ __forceinline__ uint32_t mix32(uint32_t x) {   // integer finaliser, for the sample jitter
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// Sample rank whose score serves as t_lo: with p = kb/n the number of sampled rows among the
// row's true top kb is about Binomial(S, p) (less spread, since the sample is stratified);
// t_lo exceeds the kb-th largest score only if that number reaches the rank.
__device__ __forceinline__ int sample_rank(int n, int kb, int n_samples = kSample) {
    const float m = (float)n_samples * (float)kb / (float)n;
    return (int)ceilf(m + 5.f * sqrtf(m) + 4.f);
}

// Tag of this launch's hint words: the host's call counter plus the device's generation word.
__device__ __forceinline__ uint32_t launch_epoch(const ScoreArgs& a) { return a.filt.epoch + a.filt.gen[0]; }

__device__ __forceinline__ void publish_hint(const ScoreArgs& a, int64_t unit, float t_lo) {
    const uint64_t word = ((uint64_t)launch_epoch(a) << 32) | (uint64_t)__float_as_uint(t_lo);
    __hip_atomic_store(a.filt.hint + unit, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The rank-th largest of the kSample scores in samp (LDS), by one wavefront: binary search on the
// order-preserving key, most significant bit first, all keys in registers (kSample/64 per lane; slots past a
// smaller sample hold -inf and never count): a bit
// stays set if at least `rank` keys are >= the probe.  No barrier, no LDS traffic in the loop.  The search
// stops after kSearchBits bits; the bits below stay zero, i.e. the result comes out a hair lower (relative
// 2^-15 of its magnitude): still a valid threshold, a handful more candidates.
__device__ __forceinline__ float rank_statistic(const float* samp, int rank, int lane) {
    constexpr int KPL = kSample / kWave;
    constexpr int kSearchBits = 24;
    uint32_t keys[KPL];
#pragma unroll
    for (int i = 0; i < KPL; ++i) keys[i] = score_key(samp[lane + i * kWave]);
    uint32_t prefix = 0;
    for (int bit = 31; bit > 31 - kSearchBits; --bit) {
        const uint32_t probe = prefix | (1u << bit);
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < KPL; ++i) cnt += __popcll(__ballot(keys[i] >= probe));
        if (cnt >= rank) prefix = probe;   // wave-uniform
    }
    const uint32_t u = (prefix & 0x80000000u) ? (prefix & 0x7fffffffu) : ~prefix;
    return __uint_as_float(u);
}

// Row number of sample i of a (b, g) with n live rows: stratified, with a jitter that differs per (b, g).
__device__ __forceinline__ int sample_row_of(int i, int n, int64_t unit, int n_samples = kSample) {
    const int stratum = n / n_samples;   // >= 1 unless the row is shorter than the sample
    int row = (int)(((int64_t)i * n) / n_samples);
    if (stratum > 1) row += (int)(mix32((uint32_t)unit * 0x9E3779B9u + (uint32_t)i) % (uint32_t)stratum);
    return row < n ? row : n - 1;
}

// Sampler workgroup of one (b, g): 512 sample scores -> t_lo.
template <typename T, int D>
__device__ __forceinline__ void sample_threshold(const ScoreArgs& a, int b, int g, float* samp) {
    constexpr int EPL = Chunk<T>::kElems;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int U = kScoreUnroll / 2;                 // fewer loads in flight than the streaming loop: the
                                                        // sampler must fit the register budget of that loop
    constexpr int ROUND_ROWS = kScoreWaves * U * RPW;   // samples per round of loads
    static_assert(kSample % (2 * ROUND_ROWS) == 0, "the sample and its half must divide over the workgroup");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int c = lane % LPR, grp = lane / LPR;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int n = live_rows_of(a, b);
    const int kb = a.filt.k < n ? a.filt.k : n;
    if (kb == 0 || kb == n) {   // the selection handles these rows without candidates
        if (tid == 0) publish_hint(a, unit, INFINITY);
        return;
    }
    const int ns = a.filt.n_samples == kSample / 2 ? kSample / 2 : kSample;   // block-uniform
    const int rounds = ns / ROUND_ROWS;
    const int rank = a.filt.rank_override > 0 ? a.filt.rank_override : sample_rank(n, kb, ns);
    if (rank > ns - ns / 8) {   // the sample cannot separate the top kb: every row is a candidate
        if (tid == 0) publish_hint(a, unit, -INFINITY);
        return;
    }
    for (int i = ns + tid; i < kSample; i += kScoreThreads) samp[i] = -INFINITY;   // the rank search reads kSample slots
    const T* kbase = static_cast<const T*>(a.k_vis) + (int64_t)b * a.k_sb + (int64_t)g * a.k_sh + c * EPL;
    Chunk<T> kc[U];
    auto request = [&](int r) {   // the U sample rows of this lane group in round r
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = r * ROUND_ROWS + (wave * U + u) * RPW + grp;   // sample number
            kc[u] = load_chunk(kbase + (int64_t)sample_row_of(i, n, unit, ns) * a.k_sn);
        }
    };
    // The rounds are a chain of dependent memory trips (the register budget of the streaming loop allows
    // U loads per lane in flight): the first round is requested before the query, so that the two share a trip.
    request(0);
    float qs[EPL];
    summed_query<T>(a, b, g, c, qs);
    for (int r = 0; r < rounds; ++r) {
        float sc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < EPL; ++i) s = fmaf(kc[u].at(i), qs[i], s);
            sc[u] = s;
        }
        if (r + 1 < rounds) request(r + 1);   // the next trip starts before the lane-group sums of this one
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float s = group_sum<LPR>(sc[u]) * a.scale;
            if (c == 0) samp[r * ROUND_ROWS + (wave * U + u) * RPW + grp] = s;
        }
    }
    __syncthreads();
    if (wave != 0) return;
    const float t_lo = rank_statistic(samp, rank, lane);
    if (tid == 0) publish_hint(a, unit, t_lo);
}

// Rows of the sample one round of loads of a sampler workgroup covers (U loads per lane, as in sample_threshold).
template <typename T, int D>
constexpr int sampler_round_rows() {
    return kScoreWaves * (kScoreUnroll / 2) * (kWave / (D / Chunk<T>::kElems));
}

// SPREAD sampling, for launches so small that all their tiles are resident at once and have streamed their rows before
// one sampler workgroup has walked through its chain of dependent trips (lengths, query, four rounds of sample rows,
// rank search: 9 us, where the tiles of one layer of a long video are done after 6).  The 256 sample rows of a (b, g)
// are dealt over `spread` sampler workgroups; each scores its share in ONE round of loads and publishes the scores as
// tagged words {epoch, score}; workgroup 0 of the (b, g) then fetches all 256 words (a bounded wait for the others,
// which run beside it), ranks them and publishes t_lo as sample_threshold does.  If the words never all carry this
// call's tag it publishes "every row is a candidate", which the selection's checks cover like any other threshold.
template <typename T, int D>
__device__ __forceinline__ void sample_threshold_spread(const ScoreArgs& a, int b, int g, int part, float* samp) {
    constexpr int EPL = Chunk<T>::kElems;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int U = kScoreUnroll / 2;
    constexpr int ns = kSample / 2, WPL = ns / kWave;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int c = lane % LPR, grp = lane / LPR;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const int n = live_rows_of(a, b);
    const int kb = a.filt.k < n ? a.filt.k : n;
    if (kb == 0 || kb == n) {   // the selection handles these rows without candidates
        if (part == 0 && tid == 0) publish_hint(a, unit, INFINITY);
        return;
    }
    const int rank = a.filt.rank_override > 0 ? a.filt.rank_override : sample_rank(n, kb, ns);
    if (rank > ns - ns / 8) {   // the sample cannot separate the top kb: every row is a candidate
        if (part == 0 && tid == 0) publish_hint(a, unit, -INFINITY);
        return;
    }
    const T* kbase = static_cast<const T*>(a.k_vis) + (int64_t)b * a.k_sb + (int64_t)g * a.k_sh + c * EPL;
    const int i0 = part * sampler_round_rows<T, D>() + wave * U * RPW + grp;   // this lane group's first sample
    Chunk<T> kc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) kc[u] = load_chunk(kbase + (int64_t)sample_row_of(i0 + u * RPW, n, unit, ns) * a.k_sn);
    float qs[EPL];
    summed_query<T>(a, b, g, c, qs);   // after the rows were requested: the two share a trip
    const uint32_t epoch = launch_epoch(a);
    uint64_t* words = a.filt.samples + unit * ns;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float sc = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) sc = fmaf(kc[u].at(i), qs[i], sc);
        sc = group_sum<LPR>(sc) * a.scale;
        if (c == 0)
            __hip_atomic_store(words + i0 + u * RPW, ((uint64_t)epoch << 32) | (uint64_t)__float_as_uint(sc),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (part != 0 || wave != 0) return;   // no barrier below: one wavefront of one workgroup ranks
    float t_lo = -INFINITY;
    for (int poll = 0; poll < kHintPolls; ++poll) {
        uint64_t w[WPL];
#pragma unroll
        for (int i = 0; i < WPL; ++i) w[i] = __hip_atomic_load(words + lane + i * kWave, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool mine = true;
#pragma unroll
        for (int i = 0; i < WPL; ++i) mine = mine && (uint32_t)(w[i] >> 32) == epoch;
        if (__ballot(!mine) == 0ull) {   // wave-uniform: all 256 words are this call's
#pragma unroll
            for (int i = 0; i < WPL; ++i) samp[lane + i * kWave] = __uint_as_float((uint32_t)w[i]);
#pragma unroll
            for (int i = WPL; i < kSample / kWave; ++i) samp[lane + i * kWave] = -INFINITY;   // the rank search reads kSample slots
            __builtin_amdgcn_wave_barrier();   // LDS traffic of one wavefront stays in program order
            t_lo = rank_statistic(samp, rank, lane);
            if (t_lo != t_lo) t_lo = -INFINITY;   // stale words that happen to carry the tag may hold anything
            break;
        }
        __builtin_amdgcn_s_sleep(16);
    }
    if (lane == 0) publish_hint(a, unit, t_lo);
}

// End of a tile, one wavefront: waits (bounded) for the row's threshold and stores the tile's record.
// s_val holds the tile's scores (-inf past the live rows), s_pair is scratch for the pairs.
__device__ __forceinline__ void emit_tile_record(const ScoreArgs& a, int64_t unit, int tile, int row_begin, int row_end,
                                                 const float* s_val, uint2* s_pair, uint64_t& hint_word, uint32_t epoch,
                                                 int lane) {
    // t_lo of the row: the sampler's word, once it carries this call's epoch
    float t_lo = -INFINITY;
    for (int poll = 0; poll < kHintPolls; ++poll) {
        if ((uint32_t)(hint_word >> 32) == epoch) {
            t_lo = __uint_as_float((uint32_t)hint_word);
            if (t_lo != t_lo) t_lo = -INFINITY;   // a stale word that happens to carry the epoch
            break;
        }
        __builtin_amdgcn_s_sleep(32);
        hint_word = __hip_atomic_load(a.filt.hint + unit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (a.filt.test_mode != 0 && tile % 3 == 1) t_lo = a.filt.test_mode == 1 ? INFINITY : -INFINITY;
    // Record of this tile, 8-byte items: {count, t_lo used}, {largest pair score, 0}, then the first kFilterPrimary
    // pairs in row order; records of consecutive tiles are adjacent.  A tile with more pairs also
    // writes all of them to its overflow rows.  Every store covers whole 128-byte lines (the
    // tail of the last line is zero-filled): a partially written line costs a fetch of the rest.
    const int64_t tile_id = unit * a.filt.n_tiles + tile;
    uint2* rec = reinterpret_cast<uint2*>(a.filt.tiles) + tile_id * (kFilterPrimary + 2);
    uint2* ovf = a.filt.overflow + tile_id * a.rows_per_block;
    const int tile_len = row_end - row_begin;
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    uint32_t count = 0;
    float top = -INFINITY;
    for (int r = lane; r - lane < tile_len; r += kWave) {   // wave-uniform trip count
        const float v = r < tile_len ? s_val[r] : -INFINITY;
        const bool is_cand = r < tile_len && v >= t_lo && v > -INFINITY;
        if (is_cand) top = fmaxf(top, v);
        const uint64_t cand_lanes = __ballot(is_cand);
        if (is_cand)
            s_pair[count + (uint32_t)__popcll(cand_lanes & lanes_below)] =
                make_uint2(__float_as_uint(v), (uint32_t)(row_begin + r));
        count += (uint32_t)__popcll(cand_lanes);
    }
    top = wave_max(top);
    __builtin_amdgcn_wave_barrier();   // LDS traffic of one wavefront stays in program order
    {
        const uint32_t items = min(count + 2u, (uint32_t)kFilterPrimary + 2u);
        if ((uint32_t)lane < ((items + 15u) & ~15u)) {
            uint2 v = make_uint2(0u, 0u);
            if (lane == 0) v = make_uint2(count, __float_as_uint(t_lo));
            else if (lane == 1) v = make_uint2(__float_as_uint(top), 0u);
            else if (lane >= 2 && (uint32_t)lane < items) v = s_pair[lane - 2];
            rec[lane] = v;
        }
    }
    if (count > (uint32_t)kFilterPrimary) {
        const uint32_t padded = min((count + 15u) & ~15u, (uint32_t)a.rows_per_block);
        for (uint32_t f = lane; f < padded; f += kWave) ovf[f] = f < count ? s_pair[f] : make_uint2(0u, 0u);
    }
}

// Eight wavefronts per SIMD (at most 64 VGPRs) is what the streaming loop is tuned for; the sampler
// role must not raise the register count of the whole kernel.
template <typename T, int D, bool kStream, bool kFilter>
__global__ __launch_bounds__(kScoreThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void score_kernel(const ScoreArgs a) {
    constexpr int EPL = Chunk<T>::kElems;   // elements per lane
    constexpr int LPR = D / EPL;            // lanes per row
    constexpr int RPW = kWave / LPR;        // rows per wavefront load
    constexpr int U = kScoreUnroll;
    constexpr int WAVE_ROWS = RPW * U;
    constexpr int BLOCK_ROWS = kScoreWaves * WAVE_ROWS;
    static_assert(U <= LPR, "store lane selection needs U <= lanes per row");
    // kFilter: the tile's scores (tile role) or the sample scores (sampler role)
    __shared__ float s_val[kFilter ? kFilterMaxTileRows : 1];
    __shared__ uint2 s_pair[kFilter ? kFilterMaxTileRows : 1];

    int b, g, tile;
    if (kFilter) {   // linear grid: samplers first, then the tiles of unit 0, unit 1, ...
        const int units = a.B * a.Hkv;
        int id = (int)blockIdx.x;
        if (id < units * a.filt.spread) {   // samplers: a.filt.spread workgroups per (b, g)
            const int u = id / a.filt.spread;
            if (a.filt.spread > 1) sample_threshold_spread<T, D>(a, u / a.Hkv, u % a.Hkv, id - u * a.filt.spread, s_val);
            else sample_threshold<T, D>(a, u / a.Hkv, u % a.Hkv, s_val);
            return;
        }
        id -= units * a.filt.spread;
        const int unit = id / a.filt.n_tiles;
        tile = id - unit * a.filt.n_tiles;
        b = unit / a.Hkv;
        g = unit - b * a.Hkv;
    } else {
        b = blockIdx.z; g = blockIdx.y; tile = blockIdx.x;
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int c = lane % LPR;     // chunk of the row this lane owns
    const int grp = lane / LPR;   // which of the RPW rows of a load

    const int n = live_rows_of(a, b);
    const int row_begin = tile * a.rows_per_block;
    const int row_end = min(row_begin + a.rows_per_block, a.n_vis_max);
    const int64_t unit = (int64_t)b * a.Hkv + g;
    float* __restrict__ srow = a.scores + unit * a.n_vis_max;

    // The row's threshold word is requested up front: all but the first tiles of the launch find it
    // ready, and the request rides along with the first loads instead of delaying the tile's end.
    uint64_t hint_word = 0;
    uint32_t epoch = 0;
    if (kFilter) {
        hint_word = __hip_atomic_load(a.filt.hint + unit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        epoch = launch_epoch(a);
    }

    float qs[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) qs[i] = 0.f;
    if (row_begin < n) summed_query<T>(a, b, g, c, qs);

    const T* kbase = static_cast<const T*>(a.k_vis) + (int64_t)b * a.k_sb + (int64_t)g * a.k_sh + c * EPL;

    for (int r0 = row_begin + wave * WAVE_ROWS; r0 < row_end; r0 += BLOCK_ROWS) {
        const float val = score_pass<T, D, kStream>(a, kbase, qs, r0, n, c, grp);
        const int row = r0 + c * RPW + grp;
        if (c < U && row < row_end) {
            if (!kFilter || a.write_scores) srow[row] = val;
            if (kFilter) s_val[row - row_begin] = val;
        }
    }
    if (kFilter) {
        __syncthreads();
        if (wave != 0) return;
        emit_tile_record(a, unit, tile, row_begin, row_end, s_val, s_pair, hint_word, epoch, lane);
    }
}

// The same hand-over for scores that already exist (sv_topk_select on long rows): the sampler workgroups
// read 512 of the row's scores, the tile workgroups read their scores instead of computing them.  One
// pass over the scores replaces the two of the three-kernel selection.
__global__ __launch_bounds__(kScoreThreads) void scores_filter_kernel(const ScoreArgs a, const int groups) {
    __shared__ float s_val[kScoreWaves][kFilterMaxTileRows];
    __shared__ uint2 s_pair[kScoreWaves][kFilterMaxTileRows];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int units = a.B * a.Hkv;
    int id = (int)blockIdx.x;
    if (id < units) {   // sampler of unit id
        const int64_t unit = id;
        const int n = live_rows_of(a, id / a.Hkv);
        const int kb = a.filt.k < n ? a.filt.k : n;
        if (kb == 0 || kb == n) {   // the selection handles these rows without candidates
            if (tid == 0) publish_hint(a, unit, INFINITY);
            return;
        }
        const int rank = a.filt.rank_override > 0 ? a.filt.rank_override : sample_rank(n, kb);
        if (rank > kSample - kSample / 8) {
            if (tid == 0) publish_hint(a, unit, -INFINITY);
            return;
        }
        const float* __restrict__ srow = a.scores + unit * a.n_vis_max;
        float* samp = &s_val[0][0];
        for (int i = tid; i < kSample; i += kScoreThreads) samp[i] = srow[sample_row_of(i, n, unit)];
        __syncthreads();
        if (wave != 0) return;
        const float t_lo = rank_statistic(samp, rank, lane);
        if (tid == 0) publish_hint(a, unit, t_lo);
        return;
    }
    // A wavefront takes kFilterTilesPerWave consecutive tiles of one row (a tile is 1-2 KB of scores: with a
    // workgroup per tile the launch was bound by the life of its 22 k tiny workgroups).  The scores of all
    // its tiles are requested at once; the records follow one after the other.
    id -= units;
    const int unit = id / groups;
    const int tile0 = ((id - unit * groups) * kScoreWaves + wave) * kFilterTilesPerWave;
    if (tile0 >= a.filt.n_tiles) return;   // wave-uniform; no barrier below
    const int n = live_rows_of(a, unit / a.Hkv);
    uint64_t hint_word = __hip_atomic_load(a.filt.hint + unit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // re-read by the
    const uint32_t epoch = launch_epoch(a);                                                                      // first record if stale
    const float* __restrict__ srow = a.scores + (int64_t)unit * a.n_vis_max;
    constexpr int PER_LANE = kFilterMaxTileRows / kWave;   // scores of one tile per lane
    float v[kFilterTilesPerWave][PER_LANE];
#pragma unroll
    for (int t = 0; t < kFilterTilesPerWave; ++t) {
        const int row_begin = (tile0 + t) * a.rows_per_block;
#pragma unroll
        for (int i = 0; i < PER_LANE; ++i) {
            const int r = i * kWave + lane;
            const int row = row_begin + r;
            v[t][i] = (r < a.rows_per_block && row < n) ? srow[row] : -INFINITY;
        }
    }
#pragma unroll
    for (int t = 0; t < kFilterTilesPerWave; ++t) {
        const int tile = tile0 + t;
        if (tile >= a.filt.n_tiles) break;   // wave-uniform
        const int row_begin = tile * a.rows_per_block;
        const int row_end = min(row_begin + a.rows_per_block, a.n_vis_max);
#pragma unroll
        for (int i = 0; i < PER_LANE; ++i) s_val[wave][i * kWave + lane] = v[t][i];
        __builtin_amdgcn_wave_barrier();   // LDS traffic of one wavefront stays in program order
        emit_tile_record(a, unit, tile, row_begin, row_end, s_val[wave], s_pair[wave], hint_word, epoch, lane);
        __builtin_amdgcn_wave_barrier();
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
    dim3 block(kScoreThreads);
    if (a.filt.tiles) {
        // a sample of 256 rows (a launch so small that it waits for its samplers) is spread over several sampler workgroups
        k.filt.spread = (a.filt.n_samples == kSample / 2 && a.filt.samples) ? (kSample / 2) / sampler_round_rows<T, D>() : 1;
        const uint64_t blocks = (uint64_t)a.B * a.Hkv * ((unsigned)k.filt.spread + tiles);
        if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
        dim3 grid((unsigned)blocks);
        if (a.stream_loads) hipLaunchKernelGGL((score_kernel<T, D, true, true>), grid, block, 0, stream, k);
        else hipLaunchKernelGGL((score_kernel<T, D, false, true>), grid, block, 0, stream, k);
    } else {
        dim3 grid(tiles, (unsigned)a.Hkv, (unsigned)a.B);
        if (a.stream_loads) hipLaunchKernelGGL((score_kernel<T, D, true, false>), grid, block, 0, stream, k);
        else hipLaunchKernelGGL((score_kernel<T, D, false, false>), grid, block, 0, stream, k);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_scores_filter(const ScoreArgs& a, hipStream_t stream) {
    if (!a.filt.tiles || a.filt.tile_rows <= 0) return hipErrorInvalidValue;
    ScoreArgs k = a;
    k.rows_per_block = a.filt.tile_rows;
    k.filt.spread = 1;   // given scores are sampled in one trip by one workgroup
    const int per_group = kScoreWaves * kFilterTilesPerWave;
    const int groups = (a.filt.n_tiles + per_group - 1) / per_group;   // workgroups per row
    const uint64_t blocks = (uint64_t)a.B * a.Hkv * (1u + (uint64_t)groups);
    if (blocks == 0) return hipSuccess;
    if (blocks > 0x7fffffffull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(scores_filter_kernel, dim3((unsigned)blocks), dim3(kScoreThreads), 0, stream, k, groups);
    return hipGetLastError();
}

int score_row_granule(int dtype, int D) {
    const int epl = dtype == 0 ? 8 : 4;
    const int lpr = D / epl;
    return kScoreWaves * (kWave / lpr) * kScoreUnroll;
}

int presample_rows() { return kSample; }

int filter_tile_rows(int dtype, int D, int requested, int n_vis_max, int max_tiles) {
    const int granule = score_row_granule(dtype, D);
    int rpb = requested < granule ? granule : requested;
    rpb = (rpb + granule - 1) / granule * granule;
    if (rpb > kFilterMaxTileRows) rpb = kFilterMaxTileRows / granule * granule;
    while ((n_vis_max + rpb - 1) / rpb > max_tiles && rpb + granule <= kFilterMaxTileRows) rpb += granule;
    return (n_vis_max + rpb - 1) / rpb > max_tiles ? 0 : rpb;
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
