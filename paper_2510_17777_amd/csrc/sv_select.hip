// Step 2 of the decode path: keep the k highest-scoring visual tokens of every
// (batch, kv head) (paper section 3.2: the highest-relevance tokens are retained).
//
// Exact selection: the kept set is {j : (s_j, -j) is among the k largest pairs}, i.e.
// ties go to the lower index, and it is emitted in ascending index order.
//
// Method (the same in both launch shapes below):
//   1. a range [lo, hi] of the scores; 2. a histogram over equal-width VALUE bins of
//   that range.  The bin map s -> trunc((s - lo) * inv), clamped, is monotone in s, so
//   every score in a higher bin is strictly larger and bins above the threshold bin are
//   kept whole.  Value bins spread a bell-shaped score distribution thinly (the top bits
//   of the float pattern do not), which keeps LDS atomic conflicts rare;
//   3. a scan of the histogram from the top finds the threshold bin and how many of
//   its members are still needed; its members (at most 1024) are ranked exactly by
//   (order-preserving uint32 key, index), which yields the threshold pair;
//   4. ordered compaction: counts of kept scores per lane (one workgroup: a lane owns consecutive
//   positions) or per wavefront (parts), prefix sums, ranks inside a lane or by ballot.
// If the range is degenerate (all scores equal) or the threshold bin is overfull, an MSD
// radix select (11 + 11 + 10 bits) on the uint32 keys takes over.  All counting is
// integer: the result does not depend on the order in which lanes or workgroups run.
//
// Launch shapes:
//   * rows of at most 16384 scores: one 1024-lane workgroup per (b, g), 4, 8 or 16 scores per
//     lane in registers, exact min/max as the range;
//   * longer rows: a single compute unit cannot pull a long row from memory fast
//     enough, so the row is cut into parts of 8192 scores (at most 8 parts) and three
//     kernels run over (part, g, b):  A. per-part histogram, the range taken from a
//     64-score strided sample that every part reads identically;  B. every part sums
//     the part histograms, finds the threshold bin, counts its own scores above it and
//     stores its threshold-bin members in its own candidate slots;  C. every part
//     gathers and ranks the candidates, derives its output offset, and emits its kept
//     indices.  No workgroup waits for another (kernel boundaries are the only
//     barriers) and no global atomic is used: a returning device-scope atomic costs
//     microseconds here.  Every kernel issues all its global loads up front, because
//     one dependent round trip through memory costs more than the arithmetic.
#include "sv_score_device.h"

#include <atomic>
#include <type_traits>
#include <cfloat>
#include <cmath>

namespace sv {
namespace {

constexpr int kBins = 2048;        // single-workgroup shape, and radix digits
constexpr int kPartBins = 2048;    // multi-part shape
constexpr int kMaxCand = 1024;
constexpr int kPartLen = 8192;
constexpr int kMaxParts = 8;
constexpr int kPartItems = kPartLen / 256;    // scores per lane when a part sits in registers
constexpr int kPartCand = kMaxCand / kMaxParts;   // candidate slots per part
constexpr int kPartThreads = 256;
constexpr int kSampleLanes = 64;
constexpr int kSingleThreads = 1024;
constexpr int kSingleMaxN = 16384;   // one workgroup holds a row of up to 16 scores per lane
// sv_decode_step takes the candidate filter only for rows beyond one workgroup's reach: up to there,
// storing the scores and selecting them in one workgroup is as fast (12.5k-token rows) or faster
// (8k-token rows: 44 against 55 us per step), the sampler's chain of memory trips being what a short
// scoring launch waits for.
constexpr int kFilterMinN = kSingleMaxN;

enum : uint32_t { kFlagOk = 0, kFlagDegenerate = 1, kFlagOverfull = 2 };

struct RowParams {   // one per (b, g), written by kernel A / B, read by B / C
    float lo, inv;
    uint32_t flag, tbin, need, in_bin, pad0, pad1;
};

__device__ __forceinline__ float wave_min_f(float x) { return -wave_max(-x); }
__device__ __forceinline__ float clamp_finite(float s) { return fminf(fmaxf(s, -FLT_MAX), FLT_MAX); }

template <int NBINS>
__device__ __forceinline__ int value_bin(float s, float lo, float inv) {
    float t = (clamp_finite(s) - lo) * inv;
    t = fminf(fmaxf(t, 0.f), (float)(NBINS - 1));
    return (int)t;
}

__device__ __forceinline__ int live_rows(const int32_t* vis_len, int b, int n_max) {
    if (!vis_len) return n_max;
    const int v = vis_len[b];
    return v < 0 ? 0 : (v < n_max ? v : n_max);
}

// Block-wide inclusive scan of one value per thread (thread order = index order).
template <int NT>
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t x, uint32_t* wave_tot, int lane, int wave) {
    constexpr int NW = NT / kWave;
    const uint32_t incl = wave_inclusive_scan(x, lane);
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) base += (w < wave) ? wave_tot[w] : 0u;
    __syncthreads();
    return incl + base;
}

struct ThresholdBin { uint32_t bin, above, in_bin; };

// Scans hist[0..NBINS) from the top for the bin that holds the need-th largest entry.
// Thread t owns the NBINS/NT bins just below NBINS - t*NBINS/NT.  `res` is LDS.
template <int NT, int NBINS>
__device__ __forceinline__ ThresholdBin find_threshold_bin(const uint32_t* hist, uint32_t need, uint32_t* wave_tot,
                                                           ThresholdBin* res, int tid, int lane, int wave) {
    constexpr int BPT = NBINS / NT;
    static_assert(BPT >= 1 && BPT * NT == NBINS, "bins must divide over threads");
    uint32_t c[BPT];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { c[i] = hist[NBINS - 1 - (tid * BPT + i)]; sum += c[i]; }
    if (tid == 0) { res->bin = 0; res->above = 0; res->in_bin = 0; }
    const uint32_t incl = block_inclusive_scan<NT>(sum, wave_tot, lane, wave);
    uint32_t run = incl - sum;
    if (run < need && need <= incl) {   // exactly one thread
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            if (run < need && need <= run + c[i]) {
                res->bin = NBINS - 1 - (tid * BPT + i);
                res->above = run;
                res->in_bin = c[i];
            }
            run += c[i];
        }
    }
    __syncthreads();
    const ThresholdBin r = *res;
    __syncthreads();
    return r;
}

struct RadixShared {
    alignas(16) uint32_t hist[kBins];
    uint32_t wave_tot[16], wave_tot2[16];
    ThresholdBin tb;
};

// MSD radix select over one whole row by one workgroup of NT lanes, re-reading the
// scores in every pass; wavefront w owns the contiguous range [w*seg, (w+1)*seg).
// `map` (or nullptr) renames position j to map[j] on output; it must ascend with j.
// `stride` (in elements) separates consecutive scores in s and consecutive names in map (2: interleaved pairs).
template <int NT>
__device__ __forceinline__ void radix_select_row(RadixShared& sh, const float* __restrict__ s,
                                                 int32_t* __restrict__ out, int n, int kb, int tid, int lane, int wave,
                                                 const int32_t* map = nullptr, int stride = 1) {
    constexpr int NW = NT / kWave;
    const int seg = ((n + NW - 1) / NW + kWave - 1) / kWave * kWave;
    const int seg_items = seg / kWave;
    const int j0 = wave * seg + lane;
    const int seg_end = min(n, wave * seg + seg);
    auto key_at = [&](int i) -> uint32_t {   // 0 = "no key" (valid keys are never 0)
        const int j = j0 + i * kWave;
        return j < seg_end ? score_key(s[(int64_t)j * stride]) : 0u;
    };
    uint32_t prefix = 0, mask = 0;
    uint32_t need = (uint32_t)kb;
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const uint32_t digit_mask = pass == 2 ? 0x3FFu : 0x7FFu;
        for (int i = tid; i < kBins; i += NT) sh.hist[i] = 0;
        __syncthreads();
        for (int i = 0; i < seg_items; ++i) {
            const uint32_t key = key_at(i);
            if (key != 0u && (key & mask) == prefix) atomicAdd(&sh.hist[(key >> shift) & digit_mask], 1u);
        }
        __syncthreads();
        const ThresholdBin tb = find_threshold_bin<NT, kBins>(sh.hist, need, sh.wave_tot, &sh.tb, tid, lane, wave);
        prefix |= tb.bin << shift;
        mask |= digit_mask << shift;
        need -= tb.above;
        if (need == tb.in_bin) break;   // the whole bin is kept: no finer digit needed
    }
    // kept(j) = (key&mask) > prefix, or (key&mask) == prefix and fewer than `need` equal keys precede j
    uint32_t n_gt = 0, n_eq = 0;
    for (int i = 0; i < seg_items; ++i) {
        const uint32_t key = key_at(i);
        const uint32_t kp = key & mask;
        n_gt += __popcll(__ballot(key != 0u && kp > prefix));
        n_eq += __popcll(__ballot(key != 0u && kp == prefix));
    }
    if (lane == 0) { sh.wave_tot[wave] = n_gt; sh.wave_tot2[wave] = n_eq; }
    __syncthreads();
    uint32_t eq_before = 0, gt_before = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        eq_before += (w < wave) ? sh.wave_tot2[w] : 0u;
        gt_before += (w < wave) ? sh.wave_tot[w] : 0u;
    }
    uint32_t pos = gt_before + (eq_before < need ? eq_before : need);
    uint32_t eq_seen = eq_before;
    const uint64_t lane_lt = (1ull << lane) - 1ull;
    for (int i = 0; i < seg_items; ++i) {
        const uint32_t key = key_at(i);
        const uint32_t kp = key & mask;
        const bool is_eq = key != 0u && kp == prefix;
        const uint64_t eq_ballot = __ballot(is_eq);
        const uint32_t eq_rank = eq_seen + (uint32_t)__popcll(eq_ballot & lane_lt);
        const bool keep = (key != 0u && kp > prefix) || (is_eq && eq_rank < need);
        const uint64_t keep_ballot = __ballot(keep);
        const uint32_t slot = pos + (uint32_t)__popcll(keep_ballot & lane_lt);
        if (keep && slot < (uint32_t)kb) {   // slot < kb holds for finite scores
            const int j = j0 + i * kWave;
            out[slot] = map ? map[(int64_t)j * stride] : j;
        }
        pos += (uint32_t)__popcll(keep_ballot);
        eq_seen += (uint32_t)__popcll(eq_ballot);
    }
}

// Exact ranking of the threshold bin's members held in LDS: finds the member with rank
// need-1 in (score descending, index ascending) order.  Threads stride over members; the
// members are read eight at a time so that a pass costs one LDS round trip, not eight.
template <int NT>
__device__ __forceinline__ void rank_candidates(const uint32_t* cand_key, const int32_t* cand_idx, uint32_t n_cand,
                                                uint32_t need, uint32_t* thr_key, int32_t* thr_idx, int tid) {
    constexpr uint32_t R = 8;
    for (uint32_t c = tid; c < n_cand; c += NT) {
        const uint32_t my_key = cand_key[c];
        const int32_t my_idx = cand_idx[c];
        uint32_t rank = 0;
        for (uint32_t u0 = 0; u0 < n_cand; u0 += R) {
            uint32_t ok[R];
            int32_t oi[R];
#pragma unroll
            for (uint32_t r = 0; r < R; ++r) {
                const uint32_t u = min(u0 + r, n_cand - 1);
                ok[r] = cand_key[u];
                oi[r] = cand_idx[u];
            }
#pragma unroll
            for (uint32_t r = 0; r < R; ++r)
                rank += (u0 + r < n_cand && (ok[r] > my_key || (ok[r] == my_key && oi[r] < my_idx))) ? 1u : 0u;
        }
        if (rank == need - 1) { *thr_key = my_key; *thr_idx = my_idx; }
    }
}

// Writes count and the -1 padding of one (b, g); returns true when nothing else is left
// to do (k_b == 0, or k_b == n where the kept set is every index).
template <int NT>
__device__ __forceinline__ bool emit_trivial(const SelectArgs& a, int64_t unit, int n, int kb, int first,
                                             int stride_blocks, int tid) {
    int32_t* out = a.idx + unit * a.k;
    if (first == 0 && tid == 0) a.count[unit] = kb;
    for (int i = kb + first * NT + tid; i < a.k; i += stride_blocks * NT) out[i] = -1;
    if (kb == 0) return true;
    if (kb == n) {
        for (int i = first * NT + tid; i < n; i += stride_blocks * NT) out[i] = i;
        return true;
    }
    return false;
}

// ------------------------------------------------------------------ single workgroup
struct SingleShared {
    RadixShared rx;
    uint32_t cand_key[kMaxCand];
    int32_t cand_idx[kMaxCand];
    float wave_min[16], wave_max[16];
    uint32_t n_cand, thr_key;
    int32_t thr_idx;
};

// Exact top-kb of the n <= ITEMS*1024 scores at s (global or LDS) by one 1024-lane workgroup;
// out[0..kb) receives the kept positions (renamed through `map` when given) in ascending order.
// Requires 0 < kb < n.  Lane t owns the ITEMS consecutive positions from t*ITEMS on, so that thread
// order is position order: the output slot of a lane's first kept score is one prefix sum over the
// lanes' kept counts away, and a score's bin is computed once and kept in a register.
// kVec: the scores and their names sit interleaved in LDS -- s points at 16-byte aligned (score, name) pairs,
// ITEMS*1024 of them readable, map is ignored -- and are read with 128-bit loads, two pairs at a time.
// With have_range the caller vouches that lo_hint <= every score and supplies an upper value for the
// binning (scores above it share the top bin); the workgroup then skips its own min/max pass.
// The ITEMS consecutive scores of lane `tid` of a row with n_cap readable scores at s, requested without
// knowing how many of them are live (0 past the capacity): a caller that fetches them before the row's length has
// arrived saves one trip through memory.
template <int ITEMS>
__device__ __forceinline__ void load_lane_items(const float* __restrict__ s, int n_cap, int tid, float (&vals)[ITEMS]) {
    const int j0 = tid * ITEMS;
    const int readable = min(max(n_cap - j0, 0), ITEMS);
    if ((reinterpret_cast<uintptr_t>(s) & 15u) == 0) {   // block-uniform: 128-bit loads inside the row
#pragma unroll
        for (int i = 0; i < ITEMS; i += 4) {
            if (i + 4 <= readable) {
                const float4 v = *reinterpret_cast<const float4*>(s + j0 + i);
                vals[i] = v.x; vals[i + 1] = v.y; vals[i + 2] = v.z; vals[i + 3] = v.w;
            } else {
#pragma unroll
                for (int e = i; e < i + 4; ++e) vals[e] = e < readable ? s[j0 + e] : 0.f;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) vals[i] = i < readable ? s[j0 + i] : 0.f;
    }
}

// pre: the lane's scores as load_lane_items fetched them (nullptr: fetched here, once n is known).
template <int ITEMS, bool kVec>
__device__ __forceinline__ void select_block(SingleShared& sh, const float* __restrict__ s, int32_t* __restrict__ out,
                                             int n, int kb, int tid, int lane, int wave,
                                             const int32_t* map = nullptr, bool have_range = false,
                                             float lo_hint = 0.f, float hi_hint = 0.f,
                                             const float (*pre)[ITEMS] = nullptr) {
    constexpr int NT = kSingleThreads, NW = NT / kWave;
    static_assert(!kVec || ITEMS % 2 == 0, "vector reads take two pairs");
    const int j0 = tid * ITEMS;
    const int my_items = min(max(n - j0, 0), ITEMS);
    float vals[ITEMS];
    int32_t pair_name[kVec ? ITEMS : 1];
    if (pre) {   // compile-time known at every call site
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) vals[i] = i < my_items ? (*pre)[i] : 0.f;
    } else if (kVec) {
#pragma unroll
        for (int i = 0; i < ITEMS; i += 2) {
            const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint2*>(s) + j0 + i);
            vals[i] = __uint_as_float(v.x); pair_name[i] = (int32_t)v.y;
            vals[i + 1] = __uint_as_float(v.z); pair_name[i + 1] = (int32_t)v.w;
        }
    } else if ((reinterpret_cast<uintptr_t>(s) & 15u) == 0) {   // block-uniform: 128-bit loads inside the row
#pragma unroll
        for (int i = 0; i < ITEMS; i += 4) {
            if (i + 4 <= my_items) {
                const float4 v = *reinterpret_cast<const float4*>(s + j0 + i);
                vals[i] = v.x; vals[i + 1] = v.y; vals[i + 2] = v.z; vals[i + 3] = v.w;
            } else {
#pragma unroll
                for (int e = i; e < i + 4; ++e) vals[e] = e < my_items ? s[j0 + e] : 0.f;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) vals[i] = i < my_items ? s[j0 + i] : 0.f;
    }

    float lo = FLT_MAX, hi = -FLT_MAX;
    if (!have_range) {   // block-uniform
#pragma unroll
        for (int i = 0; i < ITEMS; ++i)
            if (i < my_items) { const float v = clamp_finite(vals[i]); lo = fminf(lo, v); hi = fmaxf(hi, v); }
        lo = wave_min_f(lo);
        hi = wave_max(hi);
        if (lane == 0) { sh.wave_min[wave] = lo; sh.wave_max[wave] = hi; }
    }
    for (int i = tid; i < kBins; i += NT) sh.rx.hist[i] = 0;
    if (tid == 0) { sh.n_cand = 0; sh.thr_key = 0; sh.thr_idx = -1; }
    __syncthreads();
    if (have_range) {
        lo = clamp_finite(lo_hint);
        hi = clamp_finite(hi_hint);
    } else {
#pragma unroll
        for (int w = 0; w < NW; ++w) { lo = fminf(lo, sh.wave_min[w]); hi = fmaxf(hi, sh.wave_max[w]); }
    }
    const float inv = (float)kBins / (hi - lo);
    const bool spread = hi > lo && inv > 0.f && inv <= FLT_MAX;   // block-uniform

    bool done = false;
    if (spread) {
        int bin[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            bin[i] = -1;   // below every bin: never kept, never a candidate
            if (i < my_items) {
                bin[i] = value_bin<kBins>(vals[i], lo, inv);
                atomicAdd(&sh.rx.hist[bin[i]], 1u);
            }
        }
        __syncthreads();
        const ThresholdBin tb =
            find_threshold_bin<NT, kBins>(sh.rx.hist, (uint32_t)kb, sh.rx.wave_tot, &sh.rx.tb, tid, lane, wave);
        const int tbin = (int)tb.bin;
        const uint32_t need = (uint32_t)kb - tb.above;
        if (tb.in_bin <= (uint32_t)kMaxCand) {
            uint32_t thr_key = 0;
            int32_t thr_idx = 0x7fffffff;   // whole bin kept unless the ranking says otherwise
            if (need < tb.in_bin) {
#pragma unroll
                for (int i = 0; i < ITEMS; ++i)
                    if (bin[i] == tbin) {
                        const uint32_t slot = atomicAdd(&sh.n_cand, 1u);
                        if (slot < (uint32_t)kMaxCand) {
                            sh.cand_key[slot] = score_key(vals[i]);
                            sh.cand_idx[slot] = j0 + i;
                        }
                    }
                __syncthreads();
                rank_candidates<NT>(sh.cand_key, sh.cand_idx, tb.in_bin, need, &sh.thr_key, &sh.thr_idx, tid);
                __syncthreads();
                thr_key = sh.thr_key;
                thr_idx = sh.thr_idx;
            }
            uint32_t keep_bits = 0;
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                bool keep = bin[i] > tbin;
                if (bin[i] == tbin) {
                    const uint32_t key = score_key(vals[i]);
                    keep = key > thr_key || (key == thr_key && (j0 + i) <= thr_idx);
                }
                keep_bits |= keep ? (1u << i) : 0u;
            }
            const uint32_t n_keep = (uint32_t)__popc(keep_bits);
            const uint32_t wincl = wave_inclusive_scan(n_keep, lane);
            if (lane == kWave - 1) sh.rx.wave_tot2[wave] = wincl;
            __syncthreads();
            uint32_t pos = wincl - n_keep;
#pragma unroll
            for (int w = 0; w < NW; ++w) pos += (w < wave) ? sh.rx.wave_tot2[w] : 0u;
            if (keep_bits) {
                int32_t name[ITEMS];
                if (kVec) {
#pragma unroll
                    for (int i = 0; i < ITEMS; ++i) name[i] = pair_name[i];
                } else {
#pragma unroll
                    for (int i = 0; i < ITEMS; ++i) name[i] = (map && i < my_items) ? map[j0 + i] : j0 + i;
                }
#pragma unroll
                for (int i = 0; i < ITEMS; ++i)
                    if (((keep_bits >> i) & 1u) && pos < (uint32_t)kb) out[pos++] = name[i];   // pos < kb holds
            }
            done = true;
        }
    }
    if (!done) {   // block-uniform
        __syncthreads();
        if (kVec) radix_select_row<NT>(sh.rx, s, out, n, kb, tid, lane, wave, reinterpret_cast<const int32_t*>(s) + 1, 2);
        else radix_select_row<NT>(sh.rx, s, out, n, kb, tid, lane, wave, map);
    }
}

__global__ __launch_bounds__(kSingleThreads) void select_single_kernel(const SelectArgs a) {
    __shared__ SingleShared sh;
    const int g = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const float* s = a.scores + unit * a.n_vis_max;
    int32_t* out = a.idx + unit * a.k;
    // Scores per lane by the row's CAPACITY, so that they can be requested before the row's length has arrived
    // (rows past the length are masked afterwards): one trip through memory instead of two.
    if (a.k == 0 || !a.scores) {   // nothing to keep (a text-only step passes no scores): count and padding only
        const int n = live_rows(a.vis_len, b, a.n_vis_max);
        emit_trivial<kSingleThreads>(a, unit, n, 0, 0, 1, tid);
        return;
    }
    auto run = [&](auto items_tag) {
        constexpr int ITEMS = decltype(items_tag)::value;
        float pre[ITEMS];
        load_lane_items<ITEMS>(s, a.n_vis_max, tid, pre);
        const int n = live_rows(a.vis_len, b, a.n_vis_max);
        const int kb = a.k < n ? a.k : n;
        if (emit_trivial<kSingleThreads>(a, unit, n, kb, 0, 1, tid)) return;
        select_block<ITEMS, false>(sh, s, out, n, kb, tid, lane, wave, nullptr, false, 0.f, 0.f, &pre);
    };
    if (a.n_vis_max <= 4 * kSingleThreads) run(std::integral_constant<int, 4>{});         // block-uniform
    else if (a.n_vis_max <= 8 * kSingleThreads) run(std::integral_constant<int, 8>{});
    else run(std::integral_constant<int, kSingleMaxN / kSingleThreads>{});
}

// ------------------------------------------------------------------ candidate-filtered shape
// One workgroup per (b, g).  The scoring kernel left, per tile of the row, a 512-byte record
// {count; the first 62 (score, row) pairs >= t_lo in row order}; the records of a row are one
// contiguous block, fetched in a single trip through memory (a second one brings the overflow of
// the few fuller tiles).  Prefix sums of the counts pack the candidates, still in row order, in
// LDS; then the same on-chip selection as for a short row runs on them, positions renamed to the
// original rows.  If fewer than k_b candidates exist (t_lo was too high) or more than fit, the
// workgroup selects from the full score row.
constexpr int kSmallLaunchTiles = 1536;   // scoring launches up to this many tiles sample 256 rows per (b, g) instead of 512
constexpr int kFiltCap = 16384;                      // candidates ranked on chip (their scores and rows fill most of the LDS)
constexpr int kFiltMaxTiles = 256;
constexpr int kFiltPrimary = kFilterRecordPairs;     // pairs in a primary record
constexpr int kFiltRec16 = kFiltPrimary / 2 + 1;     // 16-byte words per primary record
constexpr int kFiltLoads = kFiltMaxTiles * kFiltRec16 / kSingleThreads;

struct FilteredShared {
    SingleShared sel;
    alignas(16) uint2 c_pair[kFiltCap];      // (score bits, row) of the candidates, in row order
    alignas(16) uint32_t tile_cnt[kFiltMaxTiles];
    float tile_tlo[kFiltMaxTiles];          // the threshold each tile used
    float tile_top[kFiltMaxTiles];          // the largest candidate score of each tile
    alignas(16) uint32_t tile_off[kFiltMaxTiles + 4];   // exclusive prefix sums of the tile counts, then their total
    uint32_t max_cnt;                        // the largest tile count
    float tlo_min[4], tlo_max[4], top_max[4];
    uint32_t n_at_or_above;
};

template <typename T, int D>
__global__ __launch_bounds__(kSingleThreads) void select_filtered_kernel(const SelectArgs a, const ScoreArgs sc) {
    constexpr int NT = kSingleThreads;
    const FilterArgs& f = sc.filt;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    FilteredShared& sh = *reinterpret_cast<FilteredShared*>(smem_raw);
    const int g = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    // one trip: word (tid + u*NT) of the row's block of records, requested before the row's length is
    // known (records of tiles past the live rows hold stale words, ignored below)
    const uint4* recs = f.tiles + unit * f.n_tiles * kFiltRec16;
    const uint2* ovf = f.overflow + unit * f.n_tiles * f.tile_rows;
    uint4 word[kFiltLoads];
#pragma unroll
    for (int u = 0; u < kFiltLoads; ++u) {
        const int w = tid + u * NT;
        word[u] = make_uint4(0u, 0u, 0u, 0u);
        if (w < f.n_tiles * kFiltRec16) word[u] = recs[w];
    }
    // The scoring launch that read the generation word is over, the next one has not begun: bump it.
    if (unit == 0 && tid == 0) f.gen[0] = f.gen[0] + 1u;
    const int n = live_rows(a.vis_len, b, a.n_vis_max);
    const int kb = a.k < n ? a.k : n;
    if (emit_trivial<NT>(a, unit, n, kb, 0, 1, tid)) return;
    int32_t* __restrict__ out = a.idx + unit * a.k;
    const int live_tiles = (n + f.tile_rows - 1) / f.tile_rows;   // <= kFiltMaxTiles (checked by the host)
#pragma unroll
    for (int u = 0; u < kFiltLoads; ++u) {
        const int w = tid + u * NT;
        if (w % kFiltRec16 == 0 && w < kFiltMaxTiles * kFiltRec16) {
            const bool live = w < live_tiles * kFiltRec16;
            sh.tile_cnt[w / kFiltRec16] = live ? min(word[u].x, (uint32_t)f.tile_rows) : 0u;
            sh.tile_tlo[w / kFiltRec16] = live ? __uint_as_float(word[u].y) : 0.f;
            sh.tile_top[w / kFiltRec16] = live ? __uint_as_float(word[u].z) : -INFINITY;
        }
    }
    if (tid == 0) sh.n_at_or_above = 0;
    __syncthreads();
    if (tid < kFiltMaxTiles) {   // wavefronts 0..3: the spread of the thresholds the tiles used
        const float t = sh.tile_tlo[tid];
        const float lo = wave_min_f(tid < live_tiles ? t : INFINITY);
        const float hi = wave_max(tid < live_tiles ? t : -INFINITY);
        const float top = wave_max(tid < live_tiles ? sh.tile_top[tid] : -INFINITY);
        if (lane == 0) { sh.tlo_min[wave] = lo; sh.tlo_max[wave] = hi; sh.top_max[wave] = top; }
    } else if (wave == kFiltMaxTiles / kWave) {   // one more wavefront: prefix sums of the tile counts, four tiles per lane
        static_assert(kFiltMaxTiles == 4 * kWave, "four tiles per lane");
        const uint4 c4 = reinterpret_cast<const uint4*>(sh.tile_cnt)[lane];
        const uint32_t s4 = c4.x + c4.y + c4.z + c4.w;
        const uint32_t incl = wave_inclusive_scan(s4, lane);
        const uint32_t base = incl - s4;
        reinterpret_cast<uint4*>(sh.tile_off)[lane] =
            make_uint4(base, base + c4.x, base + c4.x + c4.y, base + c4.x + c4.y + c4.z);
        const float big = wave_max((float)max(max(c4.x, c4.y), max(c4.z, c4.w)));   // counts <= 512: exact in fp32
        if (lane == kWave - 1) { sh.tile_off[kFiltMaxTiles] = incl; sh.max_cnt = (uint32_t)big; }
    }
    __syncthreads();
    const uint32_t m = sh.tile_off[kFiltMaxTiles];   // candidates of the row

    // Whole-row selection for a row the filter missed.  If the scoring launch did not store the scores,
    // this workgroup computes the row's scores first (slow: one compute unit streams the row's keys).
    auto select_whole_row = [&]() {
        float* row_scores = sc.scores + unit * a.n_vis_max;
        if (!sc.write_scores) {
            score_row_by_workgroup<T, D>(sc, b, g, row_scores);
            __syncthreads();
        }
        radix_select_row<NT>(sh.sel.rx, row_scores, out, n, kb, tid, lane, wave);
    };
    if (m < (uint32_t)kb || m > (uint32_t)kFiltCap) {   // block-uniform: too few or too many candidates
        select_whole_row();
        return;
    }
#pragma unroll
    for (int u = 0; u < kFiltLoads; ++u) {
        const int w = tid + u * NT;
        const int tile = w / kFiltRec16, q = w % kFiltRec16;
        if (tile < live_tiles && q > 0) {
            const uint32_t off = sh.tile_off[tile], cnt = sh.tile_cnt[tile];
            const uint32_t e = 2 * (q - 1);
            if (e < cnt) sh.c_pair[off + e] = make_uint2(word[u].x, word[u].y);
            if (e + 1 < cnt) sh.c_pair[off + e + 1] = make_uint2(word[u].z, word[u].w);
        }
    }
    // The fuller tiles: their remaining pairs from the overflow rows (which hold all pairs of such a tile).
    // Lane q of a tile's 31 takes pairs 62 + (q - 1) + 31 i.  The loads of i < 2 (tiles of up to 124
    // candidates) are all issued before any is used: one more trip through memory, not one per tile.
    if (sh.max_cnt > (uint32_t)kFiltPrimary) {   // block-uniform
        constexpr uint32_t kStride = kFiltRec16 - 1;
        uint2 ov[kFiltLoads][2];
#pragma unroll
        for (int u = 0; u < kFiltLoads; ++u) {
            const int w = tid + u * NT;
            const int tile = w / kFiltRec16, q = w % kFiltRec16;
            const uint32_t cnt = (tile < live_tiles && q > 0) ? sh.tile_cnt[tile] : 0u;
#pragma unroll
            for (uint32_t i = 0; i < 2; ++i) {
                const uint32_t x = kFiltPrimary + (q - 1) + i * kStride;
                ov[u][i] = make_uint2(0u, 0u);
                if (x < cnt) ov[u][i] = ovf[(int64_t)tile * f.tile_rows + x];
            }
        }
#pragma unroll
        for (int u = 0; u < kFiltLoads; ++u) {
            const int w = tid + u * NT;
            const int tile = w / kFiltRec16, q = w % kFiltRec16;
            if (tile < live_tiles && q > 0) {
                const uint32_t off = sh.tile_off[tile], cnt = sh.tile_cnt[tile];
#pragma unroll
                for (uint32_t i = 0; i < 2; ++i) {
                    const uint32_t x = kFiltPrimary + (q - 1) + i * kStride;
                    if (x < cnt) sh.c_pair[off + x] = ov[u][i];
                }
                for (uint32_t x = kFiltPrimary + (q - 1) + 2 * kStride; x < cnt; x += kStride)   // rare: > 124 candidates
                    sh.c_pair[off + x] = ovf[(int64_t)tile * f.tile_rows + x];
            }
        }
    }
    __syncthreads();
    // Tiles that used different thresholds: a score below its tile's threshold is missing here, so
    // the k_b-th largest candidate must not lie below the largest threshold used.
    const float t_min = fminf(fminf(sh.tlo_min[0], sh.tlo_min[1]), fminf(sh.tlo_min[2], sh.tlo_min[3]));
    const float t_max = fmaxf(fmaxf(sh.tlo_max[0], sh.tlo_max[1]), fmaxf(sh.tlo_max[2], sh.tlo_max[3]));
    if (t_min != t_max) {   // block-uniform
        uint32_t c = 0;
        for (uint32_t i = tid; i < m; i += NT) c += __uint_as_float(sh.c_pair[i].x) >= t_max ? 1u : 0u;
        c = wave_inclusive_scan(c, lane);
        if (lane == kWave - 1 && c > 0) atomicAdd(&sh.n_at_or_above, c);
        __syncthreads();
        if (sh.n_at_or_above < (uint32_t)kb) {
            select_whole_row();
            return;
        }
    }
    if (m == (uint32_t)kb) {   // every candidate is kept
        for (uint32_t i = tid; i < m; i += NT) out[i] = (int32_t)sh.c_pair[i].y;
        return;
    }
    // every candidate is >= its tile's threshold >= t_min, and none exceeds the largest tile maximum
    const float top = fmaxf(fmaxf(sh.top_max[0], sh.top_max[1]), fmaxf(sh.top_max[2], sh.top_max[3]));
    const bool have_range = t_min > -INFINITY && top < INFINITY && top > t_min;
    const float* pairs = reinterpret_cast<const float*>(sh.c_pair);
    if (m <= (uint32_t)(8 * NT))   // block-uniform: the usual case keeps eight candidates per lane
        select_block<8, true>(sh.sel, pairs, out, (int)m, kb, tid, lane, wave, nullptr, have_range, t_min, top);
    else
        select_block<kFiltCap / NT, true>(sh.sel, pairs, out, (int)m, kb, tid, lane, wave, nullptr, have_range, t_min, top);
}

// ------------------------------------------------------------------ multi-part shape
struct PartView {   // how one 256-lane workgroup sees its part of the row
    int items;      // item slots per lane: part_len / 256
    int j0;         // index of this lane's item 0
    int my_items;   // live items of this lane
};

__device__ __forceinline__ PartView part_view(int part, int part_len, int n, int lane, int wave) {
    PartView v;
    v.items = part_len / kPartThreads;
    const int wave_len = part_len / (kPartThreads / kWave);   // contiguous range of one wavefront
    v.j0 = part * part_len + wave * wave_len + lane;
    const int end = min(n, part * part_len + (wave + 1) * wave_len);
    v.my_items = v.j0 < end ? (end - v.j0 + kWave - 1) / kWave : 0;
    return v;
}

// Runs the statement(s) on this lane's live items with `i` the item number and `v` its
// score: from registers when ITEMS > 0, else from memory.
#define SV_PART_ITEMS(...)                                                                          \
    if (ITEMS > 0) {                                                                                \
        _Pragma("unroll") for (int i = 0; i < (ITEMS > 0 ? ITEMS : 1); ++i) {                       \
            if (i < pv.my_items) { const float v = vals[i]; __VA_ARGS__ }                           \
        }                                                                                           \
    } else {                                                                                        \
        for (int i = 0; i < pv.my_items; ++i) { const float v = s[pv.j0 + i * kWave]; __VA_ARGS__ } \
    }

// Issues the loads of this lane's items (register-resident shape only).
#define SV_PART_LOAD()                                                      \
    float vals[ITEMS > 0 ? ITEMS : 1];                                      \
    if (ITEMS > 0) {                                                        \
        _Pragma("unroll") for (int i = 0; i < (ITEMS > 0 ? ITEMS : 1); ++i) \
            vals[i] = i < pv.my_items ? s[pv.j0 + i * kWave] : 0.f;         \
    }                                                                       \
    (void)vals;

struct PartMeta { uint32_t above, n_cand; };   // n_cand > kPartCand: this part overflowed its slots

struct SelectWorkspace {
    uint16_t* part_hist;    // [units][parts][kPartBins], saturating at 65535
    PartMeta* part_meta;    // [units][parts]
    uint2* cand;            // [units][parts][kPartCand]  (key, index); key 0 = empty slot
    RowParams* params;      // [units]
};

// A. per-part value histogram; the bin range comes from a strided 64-score sample.
template <int ITEMS>
__global__ __launch_bounds__(kPartThreads) void select_hist_kernel(const SelectArgs a, const SelectWorkspace ws,
                                                                  const int parts, const int part_len) {
    __shared__ uint32_t hist[kPartBins];
    __shared__ float range_sh[2];
    const int part = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const float* __restrict__ s = a.scores + unit * a.n_vis_max;
    const int n = live_rows(a.vis_len, b, a.n_vis_max);
    const int kb = a.k < n ? a.k : n;
    if (kb == 0 || kb == n) return;   // kernel C handles these without the histogram

    const PartView pv = part_view(part, part_len, n, lane, wave);
    SV_PART_LOAD()
    // Range estimate: every part of the row reads the same sample, hence the same range.
    if (wave == 0) {
        const float sv = clamp_finite(s[(int)(((int64_t)lane * n) / kSampleLanes)]);
        const float lo = wave_min_f(sv), hi = wave_max(sv);
        if (lane == 0) { range_sh[0] = lo; range_sh[1] = hi; }
    }
#pragma unroll
    for (int i = 0; i < kPartBins / kPartThreads; ++i) hist[tid + i * kPartThreads] = 0;
    __syncthreads();
    // widen by the sample range on both sides: scores outside the sample's span still
    // land in distinct bins; anything beyond clamps into the end bins
    const float r = range_sh[1] - range_sh[0];
    const float lo_w = range_sh[0] - r;
    const float inv = (float)kPartBins / (3.f * r);
    const bool ok = r > 0.f && r <= FLT_MAX / 4.f && inv > 0.f && inv <= FLT_MAX;
    if (part == 0 && tid == 0) {
        RowParams p{};
        p.lo = lo_w; p.inv = inv; p.flag = ok ? kFlagOk : kFlagDegenerate;
        ws.params[unit] = p;
    }
    if (!ok) return;   // block-uniform, and the same in every part of the row

    SV_PART_ITEMS(atomicAdd(&hist[value_bin<kPartBins>(v, lo_w, inv)], 1u);)
    __syncthreads();
    uint16_t* dst = ws.part_hist + (unit * parts + part) * kPartBins;
#pragma unroll
    for (int i = 0; i < kPartBins / kPartThreads; ++i) {
        const uint32_t c = hist[tid + i * kPartThreads];
        dst[tid + i * kPartThreads] = (uint16_t)(c < 65535u ? c : 65535u);
    }
}

// B. threshold bin of the row; this part's count above it; its threshold-bin members.
template <int ITEMS>
__global__ __launch_bounds__(kPartThreads) void select_threshold_kernel(const SelectArgs a, const SelectWorkspace ws,
                                                                       const int parts, const int part_len) {
    constexpr int BPT = kPartBins / kPartThreads;   // 8 consecutive bins per thread
    __shared__ uint32_t hist[kPartBins];
    __shared__ uint2 cand_sh[kPartCand];
    __shared__ uint32_t wave_tot[4];
    __shared__ ThresholdBin tb_sh;
    __shared__ uint32_t n_cand_sh, saturated_sh;
    const int part = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const float* __restrict__ s = a.scores + unit * a.n_vis_max;
    const int n = live_rows(a.vis_len, b, a.n_vis_max);
    const int kb = a.k < n ? a.k : n;
    if (kb == 0 || kb == n) return;

    // all global loads first: parameters, the part histograms (8 bins per thread per part), own scores
    const RowParams rp = ws.params[unit];
    const int live_parts = (n + part_len - 1) / part_len;
    const uint16_t* src = ws.part_hist + unit * parts * kPartBins + tid * BPT;
    uint4 hraw[kMaxParts];
#pragma unroll
    for (int p = 0; p < kMaxParts; ++p)
        hraw[p] = p < live_parts ? *reinterpret_cast<const uint4*>(src + p * kPartBins) : make_uint4(0, 0, 0, 0);
    const PartView pv = part_view(part, part_len, n, lane, wave);
    SV_PART_LOAD()
    if (rp.flag != kFlagOk) return;

    uint32_t sum[BPT];
    bool sat = false;
#pragma unroll
    for (int i = 0; i < BPT; ++i) sum[i] = 0;
#pragma unroll
    for (int p = 0; p < kMaxParts; ++p) {
        const uint32_t w[4] = {hraw[p].x, hraw[p].y, hraw[p].z, hraw[p].w};
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            const uint32_t c = (w[i / 2] >> (16 * (i & 1))) & 0xFFFFu;
            sat |= c == 65535u;
            sum[i] += c;
        }
    }
    if (tid == 0) { n_cand_sh = 0; saturated_sh = 0; }
#pragma unroll
    for (int i = 0; i < BPT; ++i) hist[tid * BPT + i] = sum[i];
    if (tid < kPartCand) cand_sh[tid] = make_uint2(0u, 0u);
    __syncthreads();
    if (sat) saturated_sh = 1;   // a 16-bit count hit its ceiling: the sums cannot be trusted
    const ThresholdBin tb =
        find_threshold_bin<kPartThreads, kPartBins>(hist, (uint32_t)kb, wave_tot, &tb_sh, tid, lane, wave);
    const bool overfull = tb.in_bin > (uint32_t)kMaxCand || saturated_sh != 0;
    if (part == 0 && tid == 0) {
        RowParams* p = ws.params + unit;
        p->tbin = tb.bin; p->need = (uint32_t)kb - tb.above; p->in_bin = tb.in_bin;
        if (overfull) p->flag = kFlagOverfull;
    }
    if (overfull) return;   // the same decision in every part of the row

    const int tbin = (int)tb.bin;
    uint32_t n_above = 0;
    SV_PART_ITEMS({
        const int bin = value_bin<kPartBins>(v, rp.lo, rp.inv);
        n_above += bin > tbin ? 1u : 0u;
        if (bin == tbin) {
            const uint32_t slot = atomicAdd(&n_cand_sh, 1u);   // LDS
            if (slot < (uint32_t)kPartCand) cand_sh[slot] = make_uint2(score_key(v), (uint32_t)(pv.j0 + i * kWave));
        }
    })
    n_above = wave_inclusive_scan(n_above, lane);   // integer sum over the workgroup
    if (lane == kWave - 1) wave_tot[wave] = n_above;
    __syncthreads();
    if (tid < kPartCand) ws.cand[(unit * parts + part) * kPartCand + tid] = cand_sh[tid];
    if (tid == 0) {
        PartMeta m;
        m.above = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        m.n_cand = n_cand_sh;
        ws.part_meta[unit * parts + part] = m;
    }
}

// C. exact threshold from the candidates, output offset of this part, ordered emission.
template <int ITEMS>
__global__ __launch_bounds__(kPartThreads) void select_emit_kernel(const SelectArgs a, const SelectWorkspace ws,
                                                                  const int parts, const int part_len) {
    __shared__ union {
        uint64_t cand[kMaxCand];   // (key << 32) | ~index: larger = earlier in (score desc, index asc) order
        RadixShared rx;
    } sh;
    __shared__ uint32_t part_kept[kMaxParts], part_above[kMaxParts];
    __shared__ uint32_t wave_tot[4];
    __shared__ uint32_t n_cand_sh, overflow_sh;
    __shared__ uint64_t thr_sh;
    const int part = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const float* __restrict__ s = a.scores + unit * a.n_vis_max;
    int32_t* __restrict__ out = a.idx + unit * a.k;
    const int n = live_rows(a.vis_len, b, a.n_vis_max);
    const int kb = a.k < n ? a.k : n;
    if (emit_trivial<kPartThreads>(a, unit, n, kb, part, parts, tid)) return;

    // all global loads first
    const RowParams rp = ws.params[unit];
    const int live_parts = (n + part_len - 1) / part_len;
    uint2 craw[kMaxParts / 2];   // thread t: slot t%128 of parts 2m + t/128
#pragma unroll
    for (int m = 0; m < kMaxParts / 2; ++m) {
        const int p = 2 * m + tid / kPartCand;
        craw[m] = p < live_parts ? ws.cand[(unit * parts + p) * kPartCand + (tid % kPartCand)] : make_uint2(0u, 0u);
    }
    PartMeta meta{};
    if (tid < live_parts) meta = ws.part_meta[unit * parts + tid];
    const PartView pv = part_view(part, part_len, n, lane, wave);
    SV_PART_LOAD()

    if (rp.flag != kFlagOk) {   // degenerate range or overfull threshold bin: one workgroup redoes the row
        if (part == 0) radix_select_row<kPartThreads>(sh.rx, s, out, n, kb, tid, lane, wave);
        return;
    }
    if (tid == 0) { n_cand_sh = 0; overflow_sh = 0; thr_sh = 0; }   // threshold 0: the whole bin is kept
    if (tid < kMaxParts) { part_kept[tid] = 0; part_above[tid] = 0; }
    __syncthreads();
    if (tid < live_parts) {
        part_above[tid] = meta.above;
        if (meta.n_cand > (uint32_t)kPartCand) overflow_sh = 1;
    }
#pragma unroll
    for (int m = 0; m < kMaxParts / 2; ++m) {
        if (craw[m].x != 0u) {
            const uint32_t slot = atomicAdd(&n_cand_sh, 1u);   // LDS; order is irrelevant to the ranking
            sh.cand[slot] = ((uint64_t)craw[m].x << 32) | (uint64_t)(0xFFFFFFFFu - craw[m].y);
        }
    }
    __syncthreads();
    if (overflow_sh) {   // a part had more threshold-bin members than slots (block-uniform)
        __syncthreads();
        if (part == 0) radix_select_row<kPartThreads>(sh.rx, s, out, n, kb, tid, lane, wave);
        return;
    }
    const int tbin = (int)rp.tbin;
    const uint32_t need = rp.need, n_cand = n_cand_sh;
    if (need < n_cand) {
        for (uint32_t c = tid; c < n_cand; c += kPartThreads) {
            const uint64_t mine = sh.cand[c];
            uint32_t rank = 0;
#pragma unroll 8
            for (uint32_t u = 0; u < n_cand; ++u) rank += sh.cand[u] > mine ? 1u : 0u;
            if (rank == need - 1) thr_sh = mine;
        }
    }
    __syncthreads();
    const uint64_t thr = thr_sh;
    // kept threshold-bin members of the parts before this one
    for (uint32_t c = tid; c < n_cand; c += kPartThreads) {
        const uint64_t e = sh.cand[c];
        const int p = (int)(0xFFFFFFFFu - (uint32_t)e) / part_len;
        if (e >= thr && p < part) atomicAdd(&part_kept[p], 1u);
    }
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int p = 0; p < kMaxParts; ++p) base += p < part ? part_above[p] + part_kept[p] : 0u;

    uint32_t keep_bits = 0, n_keep = 0;
    auto is_kept = [&](float v, int i) -> bool {
        const int bin = value_bin<kPartBins>(v, rp.lo, rp.inv);
        if (bin != tbin) return bin > tbin;
        const uint64_t e = ((uint64_t)score_key(v) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)(pv.j0 + i * kWave));
        return e >= thr;
    };
    if (ITEMS > 0) {
#pragma unroll
        for (int i = 0; i < (ITEMS > 0 ? ITEMS : 1); ++i) {
            const bool keep = i < pv.my_items && is_kept(vals[i], i);
            keep_bits |= keep ? (1u << i) : 0u;
            n_keep += (uint32_t)__popcll(__ballot(keep));
        }
    } else {
        for (int i = 0; i < pv.items; ++i) {
            const bool keep = i < pv.my_items && is_kept(s[pv.j0 + i * kWave], i);
            n_keep += (uint32_t)__popcll(__ballot(keep));
        }
    }
    if (lane == 0) wave_tot[wave] = n_keep;
    __syncthreads();
    uint32_t pos = base;
#pragma unroll
    for (int w = 0; w < kPartThreads / kWave; ++w) pos += (w < wave) ? wave_tot[w] : 0u;
    const uint64_t lane_lt = (1ull << lane) - 1ull;
    auto emit = [&](bool keep, int i) {
        const uint64_t ballot = __ballot(keep);
        const uint32_t slot = pos + (uint32_t)__popcll(ballot & lane_lt);
        if (keep && slot < (uint32_t)kb) out[slot] = pv.j0 + i * kWave;
        pos += (uint32_t)__popcll(ballot);
    };
    if (ITEMS > 0) {
#pragma unroll
        for (int i = 0; i < (ITEMS > 0 ? ITEMS : 1); ++i) emit((keep_bits >> i) & 1u, i);
    } else {
        for (int i = 0; i < pv.items; ++i) emit(i < pv.my_items && is_kept(s[pv.j0 + i * kWave], i), i);
    }
}

#undef SV_PART_ITEMS
#undef SV_PART_LOAD

struct SelectPlan { bool single; int parts, part_len, items; };   // items == 0: scores re-read from memory

SelectPlan plan_select(int n_vis_max) {
    SelectPlan p{};
    if (n_vis_max <= kSingleMaxN) { p.single = true; p.parts = 1; p.part_len = kSingleMaxN; p.items = kSingleMaxN / kSingleThreads; return p; }
    if (n_vis_max <= kPartLen * kMaxParts) {
        p.parts = (n_vis_max + kPartLen - 1) / kPartLen;
        p.part_len = kPartLen;
        p.items = kPartItems;
        return p;
    }
    p.parts = kMaxParts;
    p.part_len = ((n_vis_max + kMaxParts - 1) / kMaxParts + kPartThreads - 1) / kPartThreads * kPartThreads;
    p.items = 0;
    return p;
}

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

struct WsLayout { size_t hist, meta, cand, params, total; };

WsLayout layout_select_ws(size_t units, int parts) {
    WsLayout l{};
    size_t off = 0;
    l.hist = off; off += align256(units * parts * kPartBins * sizeof(uint16_t));
    l.meta = off; off += align256(units * parts * sizeof(PartMeta));
    l.cand = off; off += align256(units * parts * kPartCand * sizeof(uint2));
    l.params = off; off += align256(units * sizeof(RowParams));
    l.total = off;
    return l;
}

}  // namespace

namespace {
struct FilterLayout { size_t hint, gen, tiles, overflow, total; };

// Sized for the smallest tile the scoring kernel can be asked for, so that the layout does not
// depend on the launch-shape knobs.
FilterLayout layout_filter_ws(int dtype, int D, size_t units, int n_vis_max) {
    FilterLayout l{};
    const int granule = score_row_granule(dtype, D);
    const size_t max_tiles = (size_t)(n_vis_max + granule - 1) / granule;
    size_t off = 0;
    l.hint = off; off += align256(units * sizeof(uint64_t));
    l.gen = off; off += align256(sizeof(uint32_t));
    l.tiles = off; off += align256(units * max_tiles * kFiltRec16 * sizeof(uint4));
    l.overflow = off; off += align256(units * ((size_t)n_vis_max + 512) * sizeof(uint2));
    l.total = off;
    return l;
}
}  // namespace

// Long rows whose expected candidate count (the sample-rank fraction of the row, plus four standard
// deviations of that fraction) fits the on-chip ranking.
namespace {
// Will the rows above the threshold of an S-row sample fit the on-chip ranking (expected count plus four sigma)?
bool candidates_fit(double S, int n_vis_max, int k) {
    const double mean = S * (double)k / (double)n_vis_max;
    const double frac = (mean + 5.0 * std::sqrt(mean) + 4.0) / S;
    if (frac >= 0.5) return false;
    const double expect = frac * n_vis_max;
    const double sigma = n_vis_max * std::sqrt(frac * (1.0 - frac) / S);
    return expect + 4.0 * sigma <= (double)kFiltCap;
}
}  // namespace

bool filtered_select_applies(int dtype, int D, int n_vis_max, int k) {
    if (n_vis_max <= kFilterMinN || k <= 0 || k >= n_vis_max) return false;
    if (filter_tile_rows(dtype, D, 0, n_vis_max, kFiltMaxTiles) == 0) return false;
    return candidates_fit(presample_rows(), n_vis_max, k);
}

size_t filtered_workspace_bytes(int dtype, int D, int B, int Hkv, int n_vis_max) {
    return layout_filter_ws(dtype, D, (size_t)B * Hkv, n_vis_max).total;
}

FilterArgs carve_filter_workspace(void* base, int dtype, int D, int B, int Hkv, int n_vis_max, int k,
                                  int requested_tile_rows) {
    const FilterLayout l = layout_filter_ws(dtype, D, (size_t)B * Hkv, n_vis_max);
    char* p = static_cast<char*>(base);
    FilterArgs f{};
    f.hint = reinterpret_cast<uint64_t*>(p + l.hint);
    f.gen = reinterpret_cast<uint32_t*>(p + l.gen);
    f.samples = nullptr;   // the caller may point it at units * 2 KB of scratch that the scoring launch may use
    f.spread = 1;
    f.tiles = reinterpret_cast<uint4*>(p + l.tiles);
    f.overflow = reinterpret_cast<uint2*>(p + l.overflow);
    f.tile_rows = filter_tile_rows(dtype, D, requested_tile_rows, n_vis_max, kFiltMaxTiles);
    f.n_tiles = (n_vis_max + f.tile_rows - 1) / f.tile_rows;
    f.k = k;
    f.rank_override = 0;
    f.epoch = 0;
    f.test_mode = 0;
    // A sampler reaches its threshold through a chain of dependent memory trips (64 sample rows per trip).  A launch
    // of a few hundred tiles has streamed its keys before eight trips are over and then waits for the threshold: it
    // gets half the sample -- a lower threshold, a quarter more candidates for the selection, four trips less.
    // (if the candidates of the smaller sample still fit the on-chip ranking).
    const bool small_launch = (int64_t)B * Hkv * f.n_tiles <= kSmallLaunchTiles;
    f.n_samples = small_launch && candidates_fit(presample_rows() / 2, n_vis_max, k) ? presample_rows() / 2 : presample_rows();
    return f;
}

namespace {
template <typename T, int D>
hipError_t launch_select_filtered_typed(const SelectArgs& a, const ScoreArgs& sc, hipStream_t stream) {
    // the kernel's LDS exceeds the default limit: raised once per device (the attribute belongs to the
    // device's copy of the kernel)
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> raised[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!raised[dev].load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(select_filtered_kernel<T, D>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                                    (int)sizeof(FilteredShared));
        if (attr != hipSuccess) return attr;
        raised[dev].store(true, std::memory_order_release);
    }
    dim3 grid((unsigned)a.Hkv, (unsigned)a.B), block(kSingleThreads);
    hipLaunchKernelGGL((select_filtered_kernel<T, D>), grid, block, sizeof(FilteredShared), stream, a, sc);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_select_filtered(const SelectArgs& a, const ScoreArgs& sc, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0) return hipSuccess;
    if (sc.dtype == 0) {
        if (sc.D == 128) return launch_select_filtered_typed<_Float16, 128>(a, sc, stream);
        if (sc.D == 64) return launch_select_filtered_typed<_Float16, 64>(a, sc, stream);
    } else {
        if (sc.D == 128) return launch_select_filtered_typed<float, 128>(a, sc, stream);
        if (sc.D == 64) return launch_select_filtered_typed<float, 64>(a, sc, stream);
    }
    return hipErrorInvalidValue;
}

size_t select_workspace_bytes(int B, int Hkv, int n_vis_max) {
    const SelectPlan p = plan_select(n_vis_max);
    if (p.single) return 0;
    return layout_select_ws((size_t)B * Hkv, p.parts).total;
}

hipError_t launch_select(const SelectArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0) return hipSuccess;
    const SelectPlan p = plan_select(a.n_vis_max);
    if (p.single) {
        dim3 grid((unsigned)a.Hkv, (unsigned)a.B), block(kSingleThreads);
        hipLaunchKernelGGL(select_single_kernel, grid, block, 0, stream, a);
        return hipGetLastError();
    }
    const WsLayout l = layout_select_ws((size_t)a.B * a.Hkv, p.parts);
    char* base = static_cast<char*>(a.ws);
    SelectWorkspace ws;
    ws.part_hist = reinterpret_cast<uint16_t*>(base + l.hist);
    ws.part_meta = reinterpret_cast<PartMeta*>(base + l.meta);
    ws.cand = reinterpret_cast<uint2*>(base + l.cand);
    ws.params = reinterpret_cast<RowParams*>(base + l.params);
    dim3 grid((unsigned)p.parts, (unsigned)a.Hkv, (unsigned)a.B), block(kPartThreads);
    if (p.items > 0) {
        hipLaunchKernelGGL((select_hist_kernel<kPartItems>), grid, block, 0, stream, a, ws, p.parts, p.part_len);
        hipLaunchKernelGGL((select_threshold_kernel<kPartItems>), grid, block, 0, stream, a, ws, p.parts, p.part_len);
        hipLaunchKernelGGL((select_emit_kernel<kPartItems>), grid, block, 0, stream, a, ws, p.parts, p.part_len);
    } else {
        hipLaunchKernelGGL((select_hist_kernel<0>), grid, block, 0, stream, a, ws, p.parts, p.part_len);
        hipLaunchKernelGGL((select_threshold_kernel<0>), grid, block, 0, stream, a, ws, p.parts, p.part_len);
        hipLaunchKernelGGL((select_emit_kernel<0>), grid, block, 0, stream, a, ws, p.parts, p.part_len);
    }
    return hipGetLastError();
}

}  // namespace sv
