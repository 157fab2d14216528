// Step 2 of the decode path: keep the k highest-scoring visual tokens of every
// (batch, kv head) (paper section 3.2: the highest-relevance tokens are retained).
//
// Exact integer selection on the order-preserving uint32 image of the fp32 score:
//   * MSD radix select (11 + 11 + 10 bits) finds the key T of the k-th largest
//     score and how many keys equal to T belong to the set;
//   * an ordered compaction emits {j : key_j > T} plus the first r keys equal to T
//     in ascending index order, so ties go to the lower index and the output
//     ascends -- the set is unique for the given scores.
// One 1024-lane workgroup owns one (b, g).  Each wavefront owns a contiguous index
// range; when the range fits (n <= 1024 * ITEMS) every lane keeps its keys in
// registers, so the scores are read from memory once; longer rows re-read them
// in every pass.  Histograms live in LDS; all counting is integer, hence the
// result does not depend on the order in which lanes arrive.
#include "sv_device.h"
#include "sv_kernels.h"

namespace sv {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;   // 16
constexpr int kBins = 2048;

struct SelShared {
    uint32_t hist[kBins];
    uint32_t wave_tot[kSelWaves];
    uint32_t wave_tot2[kSelWaves];
    uint32_t bin, above, in_bin;
};

// Block-wide inclusive scan of one value per thread (thread order = index order).
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t x, uint32_t* wave_tot,
                                                         int lane, int wave) {
    const uint32_t incl = wave_inclusive_scan(x, lane);
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) base += (w < wave) ? wave_tot[w] : 0u;
    __syncthreads();
    return incl + base;
}

// ITEMS > 0: keys register-resident (n <= 1024*ITEMS).  ITEMS == 0: re-read per pass.
template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectArgs a) {
    __shared__ SelShared sh;
    const int g = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t unit = (int64_t)b * a.Hkv + g;
    const float* __restrict__ s = a.scores + unit * a.n_vis_max;
    int32_t* __restrict__ out = a.idx + unit * a.k;

    int n = a.n_vis_max;
    if (a.vis_len) {
        const int v = a.vis_len[b];
        n = v < 0 ? 0 : (v < n ? v : n);
    }
    const int kb = a.k < n ? a.k : n;
    if (tid == 0) a.count[unit] = kb;
    for (int i = kb + tid; i < a.k; i += kSelThreads) out[i] = -1;
    if (kb == 0) return;
    if (kb == n) {   // everything is kept
        for (int i = tid; i < n; i += kSelThreads) out[i] = i;
        return;
    }

    // Index range of this wavefront: [wave*seg, wave*seg + seg) clipped to n.
    const int seg = ((n + kSelWaves - 1) / kSelWaves + kWave - 1) / kWave * kWave;
    const int seg_items = seg / kWave;
    const int j0 = wave * seg + lane;

    constexpr int R = ITEMS > 0 ? ITEMS : 1;
    uint32_t keys[R];
    if (ITEMS > 0) {
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int j = j0 + i * kWave;
            keys[i] = (i < seg_items && j < n) ? score_key(s[j]) : 0u;   // 0 = "no key"
        }
    }
    // key of item i (valid keys are never 0: the smallest is the image of -inf)
    auto key_at = [&](int i) -> uint32_t {
        if (ITEMS > 0) return keys[i];
        const int j = j0 + i * kWave;
        return j < n ? score_key(s[j]) : 0u;
    };
    const int n_items = ITEMS > 0 ? R : seg_items;

    uint32_t prefix = 0, mask = 0;
    uint32_t need = (uint32_t)kb;   // how many keys with (key & mask) == prefix are kept
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const uint32_t digit_mask = pass == 2 ? 0x3FFu : 0x7FFu;
        sh.hist[tid] = 0;
        sh.hist[tid + kSelThreads] = 0;
        if (tid == 0) { sh.bin = 0; sh.above = 0; sh.in_bin = 0; }
        __syncthreads();
        if (ITEMS > 0) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const uint32_t key = key_at(i);
                if (key != 0u && (key & mask) == prefix)
                    atomicAdd(&sh.hist[(key >> shift) & digit_mask], 1u);
            }
        } else {
            for (int i = 0; i < n_items; ++i) {
                const uint32_t key = key_at(i);
                if (key != 0u && (key & mask) == prefix)
                    atomicAdd(&sh.hist[(key >> shift) & digit_mask], 1u);
            }
        }
        __syncthreads();
        // Scan the bins from the top: thread t owns bins 2047-2t and 2046-2t.
        const uint32_t c0 = sh.hist[kBins - 1 - 2 * tid];
        const uint32_t c1 = sh.hist[kBins - 2 - 2 * tid];
        const uint32_t incl = block_inclusive_scan(c0 + c1, sh.wave_tot, lane, wave);
        const uint32_t excl = incl - (c0 + c1);
        if (excl < need && need <= incl) {   // exactly one thread
            if (need <= excl + c0) { sh.bin = kBins - 1 - 2 * tid; sh.above = excl; sh.in_bin = c0; }
            else { sh.bin = kBins - 2 - 2 * tid; sh.above = excl + c0; sh.in_bin = c1; }
        }
        __syncthreads();
        prefix |= sh.bin << shift;
        mask |= digit_mask << shift;
        need -= sh.above;
        const uint32_t in_bin = sh.in_bin;
        __syncthreads();
        if (need == in_bin) break;   // the whole bin is kept: no finer digit needed
    }

    // ---- ordered compaction ----
    // kept(j) = (key&mask) > prefix, or (key&mask) == prefix and fewer than `need`
    // equal keys precede j.  Per-wave counts of "greater" and "equal" keys first.
    uint32_t n_gt = 0, n_eq = 0;
    auto count_item = [&](int i) {
        const uint32_t key = key_at(i);
        const uint32_t kp = key & mask;
        n_gt += __popcll(__ballot(key != 0u && kp > prefix));
        n_eq += __popcll(__ballot(key != 0u && kp == prefix));
    };
    if (ITEMS > 0) {
#pragma unroll
        for (int i = 0; i < R; ++i) count_item(i);
    } else {
        for (int i = 0; i < n_items; ++i) count_item(i);
    }
    if (lane == 0) { sh.wave_tot[wave] = n_gt; sh.wave_tot2[wave] = n_eq; }
    __syncthreads();
    uint32_t eq_before = 0, gt_before = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        eq_before += (w < wave) ? sh.wave_tot2[w] : 0u;
        gt_before += (w < wave) ? sh.wave_tot[w] : 0u;
    }
    // kept keys before this wave = greater ones + min(equal ones, need)
    uint32_t pos = gt_before + (eq_before < need ? eq_before : need);
    uint32_t eq_seen = eq_before;
    const uint64_t lane_lt = (1ull << lane) - 1ull;
    auto emit_item = [&](int i) {
        const uint32_t key = key_at(i);
        const uint32_t kp = key & mask;
        const bool is_eq = key != 0u && kp == prefix;
        const uint64_t eq_ballot = __ballot(is_eq);
        const uint32_t eq_rank = eq_seen + (uint32_t)__popcll(eq_ballot & lane_lt);
        const bool keep = (key != 0u && kp > prefix) || (is_eq && eq_rank < need);
        const uint64_t keep_ballot = __ballot(keep);
        const uint32_t slot = pos + (uint32_t)__popcll(keep_ballot & lane_lt);
        if (keep && slot < (uint32_t)kb) out[slot] = j0 + i * kWave;   // slot < kb always holds for finite scores
        pos += (uint32_t)__popcll(keep_ballot);
        eq_seen += (uint32_t)__popcll(eq_ballot);
    };
    if (ITEMS > 0) {
#pragma unroll
        for (int i = 0; i < R; ++i) emit_item(i);
    } else {
        for (int i = 0; i < n_items; ++i) emit_item(i);
    }
}

}  // namespace

hipError_t launch_select(const SelectArgs& a, hipStream_t stream) {
    if (a.B == 0 || a.Hkv == 0) return hipSuccess;
    dim3 grid((unsigned)a.Hkv, (unsigned)a.B), block(kSelThreads);
    const int n = a.n_vis_max;
    // register-resident variants up to 50 keys per lane (128 VGPRs at 1024 lanes per workgroup)
    if (n <= kSelThreads * 4)
        hipLaunchKernelGGL((select_kernel<4>), grid, block, 0, stream, a);
    else if (n <= kSelThreads * 16)
        hipLaunchKernelGGL((select_kernel<16>), grid, block, 0, stream, a);
    else if (n <= kSelThreads * 32)
        hipLaunchKernelGGL((select_kernel<32>), grid, block, 0, stream, a);
    else if (n <= kSelThreads * 50)
        hipLaunchKernelGGL((select_kernel<50>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((select_kernel<0>), grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace sv
