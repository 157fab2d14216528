// Device code shared by the scoring kernel and the selection's whole-row fallback: the summed
// query of a GQA group and the scoring of a run of rows by one workgroup.
//   scores[b,g,j] = sum_{h in group g} scale * <q[b,h,:], K_vis[b,g,j,:]>   (paper section 3.2)
#pragma once
#include "sv_device.h"
#include "sv_kernels.h"

namespace sv {

constexpr int kScoreUnroll = 8;   // independent row loads in flight per lane

__device__ __forceinline__ int live_rows_of(const ScoreArgs& a, int b) {
    int n = a.n_vis_max;
    if (a.vis_len) {
        const int v = a.vis_len[b];
        n = v < 0 ? 0 : (v < n ? v : n);
    }
    return n;
}

// Summed query of group g, the EPL dims of chunk c.
template <typename T>
__device__ __forceinline__ void summed_query(const ScoreArgs& a, int b, int g, int c, float (&qs)[Chunk<T>::kElems]) {
    constexpr int EPL = Chunk<T>::kElems;
#pragma unroll
    for (int i = 0; i < EPL; ++i) qs[i] = 0.f;
    const T* qp = static_cast<const T*>(a.q) + (int64_t)b * a.q_sb + (int64_t)g * a.G * a.q_sh + c * EPL;
    // Eight rows are requested at once (on clamped row numbers) and then added in row order: a loop of load, wait,
    // add per head is G trips through the cache in front of every tile -- 3.6 us of a 13.6 us scoring launch over one
    // layer of a long video, measured.  The order of the additions, and with it every bit of the sum, is unchanged.
    constexpr int kRowsInFlight = 8;
    for (int h0 = 0; h0 < a.G; h0 += kRowsInFlight) {
        Chunk<T> qc[kRowsInFlight];
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) qc[j] = load_chunk(qp + (int64_t)min(h0 + j, a.G - 1) * a.q_sh);
#pragma unroll
        for (int j = 0; j < kRowsInFlight; ++j) {
            if (h0 + j < a.G) {
#pragma unroll
                for (int i = 0; i < EPL; ++i) qs[i] += qc[j].at(i);
            }
        }
    }
}

// One pass of a wavefront: the scores of rows [r0, r0 + WAVE_ROWS) of (b, g); lane (grp, c) with
// c < kScoreUnroll returns the score of row r0 + c * RPW + grp (-inf past the live rows), so that
// a wavefront can store WAVE_ROWS consecutive floats with one instruction.
template <typename T, int D, bool kStream>
__device__ __forceinline__ float score_pass(const ScoreArgs& a, const T* kbase, const float (&qs)[Chunk<T>::kElems],
                                            int r0, int n, int c, int grp) {
    constexpr int EPL = Chunk<T>::kElems;
    constexpr int LPR = D / EPL;            // lanes per row
    constexpr int RPW = kWave / LPR;        // rows per wavefront load
    constexpr int U = kScoreUnroll;
    constexpr int WAVE_ROWS = RPW * U;
    static_assert(U <= LPR, "store lane selection needs U <= lanes per row");
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
    float o = acc[0];
#pragma unroll
    for (int u = 1; u < U; ++u) o = (c == u) ? acc[u] : o;
    const int row = r0 + c * RPW + grp;
    return row < n ? o * a.scale : -INFINITY;
}

// All scores of row (b, g) by one workgroup of any size, written to dst[0 .. n_vis_max).
template <typename T, int D>
__device__ __forceinline__ void score_row_by_workgroup(const ScoreArgs& a, int b, int g, float* __restrict__ dst) {
    constexpr int EPL = Chunk<T>::kElems;
    constexpr int LPR = D / EPL;
    constexpr int RPW = kWave / LPR;
    constexpr int WAVE_ROWS = RPW * kScoreUnroll;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
    const int c = lane % LPR, grp = lane / LPR;
    const int n = live_rows_of(a, b);
    float qs[EPL];
    summed_query<T>(a, b, g, c, qs);
    const T* kbase = static_cast<const T*>(a.k_vis) + (int64_t)b * a.k_sb + (int64_t)g * a.k_sh + c * EPL;
    for (int r0 = wave * WAVE_ROWS; r0 < a.n_vis_max; r0 += waves * WAVE_ROWS) {
        const float val = score_pass<T, D, false>(a, kbase, qs, r0, n, c, grp);
        const int row = r0 + c * RPW + grp;
        if (c < kScoreUnroll && row < a.n_vis_max) dst[row] = val;
    }
}

}  // namespace sv
