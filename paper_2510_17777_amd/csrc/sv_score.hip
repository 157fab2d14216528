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
#include "sv_device.h"
#include "sv_kernels.h"

namespace sv {
namespace {

constexpr int kScoreUnroll = 8;   // independent row loads in flight per lane
constexpr int kScoreWaves = 4;    // wavefronts per workgroup

template <typename T, int D, bool kStream>
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
    float* __restrict__ srow = a.scores + ((int64_t)b * a.Hkv + g) * a.n_vis_max;

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
        if (c < U && row < row_end) srow[row] = row < n ? o * a.scale : -INFINITY;
    }
}

template <typename T, int D>
hipError_t launch_typed(const ScoreArgs& a, hipStream_t stream) {
    const int granule = score_row_granule(a.dtype, D);
    ScoreArgs k = a;
    int rpb = a.rows_per_block < granule ? granule : a.rows_per_block;
    rpb = (rpb + granule - 1) / granule * granule;
    k.rows_per_block = rpb;
    const unsigned tiles = (unsigned)((a.n_vis_max + rpb - 1) / rpb);
    if (tiles == 0 || a.B == 0) return hipSuccess;
    dim3 grid(tiles, (unsigned)a.Hkv, (unsigned)a.B), block(kScoreWaves * kWave);
    if (a.stream_loads)
        hipLaunchKernelGGL((score_kernel<T, D, true>), grid, block, 0, stream, k);
    else
        hipLaunchKernelGGL((score_kernel<T, D, false>), grid, block, 0, stream, k);
    return hipGetLastError();
}

}  // namespace

int score_row_granule(int dtype, int D) {
    const int epl = dtype == 0 ? 8 : 4;
    const int lpr = D / epl;
    return kScoreWaves * (kWave / lpr) * kScoreUnroll;
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
