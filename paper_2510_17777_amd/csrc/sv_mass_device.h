// Device helpers shared by the two attention-mass computations (retrieval with a multi-token query,
// section 3.2; query-agnostic salience of an encoder layer, section 3.1): 16-row tiles on the matrix
// cores (v_mfma_f32_16x16x32_f16), the streamed operand staged through LDS 64 rows at a time, and the
// row statistics of pass 1.
#pragma once
#include "sv_device.h"

// Between the steps of a stage: the scheduler may not move instructions across it.
#define SV_STAGE_FENCE() __builtin_amdgcn_sched_barrier(0)

namespace sv {

constexpr int kMassWaves = 4;
constexpr int kMassThreads = kMassWaves * kWave;
constexpr int kMaxRowTiles = 16;                  // R <= 256
constexpr int kTilesPerWave = kMaxRowTiles / kMassWaves;
constexpr int kStageKeys = 16 * kMassWaves;       // keys per LDS stage: one key tile per wavefront
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kSumLimit = 0x1p100f;             // pass 1: a row sum outside [1 / this, this) (or NaN) sends its key block to the exact path
constexpr int kTargetGroups = 3072;               // the streamed side is cut into blocks until this many workgroups exist

__device__ __forceinline__ int live_len(const int32_t* p, int i, int cap) {
    if (!p) return cap;
    const int v = p[i];
    return v < 0 ? 0 : (v < cap ? v : cap);
}

// The row tiles of a wavefront: tile slot t of wavefront w is row tile (w + rot) % 4 + 4t, where rot
// differs from workgroup to workgroup so that the SIMDs of a compute unit get equal shares when the
// last row tiles are missing.
__device__ __forceinline__ int row_tile_of(int wave, int rot, int t) { return ((wave + rot) & (kMassWaves - 1)) + t * kMassWaves; }
// How many of the wavefront's tile slots hold rows below R (the live slots come first); wave-uniform.
__device__ __forceinline__ int live_tiles_of(int wave, int rot, int R) {
    const int tiles = (R + 15) / 16, first = (wave + rot) & (kMassWaves - 1);
    const int n = tiles > first ? (tiles - first + kMassWaves - 1) / kMassWaves : 0;
    return __builtin_amdgcn_readfirstlane(n);
}

// B operand of one key tile: lane (row, quad) supplies dims 8*quad + 32*kb .. +8 of key `key_row`.
template <int KB>
__device__ __forceinline__ void load_key_tile(const _Float16* base, int64_t sn, int key_row, int quad,
                                              half8_t (&kf)[KB]) {
    const _Float16* p = base + (int64_t)key_row * sn + quad * 8;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) kf[kb] = __builtin_nontemporal_load(reinterpret_cast<const half8_t*>(p + 32 * kb));
}

// One LDS stage: [key tile][kb][lane], the operand words in the lane order they are fetched and used in.
template <int KB>
struct KeyStage { half8_t w[kMassWaves][KB][kWave]; };

template <int KB>
__device__ __forceinline__ void read_key_tile(const KeyStage<KB>& st, int kt, int lane, half8_t (&kf)[KB]) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) kf[kb] = st.w[kt][kb][lane];
}

// Logits of the first NTL row tiles of this wavefront against one key tile: lane (row, quad) gets rows
// 4*quad + rr of each row tile at key column `row`.  The chains of the row tiles are interleaved so that
// consecutive matrix instructions do not depend on each other.
template <int KB, int NTL>
__device__ __forceinline__ void tile_logits(const half8_t (&qa)[kTilesPerWave][KB], const half8_t (&kf)[KB],
                                            float4_t (&sv)[kTilesPerWave]) {
#pragma unroll
    for (int t = 0; t < NTL; ++t) sv[t] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < NTL; ++t) sv[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[kb], sv[t], 0, 0, 0);
}

// Maximum over the 16 lanes that hold one query row's key columns.
__device__ __forceinline__ float row_max16(float x) {
    x = fmaxf(x, dpp_move<kDppQuadXor1>(x));
    x = fmaxf(x, dpp_move<kDppQuadXor2>(x));
    x = fmaxf(x, dpp_move<kDppRowHalfMirror>(x));
    x = fmaxf(x, dpp_move<kDppRowMirror>(x));
    return x;
}

// The loads of the query tiles must not count as outstanding inside the key loops: the wait inserted
// for them there would also wait for the keys fetched one stage ahead.
__device__ __forceinline__ void wait_for_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// Pass 1 on the fast path.  One reference per wavefront -- the largest logit of its live rows against the first 16
// keys of the key block (rowstat_init_ref), a scalar register -- that is never raised: a logit far above it makes a
// large term and a row far below it small ones, which fp32 sums as accurately as terms near 1; only a distance of
// more than ~2^100 would overflow or underflow, and the kernel checks every row sum for that after the block and
// redoes the block on the exact path (a reference per row with a running maximum).  So an element costs a
// multiply-add, an exponential and an add, as in pass 2, with no maximum, no vote and no branch, and the loop holds
// no reference registers: with 16 of them per lane, or with the references set by a variant of the stage code inside
// the loop, the kernel needed more than the 168 registers that three wavefronts per SIMD leave.  The ragged last
// stage of a key block runs the same code (rowstat_fast_stage masks its dead columns through the reference).
// rows_live: rows of this workgroup below it exist (the others are zero rows and must not set the reference).
template <int KB, int NTL>
__device__ __forceinline__ float rowstat_init_ref(const KeyStage<KB>& st, int lane, int wave, int rot, int rows_live,
                                                  const half8_t (&qa)[kTilesPerWave][KB], float c2) {
    const int quad = lane >> 4;
    half8_t kf[KB];
    float4_t sv[kTilesPerWave];
    read_key_tile<KB>(st, 0, lane, kf);
    tile_logits<KB, NTL>(qa, kf, sv);
    float m = -INFINITY;
#pragma unroll
    for (int t = 0; t < NTL; ++t)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr)
            if (row_tile_of(wave, rot, t) * 16 + 4 * quad + rr < rows_live) m = fmaxf(m, sv[t][rr] * c2);
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, wave_max(m))));
}

// A stage of which the first live_cols (1..64, wave-uniform) key columns are live: the matrix instructions of the next
// key tile go between the vector instructions of this one.  A dead column (the ragged end of a key block; its key is
// a copy of the last live one) takes -inf in place of the reference in the multiply-add, so its term is exactly 0 at
// no cost per element: one compare and one select per key tile.
template <int KB, int NTL>
__device__ __forceinline__ void rowstat_fast_stage(const KeyStage<KB>& st, int lane, const half8_t (&qa)[kTilesPerWave][KB],
                                                   float c2, float ref, int live_cols, float (&l)[kTilesPerWave][4]) {
    half8_t kf[2][KB];
    float4_t sv[2][kTilesPerWave];
    read_key_tile<KB>(st, 0, lane, kf[0]);
    tile_logits<KB, NTL>(qa, kf[0], sv[0]);
    constexpr int n_m = KB * NTL, n_e = 4 * NTL;
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
        const float nref = kt * 16 + (lane & 15) < live_cols ? -ref : -INFINITY;
        float y[n_e1], pr[n_e1];
#pragma unroll
        for (int step = 0; step < n_e + 2; ++step) {
            if (has_next && step < n_e) {
#pragma unroll
                for (int m = step * n_m / n_e1; m < (step + 1) * n_m / n_e1; ++m) {
                    const int kb = m / NT1, t = m % NT1;
                    sv[nxt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[t][kb], kf[nxt][kb], sv[nxt][t], 0, 0, 0);
                }
            }
            if (step < n_e) y[step] = fmaf(sv[cur][step / 4][step % 4], c2, nref);
            if (step >= 1 && step - 1 < n_e) pr[step - 1] = __builtin_amdgcn_exp2f(y[step - 1]);
            if (step >= 2) l[(step - 2) / 4][(step - 2) % 4] += pr[step - 2];
            SV_STAGE_FENCE();
        }
    }
}

// Block-wide OR of a per-thread flag through one LDS word that is zero on entry (every thread of the workgroup
// calls it; the word is left zero again).  The library's __syncthreads_or keeps the thread-index register alive
// across everything before it, a register that pass 1 does not have to spare.
__device__ __forceinline__ bool block_any(bool mine, int* s_word) {
    if (__ballot(mine) != 0ull) *s_word = 1;   // wave-uniform branch; every lane stores the same value
    __syncthreads();
    const bool any = *s_word != 0;
    __syncthreads();
    *s_word = 0;
    return any;
}

// Length of the blocks the streamed side (n rows) is cut into when `units` workgroup rows stream it: cut only as far
// as it takes to fill the chip -- a workgroup pays for loading the rows it holds and for a merge at the end, so long
// blocks are cheaper -- never below min_len rows, a multiple of the 64-row stage.
inline int planned_block_len(int64_t units, int n, int min_len) {
    if (n < 1) return kStageKeys;
    if (units < 1) units = 1;
    int64_t want = (kTargetGroups + units - 1) / units;
    const int64_t most = n / min_len > 1 ? n / min_len : 1;
    if (want > most) want = most;
    if (want < 1) want = 1;
    const int len = (int)((n + want - 1) / want);
    return (len + kStageKeys - 1) / kStageKeys * kStageKeys;
}

}  // namespace sv
