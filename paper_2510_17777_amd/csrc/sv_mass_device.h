// Device helpers shared by the two attention-mass computations (retrieval with a multi-token query,
// section 3.2; query-agnostic salience of an encoder layer, section 3.1): 16-row tiles on the matrix
// cores (v_mfma_f32_16x16x32_f16), the streamed operand staged through LDS 64 rows at a time, and the
// row statistics of pass 1.
#pragma once
#include "sv_device.h"

namespace sv {

constexpr int kMassWaves = 4;
constexpr int kMassThreads = kMassWaves * kWave;
constexpr int kMaxRowTiles = 16;                  // R <= 256
constexpr int kTilesPerWave = kMaxRowTiles / kMassWaves;
constexpr int kStageKeys = 16 * kMassWaves;       // keys per LDS stage: one key tile per wavefront
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRaiseAbove = 8.f;                // pass 1: a reference is raised when a logit tops it by 2^8

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

// Pass 1, a stage of 64 live keys that every row sees: per lane, for rows 4*quad + rr of each row tile over
// the key columns the lane meets, a reference value ref and l = sum 2^(logit - ref), in base 2.  kInit: nothing was seen before, the first
// key tile sets the references.  The logits of key tile k + 1 are issued before those of tile k are used.
template <int KB, int NTL, bool kInit>
__device__ __forceinline__ void rowstat_plain_stage(const KeyStage<KB>& st, int lane, const half8_t (&qa)[kTilesPerWave][KB],
                                                    float c2, float (&ref)[kTilesPerWave][4], float (&l)[kTilesPerWave][4]) {
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
        float4_t(&y)[kTilesPerWave] = sv[kt & 1];
        if (kInit && kt == 0) {
            // the reference of a row: the largest of its first 16 logits, shared by the row's 16 lanes.  (A lane's
            // own first logit is a poor reference: one lane-row in fifty then meets a logit 2^8 above it
            // later in the block, and every such meeting sends the whole wavefront through the raise path.)
#pragma unroll
            for (int t = 0; t < NTL; ++t)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const float x = y[t][rr] * c2;
                    const float r0 = row_max16(x);
                    ref[t][rr] = r0;
                    l[t][rr] = __builtin_amdgcn_exp2f(x - r0);
                }
            continue;
        }
        float top = -INFINITY;
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                y[t][rr] = fmaf(y[t][rr], c2, -ref[t][rr]);   // logit - ref, base 2
                top = fmaxf(top, y[t][rr]);
            }
        if (__ballot(top > kRaiseAbove) != 0ull) {   // rare: some reference is raised to the logit that tops it
            asm volatile("" ::: "memory");   // emits nothing; keeps this block a real branch (as straight-line
                                             // selects it cost every key tile 16 more exponentials per lane)
#pragma unroll
            for (int t = 0; t < NTL; ++t)
#pragma unroll
                for (int rr = 0; rr < 4; ++rr)
                    if (y[t][rr] > kRaiseAbove) {
                        l[t][rr] *= __builtin_amdgcn_exp2f(-y[t][rr]);
                        ref[t][rr] += y[t][rr];
                        y[t][rr] = 0.f;
                    }
        }
#pragma unroll
        for (int t = 0; t < NTL; ++t)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) l[t][rr] += __builtin_amdgcn_exp2f(y[t][rr]);
    }
}

}  // namespace sv
