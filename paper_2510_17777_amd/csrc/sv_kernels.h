// Host-side view of the kernels: plain argument structs and one launcher per stage.
// The launchers assume arguments already validated by the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sv {

// Candidate filter of sv_decode_step for long rows.  Sampler workgroups at the head of the scoring
// launch publish, per (b, g), a threshold t_lo (an order statistic of the scores of a small sample
// of the row) that lies below the k-th largest score with overwhelming probability.  Every scoring
// workgroup stores the (score bits, row) pairs of its tile with score >= t_lo, in row order: a
// 512-byte primary record per tile ({count, t_lo used, largest pair score, 0}, then the first 62 pairs; records of
// consecutive tiles are adjacent) and, for fuller tiles, pair number f >= 62 at position f of the
// tile's overflow rows.  The selection ranks those few candidates on chip.  t_lo is only a hint:
// the selection checks on the device that the candidates determine the kept set (at least k of them
// at or above the largest t_lo any tile used, and no more than fit); a row that fails is selected
// from all its scores.
constexpr int kFilterRecordPairs = 62;   // pairs in a primary record: 16-byte header + 62 * 8 bytes = 512 bytes

struct FilterArgs {
    uint64_t* hint;         // [units]  {epoch << 32 | t_lo bits}, written by the samplers
    uint4* tiles;           // [units][n_tiles][32]
    uint2* overflow;        // [units][n_tiles][tile_rows]
    int32_t n_tiles;        // ceil(n_vis_max / tile_rows)
    int32_t tile_rows;      // rows per scoring workgroup while the filter is on
    int32_t k;
    int32_t rank_override;  // > 0: use this sample rank for t_lo (tests force the fallbacks with it)
    uint32_t epoch;         // differs from call to call: marks the hint words of this call
    uint32_t* gen;          // [1] bumped by every filtered selection: added to epoch on the device, so that replays
                            // of a captured call (same arguments, same epoch) still tag their hint words apart
    int32_t test_mode;      // 0; tests: every third tile ignores the hint (1: keeps nothing, 2: keeps all)
    int32_t n_samples;      // rows sampled per (b, g): 512, or 256 in a launch so small that it waits for its samplers
    uint64_t* samples;      // [units][256] {epoch << 32 | score bits}: the sample scores of a spread sample; may be nullptr
    int32_t spread;         // set by the launcher: sampler workgroups per (b, g).  1: one workgroup scores the whole sample
                            // in rounds of dependent loads; > 1 (256 samples, `samples` given): each scores its share in
                            // ONE round and publishes the scores, the first of them ranks all 256 and publishes t_lo
};

struct ScoreArgs {
    const void* q;
    const void* k_vis;
    float* scores;            // [B, Hkv, n_vis_max]
    const int32_t* vis_len;   // device [B] or nullptr
    int32_t B, Hkv, G, D, n_vis_max;
    int32_t dtype;            // 0 = f16, 1 = f32
    float scale;
    int64_t q_sb, q_sh;       // element strides
    int64_t k_sb, k_sh, k_sn;
    int32_t rows_per_block;   // tuning; rounded up to the kernel's granule by the launcher
    int32_t stream_loads;     // 1: non-temporal K loads
    int32_t write_scores;     // candidate filter on: 0 = the scores themselves are not stored (the selection
                              // recomputes a row's scores in the rare case it needs them all)
    FilterArgs filt;          // filt.tiles == nullptr: no candidate emission
};

struct SelectArgs {
    const float* scores;      // [B, Hkv, n_vis_max]
    int32_t* idx;             // [B, Hkv, k]
    int32_t* count;           // [B, Hkv]
    const int32_t* vis_len;
    void* ws;                 // select_workspace_bytes() bytes, 256-byte aligned (unused when that is 0)
    int32_t B, Hkv, n_vis_max, k;
};

struct AttnArgs {
    const void* q;
    const void* k_vis; const void* v_vis;
    const void* k_txt; const void* v_txt;
    const int32_t* idx;       // [B, Hkv, k]; nullptr: k == 0, or the visual segment is packed (token i is row i)
    const int32_t* count;     // [B, Hkv]    or nullptr when k == 0
    const int32_t* txt_len;   // device [B] or nullptr
    float* part_acc;          // [B, Hq, S, D]  un-normalised chunk outputs
    float* part_ml;           // [B, Hq, S, 2]  chunk max and chunk sum of exp
    float* out;               // [B, Hq, D]
    float* lse;               // [B, Hq] or nullptr
    int32_t B, Hq, Hkv, G, D, n_vis_max, n_txt_max, k;
    int32_t dtype;
    float scale;
    int64_t q_sb, q_sh;
    int64_t vis_sb, vis_sh, vis_sn;
    int64_t txt_sb, txt_sh, txt_sn;
    int32_t chunk;            // tokens per workgroup
    int32_t use_mfma;         // fp16 caches: 1 = logits on the matrix cores, 0 = vector FMA path
    int32_t n_chunks;         // S: partial-result slots per query head
    int32_t split_base;       // < 0: chunks cut the joint list (text, then kept visual tokens), S = ceil((n_txt_max +
                              // k) / chunk); >= 0: chunks [0, split_base) cut the text tokens, chunks [split_base, S)
                              // the kept visual tokens
    int32_t chunk_vis;        // split lists: tokens per workgroup of the visual range (`chunk` is that of the text range)
};

struct PackArgs {
    const void* k_vis; const void* v_vis;
    const int32_t* idx;       // [B, Hkv, k]
    const int32_t* count;     // [B, Hkv]
    void* k_pack; void* v_pack;   // dense [B, Hkv, k, D]
    int32_t B, Hkv, n_vis_max, k;
    int32_t elem;             // bytes per element
    int32_t row_bytes;        // D * elem, a multiple of 16 that divides 4096
    int64_t vis_sb, vis_sh, vis_sn;   // element strides of the source
    int32_t rows_per_block;   // set by the launcher
};

// Attention-mass retrieval scores of a multi-token query (sv_score_visual_mass).
struct MassArgs {
    const void* q;            // [B, Tq, Hq, D] through q_sb, q_st, q_sh (fp16)
    const void* k_vis; const void* k_txt;
    const int32_t* vis_len; const int32_t* txt_len;
    float* scores;            // [B, Hkv, n_vis_max]
    float* lse;               // [B, Tq, Hq]
    float* part;              // mass_workspace_bytes() bytes: per key block (max, sum) of every query row
    int32_t B, Hq, Hkv, G, D, Tq, n_vis_max, n_txt_max;
    float scale;
    int64_t q_sb, q_st, q_sh;
    int64_t vis_sb, vis_sh, vis_sn;
    int64_t txt_sb, txt_sh, txt_sn;
    // set by the launcher: visual / text keys per workgroup in pass 1 (pass 2 uses the visual length), the text blocks
    // of a row and all its blocks
    int32_t stat_block_keys, txt_block_keys, n_txt_blocks, n_stat_blocks;
};
hipError_t launch_mass(const MassArgs& a, hipStream_t stream);
size_t mass_workspace_bytes(int B, int Hkv, int n_txt_max, int n_vis_max);
int mass_max_rows();   // most query rows (tokens x heads of a group) the kernels hold

// Query-agnostic salience of an encoder layer (sv_salience_self).
struct SalienceArgs {
    const void* q;            // [B, N, H, D] through q_sb, q_st, q_sh (fp16)
    const void* k;            // [B, H, N, D] through k_sb, k_sh, k_sn (fp16)
    const int32_t* vis_len;
    float* salience;          // [B, N]
    float* lse;               // [B, N, H]
    float* part;              // SaliencePlan::part_bytes: per key block (max, sum) of every query row
    float* colpart;           // SaliencePlan::colpart_bytes: per query segment and head, the mass of every key
    int32_t B, H, D, N;
    float scale;
    int64_t q_sb, q_st, q_sh;
    int64_t k_sb, k_sh, k_sn;
    int32_t n_row_chunks, stat_block_keys, n_stat_blocks, seg_len, n_seg;   // set by the launcher from the plan
};
struct SaliencePlan {
    int n_row_chunks;        // groups of 256 tokens
    int stat_block_keys, n_stat_blocks;   // pass 1: keys per workgroup, key blocks per row
    int seg_len, n_seg;      // pass 2: query tokens per workgroup, segments per row
    size_t part_bytes, colpart_bytes;
};
SaliencePlan salience_plan(int B, int H, int N);   // all zero for an empty problem
hipError_t launch_salience(const SalienceArgs& a, hipStream_t stream);

hipError_t launch_score(const ScoreArgs& a, hipStream_t stream);
// Scores given (a.scores, read only): sampler + tile workgroups hand the selection the candidates of every row
// (a.filt from carve_filter_workspace); then launch_select_filtered with a.write_scores = 1.
hipError_t launch_scores_filter(const ScoreArgs& a, hipStream_t stream);
hipError_t launch_pack(const PackArgs& a, hipStream_t stream);
hipError_t launch_select(const SelectArgs& a, hipStream_t stream);
hipError_t launch_attend(const AttnArgs& a, hipStream_t stream);   // partials + combine

// Candidate-filtered selection (sv_decode_step only).  filtered_select_applies(): is the shape
// inside the limits of the on-chip ranking and is the expected candidate count small enough?
bool filtered_select_applies(int dtype, int D, int n_vis_max, int k);
size_t filtered_workspace_bytes(int dtype, int D, int B, int Hkv, int n_vis_max);   // for any tile_rows
FilterArgs carve_filter_workspace(void* base, int dtype, int D, int B, int Hkv, int n_vis_max, int k,
                                  int requested_tile_rows);
// Tile rows the filter will use: `requested` rounded to the scoring kernel's granule, at most 512, raised
// until the row has at most max_tiles tiles; 0 if that is impossible.
int filter_tile_rows(int dtype, int D, int requested, int n_vis_max, int max_tiles);
int presample_rows();                                                  // rows sampled per (b, g)
// sc: the scoring arguments of the same call (sc.filt = the candidate records; sc.scores = a.scores, which
// holds the scores if sc.write_scores and serves as scratch for a row's recomputed scores otherwise).
hipError_t launch_select_filtered(const SelectArgs& a, const ScoreArgs& sc, hipStream_t stream);

// Scratch the selection needs for rows too long for one workgroup (0 for short rows).
size_t select_workspace_bytes(int B, int Hkv, int n_vis_max);

// Plain copy of `bytes` (multiple of 16) device bytes; calibration aid for traffic counters.
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
constexpr int kReadSinkWords = 1024;   // words of the sink buffer of launch_read (a power of two)
hipError_t launch_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t stream);

// Tokens per workgroup of the matrix-core attention kernel for head_dim 64 (fixed by its register layout).
int attn_mfma_chunk();
// head_dim 128: tokens per workgroup of the text range and of the visual range, for `units` = B * Hkv *
// (head blocks) and the longest text / kept lengths; forced_batches 1..8 overrides the plan (32-token
// batches per wavefront, both ranges), 0 = plan.
void attn_flash_plan(int64_t units, int n_txt, int n_kept, int forced_batches, int* chunk_txt, int* chunk_vis);

// Row granule of the scoring kernel for a dtype/head_dim (rows one workgroup pass covers).
int score_row_granule(int dtype, int D);

// Rows one wavefront pass of the scoring kernel covers (= rows of one candidate slot).
int score_wave_rows(int dtype, int D);

}  // namespace sv
