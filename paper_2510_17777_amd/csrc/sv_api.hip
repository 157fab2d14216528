// C-ABI layer of the sparse decode library: argument validation on the host (a
// failed call launches nothing), workspace carving, and dispatch to the three
// kernel stages.  See include/sparsevila.h for the contract of every entry point.
#include "../../include/sparsevila.h"

#include <atomic>
#include <cmath>
#include <cstring>

#include "sv_kernels.h"

namespace {

constexpr size_t kAlign = 256;
constexpr int kMinChunk = 64;      // smallest attention chunk; sizes the workspace
constexpr int kMaxChunk = 1024;
constexpr int kMaxGridYZ = 65535;

// Launch-shape knobs.  Each is one atomic word, read once per call into a plain snapshot, so a call sees
// one consistent value of every knob and a concurrent sv_set_tuning cannot tear anything.
enum Knob : int {
    kScoreRowsPerBlock, kAttnChunk, kScoreStreamLoads, kAttnMfma, kAttnBatches, kSelectFilter, kFilterRank,
    kFilterSamples, kFilterSpread,
#ifdef SV_TEST_HOOKS
    kFilterTestMode, kStepStages,   // exist only in the test build of the library (libsparsevila_hooks.so)
#endif
    kNumKnobs
};
struct KnobSpec { const char* name; int32_t init; };
constexpr KnobSpec kKnobSpecs[kNumKnobs] = {
    {"score_rows_per_block", 0},   // 0 = default
    {"attn_chunk", 0},
    {"score_stream_loads", -1},    // -1 = default
    {"attn_mfma", -1},
    {"attn_batches", 0},           // 0 = planned per launch
    {"select_filter", -1},
    {"filter_rank", 0},            // 0 = derived from k / n
    {"filter_samples", 0},         // 0 = by the size of the launch; 256 or 512
    {"filter_spread", 1},          // 1 = a 256-row sample is spread over several sampler workgroups
#ifdef SV_TEST_HOOKS
    {"filter_test_mode", 0},
    {"step_stages", 3},            // sv_decode_step stops after this many stages
#endif
};
struct Knobs {
    std::atomic<int32_t> v[kNumKnobs];
    Knobs() { for (int i = 0; i < kNumKnobs; ++i) v[i].store(kKnobSpecs[i].init, std::memory_order_relaxed); }
};
Knobs g_knobs;

struct Tuning {   // one call's view of the knobs
    int32_t score_rows_per_block, attn_chunk, score_stream_loads, attn_mfma, attn_batches, select_filter, filter_rank,
        filter_samples, filter_spread, filter_test_mode, step_stages;
};
inline Tuning tuning_snapshot() {
    auto get = [](int k) { return g_knobs.v[k].load(std::memory_order_relaxed); };
    Tuning t{};
    t.score_rows_per_block = get(kScoreRowsPerBlock); t.attn_chunk = get(kAttnChunk);
    t.score_stream_loads = get(kScoreStreamLoads); t.attn_mfma = get(kAttnMfma); t.attn_batches = get(kAttnBatches);
    t.select_filter = get(kSelectFilter); t.filter_rank = get(kFilterRank); t.filter_samples = get(kFilterSamples);
    t.filter_spread = get(kFilterSpread);
#ifdef SV_TEST_HOOKS
    t.filter_test_mode = get(kFilterTestMode); t.step_stages = get(kStepStages);
#else
    t.filter_test_mode = 0; t.step_stages = 3;
#endif
    return t;
}
std::atomic<uint32_t> g_epoch{0x5eed0001u};   // tags the threshold words of one sv_decode_step call

constexpr int kDefaultScoreRows = 256;
constexpr int kDefaultAttnChunk = 128;
constexpr int kDefaultStreamLoads = 1;
constexpr int kDefaultAttnMfma = 1;
constexpr int kDefaultSelectFilter = 1;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int elem_size(int dtype) { return dtype == SV_F16 ? 2 : 4; }

// Which parts of the shape a call depends on.
enum : unsigned { kNeedQ = 1, kNeedVis = 2, kNeedTxt = 4, kAllowD96 = 8 };   // kAllowD96: the two attention-mass calls

sv_status check_shape(const sv_shape* s, unsigned need) {
    if (!s) return SV_ERR_NULL;
    if (s->dtype != SV_F16 && s->dtype != SV_F32) return SV_ERR_DTYPE;
    if (s->reserved != 0) return SV_ERR_SHAPE;
    if (s->batch < 1 || s->batch > kMaxGridYZ) return SV_ERR_SHAPE;
    if (s->n_kv_heads < 1 || s->n_q_heads < 1 || s->n_q_heads % s->n_kv_heads != 0) return SV_ERR_SHAPE;
    if ((int64_t)s->n_kv_heads * ((s->n_q_heads / s->n_kv_heads + 7) / 8) > kMaxGridYZ) return SV_ERR_SHAPE;
    if (s->n_q_heads > kMaxGridYZ) return SV_ERR_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 128 && !((need & kAllowD96) && s->head_dim == 96)) return SV_ERR_SHAPE;
    if (s->n_vis_max < 0 || s->n_txt_max < 0 || s->k < 0) return SV_ERR_SHAPE;
    if (!(s->scale >= 0.f) || std::isinf(s->scale)) return SV_ERR_SHAPE;
    const int64_t D = s->head_dim;
    const int es = elem_size(s->dtype);
    if (need & kNeedQ) {
        if (s->q_stride_h < D || s->q_stride_b < 0) return SV_ERR_SHAPE;
        if ((s->q_stride_h * es) % 16 || (s->q_stride_b * es) % 16) return SV_ERR_ALIGN;
    }
    if ((need & kNeedVis) && s->n_vis_max > 0) {
        if (s->kv_vis_stride_n < D || s->kv_vis_stride_h < 0 || s->kv_vis_stride_b < 0) return SV_ERR_SHAPE;
        if ((s->kv_vis_stride_n * es) % 16 || (s->kv_vis_stride_h * es) % 16 || (s->kv_vis_stride_b * es) % 16)
            return SV_ERR_ALIGN;
    }
    if ((need & kNeedTxt) && s->n_txt_max > 0) {
        if (s->kv_txt_stride_n < D || s->kv_txt_stride_h < 0 || s->kv_txt_stride_b < 0) return SV_ERR_SHAPE;
        if ((s->kv_txt_stride_n * es) % 16 || (s->kv_txt_stride_h * es) % 16 || (s->kv_txt_stride_b * es) % 16)
            return SV_ERR_ALIGN;
    }
    return SV_OK;
}

inline float effective_scale(const sv_shape* s) {
    return s->scale > 0.f ? s->scale : 1.0f / std::sqrt((float)s->head_dim);
}

inline int kept_max(const sv_shape* s) { return s->k < s->n_vis_max ? s->k : s->n_vis_max; }

struct Workspace {
    size_t scores_off, scores_bytes;
    size_t acc_off, acc_bytes;
    size_t ml_off, ml_bytes;
    size_t sel_off, sel_bytes;
    size_t filt_off, filt_bytes;   // candidate filter of sv_decode_step; 0 bytes when the shape does not qualify
    size_t total;
};

// Sized for the smallest chunk so that the layout never depends on the tuning knobs.
Workspace plan_workspace(const sv_shape* s) {
    Workspace w{};
    const size_t B = (size_t)s->batch, Hq = (size_t)s->n_q_heads, Hkv = (size_t)s->n_kv_heads;
    // slots of a split token list (text chunks, then visual chunks); never fewer than the joint list needs
    const size_t S = ((size_t)s->n_txt_max + kMinChunk - 1) / kMinChunk + ((size_t)kept_max(s) + kMinChunk - 1) / kMinChunk;
    w.scores_off = 0;
    w.scores_bytes = align_up(B * Hkv * (size_t)s->n_vis_max * sizeof(float));
    w.acc_off = w.scores_off + w.scores_bytes;
    w.acc_bytes = align_up(B * Hq * S * (size_t)s->head_dim * sizeof(float));
    w.ml_off = w.acc_off + w.acc_bytes;
    w.ml_bytes = align_up(B * Hq * S * 2 * sizeof(float));
    w.sel_off = w.ml_off + w.ml_bytes;
    w.sel_bytes = align_up(sv::select_workspace_bytes(s->batch, s->n_kv_heads, s->n_vis_max));
    w.filt_off = w.sel_off + w.sel_bytes;
    w.filt_bytes = 0;
    if (sv::filtered_select_applies(s->dtype, s->head_dim, s->n_vis_max, s->k))
        w.filt_bytes = align_up(sv::filtered_workspace_bytes(s->dtype, s->head_dim, s->batch, s->n_kv_heads, s->n_vis_max));
    w.total = w.filt_off + w.filt_bytes;
    if (w.total == 0) w.total = kAlign;
    return w;
}

// sv_topk_select carves the workspace on its own -- [selection scratch][candidate records] from offset 0 -- as a
// function of batch, n_kv_heads, n_vis_max and k alone: the call reads nothing else of the shape.  The records of
// given scores are laid out for the finest tiling any scoring kernel uses (that of fp32 rows of 128 dims).
constexpr int kSelectDtype = SV_F32, kSelectDim = 128;
struct SelectOnlyWorkspace { size_t sel_bytes, filt_off, filt_bytes, total; };

SelectOnlyWorkspace plan_select_workspace(const sv_shape* s) {
    SelectOnlyWorkspace w{};
    w.sel_bytes = align_up(sv::select_workspace_bytes(s->batch, s->n_kv_heads, s->n_vis_max));
    w.filt_off = w.sel_bytes;
    if (w.sel_bytes > 0 && sv::filtered_select_applies(kSelectDtype, kSelectDim, s->n_vis_max, s->k))
        w.filt_bytes = align_up(sv::filtered_workspace_bytes(kSelectDtype, kSelectDim, s->batch, s->n_kv_heads, s->n_vis_max));
    w.total = w.filt_off + w.filt_bytes;
    return w;
}

// What sv_workspace_bytes reports: enough for each of the three calls.
size_t workspace_total(const sv_shape* s) {
    const size_t step = plan_workspace(s).total, sel = plan_select_workspace(s).total;
    return step > sel ? step : sel;
}

sv_status check_workspace(const Workspace& w, const void* ws, size_t bytes) {
    if (!ws) return SV_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % kAlign) return SV_ERR_WORKSPACE;
    if (bytes < w.total) return SV_ERR_WORKSPACE;
    return SV_OK;
}

sv::ScoreArgs make_score_args(const sv_shape* s, const Tuning& tune, const void* q, const void* k_vis, float* scores) {
    sv::ScoreArgs a{};
    a.q = q; a.k_vis = k_vis; a.scores = scores; a.vis_len = s->vis_len;
    a.B = s->batch; a.Hkv = s->n_kv_heads; a.G = s->n_q_heads / s->n_kv_heads;
    a.D = s->head_dim; a.n_vis_max = s->n_vis_max; a.dtype = s->dtype;
    a.scale = effective_scale(s);
    a.q_sb = s->q_stride_b; a.q_sh = s->q_stride_h;
    a.k_sb = s->kv_vis_stride_b; a.k_sh = s->kv_vis_stride_h; a.k_sn = s->kv_vis_stride_n;
    a.rows_per_block = tune.score_rows_per_block > 0 ? tune.score_rows_per_block : kDefaultScoreRows;
    a.stream_loads = tune.score_stream_loads >= 0 ? tune.score_stream_loads : kDefaultStreamLoads;
    a.write_scores = 1;
    return a;
}

sv::SelectArgs make_select_args(const sv_shape* s, const Workspace& w, void* ws, const float* scores,
                                int32_t* idx, int32_t* count) {
    sv::SelectArgs a{};
    a.scores = scores; a.idx = idx; a.count = count; a.vis_len = s->vis_len;
    a.ws = ws ? static_cast<char*>(ws) + w.sel_off : nullptr;
    a.B = s->batch; a.Hkv = s->n_kv_heads; a.n_vis_max = s->n_vis_max; a.k = s->k;
    return a;
}

sv::AttnArgs make_attn_args(const sv_shape* s, const Tuning& tune, const Workspace& w, void* ws, const void* q,
                            const void* k_vis, const void* v_vis, const void* k_txt, const void* v_txt,
                            const int32_t* idx, const int32_t* count, float* out, float* lse) {
    sv::AttnArgs a{};
    a.q = q; a.k_vis = k_vis; a.v_vis = v_vis; a.k_txt = k_txt; a.v_txt = v_txt;
    a.idx = idx; a.count = count; a.txt_len = s->txt_len;
    a.part_acc = reinterpret_cast<float*>(static_cast<char*>(ws) + w.acc_off);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(ws) + w.ml_off);
    a.out = out; a.lse = lse;
    a.B = s->batch; a.Hq = s->n_q_heads; a.Hkv = s->n_kv_heads; a.G = s->n_q_heads / s->n_kv_heads;
    a.D = s->head_dim; a.n_vis_max = s->n_vis_max; a.n_txt_max = s->n_txt_max;
    a.k = kept_max(s) > 0 ? s->k : 0;
    a.dtype = s->dtype; a.scale = effective_scale(s);
    a.q_sb = s->q_stride_b; a.q_sh = s->q_stride_h;
    a.vis_sb = s->kv_vis_stride_b; a.vis_sh = s->kv_vis_stride_h; a.vis_sn = s->kv_vis_stride_n;
    a.txt_sb = s->kv_txt_stride_b; a.txt_sh = s->kv_txt_stride_h; a.txt_sn = s->kv_txt_stride_n;
    a.chunk = tune.attn_chunk > 0 ? tune.attn_chunk : kDefaultAttnChunk;
    a.use_mfma = (s->dtype == SV_F16) && (tune.attn_mfma >= 0 ? tune.attn_mfma : kDefaultAttnMfma);
    if (a.use_mfma) a.chunk = sv::attn_mfma_chunk();   // the attn_chunk knob shapes the vector path only
    a.chunk_vis = a.chunk;
    const int64_t t_max = (int64_t)s->n_txt_max + kept_max(s);
    a.n_chunks = (int32_t)((t_max + a.chunk - 1) / a.chunk);
    a.split_base = -1;
    if (a.use_mfma && s->head_dim == 128) {   // that kernel gives text and visual tokens chunks of their own
        const int hblk = a.G > 8 ? (a.G + 7) / 8 : 1;
        sv::attn_flash_plan((int64_t)a.B * a.Hkv * hblk, s->n_txt_max, kept_max(s), tune.attn_batches, &a.chunk,
                            &a.chunk_vis);
        a.split_base = (s->n_txt_max + a.chunk - 1) / a.chunk;
        a.n_chunks = a.split_base + (kept_max(s) + a.chunk_vis - 1) / a.chunk_vis;
    }
    return a;
}

sv_status check_attn_pointers(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis,
                              const void* k_txt, const void* v_txt, const int32_t* idx,
                              const int32_t* count, const float* out) {
    (void)idx;   // NULL with k > 0: the visual segment is packed
    if (!q || !out) return SV_ERR_NULL;
    const bool has_vis = kept_max(s) > 0;
    if (has_vis && (!k_vis || !v_vis || !count)) return SV_ERR_NULL;   // idx == NULL: packed visual segment
    if (s->n_txt_max > 0 && (!k_txt || !v_txt)) return SV_ERR_NULL;
    if (!aligned16(q)) return SV_ERR_ALIGN;
    if (has_vis && (!aligned16(k_vis) || !aligned16(v_vis))) return SV_ERR_ALIGN;
    if (s->n_txt_max > 0 && (!aligned16(k_txt) || !aligned16(v_txt))) return SV_ERR_ALIGN;
    return SV_OK;
}

inline sv_status from_hip(hipError_t e) { return e == hipSuccess ? SV_OK : SV_ERR_LAUNCH; }

}  // namespace

extern "C" {

void sv_shape_set_contiguous(sv_shape* s) {
    if (!s) return;
    const int64_t D = s->head_dim;
    s->q_stride_h = D;
    s->q_stride_b = D * s->n_q_heads;
    s->kv_vis_stride_n = D;
    s->kv_vis_stride_h = D * s->n_vis_max;
    s->kv_vis_stride_b = D * s->n_vis_max * s->n_kv_heads;
    s->kv_txt_stride_n = D;
    s->kv_txt_stride_h = D * s->n_txt_max;
    s->kv_txt_stride_b = D * s->n_txt_max * s->n_kv_heads;
}

size_t sv_workspace_bytes(const sv_shape* s) {
    if (check_shape(s, 0) != SV_OK) return 0;
    return workspace_total(s);
}

size_t sv_select_workspace_bytes(const sv_shape* s) {
    if (check_shape(s, 0) != SV_OK) return 0;
    return plan_select_workspace(s).total;
}

sv_status sv_score_visual(const sv_shape* s, const void* q, const void* k_vis, float* scores, void* stream) {
    sv_status st = check_shape(s, kNeedQ | kNeedVis);
    if (st != SV_OK) return st;
    if (s->n_vis_max == 0) return SV_OK;
    if (!q || !k_vis || !scores) return SV_ERR_NULL;
    if (!aligned16(q) || !aligned16(k_vis)) return SV_ERR_ALIGN;
    return from_hip(sv::launch_score(make_score_args(s, tuning_snapshot(), q, k_vis, scores), static_cast<hipStream_t>(stream)));
}

sv_status sv_topk_select(const sv_shape* s, const float* scores, int32_t* idx, int32_t* count,
                         void* workspace, size_t workspace_bytes, void* stream) {
    sv_status st = check_shape(s, 0);
    if (st != SV_OK) return st;
    if (!count) return SV_ERR_NULL;
    if (s->k > 0 && !idx) return SV_ERR_NULL;
    if (s->n_vis_max > 0 && !scores) return SV_ERR_NULL;
    const SelectOnlyWorkspace w = plan_select_workspace(s);
    if (w.total > 0) {   // short rows are selected entirely on chip and need no workspace
        if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign || workspace_bytes < w.total)
            return SV_ERR_WORKSPACE;
    }
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const Tuning tune = tuning_snapshot();
    sv::SelectArgs sel{};
    sel.scores = scores; sel.idx = idx; sel.count = count; sel.vis_len = s->vis_len;
    sel.ws = w.total > 0 ? workspace : nullptr;
    sel.B = s->batch; sel.Hkv = s->n_kv_heads; sel.n_vis_max = s->n_vis_max; sel.k = s->k;
    const bool filter = w.filt_bytes > 0 && (tune.select_filter >= 0 ? tune.select_filter : kDefaultSelectFilter) != 0;
    if (filter) {   // long rows: one pass over the scores hands the on-chip selection its candidates
        sv::ScoreArgs sa{};
        sa.scores = const_cast<float*>(scores);   // read only: write_scores = 1 keeps the selection's fallback off it
        sa.vis_len = s->vis_len;
        sa.B = s->batch; sa.Hkv = s->n_kv_heads; sa.G = 1;
        sa.D = kSelectDim; sa.n_vis_max = s->n_vis_max; sa.dtype = kSelectDtype;
        sa.write_scores = 1;
        sa.filt = sv::carve_filter_workspace(static_cast<char*>(workspace) + w.filt_off, kSelectDtype, kSelectDim,
                                             s->batch, s->n_kv_heads, s->n_vis_max, s->k,
                                             tune.score_rows_per_block > 0 ? tune.score_rows_per_block : kDefaultScoreRows);
        sa.filt.rank_override = tune.filter_rank;
        sa.filt.test_mode = tune.filter_test_mode;
        if (tune.filter_samples > 0) sa.filt.n_samples = tune.filter_samples;
        sa.filt.epoch = g_epoch.fetch_add(1u, std::memory_order_relaxed);
        if (sv::launch_scores_filter(sa, hs) != hipSuccess) return SV_ERR_LAUNCH;
        return from_hip(sv::launch_select_filtered(sel, sa, hs));
    }
    return from_hip(sv::launch_select(sel, hs));
}

sv_status sv_sparse_decode_attn(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis,
                                const void* k_txt, const void* v_txt, const int32_t* idx,
                                const int32_t* count, float* out, float* lse, void* workspace,
                                size_t workspace_bytes, void* stream) {
    sv_status st = check_shape(s, kNeedQ | kNeedVis | kNeedTxt);
    if (st != SV_OK) return st;
    st = check_attn_pointers(s, q, k_vis, v_vis, k_txt, v_txt, idx, count, out);
    if (st != SV_OK) return st;
    const Workspace w = plan_workspace(s);
    st = check_workspace(w, workspace, workspace_bytes);
    if (st != SV_OK) return st;
    const sv::AttnArgs a = make_attn_args(s, tuning_snapshot(), w, workspace, q, k_vis, v_vis, k_txt, v_txt, idx, count, out, lse);
    return from_hip(sv::launch_attend(a, static_cast<hipStream_t>(stream)));
}

namespace {

// Workspace of sv_decode_step_static: one array per device, inside the library's code object, so that
// the call needs no allocation by anyone.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address that kernels and copies may use is looked up once per device.
constexpr size_t kStaticScratchBytes = SV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of the current device's copy of `scratch`; looked up on the first call on that device.
sv_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SV_ERR_LAUNCH;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SV_ERR_LAUNCH;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread finds the same address
    }
    *out = p;
    return SV_OK;
}

sv_status decode_step_impl(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis,
                           const void* k_txt, const void* v_txt, float* scores, int32_t* idx,
                           int32_t* count, float* out, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream);

// Everything about a step's arguments that the host can check, short of the workspace.
sv_status check_step_args(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis, const void* k_txt,
                          const void* v_txt, const int32_t* idx, const int32_t* count, const float* out) {
    const sv_status st = check_shape(s, kNeedQ | kNeedVis | kNeedTxt);
    if (st != SV_OK) return st;
    if (kept_max(s) > 0 && (!idx || !count)) return SV_ERR_NULL;
    return check_attn_pointers(s, q, k_vis, v_vis, k_txt, v_txt, idx, count, out);
}

}  // namespace

sv_status sv_decode_step(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis,
                         const void* k_txt, const void* v_txt, float* scores, int32_t* idx,
                         int32_t* count, float* out, float* lse, void* workspace,
                         size_t workspace_bytes, void* stream) {
    return decode_step_impl(s, q, k_vis, v_vis, k_txt, v_txt, scores, idx, count, out, lse, workspace,
                            workspace_bytes, stream);
}

sv_status sv_decode_step_static(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis,
                                const void* k_txt, const void* v_txt, float* scores, int32_t* idx,
                                int32_t* count, float* out, float* lse, void* stream) {
    sv_status st = check_step_args(s, q, k_vis, v_vis, k_txt, v_txt, idx, count, out);
    if (st != SV_OK) return st;
    if (workspace_total(s) > kStaticScratchBytes) return SV_ERR_WORKSPACE;   // before anything touches the device
    void* ws = nullptr;
    st = static_scratch(&ws);
    if (st != SV_OK) return st;
    // Nothing in the workspace has to start at zero: partial results and candidate records are written
    // before they are read, and the threshold words carry a per-call tag, so what the previous call
    // (of any shape) left behind is never taken for this call's.
    return decode_step_impl(s, q, k_vis, v_vis, k_txt, v_txt, scores, idx, count, out, lse, ws,
                            kStaticScratchBytes, stream);
}

namespace {

sv_status decode_step_impl(const sv_shape* s, const void* q, const void* k_vis, const void* v_vis,
                           const void* k_txt, const void* v_txt, float* scores, int32_t* idx,
                           int32_t* count, float* out, float* lse, void* workspace,
                           size_t workspace_bytes, void* stream) {
    sv_status st = check_step_args(s, q, k_vis, v_vis, k_txt, v_txt, idx, count, out);
    if (st != SV_OK) return st;
    const bool has_vis = kept_max(s) > 0;
    const Workspace w = plan_workspace(s);
    st = check_workspace(w, workspace, workspace_bytes);
    if (st != SV_OK) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const Tuning tune = tuning_snapshot();
    if (has_vis) {
        float* sc = scores ? scores : reinterpret_cast<float*>(static_cast<char*>(workspace) + w.scores_off);
        sv::ScoreArgs sa = make_score_args(s, tune, q, k_vis, sc);
        const bool filter = w.filt_bytes > 0 &&
                            (tune.select_filter >= 0 ? tune.select_filter : kDefaultSelectFilter) != 0;
        if (filter) {   // long rows: sample a threshold, let the scoring kernel emit the candidates above it
            sa.filt = sv::carve_filter_workspace(static_cast<char*>(workspace) + w.filt_off, s->dtype, s->head_dim,
                                                 s->batch, s->n_kv_heads, s->n_vis_max, s->k, sa.rows_per_block);
            sa.filt.rank_override = tune.filter_rank;
            sa.filt.test_mode = tune.filter_test_mode;
            if (tune.filter_samples > 0) sa.filt.n_samples = tune.filter_samples;
            sa.filt.epoch = g_epoch.fetch_add(1u, std::memory_order_relaxed);
            sa.write_scores = scores != nullptr;   // nobody asked for the scores: do not spend HBM writes on them
            // Scratch for a spread sample (2 KB per (b, g)): the head of the workspace's score region, which this launch
            // does not write (the scores go to the caller's buffer or nowhere; a row the selection re-scores comes later).
            sa.filt.samples = tune.filter_spread
                                  ? reinterpret_cast<uint64_t*>(static_cast<char*>(workspace) + w.scores_off) : nullptr;
        }
        hipError_t e = sv::launch_score(sa, hs);
        if (e != hipSuccess) return SV_ERR_LAUNCH;
        if (tune.step_stages < 2) return SV_OK;
        const sv::SelectArgs sel = make_select_args(s, w, workspace, sc, idx, count);
        e = filter ? sv::launch_select_filtered(sel, sa, hs) : sv::launch_select(sel, hs);
        if (e != hipSuccess) return SV_ERR_LAUNCH;
    } else if (count && (idx || s->k == 0)) {
        // nothing can be kept (k == 0 or no visual rows): the kept sets are empty, count = 0
        hipError_t e = sv::launch_select(make_select_args(s, w, workspace, scores, idx, count), hs);
        if (e != hipSuccess) return SV_ERR_LAUNCH;
    }
    if (tune.step_stages < 3) return SV_OK;
    const sv::AttnArgs a = make_attn_args(s, tune, w, workspace, q, k_vis, v_vis, k_txt, v_txt, idx, count, out, lse);
    return from_hip(sv::launch_attend(a, hs));
}

}  // namespace

size_t sv_mass_workspace_bytes(const sv_shape* s, int32_t n_query_tokens) {
    if (check_shape(s, kAllowD96) != SV_OK || n_query_tokens < 1) return 0;
    const size_t lse = align_up((size_t)s->batch * n_query_tokens * s->n_q_heads * sizeof(float));
    const size_t part = align_up(sv::mass_workspace_bytes(s->batch, s->n_kv_heads, s->n_txt_max, s->n_vis_max));
    return lse + part + kAlign;
}

sv_status sv_score_visual_mass(const sv_shape* s, const void* q_multi, int32_t n_query_tokens, int64_t q_stride_t,
                               const void* k_vis, const void* k_txt, float* scores, float* lse, void* workspace,
                               size_t workspace_bytes, void* stream) {
    sv_status st = check_shape(s, kNeedQ | kNeedVis | kNeedTxt | kAllowD96);
    if (st != SV_OK) return st;
    if (s->dtype != SV_F16) return SV_ERR_DTYPE;
    const int G = s->n_q_heads / s->n_kv_heads;
    if (n_query_tokens < 1 || (int64_t)n_query_tokens * G > sv::mass_max_rows()) return SV_ERR_SHAPE;
    if (q_stride_t < 0 || (q_stride_t * 2) % 16) return q_stride_t < 0 ? SV_ERR_SHAPE : SV_ERR_ALIGN;
    if (s->n_vis_max == 0) return SV_OK;
    if (!q_multi || !k_vis || !scores || (s->n_txt_max > 0 && !k_txt)) return SV_ERR_NULL;
    if (!aligned16(q_multi) || !aligned16(k_vis) || (s->n_txt_max > 0 && !aligned16(k_txt))) return SV_ERR_ALIGN;
    const size_t lse_bytes = align_up((size_t)s->batch * n_query_tokens * s->n_q_heads * sizeof(float));
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign ||
        workspace_bytes < sv_mass_workspace_bytes(s, n_query_tokens))
        return SV_ERR_WORKSPACE;
    sv::MassArgs a{};
    a.q = q_multi; a.k_vis = k_vis; a.k_txt = k_txt; a.vis_len = s->vis_len; a.txt_len = s->txt_len;
    a.scores = scores;
    a.lse = lse ? lse : reinterpret_cast<float*>(workspace);
    a.part = reinterpret_cast<float*>(static_cast<char*>(workspace) + lse_bytes);
    a.B = s->batch; a.Hq = s->n_q_heads; a.Hkv = s->n_kv_heads; a.G = G; a.D = s->head_dim;
    a.Tq = n_query_tokens; a.n_vis_max = s->n_vis_max; a.n_txt_max = s->n_txt_max;
    a.scale = effective_scale(s);
    a.q_sb = s->q_stride_b; a.q_st = q_stride_t; a.q_sh = s->q_stride_h;
    a.vis_sb = s->kv_vis_stride_b; a.vis_sh = s->kv_vis_stride_h; a.vis_sn = s->kv_vis_stride_n;
    a.txt_sb = s->kv_txt_stride_b; a.txt_sh = s->kv_txt_stride_h; a.txt_sn = s->kv_txt_stride_n;
    return from_hip(sv::launch_mass(a, static_cast<hipStream_t>(stream)));
}

namespace {
// The fields sv_salience_self uses; head_dim 96 is allowed here only.
sv_status check_salience_shape(const sv_shape* s) {
    if (!s) return SV_ERR_NULL;
    if (s->dtype != SV_F16 && s->dtype != SV_F32) return SV_ERR_DTYPE;
    if (s->reserved != 0) return SV_ERR_SHAPE;
    if (s->batch < 1 || s->batch > kMaxGridYZ) return SV_ERR_SHAPE;
    if (s->n_kv_heads < 1 || s->n_q_heads != s->n_kv_heads) return SV_ERR_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 96 && s->head_dim != 128) return SV_ERR_SHAPE;
    if (s->n_vis_max < 0) return SV_ERR_SHAPE;
    if (!(s->scale >= 0.f) || std::isinf(s->scale)) return SV_ERR_SHAPE;
    if (s->dtype != SV_F16) return SV_ERR_DTYPE;
    const int64_t D = s->head_dim;
    if (s->q_stride_h < D || s->q_stride_b < 0) return SV_ERR_SHAPE;
    if ((s->q_stride_h * 2) % 16 || (s->q_stride_b * 2) % 16) return SV_ERR_ALIGN;
    if (s->n_vis_max > 0) {
        if (s->kv_vis_stride_n < D || s->kv_vis_stride_h < 0 || s->kv_vis_stride_b < 0) return SV_ERR_SHAPE;
        if ((s->kv_vis_stride_n * 2) % 16 || (s->kv_vis_stride_h * 2) % 16 || (s->kv_vis_stride_b * 2) % 16)
            return SV_ERR_ALIGN;
        const sv::SaliencePlan p = sv::salience_plan(s->batch, s->n_kv_heads, s->n_vis_max);
        if ((int64_t)s->n_kv_heads * p.n_row_chunks > kMaxGridYZ || (int64_t)s->n_kv_heads * p.n_seg > kMaxGridYZ)
            return SV_ERR_SHAPE;
    }
    return SV_OK;
}
}  // namespace

size_t sv_salience_workspace_bytes(const sv_shape* s) {
    if (check_salience_shape(s) != SV_OK) return 0;
    const sv::SaliencePlan p = sv::salience_plan(s->batch, s->n_kv_heads, s->n_vis_max);
    const size_t lse = align_up((size_t)s->batch * s->n_vis_max * s->n_kv_heads * sizeof(float));
    return lse + align_up(p.part_bytes) + align_up(p.colpart_bytes) + kAlign;
}

sv_status sv_salience_self(const sv_shape* s, const void* q_all, int64_t q_stride_t, const void* k_all, float* salience,
                           float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    sv_status st = check_salience_shape(s);
    if (st != SV_OK) return st;
    if (q_stride_t < s->head_dim) return SV_ERR_SHAPE;
    if ((q_stride_t * 2) % 16) return SV_ERR_ALIGN;
    if (s->n_vis_max == 0) return SV_OK;
    if (!q_all || !k_all || !salience) return SV_ERR_NULL;
    if (!aligned16(q_all) || !aligned16(k_all)) return SV_ERR_ALIGN;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign ||
        workspace_bytes < sv_salience_workspace_bytes(s))
        return SV_ERR_WORKSPACE;
    const sv::SaliencePlan p = sv::salience_plan(s->batch, s->n_kv_heads, s->n_vis_max);
    const size_t lse_bytes = align_up((size_t)s->batch * s->n_vis_max * s->n_kv_heads * sizeof(float));
    char* ws = static_cast<char*>(workspace);
    sv::SalienceArgs a{};
    a.q = q_all; a.k = k_all; a.vis_len = s->vis_len; a.salience = salience;
    a.lse = lse ? lse : reinterpret_cast<float*>(ws);
    a.part = reinterpret_cast<float*>(ws + lse_bytes);
    a.colpart = reinterpret_cast<float*>(ws + lse_bytes + align_up(p.part_bytes));
    a.B = s->batch; a.H = s->n_kv_heads; a.D = s->head_dim; a.N = s->n_vis_max;
    a.scale = effective_scale(s);
    a.q_sb = s->q_stride_b; a.q_st = q_stride_t; a.q_sh = s->q_stride_h;
    a.k_sb = s->kv_vis_stride_b; a.k_sh = s->kv_vis_stride_h; a.k_sn = s->kv_vis_stride_n;
    return from_hip(sv::launch_salience(a, static_cast<hipStream_t>(stream)));
}

sv_status sv_pack_selected(const sv_shape* s, const void* k_vis, const void* v_vis, const int32_t* idx,
                           const int32_t* count, void* k_pack, void* v_pack, void* stream) {
    sv_status st = check_shape(s, kNeedVis);
    if (st != SV_OK) return st;
    if (s->k == 0) return SV_OK;
    if (!idx || !count || !k_pack || !v_pack) return SV_ERR_NULL;
    if (s->n_vis_max == 0) return SV_ERR_SHAPE;
    if (!k_vis || !v_vis) return SV_ERR_NULL;
    if (!aligned16(k_vis) || !aligned16(v_vis) || !aligned16(k_pack) || !aligned16(v_pack)) return SV_ERR_ALIGN;
    sv::PackArgs a{};
    a.k_vis = k_vis; a.v_vis = v_vis; a.idx = idx; a.count = count; a.k_pack = k_pack; a.v_pack = v_pack;
    a.B = s->batch; a.Hkv = s->n_kv_heads; a.n_vis_max = s->n_vis_max; a.k = s->k;
    a.elem = elem_size(s->dtype); a.row_bytes = s->head_dim * a.elem;
    a.vis_sb = s->kv_vis_stride_b; a.vis_sh = s->kv_vis_stride_h; a.vis_sn = s->kv_vis_stride_n;
    return from_hip(sv::launch_pack(a, static_cast<hipStream_t>(stream)));
}

sv_status sv_copy_bytes(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return SV_ERR_NULL;
    if (bytes % 16 || !aligned16(dst) || !aligned16(src)) return SV_ERR_ALIGN;
    return from_hip(sv::launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)));
}

sv_status sv_read_bytes(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink) return SV_ERR_NULL;
    if (bytes % 16 || !aligned16(src) || !aligned16(sink)) return SV_ERR_ALIGN;
    return from_hip(sv::launch_read(src, bytes, sink, static_cast<hipStream_t>(stream)));
}

const char* sv_strerror(int status) {
    switch (status) {
        case SV_OK: return "ok";
        case SV_ERR_NULL: return "a required pointer is NULL";
        case SV_ERR_SHAPE: return "invalid shape, stride or knob value";
        case SV_ERR_DTYPE: return "unsupported dtype";
        case SV_ERR_ALIGN: return "pointer or row stride not 16-byte aligned";
        case SV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SV_ERR_LAUNCH: return "HIP launch failed";
    }
    return "unknown status";
}

sv_status sv_set_tuning(const char* name, int32_t value) {
    if (!name) return SV_ERR_NULL;
    int k = 0;
    while (k < kNumKnobs && std::strcmp(name, kKnobSpecs[k].name)) ++k;
    bool ok = false;
    switch (k) {
        case kScoreRowsPerBlock: ok = value == 0 || (value >= 64 && value <= 65536); break;
        case kAttnChunk: ok = value == 0 || (value >= kMinChunk && value <= kMaxChunk && value % 64 == 0); break;
        case kScoreStreamLoads: case kAttnMfma: case kSelectFilter: ok = value >= -1 && value <= 1; break;
        case kAttnBatches: ok = value >= 0 && value <= 8; break;
        case kFilterRank: ok = value >= 0 && value <= 448; break;
        case kFilterSamples: ok = value == 0 || value == 256 || value == 512; break;
        case kFilterSpread: ok = value == 0 || value == 1; break;
#ifdef SV_TEST_HOOKS
        case kFilterTestMode: ok = value >= 0 && value <= 2; break;
        case kStepStages: ok = value >= 1 && value <= 3; break;
#endif
        default: break;   // unknown name
    }
    if (!ok) return SV_ERR_SHAPE;
    g_knobs.v[k].store(value, std::memory_order_relaxed);
    return SV_OK;
}

int32_t sv_get_tuning(const char* name) {
    if (!name) return -1;
    int k = 0;
    while (k < kNumKnobs && std::strcmp(name, kKnobSpecs[k].name)) ++k;
    if (k == kNumKnobs) return -1;
    const int32_t v = g_knobs.v[k].load(std::memory_order_relaxed);
    switch (k) {   // knobs with a "default" value report what that default is
        case kScoreRowsPerBlock: return v > 0 ? v : kDefaultScoreRows;
        case kAttnChunk: return v > 0 ? v : kDefaultAttnChunk;
        case kScoreStreamLoads: return v >= 0 ? v : kDefaultStreamLoads;
        case kAttnMfma: return v >= 0 ? v : kDefaultAttnMfma;
        case kSelectFilter: return v >= 0 ? v : kDefaultSelectFilter;
        default: return v;
    }
}

int32_t sv_has_test_hooks(void) {
#ifdef SV_TEST_HOOKS
    return 1;
#else
    return 0;
#endif
}

}  // extern "C"
