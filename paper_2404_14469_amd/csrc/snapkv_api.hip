// Host side of the C ABI declared in include/snapkv.h: argument validation, scratch layout and
// the launch plan.  Nothing here synchronises the stream.
#include "../../include/snapkv.h"
#include "snapkv_internal.h"

#include <algorithm>
#include <cmath>
#include <atomic>
#include <mutex>
#include <vector>

// Scratch of snapkv_compress_static: a fixed array in the library's own device image, so that entry point
// neither allocates nor takes a workspace.  In host code this name is only a stand-in for the symbol:
// the array's device address is looked up once per device (static_scratch below) and that address is
// what the kernels get.
static __device__ __align__(256) unsigned char scratch[SNAPKV_STATIC_SCRATCH_BYTES];

namespace {

using namespace snapkv;

constexpr int kMaxDevices = 64;
constexpr size_t kLayersScratchCap = (size_t)6 << 30;   // snapkv_compress_layers: most scratch one run of layers may take
// What the last call's final kernel left ready at the start of the library's own buffer, so that
// the next call needs no preparing launch: the selection's counters (zero) for `hkv` heads and,
// behind them in a region of `fused_bytes` bytes, `ones` hand-off words holding the "not
// published" pattern.  ones < 0: nothing is known.  Anything else that touches the buffer
// resets it.
struct CleanState {
    int hkv = 0, hq = 0;
    size_t fused_bytes = 0;
    int64_t ones = -1;
    hipStream_t stream = nullptr;   // the stream the call that left this state was enqueued on
};
struct DeviceScratch {
    void* ptr = nullptr;
    size_t bytes = 0;
    CleanState clean;
    unsigned* sticky = nullptr;   // pinned host word the device sets when a call on this scratch had a wait give up
};
DeviceScratch g_scratch[kMaxDevices];
std::mutex g_mu;
DeviceScratch g_decode_scratch[kMaxDevices];   // partial results of decode attention and the hit-rate probe's logits:
                                               // kept apart so that they leave the compression scratch's ready state alone

// The auxiliary buffer of the current device, grown when needed (need > 0).
int aux_scratch(size_t need, void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SNAPKV_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceScratch& s = g_decode_scratch[dev];
    if (s.bytes < need) {
        if (s.ptr && hipFree(s.ptr) != hipSuccess) return SNAPKV_ERR_HIP;   // waits for work still using it
        s.ptr = nullptr;
        s.bytes = 0;
        if (hipMalloc(&s.ptr, need * 2) != hipSuccess) {
            s.ptr = nullptr;
            (void)hipGetLastError();
            return SNAPKV_ERR_HIP;
        }
        s.bytes = need * 2;
    }
    *out = s.ptr;
    return SNAPKV_OK;
}

// Optional per-stage timing: events recorded on the caller's stream at stage boundaries.
struct Profile {
    bool active = false;
    int max_calls = 0;
    int calls = 0;            // calls begun
    bool in_call = false;     // between kStageBegin and kStageGather of a recorded call
    std::vector<hipEvent_t> ev;   // [max_calls][kNumStageMarks]
    std::vector<char> set;        // which marks were recorded
};
Profile g_prof;
bool g_allow_fused = true;   // snapkv_set_scoring_scheme: tests can force the two-pass kernels
bool g_allow_pool_select = true;   // ... and the separate pooling and selection kernels

std::atomic<long long> g_wait_limit{-1};   // snapkv_debug_set_wait_limit: < 0 = the kernels' own bounds

bool valid_dtype(int dtype) { return dtype == SNAPKV_DTYPE_BF16 || dtype == SNAPKV_DTYPE_F32 || dtype == SNAPKV_DTYPE_F16; }
int elem_bytes(int dtype) { return dtype == SNAPKV_DTYPE_F32 ? 4 : 2; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape checks shared by every entry point that scores (steps 1-3).
int check_score_args(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D, int W,
                     int pool_kind, int p) {
    if (!q_win || !k) return SNAPKV_ERR_INVALID_ARG;
    if (L < 1 || W < 1 || W > L || Hq < 1 || Hkv < 1 || Hq % Hkv != 0) return SNAPKV_ERR_INVALID_ARG;
    if (p < 1 || (p & 1) == 0) return SNAPKV_ERR_INVALID_ARG;
    if (pool_kind != SNAPKV_POOL_MAX && pool_kind != SNAPKV_POOL_AVG) return SNAPKV_ERR_INVALID_ARG;
    if (D != 64 && D != 128) return SNAPKV_ERR_UNSUPPORTED;
    if (p > 129) return SNAPKV_ERR_UNSUPPORTED;
    if (L >= (int64_t)1 << 31) return SNAPKV_ERR_UNSUPPORTED;
    if (L > W && !select_chunked_ok(L - W)) return SNAPKV_ERR_UNSUPPORTED;   // prefixes of more than 2^24 positions
    if ((int64_t)(Hq / Hkv) * ((W + 31) / 32) > 4096) return SNAPKV_ERR_UNSUPPORTED;
    if (Hkv > 65535) return SNAPKV_ERR_UNSUPPORTED;
    if (!aligned16(q_win) || !aligned16(k)) return SNAPKV_ERR_MISALIGNED;
    return SNAPKV_OK;
}

// The entries that use the library's own scratch keep a host-side record of the state their last kernel
// leaves it in, and may allocate; neither survives being recorded into a graph and replayed later, so
// they refuse a stream that is capturing (snapkv_compress_ws and snapkv_compress_static are the forms to capture).
bool capturing(hipStream_t st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs != hipStreamCaptureStatusNone;
}

// Hands out the device's buffer.  Whoever takes it may leave it in any state, so the record of a
// ready-made state is handed to the caller (*was_clean, may be null) and dropped.
int internal_scratch(size_t need, void** out, CleanState* was_clean = nullptr, unsigned** sticky = nullptr) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SNAPKV_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceScratch& s = g_scratch[dev];
    if (!s.sticky) {   // allocated, not registered: a few bytes of pinned host memory the kernels can write
        void* p = nullptr;
        if (hipHostMalloc(&p, 64, hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            return SNAPKV_ERR_HIP;
        }
        s.sticky = static_cast<unsigned*>(p);
        *s.sticky = 0u;
    }
    if (sticky) *sticky = s.sticky;
    if (s.bytes < need) s.clean = CleanState{};
    if (was_clean) *was_clean = s.clean;
    s.clean = CleanState{};
    if (s.bytes < need) {
        if (s.ptr) {
            // hipFree waits for the device, so work still reading the old buffer has finished
            if (hipFree(s.ptr) != hipSuccess) return SNAPKV_ERR_HIP;
            s.ptr = nullptr;
            s.bytes = 0;
        }
        const size_t want = need + need / 4;
        if (hipMalloc(&s.ptr, want) != hipSuccess) {
            s.ptr = nullptr;
            (void)hipGetLastError();
            return SNAPKV_ERR_HIP;
        }
        s.bytes = want;
    }
    *out = s.ptr;
    return SNAPKV_OK;
}

// Device address of `scratch` on the current device.  Every GPU holds its own copy of the array at its
// own address, so the address is asked for with that device current, the first time the device is seen.
void* g_static_scratch[kMaxDevices] = {nullptr};

int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SNAPKV_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_static_scratch[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return SNAPKV_ERR_HIP;
        }
        g_static_scratch[dev] = ptr;
    }
    *out = g_static_scratch[dev];
    return SNAPKV_OK;
}

// Steps 1-3.  With score == nullptr the pooling kernel is left out (the caller pools and selects
// in one launch) and *Gv tells how the votes are laid out.
// Which kernels score a prompt: the single-read kernel (its hand-off words are in use; *F is its plan), the
// single-read kernel on the front part of a prompt too long for it and streaming passes on the rest (the
// same, *F = LP->Ff), two streaming passes (the hand-off words stay untouched; *F is their plan), or the
// 32x32 two-pass kernels.
enum { kPathNone = 0, kPathFused = 1, kPathStream = 2, kPathLong = 3 };
int scoring_path(int dtype, int D, const ScoreGeom& G, bool lse_given, bool allow_blocks, bool allow_long,
                 FusedGeom* F, LongPlan* LP) {
    if (!lse_given && g_allow_fused) {
        if (fused_plan(dtype, D, G, F, allow_blocks)) return kPathFused;
        if (allow_long && long_plan(dtype, D, G, LP)) {
            *F = LP->Ff;
            return kPathLong;
        }
    }
    return lse_plan(dtype, D, G, F, allow_blocks && !lse_given) ? kPathStream : kPathNone;
}

// Whether the heads of several separately allocated layers can go through the kernels as one call: the scoring
// kernels must take the prompt in their plain form (no 32-row blocks), and the single-read kernel, where it is
// used, must keep its grid resident in the form that reads its Q and K rows through a table of layers.
bool layers_table_ok(int dtype, int D, const ScoreGeom& G, int kv_heads_per_layer) {
    FusedGeom F;
    LongPlan LP;
    // (a window that a single call would score in 32-row blocks is left to single calls: the table form has no blocks)
    const int path = scoring_path(dtype, D, G, false, true, true, &F, &LP);
    if (path == kPathNone || F.BH != 1) return false;
    ScoreLayers probe{};
    probe.count = G.Hkv / kv_heads_per_layer;
    probe.kv_heads = kv_heads_per_layer;
    if (probe.count < 1 || probe.count > kMaxLayerPtrs) return false;
    if (path == kPathStream) return true;   // nothing there needs a resident grid
    // (for a long prompt F is the plan of the front part)
    const hipError_t e = launch_score_fused_layers(dtype, D, probe, path == kPathLong ? LP.Gf : G, F, FusedSync{}, nullptr, nullptr, true);
    if (e != hipSuccess) (void)hipGetLastError();
    return e == hipSuccess;
}

int run_scores(int dtype, const void* q_win, const void* k, int D, const ScoreGeom& G,
               const Workspace& ws, int pool_kind, int p, float* score, unsigned* minmax,
               bool prepare_select, ScoreGeom* Gv, hipStream_t st, bool already_prepared = false,
               CleanJob* clean = nullptr, const float* lse = nullptr, bool allow_blocks = false,
               bool allow_long = false, const ScoreLayers* layers = nullptr) {
    FusedGeom F;
    ScoreGeom Gp = G;
    if (layers && (lse || allow_blocks)) return SNAPKV_ERR_UNSUPPORTED;
    if (lse) {   // the rows' normalisers are given: one streaming pass, nothing handed between workgroups
        if (!lse_plan(dtype, D, G, &F)) return SNAPKV_ERR_UNSUPPORTED;
        if (!already_prepared) {
            if (launch_prepare(nullptr, 0, prepare_select ? &ws.sel : nullptr, G.Hkv * G.g, st, ws.status_flag) != hipSuccess)
                return SNAPKV_ERR_HIP;
            stage_done(st, kStagePrepare);
        }
        if (launch_score_lse(dtype, D, q_win, k, lse, G, F, ws.vote, st) != hipSuccess) return SNAPKV_ERR_HIP;
        stage_done(st, kStageFused);
        Gp.NV = G.g;
        Gp.VB = 1;
        if (Gv) *Gv = Gp;
        if (!score) return SNAPKV_OK;
        if (launch_pool(Gp, ws.vote, pool_kind, p, score, minmax, st) != hipSuccess) return SNAPKV_ERR_HIP;
        stage_done(st, kStagePool);
        return SNAPKV_OK;
    }
    LongPlan LP;
    const int path = scoring_path(dtype, D, G, false, allow_blocks, allow_long, &F, &LP);
    const bool fused = path == kPathFused, split_read = path == kPathLong;
    if (layers && (path == kPathNone || F.BH != 1)) return SNAPKV_ERR_UNSUPPORTED;   // (callers ask layers_table_ok first)
    FusedSync S;
    if (fused) fused_sync_layout(G, F, &S, ws.fused);
    if (split_read) fused_sync_layout(LP.Gf, F, &S, ws.fused);   // F is the front part's plan
    const bool handoff = fused || split_read;
    if (handoff) S.gave_up_flag = ws.status_flag;
    if (!already_prepared) {
        if (launch_prepare(handoff ? S.part : nullptr, handoff ? fused_sync_pairs(F) : 0,
                           prepare_select ? &ws.sel : nullptr, G.Hkv * G.g, st, ws.status_flag) != hipSuccess)   // scratch is laid out per query head
            return SNAPKV_ERR_HIP;
        stage_done(st, kStagePrepare);
    }
    if (clean && handoff) {
        clean->ones = reinterpret_cast<unsigned long long*>(S.part);
        clean->nones = fused_sync_pairs(F);
    }
    if (fused) {   // K is read once; otherwise two passes over K, or over the part of it the chip cannot hold
        if ((layers ? launch_score_fused_layers(dtype, D, *layers, G, F, S, ws.vote, st)
                    : launch_score_fused(dtype, D, q_win, k, G, F, S, ws.vote, st)) != hipSuccess)
            return SNAPKV_ERR_HIP;
        stage_done(st, kStageFused);
        Gp.NV = G.g * F.BH;   // one vote row per query head, or per 32-row block of its window
        Gp.VB = F.BH;
    } else if (split_read) {
        // the rest's key 0 is key `front` of the prompt: an address offset, or (paged K) a logical row offset
        const char* k_rest = static_cast<const char*>(k) + (G.k_table ? 0 : LP.front * G.k_rs);
        // where a key's window logits are fewer bytes than its K row, the rest's keys are read once too: the
        // statistics pass keeps its logits and the votes come from those
        const bool keep_logits = LP.Fr.RUW == 1 && LP.Fr.gs == 1 && ws.long_logit &&
                                 (size_t)LP.Fr.units * (size_t)long_logit_keys(LP.Fr) * 16 * sizeof(float) <= ws.long_logit_bytes;
        ScoreLayers rest_layers;   // separately allocated layers: every layer's rest starts `front` rows into its K
        if (layers) {
            rest_layers = *layers;
            for (int x = 0; x < rest_layers.count; ++x)
                rest_layers.k[x] = static_cast<const char*>(layers->k[x]) + LP.front * G.k_rs;
        }
        const ScoreLayers* const rl = layers ? &rest_layers : nullptr;
        if (launch_row_lse(dtype, D, q_win, k_rest, LP.Gr, LP.Fr, ws.stat_part, nullptr, st,
                           keep_logits ? ws.long_logit : nullptr, rl) != hipSuccess)
            return SNAPKV_ERR_HIP;
        if (launch_publish_rest(ws.stat_part, S, LP, st) != hipSuccess) return SNAPKV_ERR_HIP;
        stage_done(st, kStageReduce);
        S.lse_out = ws.lse;
        if ((layers ? launch_score_fused_layers(dtype, D, *layers, LP.Gf, LP.Ff, S, ws.vote, st)
                    : launch_score_fused(dtype, D, q_win, k, LP.Gf, LP.Ff, S, ws.vote, st)) != hipSuccess)
            return SNAPKV_ERR_HIP;
        stage_done(st, kStageFused);
        if ((keep_logits ? launch_votes_from_logits(ws.long_logit, ws.lse, ws.vote + LP.front, LP, st)
                         : launch_score_lse(dtype, D, q_win, k_rest, ws.lse, LP.Gr, LP.Fr, ws.vote + LP.front, st, rl)) != hipSuccess)
            return SNAPKV_ERR_HIP;
        stage_done(st, kStagePass2);
        Gp.NV = G.g;
        Gp.VB = 1;
    } else if (path == kPathStream) {
        // two streaming passes over K with nothing handed between workgroups: the rows'
        // log-sum-exp first, then the probabilities from it
        if (launch_row_lse(dtype, D, q_win, k, G, F, ws.stat_part, ws.lse, st, nullptr, layers) != hipSuccess) return SNAPKV_ERR_HIP;
        if (launch_score_lse(dtype, D, q_win, k, ws.lse, G, F, ws.vote, st, layers) != hipSuccess) return SNAPKV_ERR_HIP;
        stage_done(st, kStagePass2);
        Gp.NV = G.g * F.BH;
        Gp.VB = F.BH;
    } else {   // a window of more than 128 rows that is not a whole number of 32-row blocks, or whose caller needs one vote row per head
        return SNAPKV_ERR_UNSUPPORTED;
    }
    if (Gv) *Gv = Gp;
    if (!score) return SNAPKV_OK;
    if (launch_pool(Gp, ws.vote, pool_kind, p, score, minmax, st) != hipSuccess) return SNAPKV_ERR_HIP;
    stage_done(st, kStagePool);
    return SNAPKV_OK;
}

// What the entry points vary on top of the plain step.
struct CompressOptions {
    void* workspace = nullptr;          // caller's workspace; null: the library's own per-device buffer
    size_t workspace_bytes = 0;
    bool own_scratch = true;
    const float* lse = nullptr;         // the window rows' log-sum-exp, when the caller hands it in
    bool with_lse = false;
    const RowLayout* k_layout = nullptr;   // null: contiguous [Hkv, L, D]
    const RowLayout* v_layout = nullptr;
    bool per_query_head = false;        // one selection and one cache per query head
    PageMap pm;                         // paged K and V
    int32_t* status = nullptr;          // device word of the caller's that receives the call's verdict
    // the heads are those of several separately allocated layers (Hq and Hkv count all of them; q_win, k, v and
    // the outputs are then taken from these tables, library's own scratch only)
    const ScoreLayers* score_layers = nullptr;
    const GatherLayers* gather_layers = nullptr;
};

int64_t compress_impl(int dtype, const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                      int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k,
                      void* out_v, int32_t* out_idx, void* stream, const CompressOptions& opt = CompressOptions{}) {
    void* const workspace = opt.workspace;
    const size_t workspace_bytes = opt.workspace_bytes;
    const bool own_scratch = opt.own_scratch, with_lse = opt.with_lse, per_query_head = opt.per_query_head;
    const float* const lse = opt.lse;
    const RowLayout *const k_layout = opt.k_layout, *const v_layout = opt.v_layout;
    const PageMap& pm = opt.pm;
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    if (with_lse && !lse) return SNAPKV_ERR_INVALID_ARG;
    if (with_lse && (reinterpret_cast<uintptr_t>(lse) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    int rc = check_score_args(q_win, k, L, Hq, Hkv, D, W, pool_kind, p);
    if (rc != SNAPKV_OK) return rc;
    if (!v || !out_k || !out_v || !out_idx) return SNAPKV_ERR_INVALID_ARG;
    if (C < 1 || W > C) return SNAPKV_ERR_INVALID_ARG;
    if (C >= (int64_t)1 << 31) return SNAPKV_ERR_UNSUPPORTED;
    if (!aligned16(v) || !aligned16(out_k) || !aligned16(out_v)) return SNAPKV_ERR_MISALIGNED;
    if ((reinterpret_cast<uintptr_t>(out_idx) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int row_bytes = D * elem_bytes(dtype);
    // byte strides of K and V: contiguous [Hkv, L, D] unless the caller says otherwise
    const RowLayout contiguous{(int64_t)L * row_bytes, (int64_t)row_bytes};
    const RowLayout kl = k_layout ? *k_layout : contiguous, vl = v_layout ? *v_layout : contiguous;
    for (const RowLayout* x : {&kl, &vl}) {
        if (x->row_stride < row_bytes || x->head_stride < 0) return SNAPKV_ERR_INVALID_ARG;
        if (((x->row_stride | x->head_stride) & 15) != 0) return SNAPKV_ERR_MISALIGNED;
    }

    // heads that select and keep rows: the KV heads, or every query head for itself
    const int Hout = per_query_head ? Hq : Hkv;
    const int head_div = per_query_head ? Hq / Hkv : 1;
    if (opt.status && (reinterpret_cast<uintptr_t>(opt.status) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    if (L <= C) {   // Listing 1, first branch: the prompt already fits
        if (launch_iota(Hout, L, C, out_idx, st) != hipSuccess) return SNAPKV_ERR_HIP;
        CleanJob verdict;
        verdict.status = opt.status;
        verdict.rows = (int32_t)L;
        if (launch_gather(k, v, out_idx, Hout, L, L, C, row_bytes, out_k, out_v, kl, vl, verdict, st, head_div, pm) != hipSuccess)
            return SNAPKV_ERR_HIP;
        return L;
    }

    ScoreGeom G = make_geom(L, Hq, Hkv, D, W);
    G.k_hs = kl.head_stride;
    G.k_rs = kl.row_stride;
    G.k_table = pm.table;
    G.k_page = pm.page;
    G.k_pages = pm.pages;
    const size_t need = workspace_layout(G, nullptr, nullptr);
    const size_t need_up = (need + 255) & ~(size_t)255;
    void* base = workspace;
    CleanState was_clean;
    unsigned* sticky = nullptr;
    const ScoreLayers* const score_layers = opt.score_layers;
    const GatherLayers* const gather_layers = opt.gather_layers;
    if ((score_layers != nullptr) != (gather_layers != nullptr)) return SNAPKV_ERR_INVALID_ARG;
    if (score_layers && (!own_scratch || per_query_head || lse || k_layout || v_layout || pm.table)) return SNAPKV_ERR_UNSUPPORTED;
    // separately allocated layers: the kept positions of all heads go to one array behind the workspace, from
    // which the gather copies them to the layers' own
    const size_t idx_tmp_bytes = score_layers ? ((size_t)Hout * (size_t)C * sizeof(int32_t) + 255) & ~(size_t)255 : 0;
    if (own_scratch) {
        if (capturing(st)) return SNAPKV_ERR_UNSUPPORTED;
        rc = internal_scratch(need_up + idx_tmp_bytes, &base, &was_clean, &sticky);
        if (rc != SNAPKV_OK) return rc;
        // An earlier call on this scratch whose kernels have finished by now had a bounded wait give up: its
        // results were invalid.  Said once, here, since that call had already returned when it happened.
        if (__hip_atomic_load(sticky, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0u) {
            __hip_atomic_store(sticky, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            return SNAPKV_ERR_TIMEOUT;
        }
    } else {
        if (!workspace || workspace_bytes < need) return SNAPKV_ERR_WORKSPACE;
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SNAPKV_ERR_MISALIGNED;
    }
    Workspace ws;
    workspace_layout(G, &ws, base);
    int32_t* const idx_dst = score_layers ? reinterpret_cast<int32_t*>(static_cast<char*>(base) + need_up) : out_idx;
    stage_done(st, kStageBegin);
    hipError_t se;
    CleanJob clean;
    clean.flag = ws.status_flag;
    clean.status = opt.status;
    clean.sticky = sticky;
    clean.rows = (int32_t)C;
    DeviceScratch* mine = nullptr;      // the library's own buffer: its state is tracked between calls
    CleanState now;
    bool streaming = false;
    // Per-query-head form: the votes are laid out [Hq][n] (one row per query head, which the
    // single-read and streaming kernels produce), so pooling and selection see Hq heads of one.
    // a window of 64, 96, ... rows may be scored block by block (one vote row per 32-row block); the
    // per-query-head form and the handed-in log-sum-exp keep one vote row per query head
    const bool blocks_ok = !per_query_head && !lse && !score_layers;
    ScoreGeom Gsel = G;
    if (per_query_head) {
        FusedGeom Ft;
        if (!lse_plan(dtype, D, G, &Ft)) return SNAPKV_ERR_UNSUPPORTED;   // more window rows than those kernels take
        Gsel.Hkv = Hq;
        Gsel.g = 1;
        Gsel.NV = 1;
        Gsel.VB = 1;
    }
    // which scoring path run_scores will take, and how many vote rows per query head it leaves
    FusedGeom Fp;
    LongPlan LPp;
    const int path = scoring_path(dtype, D, G, lse != nullptr, blocks_ok, true, &Fp, &LPp);
    if (path == kPathNone) return SNAPKV_ERR_UNSUPPORTED;
    if (!per_query_head && (path == kPathFused || path == kPathStream)) {
        Gsel.VB = Fp.BH;
        Gsel.NV = G.g * Fp.BH;
    }
    if (g_allow_pool_select && pool_select_ok(Gsel, pool_kind, p, C - W)) {   // pooling and selection in one launch
        bool prepared = false;
        streaming = path == kPathStream;
        if (own_scratch && path != kPathNone) {
            int dev = 0;
            if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) {
                // the streaming path does not touch the hand-off words
                const int64_t nones = streaming ? 0 : fused_sync_pairs(Fp);
                now.hkv = Hkv;
                now.hq = Hq;
                now.fused_bytes = fused_sync_bytes(G);
                now.stream = st;
                // (a call on another stream is not ordered behind the kernel that left the state)
                const bool same = was_clean.ones >= 0 && was_clean.hkv == now.hkv && was_clean.hq == now.hq &&
                                  was_clean.fused_bytes == now.fused_bytes && was_clean.stream == st;
                prepared = same && was_clean.ones >= nones;
                now.ones = same && was_clean.ones > nones ? was_clean.ones : nones;
                mine = &g_scratch[dev];
            }
        }
        ScoreGeom Gv = G;
        rc = run_scores(dtype, q_win, k, D, G, ws, pool_kind, p, nullptr, nullptr, true, &Gv, st, prepared,
                        mine ? &clean : nullptr, lse, blocks_ok, true, score_layers);
        if (rc != SNAPKV_OK) return rc;
        if (per_query_head) Gv = Gsel;
        se = launch_pool_select(Gv, ws.vote, pool_kind, p, C - W, C, W, idx_dst, ws.sel, st);
        if (mine) {
            clean.zeros = ws.sel.ps_arrive;
            clean.nzeros = ws.sel.ps_zero_words;
        }
    } else {
        if (per_query_head) {   // votes first, then pooled per query head
            ScoreGeom Gv = G;
            rc = run_scores(dtype, q_win, k, D, G, ws, pool_kind, p, nullptr, nullptr, true, &Gv, st, false, nullptr, lse,
                            false, true);
            if (rc != SNAPKV_OK) return rc;
            if (Gv.VB != 1 || Gv.NV != G.g) return SNAPKV_ERR_UNSUPPORTED;
            if (launch_pool(Gsel, ws.vote, pool_kind, p, ws.score, ws.sel.minmax, st) != hipSuccess)
                return SNAPKV_ERR_HIP;
            stage_done(st, kStagePool);
        } else {
            rc = run_scores(dtype, q_win, k, D, G, ws, pool_kind, p, ws.score, ws.sel.minmax,
                            true, nullptr, st, false, nullptr, lse, blocks_ok, true, score_layers);
            if (rc != SNAPKV_OK) return rc;
        }
        se = launch_select_chunked(ws.score, Hout, G.n, C - W, C, W, idx_dst, ws.sel, pool_tiles(G.n), st);
    }
    if (se != hipSuccess) return SNAPKV_ERR_HIP;
    stage_done(st, kStageSelect);
    if ((gather_layers ? launch_gather_layers(*gather_layers, idx_dst, L, C, C, row_bytes, clean, st)
                       : launch_gather(k, v, out_idx, Hout, L, C, C, row_bytes, out_k, out_v, kl, vl, clean, st, head_div, pm)) != hipSuccess)
        return SNAPKV_ERR_HIP;
    if (mine && (clean.ones || streaming) && clean.zeros) {
        std::lock_guard<std::mutex> lock(g_mu);
        mine->clean = now;
    }
    stage_done(st, kStageGather);
    return C;
}

int scores_impl(int dtype, const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D, int W,
                int pool_kind, int p, float* out_scores, void* stream, const float* lse = nullptr,
                bool with_lse = false) {
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    int rc = check_score_args(q_win, k, L, Hq, Hkv, D, W, pool_kind, p);
    if (rc != SNAPKV_OK) return rc;
    if (with_lse && !lse) return SNAPKV_ERR_INVALID_ARG;
    if (with_lse && (reinterpret_cast<uintptr_t>(lse) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    if (!out_scores) return SNAPKV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(out_scores) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    if (L == W) return SNAPKV_OK;   // empty prefix: nothing to score
    ScoreGeom G = make_geom(L, Hq, Hkv, D, W);
    G.k_rs = (int64_t)D * elem_bytes(dtype);
    G.k_hs = G.k_rs * L;
    void* base = nullptr;
    if (capturing(static_cast<hipStream_t>(stream))) return SNAPKV_ERR_UNSUPPORTED;
    rc = internal_scratch(workspace_layout(G, nullptr, nullptr), &base);
    if (rc != SNAPKV_OK) return rc;
    Workspace ws;
    workspace_layout(G, &ws, base);
    return run_scores(dtype, q_win, k, D, G, ws, pool_kind, p, out_scores, nullptr, false, nullptr,
                      static_cast<hipStream_t>(stream), false, nullptr, lse, !lse, true);
}

}  // namespace

namespace snapkv {
void stage_done(hipStream_t st, int stage);
}

namespace {

// Selection and gather of several prompts of one model in one launch each (the scoring kernel still
// runs once per prompt, into vote rows padded to the longest prefix).  Returns SNAPKV_OK, a negative
// error, or 1 when this batch has to be done prompt by prompt (shapes the joint kernels do not take).
int compress_batch(int dtype, int count, const void* const* q_win, const void* const* k, const void* const* v,
                   const int64_t* L, int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                   void* const* out_k, void* const* out_v, int32_t* const* out_idx, hipStream_t st) {
    if (count < 2 || count > kMaxBatch || !g_allow_pool_select) return 1;
    if (capturing(st)) return SNAPKV_ERR_UNSUPPORTED;
    if ((int64_t)Hkv * count > 65535) return 1;   // the joint gather has one grid row per head of the batch
    const int g = Hq / Hkv;
    const int row_bytes = D * elem_bytes(dtype);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    ScoreGeom G[kMaxBatch];
    int64_t nmax = 0;
    size_t per_prompt[kMaxBatch], stats = 0, handoff = 0;   // handoff: bytes of hand-off words per prompt
    for (int i = 0; i < count; ++i) {
        G[i] = make_geom(L[i], Hq, Hkv, D, W);
        G[i].k_rs = row_bytes;
        G[i].k_hs = (int64_t)row_bytes * L[i];
        FusedGeom F;
        if (!lse_plan(dtype, D, G[i], &F)) return 1;   // more window rows than the one-row-per-head kernels take
        if (g_allow_fused && fused_plan(dtype, D, G[i], &F)) {   // hand-off words this prompt's launch will use
            const size_t words = (size_t)fused_sync_pairs(F) * sizeof(unsigned long long);
            handoff = words > handoff ? words : handoff;
        }
        nmax = G[i].n > nmax ? G[i].n : nmax;
        per_prompt[i] = up(stream_stat_bytes(G[i])) + up(sizeof(float) * (size_t)Hq * W);
        stats += per_prompt[i];
    }
    const int64_t npad = (nmax + 3) & ~(int64_t)3;
    const int Htot = Hkv * count;
    ScoreGeom Gb = make_geom(npad + W, Hq * count, Htot, D, W);   // the batch as one prompt of count * Hkv heads
    Gb.NV = g;
    Gb.VB = 1;
    if (!pool_select_ok(Gb, pool_kind, p, C - W)) return 1;

    const size_t counters = select_counter_bytes(Htot);
    handoff = up(handoff);
    const size_t votes = up(sizeof(float) * (size_t)Hq * count * (size_t)npad);
    const size_t idx_tmp = up(sizeof(int32_t) * (size_t)Htot * (size_t)C);
    const size_t nvalid = up(sizeof(int32_t) * (size_t)Htot);
    const size_t sel = select_layout(Htot, npad, nullptr, nullptr, false, nullptr);
    const size_t need = counters + handoff * count + votes + stats + idx_tmp + nvalid + sel;
    void* base = nullptr;
    int rc = internal_scratch(need, &base);
    if (rc != SNAPKV_OK) return rc;
    char* b = static_cast<char*>(base);
    char* handoff_p = b + counters;
    float* votes_p = reinterpret_cast<float*>(handoff_p + handoff * count);
    char* stats_p = reinterpret_cast<char*>(votes_p) + votes;
    int32_t* idx_p = reinterpret_cast<int32_t*>(stats_p + stats);
    int32_t* nvalid_p = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(idx_p) + idx_tmp);
    SelectScratch Sb;
    select_layout(Htot, npad, &Sb, reinterpret_cast<char*>(nvalid_p) + nvalid, false, b);

    BatchDesc B;
    B.count = count;
    B.Hkv = Hkv;
    for (int i = 0; i < count; ++i) {
        B.L[i] = L[i];
        B.n[i] = G[i].n;
        B.k[i] = k[i];
        B.v[i] = v[i];
        B.out_k[i] = out_k[i];
        B.out_v[i] = out_v[i];
        B.out_idx[i] = out_idx[i];
    }
    stage_done(st, kStageBegin);
    if (launch_prepare(handoff_p, (int64_t)(handoff * count / sizeof(unsigned long long)), &Sb, Htot, st) != hipSuccess)
        return SNAPKV_ERR_HIP;
    if (launch_batch_lengths(B, nvalid_p, st) != hipSuccess) return SNAPKV_ERR_HIP;
    stage_done(st, kStagePrepare);
    // scoring: the prompts, longest first, share launches of the single-read kernel as far as they fit
    // the chip together; a prompt that kernel does not take is scored by a launch sequence of its own
    Workspace wsp[kMaxBatch];
    char* sp = stats_p;
    for (int i = 0; i < count; ++i) {
        wsp[i] = Workspace{};
        wsp[i].fused = handoff_p + handoff * i;
        wsp[i].vote = votes_p + (size_t)i * Hq * (size_t)npad;
        wsp[i].stat_part = reinterpret_cast<float2*>(sp);
        wsp[i].lse = reinterpret_cast<float*>(sp + up(stream_stat_bytes(G[i])));
        sp += per_prompt[i];
        G[i].vpitch = npad;
    }
    int rest[kMaxBatch], nrest = count;
    for (int i = 0; i < count; ++i) rest[i] = i;
    std::sort(rest, rest + count, [&](int a, int b) { return L[a] != L[b] ? L[a] > L[b] : a < b; });
    while (nrest > 0) {
        ScoreGeom Gr[kMaxBatch];
        FusedGeom Fr[kMaxBatch];
        for (int r = 0; r < nrest; ++r) Gr[r] = G[rest[r]];
        int take[kMaxJointPrompts], wg_begin[kMaxJointPrompts], grid = 0;
        const int taken = g_allow_fused ? fused_joint_plan(dtype, D, nrest, Gr, Fr, take, wg_begin, &grid) : 0;
        if (taken == 0) {   // the longest of the rest goes alone
            const int i = rest[0];
            ScoreGeom Gv = G[i];
            rc = run_scores(dtype, q_win[i], k[i], D, G[i], wsp[i], pool_kind, p, nullptr, nullptr, false, &Gv, st, true);
            if (rc != SNAPKV_OK) return rc;
            if (Gv.VB != 1 || Gv.NV != g) return SNAPKV_ERR_UNSUPPORTED;   // not reached: lse_plan held above
            for (int r = 1; r < nrest; ++r) rest[r - 1] = rest[r];
            --nrest;
            continue;
        }
        const void *jq[kMaxJointPrompts], *jk[kMaxJointPrompts];
        float* jv[kMaxJointPrompts];
        ScoreGeom jG[kMaxJointPrompts];
        FusedGeom jF[kMaxJointPrompts];
        FusedSync jS[kMaxJointPrompts];
        for (int t = 0; t < taken; ++t) {
            const int i = rest[take[t]];
            jq[t] = q_win[i];
            jk[t] = k[i];
            jv[t] = wsp[i].vote;
            jG[t] = G[i];
            jF[t] = Fr[take[t]];
            fused_sync_layout(jG[t], jF[t], &jS[t], wsp[i].fused);
        }
        if (launch_score_fused_joint(dtype, D, taken, jq, jk, jG, jF, jS, jv, wg_begin, grid, st) != hipSuccess)
            return SNAPKV_ERR_HIP;
        stage_done(st, kStageFused);
        int keep = 0;
        for (int r = 0, t = 0; r < nrest; ++r) {
            if (t < taken && take[t] == r) ++t;
            else rest[keep++] = rest[r];
        }
        nrest = keep;
    }
    if (launch_pool_select(Gb, votes_p, pool_kind, p, C - W, C, W, idx_p, Sb, st, nvalid_p) != hipSuccess)
        return SNAPKV_ERR_HIP;
    stage_done(st, kStageSelect);
    if (launch_gather_batch(B, idx_p, C, row_bytes, CleanJob{}, st) != hipSuccess) return SNAPKV_ERR_HIP;
    stage_done(st, kStageGather);
    return SNAPKV_OK;
}

}  // namespace

namespace snapkv {
unsigned wait_limit(unsigned dflt) {
    const long long v = g_wait_limit.load();
    return v < 0 ? dflt : (unsigned)v;
}

void stage_done(hipStream_t st, int stage) {
    if (!g_prof.active) return;
    if (stage == kStageBegin) {
        if (g_prof.calls >= g_prof.max_calls) return;
        ++g_prof.calls;
        g_prof.in_call = true;
    }
    if (!g_prof.in_call) return;   // e.g. a scores-only call: not a recorded call
    const size_t at = (size_t)(g_prof.calls - 1) * kNumStageMarks + stage;
    if (hipEventRecord(g_prof.ev[at], st) == hipSuccess) g_prof.set[at] = 1;
    if (stage == kStageGather) g_prof.in_call = false;
}
}  // namespace snapkv

extern "C" {

int snapkv_profile_start(int max_calls) {
    if (max_calls < 1 || max_calls > 4096) return SNAPKV_ERR_INVALID_ARG;
    if (g_prof.active) return SNAPKV_ERR_INVALID_ARG;
    g_prof.ev.assign((size_t)max_calls * kNumStageMarks, nullptr);
    g_prof.set.assign((size_t)max_calls * kNumStageMarks, 0);
    for (auto& e : g_prof.ev)
        if (hipEventCreate(&e) != hipSuccess) return SNAPKV_ERR_HIP;
    g_prof.max_calls = max_calls;
    g_prof.calls = 0;
    g_prof.in_call = false;
    g_prof.active = true;
    return SNAPKV_OK;
}

int snapkv_profile_stop(double* stage_ms, int* calls) {
    if (!g_prof.active) return SNAPKV_ERR_INVALID_ARG;
    g_prof.active = false;
    int rc = SNAPKV_OK;
    if (hipDeviceSynchronize() != hipSuccess) rc = SNAPKV_ERR_HIP;
    double sum[kNumStageMarks] = {0};
    int counted = 0;
    for (int c = 0; c < g_prof.calls && rc == SNAPKV_OK; ++c) {
        const size_t base = (size_t)c * kNumStageMarks;
        if (!g_prof.set[base + kStageBegin] || !g_prof.set[base + kStageGather]) continue;
        int prev = kStageBegin;   // a stage that did not run has no mark and keeps a zero duration
        for (int s = 1; s < kNumStageMarks; ++s) {
            if (!g_prof.set[base + s]) continue;
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, g_prof.ev[base + prev], g_prof.ev[base + s]) != hipSuccess)
                rc = SNAPKV_ERR_HIP;
            sum[s] += ms;
            prev = s;
        }
        ++counted;
    }
    for (auto& e : g_prof.ev)
        if (e) (void)hipEventDestroy(e);
    g_prof.ev.clear();
    g_prof.set.clear();
    if (stage_ms)
        for (int s = 1; s < kNumStageMarks; ++s) stage_ms[s - 1] = counted ? sum[s] / counted : 0.0;
    if (calls) *calls = counted;
    return rc;
}

int snapkv_debug_set_wait_limit(long long polls) {
    g_wait_limit.store(polls < 0 ? -1 : (polls > 0x7fffffffLL ? 0x7fffffffLL : polls));
    if (polls == -2 && (!reset_sync_timeouts() || !reset_select_timeouts())) return SNAPKV_ERR_HIP;
    return SNAPKV_OK;
}

int snapkv_set_scoring_scheme(int scheme) {
    if (scheme < 0 || scheme > 7) return SNAPKV_ERR_INVALID_ARG;
    g_allow_fused = (scheme & 1) == 0;
    g_allow_pool_select = (scheme & 2) == 0;
    g_fused_slot_cap = (scheme & 4) ? 16 : 0;
    return SNAPKV_OK;
}

int64_t snapkv_sync_timeouts(void) {
    const unsigned v = read_sync_timeouts(), u = read_select_timeouts();
    return (v == ~0u || u == ~0u) ? (int64_t)SNAPKV_ERR_HIP : (int64_t)v + (int64_t)u;
}

int snapkv_num_stages(void) { return kNumStageMarks - 1; }

const char* snapkv_stage_name(int stage) {
    static const char* names[] = {"prepare_scratch", "score_stats", "score_merge", "score_fused", "score_stream",
                                  "pool_group", "select_topk", "gather_rows"};
    return stage >= 0 && stage < kNumStageMarks - 1 ? names[stage] : "";
}

int snapkv_version(void) { return 100; }

const char* snapkv_strerror(int code) {
    switch (code) {
        case SNAPKV_OK: return "ok";
        case SNAPKV_ERR_INVALID_ARG: return "invalid argument";
        case SNAPKV_ERR_UNSUPPORTED: return "unsupported shape";
        case SNAPKV_ERR_MISALIGNED: return "pointer not sufficiently aligned";
        case SNAPKV_ERR_WORKSPACE: return "workspace missing or too small";
        case SNAPKV_ERR_HIP: return "HIP call failed";
        case SNAPKV_ERR_TIMEOUT: return "a bounded wait inside a kernel gave up";
        default: return code > 0 ? "ok" : "unknown error";
    }
}

int64_t snapkv_compress(const void* q_win, const void* k, const void* v, int64_t L, int Hq, int Hkv,
                        int D, int W, int pool_kind, int p, int64_t C, void* out_k, void* out_v,
                        int32_t* out_idx, void* stream) {
    return compress_impl(SNAPKV_DTYPE_BF16, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k,
                         out_v, out_idx, stream);
}

int64_t snapkv_compress_f32(const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                            int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k,
                            void* out_v, int32_t* out_idx, void* stream) {
    return compress_impl(SNAPKV_DTYPE_F32, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k,
                         out_v, out_idx, stream);
}

int64_t snapkv_compress_ws(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                           int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                           void* out_k, void* out_v, int32_t* out_idx, void* workspace,
                           size_t workspace_bytes, void* stream) {
    CompressOptions opt;
    opt.workspace = workspace;
    opt.workspace_bytes = workspace_bytes;
    opt.own_scratch = false;
    return compress_impl(dtype, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int64_t snapkv_compress_static(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                               int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                               void* out_k, void* out_v, int32_t* out_idx, void* stream) {
    // the size is checked first: a shape that does not fit is refused before anything else happens
    if (L >= 1 && W >= 1 && W <= L && Hq >= 1 && Hkv >= 1 && Hq % Hkv == 0 && (D == 64 || D == 128) &&
        L < ((int64_t)1 << 31) && L > C &&
        workspace_layout(make_geom(L, Hq, Hkv, D, W), nullptr, nullptr) > (size_t)SNAPKV_STATIC_SCRATCH_BYTES)
        return SNAPKV_ERR_WORKSPACE;
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != SNAPKV_OK) return rc;
    CompressOptions opt;
    opt.workspace = ptr;                   // the looked-up device address, never the array's name
    opt.workspace_bytes = SNAPKV_STATIC_SCRATCH_BYTES;
    opt.own_scratch = false;               // everything that must start at zero is cleared by the call's first kernel
    return compress_impl(dtype, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int64_t snapkv_compress_ws_status(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                                  int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                                  void* out_k, void* out_v, int32_t* out_idx, void* workspace,
                                  size_t workspace_bytes, int32_t* status, void* stream) {
    if (!status) return SNAPKV_ERR_INVALID_ARG;
    CompressOptions opt;
    opt.workspace = workspace;
    opt.workspace_bytes = workspace_bytes;
    opt.own_scratch = false;
    opt.status = status;
    return compress_impl(dtype, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int snapkv_pooled_scores(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D, int W,
                         int pool_kind, int p, float* out_scores, void* stream) {
    return scores_impl(SNAPKV_DTYPE_BF16, q_win, k, L, Hq, Hkv, D, W, pool_kind, p, out_scores, stream);
}

int snapkv_pooled_scores_f32(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D,
                             int W, int pool_kind, int p, float* out_scores, void* stream) {
    return scores_impl(SNAPKV_DTYPE_F32, q_win, k, L, Hq, Hkv, D, W, pool_kind, p, out_scores, stream);
}

int64_t snapkv_compress_f16(const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                            int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k,
                            void* out_v, int32_t* out_idx, void* stream) {
    return compress_impl(SNAPKV_DTYPE_F16, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k,
                         out_v, out_idx, stream);
}

int snapkv_pooled_scores_f16(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D,
                             int W, int pool_kind, int p, float* out_scores, void* stream) {
    return scores_impl(SNAPKV_DTYPE_F16, q_win, k, L, Hq, Hkv, D, W, pool_kind, p, out_scores, stream);
}

int64_t snapkv_compress_lse(int dtype, const void* q_win, const void* k, const void* v, const float* lse,
                            int64_t L, int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                            void* out_k, void* out_v, int32_t* out_idx, void* stream) {
    CompressOptions opt;
    opt.lse = lse;
    opt.with_lse = true;
    return compress_impl(dtype, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int snapkv_pooled_scores_lse(int dtype, const void* q_win, const void* k, const float* lse, int64_t L,
                             int Hq, int Hkv, int D, int W, int pool_kind, int p, float* out_scores,
                             void* stream) {
    return scores_impl(dtype, q_win, k, L, Hq, Hkv, D, W, pool_kind, p, out_scores, stream, lse, true);
}

int64_t snapkv_compress_strided(int dtype, const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                                int Hkv, int D, int W, int64_t k_head_stride, int64_t k_row_stride,
                                int64_t v_head_stride, int64_t v_row_stride, int pool_kind, int p, int64_t C,
                                void* out_k, void* out_v, int32_t* out_idx, void* stream) {
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    const int64_t es = elem_bytes(dtype);
    if (k_head_stride < 0 || v_head_stride < 0 || k_row_stride < D || v_row_stride < D) return SNAPKV_ERR_INVALID_ARG;
    const int64_t lim = (int64_t)1 << 56;
    if (k_head_stride > lim || v_head_stride > lim || k_row_stride > lim || v_row_stride > lim) return SNAPKV_ERR_UNSUPPORTED;
    const RowLayout kl{k_head_stride * es, k_row_stride * es}, vl{v_head_stride * es, v_row_stride * es};
    CompressOptions opt;
    opt.k_layout = &kl;
    opt.v_layout = &vl;
    return compress_impl(dtype, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int64_t snapkv_compress_paged(int dtype, const void* q_win, const void* k_pages, const void* v_pages,
                              const int32_t* block_table, int64_t num_pages, int page_size, int64_t L, int Hq,
                              int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k, void* out_v,
                              int32_t* out_idx, void* stream) {
    if (!valid_dtype(dtype) || !block_table) return SNAPKV_ERR_INVALID_ARG;
    if (page_size < 1 || num_pages < 1 || L < 1 || (L + page_size - 1) / page_size > num_pages) return SNAPKV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(block_table) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    if (num_pages >= (int64_t)1 << 31 || Hkv < 1) return SNAPKV_ERR_UNSUPPORTED;
    // rows of a page are token-major: [num_pages, page_size, Hkv, D]
    const int64_t row = (int64_t)D * elem_bytes(dtype);
    const RowLayout lay{row, row * Hkv};
    PageMap pm;
    pm.table = block_table;
    pm.page = page_size;
    pm.pages = num_pages;
    CompressOptions opt;
    opt.k_layout = &lay;
    opt.v_layout = &lay;
    opt.pm = pm;
    return compress_impl(dtype, q_win, k_pages, v_pages, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int snapkv_compress_varlen(int dtype, int n_prompts, const void* const* q_win, const void* const* k,
                           const void* const* v, const int64_t* L, int Hq, int Hkv, int D, int W, int pool_kind,
                           int p, int64_t C, void* const* out_k, void* const* out_v, int32_t* const* out_idx,
                           int64_t* kept, void* stream) {
    if (n_prompts < 0 || (n_prompts > 0 && (!q_win || !k || !v || !L || !out_k || !out_v || !out_idx)))
        return SNAPKV_ERR_INVALID_ARG;
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    // every prompt is checked before anything is enqueued
    for (int i = 0; i < n_prompts; ++i) {
        int rc = check_score_args(q_win[i], k[i], L[i], Hq, Hkv, D, W, pool_kind, p);
        if (rc != SNAPKV_OK) return rc;
        if (!v[i] || !out_k[i] || !out_v[i] || !out_idx[i]) return SNAPKV_ERR_INVALID_ARG;
        if (C < 1 || W > C) return SNAPKV_ERR_INVALID_ARG;
        if (C >= (int64_t)1 << 31) return SNAPKV_ERR_UNSUPPORTED;
        if (!aligned16(v[i]) || !aligned16(out_k[i]) || !aligned16(out_v[i])) return SNAPKV_ERR_MISALIGNED;
        if ((reinterpret_cast<uintptr_t>(out_idx[i]) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    int order[kMaxBatch];
    int i = 0;
    while (i < n_prompts) {
        // the next run of prompts that need compressing (L > C), at most kMaxBatch of them
        int cnt = 0, j = i;
        for (; j < n_prompts && cnt < kMaxBatch; ++j) {
            if (L[j] > C) order[cnt++] = j;
            else {   // Listing 1, first branch: returned unchanged
                const int64_t r = compress_impl(dtype, q_win[j], k[j], v[j], L[j], Hq, Hkv, D, W, pool_kind, p, C,
                                                out_k[j], out_v[j], out_idx[j], stream);
                if (r < 0) return (int)r;
                if (kept) kept[j] = r;
            }
        }
        const void *bq[kMaxBatch], *bk[kMaxBatch], *bv[kMaxBatch];
        void *bok[kMaxBatch], *bov[kMaxBatch];
        int32_t* boi[kMaxBatch];
        int64_t bl[kMaxBatch];
        for (int c = 0; c < cnt; ++c) {
            const int s = order[c];
            bq[c] = q_win[s]; bk[c] = k[s]; bv[c] = v[s]; bok[c] = out_k[s]; bov[c] = out_v[s]; boi[c] = out_idx[s];
            bl[c] = L[s];
        }
        int rc = cnt > 0 ? compress_batch(dtype, cnt, bq, bk, bv, bl, Hq, Hkv, D, W, pool_kind, p, C, bok, bov, boi, st) : SNAPKV_OK;
        if (rc < 0) return rc;
        for (int c = 0; c < cnt; ++c) {
            const int s = order[c];
            if (rc == 1) {   // prompt by prompt
                const int64_t r = compress_impl(dtype, bq[c], bk[c], bv[c], bl[c], Hq, Hkv, D, W, pool_kind, p, C,
                                                bok[c], bov[c], boi[c], stream);
                if (r < 0) return (int)r;
            }
            if (kept) kept[s] = C;
        }
        i = j;
    }
    return SNAPKV_OK;
}

int snapkv_compress_layers(int dtype, int n_layers, const void* const* q_win, const void* const* k,
                           const void* const* v, int64_t L, int Hq, int Hkv, int D, int W, int pool_kind, int p,
                           int64_t C, void* const* out_k, void* const* out_v, int32_t* const* out_idx, void* stream) {
    if (n_layers < 0 || (n_layers > 0 && (!q_win || !k || !v || !out_k || !out_v || !out_idx))) return SNAPKV_ERR_INVALID_ARG;
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    for (int i = 0; i < n_layers; ++i) {   // every layer is checked before anything is enqueued
        const int rc = check_score_args(q_win[i], k[i], L, Hq, Hkv, D, W, pool_kind, p);
        if (rc != SNAPKV_OK) return rc;
        if (!v[i] || !out_k[i] || !out_v[i] || !out_idx[i]) return SNAPKV_ERR_INVALID_ARG;
        if (C < 1 || W > C) return SNAPKV_ERR_INVALID_ARG;
        if (C >= (int64_t)1 << 31) return SNAPKV_ERR_UNSUPPORTED;
        if (!aligned16(v[i]) || !aligned16(out_k[i]) || !aligned16(out_v[i])) return SNAPKV_ERR_MISALIGNED;
        if ((reinterpret_cast<uintptr_t>(out_idx[i]) & 3u) != 0) return SNAPKV_ERR_MISALIGNED;
    }
    // Layers that lie one behind the other in memory (a stacked [layers, heads, ...] tensor for each of the
    // seven arguments) are to the kernels one layer with that many more heads: heads are independent, and
    // a head's result does not depend on how many others the call has.
    const int64_t e = elem_bytes(dtype);
    const int64_t dq = (int64_t)Hq * W * D * e, dk = (int64_t)Hkv * L * D * e, dok = (int64_t)Hkv * C * D * e,
                  di = (int64_t)Hkv * C * (int64_t)sizeof(int32_t);
    auto follows = [&](int i) {   // layer i + 1 lies directly behind layer i in all seven tensors
        auto gap = [](const void* a, const void* b) { return static_cast<const char*>(b) - static_cast<const char*>(a); };
        return gap(q_win[i], q_win[i + 1]) == dq && gap(k[i], k[i + 1]) == dk && gap(v[i], v[i + 1]) == dk &&
               gap(out_k[i], out_k[i + 1]) == dok && gap(out_v[i], out_v[i + 1]) == dok &&
               gap(out_idx[i], out_idx[i + 1]) == di;
    };
    // the scratch of a run grows with its heads: runs are cut so that it stays under kLayersScratchCap
    const size_t per_layer = L > C ? workspace_layout(make_geom(L, Hq, Hkv, D, W), nullptr, nullptr) : 0;
    int most = (int)(kLayersScratchCap / (per_layer > 0 ? per_layer : 1));
    most = most < 1 ? 1 : most;
    if ((int64_t)most * Hkv > 65535) most = 65535 / Hkv;
    if (L <= C) most = 1;                  // prompts that fit are copied layer by layer (out rows [L, C) stay untouched)
    // Layers that are separate allocations go through the same launches by a table of their addresses (at most
    // kMaxLayerPtrs per run), where the single-read scoring kernel takes the prompt in that form; otherwise
    // one by one.
    int most_sep = most < kMaxLayerPtrs ? most : kMaxLayerPtrs;
    if (L <= C || (elem_bytes(dtype) != 2)) most_sep = 1;
    int i = 0;
    while (i < n_layers) {
        int r = 1;
        while (i + r < n_layers && r < most && follows(i + r - 1)) ++r;
        if (r == 1 && most_sep > 1) {   // a run of layers none of which lies behind its predecessor
            int t = 1;
            // (a layer that starts a stacked run is left to that run)
            while (i + t < n_layers && t < most_sep && (i + t + 1 >= n_layers || !follows(i + t))) ++t;
            if (t > 1) {
                ScoreGeom Gt = make_geom(L, Hq * t, Hkv * t, D, W);
                Gt.k_rs = (int64_t)D * e;
                Gt.k_hs = Gt.k_rs * L;
                if (layers_table_ok(dtype, D, Gt, Hkv)) {
                    ScoreLayers SL{};
                    GatherLayers GL{};
                    SL.count = GL.count = t;
                    SL.kv_heads = GL.heads = Hkv;
                    for (int x = 0; x < t; ++x) {
                        SL.q[x] = q_win[i + x];
                        SL.k[x] = GL.k[x] = k[i + x];
                        GL.v[x] = v[i + x];
                        GL.out_k[x] = out_k[i + x];
                        GL.out_v[x] = out_v[i + x];
                        GL.out_idx[x] = out_idx[i + x];
                    }
                    CompressOptions opt;
                    opt.score_layers = &SL;
                    opt.gather_layers = &GL;
                    const int64_t got = compress_impl(dtype, q_win[i], k[i], v[i], L, Hq * t, Hkv * t, D, W, pool_kind, p, C,
                                                      out_k[i], out_v[i], out_idx[i], stream, opt);
                    if (got < 0) return (int)got;
                    i += t;
                    continue;
                }
            }
        }
        const int64_t got = compress_impl(dtype, q_win[i], k[i], v[i], L, Hq * r, Hkv * r, D, W, pool_kind, p, C, out_k[i],
                                          out_v[i], out_idx[i], stream);
        if (got < 0) return (int)got;
        i += r;
    }
    return SNAPKV_OK;
}

int64_t snapkv_compress_per_query_head(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                                       int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                                       void* out_k, void* out_v, int32_t* out_idx, void* stream) {
    CompressOptions opt;
    opt.per_query_head = true;
    return compress_impl(dtype, q_win, k, v, L, Hq, Hkv, D, W, pool_kind, p, C, out_k, out_v, out_idx, stream, opt);
}

int64_t snapkv_capacity_for_rate(int64_t L, int W, double rate) {
    if (!(rate >= 0.0 && rate <= 1.0) || W < 1 || W > L) return SNAPKV_ERR_INVALID_ARG;
    return (int64_t)W + (int64_t)std::floor(rate * (double)(L - W));
}

size_t snapkv_workspace_bytes(int64_t L, int Hq, int Hkv, int D, int W) {
    if (L < 1 || W < 1 || W > L || Hq < 1 || Hkv < 1 || Hq % Hkv != 0) return 0;
    if (D != 64 && D != 128) return 0;
    if (L >= (int64_t)1 << 31) return 0;
    return workspace_layout(make_geom(L, Hq, Hkv, D, W), nullptr, nullptr);
}

int snapkv_select_topk(const float* scores, int H, int64_t n, int64_t kcount, int32_t* out_idx,
                       void* stream) {
    if (!scores || !out_idx) return SNAPKV_ERR_INVALID_ARG;
    if (H < 1 || n < 1 || kcount < 0 || kcount > n) return SNAPKV_ERR_INVALID_ARG;
    if (!select_chunked_ok(n)) return SNAPKV_ERR_UNSUPPORTED;
    if (kcount == 0) return SNAPKV_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void* base = nullptr;
    const int rc = internal_scratch(select_layout(H, n, nullptr, nullptr), &base);
    if (rc != SNAPKV_OK) return rc;
    SelectScratch S;
    select_layout(H, n, &S, base);
    if (launch_select_init(S, H, st) != hipSuccess) return SNAPKV_ERR_HIP;
    if (launch_select_chunked(scores, H, n, kcount, kcount, 0, out_idx, S, 0, st) != hipSuccess)
        return SNAPKV_ERR_HIP;
    return SNAPKV_OK;
}

int snapkv_decode_attention(int dtype, const void* q, const void* k_cache, const void* v_cache,
                            const int32_t* lens, int B, int Hq, int Hkv, int D, int64_t S, int64_t cap,
                            float* out, float* out_lse, void* stream) {
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    if (!q || !k_cache || !v_cache || !out) return SNAPKV_ERR_INVALID_ARG;
    if (B < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || cap < 1 || S < 1 || S > cap) return SNAPKV_ERR_INVALID_ARG;
    if (dtype == SNAPKV_DTYPE_F32 || (D != 64 && D != 128)) return SNAPKV_ERR_UNSUPPORTED;
    if (Hq / Hkv > 16 || Hkv > 65535 || B > 65535 || cap >= (int64_t)1 << 31) return SNAPKV_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return SNAPKV_ERR_MISALIGNED;
    if ((reinterpret_cast<uintptr_t>(out) & 3u) != 0 || (reinterpret_cast<uintptr_t>(out_lse) & 3u) != 0 ||
        (reinterpret_cast<uintptr_t>(lens) & 3u) != 0)
        return SNAPKV_ERR_MISALIGNED;
    const int nsplit = decode_splits(B, Hkv, S);
    const size_t need = decode_scratch_bytes(B, Hq, D, nsplit);
    void* base = nullptr;
    if (need > 0) {
        const int rc = aux_scratch(need, &base);
        if (rc != SNAPKV_OK) return rc;
    }
    return launch_decode(dtype, D, q, k_cache, v_cache, lens, B, Hq, Hkv, S, cap, nsplit, base, out, out_lse,
                         static_cast<hipStream_t>(stream)) == hipSuccess
               ? SNAPKV_OK
               : SNAPKV_ERR_HIP;
}

int snapkv_hit_rate(int dtype, const void* q_cur, const void* k, int64_t Lk, int64_t n, int Hq, int Hkv, int D,
                    const int32_t* idx, int Hidx, int64_t kcount, int64_t idx_stride, float theta,
                    int32_t* out_counts, void* stream) {
    if (!valid_dtype(dtype)) return SNAPKV_ERR_INVALID_ARG;
    if (!q_cur || !k || !out_counts) return SNAPKV_ERR_INVALID_ARG;
    if (Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || Lk < 1 || n < 0 || n > Lk) return SNAPKV_ERR_INVALID_ARG;
    if (Hidx < 1 || Hq % Hidx != 0 || kcount < 0 || kcount > idx_stride || (kcount > 0 && !idx)) return SNAPKV_ERR_INVALID_ARG;
    if (!(theta == theta)) return SNAPKV_ERR_INVALID_ARG;
    if (dtype == SNAPKV_DTYPE_F32 || (D != 64 && D != 128)) return SNAPKV_ERR_UNSUPPORTED;
    if (Hq / Hkv > 16 || Hkv > 65535 || Hq > 65535 || Lk >= (int64_t)1 << 31) return SNAPKV_ERR_UNSUPPORTED;
    if (!aligned16(q_cur) || !aligned16(k)) return SNAPKV_ERR_MISALIGNED;
    if ((reinterpret_cast<uintptr_t>(idx) & 3u) != 0 || (reinterpret_cast<uintptr_t>(out_counts) & 3u) != 0)
        return SNAPKV_ERR_MISALIGNED;
    void* base = nullptr;
    const int rc = aux_scratch(hit_rate_scratch_bytes(Hq, Lk), &base);
    if (rc != SNAPKV_OK) return rc;
    return launch_hit_rate(dtype, D, q_cur, k, Lk, n, Hq, Hkv, idx, Hidx, kcount, idx_stride, theta, base, out_counts,
                           static_cast<hipStream_t>(stream)) == hipSuccess
               ? SNAPKV_OK
               : SNAPKV_ERR_HIP;
}

void snapkv_release(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (int d = 0; d < kMaxDevices; ++d) {
        if (!g_scratch[d].ptr) continue;
        if (hipSetDevice(d) == hipSuccess) (void)hipFree(g_scratch[d].ptr);
        g_scratch[d].ptr = nullptr;
        g_scratch[d].bytes = 0;
        g_scratch[d].clean = CleanState{};
    }
    for (int d = 0; d < kMaxDevices; ++d) {
        if (!g_scratch[d].sticky) continue;
        if (hipSetDevice(d) == hipSuccess) (void)hipHostFree(g_scratch[d].sticky);
        g_scratch[d].sticky = nullptr;
    }
    for (int d = 0; d < kMaxDevices; ++d) {
        if (!g_decode_scratch[d].ptr) continue;
        if (hipSetDevice(d) == hipSuccess) (void)hipFree(g_decode_scratch[d].ptr);
        g_decode_scratch[d].ptr = nullptr;
        g_decode_scratch[d].bytes = 0;
    }
    if (have_cur) (void)hipSetDevice(cur);
}

}  // extern "C"
