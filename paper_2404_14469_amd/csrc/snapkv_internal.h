// Internal declarations shared by the host dispatcher and the kernel translation units.
// Nothing here is part of the public ABI (include/snapkv.h).
#ifndef SNAPKV_INTERNAL_H_
#define SNAPKV_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace snapkv {

// Geometry of a scoring call.  A "vote row" is one fp32 vector of length n: one per query head, or (windows of
// 64, 96, ... rows scored block by block) one per 32-row block of a query head's window.
struct ScoreGeom {
    int64_t L;       // prompt length
    int64_t n;       // prefix length L - W
    int W;           // observation window
    int g;           // query heads per KV head
    int Hkv;         // KV heads
    int BH;          // 32-row blocks per query head, ceil(W / 32)
    int NV;          // vote rows per KV head
    int VB;          // vote rows per query head
    float c2;        // log2(e) / sqrt(D): logits are kept in the base-2 domain
    int64_t k_hs;    // bytes between the K rows of consecutive KV heads (contiguous: L * D * element size)
    int64_t k_rs;    // bytes between consecutive K rows of a head (contiguous: D * element size)
    int64_t vpitch;  // floats between the vote rows of consecutive query heads (n unless a batch pads them)
    // paged K: logical row j lives at physical row k_table[j / k_page] * k_page + j % k_page (null: j itself)
    const int32_t* k_table;
    int k_page;
    int64_t k_pages;
    int64_t k_row0;  // paged K only: logical row of the cache at which this call's key 0 sits (the rest of a long prompt)
};

// Physical row of logical row j of a possibly paged tensor; page ids outside [0, pages) are clamped
// so that a bad table cannot send a load outside the allocation.
__device__ __forceinline__ int64_t physical_row(const int32_t* table, int page, int64_t pages, int64_t j) {
    if (!table) return j;
    int64_t pg = table[j / page];
    pg = pg < 0 ? 0 : (pg >= pages ? pages - 1 : pg);
    return pg * page + j % page;
}

// Layers of one prompt that are separate allocations (passed to kernels by value).  Head h of the call is head
// h % kv_heads of layer h / kv_heads; every layer has the contiguous [heads, rows, D] layout.
constexpr int kMaxLayerPtrs = 32;
struct ScoreLayers {
    int count, kv_heads;
    const void* q[kMaxLayerPtrs];
    const void* k[kMaxLayerPtrs];
};
struct GatherLayers {
    int count, heads;        // heads: output heads per layer
    const void* k[kMaxLayerPtrs];
    const void* v[kMaxLayerPtrs];
    void* out_k[kMaxLayerPtrs];
    void* out_v[kMaxLayerPtrs];
    int32_t* out_idx[kMaxLayerPtrs];
};

// Plan of the single-read scoring kernel (snapkv_fused.hip).  A unit is a KV head or one of
// `split` equal parts of its query heads; its window
// rows form RU units of 16 rows (UH per query head), padded to RUW, a power of two; a wave keeps
// KT tiles of 16 keys per row unit; Gg workgroups share one unit's keys; NG groups run at once.
struct FusedGeom {
    int RU, UH, RUW, KT, NW, Gg, NG, NB, units;   // NW waves per workgroup; NB blocks of 32 slices per row
    int NBX;                 // level-1 words per row a reader merges: NB, or NB + 1 when the word behind them is
                             // published before the launch (statistics of keys this launch does not read)
    int split, gs;           // units per KV head; query heads per unit (g = split * gs)
    int BH;                  // 1, or: every 32-row block of the window is a query head of its own to the
                             // kernel (BH blocks per real head; g, split and gs then count such blocks)
    int64_t ntiles;          // ceil(L / 16)
    unsigned spin_limit;     // bound on the hand-off wait, in polls
};

struct FusedSync {
    float2* part;            // [units][Gg][RUW*16] per-slice (row max, row sum-exp), base-2 domain
    float2* l1;              // [units][RUW*16][NB] the same merged over blocks of 32 slices
    unsigned* gave_up_flag;  // null, or a word of the call's scratch that is set when a bounded wait gives up
    float* lse_out;          // null, or [query heads][W]: the window rows' natural log-sum-exp, stored by the
                             // first workgroup of every group
};

// Scratch of the chunked top-k selection (snapkv_topk.hip), per head h of H heads.
struct SelectScratch {
    unsigned* minmax;      // [H][parts][2] smallest / largest score bit pattern per producer part
    unsigned* hist;        // [H][2048]   first-digit histogram
    unsigned* cand_count;  // [H][chunks] entries in each chunk's part of the candidate list
    unsigned* info;        // [H][4]      threshold search state; finally {T, -, need_eq, flat}
    unsigned* chunk_gt;    // [H][chunks] positions in bins above the threshold bin
    unsigned* chunk_off;   // [H][chunks][2] output offsets: (#greater, #equal) before the chunk
    uint2* cand;           // [H][n]      (pattern, position) of positions inside the threshold bin, by chunk
    // scratch of the cooperative pooling + selection kernel (pool_select), which keeps its candidates
    // in `cand` above; the first two arrays are contiguous and must be zero when the kernel starts
    // (ps_zero_words words from ps_arrive)
    unsigned* ps_arrive;   // [H][8]        arrival counters of the group-wide rendezvous points
    unsigned* ps_hist;     // [H][3][2048]  digit histograms, one per refinement level
    unsigned* ps_range;    // [H][512][2]   per-workgroup (smallest, largest) score bit pattern
    unsigned* ps_part;     // [H][512][2]   per-workgroup (#above the threshold bin, #inside it)
    int64_t ps_zero_words;
    unsigned* ps_flag;     // null, or a word of the call's scratch that is set when a bounded wait gives up
};

struct Workspace {
    unsigned* status_flag;   // first word of the block: set by a kernel whose bounded wait gave up, read and cleared by
                             // the call's last kernel
    float* vote;     // [Hkv][NV][n]
    float* score;    // [Hkv][n]
    char* fused;     // hand-off buffers of the single-read path (see fused_sync_layout)
    float2* stat_part;   // [units][Gg][R] per-slice (row max, row sum-exp) of the streaming statistics pass
    float* lse;          // [Hq][W] the window rows' log-sum-exp computed from them
    float* long_logit;   // null, or [units][keys][16] masked window logits of the keys a long prompt's single-read
    size_t long_logit_bytes;   // launch does not take (windows of at most 16 rows, one query head per KV head)
    SelectScratch sel;
};

ScoreGeom make_geom(int64_t L, int Hq, int Hkv, int D, int W);
size_t workspace_layout(const ScoreGeom& G, Workspace* ws, void* base);

// Stage boundaries for the optional per-stage timing (snapkv_profile_start/stop): when timing is
// active, stage_done records an event on the stream after the stage's launch; otherwise it is a
// no-op.  kStageBegin marks the start of a call.
enum Stage { kStageBegin = 0, kStagePrepare, kStagePass1, kStageReduce, kStageFused, kStagePass2,
             kStagePool, kStageSelect, kStageGather, kNumStageMarks };
void stage_done(hipStream_t st, int stage);

// All launchers enqueue on `st` and return the launch status.
size_t fused_sync_bytes(const ScoreGeom& G);
// allow_blocks: the plan may treat the 32-row blocks of a window longer than 32 rows as query heads
// of their own (F->BH > 1); the votes then have one row per block (NV = g * BH, VB = BH).
bool fused_plan(int dtype, int D, const ScoreGeom& G, FusedGeom* F, bool allow_blocks = false);
size_t fused_sync_layout(const ScoreGeom& G, const FusedGeom& F, FusedSync* S, void* base);
// A prompt of which one head's logits do not fit the chip's registers: the single-read kernel takes the
// first `front` keys (geometry Gf, plan Ff: as many as stay resident), the streaming kernels the rest
// (Gr, Fr: a prompt of L - front keys that ends in the same window), whose keys are so read twice.
// Order of the launches: row statistics of the rest; their merge into one hand-off word per row
// (launch_publish_rest); the single-read kernel, which merges that word with its own slices', votes on
// its keys and stores the rows' log-sum-exp; the streaming pass that votes on the rest from it.
struct LongPlan {
    ScoreGeom Gf, Gr;
    FusedGeom Ff, Fr;
    int64_t front;
};
bool long_plan(int dtype, int D, const ScoreGeom& G, LongPlan* P);
hipError_t launch_publish_rest(const float2* stat_part, const FusedSync& S, const LongPlan& P, hipStream_t st);
// (test hook) 0, or the number of workgroups the plans of the single-read kernel may count as resident
extern int g_fused_slot_cap;
// Several prompts of one model in one launch of the single-read kernel (snapkv_fused.hip).
constexpr int kMaxJointPrompts = 8;
int fused_joint_plan(int dtype, int D, int count, const ScoreGeom* G, FusedGeom* F, int* take, int* wg_begin,
                     int* grid);
hipError_t launch_score_fused_joint(int dtype, int D, int count, const void* const* q, const void* const* k,
                                    const ScoreGeom* G, const FusedGeom* F, const FusedSync* S, float* const* vote,
                                    const int* wg_begin, int grid, hipStream_t st);
hipError_t launch_score_fused(int dtype, int D, const void* q, const void* k, const ScoreGeom& G,
                              const FusedGeom& F, const FusedSync& S, float* vote, hipStream_t st);
// The same launch over the heads of SL.count layers (two-byte element types, F.BH == 1); returns
// hipErrorCooperativeLaunchTooLarge when this form of the kernel cannot keep the plan's grid resident.
hipError_t launch_score_fused_layers(int dtype, int D, const ScoreLayers& SL, const ScoreGeom& G, const FusedGeom& F,
                                     const FusedSync& S, float* vote, hipStream_t st, bool probe_only = false);
unsigned read_sync_timeouts();
bool reset_sync_timeouts();     // (test hook) both synchronise the device
bool reset_select_timeouts();
hipError_t launch_pool(const ScoreGeom& G, const float* vote, int pool_kind, int p, float* score,
                       unsigned* minmax, hipStream_t st);
size_t select_counter_bytes(int H);
size_t select_layout(int H, int64_t n, SelectScratch* S, void* base, bool own_counters = true,
                     void* counters = nullptr);
bool select_chunked_ok(int64_t n);   // rows of up to 4096 x 4096 positions
hipError_t launch_select_init(const SelectScratch& S, int H, hipStream_t st);
// flag (may be null): the status word of the call's scratch, cleared too (default: S->ps_flag).
hipError_t launch_prepare(void* pairs, int64_t npairs, const SelectScratch* S, int H, hipStream_t st,
                          unsigned* flag = nullptr);
int64_t fused_sync_pairs(const FusedGeom& F);
// allow_blocks: as for fused_plan, taken only where a window has more rows than the plain form tracks
bool lse_plan(int dtype, int D, const ScoreGeom& G, FusedGeom* F, bool allow_blocks = false);
// layers (may be null; two-byte element types): the heads are those of separately allocated layers, q and k unused
hipError_t launch_score_lse(int dtype, int D, const void* q, const void* k, const float* lse,
                            const ScoreGeom& G, const FusedGeom& F, float* vote, hipStream_t st,
                            const ScoreLayers* layers = nullptr);
size_t stream_stat_bytes(const ScoreGeom& G);
// lse_out == nullptr: the per-slice statistics only.  logit_out (may be null; plans with one row unit only):
// the pass also stores its masked logits there, [units][long_logit_keys(F)][16] floats (rows beyond the window
// hold what the padding produced and are ignored by the reader).
hipError_t launch_row_lse(int dtype, int D, const void* q, const void* k, const ScoreGeom& G,
                          const FusedGeom& F, float2* stat_part, float* lse_out, hipStream_t st,
                          float* logit_out = nullptr, const ScoreLayers* layers = nullptr);
int64_t long_logit_keys(const FusedGeom& F);
// Bytes that hold the logits of the rest of any long prompt of this shape on the current device (0: shapes whose
// logits are not kept: it is then cheaper, or as cheap, to read the rest's keys again).
size_t long_logit_bytes(const ScoreGeom& G);
// Votes of the rest from its kept logits and the rows' log-sum-exp (in place of the second streaming pass).
hipError_t launch_votes_from_logits(const float* logit, const float* lse, float* vote, const LongPlan& P,
                                    hipStream_t st);
// Pooling and selection in one cooperative launch (reads votes, writes the kept positions).
// pool_select_ok says whether the shape fits and the grid can be resident on the current device.
bool pool_select_ok(const ScoreGeom& G, int pool_kind, int p, int64_t kcount);
// nvalid (may be null): per head the number of valid positions, at most G.n, which is then only the
// pitch of the vote rows and of the candidate lists.
hipError_t launch_pool_select(const ScoreGeom& G, const float* vote, int pool_kind, int p, int64_t kcount,
                              int64_t out_stride, int W_tail, int32_t* out_idx, const SelectScratch& S,
                              hipStream_t st, const int32_t* nvalid = nullptr);
unsigned read_select_timeouts();

// Hit rate of the voting (snapkv_hitrate.hip).
size_t hit_rate_scratch_bytes(int Hq, int64_t Lk);
hipError_t launch_hit_rate(int dtype, int D, const void* q, const void* k, int64_t Lk, int64_t n, int Hq, int Hkv,
                           const int32_t* idx, int Hidx, int64_t kcount, int64_t idx_stride, float theta,
                           void* scratch, int32_t* counts, hipStream_t st);

// One decoding step of attention over a cache of [B, Hkv, cap, D] rows (snapkv_decode.hip).
int decode_splits(int B, int Hkv, int64_t S);
size_t decode_scratch_bytes(int B, int Hq, int D, int nsplit);
hipError_t launch_decode(int dtype, int D, const void* q, const void* k, const void* v, const int32_t* lens,
                         int B, int Hq, int Hkv, int64_t S, int64_t cap, int nsplit, void* scratch,
                         float* out, float* lse, hipStream_t st);
hipError_t launch_select_chunked(const float* score, int H, int64_t n, int64_t kcount,
                                 int64_t out_stride, int W_tail, int32_t* out_idx,
                                 const SelectScratch& S, int minmax_parts, hipStream_t st);
int pool_tiles(int64_t n);
hipError_t launch_iota(int H, int64_t rows, int64_t out_stride, int32_t* out_idx, hipStream_t st);
// Scratch a call's last kernel puts back into the state the next call expects (hand-off words
// all-ones, counters zero); all-null = nothing to do.
struct CleanJob {
    unsigned long long* ones = nullptr;
    int64_t nones = 0;
    unsigned* zeros = nullptr;
    int64_t nzeros = 0;
    // The call's verdict: if *flag is set (a bounded wait gave up in one of the call's kernels) the
    // last kernel writes SNAPKV_ERR_TIMEOUT to *status (device memory of the caller's, may be null) and 1
    // to *sticky (pinned host memory of the library's, may be null), otherwise `rows` to *status; then it
    // clears *flag.  flag == nullptr: nothing of this.
    unsigned* flag = nullptr;
    int32_t* status = nullptr;
    unsigned* sticky = nullptr;
    int32_t rows = 0;
};
constexpr int32_t kStatusTimeout = -6;   // SNAPKV_ERR_TIMEOUT
// Polls a bounded wait makes before it gives up: `dflt`, unless a test has set another bound
// (snapkv_debug_set_wait_limit).
unsigned wait_limit(unsigned dflt);
// Byte strides of a [heads, rows, D] tensor whose rows are contiguous.  launch_gather writes H
// output heads; output head h reads source head h / head_div.
struct RowLayout {
    int64_t head_stride, row_stride;
};
// Paging of K and V (one table for both); table == nullptr: rows are not paged.
struct PageMap {
    const int32_t* table = nullptr;
    int page = 1;
    int64_t pages = 0;
};
// A batch of prompts of one model (same heads, window and capacity, different lengths) whose
// selection and gather run as one launch each.  Passed by value to the kernels.
constexpr int kMaxBatch = 32;
struct BatchDesc {
    int count, Hkv;
    int64_t L[kMaxBatch], n[kMaxBatch];
    const void* k[kMaxBatch];
    const void* v[kMaxBatch];
    void* out_k[kMaxBatch];
    void* out_v[kMaxBatch];
    int32_t* out_idx[kMaxBatch];
};
hipError_t launch_batch_lengths(const BatchDesc& B, int32_t* nvalid, hipStream_t st);
hipError_t launch_gather_batch(const BatchDesc& B, const int32_t* idx, int64_t C, int row_bytes,
                               const CleanJob& clean, hipStream_t st);

hipError_t launch_gather(const void* k, const void* v, const int32_t* idx, int H, int64_t L,
                         int64_t rows, int64_t out_stride, int row_bytes, void* out_k, void* out_v,
                         const RowLayout& kl, const RowLayout& vl, const CleanJob& clean, hipStream_t st,
                         int head_div = 1, const PageMap& pm = PageMap{});
// The gather over the heads of GL.count separately allocated layers (contiguous rows, not paged): positions come
// from idx [GL.count * GL.heads, out_stride] and are copied to the layers' own out_idx as well.
hipError_t launch_gather_layers(const GatherLayers& GL, const int32_t* idx, int64_t L, int64_t rows, int64_t out_stride,
                                int row_bytes, const CleanJob& clean, hipStream_t st);

}  // namespace snapkv
#endif
