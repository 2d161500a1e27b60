// Geometry of a scoring call and the layout of its workspace (shared by the host dispatcher and the kernel
// translation units).
#include "snapkv_internal.h"

namespace snapkv {

ScoreGeom make_geom(int64_t L, int Hq, int Hkv, int D, int W) {
    ScoreGeom G;
    G.L = L;
    G.n = L - W;
    G.W = W;
    G.g = Hq / Hkv;
    G.Hkv = Hkv;
    G.BH = (W + 31) / 32;
    G.VB = 1;          // the scoring launch says how many vote rows it left per query head
    G.NV = G.g;
    G.c2 = (float)(1.4426950408889634 / __builtin_sqrt((double)D));
    G.k_rs = 0;   // set by the caller once the element size is known
    G.k_hs = 0;
    G.vpitch = G.n;
    G.k_table = nullptr;
    G.k_page = 1;
    G.k_pages = 0;
    G.k_row0 = 0;
    return G;
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// The two regions whose contents carry over between calls come first, at offsets that depend on
// the number of KV heads only: pool_select's counters (zero when idle), then the hand-off words of
// the single-read scoring kernel (all-ones when idle).  The selection's scratch and the scores are
// sized for one selection per query head, which the per-query-head form of the step runs.
size_t workspace_layout(const ScoreGeom& G, Workspace* ws, void* base) {
    constexpr size_t kHeader = 256;      // the status word (see Workspace::status_flag)
    char* b = static_cast<char*>(base) + (base ? kHeader : 0);
    const int Hsel = G.Hkv * G.g;
    const size_t counters = select_counter_bytes(Hsel);
    const size_t fused = fused_sync_bytes(G);
    // one vote row per query head, or per 32-row block of a window of 64, 96, ... rows
    const size_t vote = align_up(sizeof(float) * (size_t)G.Hkv * G.g * G.BH * (size_t)(G.n > 0 ? G.n : 1));
    const size_t score = align_up(sizeof(float) * (size_t)Hsel * (size_t)(G.n > 0 ? G.n : 1));
    const size_t stat = stream_stat_bytes(G);
    const size_t lse = align_up(sizeof(float) * (size_t)G.Hkv * G.g * G.W);
    const size_t logit = long_logit_bytes(G);
    const size_t off = counters + fused;
    if (ws) {
        ws->status_flag = reinterpret_cast<unsigned*>(base);
        ws->fused = b + counters;
        ws->vote = reinterpret_cast<float*>(b + off);
        ws->score = reinterpret_cast<float*>(b + off + vote);
        ws->stat_part = reinterpret_cast<float2*>(b + off + vote + score);
        ws->lse = reinterpret_cast<float*>(b + off + vote + score + stat);
        ws->long_logit = logit ? reinterpret_cast<float*>(b + off + vote + score + stat + lse) : nullptr;
        ws->long_logit_bytes = logit;
    }
    const size_t sel = select_layout(Hsel, G.n, ws ? &ws->sel : nullptr,
                                     ws ? b + off + vote + score + stat + lse + logit : nullptr, false,
                                     ws ? b : nullptr);
    if (ws) ws->sel.ps_flag = ws->status_flag;
    return kHeader + off + vote + score + stat + lse + logit + sel;
}

}  // namespace snapkv
