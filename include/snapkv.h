/*
 * snapkv.h - C ABI of the MI355X (gfx950) SnapKV prompt-KV compression library.
 *
 * The operation is the one defined in Sec. 4.1 / Listing 1 and Eq. 1-2 of "SnapKV: LLM Knows
 * What You are Looking for Before Generation" (arXiv 2404.14469): for every attention head,
 * score all prompt keys against the last W prompt queries (the observation window) with a
 * causal row softmax, sum the probabilities over the window (voting, Eq. 1), pool the votes
 * along the sequence (Sec. 4.3), keep the top C-W prefix positions per head (Eq. 2) and store
 * their K/V rows followed by the W window rows.
 *
 * Conventions fixed by this library where the paper is silent:
 *   - logits are scaled by 1/sqrt(D); window query i sits at position (L-W)+i and cannot see
 *     later keys (prompt-phase causal mask); the softmax runs over all visible keys.
 *   - pooling is stride 1 with padding p/2: max ignores the padding, average counts it as
 *     zeros and always divides by p.  p must be odd; p = 1 means no pooling.
 *   - grouped-query attention: votes are pooled per query head, then summed over the
 *     g = Hq/Hkv query heads that share a KV head; selection is per KV head.
 *   - ties in the top-(C-W) go to the lower position; kept positions are emitted ascending.
 *   - prompts with L <= C are returned unchanged (Listing 1, first branch).
 *
 * All pointers named "device" are GPU global memory owned by the caller, row-major and
 * contiguous, 16-byte aligned.  Inputs are read-only and must not alias outputs.  Calls only
 * enqueue work on `stream` (a hipStream_t passed as void*, NULL = the default stream); outputs are
 * valid once the stream reaches the end of the enqueued work.  They do not synchronise, with one
 * exception: an entry that uses a scratch buffer of the library's and finds it too small frees it and
 * allocates a larger one, and hipFree waits for the device (the first calls of a process, or the first
 * call of a larger shape; snapkv_compress_ws, snapkv_compress_ws_status and snapkv_compress_static never
 * do).  snapkv_sync_timeouts, snapkv_profile_stop, snapkv_release and the test hook say so themselves.
 * Every entry point validates its arguments on the host before touching the GPU and returns
 * a negative SNAPKV_ERR_* code on failure; nothing has been enqueued in that case unless the
 * code is SNAPKV_ERR_HIP.
 */
#ifndef SNAPKV_H_
#define SNAPKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SNAPKV_POOL_MAX 0
#define SNAPKV_POOL_AVG 1

#define SNAPKV_DTYPE_BF16 0 /* bfloat16 q/k/v */
#define SNAPKV_DTYPE_F32 1  /* IEEE float32 q/k/v */
#define SNAPKV_DTYPE_F16 2  /* IEEE float16 q/k/v */

#define SNAPKV_OK 0
#define SNAPKV_ERR_INVALID_ARG (-1) /* null pointer, L<1, W<1, W>L, W>C, even p, bad pool_kind, Hq%Hkv!=0 */
#define SNAPKV_ERR_UNSUPPORTED (-2) /* D not in {64,128}, p>129, L-W>2^24, a window length the kernels do not take */
#define SNAPKV_ERR_MISALIGNED (-3)  /* a q/k/v/out_k/out_v pointer is not 16-byte aligned */
#define SNAPKV_ERR_WORKSPACE (-4)   /* workspace missing or smaller than snapkv_workspace_bytes() */
#define SNAPKV_ERR_HIP (-5)         /* a HIP call (allocation or launch) failed */
#define SNAPKV_ERR_TIMEOUT (-6)     /* a bounded wait inside a kernel gave up: the results of that call are invalid */

/* Library version: major*10000 + minor*100 + patch. */
int snapkv_version(void);

/* Static, human-readable text for a SNAPKV_ERR_* code (never NULL). */
const char* snapkv_strerror(int code);

/*
 * The whole compression step for one prompt and one layer (Listing 1; Eq. 1-2), bf16 storage.
 *
 *   q_win   [Hq, W, D]   device, bf16: the last W prompt queries of every query head
 *   k, v    [Hkv, L, D]  device, bf16: all prompt keys / values
 *   L       prompt length (L - W <= 2^24); Hq, Hkv head counts (Hq % Hkv == 0); D in {64, 128}; W window length:
 *           1..128 rows, or more in whole blocks of 32 rows (160, 192, ...; such a window is scored block by
 *           block); other lengths return SNAPKV_ERR_UNSUPPORTED (the paper's settings are 16, 32 and 64)
 *   pool_kind SNAPKV_POOL_MAX or SNAPKV_POOL_AVG; p odd pooling width (1..129); C capacity (>= W)
 *   out_k, out_v [Hkv, C, D] device, bf16: kept rows, prefix rows in ascending position order
 *                            followed by the W window rows
 *   out_idx [Hkv, C]     device, int32: the kept positions; the last W are L-W .. L-1
 *
 * Returns the number of rows kept per head, min(C, L).  When L <= C the prompt is copied
 * unchanged into the first L rows of each head of out_k/out_v/out_idx and rows [L, C) are not
 * written.  Scratch memory comes from a per-device buffer the library allocates on first use
 * and grows when a larger problem arrives (hipMalloc; see snapkv_compress_ws for a variant that
 * never allocates); concurrent calls on different streams of one device would share it and race.
 * Calls that use this buffer (this entry and every entry below that says so) must come from one host
 * thread at a time and be ordered by the stream(s) they are enqueued on; on a stream that is being
 * captured into a graph they return SNAPKV_ERR_UNSUPPORTED (the library keeps a host-side record of the
 * state the buffer is left in, which a replay would bypass): capture snapkv_compress_ws or
 * snapkv_compress_static instead.
 */
int64_t snapkv_compress(const void* q_win, const void* k, const void* v, int64_t L, int Hq, int Hkv,
                        int D, int W, int pool_kind, int p, int64_t C, void* out_k, void* out_v,
                        int32_t* out_idx, void* stream);

/* Same operation with float32 q/k/v and float32 out_k/out_v. */
int64_t snapkv_compress_f32(const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                            int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k,
                            void* out_v, int32_t* out_idx, void* stream);

/* Same operation with IEEE float16 q/k/v and float16 out_k/out_v (fp32 accumulation and softmax). */
int64_t snapkv_compress_f16(const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                            int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k,
                            void* out_v, int32_t* out_idx, void* stream);

/*
 * Steps 1-3 only (window scores, voting per Eq. 1, pooling per Sec. 4.3, group sum):
 *   out_scores [Hkv, L-W] device, float32: the pooled score of every prefix position.
 * These are bit-for-bit the scores snapkv_compress selects from.  Returns SNAPKV_OK or <0.
 */
int snapkv_pooled_scores(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D, int W,
                         int pool_kind, int p, float* out_scores, void* stream);
int snapkv_pooled_scores_f32(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D,
                             int W, int pool_kind, int p, float* out_scores, void* stream);
int snapkv_pooled_scores_f16(const void* q_win, const void* k, int64_t L, int Hq, int Hkv, int D,
                             int W, int pool_kind, int p, float* out_scores, void* stream);

/*
 * Bytes of device scratch one call with these shapes needs (0 if the shapes are invalid).
 * The size does not depend on dtype, pooling or C; for prompts longer than the single-read scoring kernel
 * holds it includes room for the window logits of the keys that kernel does not take (windows of at most
 * 16 rows with Hq == Hkv), which depends on the compute units of the CURRENT device: ask on the device
 * the call will run on.
 */
size_t snapkv_workspace_bytes(int64_t L, int Hq, int Hkv, int D, int W);

/*
 * snapkv_compress / snapkv_compress_f32 with caller-provided scratch: `dtype` is
 * SNAPKV_DTYPE_*, `workspace` is device memory, 256-byte aligned, of at least
 * snapkv_workspace_bytes(L, Hq, Hkv, D, W) bytes, owned by the caller and free to reuse once
 * the enqueued work has finished.  The library keeps no pointer to it after the stream has
 * drained.  Calls that use distinct workspaces may run concurrently on different streams.
 */
int64_t snapkv_compress_ws(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                           int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                           void* out_k, void* out_v, int32_t* out_idx, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * snapkv_compress_ws that also leaves the call's verdict in device memory.  The single-read scoring
 * kernel and the cooperative pooling + selection kernel hand data between workgroups that must all be
 * resident at the same time; the host checks that the device CAN keep them resident, but cannot know
 * what else occupies it, so every such wait is bounded, and a wait that gives up leaves the call's
 * outputs invalid (memory-safe, but not the kept rows).  Once the stream has reached the end of the call,
 *   *status = rows kept per head (min(C, L)), or SNAPKV_ERR_TIMEOUT if a wait gave up in this call.
 *   status  device int32 of the caller's (4-byte aligned), written by the call's last kernel
 * The caller reads it where it synchronises anyway; the library never synchronises for it.  The other
 * arguments and the return value are those of snapkv_compress_ws.
 *
 * The entries that use the library's own scratch (snapkv_compress and its variants) report the same
 * condition one call late: the device records it in pinned host memory when it happens, and the next
 * such call on that device that finds the record returns SNAPKV_ERR_TIMEOUT (once) instead of enqueuing
 * anything: a call before it, already returned, produced invalid results.  They must be used from one
 * stream at a time per device (calls on different streams are not ordered against each other and share
 * the scratch) and not from several host threads at once.
 */
int64_t snapkv_compress_ws_status(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                                  int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                                  void* out_k, void* out_v, int32_t* out_idx, void* workspace,
                                  size_t workspace_bytes, int32_t* status, void* stream);

/*
 * snapkv_compress_ws for callers that cannot allocate and have no workspace to hand in: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch is a fixed array of
 * SNAPKV_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library runs on holds it
 * until the process ends); the call allocates nothing and frees nothing.  Shapes whose
 * snapkv_workspace_bytes(L, Hq, Hkv, D, W) exceeds SNAPKV_STATIC_SCRATCH_BYTES are refused with
 * SNAPKV_ERR_WORKSPACE before anything is enqueued (32 heads x 16384 tokens and 32/8 heads x 32768 tokens
 * fit; 32 heads x 131072 tokens do not).  Arguments, outputs and results are those of snapkv_compress_ws.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents (the call's first kernel
 * clears what must start at zero): calls that overlap on one GPU, on whatever streams, race.
 */
#define SNAPKV_STATIC_SCRATCH_BYTES (32u << 20)
int64_t snapkv_compress_static(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                               int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                               void* out_k, void* out_v, int32_t* out_idx, void* stream);

/*
 * The same step when the softmax normalisers of the window rows are already known (an attention
 * prefill that works block by block keeps, for every query row, the log of its softmax
 * denominator; Sec. 4.1 runs the compression at the end of prompt encoding, so they exist).
 *
 *   lse [Hq, W] device, float32: natural-log-sum-exp of window row i of query head h over the keys
 *   it may see, lse[h][i] = log sum_{j <= L-W+i} exp(q_win[h][i] . k[kv(h)][j] / sqrt(D)).
 *
 * Probabilities are then exp(logit - lse) (Sec. 4; Eq. 1 sums them unchanged), so K is streamed once
 * with no exchange between workgroups.  All other arguments, the outputs and the return values are
 * those of snapkv_compress / snapkv_pooled_scores; `dtype` is SNAPKV_DTYPE_*.  An lse that is not
 * the rows' own scales row i of the probabilities by exp(true - given); the library does not check
 * it.  SNAPKV_ERR_UNSUPPORTED if the window rows of a query head exceed what a wave tracks
 * (W > 128).  Scratch comes from the library's per-device buffer, as for snapkv_compress.
 */
int64_t snapkv_compress_lse(int dtype, const void* q_win, const void* k, const void* v, const float* lse,
                            int64_t L, int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                            void* out_k, void* out_v, int32_t* out_idx, void* stream);
int snapkv_pooled_scores_lse(int dtype, const void* q_win, const void* k, const float* lse, int64_t L,
                             int Hq, int Hkv, int D, int W, int pool_kind, int p, float* out_scores,
                             void* stream);

/*
 * snapkv_compress / snapkv_compress_f32 for K and V that are not laid out [Hkv, L, D] contiguously,
 * e.g. the token-major [L, Hkv, D] caches of attention libraries (Listing 1 indexes the tensors by
 * (head, position), whatever their storage order).  Row r of KV head h of k starts
 * k_head_stride * h + k_row_stride * r ELEMENTS after `k` (likewise v); the D elements of a row are
 * contiguous.  Strides must keep every row 16-byte aligned (multiples of 8 bf16 / 4 float32 elements),
 * k_row_stride and v_row_stride are at least D, and distinct (head, row) pairs must not overlap.
 * q_win, out_k, out_v and out_idx are contiguous as for snapkv_compress; `dtype` is SNAPKV_DTYPE_*.
 * Scratch comes from the library's per-device buffer.
 */
int64_t snapkv_compress_strided(int dtype, const void* q_win, const void* k, const void* v, int64_t L, int Hq,
                                int Hkv, int D, int W, int64_t k_head_stride, int64_t k_row_stride,
                                int64_t v_head_stride, int64_t v_row_stride, int pool_kind, int p, int64_t C,
                                void* out_k, void* out_v, int32_t* out_idx, void* stream);

/*
 * The compression step for a batch of prompts of one model (same heads, window, pooling and capacity,
 * different lengths), e.g. the prompts of one serving step.  Every prompt gets exactly the result of its
 * own snapkv_compress call; the batch only saves launches and idle compute units: prompts share scoring
 * launches as far as they fit the chip together, and pooling with selection and the gather run once for
 * up to 32 prompts.
 *
 *   n_prompts >= 0
 *   q_win, k, v, out_k, out_v, out_idx   HOST arrays of n_prompts DEVICE pointers, each as the argument of
 *           the same name of snapkv_compress for that prompt (k[i], v[i] are [Hkv, L[i], D], ...)
 *   L       HOST array of n_prompts prompt lengths
 *   kept    HOST array of n_prompts, or NULL: rows kept per head of each prompt, min(C, L[i])
 *   dtype   SNAPKV_DTYPE_*; the other arguments as for snapkv_compress
 *
 * The host arrays are read before the call returns.  All prompts are validated before anything is enqueued;
 * returns SNAPKV_OK or a negative SNAPKV_ERR_* code.  Shapes the joint kernels do not take (windows of more
 * than 128 rows per query head, a batch that is not resident at once) run prompt by prompt inside the call.
 * Scratch comes from the library's per-device buffer.
 */
int snapkv_compress_varlen(int dtype, int n_prompts, const void* const* q_win, const void* const* k,
                           const void* const* v, const int64_t* L, int Hq, int Hkv, int D, int W, int pool_kind,
                           int p, int64_t C, void* const* out_k, void* const* out_v, int32_t* const* out_idx,
                           int64_t* kept, void* stream);

/*
 * The compression step for several layers of one prompt in one call (Listing 1 runs once per layer; the
 * layers of a prompt have the same shape and are independent of each other, Sec. 4.1).  Every layer gets
 * exactly the result of its own snapkv_compress call.  What the call saves: the layers go through the
 * kernels as ONE layer with that many more heads, so the scoring kernel streams all their keys in a single
 * launch and pays its start-up and drain once, and pooling, selection and gather run as a few large launches
 * instead of three per layer.  With the whole uncompressed prompt cache resident (68.7 GB at 32 layers x
 * 32 heads x 131072 tokens: this is what 288 GB of HBM are for) that is the fastest form of the step.
 * Layers whose tensors lie one directly behind the other in memory (slices of stacked [layers, heads, ...]
 * tensors, for q_win, k, v, out_k, out_v and out_idx alike) are taken as they lie; layers that are separate
 * allocations are reached through a table of their addresses, up to 32 of them per run of launches (two-byte
 * element types; every prompt length; windows that a single call would not score in 32-row blocks, i.e. of
 * at most 32 rows, or of 33-128 rows that are not a whole number of such blocks).  What fits neither is done
 * one layer after the other inside the call.
 *
 *   n_layers >= 0
 *   q_win, k, v, out_k, out_v, out_idx   HOST arrays of n_layers DEVICE pointers, each as the argument of the
 *           same name of snapkv_compress for that layer
 *   dtype   SNAPKV_DTYPE_*; the other arguments as for snapkv_compress
 *
 * The host arrays are read before the call returns.  All layers are validated before anything is enqueued;
 * returns SNAPKV_OK or a negative SNAPKV_ERR_* code.  Scratch comes from the library's per-device buffer
 * and grows with the number of layers that run together (at most 6 GiB; longer runs are cut).
 */
int snapkv_compress_layers(int dtype, int n_layers, const void* const* q_win, const void* const* k,
                           const void* const* v, int64_t L, int Hq, int Hkv, int D, int W, int pool_kind, int p,
                           int64_t C, void* const* out_k, void* const* out_v, int32_t* const* out_idx, void* stream);

/*
 * The compression step on a paged cache (Listing 1 indexes K and V by (head, position), whatever their
 * storage): k_pages and v_pages are [num_pages, page_size, Hkv, D] (the rows of a page are token-major)
 * and logical position j of every head lives in physical page block_table[j / page_size], row
 * j % page_size.  One table serves K and V.
 *
 *   block_table  [ceil(L / page_size)] device int32, entries in [0, num_pages) (entries outside are
 *                clamped to that range, so a bad table gives wrong results, not a wild access)
 *   page_size >= 1 (16 or more for coalesced reads), ceil(L / page_size) <= num_pages
 * Other arguments, outputs (contiguous out_k/out_v [Hkv, C, D], out_idx [Hkv, C] in logical positions)
 * and the return value as for snapkv_compress; `dtype` is SNAPKV_DTYPE_*.  Scratch comes from the
 * library's per-device buffer.
 */
int64_t snapkv_compress_paged(int dtype, const void* q_win, const void* k_pages, const void* v_pages,
                              const int32_t* block_table, int64_t num_pages, int page_size, int64_t L, int Hq,
                              int Hkv, int D, int W, int pool_kind, int p, int64_t C, void* out_k, void* out_v,
                              int32_t* out_idx, void* stream);

/*
 * The compression step with one cache per QUERY head (Listing 1 as printed has equal head counts;
 * a grouped-query model reaches them by repeating every KV head for the g = Hq / Hkv query heads that
 * read it).  Query head h scores the keys of KV head h / g, and votes, pools and selects alone (no
 * sum over the group); its kept rows are gathered from that KV head.  Arguments as for
 * snapkv_compress except:
 *   dtype   SNAPKV_DTYPE_*
 *   out_k, out_v [Hq, C, D] device, dtype;   out_idx [Hq, C] device int32
 * With Hq == Hkv the result equals snapkv_compress.  SNAPKV_ERR_UNSUPPORTED for windows of more than
 * 128 rows per query head.  Scratch comes from the library's per-device buffer.
 */
int64_t snapkv_compress_per_query_head(int dtype, const void* q_win, const void* k, const void* v, int64_t L,
                                       int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C,
                                       void* out_k, void* out_v, int32_t* out_idx, void* stream);

/*
 * Capacity for the rate form of the selection size (Sec. 4, "Voting": k = floor(rate * L_prefix) prefix
 * positions are kept, L_prefix = L - W): returns C = W + floor(rate * (L - W)), the value to pass as `C`
 * to the compress entry points.  The product is taken in IEEE double.  Host-only arithmetic; returns
 * SNAPKV_ERR_INVALID_ARG unless 0 <= rate <= 1 and 1 <= W <= L.
 */
int64_t snapkv_capacity_for_rate(int64_t L, int W, double rate);

/*
 * Hit rate of the voting (Sec. 4, "Hit Rate", Eq. 3-7), as counts: a quality probe.  A_cur is the
 * softmax-normalised attention of the query of a token being generated over all Lk keys it sees, cut to
 * the n prefix positions; a position is important when A_cur > theta; a hit is an important position
 * that the voting selected.  The hit rate is H = sum(hits) / sum(important).
 *
 *   dtype   SNAPKV_DTYPE_BF16 or SNAPKV_DTYPE_F16 (float32 storage: SNAPKV_ERR_UNSUPPORTED)
 *   q_cur   [Hq, D] device, dtype;  k [Hkv, Lk, D] device, dtype (query head h reads KV head h / g, g <= 16)
 *   n       0 <= n <= Lk prefix positions
 *   idx     [Hidx, idx_stride] device int32: the first kcount entries of a row are the selected prefix
 *           positions in ascending order (the out_idx of a compress call with kcount = C - W and
 *           idx_stride = C).  Hidx divides Hq: Hkv rows for snapkv_compress (query head h is checked
 *           against row h / g), Hq rows for snapkv_compress_per_query_head.
 *   out_counts [Hq, 2] device int32: per query head (important, hits); overwritten.
 *
 * The logits of the call live in the per-device auxiliary buffer the decoding step also uses (hipMalloc
 * on first use and on growth; concurrent calls on one device would race).
 */
int snapkv_hit_rate(int dtype, const void* q_cur, const void* k, int64_t Lk, int64_t n, int Hq, int Hkv, int D,
                    const int32_t* idx, int Hidx, int64_t kcount, int64_t idx_stride, float theta,
                    int32_t* out_counts, void* stream);

/*
 * One decoding step of attention over the compacted cache (Sec. 5.1.2: after compression a
 * generated token attends to the C kept rows plus the rows appended since, so the cost of a step no
 * longer grows with the prompt).  For every sequence b and query head h (reading KV head h / g):
 *     out[b, h, :] = sum_j softmax_j(q[b, h] . k[b, h/g, j] / sqrt(D)) v[b, h/g, j],  j < S_b
 *     out_lse[b, h] = log sum_j exp(q[b, h] . k[b, h/g, j] / sqrt(D))     (natural logarithm)
 * The new token sees every valid row; the order of the rows does not matter.
 *
 *   dtype   SNAPKV_DTYPE_BF16 or SNAPKV_DTYPE_F16 (float32 storage: SNAPKV_ERR_UNSUPPORTED)
 *   q       [B, Hq, D]        device, dtype: the new token's queries
 *   k_cache, v_cache [B, Hkv, cap, D] device, dtype: row capacity `cap` per head, finite values
 *   lens    [B] device int32 valid rows per sequence, or NULL: every sequence has S rows.  Values
 *           are clamped to [0, cap]; a sequence with no rows gets out = 0 and out_lse = -inf.
 *   S       1 <= S <= cap: the valid rows when lens is NULL, otherwise a hint of the typical
 *           length (used only to choose how finely the keys are split over workgroups)
 *   Hq % Hkv == 0, Hq / Hkv <= 16, D in {64, 128}
 *   out     [B, Hq, D] device float32;  out_lse [B, Hq] device float32 or NULL
 *
 * Partial results of split key ranges live in a per-device buffer of their own that the library
 * allocates on first use and grows when needed (hipMalloc); concurrent calls on different streams
 * of one device would share it and race.  Returns SNAPKV_OK or a negative SNAPKV_ERR_* code.
 */
int snapkv_decode_attention(int dtype, const void* q, const void* k_cache, const void* v_cache,
                            const int32_t* lens, int B, int Hq, int Hkv, int D, int64_t S, int64_t cap,
                            float* out, float* out_lse, void* stream);

/*
 * Top-(kcount) selection alone (Eq. 2), exposed for testing the selector on arbitrary scores:
 *   scores [H, n] device float32, all values >= +0 (their bit patterns are compared as unsigned
 *   integers); out_idx [H, kcount] device int32: the kcount best positions per row under
 *   (score descending, position ascending), emitted ascending.  0 <= kcount <= n <= 2^24.
 */
int snapkv_select_topk(const float* scores, int H, int64_t n, int64_t kcount, int32_t* out_idx,
                       void* stream);

/*
 * Per-stage timing for benchmarks (not part of the method).  Between snapkv_profile_start and
 * snapkv_profile_stop every compressing call (L > C) records a HIP event on its stream after
 * each kernel of the path, for at most max_calls (1..4096) calls.  snapkv_profile_stop waits for
 * the device, writes the mean duration in milliseconds of each stage over the recorded calls to
 * stage_ms[0 .. snapkv_num_stages()) (host memory, may be NULL) and the number of calls averaged
 * to *calls (host, may be NULL).  A stage is one kernel (the selection stage: its few kernels);
 * snapkv_stage_name(i) names it, and a stage the calls did not run reports 0.
 * Not thread-safe; one profiling session at a time.
 */
int snapkv_profile_start(int max_calls);
int snapkv_profile_stop(double* stage_ms, int* calls);
int snapkv_num_stages(void);
const char* snapkv_stage_name(int stage);

/*
 * Kernel scheme, a bit set (default 0).  Bit 0 clear: prompts whose window logits fit the chip's
 * register files are scored by the single-read kernel (K is streamed once); of a longer prompt that
 * kernel takes the keys that fit and two streaming passes the rest (those keys are streamed twice; the
 * streaming passes hand nothing between workgroups); bit 0 set: always two streaming passes over
 * all keys.  Bit 2 set (test hook): plans of the single-read kernel count 16 workgroups as resident, so
 * that prompts of a few thousand tokens already take the path of the long ones.  Bit 1 clear:
 * pooling and top-k selection run as one cooperative launch where a head's scores fit the
 * resident workgroups, otherwise as separate kernels; bit 1 set: always the separate kernels.
 * All schemes give the scores of Eq. 1 to within rounding, and the selection of Eq. 2 exactly
 * for the scores they computed; the setting is process-wide and meant for tests and measurements.
 */
int snapkv_set_scoring_scheme(int scheme);

/*
 * The single-read scoring kernel and the cooperative pooling + selection kernel hand data
 * between resident workgroups and bound every wait; a wait that gives up is counted here (0 in
 * correct operation; the results of such a call are invalid).  Synchronises the
 * device.  Returns the count since the library was loaded, or a negative SNAPKV_ERR_* code.
 */
int64_t snapkv_sync_timeouts(void);

/*
 * Test hook, not for production: bounds every wait inside the kernels to `polls` polls (0: every wait gives
 * up at once; negative: the kernels' own bounds, tens of milliseconds).  With a bound of 0 all kernels
 * still run to their end and stay inside their buffers, the results are invalid and the condition is
 * reported as described at snapkv_compress_ws_status.  Process-wide.  -2 also sets the count of
 * snapkv_sync_timeouts back to zero (and synchronises the device for it).
 */
int snapkv_debug_set_wait_limit(long long polls);

/* Frees the library's per-device scratch buffers (synchronises each device that has one). */
void snapkv_release(void);

#ifdef __cplusplus
}
#endif
#endif /* SNAPKV_H_ */
