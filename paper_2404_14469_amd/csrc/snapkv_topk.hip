// Per-head top-k selection (Eq. 2; Listing 1, the topk call) spread over the whole chip.
//
// Scores are >= +0, so their fp32 bit patterns order like unsigned integers.  Per head the bit
// pattern T of the kcount-th largest score is found by an adaptive most-significant-digit-first
// search, then every position with pattern > T and the first (kcount - #greater) positions with
// pattern == T are emitted in position order: exactly the top-kcount under (score descending,
// position ascending), already sorted by position.  Integer arithmetic only; the result does
// not depend on the order in which workgroups run.
//
//   sel_hist      chunks of 4096 positions: histogram of (x - lo) >> sh over 512 bins, where
//                 [lo, hi] is the head's range of patterns and sh makes the range fit the bins
//                 (the digit adapts to the data, so a narrow score field still spreads out)
//   sel_compact   finds the bin b1 holding the kcount-th largest, counts per chunk the positions
//                 in higher bins and copies the few positions inside b1 to a candidate list
//   sel_threshold one workgroup per head: finishes the search on the candidates (11 bits per
//                 round), then turns per-chunk counts into per-chunk output offsets
//   sel_emit      chunks again: ordered emission by wavefront ballot / prefix counts
#include "snapkv_internal.h"

namespace snapkv {

constexpr int kSelChunk = 4096;        // positions per workgroup in the chunked kernels
constexpr int kSelBins1 = 512;         // first digit (whole row, global histogram): 9 bits
constexpr int kSelBins = 2048;         // later digits (candidates only, LDS histogram): 11 bits
constexpr int kSelMaxChunks = 4096;    // LDS arrays of sel_threshold; longer rows use one workgroup

__device__ __forceinline__ int range_shift(unsigned range) {
    // smallest shift with (range >> shift) < kSelBins1
    const int bits = 32 - __clz(range | 1u);
    return bits > 9 ? bits - 9 : 0;
}

// Exclusive prefix sum over the block (NT threads, NT a multiple of 64, at most 1024); returns
// the sum of the values of lower thread ids, *total gets the block total.  sh needs 16 words.
template <int NT>
__device__ __forceinline__ unsigned block_exclusive_scan(unsigned v, unsigned* sh, unsigned* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    __syncthreads();                      // sh may still be read from an earlier call
    if (lane == 63) sh[wave] = incl;
    __syncthreads();
    unsigned base = 0, tot = 0;
#pragma unroll
    for (int w2 = 0; w2 < NT / 64; ++w2) {
        const unsigned x = sh[w2];
        if (w2 < wave) base += x;
        tot += x;
    }
    if (total) *total = tot;
    return base + incl - v;
}

// Walking the bins of hist[0..NBINS) from the top, find the bin where the running count first
// reaches krem (1 <= krem <= total count).  out[0] = bin, out[1] = krem - count above the bin.
template <int NT, int NBINS>
__device__ __forceinline__ void load_bins_from_top(const unsigned* hist, unsigned (&c)[NBINS / NT]) {
#pragma unroll
    for (int e = 0; e < NBINS / NT; ++e) c[e] = hist[NBINS - 1 - (threadIdx.x * (NBINS / NT) + e)];
}

template <int NT, int NBINS>
__device__ __forceinline__ void find_bin_from_top(const unsigned (&c)[NBINS / NT], unsigned krem,
                                                  unsigned* sh, unsigned* out) {
    constexpr int BPT = NBINS / NT;
    const int tid = threadIdx.x;
    unsigned mine = 0;
#pragma unroll
    for (int e = 0; e < BPT; ++e) mine += c[e];
    unsigned above = block_exclusive_scan<NT>(mine, sh, nullptr);
#pragma unroll
    for (int e = 0; e < BPT; ++e) {
        if (above < krem && krem <= above + c[e]) {
            out[0] = (unsigned)(NBINS - 1 - (tid * BPT + e));
            out[1] = krem - above;
        }
        above += c[e];
    }
    __syncthreads();
}

// Range [lo, hi] of a head's score bit patterns from the per-part ranges its producer left
// (one pair per pooling tile or per chunk); every workgroup computes the same values.
__device__ __forceinline__ void head_range(const unsigned* mm, int nparts, unsigned* sh4,
                                           unsigned& lo, unsigned& hi) {
    lo = 0xFFFFFFFFu;
    hi = 0u;
    for (int i = threadIdx.x; i < nparts; i += blockDim.x) {
        const unsigned a = mm[2 * i], b = mm[2 * i + 1];
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned a = __shfl_xor(lo, d, 64), b = __shfl_xor(hi, d, 64);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        sh4[2 * wave] = lo;
        sh4[2 * wave + 1] = hi;
    }
    __syncthreads();
    for (int w2 = 0; w2 < nw; ++w2) {
        lo = sh4[2 * w2] < lo ? sh4[2 * w2] : lo;
        hi = sh4[2 * w2 + 1] > hi ? sh4[2 * w2 + 1] : hi;
    }
}

__global__ void sel_init(SelectScratch S, int H) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < H * kSelBins1) S.hist[i] = 0u;
    if (i < H) S.cand_count[i] = 0u;
}

// Range of bit patterns per head (when the scores were not produced by the pooling kernel).
__global__ __launch_bounds__(256) void sel_minmax(const float* __restrict__ score, int64_t n,
                                                  SelectScratch S) {
    __shared__ unsigned sh_lo[4], sh_hi[4];
    const int h = blockIdx.y;
    const unsigned* s = reinterpret_cast<const unsigned*>(score) + (int64_t)h * n;
    unsigned lo = 0xFFFFFFFFu, hi = 0u;
    const int64_t base = (int64_t)blockIdx.x * kSelChunk;
    for (int e = 0; e < kSelChunk / 256; ++e) {
        const int64_t j = base + e * 256 + threadIdx.x;
        if (j < n) {
            const unsigned x = s[j];
            lo = x < lo ? x : lo;
            hi = x > hi ? x : hi;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned a = __shfl_xor(lo, d, 64), b = __shfl_xor(hi, d, 64);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
    if ((threadIdx.x & 63) == 0) {
        sh_lo[threadIdx.x >> 6] = lo;
        sh_hi[threadIdx.x >> 6] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w) {
            lo = sh_lo[w] < lo ? sh_lo[w] : lo;
            hi = sh_hi[w] > hi ? sh_hi[w] : hi;
        }
        unsigned* mm = S.minmax + 2 * ((int64_t)h * gridDim.x + blockIdx.x);
        mm[0] = lo;
        mm[1] = hi;
    }
}

constexpr int kHistChunk = 16384;      // positions per workgroup of sel_hist (1024 threads)

__global__ __launch_bounds__(1024) void sel_hist(const float* __restrict__ score, int64_t n,
                                                 int nparts, SelectScratch S) {
    __shared__ unsigned hist[kSelBins1];
    __shared__ unsigned sh4[32];
    const int h = blockIdx.y, tid = threadIdx.x;
    const unsigned* s = reinterpret_cast<const unsigned*>(score) + (int64_t)h * n;
    const int64_t base = (int64_t)blockIdx.x * kHistChunk;
    unsigned x[kHistChunk / 1024];          // the chunk's scores are requested before anything else
#pragma unroll
    for (int e = 0; e < kHistChunk / 1024; ++e) {
        const int64_t j = base + e * 1024 + tid;
        x[e] = j < n ? s[j] : 0u;
    }
    for (int b = tid; b < kSelBins1; b += 1024) hist[b] = 0u;
    unsigned lo, hi;
    head_range(S.minmax + 2 * (int64_t)h * nparts, nparts, sh4, lo, hi);
    if (hi <= lo) return;                 // flat row: the threshold is known without a search
    const int sh = range_shift(hi - lo);
#pragma unroll
    for (int e = 0; e < kHistChunk / 1024; ++e) {
        const int64_t j = base + e * 1024 + tid;
        if (j < n) atomicAdd(&hist[(x[e] - lo) >> sh], 1u);
    }
    __syncthreads();
    for (int b = tid; b < kSelBins1; b += 1024) {
        const unsigned c = hist[b];
        if (c) atomicAdd(&S.hist[h * kSelBins1 + b], c);
    }
}

__global__ __launch_bounds__(256) void sel_compact(const float* __restrict__ score, int64_t n,
                                                   int64_t kcount, int nch, int nparts,
                                                   SelectScratch S) {
    __shared__ unsigned sh4[8];
    __shared__ unsigned sh_scan[16];
    __shared__ unsigned sh_out[2];
    __shared__ unsigned sh_cnt, sh_gt;
    const int h = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const unsigned* s = reinterpret_cast<const unsigned*>(score) + (int64_t)h * n;
    const int64_t base = (int64_t)c * kSelChunk;
    // everything this workgroup reads is requested up front: one round trip to memory
    unsigned xs[kSelChunk / 256];
#pragma unroll
    for (int e = 0; e < kSelChunk / 256; ++e) {
        const int64_t j = base + e * 256 + tid;
        xs[e] = j < n ? s[j] : 0u;
    }
    unsigned bins[kSelBins1 / 256];
    load_bins_from_top<256, kSelBins1>(S.hist + h * kSelBins1, bins);
    if (tid == 0) {
        sh_cnt = 0u;
        sh_gt = 0u;
    }
    unsigned lo, hi;
    head_range(S.minmax + 2 * (int64_t)h * nparts, nparts, sh4, lo, hi);
    if (hi <= lo) {                       // flat row: every position equals the threshold
        if (c == 0 && tid == 0) {
            S.info[4 * h + 0] = lo;
            S.info[4 * h + 1] = 0u;
            S.info[4 * h + 2] = (unsigned)kcount;
            S.info[4 * h + 3] = 1u;       // flat
        }
        if (tid == 0) {
            S.chunk_gt[(int64_t)h * nch + c] = 0u;
            S.cand_count[(int64_t)h * nch + c] = 0u;
        }
        return;
    }
    const int sh = range_shift(hi - lo);
    find_bin_from_top<256, kSelBins1>(bins, (unsigned)kcount, sh_scan, sh_out);
    const unsigned b1 = sh_out[0];
    if (c == 0 && tid == 0) {
        S.info[4 * h + 0] = lo + (b1 << sh);   // lowest pattern of the bin
        S.info[4 * h + 1] = (unsigned)sh;      // the bin spans 2^sh patterns
        S.info[4 * h + 2] = sh_out[1];         // rank wanted inside the bin (from its top)
        S.info[4 * h + 3] = 0u;
    }
    // positions inside the threshold bin go to this chunk's part of the candidate list
    uint2* dst = S.cand + (int64_t)h * n + base;
    unsigned gt = 0;
#pragma unroll
    for (int e = 0; e < kSelChunk / 256; ++e) {
        const int64_t j = base + e * 256 + tid;
        if (j < n) {
            const unsigned x = xs[e];
            const unsigned b = (x - lo) >> sh;
            gt += b > b1;
            if (b == b1) dst[atomicAdd(&sh_cnt, 1u)] = make_uint2(x, (unsigned)j);
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) gt += __shfl_xor(gt, d, 64);
    if ((tid & 63) == 0 && gt) atomicAdd(&sh_gt, gt);
    __syncthreads();
    if (tid == 0) {
        S.chunk_gt[(int64_t)h * nch + c] = sh_gt;
        S.cand_count[(int64_t)h * nch + c] = sh_cnt;
    }
}

constexpr int kSelLdsCand = 2048;      // candidates of a head kept in LDS by sel_threshold

__global__ __launch_bounds__(1024) void sel_threshold(int64_t n, int nch, SelectScratch S) {
    __shared__ unsigned hist[kSelBins];
    __shared__ unsigned sh_scan[16];
    __shared__ unsigned sh_out[2];
    __shared__ unsigned cgt[kSelMaxChunks], ceq[kSelMaxChunks];   // also: chunk starts in the flat list
    __shared__ uint2 lcand[kSelLdsCand];
    const int h = blockIdx.x, tid = threadIdx.x;
    constexpr int CPT = kSelMaxChunks / 1024;
    // requested up front: search state, per-chunk candidate counts and higher-bin counts
    unsigned cn[CPT], cg[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        const int c = tid * CPT + e;
        cn[e] = c < nch ? S.cand_count[(int64_t)h * nch + c] : 0u;
        cg[e] = c < nch ? S.chunk_gt[(int64_t)h * nch + c] : 0u;
    }
    unsigned cur_lo = S.info[4 * h + 0];
    int cur_sh = (int)S.info[4 * h + 1];
    unsigned krem = S.info[4 * h + 2];
    const bool flat = S.info[4 * h + 3] != 0u;

    // flatten the per-chunk lists: ceq[c] = index of chunk c's first candidate
    unsigned csum = 0;
#pragma unroll
    for (int e = 0; e < CPT; ++e) csum += cn[e];
    unsigned m = 0;
    unsigned start = block_exclusive_scan<1024>(csum, sh_scan, &m);
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        const int c = tid * CPT + e;
        if (c < nch) {
            ceq[c] = start;
            cgt[c] = cn[e];
        }
        start += cn[e];
    }
    __syncthreads();
    const bool in_lds = m <= (unsigned)kSelLdsCand;
    const uint2* gcand = S.cand + (int64_t)h * n;
    if (in_lds) {   // usual case: copy the candidates next to each other into LDS
        for (int v = tid; v < nch * 64; v += 1024) {
            const int c = v >> 6;
            const unsigned cnt = cgt[c], at = ceq[c];
            for (unsigned i = v & 63; i < cnt; i += 64) lcand[at + i] = gcand[(int64_t)c * kSelChunk + i];
        }
    }
    __syncthreads();
    // candidate i of the flat list (LDS copy, or looked up in its chunk's part of the global list)
    auto cand_at = [&](unsigned i) -> uint2 {
        if (in_lds) return lcand[i];
        int a = 0, b = nch - 1;               // last chunk whose start is <= i
        while (a < b) {
            const int mid = (a + b + 1) >> 1;
            if (ceq[mid] <= i) a = mid; else b = mid - 1;
        }
        return gcand[(int64_t)a * kSelChunk + (i - ceq[a])];
    };

    while (cur_sh > 0) {                  // 11 more bits of the threshold per round
        const int nsh = cur_sh > 11 ? cur_sh - 11 : 0;
        for (int b = tid; b < kSelBins; b += 1024) hist[b] = 0u;
        __syncthreads();
        for (unsigned i = tid; i < m; i += 1024) {
            const unsigned d = cand_at(i).x - cur_lo;       // wraps to a huge value if below range
            if ((d >> cur_sh) == 0u) atomicAdd(&hist[d >> nsh], 1u);
        }
        __syncthreads();
        unsigned bins[kSelBins / 1024];
        load_bins_from_top<1024, kSelBins>(hist, bins);
        find_bin_from_top<1024, kSelBins>(bins, krem, sh_scan, sh_out);
        cur_lo += sh_out[0] << nsh;
        krem = sh_out[1];
        cur_sh = nsh;
        __syncthreads();
    }
    const unsigned T = cur_lo, need_eq = krem;

    // per-chunk counts of candidates above / equal to T.  The chunk starts in ceq are no longer
    // needed once every candidate has been fetched, so fetch first, then reuse the array.
    uint2 mine[4];
    unsigned nmine = 0;
    bool overflow = false;
    for (unsigned i = tid; i < m; i += 1024) {
        if (nmine < 4) mine[nmine++] = cand_at(i); else overflow = true;
    }
    const bool any_overflow = __syncthreads_or(overflow);
    for (int c = tid; c < nch; c += 1024) {
        cgt[c] = 0u;
        if (!any_overflow) {
            int64_t left = n - (int64_t)c * kSelChunk;
            ceq[c] = flat ? (unsigned)(left < kSelChunk ? left : kSelChunk) : 0u;
        }
    }
    __syncthreads();
    if (!any_overflow) {
        for (unsigned x = 0; x < nmine; ++x) {
            if (mine[x].x > T) atomicAdd(&cgt[mine[x].y / kSelChunk], 1u);
            else if (mine[x].x == T) atomicAdd(&ceq[mine[x].y / kSelChunk], 1u);
        }
        __syncthreads();
    } else {
        // very long candidate lists (heavy ties): count straight from the chunks' global lists
        unsigned q[CPT];
#pragma unroll
        for (int e = 0; e < CPT; ++e) q[e] = 0u;
        __syncthreads();
        for (int e = 0; e < CPT; ++e) {
            const int c = tid * CPT + e;
            if (c >= nch) continue;
            unsigned g2 = 0, q2 = 0;
            for (unsigned i = 0; i < cn[e]; ++i) {
                const unsigned x = gcand[(int64_t)c * kSelChunk + i].x;
                g2 += x > T;
                q2 += x == T;
            }
            cgt[c] = g2;
            q[e] = q2;
        }
        __syncthreads();
        for (int e = 0; e < CPT; ++e) {
            const int c = tid * CPT + e;
            if (c < nch) ceq[c] = q[e];
        }
        __syncthreads();
    }
    // per-chunk output offsets: positions greater than T and positions equal to T before the chunk
    unsigned g[CPT], q[CPT], gsum = 0, qsum = 0;
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        const int c = tid * CPT + e;
        g[e] = c < nch ? cg[e] + cgt[c] : 0u;
        q[e] = c < nch ? ceq[c] : 0u;
        gsum += g[e];
        qsum += q[e];
    }
    unsigned gbase = block_exclusive_scan<1024>(gsum, sh_scan, nullptr);
    unsigned qbase = block_exclusive_scan<1024>(qsum, sh_scan, nullptr);
#pragma unroll
    for (int e = 0; e < CPT; ++e) {
        const int c = tid * CPT + e;
        if (c < nch) {
            S.chunk_off[2 * ((int64_t)h * nch + c)] = gbase;
            S.chunk_off[2 * ((int64_t)h * nch + c) + 1] = qbase;
        }
        gbase += g[e];
        qbase += q[e];
    }
    if (tid == 0) {
        S.info[4 * h + 0] = T;
        S.info[4 * h + 2] = need_eq;
    }
}

__global__ __launch_bounds__(256) void sel_emit(const float* __restrict__ score, int64_t n,
                                                int64_t kcount, int nch, int64_t out_stride, int W_tail,
                                                SelectScratch S, int32_t* __restrict__ out_idx) {
    __shared__ unsigned sh_gt[4], sh_eq[4];
    const int h = blockIdx.y, c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int32_t* out = out_idx + (int64_t)h * out_stride;
    if (c == 0)   // window positions n .. n + W_tail - 1 follow the selected prefix positions
        for (int t = tid; t < W_tail; t += 256) out[kcount + t] = (int32_t)(n + t);
    if (kcount <= 0) return;
    const unsigned* s = reinterpret_cast<const unsigned*>(score) + (int64_t)h * n;
    const int64_t base = (int64_t)c * kSelChunk + wave * (kSelChunk / 4);
    unsigned x[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int64_t j = base + e * 64 + lane;
        x[e] = j < n ? s[j] : 0u;
    }
    const unsigned T = S.info[4 * h + 0], need_eq = S.info[4 * h + 2];
    unsigned gt_b = S.chunk_off[2 * ((int64_t)h * nch + c)];
    unsigned eq_b = S.chunk_off[2 * ((int64_t)h * nch + c) + 1];
    unsigned cg = 0, ce = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int64_t j = base + e * 64 + lane;
        cg += j < n && x[e] > T;
        ce += j < n && x[e] == T;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        cg += __shfl_xor(cg, d, 64);
        ce += __shfl_xor(ce, d, 64);
    }
    if (lane == 0) {
        sh_gt[wave] = cg;
        sh_eq[wave] = ce;
    }
    __syncthreads();
    for (int w2 = 0; w2 < wave; ++w2) {
        gt_b += sh_gt[w2];
        eq_b += sh_eq[w2];
    }
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int64_t j = base + e * 64 + lane;
        const bool gt = j < n && x[e] > T;
        const bool eq = j < n && x[e] == T;
        const unsigned long long mgt = __ballot(gt), meq = __ballot(eq);
        const unsigned gt_before = gt_b + (unsigned)__popcll(mgt & lt_mask);
        const unsigned eq_before = eq_b + (unsigned)__popcll(meq & lt_mask);
        if (gt || (eq && eq_before < need_eq))
            out[gt_before + (eq_before < need_eq ? eq_before : need_eq)] = (int32_t)j;
        gt_b += (unsigned)__popcll(mgt);
        eq_b += (unsigned)__popcll(meq);
    }
}

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t select_layout(int H, int64_t n, SelectScratch* S, void* base) {
    const int64_t nn = n > 0 ? n : 1;
    const int64_t nch = (nn + kSelChunk - 1) / kSelChunk;
    const size_t minmax = up256(sizeof(unsigned) * 2 * (size_t)H * (size_t)((nn + 1023) / 1024));
    const size_t hist = up256(sizeof(unsigned) * kSelBins1 * (size_t)H);
    const size_t count = up256(sizeof(unsigned) * (size_t)H * nch);
    const size_t info = up256(sizeof(unsigned) * 4 * (size_t)H);
    const size_t cgt = up256(sizeof(unsigned) * (size_t)H * nch);
    const size_t coff = up256(sizeof(unsigned) * 2 * (size_t)H * nch);
    const size_t cand = up256(sizeof(uint2) * (size_t)H * nn);
    if (S) {
        char* b = static_cast<char*>(base);
        S->minmax = reinterpret_cast<unsigned*>(b);
        S->hist = reinterpret_cast<unsigned*>(b + minmax);
        S->cand_count = reinterpret_cast<unsigned*>(b + minmax + hist);
        S->info = reinterpret_cast<unsigned*>(b + minmax + hist + count);
        S->chunk_gt = reinterpret_cast<unsigned*>(b + minmax + hist + count + info);
        S->chunk_off = reinterpret_cast<unsigned*>(b + minmax + hist + count + info + cgt);
        S->cand = reinterpret_cast<uint2*>(b + minmax + hist + count + info + cgt + coff);
    }
    return minmax + hist + count + info + cgt + coff + cand;
}

bool select_chunked_ok(int64_t n) { return (n + kSelChunk - 1) / kSelChunk <= kSelMaxChunks; }

// One launch that readies all scratch a call needs: the hand-off words of the single-read scoring
// kernel (all-ones = "not published yet") and the selection's histogram and list counters (zero).
__global__ __launch_bounds__(256) void prepare_scratch(unsigned long long* pairs, int64_t npairs,
                                                      unsigned* hist, int nhist, unsigned* cand_count,
                                                      int H) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = i; j < npairs; j += stride) pairs[j] = ~0ull;
    for (int64_t j = i; j < nhist; j += stride) hist[j] = 0u;
    if (i < H) cand_count[i] = 0u;
}

hipError_t launch_prepare(void* pairs, int64_t npairs, const SelectScratch* S, int H, hipStream_t st) {
    const int nhist = S ? H * kSelBins1 : 0;
    int64_t work = npairs > nhist ? npairs : nhist;
    if (work < H) work = H;
    if (work <= 0) return hipSuccess;
    int64_t blocks = (work + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(prepare_scratch, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<unsigned long long*>(pairs), npairs, S ? S->hist : nullptr, nhist,
                       S ? S->cand_count : nullptr, S ? H : 0);
    return hipGetLastError();
}

hipError_t launch_select_init(const SelectScratch& S, int H, hipStream_t st) {
    const int items = H * kSelBins1;
    hipLaunchKernelGGL(sel_init, dim3((items + 255) / 256), dim3(256), 0, st, S, H);
    return hipGetLastError();
}

hipError_t launch_select_chunked(const float* score, int H, int64_t n, int64_t kcount,
                                 int64_t out_stride, int W_tail, int32_t* out_idx,
                                 const SelectScratch& S, int minmax_parts, hipStream_t st) {
    if (H <= 0) return hipSuccess;
    const int nch = (int)((n + kSelChunk - 1) / kSelChunk);
    const dim3 grid(nch, H);
    if (kcount > 0) {
        int nparts = minmax_parts;   // per-part ranges already left by the pooling kernel, or none
        if (nparts <= 0) {
            hipLaunchKernelGGL(sel_minmax, grid, dim3(256), 0, st, score, n, S);
            nparts = nch;
        }
        hipLaunchKernelGGL(sel_hist, dim3((unsigned)((n + kHistChunk - 1) / kHistChunk), H), dim3(1024), 0, st,
                           score, n, nparts, S);
        hipLaunchKernelGGL(sel_compact, grid, dim3(256), 0, st, score, n, kcount, nch, nparts, S);
        hipLaunchKernelGGL(sel_threshold, dim3(H), dim3(1024), 0, st, n, nch, S);
    }
    hipLaunchKernelGGL(sel_emit, grid, dim3(256), 0, st, score, n, kcount, nch, out_stride, W_tail, S,
                       out_idx);
    return hipGetLastError();
}

}  // namespace snapkv
