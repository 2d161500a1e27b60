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
constexpr int kPsThreads = 1024;       // cooperative pooling + selection kernel: threads per workgroup
constexpr int kPsCandCap = 4096;       //   candidates of a head that fit its LDS list
constexpr int kPsBinBits = 11;         //   bits per refinement level
constexpr int kPsBins = 1 << kPsBinBits;
constexpr int kPsLevels = 3;           //   refinement levels (cover all 32 bits)
constexpr int kPsStages = 8;           //   rendezvous points per head: ranges, levels, final
constexpr int kPsMaxGroup = 512;       //   workgroups per head at most

__device__ __forceinline__ int range_shift(unsigned range) {
    // smallest shift with (range >> shift) < kSelBins1
    const int bits = 32 - __clz(range | 1u);
    return bits > 9 ? bits - 9 : 0;
}

__device__ __forceinline__ int range_shift_bits(unsigned range, int digit_bits) {
    // smallest shift with (range >> shift) < 2^digit_bits
    const int bits = 32 - __clz(range | 1u);
    return bits > digit_bits ? bits - digit_bits : 0;
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
                                                  unsigned* sh, unsigned* out, unsigned* out_count = nullptr) {
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
            if (out_count) *out_count = c[e];
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


// ------------------------------------------------------------------------------------------------
// Pooling (Sec. 4.3), group sum and top-k selection (Eq. 2) in ONE cooperative launch.
//
// The Wh workgroups of a KV head each pool a contiguous chunk of the head's votes straight into
// registers (the pooled scores are never written to memory), then agree on the threshold through
// a few rendezvous points in global memory: the head's range of bit patterns, one 512-bin digit
// histogram per refinement level, and finally the few positions inside the threshold bin (or, when
// the bin is a single value, only their number).  Every workgroup then knows the threshold T, how
// many positions equal to T are kept, and how many kept positions lie before its chunk, and emits
// its own kept positions in order.  The arithmetic of the pooled score is that of pool_group, in
// the same order, so the scores are bit-identical to snapkv_pooled_scores; everything after it is
// integer work on bit patterns and does not depend on timing.
//
// All workgroups of the grid must be resident at once (checked by the host).  Waits are bounded:
// if one gives up, later ones are skipped, a counter is raised and the kernel still ends.
// ------------------------------------------------------------------------------------------------
__device__ unsigned g_select_timeouts = 0;


bool reset_select_timeouts() {
    const unsigned zero = 0;
    return hipMemcpyToSymbol(HIP_SYMBOL(g_select_timeouts), &zero, sizeof zero) == hipSuccess;
}

unsigned read_select_timeouts() {
    unsigned v = 0;
    if (hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_select_timeouts), sizeof v) != hipSuccess) return ~0u;
    return v;
}

__device__ __forceinline__ unsigned coherent_load(const unsigned* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Hand-over stores and additions are issued as atomics WITH a return value, and the wave waits for
// all of them before the rendezvous below.  A store, or an addition whose result nobody asks for,
// only has to be on its way when the wave's memory counter lets go of it; the returning form
// completes when it has been performed where all dies see it.  The callers fold the returned
// values into a dummy so that several can be in flight, and hand the dummy to hand_over_done().
__device__ __forceinline__ unsigned coherent_store(unsigned* p, unsigned v) {
    return __hip_atomic_exchange(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned coherent_store64(unsigned long long* p, unsigned long long v) {
    return (unsigned)__hip_atomic_exchange(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned coherent_add(unsigned* p, unsigned v) {
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Operand of s_waitcnt that waits for ALL of the wave's outstanding vector-memory operations and for
// nothing else.  gfx9-family layout of the 16-bit operand (gfx950 included): vmcnt is split over bits
// [3:0] (low four bits) and [15:14] (high two), expcnt is bits [6:4], lgkmcnt bits [11:8]; a counter field
// at its maximum means "do not wait for this counter".  vmcnt = 0 (all six bits clear), expcnt = 7,
// lgkmcnt = 15:
constexpr int kWaitVmcnt0 = (0 << 0) | (7 << 4) | (15 << 8) | (0 << 14);
static_assert(kWaitVmcnt0 == 0x0F70, "s_waitcnt vmcnt(0) on the gfx9 family");

// Every hand-over of this thread has been performed once this returns: a hand-over is an atomic WITH a
// return value, and the value can only come back from the place where the device's dies agree on the
// word's contents (the atomic has been carried out there by then).
__device__ __forceinline__ void hand_over_done(unsigned folded) {
    asm volatile("" ::"v"(folded));            // the returned values are needed here: the wave waits for them
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);   // and for anything else it has outstanding
}

// Rendezvous of the `expect` workgroups that share `ctr` (zero before the first arrival).  What a
// workgroup handed over before the call with coherent_store / coherent_add (and waited for with
// hand_over_done) can be read by all of them after it with coherent_load.  No cache write-back or
// invalidate is involved: those accesses are performed at the device's coherence point.  Every wave
// waits for its own outstanding memory operations before the barrier (a workgroup-scope fence does
// not: inside a compute unit it has nothing to wait for), and only then does thread 0 count the
// workgroup in.
__device__ __forceinline__ void group_rendezvous(unsigned* ctr, unsigned expect, unsigned limit,
                                                 unsigned* gave_up) {
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (threadIdx.x == 0 && !*gave_up) {
        __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < expect) {
            if (++spins > limit) {
                *gave_up = 1u;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
    }
    __syncthreads();
}

// Sums of up to three values over the block, one barrier pair for all of them; every thread gets
// the totals.  sh needs 3 * NT / 64 words and may be reused right after the call returns.
template <int NT>
__device__ __forceinline__ void block_sum3(unsigned& a, unsigned& b, unsigned& c, unsigned* sh) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        a += __shfl_xor(a, d, 64);
        b += __shfl_xor(b, d, 64);
        c += __shfl_xor(c, d, 64);
    }
    __syncthreads();
    if (lane == 0) {
        sh[wave] = a;
        sh[NT / 64 + wave] = b;
        sh[2 * (NT / 64) + wave] = c;
    }
    __syncthreads();
    a = b = c = 0u;
#pragma unroll
    for (int w2 = 0; w2 < NT / 64; ++w2) {
        a += sh[w2];
        b += sh[NT / 64 + w2];
        c += sh[2 * (NT / 64) + w2];
    }
}

template <int EPT, int P, int KIND>   // KIND: 0 max pooling, 1 average pooling
__global__ __launch_bounds__(kPsThreads) void pool_select(
    const float* __restrict__ vote, const ScoreGeom G, const int p_arg,
    const int64_t kcount, const int64_t out_stride, const int W_tail, int32_t* __restrict__ out_idx,
    const SelectScratch S, const int Wh, const int chunk, const unsigned spin_limit,
    const int32_t* __restrict__ nvalid) {
    constexpr int NT = kPsThreads;
    constexpr int NWV = NT / 64;
    // One dynamic LDS block, used in turn as the staging area of the votes (chunk plus a halo of
    // p/2 positions on either side) and, once the scores sit in registers, as digit histogram
    // (kPsBins words) followed by the candidate list (kPsCandCap pairs).
    extern __shared__ __attribute__((aligned(16))) unsigned ps_lds[];
    float* const stage = reinterpret_cast<float*>(ps_lds);
    unsigned* const sh_hist = ps_lds;
    uint2* const sh_cand = reinterpret_cast<uint2*>(ps_lds + kPsBins);
    __shared__ unsigned sh_tab[2][(EPT / 4) * NWV]; // per (run row, wave) counts for the ordered emission
    __shared__ unsigned sh_scan[16], sh_out[2], sh_red[3 * NWV], sh_gave_up, sh_bin_count;
    __shared__ unsigned sh_off[kPsMaxGroup + 1];    // start of each workgroup's candidates in the merged list
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x / Wh, c = blockIdx.x % Wh;
    // rows of votes and candidate lists are G.n apart; a head may have fewer valid positions (a
    // batch of prompts of different lengths shares one launch)
    const int64_t pitch = G.n;
    int64_t n = pitch;
    if (nvalid) {
        n = nvalid[h];
        n = n < 0 ? 0 : (n > pitch ? pitch : n);
    }
    const int64_t chunk0 = (int64_t)c * chunk;
    const int64_t chunk1 = chunk0 + chunk < n ? chunk0 + chunk : n;
    const int len = chunk1 > chunk0 ? (int)(chunk1 - chunk0) : 0;
    int32_t* out = out_idx + (int64_t)h * out_stride;
    if (c == 0)   // window positions follow the selected prefix positions
        for (int t = tid; t < W_tail; t += NT) out[kcount + t] = (int32_t)(n + t);
    if (kcount <= 0) return;
    if (tid == 0) sh_gave_up = 0u;

    // ---- pooled, group-summed scores of this thread's positions, in the arithmetic and order of
    // pool_group.  A thread owns EPT / 4 runs of four consecutive positions: element e = 4 * e4 + k
    // is position chunk0 + e4 * 4 * NT + 4 * tid + k, so that position order is (e4, thread, k).
    // Per query head the chunk's votes and a halo on either side pass through LDS once (as
    // 16-byte pieces where the rows are aligned); the taps of four positions are then a few
    // 16-byte LDS reads.
    static_assert(EPT % 4 == 0, "positions are owned in runs of four");
    constexpr int E4 = EPT / 4;
    const int p = P > 0 ? P : p_arg;
    const int r = p >> 1;
    const int HQ = 4 * ((r + 3) / 4);            // halo, rounded up to whole 16-byte pieces
    constexpr int pool_kind = KIND;
    const float pad = KIND == 0 ? -INFINITY : 0.f;
    const int nf4 = ((len + 3) / 4) + 2 * (HQ / 4);   // 16-byte pieces to stage
    const bool rows_aligned = ((n | pitch) & 3) == 0 && (reinterpret_cast<uintptr_t>(vote) & 15u) == 0;
    auto pos_local = [&](int e) { return (e >> 2) * (4 * NT) + 4 * tid + (e & 3); };
    const int nn = (int)n, kc = (int)kcount;
    unsigned x[EPT];
    {
        float acc[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) acc[e] = 0.f;
        for (int hq = 0; hq < G.g; ++hq) {
            const float* vb = vote + ((int64_t)h * G.NV + (int64_t)hq * G.VB) * pitch;
            if (hq > 0) __syncthreads();          // the previous head's taps have been read
            float4 land[E4 + 1];                  // all loads are in flight before the first LDS write
#pragma unroll
            for (int e4 = 0; e4 <= E4; ++e4) {
                const int f = e4 * NT + tid;
                const int q0 = (int)chunk0 - HQ + 4 * f;     // positions fit 32 bits (n < 2^31)
                float4 t4 = make_float4(pad, pad, pad, pad);
                if (f < nf4) {
                    if (P > 0 && rows_aligned) {
                        if (q0 >= 0 && q0 < nn) {
                            t4 = *reinterpret_cast<const float4*>(vb + q0);
                            if constexpr (EPT <= 4) {   // (at 16 positions per thread this sum costs registers the kernel does not have)
                                for (int b = 1; b < G.VB; ++b) {   // the vote rows of a query head, in order
                                    const float4 u = *reinterpret_cast<const float4*>(vb + (int64_t)b * pitch + q0);
                                    t4.x += u.x;
                                    t4.y += u.y;
                                    t4.z += u.z;
                                    t4.w += u.w;
                                }
                            }
                        }
                    } else {
                        float t[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const int q = q0 + k;
                            t[k] = pad;
                            if (q >= 0 && q < nn) {
                                t[k] = vb[q];
                                if (P == 0 || EPT <= 4)   // several vote rows per query head: the loop form, or the light kernel
                                    for (int b = 1; b < G.VB; ++b) t[k] += vb[(int64_t)b * pitch + q];
                            }
                        }
                        t4 = make_float4(t[0], t[1], t[2], t[3]);
                    }
                }
                land[e4] = t4;
            }
#pragma unroll
            for (int e4 = 0; e4 <= E4; ++e4) {
                const int f = e4 * NT + tid;
                if (f < nf4) reinterpret_cast<float4*>(stage)[f] = land[e4];
            }
            __syncthreads();
#pragma unroll
            for (int e4 = 0; e4 < E4; ++e4) {
                const int i0 = e4 * (4 * NT) + 4 * tid;      // first of the four positions; its taps
                if (i0 >= len) continue;                     // start at stage[i0 + HQ - r]
                if (P > 0) {
                    constexpr int RQ = (P / 2 + 3) / 4, NV4 = 2 * RQ + 1;
                    float v[4 * NV4];
#pragma unroll
                    for (int b4 = 0; b4 < NV4; ++b4) {
                        const float4 q4 = reinterpret_cast<const float4*>(stage)[(i0 >> 2) + b4];
                        v[4 * b4] = q4.x;
                        v[4 * b4 + 1] = q4.y;
                        v[4 * b4 + 2] = q4.z;
                        v[4 * b4 + 3] = q4.w;
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        float val = v[4 * RQ + k - P / 2];
#pragma unroll
                        for (int d = 1; d < P; ++d)
                            val = pool_kind == 0 ? fmaxf(val, v[4 * RQ + k - P / 2 + d]) : val + v[4 * RQ + k - P / 2 + d];
                        if (pool_kind != 0) val = val / (float)P;
                        acc[4 * e4 + k] += val;
                    }
                } else if (p >= 5) {
                    // The four positions share all but three of their taps: every staged value is read
                    // once and goes to the positions whose window holds it, each position taking its
                    // taps in increasing order (the order of the plain loop below, so sums agree bit for bit).
                    const int s0 = i0 + HQ - r;
                    auto op = [](float a, float b) { return KIND == 0 ? fmaxf(a, b) : a + b; };
                    const float t0 = stage[s0], t1 = stage[s0 + 1], t2 = stage[s0 + 2];
                    float v0 = op(op(t0, t1), t2), v1 = op(t1, t2), v2 = t2;
                    float t = stage[s0 + 3];
                    v0 = op(v0, t);
                    v1 = op(v1, t);
                    v2 = op(v2, t);
                    float v3 = t;
                    for (int d = 4; d < p; ++d) {
                        t = stage[s0 + d];
                        v0 = op(v0, t);
                        v1 = op(v1, t);
                        v2 = op(v2, t);
                        v3 = op(v3, t);
                    }
                    t = stage[s0 + p];
                    v1 = op(v1, t);
                    v2 = op(v2, t);
                    v3 = op(v3, t);
                    t = stage[s0 + p + 1];
                    v2 = op(v2, t);
                    v3 = op(v3, t);
                    v3 = op(v3, stage[s0 + p + 2]);
                    if (pool_kind != 0) {
                        v0 = v0 / (float)p;
                        v1 = v1 / (float)p;
                        v2 = v2 / (float)p;
                        v3 = v3 / (float)p;
                    }
                    acc[4 * e4] += v0;
                    acc[4 * e4 + 1] += v1;
                    acc[4 * e4 + 2] += v2;
                    acc[4 * e4 + 3] += v3;
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int s0 = i0 + k + HQ - r;
                        float val = stage[s0];
                        for (int d = 1; d < p; ++d) val = pool_kind == 0 ? fmaxf(val, stage[s0 + d]) : val + stage[s0 + d];
                        if (pool_kind != 0) val = val / (float)p;
                        acc[4 * e4 + k] += val;
                    }
                }
            }
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) x[e] = __float_as_uint(acc[e]);
    }
    unsigned active = 0;        // bit e: position e is valid and still inside the searched range
#pragma unroll
    for (int e = 0; e < EPT; ++e)
        if (pos_local(e) < len) active |= 1u << e;
    const unsigned valid = active;

    // ---- the head's range of bit patterns
    unsigned lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int e = 0; e < EPT; ++e)
        if (valid >> e & 1u) {
            lo = x[e] < lo ? x[e] : lo;
            hi = x[e] > hi ? x[e] : hi;
        }
    auto block_range = [&]() {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const unsigned a = __shfl_xor(lo, d, 64), b = __shfl_xor(hi, d, 64);
            lo = a < lo ? a : lo;
            hi = b > hi ? b : hi;
        }
        __syncthreads();
        if (lane == 0) {
            sh_red[2 * wave] = lo;
            sh_red[2 * wave + 1] = hi;
        }
        __syncthreads();
#pragma unroll
        for (int w2 = 0; w2 < NWV; ++w2) {
            lo = sh_red[2 * w2] < lo ? sh_red[2 * w2] : lo;
            hi = sh_red[2 * w2 + 1] > hi ? sh_red[2 * w2 + 1] : hi;
        }
    };
    block_range();
    if (tid == 0) {
        unsigned done = coherent_store(&S.ps_range[2 * ((int64_t)h * kPsMaxGroup + c)], lo);
        done ^= coherent_store(&S.ps_range[2 * ((int64_t)h * kPsMaxGroup + c) + 1], hi);
        hand_over_done(done);
    }
    unsigned* arrive = S.ps_arrive + (int64_t)h * kPsStages;
    group_rendezvous(arrive + 0, (unsigned)Wh, spin_limit, &sh_gave_up);
    lo = 0xFFFFFFFFu;
    hi = 0u;
    for (int i = lane; i < Wh; i += 64) {     // every wave reads all of them: no barrier needed
        const unsigned a = coherent_load(&S.ps_range[2 * ((int64_t)h * kPsMaxGroup + i)]);
        const unsigned b = coherent_load(&S.ps_range[2 * ((int64_t)h * kPsMaxGroup + i) + 1]);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned a = __shfl_xor(lo, d, 64), b = __shfl_xor(hi, d, 64);
        lo = a < lo ? a : lo;
        hi = b > hi ? b : hi;
    }

    // ---- threshold bin: 11 bits per level until the bin is a single value or holds few positions
    unsigned cur_lo = lo, krem = (unsigned)kcount, above = 0, bin_count = 0, T = lo, need_eq = 0;
    int cur_sh = hi > lo ? range_shift_bits(hi - lo, kPsBinBits) : 0;
    bool exact = hi <= lo;      // T is known exactly (all remaining positions are equal to it)
    if (exact) need_eq = krem;
    for (int lvl = 0; lvl < kPsLevels && !exact; ++lvl) {
        __syncthreads();
        for (int b = tid; b < kPsBins; b += NT) sh_hist[b] = 0u;
        if (tid == 0) {
            sh_out[0] = 0u;
            sh_out[1] = 1u;
            sh_bin_count = 0u;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (active >> e & 1u) atomicAdd(&sh_hist[((x[e] - cur_lo) >> cur_sh) & (kPsBins - 1)], 1u);
        __syncthreads();
        unsigned* gh = S.ps_hist + ((int64_t)h * kPsLevels + lvl) * kPsBins;
        unsigned done = 0;
        for (int b = tid; b < kPsBins; b += NT) {
            const unsigned cnt = sh_hist[b];
            if (cnt) done ^= coherent_add(&gh[b], cnt);
        }
        hand_over_done(done);
        group_rendezvous(arrive + 1 + lvl, (unsigned)Wh, spin_limit, &sh_gave_up);
        unsigned bins[kPsBins / NT];
#pragma unroll
        for (int e = 0; e < kPsBins / NT; ++e)
            bins[e] = coherent_load(&gh[kPsBins - 1 - (tid * (kPsBins / NT) + e)]);
        find_bin_from_top<NT, kPsBins>(bins, krem, sh_scan, sh_out, &sh_bin_count);
        const unsigned b1 = sh_out[0] & (kPsBins - 1);
        krem = sh_out[1];
        bin_count = sh_bin_count;
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (active >> e & 1u) {
                const unsigned d = ((x[e] - cur_lo) >> cur_sh) & (kPsBins - 1);
                if (d > b1) ++above;
                if (d != b1) active &= ~(1u << e);
            }
        cur_lo += b1 << cur_sh;
        if (cur_sh == 0) {
            exact = true;
            T = cur_lo;
            need_eq = krem;
        } else if (bin_count <= (unsigned)kPsCandCap) {
            break;
        } else {
            cur_sh = range_shift_bits((1u << cur_sh) - 1u, kPsBinBits);
        }
    }

    // ---- final exchange: counts per workgroup, and the candidates unless T is already exact
    const unsigned mine_in = (unsigned)__popc(active);
    unsigned in_total = 0;
    const unsigned in_before = block_exclusive_scan<NT>(mine_in, sh_scan, &in_total);
    unsigned above_total = above, z1 = 0, z2 = 0;
    block_sum3<NT>(above_total, z1, z2, sh_red);
    if (!exact) {   // this workgroup's candidates go to the start of its own stretch of the head's list
        unsigned slot = in_before, done = 0;
        unsigned long long* const my_cand = reinterpret_cast<unsigned long long*>(S.cand + (int64_t)h * pitch + chunk0);
#pragma unroll
        for (int e = 0; e < EPT; ++e)
            if (active >> e & 1u) {
                if (slot < (unsigned)len)
                    done ^= coherent_store64(my_cand + slot,
                                             ((unsigned long long)(unsigned)((int)chunk0 + pos_local(e)) << 32) | x[e]);
                ++slot;
            }
        hand_over_done(done);
    }
    if (tid == 0) {
        unsigned done = coherent_store(&S.ps_part[2 * ((int64_t)h * kPsMaxGroup + c)], above_total);
        done ^= coherent_store(&S.ps_part[2 * ((int64_t)h * kPsMaxGroup + c) + 1], in_total);
        hand_over_done(done);
    }
    group_rendezvous(arrive + 1 + kPsLevels, (unsigned)Wh, spin_limit, &sh_gave_up);

    // kept positions of the head before this chunk.  Every wave sums the per-workgroup counts
    // itself (no barrier); without an exact T the candidates are fetched, workgroup by workgroup.
    unsigned gt_before = 0, eq_before = 0;
    {
        unsigned run = 0;           // candidates of the workgroups before `base`
        for (int base = 0; base < Wh; base += 64) {
            const int i = base + lane;
            unsigned ab = 0, cnt = 0;
            if (i < Wh) {
                ab = coherent_load(&S.ps_part[2 * ((int64_t)h * kPsMaxGroup + i)]);
                cnt = coherent_load(&S.ps_part[2 * ((int64_t)h * kPsMaxGroup + i) + 1]);
            }
            if (i < c) {
                gt_before += ab;
                eq_before += cnt;
            }
            if (!exact && wave == 0) {   // where each workgroup's candidates start in the merged list
                unsigned inc = cnt;
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const unsigned up = __shfl_up(inc, d, 64);
                    if (lane >= d) inc += up;
                }
                if (i < Wh) sh_off[i] = run + inc - cnt;
                run += __shfl(inc, 63, 64);
            }
        }
        if (!exact && wave == 0 && lane == 0) sh_off[Wh] = run;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        gt_before += __shfl_xor(gt_before, d, 64);
        eq_before += __shfl_xor(eq_before, d, 64);
    }
    if (!exact) {
        eq_before = 0;              // positions inside the bin are counted from the candidate list
        const unsigned m = bin_count < (unsigned)kPsCandCap ? bin_count : (unsigned)kPsCandCap;
        __syncthreads();
        for (unsigned i = tid; i < m; i += NT) {
            int a2 = 0, b2 = Wh;            // largest c2 with sh_off[c2] <= i
            while (b2 - a2 > 1) {
                const int mid = (a2 + b2) >> 1;
                if (sh_off[mid] <= i) a2 = mid; else b2 = mid;
            }
            int64_t at = (int64_t)a2 * chunk + (i - sh_off[a2]);
            at = at < pitch ? at : pitch - 1;       // only counts that a failed rendezvous left inconsistent get here
            const unsigned long long both = __hip_atomic_load(
                reinterpret_cast<const unsigned long long*>(&S.cand[(int64_t)h * pitch + at]),
                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sh_cand[i] = make_uint2((unsigned)(both & 0xffffffffull), (unsigned)(both >> 32));
        }
        int rem_sh = cur_sh;            // bits of the pattern still undecided inside the bin
        while (rem_sh > 0) {
            const int nsh = rem_sh > kPsBinBits ? rem_sh - kPsBinBits : 0;
            for (int b = tid; b < kPsBins; b += NT) sh_hist[b] = 0u;
            if (tid == 0) {
                sh_out[0] = 0u;
                sh_out[1] = 1u;
            }
            __syncthreads();
            for (unsigned i = tid; i < m; i += NT) {
                const unsigned v = sh_cand[i].x;
                if (v >= cur_lo && ((v - cur_lo) >> rem_sh) == 0u)
                    atomicAdd(&sh_hist[((v - cur_lo) >> nsh) & (kPsBins - 1)], 1u);
            }
            __syncthreads();
            unsigned bins[kPsBins / NT];
            load_bins_from_top<NT, kPsBins>(sh_hist, bins);
            find_bin_from_top<NT, kPsBins>(bins, krem, sh_scan, sh_out);
            cur_lo += (sh_out[0] & (kPsBins - 1)) << nsh;
            krem = sh_out[1];
            rem_sh = nsh;
            __syncthreads();
        }
        __syncthreads();
        T = cur_lo;
        need_eq = krem;
        unsigned g2 = 0, q2 = 0, z = 0;   // candidates before this chunk: greater than / equal to T
        for (unsigned i = tid; i < m; i += NT) {
            const uint2 cd = sh_cand[i];
            if ((int64_t)cd.y < chunk0) {
                g2 += cd.x > T;
                q2 += cd.x == T;
            }
        }
        block_sum3<NT>(g2, q2, z, sh_red);
        gt_before += g2;
        eq_before = q2;
    }

    // ---- ordered emission: position order is (run e4, wave, lane, k).  Every wave leaves the
    // counts of its part of each run row in a table; lane e4 of a wave then turns row e4 of the
    // table into the number of kept positions before the wave's part of that row.
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    unsigned inc_g[E4], inc_q[E4], cnt_g[E4], cnt_q[E4];   // per row: this thread's counts, scanned over the wave
#pragma unroll
    for (int e4 = 0; e4 < E4; ++e4) {
        unsigned cg = 0, cq = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = 4 * e4 + k;
            const bool ok = valid >> e & 1u;
            cg += ok && x[e] > T;
            cq += ok && x[e] == T;
        }
        // counts are at most 4: the wave-wide inclusive scan is three ballots per count
        unsigned ig = cg, iq = cq;
#pragma unroll
        for (int bit = 0; bit < 3; ++bit) {
            ig += (unsigned)__popcll(__ballot(cg >> bit & 1u) & lt_mask) << bit;
            iq += (unsigned)__popcll(__ballot(cq >> bit & 1u) & lt_mask) << bit;
        }
        cnt_g[e4] = cg;
        cnt_q[e4] = cq;
        inc_g[e4] = ig;
        inc_q[e4] = iq;
        if (lane == 63) {
            sh_tab[0][e4 * NWV + wave] = ig;
            sh_tab[1][e4 * NWV + wave] = iq;
        }
    }
    __syncthreads();
    unsigned base_gt = 0, base_eq = 0;          // lane e4 < E4: kept positions before (row e4, this wave)
    {
        unsigned row_gt = 0, row_eq = 0, mine_gt = 0, mine_eq = 0;
        if (lane < E4) {
#pragma unroll
            for (int w2 = 0; w2 < NWV; ++w2) {
                const unsigned a2 = sh_tab[0][lane * NWV + w2], q2 = sh_tab[1][lane * NWV + w2];
                row_gt += a2;
                row_eq += q2;
                if (w2 < wave) {
                    mine_gt += a2;
                    mine_eq += q2;
                }
            }
        }
        unsigned ig = row_gt, iq = row_eq;      // inclusive scan over the rows (lanes 0..E4-1)
#pragma unroll
        for (int d = 1; d < E4; d <<= 1) {
            const unsigned ug = __shfl_up(ig, d, 64), uq = __shfl_up(iq, d, 64);
            if (lane >= d) {
                ig += ug;
                iq += uq;
            }
        }
        base_gt = gt_before + ig - row_gt + mine_gt;
        base_eq = eq_before + iq - row_eq + mine_eq;
    }
#pragma unroll
    for (int e4 = 0; e4 < E4; ++e4) {
        unsigned gb = __shfl(base_gt, e4, 64) + inc_g[e4] - cnt_g[e4];
        unsigned qb = __shfl(base_eq, e4, 64) + inc_q[e4] - cnt_q[e4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int e = 4 * e4 + k;
            const bool ok = valid >> e & 1u;
            const bool gt = ok && x[e] > T, eq = ok && x[e] == T;
            if (gt || (eq && qb < need_eq)) {
                const unsigned at = gb + (qb < need_eq ? qb : need_eq);
                if (at < (unsigned)kc) out[at] = (int32_t)chunk0 + pos_local(e);
            }
            gb += gt;
            qb += eq;
        }
    }
    if (tid == 0 && sh_gave_up) {
        atomicAdd(&g_select_timeouts, 1u);
        if (S.ps_flag) __hip_atomic_store(S.ps_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t select_counter_bytes(int H) {
    return up256(sizeof(unsigned) * (size_t)H * (kPsStages + kPsLevels * kPsBins));
}

// own_counters: the arrival counters and digit histograms of pool_select sit at the end of this
// layout; otherwise they are not part of it and are placed at `counters`
// (select_counter_bytes(H) bytes), so that a caller can keep them at an address that does not
// move with n.
size_t select_layout(int H, int64_t n, SelectScratch* S, void* base, bool own_counters, void* counters) {
    const int64_t nn = n > 0 ? n : 1;
    const int64_t nch = (nn + kSelChunk - 1) / kSelChunk;
    const size_t minmax = up256(sizeof(unsigned) * 2 * (size_t)H * (size_t)((nn + 1023) / 1024));
    const size_t hist = up256(sizeof(unsigned) * kSelBins1 * (size_t)H);
    const size_t count = up256(sizeof(unsigned) * (size_t)H * nch);
    const size_t info = up256(sizeof(unsigned) * 4 * (size_t)H);
    const size_t cgt = up256(sizeof(unsigned) * (size_t)H * nch);
    const size_t coff = up256(sizeof(unsigned) * 2 * (size_t)H * nch);
    const size_t cand = up256(sizeof(uint2) * (size_t)H * nn);
    const size_t ps_range = up256(sizeof(unsigned) * 2 * (size_t)H * kPsMaxGroup);
    const size_t ps_zero = select_counter_bytes(H);
    if (S) {
        char* b = static_cast<char*>(base);
        S->minmax = reinterpret_cast<unsigned*>(b);
        S->hist = reinterpret_cast<unsigned*>(b + minmax);
        S->cand_count = reinterpret_cast<unsigned*>(b + minmax + hist);
        S->info = reinterpret_cast<unsigned*>(b + minmax + hist + count);
        S->chunk_gt = reinterpret_cast<unsigned*>(b + minmax + hist + count + info);
        S->chunk_off = reinterpret_cast<unsigned*>(b + minmax + hist + count + info + cgt);
        S->cand = reinterpret_cast<uint2*>(b + minmax + hist + count + info + cgt + coff);
        char* q = b + minmax + hist + count + info + cgt + coff + cand;
        S->ps_range = reinterpret_cast<unsigned*>(q);
        S->ps_part = reinterpret_cast<unsigned*>(q + ps_range);
        S->ps_arrive = reinterpret_cast<unsigned*>(own_counters ? q + 2 * ps_range : static_cast<char*>(counters));
        S->ps_hist = S->ps_arrive + (size_t)H * kPsStages;
        S->ps_zero_words = (int64_t)H * (kPsStages + kPsLevels * kPsBins);
        S->ps_flag = nullptr;
    }
    return minmax + hist + count + info + cgt + coff + cand + 2 * ps_range + (own_counters ? ps_zero : 0);
}

bool select_chunked_ok(int64_t n) { return (n + kSelChunk - 1) / kSelChunk <= kSelMaxChunks; }

// One launch that readies all scratch a call needs: the hand-off words of the single-read scoring
// kernel (all-ones = "not published yet") and the selection's histogram and list counters (zero).
__global__ __launch_bounds__(256) void prepare_scratch(unsigned long long* pairs, int64_t npairs,
                                                      unsigned* hist, int nhist, unsigned* cand_count,
                                                      int H, unsigned* ps_zero, int64_t ps_words, unsigned* flag) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && flag) *flag = 0u;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = i; j < npairs; j += stride) pairs[j] = ~0ull;
    for (int64_t j = i; j < nhist; j += stride) hist[j] = 0u;
    for (int64_t j = i; j < ps_words; j += stride) ps_zero[j] = 0u;
    if (i < H) cand_count[i] = 0u;
}

hipError_t launch_prepare(void* pairs, int64_t npairs, const SelectScratch* S, int H, hipStream_t st, unsigned* flag) {
    const int nhist = S ? H * kSelBins1 : 0;
    int64_t work = npairs > nhist ? npairs : nhist;
    if (S && work < S->ps_zero_words) work = S->ps_zero_words;
    if (work < H) work = H;
    if (!flag && S) flag = S->ps_flag;
    if (work <= 0 && flag) work = 1;
    if (work <= 0) return hipSuccess;
    int64_t blocks = (work + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(prepare_scratch, dim3((unsigned)blocks), dim3(256), 0, st,
                       static_cast<unsigned long long*>(pairs), npairs, S ? S->hist : nullptr, nhist,
                       S ? S->cand_count : nullptr, S ? H : 0, S ? S->ps_arrive : nullptr,
                       S ? S->ps_zero_words : 0, flag);
    return hipGetLastError();
}

// ---- host side of the cooperative kernel
struct PoolSelCall {
    const float* vote;
    const ScoreGeom* G;
    int pool_kind, p;
    int64_t kcount, out_stride;
    int W_tail;
    int32_t* out_idx;
    const SelectScratch* S;
    int Wh, chunk;
    hipStream_t st;
    const int32_t* nvalid;
};

constexpr unsigned kPsSpinLimit = 1u << 14;    // polls before a rendezvous gives up (tens of ms)

// With call == nullptr: returns in *occ how many workgroups of this instantiation one compute unit
// keeps resident.  Otherwise launches.
template <int EPT, int P, int KIND>
static hipError_t pool_select_instance(const PoolSelCall* call, int* occ) {
    auto kern = pool_select<EPT, P, KIND>;
    // staging area of the votes (chunk + halo for p <= 129) or histogram + candidate list
    constexpr size_t kStage = sizeof(float) * ((size_t)EPT * kPsThreads + 128);
    constexpr size_t kSearch = sizeof(unsigned) * kPsBins + sizeof(uint2) * kPsCandCap;
    constexpr size_t kLds = kStage > kSearch ? kStage : kSearch;
    if (!call) {
        static int cached[64] = {0};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        if (cached[dev] == 0) {
            int nb = 0;
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
            if (e != hipSuccess) return e;
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, kPsThreads, kLds);
            if (e != hipSuccess) return e;
            cached[dev] = nb > 0 ? nb : -1;
        }
        *occ = cached[dev] > 0 ? cached[dev] : 0;
        return hipSuccess;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(call->G->Hkv * call->Wh)), dim3(kPsThreads), kLds, call->st,
                       call->vote, *call->G, call->p, call->kcount, call->out_stride,
                       call->W_tail, call->out_idx, *call->S, call->Wh, call->chunk, wait_limit(kPsSpinLimit), call->nvalid);
    return hipGetLastError();
}

template <int EPT, int KIND>
static hipError_t pool_select_by_width(int pw, const PoolSelCall* call, int* occ) {
    switch (pw) {   // the widths the paper uses (Sec. 5) get unrolled taps
        case 5: return pool_select_instance<EPT, 5, KIND>(call, occ);
        case 7: return pool_select_instance<EPT, 7, KIND>(call, occ);
        case 13:   // 13 taps of 16 positions do not fit the registers: the loop form is faster there
            if constexpr (EPT <= 4) return pool_select_instance<EPT, 13, KIND>(call, occ);
            return pool_select_instance<EPT, 0, KIND>(call, occ);
        default: return pool_select_instance<EPT, 0, KIND>(call, occ);
    }
}

static hipError_t pool_select_dispatch(int ept, int pw, int kind, const PoolSelCall* call, int* occ) {
    if (ept == 4) return kind == 0 ? pool_select_by_width<4, 0>(pw, call, occ) : pool_select_by_width<4, 1>(pw, call, occ);
    return kind == 0 ? pool_select_by_width<16, 0>(pw, call, occ) : pool_select_by_width<16, 1>(pw, call, occ);
}

static int ps_cu_count() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int nc = 0;
        if (hipDeviceGetAttribute(&nc, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev] = nc;
    }
    return cached[dev];
}

// Width the kernel is instantiated for (unrolled taps), or 0 for the loop form.  With several vote rows
// per query head only the kernel for 4 positions per thread has the unrolled form.
static int ps_width(const ScoreGeom& G, int p, int ept) {
    return ((G.VB == 1 || ept <= 4) && (p == 5 || p == 7 || p == 13)) ? p : 0;
}

static bool pool_select_plan(const ScoreGeom& G, int pool_kind, int p, int64_t kcount, int* Wh, int* chunk, int* ept) {
    if (G.n < 1 || kcount < 0 || kcount > G.n || G.Hkv < 1) return false;
    const int cus = ps_cu_count();
    if (cus <= 0) return false;
    for (int e : {4, 16}) {   // positions per thread: the lighter variant when the chunks allow it
        int occ = 0;
        if (pool_select_dispatch(e, ps_width(G, p, e), pool_kind, nullptr, &occ) != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        const int64_t resident = (int64_t)cus * occ;
        if (occ <= 0 || G.Hkv > resident) continue;
        int64_t w = resident / G.Hkv;
        if (w > kPsMaxGroup) w = kPsMaxGroup;
        const int64_t want = G.n / 2048 > 1 ? G.n / 2048 : 1;   // at least 2048 positions per workgroup
        if (w > want) w = want;
        const int64_t ch = ((G.n + w - 1) / w + 3) & ~(int64_t)3;   // whole runs of four positions
        if (ch > (int64_t)e * kPsThreads) continue;   // does not fit the workgroups' registers
        *Wh = (int)w;
        *chunk = (int)ch;
        *ept = e;
        return true;
    }
    return false;
}

bool pool_select_ok(const ScoreGeom& G, int pool_kind, int p, int64_t kcount) {
    int Wh = 0, chunk = 0, ept = 0;
    return pool_select_plan(G, pool_kind, p, kcount, &Wh, &chunk, &ept);
}

hipError_t launch_pool_select(const ScoreGeom& G, const float* vote, int pool_kind, int p, int64_t kcount,
                              int64_t out_stride, int W_tail, int32_t* out_idx, const SelectScratch& S,
                              hipStream_t st, const int32_t* nvalid) {
    int Wh = 0, chunk = 0, ept = 0;
    if (!pool_select_plan(G, pool_kind, p, kcount, &Wh, &chunk, &ept)) return hipErrorInvalidValue;
    const PoolSelCall call{vote, &G, pool_kind, p, kcount, out_stride, W_tail, out_idx, &S, Wh, chunk, st, nvalid};
    int occ = 0;
    return pool_select_dispatch(ept, ps_width(G, p, ept), pool_kind, &call, &occ);
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

