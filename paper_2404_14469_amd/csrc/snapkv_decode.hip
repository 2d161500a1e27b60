// One decoding step of attention over a compacted KV cache (Sec. 5.1.2: every generated token
// attends to the C kept rows of Listing 1 plus the rows appended since).  The step reads every
// cached K and V row once and is bound by that traffic; all arithmetic rides on MFMA so that the
// vector units only convert and exponentiate.
//
// Work split.  A workgroup of four waves owns a range of keys of one (sequence, KV head) and all
// g query heads that read it; a wave walks its keys 32 at a time (two 16-key tiles X and Y).
// With few (sequence, head) pairs the keys of a pair are split over several workgroups, which
// leave (max, sum, unnormalised output) partials that a second small kernel merges.
//
// MFMA layout (16x16x32, 64 lanes): lane l supplies row/column l%16 and contraction slice l/16
// (eight elements); accumulator register r of lane l is row 4*(l/16) + r, column l%16.
//
//   logits^T = K Q^T: a lane loads the 16-byte pieces 4c + l/16 of key row l%16 (the natural
//     row-major read) and of query row l%16; the result puts four consecutive keys of one query
//     head into each lane, which is exactly the per-lane contraction slice the last product
//     needs, so the probabilities never move between lanes.
//   V^T by MFMA: the value rows arrive the same way (a lane holds eight head-dim elements of one
//     key) but the last product contracts over keys.  Multiplying a 16-key tile by a 0/1
//     selection matrix (one MFMA per 16 head-dim columns) returns the same numbers with four
//     consecutive keys of one head-dim column per lane: an exact transposition in registers,
//     with no LDS traffic.  Non-finite values would spread along the contraction, so V is
//     assumed finite.
//   out^T = V^T P^T: contraction slice j of lane l stands for key 4*(l/16) + j of tile X
//     (j < 4) or of tile Y (j >= 4) in both operands.  P is split into a high and a low part of
//     the storage type, two MFMAs, so that the product is accurate to about 2^-16.
//
// The softmax is the usual running one: per 32 keys the row maximum is refreshed (two
// cross-lane steps), the accumulators and the running sum are rescaled, and the new
// exponentials are taken to base two with log2(e)/sqrt(D) folded into the logit scale.
#include "snapkv_internal.h"

#include <algorithm>
#include <cmath>

namespace snapkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 dbf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 df16x8;
typedef __attribute__((ext_vector_type(4))) float dfx4;
typedef __attribute__((ext_vector_type(2))) _Float16 df16x2;

struct dec_bf16 {};
struct dec_f16 {};

__device__ __forceinline__ dfx4 mma(dec_bf16, uint4 a, uint4 b, dfx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(dbf16x8, a), __builtin_bit_cast(dbf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ dfx4 mma(dec_f16, uint4 a, uint4 b, dfx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(df16x8, a), __builtin_bit_cast(df16x8, b), c, 0, 0, 0);
}

// Two fp32 values that are exactly representable in the storage type, packed (first in the low half).
__device__ __forceinline__ unsigned pack_exact(dec_bf16, float a, float b) {
    return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xFFFF0000u);
}
__device__ __forceinline__ unsigned pack_exact(dec_f16, float a, float b) {
    const df16x2 h = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, h);
}

// p >= 0 split into hi + lo of the storage type (hi by truncation, lo the rounded remainder).
__device__ __forceinline__ void split2(dec_bf16, float a, float b, unsigned& hi, unsigned& lo) {
    const unsigned ua = __float_as_uint(a) & 0xFFFF0000u, ub = __float_as_uint(b) & 0xFFFF0000u;
    hi = (ua >> 16) | ub;
    const float ra = a - __uint_as_float(ua), rb = b - __uint_as_float(ub);
    lo = (__float_as_uint(ra) >> 16) | (__float_as_uint(rb) & 0xFFFF0000u);
}
__device__ __forceinline__ void split2(dec_f16, float a, float b, unsigned& hi, unsigned& lo) {
    const df16x2 h = __builtin_bit_cast(df16x2, __builtin_amdgcn_cvt_pkrtz(a, b));
    hi = __builtin_bit_cast(unsigned, h);
    const float ra = a - (float)h.x, rb = b - (float)h.y;
    lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(ra, rb));
}

template <typename T> __device__ __forceinline__ unsigned one_bits();
template <> __device__ __forceinline__ unsigned one_bits<dec_bf16>() { return 0x3F80u; }
template <> __device__ __forceinline__ unsigned one_bits<dec_f16>() { return 0x3C00u; }

// Selection operand: column n = l%16 of the 32 x 16 matrix that copies contraction element
// 16*half + n.  A lane's slice covers elements 8*(l/16) .. +7.
template <typename T> __device__ __forceinline__ uint4 selector(int lane, int half) {
    const int n = lane & 15, kg = lane >> 4;
    const int e = 16 * half + n - 8 * kg;   // which of this lane's eight elements, if any
    unsigned w[4] = {0u, 0u, 0u, 0u};
    if (e >= 0 && e < 8) w[e >> 1] = one_bits<T>() << (16 * (e & 1));
    return make_uint4(w[0], w[1], w[2], w[3]);
}

struct DecodeArgs {
    const char* q;        // [B, Hq, D]
    const char* k;        // [B, Hkv, cap, D]
    const char* v;
    const int32_t* lens;  // [B] or null
    int64_t S_all;        // valid rows when lens is null
    int64_t cap;
    int Hq, Hkv, g, nsplit;
    float scale2;         // log2(e) / sqrt(D)
    float* out;           // [B, Hq, D]
    float* lse;           // [B, Hq] or null
    float* part_acc;      // [B, Hq, nsplit, D]   (nsplit > 1)
    float2* part_ml;      // [B, Hq, nsplit]
};

constexpr int kDecWaves = 4;   // four or eight waves measure the same; four keeps short caches unsplit

template <typename T, int D>
__global__ __launch_bounds__(kDecWaves * 64) void decode_attn(const DecodeArgs A) {
    constexpr int NP = D / 32;        // 16-byte pieces per lane and row (2-byte elements)
    constexpr int NB = D / 16;        // 16-column blocks of the output
    constexpr int ROW = D * 2;        // bytes per row
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, kg = lane >> 4;
    const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    int64_t S = A.lens ? (int64_t)A.lens[b] : A.S_all;
    S = S < 0 ? 0 : (S > A.cap ? A.cap : S);
    const int64_t npairs = (S + 31) / 32;
    const int64_t pps = (npairs + A.nsplit - 1) / A.nsplit;
    const int64_t p_begin = (int64_t)split * pps;
    const int64_t p_end = p_begin + pps < npairs ? p_begin + pps : npairs;

    const char* kbase = A.k + ((int64_t)b * A.Hkv + kvh) * A.cap * ROW;
    const char* vbase = A.v + ((int64_t)b * A.Hkv + kvh) * A.cap * ROW;

    // the query rows of this KV head: row n16 of the operand is query head kvh*g + n16
    uint4 qf[NP];
#pragma unroll
    for (int c = 0; c < NP; ++c) qf[c] = make_uint4(0, 0, 0, 0);
    if (n16 < A.g) {
        const char* qrow = A.q + ((int64_t)b * A.Hq + (int64_t)kvh * A.g + n16) * ROW;
#pragma unroll
        for (int c = 0; c < NP; ++c) qf[c] = *reinterpret_cast<const uint4*>(qrow + (4 * c + kg) * 16);
    }
    const uint4 sel0 = selector<T>(lane, 0), sel1 = selector<T>(lane, 1);

    float m = -INFINITY, lsum = 0.f;
    dfx4 acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = dfx4{0.f, 0.f, 0.f, 0.f};

    const int64_t last_row = S > 0 ? S - 1 : 0;
    auto row_of = [&](int64_t pair, int tile) {
        const int64_t r = pair * 32 + tile * 16 + n16;
        return r < last_row ? r : last_row;   // rows past the end are read from the last valid row and masked
    };

    // Both operands of a pair are requested one pair ahead into the other of two register sets,
    // so a pair's arithmetic never waits for its own loads.  Every request is unconditional (past
    // the end it repeats an in-range pair), which lets the compiler count the loads in flight.
    struct PairRegs {
        uint4 kx[NP], ky[NP], vx[NP], vy[NP];
    };
    auto request = [&](PairRegs& P, int64_t pr) {
        const int64_t rx = row_of(pr, 0) * ROW, ry = row_of(pr, 1) * ROW;
#pragma unroll
        for (int c = 0; c < NP; ++c) {
            P.kx[c] = *reinterpret_cast<const uint4*>(kbase + rx + (4 * c + kg) * 16);
            P.ky[c] = *reinterpret_cast<const uint4*>(kbase + ry + (4 * c + kg) * 16);
        }
#pragma unroll
        for (int c = 0; c < NP; ++c) {
            P.vx[c] = *reinterpret_cast<const uint4*>(vbase + rx + (4 * c + kg) * 16);
            P.vy[c] = *reinterpret_cast<const uint4*>(vbase + ry + (4 * c + kg) * 16);
        }
        __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the arithmetic that follows
    };
    auto process = [&](const PairRegs& P, int64_t pair) {
        // logits^T: lane (query n16, key group kg) gets keys 4*kg + r of X and of Y
        dfx4 sx = {0.f, 0.f, 0.f, 0.f}, sy = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NP; ++c) {
            sx = mma(T{}, P.kx[c], qf[c], sx);
            sy = mma(T{}, P.ky[c], qf[c], sy);
        }
        const int64_t key0 = pair * 32 + 4 * kg;
        float e[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            e[r] = key0 + r < S ? sx[r] * A.scale2 : -INFINITY;
            e[4 + r] = key0 + 16 + r < S ? sy[r] * A.scale2 : -INFINITY;
            tmax = fmaxf(tmax, fmaxf(e[r], e[4 + r]));
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float mn = fmaxf(m, tmax);            // finite: a pair always holds a valid key
        const float alpha = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mn);
        m = mn;
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            e[j] = __builtin_amdgcn_exp2f(e[j] - mn);
            psum += e[j];
        }
        lsum = lsum * alpha + psum;
        uint4 ph, pl;
        split2(T{}, e[0], e[1], ph.x, pl.x);
        split2(T{}, e[2], e[3], ph.y, pl.y);
        split2(T{}, e[4], e[5], ph.z, pl.z);
        split2(T{}, e[6], e[7], ph.w, pl.w);
#pragma unroll
        for (int i = 0; i < NB; ++i) acc[i] *= alpha;
        // V^T blocks and out^T += V^T P^T
#pragma unroll
        for (int c = 0; c < NP; ++c) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const dfx4 z = {0.f, 0.f, 0.f, 0.f};
                const dfx4 tx = mma(T{}, P.vx[c], half ? sel1 : sel0, z);
                const dfx4 ty = mma(T{}, P.vy[c], half ? sel1 : sel0, z);
                uint4 vt;
                vt.x = pack_exact(T{}, tx[0], tx[1]);
                vt.y = pack_exact(T{}, tx[2], tx[3]);
                vt.z = pack_exact(T{}, ty[0], ty[1]);
                vt.w = pack_exact(T{}, ty[2], ty[3]);
                dfx4 o = acc[2 * c + half];
                o = mma(T{}, vt, ph, o);
                o = mma(T{}, vt, pl, o);
                acc[2 * c + half] = o;
            }
        }
    };
    PairRegs R0, R1;
    int64_t pair = p_begin + wave;
    if (pair < p_end) {
        request(R0, pair);
        for (;;) {
            request(R1, pair + kDecWaves < p_end ? pair + kDecWaves : pair);
            process(R0, pair);
            pair += kDecWaves;
            if (pair >= p_end) break;
            request(R0, pair + kDecWaves < p_end ? pair + kDecWaves : pair);
            process(R1, pair);
            pair += kDecWaves;
            if (pair >= p_end) break;
        }
    }
    lsum += __shfl_xor(lsum, 16);
    lsum += __shfl_xor(lsum, 32);

    // merge the four waves: acc[i][r] of lane (n16, kg) is out[query n16][16*i + 4*kg + r]
    __shared__ float s_acc[kDecWaves][16][D + 4];
    __shared__ float s_m[kDecWaves][16], s_l[kDecWaves][16];
#pragma unroll
    for (int i = 0; i < NB; ++i)
        *reinterpret_cast<float4*>(&s_acc[wave][n16][16 * i + 4 * kg]) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    if (kg == 0) {
        s_m[wave][n16] = m;
        s_l[wave][n16] = lsum;
    }
    __syncthreads();
    constexpr int DT = D / 16;         // head-dim elements per thread in the merge
    const int qi = tid >> 4, d0 = (tid & 15) * DT;
    if (qi < A.g) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) M = fmaxf(M, s_m[w][qi]);
        float Lq = 0.f, o[DT];
#pragma unroll
        for (int d = 0; d < DT; ++d) o[d] = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float mw = s_m[w][qi];
            const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
            Lq += s_l[w][qi] * f;
#pragma unroll
            for (int d = 0; d < DT; ++d) o[d] += s_acc[w][qi][d0 + d] * f;
        }
        const int64_t hq = (int64_t)b * A.Hq + (int64_t)kvh * A.g + qi;
        if (A.nsplit == 1) {
            const float inv = Lq > 0.f ? 1.f / Lq : 0.f;
#pragma unroll
            for (int d = 0; d < DT; ++d) A.out[hq * D + d0 + d] = o[d] * inv;
            if (A.lse && (tid & 15) == 0)
                A.lse[hq] = Lq > 0.f ? (M + __builtin_amdgcn_logf(Lq)) * 0.6931471805599453f : -INFINITY;
        } else {
            float* pa = A.part_acc + (hq * A.nsplit + split) * D;
#pragma unroll
            for (int d = 0; d < DT; ++d) pa[d0 + d] = o[d];
            if ((tid & 15) == 0) A.part_ml[hq * A.nsplit + split] = make_float2(M, Lq);
        }
    }
}

// Merges the partials of the splits of one query head: one workgroup of D threads per head.
template <int D>
__global__ __launch_bounds__(D) void decode_merge(const float* part_acc, const float2* part_ml, int nsplit,
                                                  float* out, float* lse) {
    const int64_t hq = blockIdx.x;
    const int d = threadIdx.x;
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part_ml[hq * nsplit + s].x);
    float Lq = 0.f, o = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float2 ml = part_ml[hq * nsplit + s];
        const float f = ml.x == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ml.x - M);
        Lq += ml.y * f;
        o += part_acc[(hq * nsplit + s) * D + d] * f;
    }
    out[hq * D + d] = Lq > 0.f ? o / Lq : 0.f;
    if (lse && d == 0) lse[hq] = Lq > 0.f ? (M + __builtin_amdgcn_logf(Lq)) * 0.6931471805599453f : -INFINITY;
}

int cu_count() {
    static int cus = -1;
    if (cus < 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            return 256;
        cus = n;
    }
    return cus;
}

}  // namespace

// Splits of a (sequence, KV head) pair's keys.  Measured: long-running workgroups, about one per
// compute unit, stream best, so the keys are split only when the pairs alone leave units idle,
// and never below 128 keys per wave.
int decode_splits(int B, int Hkv, int64_t S) {
    const int64_t pairs = (int64_t)B * Hkv;
    const int64_t want = (cu_count() + pairs / 2) / pairs;
    const int64_t most = std::max<int64_t>(1, S / (128 * kDecWaves));
    return (int)std::max<int64_t>(1, std::min<int64_t>(std::min(want, most), 64));
}

size_t decode_scratch_bytes(int B, int Hq, int D, int nsplit) {
    if (nsplit <= 1) return 0;
    const size_t heads = (size_t)B * Hq;
    return ((heads * nsplit * D * sizeof(float) + 255) & ~(size_t)255) + heads * nsplit * sizeof(float2);
}

hipError_t launch_decode(int dtype, int D, const void* q, const void* k, const void* v, const int32_t* lens,
                         int B, int Hq, int Hkv, int64_t S, int64_t cap, int nsplit, void* scratch,
                         float* out, float* lse, hipStream_t st) {
    DecodeArgs A;
    A.q = static_cast<const char*>(q);
    A.k = static_cast<const char*>(k);
    A.v = static_cast<const char*>(v);
    A.lens = lens;
    A.S_all = S;
    A.cap = cap;
    A.Hq = Hq;
    A.Hkv = Hkv;
    A.g = Hq / Hkv;
    A.nsplit = nsplit;
    A.scale2 = (float)(1.4426950408889634 / std::sqrt((double)D));
    A.out = out;
    A.lse = lse;
    A.part_acc = nullptr;
    A.part_ml = nullptr;
    if (nsplit > 1) {
        const size_t heads = (size_t)B * Hq;
        A.part_acc = static_cast<float*>(scratch);
        A.part_ml = reinterpret_cast<float2*>(static_cast<char*>(scratch) +
                                              ((heads * nsplit * D * sizeof(float) + 255) & ~(size_t)255));
    }
    const dim3 grid(nsplit, Hkv, B), block(kDecWaves * 64);
    if (dtype == 0 && D == 128) hipLaunchKernelGGL((decode_attn<dec_bf16, 128>), grid, block, 0, st, A);
    else if (dtype == 0 && D == 64) hipLaunchKernelGGL((decode_attn<dec_bf16, 64>), grid, block, 0, st, A);
    else if (dtype == 2 && D == 128) hipLaunchKernelGGL((decode_attn<dec_f16, 128>), grid, block, 0, st, A);
    else if (dtype == 2 && D == 64) hipLaunchKernelGGL((decode_attn<dec_f16, 64>), grid, block, 0, st, A);
    else return hipErrorInvalidValue;
    if (nsplit > 1) {
        const unsigned heads = (unsigned)((int64_t)B * Hq);
        if (D == 128) hipLaunchKernelGGL((decode_merge<128>), dim3(heads), dim3(128), 0, st, A.part_acc, A.part_ml, nsplit, out, lse);
        else hipLaunchKernelGGL((decode_merge<64>), dim3(heads), dim3(64), 0, st, A.part_acc, A.part_ml, nsplit, out, lse);
    }
    return hipGetLastError();
}

}  // namespace snapkv
