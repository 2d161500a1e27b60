// Hit rate of the voting (Sec. 4, "Hit Rate", Eq. 3-7): of the prefix positions that the query of
// a generated token attends to above a threshold, how many had the voting kept.  A quality probe,
// not part of the compression path.
//
//   hit_logits:  one pass over K.  Logits of the g query heads of a KV head against 16 keys per
//                MFMA tile (16x16x32, the layout of the decoding step: lane l holds query head l%16
//                and keys 4*(l/16) + r of the tile); the logits go to a scratch row per query head in
//                the base-2 domain, and every workgroup leaves its (max, sum 2^(s - max)) per head.
//   hit_count:   per query head and chunk of prefix positions: the head's log-sum-exp from those
//                partials, A_cur = 2^(s - lse) > theta, membership of the position in the head's
//                ascending selection by binary search, integer counts added with atomics.
// The counts are integers; only the comparison with theta depends on fp32 rounding.
#include "snapkv_internal.h"

#include <algorithm>
#include <cmath>

namespace snapkv {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 hbf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 hf16x8;
typedef __attribute__((ext_vector_type(4))) float hfx4;

struct hr_bf16 {};
struct hr_f16 {};
__device__ __forceinline__ hfx4 hmma(hr_bf16, uint4 a, uint4 b, hfx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(hbf16x8, a), __builtin_bit_cast(hbf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ hfx4 hmma(hr_f16, uint4 a, uint4 b, hfx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(hf16x8, a), __builtin_bit_cast(hf16x8, b), c, 0, 0, 0);
}

constexpr int kHrWaves = 4;

struct HitArgs {
    const char* q;       // [Hq, D]
    const char* k;       // [Hkv, Lk, D]
    int64_t Lk, pitch;   // keys; floats per logits row (Lk rounded up to whole 16-key tiles)
    int Hq, g, nblk;
    float scale2;
    float* logits;       // [Hq][pitch] base-2 logits
    float2* part;        // [Hq][nblk] (max, sum) per workgroup
    int32_t* counts;     // [Hq][2], zeroed here for hit_count
};

template <typename T, int D>
__global__ __launch_bounds__(kHrWaves * 64) void hit_logits(const HitArgs A) {
    constexpr int NP = D / 32, ROW = D * 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, kg = lane >> 4;
    const int blk = blockIdx.x, kvh = blockIdx.y;
    if (blk == 0 && kvh == 0)
        for (int i = tid; i < 2 * A.Hq; i += kHrWaves * 64) A.counts[i] = 0;
    const int64_t ntiles = (A.Lk + 15) / 16;
    const int64_t per = (ntiles + A.nblk - 1) / A.nblk;
    const int64_t t_begin = (int64_t)blk * per;
    const int64_t t_end = t_begin + per < ntiles ? t_begin + per : ntiles;
    const char* kbase = A.k + (int64_t)kvh * A.Lk * ROW;
    uint4 qf[NP];
#pragma unroll
    for (int c = 0; c < NP; ++c) qf[c] = make_uint4(0, 0, 0, 0);
    const int hq = kvh * A.g + n16;
    if (n16 < A.g) {
        const char* qrow = A.q + (int64_t)hq * ROW;
#pragma unroll
        for (int c = 0; c < NP; ++c) qf[c] = *reinterpret_cast<const uint4*>(qrow + (4 * c + kg) * 16);
    }
    float m = -INFINITY, l = 0.f;
    for (int64_t t = t_begin + wave; t < t_end; t += kHrWaves) {
        int64_t row = t * 16 + n16;
        row = row < A.Lk ? row : A.Lk - 1;   // rows past the end repeat the last row and are masked
        const char* rp = kbase + row * ROW;
        hfx4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NP; ++c)
            s = hmma(T{}, *reinterpret_cast<const uint4*>(rp + (4 * c + kg) * 16), qf[c], s);
        const int64_t key0 = t * 16 + 4 * kg;
        float e[4];
        float tm = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            e[r] = key0 + r < A.Lk ? s[r] * A.scale2 : -INFINITY;
            tm = fmaxf(tm, e[r]);
        }
        if (n16 < A.g)   // a row holds whole tiles and key0 is a multiple of four: an aligned 16-byte store inside the row
            *reinterpret_cast<float4*>(A.logits + (int64_t)hq * A.pitch + key0) = make_float4(e[0], e[1], e[2], e[3]);
        if (tm > -INFINITY) {
            const float mn = fmaxf(m, tm);
            float add = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) add += __builtin_amdgcn_exp2f(e[r] - mn);
            l = (m == -INFINITY ? 0.f : l * __builtin_amdgcn_exp2f(m - mn)) + add;
            m = mn;
        }
    }
    // merge the four key groups of a query head, then the waves
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float pm = __shfl_xor(m, off), pl = __shfl_xor(l, off);
        const float mn = fmaxf(m, pm);
        if (mn > -INFINITY) {
            l = (m == -INFINITY ? 0.f : l * __builtin_amdgcn_exp2f(m - mn)) +
                (pm == -INFINITY ? 0.f : pl * __builtin_amdgcn_exp2f(pm - mn));
            m = mn;
        }
    }
    __shared__ float sm[kHrWaves][16], sl[kHrWaves][16];
    if (kg == 0) {
        sm[wave][n16] = m;
        sl[wave][n16] = l;
    }
    __syncthreads();
    if (tid < A.g) {
        float M = -INFINITY, Ls = 0.f;
#pragma unroll
        for (int w = 0; w < kHrWaves; ++w) M = fmaxf(M, sm[w][tid]);
#pragma unroll
        for (int w = 0; w < kHrWaves; ++w)
            if (sm[w][tid] > -INFINITY) Ls += sl[w][tid] * __builtin_amdgcn_exp2f(sm[w][tid] - M);
        A.part[(int64_t)(kvh * A.g + tid) * A.nblk + blk] = make_float2(M, Ls);
    }
}

struct CountArgs {
    const float* logits;
    const float2* part;
    int64_t pitch, n, kcount, idx_stride;
    int nblk, idx_div;      // query heads per row of idx
    const int32_t* idx;     // [Hq / idx_div][idx_stride], the first kcount of a row ascending
    float theta;
    int32_t* counts;
};

constexpr int kCountThreads = 256;
constexpr int kCountChunk = 8192;   // prefix positions per workgroup

__global__ __launch_bounds__(kCountThreads) void hit_count(const CountArgs A) {
    const int tid = threadIdx.x, hq = blockIdx.y;
    __shared__ float red[kCountThreads];
    __shared__ int ired[2][kCountThreads / 64];
    // the head's log-sum-exp (base 2) from the workgroups' partials
    float M = -INFINITY;
    for (int i = tid; i < A.nblk; i += kCountThreads) M = fmaxf(M, A.part[(int64_t)hq * A.nblk + i].x);
    red[tid] = M;
    __syncthreads();
    for (int s = kCountThreads / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] = fmaxf(red[tid], red[tid + s]);
        __syncthreads();
    }
    M = red[0];
    __syncthreads();
    float Ls = 0.f;
    for (int i = tid; i < A.nblk; i += kCountThreads) {
        const float2 p = A.part[(int64_t)hq * A.nblk + i];
        if (p.x > -INFINITY) Ls += p.y * __builtin_amdgcn_exp2f(p.x - M);
    }
    red[tid] = Ls;
    __syncthreads();
    for (int s = kCountThreads / 2; s > 0; s >>= 1) {   // a fixed tree: the same sum in every workgroup of the head
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    const float lse2 = M + __builtin_amdgcn_logf(red[0]);
    const int32_t* sel = A.idx + (int64_t)(hq / A.idx_div) * A.idx_stride;
    const float* row = A.logits + (int64_t)hq * A.pitch;
    const int64_t j0 = (int64_t)blockIdx.x * kCountChunk;
    const int64_t j1 = j0 + kCountChunk < A.n ? j0 + kCountChunk : A.n;
    int imp = 0, hit = 0;
    for (int64_t j = j0 + tid; j < j1; j += kCountThreads) {
        const float a = __builtin_amdgcn_exp2f(row[j] - lse2);
        if (a > A.theta) {
            ++imp;
            int64_t lo = 0, hi = A.kcount;   // first entry >= j of the ascending selection
            while (lo < hi) {
                const int64_t mid = (lo + hi) >> 1;
                if (sel[mid] < j) lo = mid + 1; else hi = mid;
            }
            if (lo < A.kcount && sel[lo] == j) ++hit;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        imp += __shfl_xor(imp, off);
        hit += __shfl_xor(hit, off);
    }
    if ((tid & 63) == 0) {
        ired[0][tid >> 6] = imp;
        ired[1][tid >> 6] = hit;
    }
    __syncthreads();
    if (tid == 0) {
        int a = 0, b = 0;
        for (int w = 0; w < kCountThreads / 64; ++w) {
            a += ired[0][w];
            b += ired[1][w];
        }
        if (a) atomicAdd(&A.counts[2 * hq], a);
        if (b) atomicAdd(&A.counts[2 * hq + 1], b);
    }
}

}  // namespace

static int hit_blocks(int64_t Lk) {
    const int64_t ntiles = (Lk + 15) / 16;
    return (int)std::max<int64_t>(1, std::min<int64_t>(ntiles / (4 * kHrWaves), 256));
}

size_t hit_rate_scratch_bytes(int Hq, int64_t Lk) {
    const size_t pitch = ((size_t)Lk + 15) & ~(size_t)15;
    return ((sizeof(float) * Hq * pitch + 255) & ~(size_t)255) + sizeof(float2) * (size_t)Hq * hit_blocks(Lk);
}

hipError_t launch_hit_rate(int dtype, int D, const void* q, const void* k, int64_t Lk, int64_t n, int Hq, int Hkv,
                           const int32_t* idx, int Hidx, int64_t kcount, int64_t idx_stride, float theta,
                           void* scratch, int32_t* counts, hipStream_t st) {
    HitArgs A;
    A.q = static_cast<const char*>(q);
    A.k = static_cast<const char*>(k);
    A.Lk = Lk;
    A.pitch = (Lk + 15) & ~(int64_t)15;
    A.Hq = Hq;
    A.g = Hq / Hkv;
    A.nblk = hit_blocks(Lk);
    A.scale2 = (float)(1.4426950408889634 / std::sqrt((double)D));
    A.logits = static_cast<float*>(scratch);
    A.part = reinterpret_cast<float2*>(static_cast<char*>(scratch) + ((sizeof(float) * Hq * (size_t)A.pitch + 255) & ~(size_t)255));
    A.counts = counts;
    const dim3 grid(A.nblk, Hkv), block(kHrWaves * 64);
    if (dtype == 0 && D == 128) hipLaunchKernelGGL((hit_logits<hr_bf16, 128>), grid, block, 0, st, A);
    else if (dtype == 0 && D == 64) hipLaunchKernelGGL((hit_logits<hr_bf16, 64>), grid, block, 0, st, A);
    else if (dtype == 2 && D == 128) hipLaunchKernelGGL((hit_logits<hr_f16, 128>), grid, block, 0, st, A);
    else if (dtype == 2 && D == 64) hipLaunchKernelGGL((hit_logits<hr_f16, 64>), grid, block, 0, st, A);
    else return hipErrorInvalidValue;
    if (n > 0) {
        CountArgs C;
        C.logits = A.logits;
        C.part = A.part;
        C.pitch = A.pitch;
        C.n = n;
        C.kcount = kcount;
        C.idx_stride = idx_stride;
        C.nblk = A.nblk;
        C.idx_div = Hq / Hidx;
        C.idx = idx;
        C.theta = theta;
        C.counts = counts;
        hipLaunchKernelGGL(hit_count, dim3((unsigned)((n + kCountChunk - 1) / kCountChunk), Hq), dim3(kCountThreads), 0, st, C);
    }
    return hipGetLastError();
}

}  // namespace snapkv
