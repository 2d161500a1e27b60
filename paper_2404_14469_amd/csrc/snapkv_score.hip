// Window scoring and voting (Listing 1: the compute_attn call and the column sum; Eq. 1).
//
// For one KV head the g*W observation-window queries form the M side of an MFMA product with
// the keys on the N side: S = Q_win * K^T, bf16 (or fp32) in, fp32 accumulate.  A wave owns one
// 32-row block of queries and a chunk of kChunkKeys keys.  Softmax needs every row's
// normaliser over all L keys before a probability can be summed down a column, so the work is
// split in two passes over the keys:
//   pass 1: per (chunk, row) the row maximum and sum of exponentials of the chunk,
//   reduce: per row the global maximum and 1 / sum of exponentials,
//   pass 2: recompute the chunk's logits, normalise, sum over the window rows of each query
//           head (the vote of Eq. 1) and store it for prefix columns.
// Logits live in the base-2 domain (scaled by log2(e)/sqrt(D)) so v_exp_f32 applies directly.
//
// MFMA operand layout (32x32 shapes, 64 lanes): lane l supplies row/column l%32 and the
// contraction slice l/32; accumulator register r of lane l is row (r/4)*8 + (l/32)*4 + r%4,
// column l%32.  A lane therefore loads half of one Q row and half of one K row, contiguous in
// memory; which head-dim elements go into which MFMA step is irrelevant as long as Q and K
// agree, so the natural memory order is used.
#include "snapkv_internal.h"

namespace snapkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct bf16_tag {};
struct f16_tag {};
struct f32_tag {};
template <typename T> struct elem_size;
template <> struct elem_size<bf16_tag> { static constexpr int value = 2; };
template <> struct elem_size<f16_tag> { static constexpr int value = 2; };
template <> struct elem_size<f32_tag> { static constexpr int value = 4; };

// Half a row of D elements as 16-byte pieces.
template <typename T, int D> struct Frag {
    static constexpr int N16 = (D / 2) * elem_size<T>::value / 16;
    uint4 v[N16];
};

template <typename T, int D>
__device__ __forceinline__ void load_frag(Frag<T, D>& f, const void* row_base, int kh) {
    const uint4* p = reinterpret_cast<const uint4*>(static_cast<const char*>(row_base) +
                                                    kh * (D / 2) * elem_size<T>::value);
#pragma unroll
    for (int s = 0; s < Frag<T, D>::N16; ++s) f.v[s] = p[s];
}

template <typename T, int D> __device__ __forceinline__ void zero_frag(Frag<T, D>& f) {
#pragma unroll
    for (int s = 0; s < Frag<T, D>::N16; ++s) f.v[s] = make_uint4(0, 0, 0, 0);
}

template <int D>
__device__ __forceinline__ void mfma_rows(const Frag<bf16_tag, D>& a, const Frag<bf16_tag, D>& b,
                                          f32x16& acc) {
#pragma unroll
    for (int s = 0; s < Frag<bf16_tag, D>::N16; ++s) {
        bf16x8 av = __builtin_bit_cast(bf16x8, a.v[s]);
        bf16x8 bv = __builtin_bit_cast(bf16x8, b.v[s]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
    }
}

template <int D>
__device__ __forceinline__ void mfma_rows(const Frag<f16_tag, D>& a, const Frag<f16_tag, D>& b,
                                          f32x16& acc) {
#pragma unroll
    for (int s = 0; s < Frag<f16_tag, D>::N16; ++s) {
        f16x8 av = __builtin_bit_cast(f16x8, a.v[s]);
        f16x8 bv = __builtin_bit_cast(f16x8, b.v[s]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc, 0, 0, 0);
    }
}

template <int D>
__device__ __forceinline__ void mfma_rows(const Frag<f32_tag, D>& a, const Frag<f32_tag, D>& b,
                                          f32x16& acc) {
#pragma unroll
    for (int s = 0; s < Frag<f32_tag, D>::N16; ++s) {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[s].x), __uint_as_float(b.v[s].x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[s].y), __uint_as_float(b.v[s].y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[s].z), __uint_as_float(b.v[s].z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[s].w), __uint_as_float(b.v[s].w), acc, 0, 0, 0);
    }
}

// Which (query head within the group, window row) a row of a 32-row block is; i >= W or
// head >= g marks a padding row.
__device__ __forceinline__ void row_to_head(const ScoreGeom& G, int rb, int row, int& head, int& i) {
    if (G.mode16) {
        head = 2 * rb + (row >> 4);
        i = row & 15;
    } else {
        head = rb / G.BH;
        i = (rb % G.BH) * 32 + row;
    }
}

struct Task {
    int hkv, chunk, rb;
    bool valid;
};

__device__ __forceinline__ Task decode_task(const ScoreGeom& G) {
    Task t;
    const int64_t id = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t total = (int64_t)G.Hkv * G.nchunks * G.R32;
    t.valid = id < total;
    t.rb = (int)(id % G.R32);
    const int64_t r = id / G.R32;
    t.chunk = (int)(r % G.nchunks);
    t.hkv = (int)(r / G.nchunks);
    return t;
}

template <typename T, int D>
__device__ __forceinline__ void load_q_block(Frag<T, D>& qf, const void* q, const ScoreGeom& G,
                                             const Task& t, int lane) {
    int head, i;
    row_to_head(G, t.rb, lane & 31, head, i);
    if (head < G.g && i < G.W) {
        const int64_t row = ((int64_t)(t.hkv * G.g + head) * G.W + i);
        load_frag<T, D>(qf, static_cast<const char*>(q) + row * D * elem_size<T>::value, lane >> 5);
    } else {
        zero_frag<T, D>(qf);
    }
}

// Logits of the wave's chunk: acc[t] is the 32x32 tile of keys [j0 + 32t, j0 + 32t + 32).
// Rows past the end of the prompt are clamped to the last key (finite values, masked later).
template <typename T, int D>
__device__ __forceinline__ void chunk_logits(f32x16 (&acc)[kTilesPerChunk], const Frag<T, D>& qf,
                                             const void* k, const ScoreGeom& G, const Task& t,
                                             int lane) {
    const int64_t j0 = (int64_t)t.chunk * kChunkKeys;
    const char* kbase = static_cast<const char*>(k) + (int64_t)t.hkv * G.k_hs;
    Frag<T, D> kf[kTilesPerChunk];
#pragma unroll
    for (int tt = 0; tt < kTilesPerChunk; ++tt) {
        int64_t j = j0 + tt * kTileKeys + (lane & 31);
        j = j < G.L ? j : G.L - 1;
        j = physical_row(G.k_table, G.k_page, G.k_pages, j);
        load_frag<T, D>(kf[tt], kbase + j * G.k_rs, lane >> 5);
    }
#pragma unroll
    for (int tt = 0; tt < kTilesPerChunk; ++tt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[tt][r] = 0.f;
        mfma_rows<D>(qf, kf[tt], acc[tt]);
    }
}

__device__ __forceinline__ float wave32_max(float x) {
#pragma unroll
    for (int m = 1; m < 32; m <<= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
    return x;
}
__device__ __forceinline__ float wave32_sum(float x) {
#pragma unroll
    for (int m = 1; m < 32; m <<= 1) x += __shfl_xor(x, m, 64);
    return x;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void score_pass1(const void* __restrict__ q,
                                                   const void* __restrict__ k,
                                                   float2* __restrict__ part, const ScoreGeom G) {
    const Task t = decode_task(G);
    if (!t.valid) return;
    const int lane = threadIdx.x & 63;
    const int kh = lane >> 5;
    Frag<T, D> qf;
    load_q_block<T, D>(qf, q, G, t, lane);
    f32x16 acc[kTilesPerChunk];
    chunk_logits<T, D>(acc, qf, k, G, t, lane);

    const int64_t j0 = (int64_t)t.chunk * kChunkKeys;
    const bool boundary = j0 + kChunkKeys > G.n;   // chunk touches window columns or the tail
    float mx[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) mx[r] = -INFINITY;
#pragma unroll
    for (int tt = 0; tt < kTilesPerChunk; ++tt) {
        const int64_t j = j0 + tt * kTileKeys + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float s = acc[tt][r] * G.c2;
            if (boundary) {
                int head, i;
                row_to_head(G, t.rb, (r >> 2) * 8 + kh * 4 + (r & 3), head, i);
                if (j > G.n + i || j >= G.L) s = -INFINITY;     // causal mask of the prompt phase
            }
            acc[tt][r] = s;
            mx[r] = fmaxf(mx[r], s);
        }
    }
    float zs[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        mx[r] = wave32_max(mx[r]);
        const float ref = mx[r] == -INFINITY ? 0.f : mx[r];
        float z = 0.f;
#pragma unroll
        for (int tt = 0; tt < kTilesPerChunk; ++tt) z += __builtin_amdgcn_exp2f(acc[tt][r] - ref);
        zs[r] = wave32_sum(z);
    }
    if ((lane & 31) == 0) {
        float2* dst = part + (((int64_t)t.hkv * G.nchunks + t.chunk) * G.R32 + t.rb) * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[(r >> 2) * 8 + kh * 4 + (r & 3)] = make_float2(mx[r], zs[r]);
    }
}

// Per row: merge the chunks' (max, sum-exp) pairs in a fixed order into (max, 1/sum).
__global__ __launch_bounds__(256) void reduce_rows(const float2* __restrict__ part,
                                                   float2* __restrict__ mz, const ScoreGeom G) {
    const int rb = blockIdx.x, hkv = blockIdx.y;
    const int row = threadIdx.x & 31, cl = threadIdx.x >> 5;
    float m = -INFINITY, z = 0.f;
    for (int c = cl; c < G.nchunks; c += 8) {
        const float2 pc = part[(((int64_t)hkv * G.nchunks + c) * G.R32 + rb) * 32 + row];
        const float nm = fmaxf(m, pc.x);
        if (nm != -INFINITY) {
            z = z * __builtin_amdgcn_exp2f(m - nm) + pc.y * __builtin_amdgcn_exp2f(pc.x - nm);
            m = nm;
        }
    }
    __shared__ float2 sh[8][32];
    sh[cl][row] = make_float2(m, z);
    __syncthreads();
    if (cl == 0) {
        for (int c = 1; c < 8; ++c) {
            const float2 pc = sh[c][row];
            const float nm = fmaxf(m, pc.x);
            if (nm != -INFINITY) {
                z = z * __builtin_amdgcn_exp2f(m - nm) + pc.y * __builtin_amdgcn_exp2f(pc.x - nm);
                m = nm;
            }
        }
        int head, i;
        row_to_head(G, rb, row, head, i);
        const bool real = head < G.g && i < G.W && z > 0.f;
        mz[((int64_t)hkv * G.R32 + rb) * 32 + row] = real ? make_float2(m, 1.0f / z) : make_float2(0.f, 0.f);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void score_pass2(const void* __restrict__ q,
                                                   const void* __restrict__ k,
                                                   const float2* __restrict__ mz,
                                                   float* __restrict__ vote, const ScoreGeom G) {
    const Task t = decode_task(G);
    if (!t.valid) return;
    const int64_t j0 = (int64_t)t.chunk * kChunkKeys;
    if (j0 >= G.n) return;                       // window-only chunk: no prefix column to vote on
    const int lane = threadIdx.x & 63;
    const int kh = lane >> 5;
    Frag<T, D> qf;
    load_q_block<T, D>(qf, q, G, t, lane);
    f32x16 acc[kTilesPerChunk];
    chunk_logits<T, D>(acc, qf, k, G, t, lane);

    float m2[16], iz[16];
    const float2* mzb = mz + ((int64_t)t.hkv * G.R32 + t.rb) * 32;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float2 x = mzb[(r >> 2) * 8 + kh * 4 + (r & 3)];
        m2[r] = x.x;
        iz[r] = x.y;
    }
    float* vbase = vote + (int64_t)t.hkv * G.NV * G.n;
#pragma unroll
    for (int tt = 0; tt < kTilesPerChunk; ++tt) {
        float lo = 0.f, hi = 0.f;                // rows 0-15 and rows 16-31 of the block
#pragma unroll
        for (int r = 0; r < 8; ++r)
            lo += __builtin_amdgcn_exp2f(fmaf(acc[tt][r], G.c2, -m2[r])) * iz[r];
#pragma unroll
        for (int r = 8; r < 16; ++r)
            hi += __builtin_amdgcn_exp2f(fmaf(acc[tt][r], G.c2, -m2[r])) * iz[r];
        lo += __shfl_xor(lo, 32, 64);
        hi += __shfl_xor(hi, 32, 64);
        const int64_t j = j0 + tt * kTileKeys + (lane & 31);
        if (j < G.n) {
            if (G.mode16) {
                const int head = 2 * t.rb + kh;  // lanes 0-31 store the first head, 32-63 the second
                if (head < G.g) vbase[(int64_t)head * G.n + j] = kh ? hi : lo;
            } else if (kh == 0) {
                vbase[(int64_t)t.rb * G.n + j] = lo + hi;
            }
        }
    }
}

ScoreGeom make_geom(int64_t L, int Hq, int Hkv, int D, int W) {
    ScoreGeom G;
    G.L = L;
    G.n = L - W;
    G.W = W;
    G.g = Hq / Hkv;
    G.Hkv = Hkv;
    G.mode16 = W <= 16 ? 1 : 0;
    G.BH = (W + 31) / 32;
    G.R32 = G.mode16 ? (G.g + 1) / 2 : G.g * G.BH;
    G.VB = G.mode16 ? 1 : G.BH;
    G.NV = G.g * G.VB;
    G.nchunks = (int)((L + kChunkKeys - 1) / kChunkKeys);
    G.c2 = (float)(1.4426950408889634 / __builtin_sqrt((double)D));
    G.k_rs = 0;   // set by the caller once the element size is known
    G.k_hs = 0;
    G.vpitch = G.n;
    G.k_table = nullptr;
    G.k_page = 1;
    G.k_pages = 0;
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
    const size_t part = align_up(sizeof(float2) * (size_t)G.Hkv * G.nchunks * G.R32 * 32);
    const size_t mz = align_up(sizeof(float2) * (size_t)G.Hkv * G.R32 * 32);
    const size_t vote = align_up(sizeof(float) * (size_t)G.Hkv * G.NV * (size_t)(G.n > 0 ? G.n : 1));
    const size_t score = align_up(sizeof(float) * (size_t)Hsel * (size_t)(G.n > 0 ? G.n : 1));
    const size_t stat = stream_stat_bytes(G);
    const size_t lse = align_up(sizeof(float) * (size_t)G.Hkv * G.g * G.W);
    const size_t logit = long_logit_bytes(G);
    const size_t off = counters + fused;
    if (ws) {
        ws->status_flag = reinterpret_cast<unsigned*>(base);
        ws->fused = b + counters;
        ws->part = reinterpret_cast<float2*>(b + off);
        ws->mz = reinterpret_cast<float2*>(b + off + part);
        ws->vote = reinterpret_cast<float*>(b + off + part + mz);
        ws->score = reinterpret_cast<float*>(b + off + part + mz + vote);
        ws->stat_part = reinterpret_cast<float2*>(b + off + part + mz + vote + score);
        ws->lse = reinterpret_cast<float*>(b + off + part + mz + vote + score + stat);
        ws->long_logit = logit ? reinterpret_cast<float*>(b + off + part + mz + vote + score + stat + lse) : nullptr;
        ws->long_logit_bytes = logit;
    }
    const size_t sel = select_layout(Hsel, G.n, ws ? &ws->sel : nullptr,
                                     ws ? b + off + part + mz + vote + score + stat + lse + logit : nullptr, false,
                                     ws ? b : nullptr);
    if (ws) ws->sel.ps_flag = ws->status_flag;
    return kHeader + off + part + mz + vote + score + stat + lse + logit + sel;
}

template <typename T, int D>
static hipError_t launch_score_t(const void* q, const void* k, const ScoreGeom& G,
                                 const Workspace& ws, hipStream_t st) {
    const int64_t tasks = (int64_t)G.Hkv * G.nchunks * G.R32;
    const unsigned blocks = (unsigned)((tasks + 3) / 4);
    hipLaunchKernelGGL((score_pass1<T, D>), dim3(blocks), dim3(256), 0, st, q, k, ws.part, G);
    stage_done(st, kStagePass1);
    hipLaunchKernelGGL(reduce_rows, dim3(G.R32, G.Hkv), dim3(256), 0, st, ws.part, ws.mz, G);
    stage_done(st, kStageReduce);
    hipLaunchKernelGGL((score_pass2<T, D>), dim3(blocks), dim3(256), 0, st, q, k, ws.mz, ws.vote, G);
    stage_done(st, kStagePass2);
    return hipGetLastError();
}

hipError_t launch_score(int dtype, int D, const void* q, const void* k, const ScoreGeom& G,
                        const Workspace& ws, hipStream_t st) {
    if (G.n <= 0) return hipSuccess;
    if (dtype == 0) {
        if (D == 128) return launch_score_t<bf16_tag, 128>(q, k, G, ws, st);
        if (D == 64) return launch_score_t<bf16_tag, 64>(q, k, G, ws, st);
    } else if (dtype == 2) {
        if (D == 128) return launch_score_t<f16_tag, 128>(q, k, G, ws, st);
        if (D == 64) return launch_score_t<f16_tag, 64>(q, k, G, ws, st);
    } else {
        if (D == 128) return launch_score_t<f32_tag, 128>(q, k, G, ws, st);
        if (D == 64) return launch_score_t<f32_tag, 64>(q, k, G, ws, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace snapkv
