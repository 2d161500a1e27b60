// Pooling + group sum (Sec. 4.3; Listing 1, the pool1d call) as a kernel of its own, and the gather of the
// kept rows (Listing 1, the two gathers and concatenations).  The top-k selection is in snapkv_topk.hip.
#include "snapkv_internal.h"
#include <type_traits>

namespace snapkv {

// ------------------------------------------------------------------------------------------
// Pooling.  One workgroup produces kPoolTile consecutive scores of one KV head; a thread owns
// positions tile + t, tile + t + 256, ... so that every load and store is lane-contiguous.  For
// each query head of the group the 2*(p/2)+1 taps of a position are read straight from the
// head's votes (neighbouring lanes read neighbouring words, so the taps are L1 hits), pooled,
// and added to the running group sum in head order.  Max pooling ignores positions outside
// [0, n); average pooling counts them as zeros and divides by p.
// ------------------------------------------------------------------------------------------
constexpr int kPoolTile = 1024;
constexpr int kPoolPerThread = kPoolTile / 256;

// P > 0: pooling width known at compile time (taps unrolled, their loads issued together);
// P == 0: width taken from the argument p.
template <int P>
__global__ __launch_bounds__(256) void pool_group(const float* __restrict__ vote,
                                                  float* __restrict__ score, const ScoreGeom G,
                                                  const int pool_kind, const int p_arg,
                                                  unsigned* __restrict__ minmax) {
    __shared__ unsigned sh_lo[4], sh_hi[4];
    const int hkv = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * kPoolTile;
    const int p = P > 0 ? P : p_arg;
    const int r = p >> 1;
    const float pad = pool_kind == 0 ? -INFINITY : 0.f;
    float acc[kPoolPerThread];
#pragma unroll
    for (int e = 0; e < kPoolPerThread; ++e) acc[e] = 0.f;
    for (int h = 0; h < G.g; ++h) {
        const float* vb = vote + ((int64_t)hkv * G.NV + (int64_t)h * G.VB) * G.n;
#pragma unroll
        for (int e = 0; e < kPoolPerThread; ++e) {
            const int64_t j = t0 + threadIdx.x + e * 256;
            if (j >= G.n) continue;
            float val;
            if (P > 0 && G.VB == 1) {
                float tap[P > 0 ? P : 1];
#pragma unroll
                for (int d = 0; d < P; ++d) {
                    const int64_t x = j + d - P / 2;
                    tap[d] = (x >= 0 && x < G.n) ? vb[x] : pad;
                }
                val = tap[0];
#pragma unroll
                for (int d = 1; d < P; ++d) val = pool_kind == 0 ? fmaxf(val, tap[d]) : val + tap[d];
            } else {
                val = pad;
                for (int d = -r; d <= r; ++d) {
                    const int64_t x = j + d;
                    float tap = pad;
                    if (x >= 0 && x < G.n) {
                        tap = vb[x];
                        for (int b = 1; b < G.VB; ++b) tap += vb[(int64_t)b * G.n + x];
                    }
                    val = d == -r ? tap : (pool_kind == 0 ? fmaxf(val, tap) : val + tap);
                }
            }
            if (pool_kind != 0) val = val / (float)p;
            acc[e] += val;
        }
    }
    unsigned lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int e = 0; e < kPoolPerThread; ++e) {
        const int64_t j = t0 + threadIdx.x + e * 256;
        if (j < G.n) {
            score[(int64_t)hkv * G.n + j] = acc[e];
            const unsigned x = __float_as_uint(acc[e]);
            lo = x < lo ? x : lo;
            hi = x > hi ? x : hi;
        }
    }
    if (minmax) {   // range of this tile's score bit patterns, for the selection that follows
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
            unsigned* mm = minmax + 2 * ((int64_t)hkv * gridDim.x + blockIdx.x);
            mm[0] = lo;
            mm[1] = hi;
        }
    }
}

// Variant for rows whose length is a multiple of four (so that every row is 16-byte aligned): a thread owns four consecutive positions and reads them and their
// taps as float4, an order of magnitude fewer instructions per position.  The first and last
// tiles of a row take the element-wise path.
template <int P>
__global__ __launch_bounds__(256) void pool_group4(const float* __restrict__ vote,
                                                   float* __restrict__ score, const ScoreGeom G,
                                                   const int pool_kind, unsigned* __restrict__ minmax) {
    constexpr int r = P / 2;
    constexpr int RQ = (r + 3) / 4;             // float4 loads on each side of the centre one
    constexpr int NV4 = 2 * RQ + 1;
    __shared__ unsigned sh_lo[4], sh_hi[4];
    const int hkv = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * kPoolTile;
    const int64_t j0 = t0 + 4 * threadIdx.x;
    const bool interior = t0 >= 4 * RQ && t0 + kPoolTile + 4 * RQ <= G.n;
    const float pad = pool_kind == 0 ? -INFINITY : 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int h = 0; h < G.g; ++h) {
        // (a query head whose window was scored in blocks has one vote row per block: they are added,
        // in order, before pooling)
        const float* vb = vote + ((int64_t)hkv * G.NV + (int64_t)h * G.VB) * G.n;
        float v[NV4 * 4];
        if (interior) {
#pragma unroll
            for (int x = 0; x < NV4; ++x) {
                const float4 q = *reinterpret_cast<const float4*>(vb + j0 + 4 * (x - RQ));
                v[4 * x] = q.x;
                v[4 * x + 1] = q.y;
                v[4 * x + 2] = q.z;
                v[4 * x + 3] = q.w;
            }
            for (int b = 1; b < G.VB; ++b) {
#pragma unroll
                for (int x = 0; x < NV4; ++x) {
                    const float4 q = *reinterpret_cast<const float4*>(vb + (int64_t)b * G.n + j0 + 4 * (x - RQ));
                    v[4 * x] += q.x;
                    v[4 * x + 1] += q.y;
                    v[4 * x + 2] += q.z;
                    v[4 * x + 3] += q.w;
                }
            }
        } else {
#pragma unroll
            for (int x = 0; x < NV4 * 4; ++x) {
                const int64_t j = j0 + x - 4 * RQ;
                v[x] = pad;
                if (j >= 0 && j < G.n) {
                    v[x] = vb[j];
                    for (int b = 1; b < G.VB; ++b) v[x] += vb[(int64_t)b * G.n + j];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float val = v[4 * RQ + i - r];
#pragma unroll
            for (int d = 1; d < P; ++d)
                val = pool_kind == 0 ? fmaxf(val, v[4 * RQ + i - r + d]) : val + v[4 * RQ + i - r + d];
            if (pool_kind != 0) val = val / (float)P;
            acc[i] += val;
        }
    }
    unsigned lo = 0xFFFFFFFFu, hi = 0u;
    if (j0 + 3 < G.n) {
        *reinterpret_cast<float4*>(score + (int64_t)hkv * G.n + j0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (j0 + i < G.n) score[(int64_t)hkv * G.n + j0 + i] = acc[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (j0 + i < G.n) {
            const unsigned x = __float_as_uint(acc[i]);
            lo = x < lo ? x : lo;
            hi = x > hi ? x : hi;
        }
    if (minmax) {   // range of this tile's score bit patterns, for the selection that follows
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
            unsigned* mm = minmax + 2 * ((int64_t)hkv * gridDim.x + blockIdx.x);
            mm[0] = lo;
            mm[1] = hi;
        }
    }
}

int pool_tiles(int64_t n) { return (int)((n + kPoolTile - 1) / kPoolTile); }

hipError_t launch_pool(const ScoreGeom& G, const float* vote, int pool_kind, int p, float* score,
                       unsigned* minmax, hipStream_t st) {
    if (G.n <= 0) return hipSuccess;
    const unsigned tiles = (unsigned)((G.n + kPoolTile - 1) / kPoolTile);
    const dim3 grid(tiles, G.Hkv);
    if (G.n % 4 == 0 && (reinterpret_cast<uintptr_t>(vote) & 15u) == 0 &&
        (reinterpret_cast<uintptr_t>(score) & 15u) == 0) {
        switch (p) {
            case 1: hipLaunchKernelGGL(pool_group4<1>, grid, dim3(256), 0, st, vote, score, G, pool_kind, minmax); return hipGetLastError();
            case 5: hipLaunchKernelGGL(pool_group4<5>, grid, dim3(256), 0, st, vote, score, G, pool_kind, minmax); return hipGetLastError();
            case 7: hipLaunchKernelGGL(pool_group4<7>, grid, dim3(256), 0, st, vote, score, G, pool_kind, minmax); return hipGetLastError();
            case 13: hipLaunchKernelGGL(pool_group4<13>, grid, dim3(256), 0, st, vote, score, G, pool_kind, minmax); return hipGetLastError();
            default: break;
        }
    }
    switch (p) {   // the widths the paper uses (Sec. 5) get unrolled taps
        case 1: hipLaunchKernelGGL(pool_group<1>, grid, dim3(256), 0, st, vote, score, G, pool_kind, p, minmax); break;
        case 5: hipLaunchKernelGGL(pool_group<5>, grid, dim3(256), 0, st, vote, score, G, pool_kind, p, minmax); break;
        case 7: hipLaunchKernelGGL(pool_group<7>, grid, dim3(256), 0, st, vote, score, G, pool_kind, p, minmax); break;
        case 13: hipLaunchKernelGGL(pool_group<13>, grid, dim3(256), 0, st, vote, score, G, pool_kind, p, minmax); break;
        default: hipLaunchKernelGGL(pool_group<0>, grid, dim3(256), 0, st, vote, score, G, pool_kind, p, minmax); break;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Identity index list for prompts that fit the capacity, and the row gather.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void iota_rows(const int64_t rows, const int64_t out_stride,
                                                 int32_t* __restrict__ out_idx) {
    int32_t* out = out_idx + (int64_t)blockIdx.y * out_stride;
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < rows; j += (int64_t)gridDim.x * 256)
        out[j] = (int32_t)j;
}

hipError_t launch_iota(int H, int64_t rows, int64_t out_stride, int32_t* out_idx, hipStream_t st) {
    if (H <= 0 || rows <= 0) return hipSuccess;
    unsigned bx = (unsigned)((rows + 255) / 256);
    if (bx > 1024) bx = 1024;
    hipLaunchKernelGGL(iota_rows, dim3(bx, H), dim3(256), 0, st, rows, out_stride, out_idx);
    return hipGetLastError();
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4_nt;

struct NoLayers {};

// Each thread moves 16 bytes of a K row and the matching 16 bytes of the V row; consecutive
// threads cover consecutive pieces of a row, so a 256-byte row is one coalesced 16-lane access.
// Every row is read once and written once: the non-temporal policy keeps both out of the way of
// the next call's K stream.  LY = GatherLayers: head h is head h % ly.heads of the separately allocated
// layer h / ly.heads (k, v, out_k and out_v are then unused) and the positions are copied to that layer's
// out_idx as well.
template <typename LY>
__device__ __forceinline__ void gather_body(const uint4* __restrict__ k, const uint4* __restrict__ v,
                                            const int32_t* __restrict__ idx, const int64_t L, const int64_t rows,
                                            const int64_t out_stride, const int pieces, uint4* __restrict__ out_k,
                                            uint4* __restrict__ out_v, const RowLayout& kl, const RowLayout& vl,
                                            const int head_div, const PageMap& pm, const CleanJob& clean, const LY& ly) {
    constexpr bool LAYERS = std::is_same<LY, GatherLayers>::value;
    const int h = blockIdx.y;
    const int64_t total = rows * pieces;
    const uint4 *kb, *vb;
    uint4 *okb, *ovb;
    int32_t* ob = nullptr;
    if constexpr (LAYERS) {
        const int layer = h / ly.heads, hh = h % ly.heads;
        kb = static_cast<const uint4*>(ly.k[layer]) + (int64_t)(hh / head_div) * kl.head_stride;
        vb = static_cast<const uint4*>(ly.v[layer]) + (int64_t)(hh / head_div) * vl.head_stride;
        okb = static_cast<uint4*>(ly.out_k[layer]) + (int64_t)hh * out_stride * pieces;
        ovb = static_cast<uint4*>(ly.out_v[layer]) + (int64_t)hh * out_stride * pieces;
        ob = ly.out_idx[layer] + (int64_t)hh * out_stride;
    } else {
        kb = k + (int64_t)(h / head_div) * kl.head_stride;
        vb = v + (int64_t)(h / head_div) * vl.head_stride;
        okb = out_k + (int64_t)h * out_stride * pieces;
        ovb = out_v + (int64_t)h * out_stride * pieces;
    }
    const int32_t* ib = idx + (int64_t)h * out_stride;
    // Four pieces per thread and pass, a grid stride apart: the positions are fetched first, then all
    // eight loads are in flight together, then the stores; a thread's two dependent memory latencies
    // (position, then row) are so paid once per four pieces.
    constexpr int U = 4;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t e0 = (int64_t)blockIdx.x * 256 + threadIdx.x; e0 < total; e0 += U * stride) {
        int64_t r[U], src[U];
        int c[U];
        int32_t raw[U];
        bool on[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = e0 + u * stride;
            on[u] = e < total;
            r[u] = on[u] ? e / pieces : 0;
            c[u] = on[u] ? (int)(e - r[u] * pieces) : 0;
            raw[u] = ib[r[u]];
            int64_t pos = raw[u];
            pos = pos < 0 ? 0 : (pos < L ? pos : L - 1);   // whatever idx holds, the read stays inside the prompt
            src[u] = pos;
        }
        u32x4_nt a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t row = physical_row(pm.table, pm.page, pm.pages, src[u]);
            a[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(&kb[row * kl.row_stride + c[u]]));
            b[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(&vb[row * vl.row_stride + c[u]]));
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (on[u]) {
                __builtin_nontemporal_store(a[u], reinterpret_cast<u32x4_nt*>(&okb[r[u] * pieces + c[u]]));
                __builtin_nontemporal_store(b[u], reinterpret_cast<u32x4_nt*>(&ovb[r[u] * pieces + c[u]]));
                if constexpr (LAYERS)
                    if (c[u] == 0) ob[r[u]] = raw[u];
            }
    }
    // the call's scratch is no longer read by anything: leave it ready for the next call
    const int64_t gid = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x;
    const int64_t gsz = (int64_t)gridDim.y * gridDim.x * 256;
    for (int64_t j = gid; j < clean.nones; j += gsz) clean.ones[j] = ~0ull;
    for (int64_t j = gid; j < clean.nzeros; j += gsz) clean.zeros[j] = 0u;
    if (gid == 0 && (clean.flag || clean.status)) {   // the call's verdict (see CleanJob)
        const unsigned gave_up = clean.flag ? *clean.flag : 0u;
        if (clean.status) *clean.status = gave_up ? kStatusTimeout : clean.rows;
        if (gave_up && clean.sticky) __hip_atomic_store(clean.sticky, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        if (clean.flag) *clean.flag = 0u;
    }
}

__global__ __launch_bounds__(256) void gather_rows(const uint4* __restrict__ k,
                                                   const uint4* __restrict__ v,
                                                   const int32_t* __restrict__ idx,
                                                   const int64_t L /* rows per head of k and v */,
                                                   const int64_t rows, const int64_t out_stride,
                                                   const int pieces /* 16-byte pieces per row */,
                                                   uint4* __restrict__ out_k,
                                                   uint4* __restrict__ out_v, const RowLayout kl,
                                                   const RowLayout vl /* strides in 16-byte pieces */,
                                                   const int head_div /* output heads per source head */,
                                                   const PageMap pm, const CleanJob clean) {
    gather_body(k, v, idx, L, rows, out_stride, pieces, out_k, out_v, kl, vl, head_div, pm, clean, NoLayers{});
}

__global__ __launch_bounds__(256) void gather_rows_layers(const GatherLayers ly, const int32_t* __restrict__ idx,
                                                          const int64_t L, const int64_t rows, const int64_t out_stride,
                                                          const int pieces, const RowLayout kl, const RowLayout vl,
                                                          const CleanJob clean) {
    gather_body(nullptr, nullptr, idx, L, rows, out_stride, pieces, nullptr, nullptr, kl, vl, 1, PageMap{}, clean, ly);
}

// Per-head valid prefix lengths of a batch: head h of the batch belongs to prompt h / Hkv.
__global__ __launch_bounds__(256) void batch_lengths(const BatchDesc B, int32_t* __restrict__ nvalid) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < B.count * B.Hkv) nvalid[i] = (int32_t)B.n[i / B.Hkv];
}

hipError_t launch_batch_lengths(const BatchDesc& B, int32_t* nvalid, hipStream_t st) {
    const int items = B.count * B.Hkv;
    hipLaunchKernelGGL(batch_lengths, dim3((items + 255) / 256), dim3(256), 0, st, B, nvalid);
    return hipGetLastError();
}

// gather_rows for a batch: head h of the grid is KV head h % Hkv of prompt h / Hkv; the kept
// positions come from one [heads, C] array and are also copied to the prompt's own out_idx.
__global__ __launch_bounds__(256) void gather_rows_batch(const BatchDesc B, const int32_t* __restrict__ idx,
                                                         const int64_t C, const int pieces, const CleanJob clean) {
    const int h = blockIdx.y, pr = h / B.Hkv, head = h % B.Hkv;
    const int64_t L = B.L[pr];
    const uint4* kb = static_cast<const uint4*>(B.k[pr]) + (int64_t)head * L * pieces;
    const uint4* vb = static_cast<const uint4*>(B.v[pr]) + (int64_t)head * L * pieces;
    uint4* okb = static_cast<uint4*>(B.out_k[pr]) + (int64_t)head * C * pieces;
    uint4* ovb = static_cast<uint4*>(B.out_v[pr]) + (int64_t)head * C * pieces;
    const int32_t* ib = idx + (int64_t)h * C;
    int32_t* ob = B.out_idx[pr] + (int64_t)head * C;
    const int64_t total = C * pieces;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t r = e / pieces;
        const int c = (int)(e - r * pieces);
        int64_t src = ib[r];
        src = src < 0 ? 0 : (src < L ? src : L - 1);   // a failed selection cannot send a read outside the prompt
        const u32x4_nt a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(&kb[src * pieces + c]));
        const u32x4_nt b = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(&vb[src * pieces + c]));
        __builtin_nontemporal_store(a, reinterpret_cast<u32x4_nt*>(&okb[r * pieces + c]));
        __builtin_nontemporal_store(b, reinterpret_cast<u32x4_nt*>(&ovb[r * pieces + c]));
        if (c == 0) ob[r] = ib[r];
    }
    const int64_t gid = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x;
    const int64_t gsz = (int64_t)gridDim.y * gridDim.x * 256;
    for (int64_t j = gid; j < clean.nones; j += gsz) clean.ones[j] = ~0ull;
    for (int64_t j = gid; j < clean.nzeros; j += gsz) clean.zeros[j] = 0u;
}

hipError_t launch_gather_batch(const BatchDesc& B, const int32_t* idx, int64_t C, int row_bytes,
                               const CleanJob& clean, hipStream_t st) {
    if (B.count <= 0 || C <= 0) return hipSuccess;
    const int pieces = row_bytes / 16;
    const int64_t total = C * pieces;
    unsigned bx = (unsigned)((total + 255) / 256);
    if (bx > 1024) bx = 1024;
    hipLaunchKernelGGL(gather_rows_batch, dim3(bx, B.count * B.Hkv), dim3(256), 0, st, B, idx, C, pieces, clean);
    return hipGetLastError();
}

hipError_t launch_gather_layers(const GatherLayers& GL, const int32_t* idx, int64_t L, int64_t rows, int64_t out_stride,
                                int row_bytes, const CleanJob& clean, hipStream_t st) {
    if (GL.count < 1 || GL.count > kMaxLayerPtrs || GL.heads < 1 || L < 1 || (int64_t)GL.count * GL.heads > 65535)
        return hipErrorInvalidValue;
    if (rows <= 0) return hipSuccess;
    const int pieces = row_bytes / 16;
    const int64_t total = rows * pieces;
    unsigned bx = (unsigned)((total + 1023) / 1024);
    if (bx > 4096) bx = 4096;
    const RowLayout rl{L * pieces, pieces};   // contiguous [heads, L, D] in 16-byte pieces
    hipLaunchKernelGGL(gather_rows_layers, dim3(bx, GL.count * GL.heads), dim3(256), 0, st, GL, idx, L, rows, out_stride,
                       pieces, rl, rl, clean);
    return hipGetLastError();
}

hipError_t launch_gather(const void* k, const void* v, const int32_t* idx, int H, int64_t L,
                         int64_t rows, int64_t out_stride, int row_bytes, void* out_k, void* out_v,
                         const RowLayout& kl, const RowLayout& vl, const CleanJob& clean, hipStream_t st,
                         int head_div, const PageMap& pm) {
    if (head_div < 1 || L < 1) return hipErrorInvalidValue;
    if (H <= 0 || rows <= 0) return hipSuccess;
    const int pieces = row_bytes / 16;
    const int64_t total = rows * pieces;
    unsigned bx = (unsigned)((total + 1023) / 1024);   // four pieces per thread
    if (bx > 4096) bx = 4096;
    const RowLayout kp{kl.head_stride / 16, kl.row_stride / 16}, vp{vl.head_stride / 16, vl.row_stride / 16};
    hipLaunchKernelGGL(gather_rows, dim3(bx, H), dim3(256), 0, st, static_cast<const uint4*>(k),
                       static_cast<const uint4*>(v), idx, L, rows, out_stride, pieces,
                       static_cast<uint4*>(out_k), static_cast<uint4*>(out_v), kp, vp, head_div, pm, clean);
    return hipGetLastError();
}

}  // namespace snapkv
