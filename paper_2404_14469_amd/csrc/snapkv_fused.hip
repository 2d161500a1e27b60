// Single-read window scoring and voting (Listing 1: the compute_attn call and the column sum;
// Eq. 1) for prompts whose logits fit on the chip.
//
// The softmax normaliser of a window row needs all L logits of that row before any probability
// can be summed down a column.  Instead of reading K twice, this kernel keeps the exponentials
// of the logits on the chip (registers, then an LDS queue) across a device-wide hand-off:
//
//   * a KV head is a "unit".  The keys of a unit are cut into slices, one per workgroup of a
//     group of Gg workgroups; NG groups work on different units at the same time.  Every
//     workgroup stays resident (one workgroup per compute unit, the grid never exceeds the
//     number of compute units).
//   * step P1 of a unit: the slice of K, loaded once, meets the window queries on MFMA
//     (16x16x32 bf16 or 16x16x4 fp32, fp32 accumulate); the slice's row maxima m_s are taken,
//     e = 2^(s - m_s) goes into the LDS queue and (m_s, sum e) per row is published.
//   * step L1, one unit later: the Gg slices of a row are merged 32 at a time by half-waves
//     spread evenly over the workgroups of the group, and the merged pairs published.
//   * step P2, another unit later: every workgroup merges the few level-1 pairs of each row
//     into (m, 1/Z), scales the queued e by 2^(m_s - m)/Z and sums them over the window rows
//     of each query head: the vote of Eq. 1, stored for prefix columns.
//   All workgroups do the same amount of merging, so none falls behind the others, and what a
//   step reads was published a whole unit earlier, so the waits normally end at once.
//
// Hand-off protocol.  Everything that crosses workgroups is a single aligned 64-bit word moved
// with relaxed device-scope atomic loads and stores: a (max, sum) pair carries its own validity
// (the host side fills the buffers with an all-ones pattern no real pair can have), so no
// ordering between different addresses is needed and the kernel issues no cache write-backs or
// invalidates.  The hand-off words of a step are requested at the top of an iteration, before
// the K loads of the next unit, so that waiting for them never waits for K (a wave's loads
// retire in order).  Every wait is bounded: if one gives up, a counter is raised and the
// kernel still terminates.
//
// MFMA layout (16x16 shapes, 64 lanes): lane l supplies row/column l%16 and contraction slice
// l/16; accumulator register r of lane l is row (l/16)*4 + r, column l%16.  Which head-dim
// elements feed which MFMA step is free as long as Q and K agree, so a lane takes the 16-byte
// pieces 4p + l/16 of its row: the four lanes of a row then read 64 contiguous bytes per load.
#include "snapkv_internal.h"

namespace snapkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct bf16_k {};
struct f32_k {};
template <typename T> struct esize;
template <> struct esize<bf16_k> { static constexpr int value = 2; };
template <> struct esize<f32_k> { static constexpr int value = 4; };

template <typename T, int D> struct Frag16 {
    static constexpr int NP = D * esize<T>::value / 64;   // 16-byte pieces per lane
    uint4 v[NP];
};

template <typename T, int D>
__device__ __forceinline__ void load_frag16(Frag16<T, D>& f, const char* row_base, int kg) {
#pragma unroll
    for (int p = 0; p < Frag16<T, D>::NP; ++p)
        f.v[p] = *reinterpret_cast<const uint4*>(row_base + (4 * p + kg) * 16);
}

template <typename T, int D> __device__ __forceinline__ void zero_frag16(Frag16<T, D>& f) {
#pragma unroll
    for (int p = 0; p < Frag16<T, D>::NP; ++p) f.v[p] = make_uint4(0, 0, 0, 0);
}

template <int D>
__device__ __forceinline__ f32x4 mfma16(const Frag16<bf16_k, D>& a, const Frag16<bf16_k, D>& b) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < Frag16<bf16_k, D>::NP; ++p)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a.v[p]),
                                                      __builtin_bit_cast(bf16x8_t, b.v[p]), acc, 0, 0, 0);
    return acc;
}

template <int D>
__device__ __forceinline__ f32x4 mfma16(const Frag16<f32_k, D>& a, const Frag16<f32_k, D>& b) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < Frag16<f32_k, D>::NP; ++p) {
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.v[p].x), __uint_as_float(b.v[p].x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.v[p].y), __uint_as_float(b.v[p].y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.v[p].z), __uint_as_float(b.v[p].z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.v[p].w), __uint_as_float(b.v[p].w), acc, 0, 0, 0);
    }
    return acc;
}

// Butterfly over the 16 lanes of a DPP row; every lane ends with the same value (the tree has
// the same shape for all lanes and both operations are commutative).
template <int CTRL> __device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_max(float x) {
    x = fmaxf(x, dpp_move<0xB1>(x));    // quad_perm [1,0,3,2]
    x = fmaxf(x, dpp_move<0x4E>(x));    // quad_perm [2,3,0,1]
    x = fmaxf(x, dpp_move<0x141>(x));   // row_half_mirror
    x = fmaxf(x, dpp_move<0x140>(x));   // row_mirror
    return x;
}
__device__ __forceinline__ float row16_sum(float x) {
    x += dpp_move<0xB1>(x);
    x += dpp_move<0x4E>(x);
    x += dpp_move<0x141>(x);
    x += dpp_move<0x140>(x);
    return x;
}

__device__ __forceinline__ void merge_pair(float& m, float& z, float pm, float pz) {
    const float nm = fmaxf(m, pm);
    if (nm != -INFINITY) {
        z = z * __builtin_amdgcn_exp2f(m - nm) + pz * __builtin_amdgcn_exp2f(pm - nm);
        m = nm;
    }
}

// Number of hand-off waits that gave up (never expected; read by snapkv_sync_timeouts()).
__device__ unsigned g_sync_timeouts = 0;

unsigned read_sync_timeouts() {
    unsigned v = 0;
    if (hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_sync_timeouts), sizeof v) != hipSuccess) return ~0u;
    return v;
}

// Optional timestamp trace for tuning builds (-DSNAPKV_FUSED_TRACE): wave 0 of every workgroup
// writes wall-clock stamps at fixed points of each unit into g_trace.  Not compiled by default.
#ifdef SNAPKV_FUSED_TRACE
__device__ long long g_trace[512 * 64 * 12];
#define TRACE(slot_) do { if (tid == 0) g_trace[((int64_t)blockIdx.x * 64 + trace_ui) * 12 + (slot_)] = wall_clock64(); } while (0)
#else
#define TRACE(slot_) do { } while (0)
#endif

constexpr unsigned long long kInvalidPair = ~0ull;   // a sum-exp is never NaN: no real pair looks like this
constexpr int kSlicesPerBlock = 32;                  // slices merged by one half-wave in step L1

__device__ __forceinline__ unsigned long long pack_pair(float m, float z) {
    return ((unsigned long long)__float_as_uint(z) << 32) | (unsigned long long)__float_as_uint(m);
}
__device__ __forceinline__ void unpack_pair(unsigned long long bits, float& m, float& z) {
    m = __uint_as_float((unsigned)(bits & 0xffffffffull));
    z = __uint_as_float((unsigned)(bits >> 32));
}
__device__ __forceinline__ void publish_pair(float2* p, float m, float z) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), pack_pair(m, z), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long load_pair_bits(const float2* p) {
    return __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
}
// Waits (bounded) until the word at p is a published pair; `bits` is what an earlier load saw.
__device__ __forceinline__ unsigned long long await_pair(const float2* p, unsigned long long bits,
                                                         unsigned limit, bool& gave_up) {
    unsigned spins = 0;
    while (bits == kInvalidPair) {
        if (++spins > limit) {
            gave_up = true;
            return pack_pair(-INFINITY, 0.f);
        }
        __builtin_amdgcn_s_sleep(2);
        bits = load_pair_bits(p);
    }
    return bits;
}

// pair buffers to the invalid pattern
__global__ void init_sync(unsigned long long* pairs, int64_t npairs) {
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < npairs;
         j += (int64_t)gridDim.x * blockDim.x)
        pairs[j] = kInvalidPair;
}

// LDS-only barrier: orders LDS traffic between the waves of the workgroup without draining the
// global loads in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <typename T, int D, int RUW, int KT, int NW>
__global__ __launch_bounds__(NW * 64) void score_fused(const void* __restrict__ qv,
                                                       const void* __restrict__ kv,
                                                       float* __restrict__ vote, const FusedSync S,
                                                       const ScoreGeom G, const FusedGeom F) {
    constexpr int R = RUW * 16;          // window rows a workgroup tracks per unit
    constexpr int NT = NW * 64;
    constexpr int NSLOT = RUW * KT;      // accumulator tiles per lane per unit
    constexpr int NBMAX = 8;             // level-1 blocks per row (Gg <= 256)
    constexpr int L2PT = (R * NBMAX + NT - 1) / NT;   // level-1 pairs a thread fetches in step P2
    constexpr int ES = esize<T>::value;
    using Frag = Frag16<T, D>;

    extern __shared__ float4 fifo[];     // [2][NSLOT][NT]: e of the two units in flight
    __shared__ float sm_wmax[NW][R];
    __shared__ float sm_wsum[NW][R];
    __shared__ float sm_ref[3][R];
    __shared__ float2 sm_l1[R * NBMAX];
    __shared__ float2 sm_fin[R];

    const char* q = static_cast<const char*>(qv);
    const char* k = static_cast<const char*>(kv);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, n16 = lane & 15, kg = lane >> 4;
    const int wg = (int)(blockIdx.x % F.Gg), group = (int)(blockIdx.x / F.Gg);
    const int64_t tile0 = ((int64_t)wg * NW + w) * KT;
    const int nu = group < F.units ? (F.units - group + F.NG - 1) / F.NG : 0;   // units of this group
    if (nu == 0) return;
    const int tasks = R * F.NB;          // level-1 merges per unit, spread over the group
    const int hw = tid >> 5, l32 = tid & 31;
    bool gave_up = false;
#ifdef SNAPKV_FUSED_TRACE
    int trace_ui = 0;
#endif

    Frag kf[KT];
    Frag qf[RUW];
    auto issue_loads = [&](int unit) {
        const char* kb = k + (int64_t)unit * G.L * D * ES;
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const int64_t tile = tile0 + t;
            if (tile < F.ntiles) {
                int64_t j = tile * 16 + n16;
                j = j < G.L ? j : G.L - 1;
                load_frag16<T, D>(kf[t], kb + j * D * ES, kg);
            } else {
                zero_frag16<T, D>(kf[t]);
            }
        }
#pragma unroll
        for (int ru = 0; ru < RUW; ++ru) {
            const int head = ru / F.UH;
            const int i = (ru % F.UH) * 16 + n16;
            if (ru < F.RU && i < G.W) {
                const int64_t row = (int64_t)(unit * G.g + head) * G.W + i;
                load_frag16<T, D>(qf[ru], q + row * D * ES, kg);
            } else {
                zero_frag16<T, D>(qf[ru]);
            }
        }
    };

    issue_loads(group);
    for (int it = 0; it < nu + 2; ++it) {
        const bool has_p1 = it < nu;
        const bool has_l1 = it >= 1 && it - 1 < nu;
        const bool has_p2 = it >= 2;
        const int unit = group + it * F.NG;
        const int unit_l1 = unit - F.NG;
        const int unit_p2 = unit - 2 * F.NG;
        TRACE(0);

        // ---- A. request this iteration's hand-off words (before the next unit's K loads)
        unsigned long long l1_bits = pack_pair(-INFINITY, 0.f);
        const float2* l1_src = nullptr;
        const int task0 = wg + hw * F.Gg;
        if (has_l1 && task0 < tasks) {
            const int row = task0 / F.NB, blk = task0 % F.NB;
            const int slice = blk * kSlicesPerBlock + l32;
            if (slice < F.Gg) {
                l1_src = &S.part[((int64_t)unit_l1 * F.Gg + slice) * R + row];
                l1_bits = load_pair_bits(l1_src);
            }
        }
        unsigned long long p2_bits[L2PT];
#pragma unroll
        for (int x = 0; x < L2PT; ++x) {
            const int idx = tid + x * NT;
            p2_bits[x] = has_p2 && idx < tasks ? load_pair_bits(&S.l1[(int64_t)unit_p2 * tasks + idx])
                                               : kInvalidPair;
        }

        f32x4 e[RUW][KT];
        if (has_p1) {
            // ---- B. logits of the slice; C. start the next unit's loads
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int t = 0; t < KT; ++t) e[ru][t] = mfma16<D>(qf[ru], kf[t]);
            if (it + 1 < nu) issue_loads(unit + F.NG);
            TRACE(1);

            // ---- D. base-2 logits, causal mask, slice row maxima
            float mx[RUW][4];
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int r = 0; r < 4; ++r) mx[ru][r] = -INFINITY;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int64_t tile = tile0 + t;
                const int64_t j = tile * 16 + n16;
                const bool live = tile < F.ntiles;
                const bool boundary = tile * 16 + 15 >= G.n;
#pragma unroll
                for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float s = e[ru][t][r] * G.c2;
                        if (!live) {
                            s = -INFINITY;
                        } else if (boundary) {
                            const int i = (ru % F.UH) * 16 + kg * 4 + r;
                            if (j > G.n + i || j >= G.L) s = -INFINITY;   // prompt-phase causal mask
                        }
                        e[ru][t][r] = s;
                        mx[ru][r] = fmaxf(mx[ru][r], s);
                    }
            }
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int r = 0; r < 4; ++r) mx[ru][r] = row16_max(mx[ru][r]);
            if (n16 == 0) {
#pragma unroll
                for (int ru = 0; ru < RUW; ++ru)
                    *reinterpret_cast<float4*>(&sm_wmax[w][ru * 16 + kg * 4]) =
                        make_float4(mx[ru][0], mx[ru][1], mx[ru][2], mx[ru][3]);
            }
        }
        TRACE(2);
        lds_barrier();
        TRACE(3);
        if (has_p1) {
            // workgroup reference, exponentials, slice row sums
            float zs[RUW][4];
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                float4 m4 = *reinterpret_cast<const float4*>(&sm_wmax[0][ru * 16 + kg * 4]);
#pragma unroll
                for (int w2 = 1; w2 < NW; ++w2) {
                    const float4 o = *reinterpret_cast<const float4*>(&sm_wmax[w2][ru * 16 + kg * 4]);
                    m4.x = fmaxf(m4.x, o.x);
                    m4.y = fmaxf(m4.y, o.y);
                    m4.z = fmaxf(m4.z, o.z);
                    m4.w = fmaxf(m4.w, o.w);
                }
                const float ref[4] = {m4.x == -INFINITY ? 0.f : m4.x, m4.y == -INFINITY ? 0.f : m4.y,
                                      m4.z == -INFINITY ? 0.f : m4.z, m4.w == -INFINITY ? 0.f : m4.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float z = 0.f;
#pragma unroll
                    for (int t = 0; t < KT; ++t) {
                        const float x = __builtin_amdgcn_exp2f(e[ru][t][r] - ref[r]);
                        e[ru][t][r] = x;
                        z += x;
                    }
                    zs[ru][r] = row16_sum(z);
                }
            }
            if (n16 == 0) {
#pragma unroll
                for (int ru = 0; ru < RUW; ++ru)
                    *reinterpret_cast<float4*>(&sm_wsum[w][ru * 16 + kg * 4]) =
                        make_float4(zs[ru][0], zs[ru][1], zs[ru][2], zs[ru][3]);
            }
        }
        lds_barrier();
        TRACE(4);
        if (has_p1 && tid < R) {   // publish the slice's (max, sum) per row
            float m = sm_wmax[0][tid], z = sm_wsum[0][tid];
#pragma unroll
            for (int w2 = 1; w2 < NW; ++w2) {
                m = fmaxf(m, sm_wmax[w2][tid]);
                z += sm_wsum[w2][tid];
            }
            publish_pair(&S.part[((int64_t)unit * F.Gg + wg) * R + tid], m, z);
            sm_ref[it % 3][tid] = m;
        }

        // ---- E. step L1 of the previous unit: merge 32 slices of one row per half-wave
        if (has_l1) {
            for (int task = task0; task < tasks; task += 2 * NW * F.Gg) {
                const int row = task / F.NB, blk = task % F.NB;
                float m = -INFINITY, z = 0.f;
                if (task == task0) {
                    if (l1_src) unpack_pair(await_pair(l1_src, l1_bits, F.spin_limit, gave_up), m, z);
                } else {
                    const int slice = blk * kSlicesPerBlock + l32;
                    if (slice < F.Gg) {
                        const float2* src = &S.part[((int64_t)unit_l1 * F.Gg + slice) * R + row];
                        unpack_pair(await_pair(src, load_pair_bits(src), F.spin_limit, gave_up), m, z);
                    }
                }
#pragma unroll
                for (int d = 1; d < 32; d <<= 1) {   // fixed tree over the half-wave's 32 slices
                    const float om = __shfl_xor(m, d, 64), oz = __shfl_xor(z, d, 64);
                    merge_pair(m, z, om, oz);
                }
                if (l32 == 0) publish_pair(&S.l1[(int64_t)unit_l1 * tasks + task], m, z);
            }
        }
        TRACE(5);

        // ---- F. step P2 of the unit before that
        if (has_p2) {
#pragma unroll
            for (int x = 0; x < L2PT; ++x) {
                const int idx = tid + x * NT;
                if (idx < tasks) {
                    float m, z;
                    unpack_pair(await_pair(&S.l1[(int64_t)unit_p2 * tasks + idx], p2_bits[x],
                                           F.spin_limit, gave_up), m, z);
                    sm_l1[idx] = make_float2(m, z);
                }
            }
        }
        lds_barrier();
        TRACE(6);
        if (has_p2 && tid < R) {   // level-1 pairs of a row, in block order, into (max, 1/sum)
            float m = -INFINITY, z = 0.f;
            for (int blk = 0; blk < F.NB; ++blk) {
                const float2 x = sm_l1[tid * F.NB + blk];
                merge_pair(m, z, x.x, x.y);
            }
            const int ru = tid >> 4;
            const int i = (ru % F.UH) * 16 + (tid & 15);
            const bool real = ru < F.RU && i < G.W && z > 0.f;
            sm_fin[tid] = real ? make_float2(m, 1.0f / z) : make_float2(0.f, 0.f);
        }
        lds_barrier();
        float4* slot = fifo + (size_t)(it & 1) * NSLOT * NT + tid;
        if (has_p2) {
            float f[RUW][4];
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = ru * 16 + kg * 4 + r;
                    const float2 mz = sm_fin[row];
                    const float ms = sm_ref[(it + 1) % 3][row];   // written two iterations ago
                    f[ru][r] = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - mz.x) * mz.y;
                }
            float* vb = vote + (int64_t)unit_p2 * G.g * G.n;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int64_t j = (tile0 + t) * 16 + n16;
                float v = 0.f;
#pragma unroll
                for (int ru = 0; ru < RUW; ++ru) {
                    const float4 ev = slot[(size_t)(ru * KT + t) * NT];
                    v = fmaf(ev.x, f[ru][0], v);
                    v = fmaf(ev.y, f[ru][1], v);
                    v = fmaf(ev.z, f[ru][2], v);
                    v = fmaf(ev.w, f[ru][3], v);
                    if ((ru + 1) % F.UH == 0) {   // last row unit of a query head: finish its vote
                        v += __shfl_xor(v, 16, 64);
                        v += __shfl_xor(v, 32, 64);
                        const int head = ru / F.UH;
                        if (kg == 0 && head < G.g && j < G.n) vb[(int64_t)head * G.n + j] = v;
                        v = 0.f;
                    }
                }
            }
        }
        // ---- G. queue this unit's exponentials (each lane owns its queue entries)
        if (has_p1) {
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int t = 0; t < KT; ++t)
                    slot[(size_t)(ru * KT + t) * NT] = make_float4(e[ru][t][0], e[ru][t][1], e[ru][t][2], e[ru][t][3]);
        }
        TRACE(7);
#ifdef SNAPKV_FUSED_TRACE
        ++trace_ui;
#endif
    }
    if (gave_up) atomicAdd(&g_sync_timeouts, 1u);
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
constexpr int kFusedWaves = 8;
constexpr int kFusedSlots = 8;          // RUW * KT: accumulator tiles a wave keeps per unit

static int g_cu_count[64] = {0};

static int cu_count() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (g_cu_count[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        g_cu_count[dev] = n;
    }
    return g_cu_count[dev];
}

// Device-independent part of the plan: how the rows and keys of a unit map onto a workgroup.
// Returns false when the window rows of a KV head exceed what one wave tracks.
bool fused_shape(const ScoreGeom& G, FusedGeom* F) {
    const int UH = (G.W + 15) / 16;
    const int RU = G.g * UH;
    if (RU > 8 || G.n <= 0) return false;
    int RUW = 1;
    while (RUW < RU) RUW *= 2;
    const int KT = kFusedSlots / RUW;
    const int64_t ntiles = (G.L + 15) / 16;
    const int64_t per_wg = (int64_t)kFusedWaves * KT;
    const int64_t Gg = (ntiles + per_wg - 1) / per_wg;
    if (Gg > 256) return false;   // level-1 merge blocks per row are capped at 8
    F->RU = RU;
    F->UH = UH;
    F->RUW = RUW;
    F->KT = KT;
    F->Gg = (int)Gg;
    F->NG = 1;
    F->NB = (int)((Gg + 31) / 32);
    F->ntiles = ntiles;
    F->units = G.Hkv;
    F->spin_limit = 1u << 24;
    return true;
}

// Whether the current device can keep a whole group resident (one workgroup per compute unit),
// and how many groups run side by side.
bool fused_plan(const ScoreGeom& G, FusedGeom* F) {
    if (!fused_shape(G, F)) return false;
    const int cus = cu_count();
    if (cus <= 0 || F->Gg > cus) return false;   // one head's logits do not fit the register files
    int NG = cus / F->Gg;
    if (NG > G.Hkv) NG = G.Hkv;
    F->NG = NG;
    return true;
}

size_t fused_sync_layout(const ScoreGeom& G, const FusedGeom& F, FusedSync* S, void* base) {
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t R = (size_t)F.RUW * 16;
    const size_t part = sizeof(float2) * (size_t)F.units * F.Gg * R;   // l1 follows part directly
    const size_t l1 = sizeof(float2) * (size_t)F.units * R * F.NB;
    if (S) {
        char* b = static_cast<char*>(base);
        S->part = reinterpret_cast<float2*>(b);
        S->l1 = reinterpret_cast<float2*>(b + part);
    }
    return up(part + l1);
}

template <typename T, int D, int RUW>
static hipError_t launch_fused_t(const void* q, const void* k, const ScoreGeom& G, const FusedGeom& F,
                                 const FusedSync& S, float* vote, hipStream_t st) {
    constexpr int KT = kFusedSlots / RUW;
    auto kern = score_fused<T, D, RUW, KT, kFusedWaves>;
    // the LDS queue: two units of exponentials; large enough that one workgroup owns a compute unit
    constexpr int kQueueBytes = 2 * kFusedSlots * kFusedWaves * 64 * 16;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kQueueBytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int64_t npairs = (int64_t)F.units * (F.RUW * 16) * (F.Gg + F.NB);   // part and l1 are adjacent
    int64_t blocks = (npairs + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(init_sync, dim3((unsigned)blocks), dim3(256), 0, st,
                       reinterpret_cast<unsigned long long*>(S.part), npairs);
    hipLaunchKernelGGL(kern, dim3(F.NG * F.Gg), dim3(kFusedWaves * 64), kQueueBytes, st, q, k, vote, S, G, F);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t launch_fused_d(const void* q, const void* k, const ScoreGeom& G, const FusedGeom& F,
                                 const FusedSync& S, float* vote, hipStream_t st) {
    switch (F.RUW) {
        case 1: return launch_fused_t<T, D, 1>(q, k, G, F, S, vote, st);
        case 2: return launch_fused_t<T, D, 2>(q, k, G, F, S, vote, st);
        case 4: return launch_fused_t<T, D, 4>(q, k, G, F, S, vote, st);
        case 8: return launch_fused_t<T, D, 8>(q, k, G, F, S, vote, st);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_score_fused(int dtype, int D, const void* q, const void* k, const ScoreGeom& G,
                              const FusedGeom& F, const FusedSync& S, float* vote, hipStream_t st) {
    if (G.n <= 0) return hipSuccess;
    if (dtype == 0) {
        if (D == 128) return launch_fused_d<bf16_k, 128>(q, k, G, F, S, vote, st);
        if (D == 64) return launch_fused_d<bf16_k, 64>(q, k, G, F, S, vote, st);
    } else {
        if (D == 128) return launch_fused_d<f32_k, 128>(q, k, G, F, S, vote, st);
        if (D == 64) return launch_fused_d<f32_k, 64>(q, k, G, F, S, vote, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace snapkv

#ifdef SNAPKV_FUSED_TRACE
extern "C" int snapkv_debug_trace(long long* out, int n) {
    if (n > 512 * 64 * 12) n = 512 * 64 * 12;
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(snapkv::g_trace), sizeof(long long) * n);
}
#endif
