// Single-read window scoring and voting (Listing 1: the compute_attn call and the column sum;
// Eq. 1) for prompts whose logits fit on the chip.
//
// The softmax normaliser of a window row needs all L logits of that row before any probability
// can be summed down a column.  Instead of reading K twice, this kernel keeps the exponentials
// of the logits in registers across a device-wide hand-off of the row normalisers:
//
//   * a "unit" is a KV head, or, when the query heads of a KV head have more window rows than a
//     wave tracks well, one of `split` equal parts of its query heads (units of one KV head then
//     run side by side in neighbouring groups, so that its keys are fetched from memory once and
//     found in the cache by the others; where the prompt is too long for that, they follow one
//     another on the same workgroups).  The keys of a unit are cut into slices, one per workgroup of a
//     group of Gg workgroups; NG groups work on different units at the same time.  Every
//     workgroup stays resident (the grid never exceeds what the device keeps resident at once).
//   * step P1 of a unit: the slice of K, loaded once, meets the window queries on MFMA
//     (16x16x32 bf16 or 16x16x4 fp32, fp32 accumulate); the slice's row maxima m_s are taken,
//     e = 2^(s - m_s) stays in the wave's registers and (m_s, sum e) per row is published.
//   * step L1, one unit later: the Gg slices of a row are merged 32 at a time by half-waves
//     spread evenly over the workgroups of the group, and the merged pairs published.
//   * step P2, another unit later: every workgroup merges the few level-1 pairs of each row
//     into (m, 1/Z), scales the kept e by 2^(m_s - m)/Z and sums them over the window rows
//     of each query head: the vote of Eq. 1, stored for prefix columns.
//   All workgroups do the same amount of merging, so none falls behind the others, and what a
//   step reads was published a whole unit earlier, so the waits normally end at once.
//
// Hand-off protocol.  Everything that crosses workgroups is a single aligned 64-bit word moved
// with relaxed device-scope atomic loads and stores: a (max, sum) pair carries its own validity
// (the host side fills the buffers with an all-ones pattern no real pair can have), so no
// ordering between different addresses is needed and the kernel issues no cache write-backs or
// invalidates.  The hand-off words of a step are requested at the top of an iteration, before
// the K loads issued in it, so that waiting for them never waits for those (a wave's loads
// retire in order).  Inside a workgroup the waves exchange their partial results through LDS
// with per-wave flags instead of barriers.  Every wait is bounded: if one gives up, a counter
// is raised and the kernel still terminates.
//
// Keeping K in flight.  A wave's K tile buffers (registers) are the landing space of the
// stream: half of them are consumed by MFMAs at the top of an iteration, half at its end, and
// each is requested again at one of four points spread over the iteration.  All loads of the
// steady state are unconditional, so that the compiler can count, on every path, how many
// younger loads may stay in flight when it waits for an older one.
//
// MFMA layout (16x16 shapes, 64 lanes): lane l supplies row/column l%16 and contraction slice
// l/16; accumulator register r of lane l is row (l/16)*4 + r, column l%16.  Which head-dim
// elements feed which MFMA step is free as long as Q and K agree, so a lane takes the 16-byte
// pieces 4p + l/16 of its row: the four lanes of a row then read 64 contiguous bytes per load.
#include "snapkv_internal.h"

#include <cstdlib>
#include <type_traits>

namespace snapkv {

// Votes are stored with device scope: the store goes through to memory at once instead of leaving a
// dirty line in the die's cache.  They are read once, by a later kernel, and as ordinary stores their
// dirty lines compete with the K stream for the cache (about 10 us per call at 131072 keys x 32 heads);
// the non-temporal policy avoids most of that, the write-through store all of it (265 us against 276 us
// per call there, same build otherwise).
#define VOTE_STORE(p_, v_) __hip_atomic_store((p_), (v_), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct bf16_k {};
struct f16_k {};
struct f32_k {};
template <typename T> struct esize;
template <> struct esize<bf16_k> { static constexpr int value = 2; };
template <> struct esize<f16_k> { static constexpr int value = 2; };
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
__device__ __forceinline__ f32x4 mfma16(const Frag16<f16_k, D>& a, const Frag16<f16_k, D>& b) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < Frag16<f16_k, D>::NP; ++p)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a.v[p]),
                                                     __builtin_bit_cast(f16x8_t, b.v[p]), acc, 0, 0, 0);
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

bool reset_sync_timeouts() {
    const unsigned zero = 0;
    return hipMemcpyToSymbol(HIP_SYMBOL(g_sync_timeouts), &zero, sizeof zero) == hipSuccess;
}

unsigned read_sync_timeouts() {
    unsigned v = 0;
    if (hipMemcpyFromSymbol(&v, HIP_SYMBOL(g_sync_timeouts), sizeof v) != hipSuccess) return ~0u;
    return v;
}


constexpr unsigned long long kInvalidPair = ~0ull;   // a sum-exp is never NaN: no real pair looks like this
constexpr int kSlicesPerBlock = 32;                  // slices merged by one half-wave in step L1
constexpr int kL1BlocksPadded = 16;                  // level-1 words per row (Gg <= 512)

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
        if (gave_up || ++spins > limit) {   // once a wait has given up, later ones do not wait again
            gave_up = true;
            return pack_pair(-INFINITY, 0.f);
        }
        __builtin_amdgcn_s_sleep(2);
        bits = load_pair_bits(p);
    }
    return bits;
}

// Hand-offs between the waves of a workgroup go through LDS without a barrier: a wave writes
// its data, then stamps its flag with the iteration number; a reader waits (bounded) until the
// flags of all waves have reached the stamp it needs.  The fences order LDS traffic only, so
// that no wave ever drains its global loads in flight for them.
__device__ __forceinline__ void lds_release() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
}
__device__ __forceinline__ void lds_stamp(int* flag, int value) {
    __hip_atomic_store(flag, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
template <int NW>
__device__ __forceinline__ void lds_await_all(int* flags, int need, unsigned limit, bool& gave_up) {
    static_assert((NW & (NW - 1)) == 0, "waves per workgroup must be a power of two");
    int* mine = flags + (threadIdx.x & (NW - 1));
    unsigned spins = 0;
    while (__hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < need) {
        if (gave_up || ++spins > limit) {
            gave_up = true;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int CTRL> __device__ __forceinline__ void dpp_merge(float& m, float& z) {
    const float om = dpp_move<CTRL>(m), oz = dpp_move<CTRL>(z);
    merge_pair(m, z, om, oz);
}

template <typename T, int D>
__device__ __forceinline__ void load_frag16p(Frag16<T, D>& f, const char* p) {
#pragma unroll
    for (int x = 0; x < Frag16<T, D>::NP; ++x) f.v[x] = *reinterpret_cast<const uint4*>(p + 64 * x);
}

// The kernel's body; `bid` is the workgroup's index inside its own launch plan (the block index,
// or the block index less the first block of the prompt when several prompts share a launch).
constexpr int kFusedSlots = 8;          // RUW * KT: accumulator tiles a wave keeps per unit (8 waves)

// The instance with one row unit per workgroup (a window of at most 16 rows, one query head per
// unit) holds eight K tile buffers per wave, twice what the others hold, and has no registers left
// for the exponentials of the two previous units: those wait for their vote in LDS instead (two
// generations of RUW * KT accumulator tiles per thread, behind the Q blocks).
template <int RUW> struct fused_parks { static constexpr bool value = RUW == 1; };

// Bytes of dynamic LDS of score_fused: the Q blocks of three units, then the parked exponentials.
template <typename T, int D, int RUW, int NW> constexpr int fused_lds_bytes() {
    return 3 * RUW * (D * esize<T>::value / 64) * 64 * 16 + (fused_parks<RUW>::value ? 2 * kFusedSlots * NW * 64 * 16 : 0);
}

// LAYERS: the heads are those of several layers of one prompt that are separate allocations; the Q and K
// rows of head h then start at SL->q / SL->k [h / heads per layer] instead of behind one another after
// qv / kv (which are then unused).
template <typename T, int D, int RUW, int KT, int NW, bool LAYERS = false>
__device__ __forceinline__ void score_fused_body(const void* __restrict__ qv, const void* __restrict__ kv,
                                                 float* __restrict__ vote, const FusedSync& S,
                                                 const ScoreGeom& G, const FusedGeom& F, const int bid,
                                                 const ScoreLayers* SL = nullptr) {
    constexpr int R = RUW * 16;          // window rows a workgroup tracks per unit
    constexpr int NT = NW * 64;
    constexpr int NSLOT = RUW * KT;      // accumulator tiles per lane per unit
    constexpr int NBP = kL1BlocksPadded; // level-1 words per row (the first F.NB are real)
    constexpr int L2PT = (R * NBP + NT - 1) / NT;   // level-1 words a thread fetches in step P2
    constexpr int ES = esize<T>::value;
    using Frag = Frag16<T, D>;

    constexpr int NP = Frag::NP;         // 16-byte pieces per lane per row
    constexpr int QCH = RUW * NP;        // 1 KB chunks of a unit's Q block, in the order the MFMAs read them
    constexpr int QPW = (QCH + NW - 1) / NW;   // chunks a wave fetches per unit
    extern __shared__ uint4 qbuf[];      // [3][QCH][64]: Q blocks of three consecutive units
    constexpr bool PARK = fused_parks<RUW>::value;
    // [2][NSLOT][NT] exponentials of the units one and two back, each thread's own (PARK only)
    f32x4* const park = reinterpret_cast<f32x4*>(qbuf + 3 * QCH * 64);
    // No barrier inside the loop.  Why the buffers may be reused when they are: a wave writes
    // them only after step E of an iteration, which has waited for level-1 words of the unit two
    // back; those exist only once every workgroup, this one included, has published that unit's
    // slice, i.e. once all its waves have passed step D of the iteration two back.  Hence a
    // buffer read up to the end of iteration `it` may be rewritten from iteration it + 3 on
    // (qbuf, sm_fin: three copies), and one read by the publishing wave before it publishes
    // from iteration it + 2 on (sm_pair: two copies).
    __shared__ float2 sm_pair[2][NW][R]; // per wave: (row max, row sum-exp) of the current unit
    __shared__ float sm_ref[3][NW][R];   // per wave: row maxima of the last three units (own wave only)
    __shared__ float2 sm_fin[3][R];      // (row max, 1 / row sum-exp) of the unit in step P2
    __shared__ int sm_flag[3][NW];       // per wave: Q chunks / sm_pair / sm_fin written up to this stamp

    const int tid = threadIdx.x, lane = tid & 63, n16 = lane & 15, kg = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = bid % F.Gg, group = bid / F.Gg;
    // Tile t of this wave is key tile tile0 + t * TS: the waves of the whole group work on the same
    // t at about the same time, and this way what they request together is one contiguous stretch
    // of K instead of one 4 KB piece out of every wave's 16 KB (which loads only part of the memory
    // channels at any moment).
    const int TS = F.Gg * NW;
    // Workgroups are handed to the chip's eight dies in turn; those of one die take neighbouring
    // stretches of keys so that the die's cache channels are loaded evenly.
    const int vwg = (F.Gg % 8 == 0) ? (wg % 8) * (F.Gg / 8) + wg / 8 : wg;
    const int tile0 = vwg * NW + w;
    const int nu = group < F.units ? (F.units - group + F.NG - 1) / F.NG : 0;   // units of this group
    if (nu == 0) return;
    // wave touches window columns, the ragged tail or tiles past the end: masks are needed
    const bool special = ((int64_t)(KT - 1) * TS + tile0 + 1) * 16 > G.n;
    const int hw = tid >> 5, l32 = tid & 31;
    const int real_tasks = R * F.NB;
    bool gave_up = false;

    // Per-lane row addresses; they advance by one group stride per iteration.  Loads are
    // unconditional (out-of-range tiles and padding rows re-read a valid row and are masked or
    // ignored later) so that the number of loads in flight behind a hand-off word is fixed.
    // first K row of KV head h, first Q row of query head qh
    auto k_head = [&](const int h) -> const char* {
        if constexpr (LAYERS)
            return static_cast<const char*>(SL->k[h / SL->kv_heads]) + (int64_t)(h % SL->kv_heads) * G.k_hs;
        else
            return static_cast<const char*>(kv) + (int64_t)h * G.k_hs;
    };
    auto q_head = [&](const int qh) -> const char* {
        if constexpr (LAYERS) {
            const int per_layer = SL->kv_heads * G.g;
            return static_cast<const char*>(SL->q[qh / per_layer]) + (int64_t)(qh % per_layer) * G.W * D * ES;
        } else {
            return static_cast<const char*>(qv) + (int64_t)qh * G.W * D * ES;
        }
    };
    const char* kp[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        int64_t j = ((int64_t)t * TS + tile0) * 16 + n16;
        j = j < G.L ? j : G.L - 1;
        j = physical_row(G.k_table, G.k_page, G.k_pages, j + G.k_row0);
        kp[t] = k_head(group / F.split) + j * G.k_rs + kg * 16;
    }
    // Q is shared by the waves: each fetches QPW of the unit's 1 KB chunks (chunk c = row unit c / NP,
    // piece c % NP, lane l = row l % 16, contraction slice l / 16) and leaves them in LDS.
    const char* qp[QPW];
#pragma unroll
    for (int x = 0; x < QPW; ++x) {
        int c = w + x * NW;
        c = c < QCH ? c : QCH - 1;
        const int ru = c / NP, pc = c % NP;
        int head = ru / F.UH, i = (ru % F.UH) * 16 + n16;
        head = head < F.gs ? head : F.gs - 1;
        i = i < G.W ? i : G.W - 1;
        qp[x] = q_head(group * F.gs + head) + (int64_t)i * D * ES + (4 * pc + kg) * 16;
    }
    // The KV head of unit u is u / split, and a group's units are NG apart.  Where whole KV heads run
    // side by side (NG a multiple of split) the K pointers move by the same amount every iteration;
    // where a prompt is so long that fewer groups than a KV head has parts fit the chip, the parts of a
    // KV head follow one another on the same workgroups (its keys then come from the cache the second
    // time) and the step from one unit to the next is zero or one head.
    const bool even_steps = F.NG % F.split == 0;
    const int64_t kstep_even = (int64_t)(F.NG / F.split) * G.k_hs;
    auto kstep_to = [&](const int itn) -> int64_t {   // from the K of the group's unit itn - 1 to that of unit itn
        if constexpr (LAYERS) return k_head((group + itn * F.NG) / F.split) - k_head((group + (itn - 1) * F.NG) / F.split);
        if (even_steps) return kstep_even;
        return (int64_t)((group + itn * F.NG) / F.split - (group + (itn - 1) * F.NG) / F.split) * G.k_hs;
    };
    const int64_t qstep_even = (int64_t)F.NG * F.gs * G.W * D * ES;
    auto qstep_to = [&](const int itn) -> int64_t {   // the same for Q (a unit's query heads lie in one layer)
        if constexpr (LAYERS) return q_head((group + itn * F.NG) * F.gs) - q_head((group + (itn - 1) * F.NG) * F.gs);
        return qstep_even;
    };

    // K tiles are consumed in two halves so that the memory pipeline never runs dry: the lower
    // KL tiles of a unit meet Q at the end of the previous iteration (their accumulators take
    // the registers the vote has just freed) and are re-requested at once for the unit after;
    // the upper tiles meet Q at the top of the unit's own iteration and are re-requested in
    // portions spread over its first steps.  Every K load so has about one iteration to land,
    // and at least half of a wave's tile buffers are in flight at any time.
    constexpr int KL = KT / 2;           // lower tiles (none when a wave holds a single tile)
    Frag kf[KT];
    uint4 qland[QPW];
    f32x4 e[RUW][KT];                    // logits, then exponentials, of the unit in step P1
#pragma unroll
    for (int t = 0; t < KT; ++t) load_frag16p<T, D>(kf[t], kp[t]);
#pragma unroll
    for (int x = 0; x < QPW; ++x) qland[x] = *reinterpret_cast<const uint4*>(qp[x]);
#pragma unroll
    for (int x = 0; x < QPW; ++x)
        if (w + x * NW < QCH) qbuf[(w + x * NW) * 64 + lane] = qland[x];
    if (tid < 3 * NW) sm_flag[tid / NW][tid % NW] = tid < NW ? 1 : 0;   // Q of unit 0 is in place
    __syncthreads();
    // exponentials of the two previous units stay in registers (or, PARK, in LDS) until their votes are taken
    f32x4 e1[PARK ? 1 : RUW][PARK ? 1 : KT], e2[PARK ? 1 : RUW][PARK ? 1 : KT];
#pragma unroll
    for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            e[ru][t] = f32x4{0.f, 0.f, 0.f, 0.f};
            if constexpr (!PARK) e1[ru][t] = e2[ru][t] = e[ru][t];
        }

    // logits of tiles [T0, T1) of the unit whose Q block sits in half `par` of qbuf
    auto mfma_tiles = [&](auto T0, auto T1, const int par) {
        constexpr int t0 = decltype(T0)::value, t1 = decltype(T1)::value;
        if constexpr (t0 < t1) {
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                Frag qf;
#pragma unroll
                for (int pc = 0; pc < NP; ++pc) qf.v[pc] = qbuf[(par * QCH + ru * NP + pc) * 64 + lane];
#pragma unroll
                for (int t = t0; t < t1; ++t) e[ru][t] = mfma16<D>(qf, kf[t]);
            }
        }
    };
    auto issue_tiles = [&](auto T0, auto T1, const int64_t step) {
        constexpr int t0 = decltype(T0)::value, t1 = decltype(T1)::value;
#pragma unroll
        for (int t = t0; t < t1; ++t) {
            kp[t] += step;
            load_frag16p<T, D>(kf[t], kp[t]);
        }
    };
    using IC0 = std::integral_constant<int, 0>;
    using ICL = std::integral_constant<int, KL>;
    using ICT = std::integral_constant<int, KT>;
    using ICLA = std::integral_constant<int, (KL + 1) / 2>;              // lower tiles [0, LA) | [LA, KL)
    using ICUA = std::integral_constant<int, KL + (KT - KL + 1) / 2>;    // upper tiles [KL, UA) | [UA, KT)
    mfma_tiles(IC0{}, ICL{}, 0);
    __builtin_amdgcn_sched_barrier(0);
    // Unconditional (a group with a single unit re-reads it): the compiler derives how long a wait
    // for older loads must be from the loads that certainly follow them on every path, so no load
    // of the steady state may sit behind a branch.
    issue_tiles(IC0{}, ICLA{}, nu > 1 ? kstep_to(1) : 0);
    __builtin_amdgcn_sched_barrier(0);

    // K requests are paced: the tile buffers are requested again at four points spread evenly
    // over an iteration (a quarter of the tiles each) instead of as soon as they are free, so
    // that the compute unit's memory pipeline sees a steady stream rather than bursts it cannot
    // absorb (a wave that issues into a full pipeline stalls).  Point 3 follows the lower tiles'
    // MFMAs at the end of an iteration (first half of the lower tiles, for the unit two ahead),
    // point 0 comes a quarter of an iteration later (their second half, by then for the next
    // unit), points 1 and 2 re-request the halves of the upper tiles for the next unit.
    auto issue_q = [&](const int64_t qstep) {
#pragma unroll
        for (int x = 0; x < QPW; ++x) {
            qp[x] += qstep;
            qland[x] = *reinterpret_cast<const uint4*>(qp[x]);
        }
    };
#define SNAPKV_ISSUE(cond_, what_)                                           \
    do {                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                   \
        if constexpr (cond_) { what_; }                                      \
        __builtin_amdgcn_sched_barrier(0);                                   \
    } while (0)

    // Loop-invariant parts of the hand-off addressing.  Step L1: this half-wave's first merge task
    // (further ones, for small groups, are addressed in the loop); step P2: this thread's words.
    const int task0 = wg + hw * F.Gg;
    const bool l1_mine = task0 < real_tasks;
    const int l1_row = l1_mine ? task0 / F.NB : 0, l1_blk = l1_mine ? task0 % F.NB : 0;
    const int l1_slice = l1_blk * kSlicesPerBlock + l32;
    const bool l1_lane = l1_mine && l1_slice < F.Gg;
    const float2* const l1_base = S.part + ((int64_t)group * F.Gg + (l1_lane ? l1_slice : 0)) * R + l1_row;
    const int64_t l1_step = (int64_t)F.NG * F.Gg * R;
    const float2* const p2_base = S.l1 + (int64_t)group * (R * NBP);
    const int64_t p2_step = (int64_t)F.NG * (R * NBP);
    bool p2_ok[L2PT];
    int p2_at[L2PT];                     // word this thread fetches (threads without one take word 0)
#pragma unroll
    for (int x = 0; x < L2PT; ++x) {
        const int idx = tid + x * NT;
        p2_ok[x] = idx < R * NBP && (idx & (NBP - 1)) < F.NBX;
        p2_at[x] = p2_ok[x] ? idx : 0;   // word 0 always exists: every wave waits for at least that one
    }

    // One iteration; MODE says (at compile time) whether the units one (bit 0) and two (bit 1)
    // steps ahead exist, so that every variant of the loop body has a fixed number of loads in
    // flight behind the hand-off words.
    auto iteration = [&](auto MODE, const int it) {
        constexpr bool kNext1 = (decltype(MODE)::value & 1) != 0;
        constexpr bool kNext2 = (decltype(MODE)::value & 2) != 0;
        const bool has_p1 = it < nu;
        const bool has_l1 = it >= 1 && it - 1 < nu;
        const bool has_p2 = it >= 2;
        const int unit = group + it * F.NG;
        const int unit_l1 = unit - F.NG;
        const int unit_p2 = unit - 2 * F.NG;
        const int64_t kstep = kNext1 ? kstep_to(it + 1) : 0;   // to the next unit's keys

        // ---- A. request this iteration's hand-off words at the very top: they are needed after
        // the arithmetic of step D, about one memory latency from now.  A wave's loads retire in
        // order: these are younger than this unit's K and Q (waited for next) and older than the
        // next unit's (issued below), so waiting for them never waits for those.
        // The loads are unconditional (lanes and iterations without a word re-read a valid one and
        // ignore it) so that their number is the same on every path.
        const float2* const l1_src = l1_base + (int64_t)(has_l1 ? it - 1 : 0) * l1_step;
        const unsigned long long l1_bits = load_pair_bits(l1_src);
        const float2* const p2_src = p2_base + (int64_t)(has_p2 ? it - 2 : 0) * p2_step;
        unsigned long long p2_bits[L2PT];
#pragma unroll
        for (int x = 0; x < L2PT; ++x) p2_bits[x] = load_pair_bits(p2_src + p2_at[x]);
        __builtin_amdgcn_sched_barrier(0);

        // ---- B. logits of the upper tiles of the slice (waits for their K; the lower tiles were
        // done at the end of the previous iteration)
        if (has_p1) mfma_tiles(ICL{}, ICT{}, it % 3);
        __builtin_amdgcn_sched_barrier(0);

        // ---- C. the next unit's Q and upper K tiles follow in portions between the steps below
        SNAPKV_ISSUE(kNext1, issue_q(qstep_to(it + 1)));

        float mref[RUW][4], zs[RUW][4];
        if (has_p1) {
            // ---- D. slice row maxima over this wave's keys (raw logits; scale is positive)
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int r = 0; r < 4; ++r) mref[ru][r] = -INFINITY;
            if (!special) {
#pragma unroll
                for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                    for (int t = 0; t < KT; ++t)
#pragma unroll
                        for (int r = 0; r < 4; ++r) mref[ru][r] = fmaxf(mref[ru][r], e[ru][t][r]);
            } else {
                // The lane's key position is made opaque to the optimiser here: otherwise the
                // (loop-invariant) mask of every accumulator element is hoisted out of the unit
                // loop and held in scalar registers for its whole duration.
                int jlane = tile0 * 16 + n16;
                asm volatile("" : "+v"(jlane));
                const int nn = (int)G.n, LL = (int)G.L;
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    const int j = jlane + t * TS * 16;
#pragma unroll
                    for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            // the row's place in the window (blocks of a longer window are heads to this kernel)
                            const int i = (ru % F.UH) * 16 + kg * 4 + r + ((unit * F.gs + ru / F.UH) % F.BH) * 32;
                            // prompt-phase causal mask; keys past the end of the prompt
                            if (j > nn + i || j >= LL) e[ru][t][r] = -INFINITY;
                            mref[ru][r] = fmaxf(mref[ru][r], e[ru][t][r]);
                        }
                }
            }
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int r = 0; r < 4; ++r) mref[ru][r] = row16_max(mref[ru][r]) * G.c2;   // base-2 domain
        }
        SNAPKV_ISSUE(kNext1, issue_tiles(ICLA{}, ICL{}, kstep));   // point 0
        if (has_p1) {
            // exponentials relative to the wave's own row maxima, and their row sums
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float ref = mref[ru][r] == -INFINITY ? 0.f : mref[ru][r];
                    float z = 0.f;
#pragma unroll
                    for (int t = 0; t < KT; ++t) {
                        const float x = __builtin_amdgcn_exp2f(fmaf(e[ru][t][r], G.c2, -ref));
                        e[ru][t][r] = x;
                        z += x;
                    }
                    zs[ru][r] = row16_sum(z);
                }
        }
        // ---- E. step P2 of the unit two back: level-1 words of a row sit in 16 neighbouring
        // lanes; merge them in a fixed tree into (max, 1/sum)
        if (has_p2) {
#pragma unroll
            for (int x = 0; x < L2PT; ++x) {
                const int idx = tid + x * NT;
                float m = -INFINITY, z = 0.f;
                const unsigned long long got = await_pair(p2_src + p2_at[x], p2_bits[x], F.spin_limit, gave_up);
                if (p2_ok[x]) unpack_pair(got, m, z);
                const float mm = row16_max(m);
                const float zz = row16_sum(m == -INFINITY ? 0.f : z * __builtin_amdgcn_exp2f(m - mm));
                if (idx < R * NBP && (idx & (NBP - 1)) == 0) {
                    const int row = idx / NBP, ru = row >> 4;
                    const int i = (ru % F.UH) * 16 + (row & 15);
                    const bool real = ru < F.RU && i < G.W && zz > 0.f;
                    sm_fin[it % 3][row] = real ? make_float2(mm, 1.0f / zz) : make_float2(0.f, 0.f);
                    if (S.lse_out && wg == 0 && real)   // for whoever scores further keys of these rows
                        S.lse_out[((int64_t)unit_p2 * F.gs + ru / F.UH) * G.W + i] = (mm + log2f(zz)) * 0.6931471805599453f;
                }
            }
        }
        if constexpr (kNext1) {   // the next unit's Q chunks
#pragma unroll
            for (int x = 0; x < QPW; ++x)
                if (w + x * NW < QCH) qbuf[(((it + 1) % 3) * QCH + w + x * NW) * 64 + lane] = qland[x];
        }
        if (has_p1 && n16 == 0) {
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                float4* dst = reinterpret_cast<float4*>(&sm_pair[it & 1][w][ru * 16 + kg * 4]);
                dst[0] = make_float4(mref[ru][0], zs[ru][0], mref[ru][1], zs[ru][1]);
                dst[1] = make_float4(mref[ru][2], zs[ru][2], mref[ru][3], zs[ru][3]);
                *reinterpret_cast<float4*>(&sm_ref[it % 3][w][ru * 16 + kg * 4]) =
                    make_float4(mref[ru][0], mref[ru][1], mref[ru][2], mref[ru][3]);
            }
        }
        // what this wave has written up to here is complete: stamp its three flags
        lds_release();
        if (lane < 3) lds_stamp(&sm_flag[lane][w], lane == 0 ? it + 2 : it + 1);
        SNAPKV_ISSUE(kNext1, issue_tiles(ICL{}, ICUA{}, kstep));   // point 1
        if (has_p1 && tid >= NT - R) {   // the last R threads merge the waves (in wave order) and publish
            const int row = tid - (NT - R);
            lds_await_all<NW>(sm_flag[1], it + 1, F.spin_limit, gave_up);
            float2 x[NW];
            float mm[NW], zz[NW];
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2) {
                x[w2] = sm_pair[it & 1][w2][row];
                mm[w2] = x[w2].x;
            }
#pragma unroll
            for (int d = 1; d < NW; d <<= 1)   // balanced trees: short dependency chains
#pragma unroll
                for (int w2 = 0; w2 + d < NW; w2 += 2 * d) mm[w2] = fmaxf(mm[w2], mm[w2 + d]);
            const float m = mm[0];
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2)
                zz[w2] = x[w2].x == -INFINITY ? 0.f : x[w2].y * __builtin_amdgcn_exp2f(x[w2].x - m);
#pragma unroll
            for (int d = 1; d < NW; d <<= 1)
#pragma unroll
                for (int w2 = 0; w2 + d < NW; w2 += 2 * d) zz[w2] += zz[w2 + d];
            publish_pair(&S.part[((int64_t)unit * F.Gg + wg) * R + row], m, zz[0]);
        }

        // ---- F. step L1 of the previous unit: merge 32 slices of one row per half-wave
        if (has_l1) {
            for (int task = task0; task < real_tasks; task += 2 * NW * F.Gg) {
                int row = l1_row, blk = l1_blk;
                float m = -INFINITY, z = 0.f;
                if (task == task0) {
                    if (l1_lane) unpack_pair(await_pair(l1_src, l1_bits, F.spin_limit, gave_up), m, z);
                } else {
                    row = task / F.NB;
                    blk = task % F.NB;
                    const int slice = blk * kSlicesPerBlock + l32;
                    if (slice < F.Gg) {
                        const float2* src = &S.part[((int64_t)unit_l1 * F.Gg + slice) * R + row];
                        unpack_pair(await_pair(src, load_pair_bits(src), F.spin_limit, gave_up), m, z);
                    }
                }
                // maximum over the half-wave's 32 slices, then the sums rescaled to it (fixed trees)
                float mm = row16_max(m);
                mm = fmaxf(mm, __shfl_xor(mm, 16, 64));
                float zz = m == -INFINITY ? 0.f : z * __builtin_amdgcn_exp2f(m - mm);
                zz = row16_sum(zz);
                zz += __shfl_xor(zz, 16, 64);
                if (l32 == 0) publish_pair(&S.l1[(int64_t)unit_l1 * (R * NBP) + row * NBP + blk], mm, zz);
            }
        }
        SNAPKV_ISSUE(kNext1, issue_tiles(ICUA{}, ICT{}, kstep));   // point 2
        if (has_p2) {
            lds_await_all<NW>(sm_flag[2], it + 1, F.spin_limit, gave_up);
            float f[RUW][4];
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                const float4* fin4 = reinterpret_cast<const float4*>(&sm_fin[it % 3][ru * 16 + kg * 4]);
                const float4 a = fin4[0], b = fin4[1];   // (m, 1/Z) of rows kg*4 .. kg*4+3
                const float4 ms = *reinterpret_cast<const float4*>(&sm_ref[(it + 1) % 3][w][ru * 16 + kg * 4]);
                f[ru][0] = (ms.x == -INFINITY || a.y == 0.f) ? 0.f : __builtin_amdgcn_exp2f(ms.x - a.x) * a.y;
                f[ru][1] = (ms.y == -INFINITY || a.w == 0.f) ? 0.f : __builtin_amdgcn_exp2f(ms.y - a.z) * a.w;
                f[ru][2] = (ms.z == -INFINITY || b.y == 0.f) ? 0.f : __builtin_amdgcn_exp2f(ms.z - b.x) * b.y;
                f[ru][3] = (ms.w == -INFINITY || b.w == 0.f) ? 0.f : __builtin_amdgcn_exp2f(ms.w - b.z) * b.w;
            }
            float* vb = vote + (int64_t)unit_p2 * F.gs * G.vpitch;
            int jst = tile0 * 16 + n16;       // opaque for the same reason as above
            asm volatile("" : "+v"(jst));
            const int nst = (int)G.n;
            float v[KT];
#pragma unroll
            for (int t = 0; t < KT; ++t) v[t] = 0.f;
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    f32x4 ev;
                    if constexpr (PARK) ev = park[((it & 1) * NSLOT + ru * KT + t) * NT + tid];   // left there at it - 2
                    else ev = e2[ru][t];
                    v[t] = fmaf(ev[0], f[ru][0], v[t]);
                    v[t] = fmaf(ev[1], f[ru][1], v[t]);
                    v[t] = fmaf(ev[2], f[ru][2], v[t]);
                    v[t] = fmaf(ev[3], f[ru][3], v[t]);
                }
                if ((ru + 1) % F.UH == 0) {   // last row unit of a query head: finish its votes
                    const int head = ru / F.UH;
                    float* vh = vb + (int64_t)head * G.vpitch;
                    // sum over the four contraction-slice lanes of a column; with several tiles
                    // the lanes split the tiles between them so that each stores its own share
                    if constexpr (KT >= 4) {
                        float a[KT / 2], b[KT / 4];
#pragma unroll
                        for (int x = 0; x < KT / 2; ++x) {
                            const float mine = (kg & 2) ? v[x + KT / 2] : v[x];
                            const float theirs = (kg & 2) ? v[x] : v[x + KT / 2];
                            a[x] = mine + __shfl_xor(theirs, 32, 64);
                        }
#pragma unroll
                        for (int x = 0; x < KT / 4; ++x) {
                            const float mine = (kg & 1) ? a[x + KT / 4] : a[x];
                            const float theirs = (kg & 1) ? a[x] : a[x + KT / 4];
                            b[x] = mine + __shfl_xor(theirs, 16, 64);
                        }
#pragma unroll
                        for (int x = 0; x < KT / 4; ++x) {
                            const int t = ((kg & 2) ? KT / 2 : 0) + ((kg & 1) ? KT / 4 : 0) + x;
                            const int j = jst + t * TS * 16;
                            if (head < F.gs && j < nst) VOTE_STORE(&vh[j], b[x]);
                        }
                    } else {
#pragma unroll
                        for (int t = 0; t < KT; ++t) {
                            float s = v[t] + __shfl_xor(v[t], 32, 64);
                            s += __shfl_xor(s, 16, 64);
                            const int j = jst + t * TS * 16;
                            if (kg == 0 && head < F.gs && j < nst) VOTE_STORE(&vh[j], s);
                        }
                    }
#pragma unroll
                    for (int t = 0; t < KT; ++t) v[t] = 0.f;
                }
            }
        }
        // ---- G. age the kept exponentials by one unit (PARK: this unit's take the place of the ones just voted on;
        // a thread reads back only what it wrote itself, in program order)
#pragma unroll
        for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                if constexpr (PARK) {
                    if (has_p1) park[((it & 1) * NSLOT + ru * KT + t) * NT + tid] = e[ru][t];
                } else {
                    e2[ru][t] = e1[ru][t];
                    e1[ru][t] = e[ru][t];
                }
            }
        // ---- H. the next unit's lower tiles meet its Q (in LDS since the barrier) and their
        // buffers are requested again for the unit after it
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kNext1) {
            lds_await_all<NW>(sm_flag[0], it + 2, F.spin_limit, gave_up);   // Q of the next unit
            mfma_tiles(IC0{}, ICL{}, (it + 1) % 3);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kNext2) issue_tiles(IC0{}, ICLA{}, kstep_to(it + 2));   // point 3
        __builtin_amdgcn_sched_barrier(0);
    };

#undef SNAPKV_ISSUE
    int it = 0;
    for (; it + 2 < nu; ++it) iteration(std::integral_constant<int, 3>{}, it);
    for (; it + 1 < nu; ++it) iteration(std::integral_constant<int, 1>{}, it);   // last but one unit
    for (; it < nu + 2; ++it) iteration(std::integral_constant<int, 0>{}, it);   // last unit, two drain steps
    if (gave_up) {
        atomicAdd(&g_sync_timeouts, 1u);
        if (S.gave_up_flag) __hip_atomic_store(S.gave_up_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <typename T, int D, int RUW, int KT, int NW>
__global__ __launch_bounds__(NW * 64) void score_fused(const void* __restrict__ qv,
                                                       const void* __restrict__ kv,
                                                       float* __restrict__ vote, const FusedSync S,
                                                       const ScoreGeom G, const FusedGeom F) {
    score_fused_body<T, D, RUW, KT, NW>(qv, kv, vote, S, G, F, (int)blockIdx.x);
}

template <typename T, int D, int RUW, int KT, int NW>
__global__ __launch_bounds__(NW * 64) void score_fused_layers(float* __restrict__ vote, const FusedSync S,
                                                              const ScoreGeom G, const FusedGeom F,
                                                              const ScoreLayers SL) {
    score_fused_body<T, D, RUW, KT, NW, true>(nullptr, nullptr, vote, S, G, F, (int)blockIdx.x, &SL);
}

// Several prompts of one model in one launch: every prompt has its own groups of workgroups
// (blocks wg_begin .. of the grid), its own hand-off words and vote rows, and runs exactly as in
// a launch of its own; together the prompts fill the chip that one short prompt leaves idle.
constexpr int kMaxJoint = kMaxJointPrompts;
struct FusedPrompt {
    const void* q;
    const void* k;
    float* vote;
    FusedSync S;
    ScoreGeom G;
    FusedGeom F;
    int wg_begin;
};
struct FusedJoint {
    int count;
    FusedPrompt p[kMaxJoint];
};

template <typename T, int D, int RUW, int KT, int NW>
__global__ __launch_bounds__(NW * 64) void score_fused_joint(const FusedJoint J) {
    int pi = 0;
    for (int i = 1; i < J.count; ++i)
        if ((int)blockIdx.x >= J.p[i].wg_begin) pi = i;
    const FusedPrompt& P = J.p[pi];
    const int bid = (int)blockIdx.x - P.wg_begin;
    if (bid >= P.F.NG * P.F.Gg) return;   // padding between two prompts' blocks
    score_fused_body<T, D, RUW, KT, NW>(P.q, P.k, P.vote, P.S, P.G, P.F, bid);
}


// ---------------------------------------------------------------------------------------------
// Scoring and voting when the window rows' log-sum-exp is handed in (the normalisers a block-wise
// attention prefill keeps per query row).  P[i, j] = exp(s[i, j] - lse[i]) needs nothing from other
// keys, so K is streamed once with no hand-off between workgroups at all: logits on MFMA, one
// exponential per logit, the column sum over the window rows of each query head (Eq. 1), store.
// Units, slices, the tile-to-key mapping, the shared Q block and the way K tile buffers are
// consumed in two halves and requested again at points spread over an iteration are those of
// score_fused; the waves of a workgroup meet at one LDS-only barrier per unit (for the Q block).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <typename T, int D, int RUW, int KT, int NW, bool STAT, bool LAYERS>
__device__ __forceinline__ void score_lse_body(const void* __restrict__ qv, const void* __restrict__ kv,
                                               const float* __restrict__ lse, float* __restrict__ vote,
                                               float2* __restrict__ stat_part, const ScoreGeom& G,
                                               const FusedGeom& F, const ScoreLayers* SL) {
    constexpr int R = RUW * 16;
    constexpr int NT = NW * 64;
    constexpr int ES = esize<T>::value;
    using Frag = Frag16<T, D>;
    constexpr int NP = Frag::NP;
    constexpr int QCH = RUW * NP;
    constexpr int QPW = (QCH + NW - 1) / NW;
    constexpr int KL = KT / 2;
    static_assert(R <= NT, "one thread per window row stages its log-sum-exp");
    extern __shared__ uint4 qbuf[];      // [2][QCH][64]: Q blocks of two consecutive units
    __shared__ __attribute__((aligned(16))) float sm_lse[2][R];   // base-2 log-sum-exp per row, +inf for padding rows
    __shared__ __attribute__((aligned(16))) float2 sm_stat[2][STAT ? NW : 1][R];   // STAT: per wave (row max, row sum-exp)

    const int tid = threadIdx.x, lane = tid & 63, n16 = lane & 15, kg = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = (int)(blockIdx.x % F.Gg), group = (int)(blockIdx.x / F.Gg);
    const int TS = F.Gg * NW;
    const int vwg = (F.Gg % 8 == 0) ? (wg % 8) * (F.Gg / 8) + wg / 8 : wg;
    const int tile0 = vwg * NW + w;
    const int nu = group < F.units ? (F.units - group + F.NG - 1) / F.NG : 0;
    if (nu == 0) return;
    const bool special = ((int64_t)(KT - 1) * TS + tile0 + 1) * 16 > G.n;

    // first K row of KV head h, first Q row of query head qh (LAYERS: as in score_fused_body)
    auto k_head = [&](const int h) -> const char* {
        if constexpr (LAYERS)
            return static_cast<const char*>(SL->k[h / SL->kv_heads]) + (int64_t)(h % SL->kv_heads) * G.k_hs;
        else
            return static_cast<const char*>(kv) + (int64_t)h * G.k_hs;
    };
    auto q_head = [&](const int qh) -> const char* {
        if constexpr (LAYERS) {
            const int per_layer = SL->kv_heads * G.g;
            return static_cast<const char*>(SL->q[qh / per_layer]) + (int64_t)(qh % per_layer) * G.W * D * ES;
        } else {
            return static_cast<const char*>(qv) + (int64_t)qh * G.W * D * ES;
        }
    };
    const char* kp[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        int64_t j = ((int64_t)t * TS + tile0) * 16 + n16;
        j = j < G.L ? j : G.L - 1;
        j = physical_row(G.k_table, G.k_page, G.k_pages, j + G.k_row0);
        kp[t] = k_head(group / F.split) + j * G.k_rs + kg * 16;
    }
    const char* qp[QPW];
#pragma unroll
    for (int x = 0; x < QPW; ++x) {
        int c = w + x * NW;
        c = c < QCH ? c : QCH - 1;
        const int ru = c / NP, pc = c % NP;
        int head = ru / F.UH, i = (ru % F.UH) * 16 + n16;
        head = head < F.gs ? head : F.gs - 1;
        i = i < G.W ? i : G.W - 1;
        qp[x] = q_head(group * F.gs + head) + (int64_t)i * D * ES + (4 * pc + kg) * 16;
    }
    // the window row whose log-sum-exp this thread stages (threads beyond R re-read row 0)
    const int lrow = tid < R ? tid : 0;
    const int lru = lrow >> 4, lhead = lru / F.UH, li = (lru % F.UH) * 16 + (lrow & 15);
    const bool lreal = tid < R && lru < F.RU && lhead < F.gs && li < G.W;
    const float* lp = lse + (int64_t)(group * F.gs + (lhead < F.gs ? lhead : F.gs - 1)) * G.W + (li < G.W ? li : G.W - 1);
    // from the rows of the group's unit itn - 1 to those of unit itn (NG is a multiple of split here)
    const int64_t kstep_even = (int64_t)(F.NG / F.split) * G.k_hs;
    const int64_t qstep_even = (int64_t)F.NG * F.gs * G.W * D * ES;
    auto kstep_to = [&](const int itn) -> int64_t {
        if constexpr (LAYERS) return k_head((group + itn * F.NG) / F.split) - k_head((group + (itn - 1) * F.NG) / F.split);
        return kstep_even;
    };
    auto qstep_to = [&](const int itn) -> int64_t {
        if constexpr (LAYERS) return q_head((group + itn * F.NG) * F.gs) - q_head((group + (itn - 1) * F.NG) * F.gs);
        return qstep_even;
    };
    const int64_t lstep = (int64_t)F.NG * F.gs * G.W;
    constexpr float kLog2e = 1.4426950408889634f;

    Frag kf[KT];
    uint4 qland[QPW];
    float lland;
    f32x4 e[RUW][KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) load_frag16p<T, D>(kf[t], kp[t]);
#pragma unroll
    for (int x = 0; x < QPW; ++x) qland[x] = *reinterpret_cast<const uint4*>(qp[x]);
    lland = STAT ? 0.f : *lp;
#pragma unroll
    for (int x = 0; x < QPW; ++x)
        if (w + x * NW < QCH) qbuf[(w + x * NW) * 64 + lane] = qland[x];
    if (tid < R) sm_lse[0][tid] = lreal ? lland * kLog2e : INFINITY;
    __syncthreads();
#pragma unroll
    for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
        for (int t = 0; t < KT; ++t) e[ru][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto mfma_tiles = [&](auto T0, auto T1, const int par) {
        constexpr int t0 = decltype(T0)::value, t1 = decltype(T1)::value;
        if constexpr (t0 < t1) {
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                Frag qf;
#pragma unroll
                for (int pc = 0; pc < NP; ++pc) qf.v[pc] = qbuf[(par * QCH + ru * NP + pc) * 64 + lane];
#pragma unroll
                for (int t = t0; t < t1; ++t) e[ru][t] = mfma16<D>(qf, kf[t]);
            }
        }
    };
    auto issue_tiles = [&](auto T0, auto T1, const int64_t step) {
        constexpr int t0 = decltype(T0)::value, t1 = decltype(T1)::value;
#pragma unroll
        for (int t = t0; t < t1; ++t) {
            kp[t] += step;
            load_frag16p<T, D>(kf[t], kp[t]);
        }
    };
    using IC0 = std::integral_constant<int, 0>;
    using ICL = std::integral_constant<int, KL>;
    using ICT = std::integral_constant<int, KT>;
    using ICLA = std::integral_constant<int, (KL + 1) / 2>;
    using ICUA = std::integral_constant<int, KL + (KT - KL + 1) / 2>;
    mfma_tiles(IC0{}, ICL{}, 0);
    __builtin_amdgcn_sched_barrier(0);
    issue_tiles(IC0{}, ICLA{}, nu > 1 ? kstep_to(1) : 0);   // unconditional: see score_fused
    __builtin_amdgcn_sched_barrier(0);

#define SNAPKV_LSE_ISSUE(cond_, what_)                                       \
    do {                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                   \
        if constexpr (cond_) { what_; }                                      \
        __builtin_amdgcn_sched_barrier(0);                                   \
    } while (0)

    auto iteration = [&](auto MODE, const int it) {
        constexpr bool kNext1 = (decltype(MODE)::value & 1) != 0;
        constexpr bool kNext2 = (decltype(MODE)::value & 2) != 0;
        const int unit = group + it * F.NG;
        const int64_t kstep = kNext1 ? kstep_to(it + 1) : 0;
        mfma_tiles(ICL{}, ICT{}, it & 1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kNext1) {   // the next unit's Q chunk and log-sum-exp
#pragma unroll
            for (int x = 0; x < QPW; ++x) {
                qp[x] += qstep_to(it + 1);
                qland[x] = *reinterpret_cast<const uint4*>(qp[x]);
            }
            if constexpr (!STAT) {
                lp += lstep;
                lland = *lp;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        SNAPKV_LSE_ISSUE(kNext1, issue_tiles(ICLA{}, ICL{}, kstep));   // point 0

        // masked logits; then probabilities (one exponential per logit, base-2 domain) or row statistics
        if (special) {
            int jlane = tile0 * 16 + n16;
            asm volatile("" : "+v"(jlane));
            const int nn = (int)G.n, LL = (int)G.L;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int j = jlane + t * TS * 16;
#pragma unroll
                for (int ru = 0; ru < RUW; ++ru)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // the row's place in the window (blocks of a longer window are heads to this kernel)
                        const int i = (ru % F.UH) * 16 + kg * 4 + r + ((unit * F.gs + ru / F.UH) % F.BH) * 32;
                        if (j > nn + i || j >= LL) e[ru][t][r] = -INFINITY;   // prompt-phase causal mask
                    }
            }
        }
        if constexpr (STAT && RUW == 1) {
            // (`vote` in this mode: null, or where the masked logits are kept for a reader that turns them
            // into votes once the rows' normalisers are known; a wave stores 1 KB per tile)
            if (vote) {
                float* lb = vote + (int64_t)unit * ((int64_t)F.Gg * NW * KT * 16) * 16;
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    const int64_t j = ((int64_t)t * TS + tile0) * 16 + n16;
                    __builtin_nontemporal_store(e[0][t], reinterpret_cast<f32x4*>(lb + j * 16 + kg * 4));
                }
            }
        }
        if constexpr (STAT) {
            // row maxima and sums of exponentials of this wave's keys (base-2 domain), left in LDS
            // for the merge over the waves after the barrier
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                float mref[4], zs[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float m = -INFINITY;
#pragma unroll
                    for (int t = 0; t < KT; ++t) m = fmaxf(m, e[ru][t][r]);
                    mref[r] = row16_max(m) * G.c2;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float ref = mref[r] == -INFINITY ? 0.f : mref[r];
                    float z = 0.f;
#pragma unroll
                    for (int t = 0; t < KT; ++t) z += __builtin_amdgcn_exp2f(fmaf(e[ru][t][r], G.c2, -ref));
                    zs[r] = row16_sum(z);
                }
                if (n16 == 0) {
                    float4* dst = reinterpret_cast<float4*>(&sm_stat[it & 1][w][ru * 16 + kg * 4]);
                    dst[0] = make_float4(mref[0], zs[0], mref[1], zs[1]);
                    dst[1] = make_float4(mref[2], zs[2], mref[3], zs[3]);
                }
            }
        } else {
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
                const float4 l2 = *reinterpret_cast<const float4*>(&sm_lse[it & 1][ru * 16 + kg * 4]);
                const float l[4] = {l2.x, l2.y, l2.z, l2.w};
#pragma unroll
                for (int t = 0; t < KT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) e[ru][t][r] = __builtin_amdgcn_exp2f(fmaf(e[ru][t][r], G.c2, -l[r]));
            }
        }
        SNAPKV_LSE_ISSUE(kNext1, issue_tiles(ICL{}, ICUA{}, kstep));   // point 1

        // votes: sum over the window rows of each query head, then over the four lanes of a column
        if constexpr (!STAT) {
            float* vb = vote + (int64_t)unit * F.gs * G.vpitch;
            int jst = tile0 * 16 + n16;
            asm volatile("" : "+v"(jst));
            const int nst = (int)G.n;
            float v[KT];
#pragma unroll
            for (int t = 0; t < KT; ++t) v[t] = 0.f;
#pragma unroll
            for (int ru = 0; ru < RUW; ++ru) {
#pragma unroll
                for (int t = 0; t < KT; ++t) {
                    const f32x4 ev = e[ru][t];
                    v[t] += (ev[0] + ev[1]) + (ev[2] + ev[3]);
                }
                if ((ru + 1) % F.UH == 0) {
                    const int head = ru / F.UH;
                    float* vh = vb + (int64_t)head * G.vpitch;
                    if constexpr (KT >= 4) {
                        float a[KT / 2], b[KT / 4];
#pragma unroll
                        for (int x = 0; x < KT / 2; ++x) {
                            const float mine = (kg & 2) ? v[x + KT / 2] : v[x];
                            const float theirs = (kg & 2) ? v[x] : v[x + KT / 2];
                            a[x] = mine + __shfl_xor(theirs, 32, 64);
                        }
#pragma unroll
                        for (int x = 0; x < KT / 4; ++x) {
                            const float mine = (kg & 1) ? a[x + KT / 4] : a[x];
                            const float theirs = (kg & 1) ? a[x] : a[x + KT / 4];
                            b[x] = mine + __shfl_xor(theirs, 16, 64);
                        }
#pragma unroll
                        for (int x = 0; x < KT / 4; ++x) {
                            const int t = ((kg & 2) ? KT / 2 : 0) + ((kg & 1) ? KT / 4 : 0) + x;
                            const int j = jst + t * TS * 16;
                            if (head < F.gs && j < nst) VOTE_STORE(&vh[j], b[x]);
                        }
                    } else {
#pragma unroll
                        for (int t = 0; t < KT; ++t) {
                            float sum = v[t] + __shfl_xor(v[t], 32, 64);
                            sum += __shfl_xor(sum, 16, 64);
                            const int j = jst + t * TS * 16;
                            if (kg == 0 && head < F.gs && j < nst) VOTE_STORE(&vh[j], sum);
                        }
                    }
#pragma unroll
                    for (int t = 0; t < KT; ++t) v[t] = 0.f;
                }
            }
        }
        SNAPKV_LSE_ISSUE(kNext1, issue_tiles(ICUA{}, ICT{}, kstep));   // point 2
        if constexpr (kNext1) {
#pragma unroll
            for (int x = 0; x < QPW; ++x)
                if (w + x * NW < QCH) qbuf[(((it + 1) & 1) * QCH + w + x * NW) * 64 + lane] = qland[x];
            if (!STAT && tid < R) sm_lse[(it + 1) & 1][tid] = lreal ? lland * kLog2e : INFINITY;
        }
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (STAT) {
            if (tid >= NT - R) {   // the last R threads merge the waves (fixed trees) and store the slice's pair
                const int row = tid - (NT - R);
                float2 x[NW];
                float mm[NW], zz[NW];
#pragma unroll
                for (int w2 = 0; w2 < NW; ++w2) {
                    x[w2] = sm_stat[it & 1][w2][row];
                    mm[w2] = x[w2].x;
                }
#pragma unroll
                for (int d = 1; d < NW; d <<= 1)
#pragma unroll
                    for (int w2 = 0; w2 + d < NW; w2 += 2 * d) mm[w2] = fmaxf(mm[w2], mm[w2 + d]);
                const float m = mm[0];
#pragma unroll
                for (int w2 = 0; w2 < NW; ++w2)
                    zz[w2] = x[w2].x == -INFINITY ? 0.f : x[w2].y * __builtin_amdgcn_exp2f(x[w2].x - m);
#pragma unroll
                for (int d = 1; d < NW; d <<= 1)
#pragma unroll
                    for (int w2 = 0; w2 + d < NW; w2 += 2 * d) zz[w2] += zz[w2 + d];
                stat_part[((int64_t)unit * F.Gg + wg) * R + row] = make_float2(m, zz[0]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kNext1) mfma_tiles(IC0{}, ICL{}, (it + 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (kNext2) issue_tiles(IC0{}, ICLA{}, kstep_to(it + 2));   // point 3
        __builtin_amdgcn_sched_barrier(0);
    };
#undef SNAPKV_LSE_ISSUE
    int it = 0;
    for (; it + 2 < nu; ++it) iteration(std::integral_constant<int, 3>{}, it);
    for (; it + 1 < nu; ++it) iteration(std::integral_constant<int, 1>{}, it);
    for (; it < nu; ++it) iteration(std::integral_constant<int, 0>{}, it);
}

template <typename T, int D, int RUW, int KT, int NW, bool STAT>
__global__ __launch_bounds__(NW * 64) void score_lse(const void* __restrict__ qv,
                                                     const void* __restrict__ kv,
                                                     const float* __restrict__ lse,
                                                     float* __restrict__ vote,
                                                     float2* __restrict__ stat_part, const ScoreGeom G,
                                                     const FusedGeom F) {
    score_lse_body<T, D, RUW, KT, NW, STAT, false>(qv, kv, lse, vote, stat_part, G, F, nullptr);
}

// The same over the heads of several separately allocated layers (see score_fused_layers).
template <typename T, int D, int RUW, int KT, int NW, bool STAT>
__global__ __launch_bounds__(NW * 64) void score_lse_layers(const float* __restrict__ lse, float* __restrict__ vote,
                                                            float2* __restrict__ stat_part, const ScoreGeom G,
                                                            const FusedGeom F, const ScoreLayers SL) {
    score_lse_body<T, D, RUW, KT, NW, STAT, true>(nullptr, nullptr, lse, vote, stat_part, G, F, &SL);
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
constexpr unsigned kSpinLimit = 1u << 15;   // polls before a hand-off wait gives up (tens of ms)

static int g_cu_count[64] = {0};
int g_fused_slot_cap = 0;

// Workgroups of the single-read kernel that are resident together, given how many fit a compute unit.
static int64_t resident_slots(int occ);

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

static int64_t resident_slots(int occ) {
    const int64_t slots = (int64_t)cu_count() * occ;
    return g_fused_slot_cap > 0 && slots > g_fused_slot_cap ? g_fused_slot_cap : slots;
}

constexpr int kFusedWaves = 8;          // waves per workgroup (two per SIMD): measured best

// Device-independent part of the plan: how the rows and keys of a unit map onto a workgroup of
// NW waves.  Returns false when the window rows of a KV head exceed what one wave tracks.
static bool fused_shape_nw(const ScoreGeom& G, int NW, int split, FusedGeom* F, bool capped = true) {
    if (split < 1 || G.g % split != 0) return false;
    const int UH = (G.W + 15) / 16;
    const int gs = G.g / split;          // query heads per unit
    const int RU = gs * UH;
    if (RU > 8 || G.n <= 0) return false;
    int RUW = 1;
    while (RUW < RU) RUW *= 2;
    const int KT = kFusedSlots / RUW;
    const int64_t ntiles = (G.L + 15) / 16;
    const int64_t per_wg = (int64_t)NW * KT;
    const int64_t Gg = (ntiles + per_wg - 1) / per_wg;
    if (capped && Gg > 32 * kL1BlocksPadded) return false;   // level-1 merge blocks per row are capped
    if (Gg > (1 << 20)) return false;
    F->RU = RU;
    F->UH = UH;
    F->RUW = RUW;
    F->KT = KT;
    F->NW = NW;
    F->Gg = (int)Gg;
    F->NG = split;
    F->NB = (int)((Gg + 31) / 32);
    F->NBX = F->NB;
    F->ntiles = ntiles;
    F->units = G.Hkv * split;
    F->split = split;
    F->gs = gs;
    F->BH = 1;
    F->spin_limit = wait_limit(kSpinLimit);
    return true;
}

// The geometry in which every 32-row block of the window counts as a query head (windows of 64, 96,
// ... rows): the rows of a block keep their softmax to themselves, so a block is to the kernel what
// a query head is, except that its rows' causal mask starts 32 * (block index) rows later.
static bool block_geom(const ScoreGeom& G, ScoreGeom* Gs) {
    if (G.W <= 32 || G.W % 32 != 0) return false;
    *Gs = G;
    Gs->g = G.g * G.BH;
    Gs->W = 32;
    Gs->BH = 1;
    Gs->VB = 1;
    Gs->NV = Gs->g;
    return true;
}

// Splits worth trying, best first: the finest one whose units still have two row units (the
// kernel's leanest form), then the others from fine to coarse.  Returns how many (at most 8).
static int fused_split_candidates(const ScoreGeom& G, int* out) {
    const int UH = (G.W + 15) / 16;
    int all[8], na = 0;
    for (int s = G.g; s >= 1 && na < 8; --s)
        if (G.g % s == 0 && (G.g / s) * UH <= 8) all[na++] = s;
    if (na == 0) return 0;
    int best = na - 1;
    for (int i = 0; i < na; ++i)
        if ((G.g / all[i]) * UH >= 2) {
            best = i;
            break;
        }
    int nc = 0;
    out[nc++] = all[best];
    for (int i = 0; i < na; ++i)
        if (i != best) out[nc++] = all[i];
    return nc;
}

size_t fused_sync_layout(const ScoreGeom& G, const FusedGeom& F, FusedSync* S, void* base);

// Bytes of hand-off buffers that cover whichever split the launch plan ends up choosing, for any
// prompt length: the size depends on the heads and the window only, so that what follows the
// buffers in a workspace never moves onto them when the length changes.
size_t fused_sync_bytes(const ScoreGeom& G) {
    size_t most = 0;
    ScoreGeom Gs;
    const ScoreGeom* geoms[2] = {&G, block_geom(G, &Gs) ? &Gs : nullptr};
    for (const ScoreGeom* g : geoms) {
        if (!g) continue;
        int cand[8];
        const int nc = fused_split_candidates(*g, cand);
        for (int i = 0; i < nc; ++i) {
            FusedGeom F;
            if (!fused_shape_nw(*g, kFusedWaves, cand[i], &F, false)) continue;
            F.Gg = 32 * kL1BlocksPadded;   // the most slices a launch can have
            const size_t b = fused_sync_layout(*g, F, nullptr, nullptr);
            most = b > most ? b : most;
        }
    }
    return most;
}

size_t fused_sync_layout(const ScoreGeom& G, const FusedGeom& F, FusedSync* S, void* base) {
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t R = (size_t)F.RUW * 16;
    const size_t part = sizeof(float2) * (size_t)F.units * F.Gg * R;   // l1 follows part directly
    const size_t l1 = sizeof(float2) * (size_t)F.units * R * kL1BlocksPadded;
    if (S) {
        char* b = static_cast<char*>(base);
        S->part = reinterpret_cast<float2*>(b);
        S->l1 = reinterpret_cast<float2*>(b + part);
        S->gave_up_flag = nullptr;
        S->lse_out = nullptr;
    }
    return up(part + l1);
}

// Hand-off words (part and l1, adjacent) that must hold the "not published" pattern at launch.
int64_t fused_sync_pairs(const FusedGeom& F) {
    return (int64_t)F.units * (F.RUW * 16) * (F.Gg + kL1BlocksPadded);
}

struct FusedCall {
    const void* q;
    const void* k;
    const ScoreGeom* G;
    const FusedGeom* F;
    const FusedSync* S;
    float* vote;
    hipStream_t st;
};

// call == nullptr: returns in *occ how many workgroups of this instance fit one compute unit
// (asked of the runtime, so that a launch never exceeds what is resident at the same time).
template <typename T, int D, int RUW, int NW>
static hipError_t fused_instance(const FusedCall* call, int* occ) {
    constexpr int KT = kFusedSlots / RUW;
    auto kern = score_fused<T, D, RUW, KT, NW>;
    constexpr int kQueueBytes = fused_lds_bytes<T, D, RUW, NW>();
    static int cached_occ = -1;
    if (cached_occ < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kQueueBytes);
        if (e != hipSuccess) return e;
        int n = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, NW * 64, kQueueBytes);
        if (e != hipSuccess) return e;
        cached_occ = n;
    }
    if (occ) *occ = cached_occ;
    if (!call) return hipSuccess;
    const FusedGeom& F = *call->F;
    if ((int64_t)F.NG * F.Gg > (int64_t)cached_occ * cu_count()) return hipErrorCooperativeLaunchTooLarge;
    hipLaunchKernelGGL(kern, dim3(F.NG * F.Gg), dim3(NW * 64), kQueueBytes, call->st, call->q, call->k,
                       call->vote, *call->S, *call->G, F);
    return hipGetLastError();
}

template <typename T, int D, int NW>
static hipError_t fused_by_rows(int RUW, const FusedCall* call, int* occ) {
    switch (RUW) {
        case 1: return fused_instance<T, D, 1, NW>(call, occ);
        case 2: return fused_instance<T, D, 2, NW>(call, occ);
        case 4: return fused_instance<T, D, 4, NW>(call, occ);
        case 8: return fused_instance<T, D, 8, NW>(call, occ);
    }
    return hipErrorInvalidValue;
}

template <typename T, int D>
static hipError_t fused_by_waves(int NW, int RUW, const FusedCall* call, int* occ) {
    if (NW == kFusedWaves) return fused_by_rows<T, D, kFusedWaves>(RUW, call, occ);
    return hipErrorInvalidValue;
}

static hipError_t fused_dispatch(int dtype, int D, int NW, int RUW, const FusedCall* call, int* occ) {
    if (dtype == 0) {
        if (D == 128) return fused_by_waves<bf16_k, 128>(NW, RUW, call, occ);
        if (D == 64) return fused_by_waves<bf16_k, 64>(NW, RUW, call, occ);
    } else if (dtype == 2) {
        if (D == 128) return fused_by_waves<f16_k, 128>(NW, RUW, call, occ);
        if (D == 64) return fused_by_waves<f16_k, 64>(NW, RUW, call, occ);
    } else {
        if (D == 128) return fused_by_waves<f32_k, 128>(NW, RUW, call, occ);
        if (D == 64) return fused_by_waves<f32_k, 64>(NW, RUW, call, occ);
    }
    return hipErrorInvalidValue;
}

// Whether the current device can keep a whole group of workgroups resident, and how many groups
// run side by side.  The number of resident workgroups comes from the runtime's occupancy
// answer for the exact kernel instance, never from an assumption.
static bool fused_plan_for(int dtype, int D, const ScoreGeom& G, FusedGeom* F);

bool fused_plan(int dtype, int D, const ScoreGeom& G, FusedGeom* F, bool allow_blocks) {
    ScoreGeom Gs;
    if (allow_blocks && block_geom(G, &Gs) && fused_plan_for(dtype, D, Gs, F)) {
        F->BH = G.BH;
        return true;
    }
    return fused_plan_for(dtype, D, G, F);
}

static bool fused_plan_for(int dtype, int D, const ScoreGeom& G, FusedGeom* F) {
    int cand[8];
    const int nc = fused_split_candidates(G, cand);
    for (int c = 0; c < nc; ++c) {
        if (!fused_shape_nw(G, kFusedWaves, cand[c], F)) continue;
        int occ = 0;
        if (fused_dispatch(dtype, D, F->NW, F->RUW, nullptr, &occ) != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        const int64_t slots = resident_slots(occ);
        if (slots <= 0 || F->Gg > slots) continue;          // one unit's logits do not fit on the chip
        int64_t NG = slots / F->Gg;
        if (NG > F->units) NG = F->units;
        if (NG >= F->split) {
            NG -= NG % F->split;  // the parts of a KV head run side by side, in neighbouring groups
        } else {                  // or, when the prompt leaves no room for that, one after another on the same groups
            while (NG > 1 && F->split % NG != 0) --NG;
        }
        if (NG < 1) continue;
        F->NG = (int)NG;
        return true;
    }
    return false;
}

// ---- prompts longer than the chip's registers hold: a front part read once, the rest read twice
bool long_plan(int dtype, int D, const ScoreGeom& G, LongPlan* P) {
    int cand[8];
    const int nc = fused_split_candidates(G, cand);
    for (int c = 0; c < nc; ++c) {
        FusedGeom F;
        if (!fused_shape_nw(G, kFusedWaves, cand[c], &F, false)) continue;
        int occ = 0;
        if (fused_dispatch(dtype, D, F.NW, F.RUW, nullptr, &occ) != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        const int64_t wg_keys = (int64_t)F.NW * F.KT * 16;
        int64_t Gg = resident_slots(occ);
        // one level-1 word per row is kept for the rest's statistics
        if (Gg > kSlicesPerBlock * (kL1BlocksPadded - 1)) Gg = kSlicesPerBlock * (kL1BlocksPadded - 1);
        Gg -= Gg % 8;
        // the rest is a prompt of its own: the window and at least one key before it
        while (Gg >= 8 && G.L - Gg * wg_keys <= G.W) Gg -= 8;
        if (Gg < 8) continue;
        P->front = Gg * wg_keys;
        P->Gf = G;
        P->Gf.L = P->front;   // every key of the front part is before the window: no causal mask, all are voted on
        P->Gf.n = P->front;
        if (!fused_shape_nw(P->Gf, kFusedWaves, cand[c], &P->Ff, true) || P->Ff.Gg != Gg) continue;
        P->Ff.NG = 1;
        P->Ff.NBX = P->Ff.NB + 1;
        P->Gr = G;
        P->Gr.L = G.L - P->front;
        P->Gr.n = G.n - P->front;
        if (G.k_table) P->Gr.k_row0 = G.k_row0 + P->front;   // paged rows: the rest starts at a logical row, not at an address
        if (!lse_plan(dtype, D, P->Gr, &P->Fr) || P->Fr.split != P->Ff.split || P->Fr.RUW != P->Ff.RUW) continue;
        return true;
    }
    return false;
}

// Per window row of a unit: the (max, sum-exp) pairs of the rest's slices merged in a fixed order into the
// level-1 word behind the single-read kernel's own.  One workgroup per unit; 1024 / R threads share a row.
__global__ __launch_bounds__(1024) void publish_rest(const float2* __restrict__ part, float2* __restrict__ l1,
                                                    const int slices, const int R, const int slot) {
    __shared__ float2 sh[1024];
    const int unit = blockIdx.x, tid = threadIdx.x;
    const int S = 1024 / R;
    const int row = tid % R, sub = tid / R;
    float m = -INFINITY, z = 0.f;
    if (sub < S)
        for (int sl = sub; sl < slices; sl += S) {
            const float2 pc = part[((int64_t)unit * slices + sl) * R + row];
            merge_pair(m, z, pc.x, pc.y);
        }
    sh[tid] = make_float2(m, z);
    __syncthreads();
    if (sub == 0) {
        for (int c = 1; c < S; ++c) {
            const float2 pc = sh[c * R + row];
            merge_pair(m, z, pc.x, pc.y);
        }
        publish_pair(&l1[(int64_t)unit * (R * kL1BlocksPadded) + row * kL1BlocksPadded + slot], m, z);
    }
}

hipError_t launch_publish_rest(const float2* stat_part, const FusedSync& S, const LongPlan& P, hipStream_t st) {
    if (P.Ff.NBX != P.Ff.NB + 1 || P.Ff.NBX > kL1BlocksPadded || P.Fr.units != P.Ff.units) return hipErrorInvalidValue;
    hipLaunchKernelGGL(publish_rest, dim3(P.Ff.units), dim3(1024), 0, st, stat_part, S.l1, P.Fr.Gg, P.Ff.RUW * 16,
                       P.Ff.NB);
    return hipGetLastError();
}

// ---- several prompts in one launch
template <typename T, int D, int RUW, int NW>
static hipError_t joint_instance(const FusedJoint* J, int grid, hipStream_t st, int* occ) {
    constexpr int KT = kFusedSlots / RUW;
    auto kern = score_fused_joint<T, D, RUW, KT, NW>;
    constexpr int kQueueBytes = fused_lds_bytes<T, D, RUW, NW>();
    static int cached_occ = -1;
    if (cached_occ < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kQueueBytes);
        if (e != hipSuccess) return e;
        int n = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, NW * 64, kQueueBytes);
        if (e != hipSuccess) return e;
        cached_occ = n;
    }
    if (occ) *occ = cached_occ;
    if (!J) return hipSuccess;
    if ((int64_t)grid > (int64_t)cached_occ * cu_count()) return hipErrorCooperativeLaunchTooLarge;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), kQueueBytes, st, *J);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t joint_by_rows(int RUW, const FusedJoint* J, int grid, hipStream_t st, int* occ) {
    switch (RUW) {
        case 1: return joint_instance<T, D, 1, kFusedWaves>(J, grid, st, occ);
        case 2: return joint_instance<T, D, 2, kFusedWaves>(J, grid, st, occ);
        case 4: return joint_instance<T, D, 4, kFusedWaves>(J, grid, st, occ);
        case 8: return joint_instance<T, D, 8, kFusedWaves>(J, grid, st, occ);
    }
    return hipErrorInvalidValue;
}

// Two-byte storage types only: the joint launch serves batches of short prompts.
static hipError_t joint_dispatch(int dtype, int D, int RUW, const FusedJoint* J, int grid, hipStream_t st, int* occ) {
    if (dtype == 0) {
        if (D == 128) return joint_by_rows<bf16_k, 128>(RUW, J, grid, st, occ);
        if (D == 64) return joint_by_rows<bf16_k, 64>(RUW, J, grid, st, occ);
    } else if (dtype == 2) {
        if (D == 128) return joint_by_rows<f16_k, 128>(RUW, J, grid, st, occ);
        if (D == 64) return joint_by_rows<f16_k, 64>(RUW, J, grid, st, occ);
    }
    return hipErrorInvalidValue;
}

static int up8(int x) { return (x + 7) & ~7; }

// Plans one joint launch over some of the prompts G[0..count), scanned in the order given (the
// caller puts the longest first): take[] gets the indices taken (at most kMaxJoint), F[i] of a taken
// prompt its shape and its number of groups, wg_begin[t] the first block of the t-th taken prompt (a
// multiple of eight, so that the die of a workgroup is the same as in a launch of its own), *grid
// the blocks of the launch.  Returns how many prompts the launch takes; 0 when G[0] cannot use the
// kernel at all.  Every prompt gets at least one group per part of a KV head; what the chip has
// left over goes, a step at a time, to the prompt with the most iterations still to run.
int fused_joint_plan(int dtype, int D, int count, const ScoreGeom* G, FusedGeom* F, int* take, int* wg_begin,
                     int* grid) {
    if (count < 1 || (dtype != 0 && dtype != 2)) return 0;
    if (!fused_plan(dtype, D, G[0], &F[0])) return 0;
    int occ = 0;
    if (joint_dispatch(dtype, D, F[0].RUW, nullptr, 0, nullptr, &occ) != hipSuccess) {
        (void)hipGetLastError();
        return 0;
    }
    const int slots = cu_count() * occ;
    int taken = 0, total = 0;
    for (int i = 0; i < count && taken < kMaxJoint; ++i) {
        if (i > 0 && (!fused_plan(dtype, D, G[i], &F[i]) || F[i].RUW != F[0].RUW || F[i].split != F[0].split ||
                      F[i].NW != F[0].NW))
            continue;
        // a prompt joins with one group (the parts of its KV heads then follow one another); the
        // spare blocks go to whoever has most iterations left
        const int least = up8(F[i].Gg);
        if (total + least > slots) {
            if (i == 0) return 0;
            continue;
        }
        F[i].NG = 1;
        total += least;
        take[taken++] = i;
    }
    // the next number of groups a prompt can have: a divisor of split below it, a multiple of it above
    auto next_groups = [](const FusedGeom& f) {
        if (f.NG >= f.split) return f.NG + f.split;
        int n = f.NG + 1;
        while (f.split % n != 0) ++n;
        return n;
    };
    for (;;) {   // hand the spare blocks out
        int best = -1, best_iters = 0;
        for (int t = 0; t < taken; ++t) {
            const FusedGeom& f = F[take[t]];
            const int nx = next_groups(f);
            if (nx > f.units) continue;
            const int more = up8(nx * f.Gg) - up8(f.NG * f.Gg);
            const int iters = (f.units + f.NG - 1) / f.NG;
            if (total + more <= slots && iters > best_iters) {
                best = t;
                best_iters = iters;
            }
        }
        if (best < 0 || best_iters <= 1) break;
        FusedGeom& f = F[take[best]];
        const int nx = next_groups(f);
        total += up8(nx * f.Gg) - up8(f.NG * f.Gg);
        f.NG = nx;
    }
    int at = 0;
    for (int t = 0; t < taken; ++t) {
        wg_begin[t] = at;
        at += up8(F[take[t]].NG * F[take[t]].Gg);
    }
    *grid = at;
    return taken;
}

hipError_t launch_score_fused_joint(int dtype, int D, int count, const void* const* q, const void* const* k,
                                    const ScoreGeom* G, const FusedGeom* F, const FusedSync* S, float* const* vote,
                                    const int* wg_begin, int grid, hipStream_t st) {
    if (count < 1 || count > kMaxJoint) return hipErrorInvalidValue;
    FusedJoint J;
    J.count = count;
    for (int i = 0; i < count; ++i) {
        if (G[i].n <= 0) return hipErrorInvalidValue;
        J.p[i].q = q[i];
        J.p[i].k = k[i];
        J.p[i].vote = vote[i];
        J.p[i].S = S[i];
        J.p[i].G = G[i];
        J.p[i].F = F[i];
        J.p[i].wg_begin = wg_begin[i];
    }
    for (int i = count; i < kMaxJoint; ++i) J.p[i] = J.p[0];
    return joint_dispatch(dtype, D, F[0].RUW, &J, grid, st, nullptr);
}

hipError_t launch_score_fused(int dtype, int D, const void* q, const void* k, const ScoreGeom& G,
                              const FusedGeom& F, const FusedSync& S, float* vote, hipStream_t st) {
    if (G.n <= 0) return hipSuccess;
    ScoreGeom Gl = G;
    if (F.BH > 1 && !block_geom(G, &Gl)) return hipErrorInvalidValue;
    const FusedCall call{q, k, &Gl, &F, &S, vote, st};
    return fused_dispatch(dtype, D, F.NW, F.RUW, &call, nullptr);
}

// ---- the heads of several separately allocated layers in one launch
template <typename T, int D, int RUW>
static hipError_t layers_instance(const ScoreLayers& SL, const ScoreGeom& G, const FusedGeom& F, const FusedSync& S,
                                  float* vote, hipStream_t st, bool probe_only) {
    constexpr int NW = kFusedWaves, KT = kFusedSlots / RUW;
    auto kern = score_fused_layers<T, D, RUW, KT, NW>;
    constexpr int kQueueBytes = fused_lds_bytes<T, D, RUW, NW>();
    static int cached_occ = -1;
    if (cached_occ < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kQueueBytes);
        if (e != hipSuccess) return e;
        int n = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, NW * 64, kQueueBytes);
        if (e != hipSuccess) return e;
        cached_occ = n;
    }
    if ((int64_t)F.NG * F.Gg > resident_slots(cached_occ)) return hipErrorCooperativeLaunchTooLarge;
    if (probe_only) return hipSuccess;
    hipLaunchKernelGGL(kern, dim3(F.NG * F.Gg), dim3(NW * 64), kQueueBytes, st, vote, S, G, F, SL);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t layers_by_rows(const ScoreLayers& SL, const ScoreGeom& G, const FusedGeom& F, const FusedSync& S,
                                 float* vote, hipStream_t st, bool probe_only) {
    switch (F.RUW) {
        case 1: return layers_instance<T, D, 1>(SL, G, F, S, vote, st, probe_only);
        case 2: return layers_instance<T, D, 2>(SL, G, F, S, vote, st, probe_only);
        case 4: return layers_instance<T, D, 4>(SL, G, F, S, vote, st, probe_only);
        case 8: return layers_instance<T, D, 8>(SL, G, F, S, vote, st, probe_only);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_score_fused_layers(int dtype, int D, const ScoreLayers& SL, const ScoreGeom& G, const FusedGeom& F,
                                     const FusedSync& S, float* vote, hipStream_t st, bool probe_only) {
    if (SL.count < 1 || SL.count > kMaxLayerPtrs || SL.kv_heads < 1 || SL.count * SL.kv_heads != G.Hkv) return hipErrorInvalidValue;
    if (F.BH != 1 || F.NW != kFusedWaves || G.k_table || G.n <= 0) return hipErrorInvalidValue;
    if (dtype == 0) {
        if (D == 128) return layers_by_rows<bf16_k, 128>(SL, G, F, S, vote, st, probe_only);
        if (D == 64) return layers_by_rows<bf16_k, 64>(SL, G, F, S, vote, st, probe_only);
    } else if (dtype == 2) {
        if (D == 128) return layers_by_rows<f16_k, 128>(SL, G, F, S, vote, st, probe_only);
        if (D == 64) return layers_by_rows<f16_k, 64>(SL, G, F, S, vote, st, probe_only);
    }
    return hipErrorInvalidValue;
}

// ---- the streaming kernel: probabilities from a given log-sum-exp, or the row statistics that give it
// Per window row: merge the slices' (max, sum-exp) pairs (base-2 domain) in a fixed order and store
// the row's natural log-sum-exp.  One workgroup per unit; 1024 / R threads share a row.
__global__ __launch_bounds__(1024) void lse_from_parts(const float2* __restrict__ part, float* __restrict__ lse,
                                                      const ScoreGeom G, const FusedGeom F) {
    __shared__ float2 sh[1024];
    const int unit = blockIdx.x, tid = threadIdx.x;
    const int R = F.RUW * 16, S = 1024 / R;
    const int row = tid % R, sub = tid / R;
    float m = -INFINITY, z = 0.f;
    if (sub < S)
        for (int sl = sub; sl < F.Gg; sl += S) {
            const float2 pc = part[((int64_t)unit * F.Gg + sl) * R + row];
            merge_pair(m, z, pc.x, pc.y);
        }
    sh[tid] = make_float2(m, z);
    __syncthreads();
    if (sub == 0) {
        for (int c = 1; c < S; ++c) {
            const float2 pc = sh[c * R + row];
            merge_pair(m, z, pc.x, pc.y);
        }
        const int ru = row >> 4, head = ru / F.UH, i = (ru % F.UH) * 16 + (row & 15);
        if (ru < F.RU && head < F.gs && i < G.W)
            lse[((int64_t)unit * F.gs + head) * G.W + i] = (m + log2f(z)) * 0.6931471805599453f;
    }
}

struct LseCall {
    const void* q;
    const void* k;
    const float* lse;
    const ScoreGeom* G;
    const FusedGeom* F;
    float* vote;
    float2* stat_part;
    hipStream_t st;
    const ScoreLayers* layers = nullptr;   // the heads are those of separately allocated layers (q and k unused)
};

// The launch over a table of layers (two-byte element types; nothing waits across workgroups, so any grid runs).
template <typename T, int D, int RUW, int NW, bool STAT>
static hipError_t lse_layers_instance(const LseCall* call) {
    constexpr int KT = kFusedSlots / RUW;
    auto kern = score_lse_layers<T, D, RUW, KT, NW, STAT>;
    constexpr int kQBytes = 2 * RUW * (D * esize<T>::value / 64) * 64 * 16;
    static bool ready = false;
    if (!ready) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kQBytes);
        if (e != hipSuccess) return e;
        ready = true;
    }
    const FusedGeom& F = *call->F;
    hipLaunchKernelGGL(kern, dim3(F.NG * F.Gg), dim3(NW * 64), kQBytes, call->st, call->lse, call->vote,
                       call->stat_part, *call->G, F, *call->layers);
    return hipGetLastError();
}

template <typename T, int D, int RUW, int NW, bool STAT>
static hipError_t lse_instance(const LseCall* call, int* occ) {
    constexpr int KT = kFusedSlots / RUW;
    auto kern = score_lse<T, D, RUW, KT, NW, STAT>;
    constexpr int kQBytes = 2 * RUW * (D * esize<T>::value / 64) * 64 * 16;   // Q blocks of two units
    static int cached_occ = -1;
    if (cached_occ < 0) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kQBytes);
        if (e != hipSuccess) return e;
        int n = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, NW * 64, kQBytes);
        if (e != hipSuccess) return e;
        cached_occ = n;
    }
    if (occ) *occ = cached_occ;
    if (!call) return hipSuccess;
    if (call->layers) {
        if constexpr (esize<T>::value == 2) return lse_layers_instance<T, D, RUW, NW, STAT>(call);
        else return hipErrorInvalidValue;
    }
    const FusedGeom& F = *call->F;
    hipLaunchKernelGGL(kern, dim3(F.NG * F.Gg), dim3(NW * 64), kQBytes, call->st, call->q, call->k,
                       call->lse, call->vote, call->stat_part, *call->G, F);
    return hipGetLastError();
}

template <typename T, int D, bool STAT>
static hipError_t lse_by_rows(int RUW, const LseCall* call, int* occ) {
    switch (RUW) {
        case 1: return lse_instance<T, D, 1, kFusedWaves, STAT>(call, occ);
        case 2: return lse_instance<T, D, 2, kFusedWaves, STAT>(call, occ);
        case 4: return lse_instance<T, D, 4, kFusedWaves, STAT>(call, occ);
        case 8: return lse_instance<T, D, 8, kFusedWaves, STAT>(call, occ);
    }
    return hipErrorInvalidValue;
}

template <bool STAT>
static hipError_t lse_dispatch(int dtype, int D, int RUW, const LseCall* call, int* occ) {
    if (dtype == 0) {
        if (D == 128) return lse_by_rows<bf16_k, 128, STAT>(RUW, call, occ);
        if (D == 64) return lse_by_rows<bf16_k, 64, STAT>(RUW, call, occ);
    } else if (dtype == 2) {
        if (D == 128) return lse_by_rows<f16_k, 128, STAT>(RUW, call, occ);
        if (D == 64) return lse_by_rows<f16_k, 64, STAT>(RUW, call, occ);
    } else {
        if (D == 128) return lse_by_rows<f32_k, 128, STAT>(RUW, call, occ);
        if (D == 64) return lse_by_rows<f32_k, 64, STAT>(RUW, call, occ);
    }
    return hipErrorInvalidValue;
}

// Launch plan of the streaming kernel (both modes share it).  Nothing waits across workgroups, so
// residency is not a condition and the prompt length is not limited by the chip; the grid is still
// sized to what is resident so that every workgroup streams from start to end.
static bool lse_plan_for(int dtype, int D, const ScoreGeom& G, FusedGeom* F);

bool lse_plan(int dtype, int D, const ScoreGeom& G, FusedGeom* F, bool allow_blocks) {
    if (lse_plan_for(dtype, D, G, F)) return true;
    // more window rows than a wave tracks: every 32-row block of the window as a query head of its own
    ScoreGeom Gs;
    if (allow_blocks && block_geom(G, &Gs) && lse_plan_for(dtype, D, Gs, F)) {
        F->BH = G.BH;
        return true;
    }
    return false;
}

static bool lse_plan_for(int dtype, int D, const ScoreGeom& G, FusedGeom* F) {
    int cand[8];
    const int nc = fused_split_candidates(G, cand);
    for (int c = 0; c < nc; ++c) {
        if (!fused_shape_nw(G, kFusedWaves, cand[c], F, false)) continue;
        int occ = 0, occ2 = 0;
        if (lse_dispatch<false>(dtype, D, F->RUW, nullptr, &occ) != hipSuccess ||
            lse_dispatch<true>(dtype, D, F->RUW, nullptr, &occ2) != hipSuccess) {
            (void)hipGetLastError();
            continue;
        }
        if (occ2 < occ) occ = occ2;
        const int64_t slots = (int64_t)cu_count() * occ;
        if (slots <= 0) continue;
        int64_t NG = slots / F->Gg;
        if (NG < F->split) NG = F->split;    // more workgroups than fit at once simply queue up
        if (NG > F->units) NG = F->units;
        NG -= NG % F->split;
        if (NG < F->split) continue;
        F->NG = (int)NG;
        return true;
    }
    return false;
}

// Bytes of per-slice row statistics that cover whichever split lse_plan ends up choosing.
size_t stream_stat_bytes(const ScoreGeom& G) {
    size_t most = 0;
    ScoreGeom Gs;
    const ScoreGeom* geoms[2] = {&G, block_geom(G, &Gs) ? &Gs : nullptr};
    for (const ScoreGeom* g : geoms) {
        if (!g) continue;
        int cand[8];
        const int nc = fused_split_candidates(*g, cand);
        for (int i = 0; i < nc; ++i) {
            FusedGeom F;
            if (!fused_shape_nw(*g, kFusedWaves, cand[i], &F, false)) continue;
            const size_t b = sizeof(float2) * (size_t)F.units * F.Gg * F.RUW * 16;
            most = b > most ? b : most;
        }
    }
    return (most + 255) & ~(size_t)255;
}

static bool layers_fit(const ScoreLayers* SL, const ScoreGeom& G, const FusedGeom& F) {
    return !SL || (SL->count >= 1 && SL->count <= kMaxLayerPtrs && SL->kv_heads >= 1 && SL->count * SL->kv_heads == G.Hkv &&
                   F.BH == 1 && !G.k_table);
}

hipError_t launch_score_lse(int dtype, int D, const void* q, const void* k, const float* lse,
                            const ScoreGeom& G, const FusedGeom& F, float* vote, hipStream_t st,
                            const ScoreLayers* layers) {
    if (G.n <= 0) return hipSuccess;
    if (!layers_fit(layers, G, F)) return hipErrorInvalidValue;
    ScoreGeom Gl = G;
    if (F.BH > 1 && !block_geom(G, &Gl)) return hipErrorInvalidValue;
    const LseCall call{q, k, lse, &Gl, &F, vote, nullptr, st, layers};
    return lse_dispatch<false>(dtype, D, F.RUW, &call, nullptr);
}

// The rows' log-sum-exp by one streaming pass over K and a small merge.
int64_t long_logit_keys(const FusedGeom& F) { return (int64_t)F.Gg * F.NW * F.KT * 16; }

size_t long_logit_bytes(const ScoreGeom& G) {
    // one row unit per unit: a key's 16 logits are 64 bytes against the 2 * D bytes or more of its K row
    if (G.W > 16 || G.g != 1) return 0;
    int64_t slots = resident_slots(1);
    slots -= slots % 8;
    const int64_t wg_keys = (int64_t)kFusedWaves * kFusedSlots * 16;
    if (slots < 8 || G.L <= slots * wg_keys) return 0;   // short enough for the single-read kernel alone
    const int64_t rest = G.L - slots * wg_keys + wg_keys;   // rounded up to the workgroups' tile grid
    return ((size_t)G.Hkv * (size_t)rest * 16 * sizeof(float) + 255) & ~(size_t)255;
}

// One quad of lanes per key: each lane exponentiates four rows' logits, the quad's sum is the vote.  A workgroup
// takes kVflKeys consecutive keys of a unit, eight per quad, all loads in flight before the first is used.
constexpr int kVflKeys = 512;
__global__ __launch_bounds__(256) void votes_from_logits(const float* __restrict__ logit, const float* __restrict__ lse,
                                                        float* __restrict__ vote, const int64_t keys, const int64_t n,
                                                        const int W, const float c2, const int64_t vpitch) {
    const int unit = blockIdx.y, part = threadIdx.x & 3, quad = threadIdx.x >> 2;
    const int64_t j0 = (int64_t)blockIdx.x * kVflKeys + quad;
    constexpr float kLog2e = 1.4426950408889634f;
    float l2[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int i = part * 4 + r;
        l2[r] = i < W ? lse[(int64_t)unit * W + i] * kLog2e : INFINITY;   // rows beyond the window vote nothing
    }
    const float* base = logit + (int64_t)unit * keys * 16 + part * 4;
    f32x4 x[kVflKeys / 64];
#pragma unroll
    for (int c = 0; c < kVflKeys / 64; ++c) {
        const int64_t j = j0 + c * 64;   // inside the unit's logits (they cover whole workgroup strides of keys)
        x[c] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(base + (j < keys ? j : keys - 1) * 16));
    }
#pragma unroll
    for (int c = 0; c < kVflKeys / 64; ++c) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) s += __builtin_amdgcn_exp2f(fmaf(x[c][r], c2, -l2[r]));
        s += __shfl_xor(s, 1, 64);
        s += __shfl_xor(s, 2, 64);
        const int64_t j = j0 + c * 64;
        if (part == 0 && j < n) VOTE_STORE(&vote[(int64_t)unit * vpitch + j], s);
    }
}

hipError_t launch_votes_from_logits(const float* logit, const float* lse, float* vote, const LongPlan& P,
                                    hipStream_t st) {
    if (P.Fr.RUW != 1 || P.Fr.gs != 1 || P.Gr.n <= 0 || P.Fr.units > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((P.Gr.n + kVflKeys - 1) / kVflKeys), (unsigned)P.Fr.units);
    hipLaunchKernelGGL(votes_from_logits, grid, dim3(256), 0, st, logit, lse, vote, long_logit_keys(P.Fr), P.Gr.n, P.Gr.W,
                       P.Gr.c2, P.Gr.vpitch);
    return hipGetLastError();
}

hipError_t launch_row_lse(int dtype, int D, const void* q, const void* k, const ScoreGeom& G,
                          const FusedGeom& F, float2* stat_part, float* lse_out, hipStream_t st, float* logit_out,
                          const ScoreLayers* layers) {
    if (G.n <= 0) return hipSuccess;
    if (logit_out && F.RUW != 1) return hipErrorInvalidValue;
    if (!layers_fit(layers, G, F)) return hipErrorInvalidValue;
    ScoreGeom Gl = G;
    if (F.BH > 1 && !block_geom(G, &Gl)) return hipErrorInvalidValue;
    const LseCall call{q, k, nullptr, &Gl, &F, logit_out, stat_part, st, layers};
    hipError_t e = lse_dispatch<true>(dtype, D, F.RUW, &call, nullptr);
    if (e != hipSuccess) return e;
    stage_done(st, kStagePass1);
    if (!lse_out) return hipGetLastError();
    // (with blocks, row i of block b of a head is row 32 b + i of its window: the same place in lse_out)
    hipLaunchKernelGGL(lse_from_parts, dim3(F.units), dim3(1024), 0, st, stat_part, lse_out, Gl, F);
    stage_done(st, kStageReduce);
    return hipGetLastError();
}

}  // namespace snapkv

