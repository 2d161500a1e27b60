/*
 * Host-side bounds model of how a prompt longer than the single-read scoring launch holds is cut in two, and of
 * where the two launches' workgroups read keys and write votes and kept logits (Eq. 1: every prefix key gets exactly
 * one vote).  The model repeats the integer arithmetic of the plan and of the kernels' tile-to-key mapping:
 *   front  = as many keys as `slots` resident workgroups hold (a multiple of eight workgroups, each NW waves x KT
 *            tiles x 16 keys), shortened until the rest keeps the W window rows and at least one key before them;
 *   rest   = a prompt of L - front keys ending in the same window, covered by ceil(tiles / (NW x KT)) workgroups;
 *   tile t of wave w of workgroup g (placed on die g mod 8) is key tile t * (G * NW) + place(g) * NW + w.
 * It then writes a vote mark for every key a launch votes on, and, for the form that keeps the rest's logits, a
 * float4 per (key, 4-row group) into an array of exactly the size the workspace layout reserves.  Under
 * -fsanitize=address,undefined any index outside an array is an error by itself; the checks on top: every prefix key
 * is voted on exactly once, no other key is, front + rest = L, and the logits of every unit fit.
 * CPU only; test infrastructure.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

enum { NW = 8, SLOTS_PER_WAVE = 8, MAX_L1_BLOCKS = 16 };

static int64_t place(int64_t g, int64_t G) { return G % 8 == 0 ? (g % 8) * (G / 8) + g / 8 : g; }

/* marks [0, limit) of `votes` for the keys < limit that a launch of G workgroups covers */
static int cover(int64_t G, int KT, int64_t limit, unsigned char* votes, int64_t base) {
    const int64_t TS = G * NW;
    for (int64_t g = 0; g < G; ++g)
        for (int w = 0; w < NW; ++w)
            for (int t = 0; t < KT; ++t) {
                const int64_t tile = (int64_t)t * TS + place(g, G) * NW + w;
                for (int n16 = 0; n16 < 16; ++n16) {
                    const int64_t j = tile * 16 + n16;
                    if (j < limit) {
                        if (votes[base + j] != 0) return 0;   /* a key voted on twice */
                        votes[base + j] = 1;
                    }
                }
            }
    return 1;
}

static int run_case(int64_t L, int W, int RUW, int64_t slots, int units) {
    const int KT = SLOTS_PER_WAVE / RUW;
    const int64_t wg_keys = (int64_t)NW * KT * 16, n = L - W;
    int64_t G = slots;
    if (G > 32 * (MAX_L1_BLOCKS - 1)) G = 32 * (MAX_L1_BLOCKS - 1);
    G -= G % 8;
    while (G >= 8 && L - G * wg_keys <= W) G -= 8;
    if (G < 8) return 1;                      /* no front part: the prompt takes two streaming passes */
    const int64_t front = G * wg_keys, Lr = L - front, nr = Lr - W;
    if (front + Lr != L || nr < 1 || front > n) return 0;
    const int64_t tiles_r = (Lr + 15) / 16, Gr = (tiles_r + NW * KT - 1) / (NW * KT), keys_pad = Gr * wg_keys;
    if (keys_pad < Lr) return 0;

    unsigned char* votes = calloc((size_t)L, 1);
    if (!votes) return 0;
    int ok = cover(G, KT, front, votes, 0);                 /* the single-read launch votes on every key of the front */
    ok = ok && cover(Gr, KT, nr, votes, front);             /* the rest's launch on its own prefix */
    for (int64_t j = 0; ok && j < L; ++j) ok = votes[j] == (j < n ? 1 : 0);
    free(votes);
    if (!ok) return 0;

    if (RUW == 1) {   /* the kept logits: sized as the workspace layout sizes them, written as the statistics pass writes them */
        int64_t s8 = slots - slots % 8;
        if (s8 < 8 || L <= s8 * wg_keys) return 1;          /* layout reserves nothing: the plan must not keep logits */
        const int64_t reserve_keys = L - s8 * wg_keys + wg_keys;
        const size_t floats = (size_t)units * (size_t)reserve_keys * 16;
        if ((size_t)units * (size_t)keys_pad * 16 > floats) {
            /* a shortened front leaves a longer rest than the layout assumed: the dispatcher then reads the keys again */
            return front < s8 * wg_keys;
        }
        float* logit = malloc(sizeof(float) * floats);
        if (!logit) return 0;
        const int64_t TS = Gr * NW;
        for (int u = 0; u < units; ++u)
            for (int64_t g = 0; g < Gr; ++g)
                for (int w = 0; w < NW; ++w)
                    for (int t = 0; t < KT; ++t)
                        for (int lane = 0; lane < 64; ++lane) {
                            const int n16 = lane & 15, kg = lane >> 4;
                            const int64_t j = ((int64_t)t * TS + place(g, Gr) * NW + w) * 16 + n16;
                            float* dst = logit + ((int64_t)u * keys_pad + j) * 16 + kg * 4;
                            dst[0] = dst[1] = dst[2] = dst[3] = (float)u;
                        }
        /* the reader: one quad of lanes per key below nr */
        double sum = 0.0;
        for (int u = 0; u < units; ++u)
            for (int64_t j = 0; j < nr; ++j)
                for (int part = 0; part < 4; ++part) sum += logit[((int64_t)u * keys_pad + j) * 16 + part * 4];
        free(logit);
        if (sum != (double)nr * 4.0 * (units * (units - 1) / 2)) return 0;
    }
    return 1;
}

int main(void) {
    const int64_t slot_counts[] = {8, 16, 24, 100, 256};
    const int windows[] = {1, 8, 16, 32, 64};
    int cases = 0;
    for (int RUW = 1; RUW <= 8; RUW *= 2)
        for (size_t s = 0; s < sizeof slot_counts / sizeof *slot_counts; ++s)
            for (size_t wi = 0; wi < sizeof windows / sizeof *windows; ++wi) {
                const int W = windows[wi];
                const int64_t wg_keys = (int64_t)NW * (SLOTS_PER_WAVE / RUW) * 16;
                const int64_t cap = (slot_counts[s] - slot_counts[s] % 8) * wg_keys;
                const int64_t lengths[] = {cap + 1, cap + W, cap + W + 1, cap + W + 17, cap + wg_keys, cap + wg_keys + W + 1,
                                           2 * cap + 333, cap + 100000 + W, 3 * cap + 5};
                for (size_t li = 0; li < sizeof lengths / sizeof *lengths; ++li) {
                    if (lengths[li] <= W || lengths[li] > 3000000) continue;
                    if (!run_case(lengths[li], W, RUW, slot_counts[s], 3)) {
                        printf("FAILED: L=%lld W=%d RUW=%d slots=%lld\n", (long long)lengths[li], W, RUW,
                               (long long)slot_counts[s]);
                        return 1;
                    }
                    ++cases;
                }
            }
    printf("%d cases: all cases passed\n", cases);
    return 0;
}
