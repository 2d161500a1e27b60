/*
 * Host-side bounds model of the ordered emission of the cooperative pooling + selection kernel (Eq. 2's
 * top-k, emitted ascending).  A head's n scores are cut into workgroup chunks; a workgroup knows the
 * threshold pattern T, how many positions equal to T are kept (need_eq), and how many positions greater
 * than / equal to T lie in the chunks before its own; position j then goes to slot
 *     (#greater before j) + min(#equal before j, need_eq)        if x[j] > T, or x[j] == T and #equal before j < need_eq.
 * The model runs exactly that arithmetic chunk by chunk into an array of k slots (under
 * -fsanitize=address,undefined an out-of-range slot is an error by itself) and checks: every slot
 * written exactly once, slots ascending in position, the kept set equal to a plain sort's top-k with ties
 * to the lower position, the per-chunk kept counts summing to k.  Heavy ties (few distinct values, as
 * max pooling produces) are the interesting inputs.  CPU only; test infrastructure.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static uint64_t rng_state = 1234567891011ull;
static uint32_t rnd32(void) {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 20);
}

typedef struct { uint32_t x; int32_t j; } item;
static int by_score_desc_pos_asc(const void* a, const void* b) {
    const item *p = a, *q = b;
    if (p->x != q->x) return p->x > q->x ? -1 : 1;
    return p->j < q->j ? -1 : (p->j > q->j ? 1 : 0);
}

static int run_case(int n, int k, int chunk, uint32_t distinct) {
    uint32_t* x = malloc(sizeof(uint32_t) * (size_t)n);
    item* sorted = malloc(sizeof(item) * (size_t)n);
    int32_t* out = malloc(sizeof(int32_t) * (size_t)(k > 0 ? k : 1));
    int* written = calloc((size_t)(k > 0 ? k : 1), sizeof(int));
    char* want = calloc((size_t)n, 1);
    for (int j = 0; j < n; ++j) {
        x[j] = distinct ? 0x38000000u + (rnd32() % distinct) * 977u : rnd32() & 0x7fffffffu;
        sorted[j].x = x[j];
        sorted[j].j = j;
    }
    int bad = 0;
    if (k > 0) {
        qsort(sorted, (size_t)n, sizeof(item), by_score_desc_pos_asc);
        const uint32_t T = sorted[k - 1].x;
        int greater = 0;
        for (int j = 0; j < n; ++j) greater += x[j] > T;
        const int need_eq = k - greater;                 /* what the threshold search hands every workgroup */
        for (int i = 0; i < k; ++i) want[sorted[i].j] = 1;
        const int nchunks = (n + chunk - 1) / chunk;
        int kept_total = 0, gt_before = 0, eq_before = 0;
        for (int c = 0; c < nchunks && !bad; ++c) {      /* one workgroup after the other; order does not matter */
            const int a = c * chunk, b = a + chunk < n ? a + chunk : n;
            int gb = gt_before, qb = eq_before, kept = 0;
            for (int j = a; j < b; ++j) {
                const int gt = x[j] > T, eq = x[j] == T;
                if (gt || (eq && qb < need_eq)) {
                    const int at = gb + (qb < need_eq ? qb : need_eq);
                    if (at >= k) { bad = 1; break; }
                    out[at] = j;                         /* a slot beyond k would be caught by the sanitizer as well */
                    ++written[at];
                    ++kept;
                    if (!want[j]) bad = 2;
                }
                gb += gt;
                qb += eq;
            }
            kept_total += kept;
            gt_before = gb;
            eq_before = qb;
        }
        if (!bad && kept_total != k) bad = 3;
        for (int i = 0; i < k && !bad; ++i) {
            if (written[i] != 1) bad = 4;
            if (i > 0 && out[i] <= out[i - 1]) bad = 5;
        }
    }
    free(x), free(sorted), free(out), free(written), free(want);
    if (bad) fprintf(stderr, "case n=%d k=%d chunk=%d distinct=%u failed check %d\n", n, k, chunk, distinct, bad);
    return bad;
}

int main(void) {
    int bad = 0;
    const int chunks[] = {4, 64, 1000, 2048, 16384};
    const uint32_t kinds[] = {0u, 1u, 2u, 7u, 300u};    /* all distinct ... a single value */
    for (unsigned ci = 0; ci < sizeof chunks / sizeof *chunks; ++ci)
        for (unsigned ki = 0; ki < sizeof kinds / sizeof *kinds; ++ki) {
            bad |= run_case(5000, 992, chunks[ci], kinds[ki]);
            bad |= run_case(4097, 4097, chunks[ci], kinds[ki]);   /* everything kept */
            bad |= run_case(777, 1, chunks[ci], kinds[ki]);
            bad |= run_case(131, 0, chunks[ci], kinds[ki]);       /* nothing but the window */
        }
    if (!bad) printf("emission model: all cases passed\n");
    return bad ? 1 : 0;
}
