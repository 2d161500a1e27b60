/*
 * Drives the plain-C oracle (oracle/snapkv_oracle.c, compiled into this program) on small seeded inputs
 * under -fsanitize=address,undefined: every configuration kind the tests use (float32 and bfloat16 storage,
 * grouped heads, max and average pooling, a window as long as the prompt allows, a prompt that fits the
 * capacity, p = 1), and checks the properties the definition fixes (Listing 1): output length, positions
 * ascending and unique, window rows last, rows copied bit for bit.  CPU only; test infrastructure.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int snapkv_oracle_pooled_scores(const void* q_win, const void* k, int is_bf16, int64_t L, int Hq, int Hkv, int D, int W,
                                int pool_kind, int p, double* out);
int64_t snapkv_oracle_compress(const void* q_win, const void* k, const void* v, int is_bf16, int64_t L, int Hq, int Hkv,
                               int D, int W, int pool_kind, int p, int64_t C, void* out_k, void* out_v, int64_t* out_idx,
                               double* score);

static uint64_t rng_state = 88172645463325252ull;
static double rnd(void) { /* xorshift64: values in (-1, 1) */
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

static void fill(void* dst, int64_t count, int is_bf16) {
    for (int64_t i = 0; i < count; ++i) {
        float f = (float)(1.5 * rnd());
        if (is_bf16) {
            uint32_t bits;
            memcpy(&bits, &f, 4);
            ((uint16_t*)dst)[i] = (uint16_t)(bits >> 16);
        } else {
            ((float*)dst)[i] = f;
        }
    }
}

static int run_case(int is_bf16, int64_t L, int Hq, int Hkv, int D, int W, int pool_kind, int p, int64_t C) {
    const size_t e = is_bf16 ? 2 : 4;
    const int64_t n = L - W, rows = L <= C ? L : C;
    void* q = malloc((size_t)Hq * W * D * e);
    void* k = malloc((size_t)Hkv * L * D * e);
    void* v = malloc((size_t)Hkv * L * D * e);
    void* ok = malloc((size_t)Hkv * C * D * e);
    void* ov = malloc((size_t)Hkv * C * D * e);
    int64_t* idx = malloc(sizeof(int64_t) * (size_t)Hkv * C);
    double* score = malloc(sizeof(double) * (size_t)Hkv * (n > 0 ? n : 1));
    double* score2 = malloc(sizeof(double) * (size_t)Hkv * (n > 0 ? n : 1));
    fill(q, (int64_t)Hq * W * D, is_bf16);
    fill(k, (int64_t)Hkv * L * D, is_bf16);
    fill(v, (int64_t)Hkv * L * D, is_bf16);
    int bad = 0;
    const int64_t kept = snapkv_oracle_compress(q, k, v, is_bf16, L, Hq, Hkv, D, W, pool_kind, p, C, ok, ov, idx,
                                                L > C ? score : NULL);
    if (kept != rows) bad = 1;
    if (n > 0 && snapkv_oracle_pooled_scores(q, k, is_bf16, L, Hq, Hkv, D, W, pool_kind, p, score2) != 0) bad = 2;
    for (int h = 0; h < Hkv && !bad; ++h) {
        const int64_t* ih = idx + (int64_t)h * C;
        for (int64_t r = 0; r < rows; ++r) {
            if (ih[r] < 0 || ih[r] >= L || (r > 0 && ih[r] <= ih[r - 1])) bad = 3;
            if (L > C && r >= C - W && ih[r] != n + (r - (C - W))) bad = 4;
            if (bad) break;
            if (memcmp((char*)ok + ((size_t)h * C + r) * D * e, (char*)k + ((size_t)h * L + ih[r]) * D * e, D * e) != 0) bad = 5;
            if (memcmp((char*)ov + ((size_t)h * C + r) * D * e, (char*)v + ((size_t)h * L + ih[r]) * D * e, D * e) != 0) bad = 6;
        }
        if (L > C && !bad)
            for (int64_t j = 0; j < n; ++j)
                if (score[(int64_t)h * n + j] != score2[(int64_t)h * n + j] || !(score[(int64_t)h * n + j] >= 0.0)) bad = 7;
    }
    free(q), free(k), free(v), free(ok), free(ov), free(idx), free(score), free(score2);
    if (bad) fprintf(stderr, "case bf16=%d L=%lld Hq=%d Hkv=%d D=%d W=%d kind=%d p=%d C=%lld failed check %d\n", is_bf16,
                     (long long)L, Hq, Hkv, D, W, pool_kind, p, (long long)C, bad);
    return bad;
}

int main(void) {
    int bad = 0;
    bad |= run_case(0, 96, 4, 4, 64, 32, 0, 7, 48);     /* float32, max pooling */
    bad |= run_case(1, 200, 8, 2, 128, 16, 1, 5, 64);   /* bfloat16, grouped heads, average pooling */
    bad |= run_case(1, 70, 2, 2, 64, 64, 0, 13, 66);    /* window nearly as long as the prompt, pooling wider than the prefix */
    bad |= run_case(0, 40, 2, 1, 64, 8, 0, 3, 64);      /* prompt fits the capacity: returned unchanged */
    bad |= run_case(0, 33, 1, 1, 64, 1, 0, 1, 9);       /* W = 1, p = 1 */
    bad |= run_case(1, 64, 2, 2, 64, 32, 1, 129, 40);   /* widest pooling */
    bad |= run_case(0, 50, 3, 3, 64, 10, 0, 5, 10);     /* C = W: nothing but the window is kept */
    if (!bad) printf("oracle driver: all cases passed\n");
    return bad ? 1 : 0;
}
