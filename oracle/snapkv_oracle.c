/*
 * Plain-C fp64 oracle for the SnapKV prompt-KV compression step (arXiv 2404.14469).
 *
 * TEST INFRASTRUCTURE ONLY: a second, independently written opinion on the numpy oracle
 * beside it, and the CPU baseline the bench times.  The product never links or loads it.
 *
 * It follows the procedure of Sec. 4.1 / Listing 1 (Eq. 1-2) in order, one KV head at a
 * time, in scalar loops: scaled dot products of the W observation-window queries with
 * every key, the prompt-phase causal mask (window query i is at position n+i and cannot
 * see keys after it), a row softmax over all keys, the column sum over the window rows
 * for prefix columns, stride-1 pooling of width p with padding p/2 (max ignores the
 * padding; average counts it as zeros and divides by p), the sum over the query heads of
 * a KV group, the top-(C-W) positions with ties to the lower index, and the copy of the
 * chosen rows in ascending position order followed by the window rows.
 *
 * Storage: is_bf16 != 0 means q/k/v are 16-bit bfloat16 patterns, else IEEE float32.
 * Layouts: q_win [Hq][W][D], k and v [Hkv][L][D], row-major.
 * Threads: KV heads are independent and are spread over OpenMP threads when built with
 * -fopenmp; the arithmetic of a head never depends on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double load_elem(const void* base, int64_t idx, int is_bf16) {
    if (is_bf16) {
        uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float*)base)[idx];
}

int snapkv_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* vote of one query head into vote[n]; scratch rows s[W][L] supplied by the caller */
static void head_vote(const void* q, int64_t q_off, const void* k, int64_t k_off, int is_bf16,
                      int64_t L, int D, int W, double* s, double* kd, double* vote) {
    const int64_t n = L - W;
    const double scale = 1.0 / sqrt((double)D);
    for (int64_t j = 0; j < L; ++j)
        for (int d = 0; d < D; ++d) kd[j * D + d] = load_elem(k, k_off + j * D + d, is_bf16);
    for (int i = 0; i < W; ++i) {
        double* row = s + (int64_t)i * L;
        double qd[1024];
        for (int d = 0; d < D; ++d) qd[d] = load_elem(q, q_off + (int64_t)i * D + d, is_bf16);
        const int64_t last_visible = n + i; /* keys 0..n+i */
        double mx = -INFINITY;
        for (int64_t j = 0; j <= last_visible; ++j) {
            double acc = 0.0;
            const double* kr = kd + j * D;
            for (int d = 0; d < D; ++d) acc += qd[d] * kr[d];
            row[j] = acc * scale;
            if (row[j] > mx) mx = row[j];
        }
        double z = 0.0;
        for (int64_t j = 0; j <= last_visible; ++j) {
            row[j] = exp(row[j] - mx);
            z += row[j];
        }
        for (int64_t j = 0; j <= last_visible; ++j) row[j] /= z;
        for (int64_t j = last_visible + 1; j < L; ++j) row[j] = 0.0;
    }
    for (int64_t j = 0; j < n; ++j) {
        double c = 0.0;
        for (int i = 0; i < W; ++i) c += s[(int64_t)i * L + j];
        vote[j] = c;
    }
}

static void pool_into(const double* vote, int64_t n, int pool_kind, int p, double* acc) {
    const int r = p / 2;
    for (int64_t j = 0; j < n; ++j) {
        int64_t lo = j - r < 0 ? 0 : j - r;
        int64_t hi = j + r > n - 1 ? n - 1 : j + r;
        double val;
        if (pool_kind == 0) {
            val = vote[lo];
            for (int64_t t = lo + 1; t <= hi; ++t)
                if (vote[t] > val) val = vote[t];
        } else {
            val = 0.0;
            for (int64_t t = lo; t <= hi; ++t) val += vote[t];
            val /= (double)p;
        }
        acc[j] += val;
    }
}

/* score[Hkv][n]; returns 0 on success, -1 on bad arguments, -2 on allocation failure */
int snapkv_oracle_pooled_scores(const void* q_win, const void* k, int is_bf16, int64_t L, int Hq,
                                int Hkv, int D, int W, int pool_kind, int p, double* score) {
    if (!q_win || !k || !score || L < 1 || W < 1 || W > L || Hkv < 1 || Hq % Hkv || D < 1 ||
        D > 1024 || p < 1 || p % 2 == 0 || (pool_kind != 0 && pool_kind != 1))
        return -1;
    const int g = Hq / Hkv;
    const int64_t n = L - W;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int hk = 0; hk < Hkv; ++hk) {
        double* s = (double*)malloc(sizeof(double) * (size_t)W * (size_t)L);
        double* kd = (double*)malloc(sizeof(double) * (size_t)L * (size_t)D);
        double* vt = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        if (!s || !kd || !vt) {
            fail = 1;
        } else {
            double* out = score + (int64_t)hk * n;
            for (int64_t j = 0; j < n; ++j) out[j] = 0.0;
            for (int h = hk * g; h < (hk + 1) * g; ++h) {
                head_vote(q_win, (int64_t)h * W * D, k, (int64_t)hk * L * D, is_bf16, L, D, W, s,
                          kd, vt);
                pool_into(vt, n, pool_kind, p, out);
            }
        }
        free(s);
        free(kd);
        free(vt);
    }
    return fail ? -2 : 0;
}

typedef struct {
    double score;
    int64_t pos;
} cand_t;

static int cand_cmp(const void* a, const void* b) {
    const cand_t* x = (const cand_t*)a;
    const cand_t* y = (const cand_t*)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int pos_cmp(const void* a, const void* b) {
    int64_t x = *(const int64_t*)a, y = *(const int64_t*)b;
    return (x > y) - (x < y);
}

/*
 * Whole step.  out_k/out_v: [Hkv][C][D] in the storage type, out_idx: [Hkv][C] int64,
 * score_out (may be NULL): [Hkv][n].  Returns rows kept per head (min(C, L)), or <0.
 * On bypass (L <= C) only the first L rows / indices of each head are written.
 */
int64_t snapkv_oracle_compress(const void* q_win, const void* k, const void* v, int is_bf16,
                               int64_t L, int Hq, int Hkv, int D, int W, int pool_kind, int p,
                               int64_t C, void* out_k, void* out_v, int64_t* out_idx,
                               double* score_out) {
    if (!q_win || !k || !v || !out_k || !out_v || !out_idx || W > C) return -1;
    const size_t esz = is_bf16 ? 2 : 4;
    const size_t row = (size_t)D * esz;
    if (L <= C) {
        if (L < 1 || Hkv < 1) return -1;
        for (int hk = 0; hk < Hkv; ++hk) {
            memcpy((char*)out_k + (size_t)hk * C * row, (const char*)k + (size_t)hk * L * row,
                   (size_t)L * row);
            memcpy((char*)out_v + (size_t)hk * C * row, (const char*)v + (size_t)hk * L * row,
                   (size_t)L * row);
            for (int64_t j = 0; j < L; ++j) out_idx[(int64_t)hk * C + j] = j;
        }
        return L;
    }
    const int64_t n = L - W;
    const int64_t kc = C - W;
    double* score = score_out ? score_out : (double*)malloc(sizeof(double) * (size_t)Hkv * n);
    if (!score) return -2;
    int rc = snapkv_oracle_pooled_scores(q_win, k, is_bf16, L, Hq, Hkv, D, W, pool_kind, p, score);
    if (rc) {
        if (!score_out) free(score);
        return rc;
    }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int hk = 0; hk < Hkv; ++hk) {
        cand_t* c = (cand_t*)malloc(sizeof(cand_t) * (size_t)n);
        if (!c) {
            fail = 1;
            continue;
        }
        for (int64_t j = 0; j < n; ++j) {
            c[j].score = score[(int64_t)hk * n + j];
            c[j].pos = j;
        }
        qsort(c, (size_t)n, sizeof(cand_t), cand_cmp);
        int64_t* idx = out_idx + (int64_t)hk * C;
        for (int64_t t = 0; t < kc; ++t) idx[t] = c[t].pos;
        qsort(idx, (size_t)kc, sizeof(int64_t), pos_cmp);
        for (int64_t t = 0; t < W; ++t) idx[kc + t] = n + t;
        for (int64_t t = 0; t < C; ++t) {
            memcpy((char*)out_k + ((size_t)hk * C + t) * row,
                   (const char*)k + ((size_t)hk * L + idx[t]) * row, row);
            memcpy((char*)out_v + ((size_t)hk * C + t) * row,
                   (const char*)v + ((size_t)hk * L + idx[t]) * row, row);
        }
        free(c);
    }
    if (!score_out) free(score);
    return fail ? -2 : C;
}
