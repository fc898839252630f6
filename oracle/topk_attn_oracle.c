/*
 * CPU oracle for top-k attention decode, plain C, double precision.
 * TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg link or call this.  It shares no code with the HIP path.
 *
 * Follows the paper's methodology section ("Top-k Attention: Accelerating
 * Decoding"): the exact ("list") k-nearest-neighbour search under the
 * dot-product metric, then Algorithm 1's attention step
 * Softmax(vals / sqrt(d)) V[I] over the retrieved rows.  Every step is the
 * plain definition: full score vector, full sort of all N (score, position)
 * pairs, max-subtracted softmax, double-precision weighted sum.
 *
 * Inputs are the storage-dtype arrays the GPU sees (fp32, fp16 or bf16 bit
 * patterns); each element is widened to double before any arithmetic, so the
 * scores are the exact scores of the stored values up to double rounding.
 *
 * Conventions: query head h searches KV head h / G (G = Hq / Hkv); each query
 * head selects its own top-k; ties go to the lower position; k_eff = min(k, N)
 * and unused slots hold idx = -1, vals = -inf.
 *
 * Pins: cross-checked against the NumPy oracle and, through it and directly,
 * against library dense attention (k = N), brute-force subset enumeration,
 * k = 1, all-equal scores and planted keys (tests/test_oracle_pins.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

static double widen_f16(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0) {
        v = ldexp((double)m, -24);                 /* subnormal: m * 2^-10 * 2^-14 */
    } else if (e == 31) {
        v = m ? NAN : INFINITY;
    } else {
        v = ldexp((double)(m | 0x400), e - 25);    /* (1 + m/1024) * 2^(e-15) */
    }
    return sign ? -v : v;
}

static double widen_bf16(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* 65536-entry table of the doubles a 16-bit pattern stands for (built per call) */
static double* build_table(int dtype) {
    if (dtype == ORACLE_F32) return NULL;
    double* t = (double*)malloc(sizeof(double) * 65536);
    if (!t) return NULL;
    for (uint32_t b = 0; b < 65536; ++b)
        t[b] = dtype == ORACLE_F16 ? widen_f16((uint16_t)b) : widen_bf16((uint16_t)b);
    return t;
}

/* widen n consecutive stored elements starting at element offset `off` */
static void widen_row(const void* base, int dtype, const double* tab, int64_t off, int n,
                      double* dst) {
    if (dtype == ORACLE_F32) {
        const float* p = (const float*)base + off;
        for (int c = 0; c < n; ++c) dst[c] = (double)p[c];
    } else {
        const uint16_t* p = (const uint16_t*)base + off;
        for (int c = 0; c < n; ++c) dst[c] = tab[p[c]];
    }
}

typedef struct { double s; int64_t i; } pair_t;

/* score descending, position ascending */
static int cmp_pair(const void* a, const void* b) {
    const pair_t* x = (const pair_t*)a;
    const pair_t* y = (const pair_t*)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    if (x->i < y->i) return -1;
    if (x->i > y->i) return 1;
    return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* scores of all query heads against keys [i0, i1) of every KV head */
static void score_block(const void* q, const void* K, int dtype, const double* tab,
                        int Hq, int Hkv, int d, int64_t N, int64_t rows, int64_t i0, int64_t i1,
                        int g, double* S, double* qd, double* kd) {
    int G = Hq / Hkv;
    for (int j = 0; j < G; ++j)
        widen_row(q, dtype, tab, (int64_t)(g * G + j) * d, d, qd + (size_t)j * d);
    for (int64_t i = i0; i < i1; ++i) {
        widen_row(K, dtype, tab, ((int64_t)g * rows + i) * d, d, kd);
        for (int j = 0; j < G; ++j) {
            const double* qh = qd + (size_t)j * d;
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += qh[c] * kd[c];
            S[(int64_t)(g * G + j) * N + i] = acc;
        }
    }
}

/*
 * S = q K^T (Eq. 1's score matrix), one row per query head; query head h is
 * scored against KV head h / G.
 * q [Hq, d], K [Hkv, N, d] in `dtype`; S [Hq, N] double.
 */
static int scores_impl(const void* q, const void* K, int dtype, int Hq, int Hkv, int d,
                       int64_t N, int64_t rows, double* S);

int oracle_scores(const void* q, const void* K, int dtype, int Hq, int Hkv, int d,
                  int64_t N, double* S) {
    return scores_impl(q, K, dtype, Hq, Hkv, d, N, N, S);
}

/* The same with the first N of `rows` stored rows per KV head scored (K [Hkv, rows, d]). */
static int scores_impl(const void* q, const void* K, int dtype, int Hq, int Hkv, int d,
                       int64_t N, int64_t rows, double* S) {
    if (!q || !K || !S || Hq < 1 || Hkv < 1 || d < 1 || N < 0 || rows < N || Hq % Hkv) return 1;
    if (dtype < 0 || dtype > 2) return 1;
    double* tab = build_table(dtype);
    if (dtype != ORACLE_F32 && !tab) return 2;
    int G = Hq / Hkv;
    const int64_t blk = 4096;
    int64_t nblk = (N + blk - 1) / blk;
    int fail = 0;
#pragma omp parallel
    {
        double* qd = (double*)malloc(sizeof(double) * (size_t)d * (size_t)G);
        double* kd = (double*)malloc(sizeof(double) * (size_t)d);
        if (!qd || !kd) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int g = 0; g < Hkv; ++g)
            for (int64_t b = 0; b < nblk; ++b) {
                if (!qd || !kd) continue;
                int64_t i0 = b * blk, i1 = i0 + blk < N ? i0 + blk : N;
                score_block(q, K, dtype, tab, Hq, Hkv, d, N, rows, i0, i1, g, S, qd, kd);
            }
        free(qd); free(kd);
    }
    free(tab);
    return fail ? 2 : 0;
}

static int topk_window_impl(const void* q, const void* K, const void* V, int dtype, int Hq, int Hkv, int d,
                            int64_t N, int64_t rows, int64_t k, int64_t window, double* out, int64_t* idx,
                            double* vals, double* lse);

/*
 * One decode step for one (layer, sequence).
 * q [Hq, d], K, V [Hkv, N, d] in `dtype`.
 * out [Hq, d] double; idx [Hq, k] int64; vals [Hq, k] double; lse [Hq] double
 * (idx, vals, lse may be NULL).  idx/vals come out in descending score order.
 * Returns 0, or 1 on invalid arguments, 2 on allocation failure.
 */
int oracle_topk_attention(const void* q, const void* K, const void* V, int dtype,
                          int Hq, int Hkv, int d, int64_t N, int64_t k,
                          double* out, int64_t* idx, double* vals, double* lse) {
    return topk_window_impl(q, K, V, dtype, Hq, Hkv, d, N, N, k, 0, out, idx, vals, lse);
}

/*
 * Decode step with the recent-token window of Algorithm 1: the last `window` cached
 * tokens (the algorithm's K_gen / V_gen) are always attended, the search runs over the
 * older prefix [0, N - window) only, and one softmax spans retrieved and window scores.
 * idx / vals report the search result over the prefix; lse covers both parts.
 */
int oracle_topk_attention_window(const void* q, const void* K, const void* V, int dtype,
                                 int Hq, int Hkv, int d, int64_t N, int64_t k, int64_t window,
                                 double* out, int64_t* idx, double* vals, double* lse) {
    if (window < 0) return 1;
    return topk_window_impl(q, K, V, dtype, Hq, Hkv, d, N, N, k, window, out, idx, vals, lse);
}

/*
 * A chunk of M queries against one cache (the multi-query use of top-k attention: the
 * paper's remark that top-k can also serve while the cache is being built).  Each query
 * is an independent decode step as above; with `causal` the queries belong to the last M
 * cached tokens and query m sees only the first N - (M - 1 - m) of them, without it every
 * query sees all N.  q [M, Hq, d]; K, V [Hkv, N, d]; out [M, Hq, d]; idx, vals [M, Hq, k];
 * lse [M, Hq].
 */
int oracle_topk_attention_multi(const void* q, const void* K, const void* V, int dtype, int M,
                                int Hq, int Hkv, int d, int64_t N, int causal, int64_t k, int64_t window,
                                double* out, int64_t* idx, double* vals, double* lse) {
    if (M < 1 || window < 0 || !q || dtype < 0 || dtype > 2) return 1;
    size_t esize = dtype == ORACLE_F32 ? 4 : 2;
    for (int m = 0; m < M; ++m) {
        int64_t n_vis = causal ? N - (M - 1 - m) : N;
        int rc = topk_window_impl((const char*)q + (size_t)m * Hq * d * esize, K, V, dtype, Hq, Hkv, d, n_vis, N,
                                  k, window, out + (size_t)m * Hq * d, idx ? idx + (size_t)m * Hq * k : NULL,
                                  vals ? vals + (size_t)m * Hq * k : NULL, lse ? lse + (size_t)m * Hq : NULL);
        if (rc) return rc;
    }
    return 0;
}

static int topk_window_impl(const void* q, const void* K, const void* V, int dtype, int Hq, int Hkv, int d,
                            int64_t N, int64_t rows, int64_t k, int64_t window, double* out, int64_t* idx,
                            double* vals, double* lse) {
    if (!q || !K || !V || !out || Hq < 1 || Hkv < 1 || d < 1 || N < 1 || k < 1 || Hq % Hkv)
        return 1;
    if (dtype < 0 || dtype > 2) return 1;
    int G = Hq / Hkv;
    int64_t W = window < N ? window : N;
    int64_t P = N - W;                           /* the search runs over positions [0, P) */
    int64_t k_eff = k < P ? k : P;
    int64_t n_att = k_eff + W;                   /* rows the softmax spans */
    double inv_sqrt_d = 1.0 / sqrt((double)d);

    /* 1. scores: raw dot product of each query with every cached key */
    double* S = (double*)malloc(sizeof(double) * (size_t)Hq * (size_t)N);
    if (!S) return 2;
    int rc = scores_impl(q, K, dtype, Hq, Hkv, d, N, rows, S);
    if (rc) { free(S); return rc; }

    double* tab = build_table(dtype);
    if (dtype != ORACLE_F32 && !tab) { free(S); return 2; }
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < Hq; ++h) {
        pair_t* p = (pair_t*)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
        double* w = (double*)malloc(sizeof(double) * (size_t)n_att);
        double* vd = (double*)malloc(sizeof(double) * (size_t)d);
        if (!p || !w || !vd) {
#pragma omp atomic write
            fail = 1;
            free(p); free(w); free(vd);
            continue;
        }
        for (int64_t i = 0; i < N; ++i) {
            p[i].s = S[(int64_t)h * N + i];
            p[i].i = i;
        }
        /* 2. exact search: full sort of the P prefix pairs, keep the first k_eff;
              the W window pairs p[P..N) follow them unsorted */
        qsort(p, (size_t)P, sizeof(pair_t), cmp_pair);
        if (k_eff < P) memmove(p + k_eff, p + P, sizeof(pair_t) * (size_t)W);
        /* 3. softmax over the retrieved and the window scores, scaled by 1/sqrt(d) */
        double m = -INFINITY;
        for (int64_t j = 0; j < n_att; ++j)
            if (p[j].s * inv_sqrt_d > m) m = p[j].s * inv_sqrt_d;
        double Z = 0.0;
        for (int64_t j = 0; j < n_att; ++j) {
            w[j] = exp(p[j].s * inv_sqrt_d - m);
            Z += w[j];
        }
        /* 4. weighted sum of the attended value rows */
        double* o = out + (int64_t)h * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int64_t j = 0; j < n_att; ++j) {
            widen_row(V, dtype, tab, ((int64_t)(h / G) * rows + p[j].i) * d, d, vd);
            double pj = w[j] / Z;
            for (int c = 0; c < d; ++c) o[c] += pj * vd[c];
        }
        if (lse) lse[h] = m + log(Z);
        for (int64_t j = 0; j < k; ++j) {
            if (idx) idx[(int64_t)h * k + j] = j < k_eff ? p[j].i : -1;
            if (vals) vals[(int64_t)h * k + j] = j < k_eff ? p[j].s : -INFINITY;
        }
        free(p); free(w); free(vd);
    }
    free(tab);
    free(S);
    return fail ? 2 : 0;
}
