/*
 * Runs the plain-C oracle on the cases of a binary file and writes every result to a
 * second file.  Built with -fsanitize=address,undefined by tests/test_sanitizers_cpu.py,
 * which compares the results with those of the oracle's ordinary build: any out-of-bounds
 * access, use after free, leak, signed overflow or misaligned access in the oracle ends
 * the run with a non-zero status.
 *
 * Input:  int64 n_cases; per case int64 {dtype, M, Hq, Hkv, d, N, causal, k, window},
 *         then q [M, Hq, d], K [Hkv, N, d], V [Hkv, N, d] in the storage type.
 * Output: per case int64 rc; if rc == 0: out [M, Hq, d] f64, idx [M, Hq, k] i64,
 *         vals [M, Hq, k] f64, lse [M, Hq] f64, scores of query 0 [Hq, N] f64.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_scores(const void* q, const void* K, int dtype, int Hq, int Hkv, int d, int64_t N, double* S);
int oracle_topk_attention(const void* q, const void* K, const void* V, int dtype, int Hq, int Hkv, int d, int64_t N,
                          int64_t k, double* out, int64_t* idx, double* vals, double* lse);
int oracle_topk_attention_window(const void* q, const void* K, const void* V, int dtype, int Hq, int Hkv, int d,
                                 int64_t N, int64_t k, int64_t window, double* out, int64_t* idx, double* vals,
                                 double* lse);
int oracle_topk_attention_multi(const void* q, const void* K, const void* V, int dtype, int M, int Hq, int Hkv, int d,
                                int64_t N, int causal, int64_t k, int64_t window, double* out, int64_t* idx,
                                double* vals, double* lse);

static void* read_block(FILE* f, size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short read\n"); exit(3); }
    return p;
}

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* in = fopen(argv[1], "rb");
    FILE* out_f = fopen(argv[2], "wb");
    if (!in || !out_f) return 2;
    int64_t n_cases = 0;
    if (fread(&n_cases, sizeof n_cases, 1, in) != 1) return 3;
    for (int64_t c = 0; c < n_cases; ++c) {
        int64_t hd[9];
        if (fread(hd, sizeof hd, 1, in) != 1) return 3;
        const int dtype = (int)hd[0], M = (int)hd[1], Hq = (int)hd[2], Hkv = (int)hd[3], d = (int)hd[4];
        const int64_t N = hd[5], k = hd[7], window = hd[8];
        const int causal = (int)hd[6];
        const size_t e = dtype == 0 ? 4 : 2;
        void* q = read_block(in, (size_t)M * Hq * d * e);
        void* K = read_block(in, (size_t)Hkv * N * d * e);
        void* V = read_block(in, (size_t)Hkv * N * d * e);
        const size_t n_out = (size_t)M * Hq * d, n_sel = (size_t)M * Hq * k, n_lse = (size_t)M * Hq;
        double* o = malloc(sizeof(double) * n_out);
        int64_t* idx = malloc(sizeof(int64_t) * n_sel);
        double* vals = malloc(sizeof(double) * n_sel);
        double* lse = malloc(sizeof(double) * n_lse);
        double* S = malloc(sizeof(double) * (size_t)Hq * N);
        if (!o || !idx || !vals || !lse || !S) return 4;
        int64_t rc;
        if (M == 1 && window == 0 && !causal)
            rc = oracle_topk_attention(q, K, V, dtype, Hq, Hkv, d, N, k, o, idx, vals, lse);
        else if (M == 1 && !causal)
            rc = oracle_topk_attention_window(q, K, V, dtype, Hq, Hkv, d, N, k, window, o, idx, vals, lse);
        else
            rc = oracle_topk_attention_multi(q, K, V, dtype, M, Hq, Hkv, d, N, causal, k, window, o, idx, vals, lse);
        if (rc == 0) rc = oracle_scores(q, K, dtype, Hq, Hkv, d, N, S);
        fwrite(&rc, sizeof rc, 1, out_f);
        if (rc == 0) {
            fwrite(o, sizeof(double), n_out, out_f);
            fwrite(idx, sizeof(int64_t), n_sel, out_f);
            fwrite(vals, sizeof(double), n_sel, out_f);
            fwrite(lse, sizeof(double), n_lse, out_f);
            fwrite(S, sizeof(double), (size_t)Hq * N, out_f);
        }
        free(q); free(K); free(V); free(o); free(idx); free(vals); free(lse); free(S);
    }
    fclose(in);
    fclose(out_f);
    return 0;
}
