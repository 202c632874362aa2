/*
 * CPU oracle for the Block-Sparse FlashAttention forward pass.  TEST INFRASTRUCTURE ONLY:
 * it is loaded by the tests, by the smoke check and by the benchmark's CPU-baseline leg,
 * never by the product path, and it shares no code with the HIP kernels.
 *
 * What it computes (paper Section 4.1, Eq. 5-6, and Algorithm 1 collapsed to its fixed point):
 * the gate decision of a key block depends only on the score tile S_ij and the threshold,
 * never on the running statistics, so the result of Algorithm 1 is the exact softmax
 * attention of Section 2.1 restricted to the kept key blocks.  The oracle therefore evaluates
 * that definition directly, two passes per query tile, no online rescaling, no blocking of
 * the reduction:
 *   1. S = Q_i K^T / sqrt(d) for every reachable key           (Section 4.1, Eq. 5)
 *   2. classify key blocks: gateable (every entry visible) or diagonal (touches the causal
 *      boundary; always processed, Section 4.1 last paragraph, Algorithm 1 diagonal step)
 *   3. block maximum s_max = max_{p,q} S_ij                    (Eq. 6)
 *      keep(i,j) = diagonal or s_max >= T                      (Section 4.1: skip iff s_max < T)
 *   4. per row: softmax over the visible entries of kept blocks, times V
 *      (Algorithm 1 update steps and finalisation, collapsed), LSE = m + log(l)
 * All arithmetic is fp64 on fp32 inputs; the gate compares the block maximum rounded to
 * fp32 with the fp32 threshold (the precision the kernel decides in).
 *
 * Layout: q [B][N][Hq][d], k and v [B][N][Hkv][d], contiguous fp32.  Query head h reads KV
 * head h / (Hq / Hkv).  Work is a list of items (b, h, i) = one query tile of one head each.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { CLS_UNREACHABLE = 0, CLS_SKIPPED = 1, CLS_KEPT = 2, CLS_DIAGONAL = 3 };

int bsfa_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Classification of key block j for query tile i (0 unreachable, 2 gateable, 3 diagonal).
 * Causal: reachable iff its first key is not after the tile's last row; gateable iff its
 * last key is not after the tile's first row (no entry needs masking).
 * Non-causal: every block is reachable; blocks overlapping the tile's own token range play
 * the role of the diagonal (always kept, so no row can lose all its keys). */
static int classify(int i, int j, int BM, int BN, int causal)
{
    long r0 = (long)i * BM, r1 = r0 + BM - 1;      /* first / last query row */
    long c0 = (long)j * BN, c1 = c0 + BN - 1;      /* first / last key       */
    if (causal) {
        if (c0 > r1) return CLS_UNREACHABLE;
        if (c1 <= r0) return CLS_KEPT;             /* gateable */
        return CLS_DIAGONAL;
    }
    if (c0 <= r1 && c1 >= r0) return CLS_DIAGONAL;
    return CLS_KEPT;
}

static int one_item(const float *q, const float *k, const float *v,
                    int N, int Hq, int Hkv, int d, int BM, int BN, int causal,
                    float tau, int b, int h, int i, const uint8_t *forced_keep,
                    float *out, float *bmax, uint8_t *cls, double *psum, float *lse)
{
    const int MKV = N / BN;
    const int g = h / (Hq / Hkv);
    const long nk = causal ? (long)(i + 1) * BM : (long)N;    /* reachable keys */
    const double scale = 1.0 / sqrt((double)d);
    double *S = (double *)malloc(sizeof(double) * (size_t)BM * (size_t)nk);
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    if (!S || !acc) { free(S); free(acc); return -1; }

    /* 1. scores, with the causal mask written as -inf */
    for (int p = 0; p < BM; ++p) {
        const long row = (long)i * BM + p;
        const float *qr = q + (((size_t)b * N + row) * Hq + h) * d;
        for (long t = 0; t < nk; ++t) {
            double s;
            if (causal && t > row) {
                s = -INFINITY;
            } else {
                const float *kr = k + (((size_t)b * N + t) * Hkv + g) * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += (double)qr[c] * (double)kr[c];
                s = dot * scale;
            }
            S[(size_t)p * nk + t] = s;
        }
    }

    /* 2.-3. classes, block maxima, gate */
    for (int j = 0; j < MKV; ++j) {
        int c = classify(i, j, BM, BN, causal);
        float bm = NAN;
        if (c == CLS_KEPT) {                       /* gateable: take the decision */
            double m = -INFINITY;
            for (int p = 0; p < BM; ++p)
                for (int t = 0; t < BN; ++t) {
                    double s = S[(size_t)p * nk + (size_t)j * BN + t];
                    if (s > m) m = s;
                }
            bm = (float)m;
            int keep = forced_keep ? (forced_keep[j] != 0) : (bm >= tau);
            c = keep ? CLS_KEPT : CLS_SKIPPED;
        }
        bmax[j] = bm;
        cls[j] = (uint8_t)c;
    }

    /* 4. softmax over the visible entries of kept blocks, times V */
    for (int p = 0; p < BM; ++p) {
        const double *Sr = S + (size_t)p * nk;
        double m = -INFINITY;
        for (long t = 0; t < nk; ++t)
            if (cls[t / BN] >= CLS_KEPT && Sr[t] > m) m = Sr[t];
        double l = 0.0;
        for (int c = 0; c < d; ++c) acc[c] = 0.0;
        for (long t = 0; t < nk; ++t) {
            if (cls[t / BN] < CLS_KEPT || Sr[t] == -INFINITY) continue;
            double e = exp(Sr[t] - m);
            l += e;
            const float *vr = v + (((size_t)b * N + t) * Hkv + g) * d;
            for (int c = 0; c < d; ++c) acc[c] += e * (double)vr[c];
        }
        for (int c = 0; c < d; ++c) out[(size_t)p * d + c] = (float)(acc[c] / l);
        if (psum) {                                 /* sum of the normalised probabilities */
            double ps = 0.0;
            for (long t = 0; t < nk; ++t)
                if (cls[t / BN] >= CLS_KEPT && Sr[t] != -INFINITY) ps += exp(Sr[t] - m) / l;
            psum[p] = ps;
        }
        if (lse) lse[p] = (float)(m + log(l));
    }
    free(S);
    free(acc);
    return 0;
}

/*
 * items        [n_items][3] = (b, h, i)
 * tau          [Hq] thresholds, or [Hq][N/BM] when tau_per_tile != 0 (one per query tile,
 *              the paper's T_{l,h,i} for a single layer and sparsity level)
 * forced_keep  NULL, or [n_items][N/BN]: nonzero keeps a gateable block whatever its maximum
 * out          [n_items][BM][d]
 * bmax         [n_items][N/BN], NaN where the block is not gateable
 * cls          [n_items][N/BN], 0 unreachable / 1 skipped / 2 kept by the gate / 3 diagonal
 * psum, lse    NULL or [n_items][BM]
 * Returns 0, -1 on allocation failure, -2 on a bad argument.
 */
int bsfa_oracle_items(const float *q, const float *k, const float *v,
                      int B, int N, int Hq, int Hkv, int d, int BM, int BN, int causal,
                      const float *tau, int tau_per_tile,
                      const int32_t *items, int n_items, const uint8_t *forced_keep,
                      float *out, float *bmax, uint8_t *cls, double *psum, float *lse)
{
    if (!q || !k || !v || !tau || !items || !out || !bmax || !cls) return -2;
    if (B < 1 || N < 1 || d < 1 || BM < 1 || BN < 1 || Hkv < 1 || Hq % Hkv) return -2;
    if (N % BM || N % BN) return -2;
    const int MQ = N / BM, MKV = N / BN;
    for (int n = 0; n < n_items; ++n) {
        const int32_t *it = items + 3 * (size_t)n;
        if (it[0] < 0 || it[0] >= B || it[1] < 0 || it[1] >= Hq || it[2] < 0 || it[2] >= MQ) return -2;
    }
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < n_items; ++n) {
        const int b = items[3 * n], h = items[3 * n + 1], i = items[3 * n + 2];
        const float t = tau_per_tile ? tau[(size_t)h * MQ + i] : tau[h];
        int rc = one_item(q, k, v, N, Hq, Hkv, d, BM, BN, causal, t, b, h, i,
                          forced_keep ? forced_keep + (size_t)n * MKV : NULL,
                          out + (size_t)n * BM * d, bmax + (size_t)n * MKV, cls + (size_t)n * MKV,
                          psum ? psum + (size_t)n * BM : NULL, lse ? lse + (size_t)n * BM : NULL);
        if (rc) {
#pragma omp atomic write
            status = rc;
        }
    }
    return status;
}
