/*
 * CPU oracle for PQTopK scoring -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may call this file.  It shares no
 * code, header, table or helper with the HIP library; it is written from the paper alone (Petrov, Macdonald,
 * Tonellotto, "Efficient Inference of Sub-Item Id-based Sequential Recommendation Models with Millions of
 * Items", RecSys '24) and is deliberately plain: no blocking, no fusion, no vector intrinsics.
 *
 * Notation as in the paper, 0-based here:
 *   N = |I| items, d embedding dim, m splits, s = d/m, b sub-ids per split, B queries, K results.
 *   codes      uint8 [N][m]       codebook G, Eq. 1 (uint16 in the *_u16 functions: the paper's G holds natural
 *                                 numbers and leaves b open; one byte per sub-id is the b <= 256 case)
 *   centroids  float [m][b][s]    sub-item embeddings Psi_k (Section 2, "Sub-Id based recommendation")
 *   queries    float [B][d]       sequence embeddings phi; phi_k is the k-th contiguous chunk of length s (Section 3)
 *   S          float [B][m][b]    sub-id score matrix, Eq. 4
 *
 * The paper fixes what is computed, not a floating-point evaluation order or a tie rule.  The readings used here:
 *   - fp32 throughout; Eq. 4 is evaluated as a left-to-right chain of fused multiply-adds over t = 0..s-1
 *     starting from 0; Eq. 5 as a left-to-right chain of fp32 additions over k = 0..m-1 starting from the k = 0
 *     term; round to nearest even; -0.0 is turned into +0.0 by adding +0.0f to the finished score.
 *   - TopK (Algorithm 1, last line) orders items by score descending and, between equal scores, by item id
 *     ascending, and returns the first K <id, score> pairs in that order.
 *
 * Every function returns 0 on success and -1 on an argument error.  All pointers are host pointers owned by the
 * caller.  Parity status: every function below is pinned by tests (hand-worked example, reconstruction brute
 * force in float64, closed forms and invariants); nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the item loop will use (1 when built without OpenMP) */
int pq_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void pq_oracle_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Eq. 4: s_{k,j} = psi_{k,j} . phi_k, for every query. */
int pq_oracle_subitem_scores(const float* queries, const float* centroids, float* S,
                             int B, int d, int m, int b) {
    if (!queries || !centroids || !S || B < 1 || d < 1 || m < 1 || b < 1 || d % m != 0) return -1;
    const int s = d / m;
    for (int q = 0; q < B; ++q) {
        for (int k = 0; k < m; ++k) {
            const float* phi_k = queries + (size_t)q * d + (size_t)k * s;
            for (int j = 0; j < b; ++j) {
                const float* psi = centroids + ((size_t)k * b + j) * s;
                float acc = 0.0f;
                for (int t = 0; t < s; ++t) acc = fmaf(psi[t], phi_k[t], acc);
                S[((size_t)q * m + k) * b + j] = acc;
            }
        }
    }
    return 0;
}

/* Eq. 5 / Algorithm 1, the loop over items: score[i] = sum_k S[k][G[i][k]] for ONE query (S is [m][b]). */
int pq_oracle_item_scores(const uint8_t* codes, const float* S, float* score, long long N, int m, int b) {
    if (!codes || !S || !score || N < 1 || m < 1 || b < 1 || b > 256) return -1;
    if (b < 256)                                   /* a uint8 sub-id is always in range when b = 256 */
        for (long long i = 0; i < N; ++i)
            for (int k = 0; k < m; ++k)
                if (codes[i * m + k] >= b) return -1;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < N; ++i) {
        const uint8_t* g = codes + i * m;
        float acc = S[g[0]];
        for (int k = 1; k < m; ++k) acc = acc + S[(size_t)k * b + g[k]];
        score[i] = acc + 0.0f;
    }
    return 0;
}

/* Algorithm 2 (RecJPQ's original scoring): same sums with the loops swapped -- the outer loop runs over splits
 * and every item keeps an accumulator.  The accumulator starts at 0 as the listing says; adding the k = 0 term
 * to +0 gives that term exactly (or +0 for a -0 term, which the final "+ 0.0f" of Algorithm 1's reading also
 * produces), so the two loop orders give the same bits. */
int pq_oracle_item_scores_split_major(const uint8_t* codes, const float* S, float* score,
                                      long long N, int m, int b) {
    if (!codes || !S || !score || N < 1 || m < 1 || b < 1 || b > 256) return -1;
    for (long long i = 0; i < N; ++i) score[i] = 0.0f;
    for (int k = 0; k < m; ++k)
        for (long long i = 0; i < N; ++i) {
            int g = codes[i * m + k];
            if (g >= b) return -1;
            score[i] += S[(size_t)k * b + g];
        }
    return 0;
}

/* strict "a ranks before b": higher score first, lower id between equal scores */
static int ranks_before(float sa, long long ia, float sb, long long ib) {
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return ia < ib;
}

/* TopK by its definition: sort every item id under the order above, keep the first K. */
typedef struct { float score; int id; } pair_t;

static int pair_cmp(const void* pa, const void* pb) {
    const pair_t* a = (const pair_t*)pa;
    const pair_t* b = (const pair_t*)pb;
    if (ranks_before(a->score, a->id, b->score, b->id)) return -1;
    if (ranks_before(b->score, b->id, a->score, a->id)) return 1;
    return 0;
}

int pq_oracle_topk_fullsort(const float* score, long long N, int K, int* out_ids, float* out_scores) {
    if (!score || !out_ids || !out_scores || N < 1 || K < 1 || K > N || N >= 2147483648LL) return -1;
    pair_t* all = (pair_t*)malloc((size_t)N * sizeof(pair_t));
    if (!all) return -1;
    for (long long i = 0; i < N; ++i) { all[i].score = score[i]; all[i].id = (int)i; }
    qsort(all, (size_t)N, sizeof(pair_t), pair_cmp);
    for (int r = 0; r < K; ++r) { out_ids[r] = all[r].id; out_scores[r] = all[r].score; }
    free(all);
    return 0;
}

/* TopK by one scan that keeps the best K seen so far in rank order (insertion into a sorted list of length K).
 * Same result as the full sort -- the tests hold the two against each other -- but linear in N, so the large
 * catalogues finish. */
int pq_oracle_topk(const float* score, long long N, int K, int* out_ids, float* out_scores) {
    if (!score || !out_ids || !out_scores || N < 1 || K < 1 || K > N || N >= 2147483648LL) return -1;
    int kept = 0;
    for (long long i = 0; i < N; ++i) {
        float sc = score[i];
        if (kept == K && !ranks_before(sc, i, out_scores[K - 1], out_ids[K - 1])) continue;
        int pos = (kept < K) ? kept : K - 1;          /* slot that is free or holds the entry to drop */
        while (pos > 0 && ranks_before(sc, i, out_scores[pos - 1], out_ids[pos - 1])) {
            out_scores[pos] = out_scores[pos - 1];
            out_ids[pos] = out_ids[pos - 1];
            --pos;
        }
        out_scores[pos] = sc;
        out_ids[pos] = (int)i;
        if (kept < K) ++kept;
    }
    return 0;
}

/* Algorithm 1 with V = I for a batch: for every query, score all items from its S, then TopK.
 * S is [B][m][b]; out_ids / out_scores are [B][K]. */
int pq_oracle_score_topk(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                         int* out_ids, float* out_scores) {
    if (!codes || !S || !out_ids || !out_scores || N < 1 || B < 1 || m < 1 || b < 1 || b > 256 || K < 1 ||
        K > N || N >= 2147483648LL)
        return -1;
    float* score = (float*)malloc((size_t)N * sizeof(float));
    if (!score) return -1;
    int rc = 0;
    for (int q = 0; q < B && rc == 0; ++q) {
        rc = pq_oracle_item_scores(codes, S + (size_t)q * m * b, score, N, m, b);
        if (rc == 0) rc = pq_oracle_topk(score, N, K, out_ids + (size_t)q * K, out_scores + (size_t)q * K);
    }
    free(score);
    return rc;
}

/* Algorithm 1 with a candidate list V (its optional argument, Section 3): for every query, score only the items
 * whose ids are listed in subset[0..n) (each id in [0, N), no id listed twice), then TopK among them under the same
 * order (score descending, lower ITEM ID first).  One candidate list serves all B queries.  The loop is the
 * algorithm's own: for each listed item, the sum over splits of S[k][G[item][k]] from the k = 0 term on. */
int pq_oracle_score_topk_subset(const uint8_t* codes, const float* S, const int* subset, long long n, long long N,
                                int B, int m, int b, int K, int* out_ids, float* out_scores) {
    if (!codes || !S || !subset || !out_ids || !out_scores || n < 1 || N < 1 || B < 1 || m < 1 || b < 1 || b > 256 ||
        K < 1 || K > n || N >= 2147483648LL)
        return -1;
    for (long long p = 0; p < n; ++p)
        if (subset[p] < 0 || subset[p] >= N) return -1;
    for (int q = 0; q < B; ++q) {
        const float* Sq = S + (size_t)q * m * b;
        int* ids = out_ids + (size_t)q * K;
        float* scs = out_scores + (size_t)q * K;
        int kept = 0;
        for (long long p = 0; p < n; ++p) {
            const long long item = subset[p];
            const uint8_t* row = codes + (size_t)item * m;
            if (row[0] >= b) return -1;
            float acc = Sq[row[0]];
            for (int k = 1; k < m; ++k) {
                if (row[k] >= b) return -1;
                acc = acc + Sq[(size_t)k * b + row[k]];
            }
            const float sc = acc + 0.0f;                       /* a sum of -0 counts as +0 */
            if (kept == K && !ranks_before(sc, item, scs[K - 1], ids[K - 1])) continue;
            int pos = (kept < K) ? kept : K - 1;
            while (pos > 0 && ranks_before(sc, item, scs[pos - 1], ids[pos - 1])) {
                scs[pos] = scs[pos - 1];
                ids[pos] = ids[pos - 1];
                --pos;
            }
            scs[pos] = sc;
            ids[pos] = (int)item;
            if (kept < K) ++kept;
        }
    }
    return 0;
}

/* The whole path from embeddings: Eq. 4, then Algorithm 1. */
int pq_oracle_pqtopk(const uint8_t* codes, const float* centroids, const float* queries,
                     long long N, int B, int d, int m, int b, int K, int* out_ids, float* out_scores) {
    if (B < 1 || m < 1 || b < 1) return -1;
    float* S = (float*)malloc((size_t)B * m * b * sizeof(float));
    if (!S) return -1;
    int rc = pq_oracle_subitem_scores(queries, centroids, S, B, d, m, b);
    if (rc == 0) rc = pq_oracle_score_topk(codes, S, N, B, m, b, K, out_ids, out_scores);
    free(S);
    return rc;
}

/* Exhaustive scoring by reconstruction, in float64: w_i is the concatenation of the item's sub-item embeddings
 * (Eq. 2), r_i = w_i . phi (Eq. 3), then TopK by full sort under the same order.  out_scores is double [B][K].
 * This is the definition PQTopK must reproduce (it is a safe method: Sections 1 and 3); meant for small N. */
typedef struct { double score; int id; } dpair_t;

static int dpair_cmp(const void* pa, const void* pb) {
    const dpair_t* a = (const dpair_t*)pa;
    const dpair_t* b = (const dpair_t*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

int pq_oracle_bruteforce_topk(const uint8_t* codes, const float* centroids, const float* queries,
                              long long N, int B, int d, int m, int b, int K, int* out_ids, double* out_scores) {
    if (!codes || !centroids || !queries || !out_ids || !out_scores || N < 1 || B < 1 || d < 1 || m < 1 ||
        b < 1 || b > 256 || d % m != 0 || K < 1 || K > N || N >= 2147483648LL)
        return -1;
    const int s = d / m;
    double* w = (double*)malloc((size_t)d * sizeof(double));
    dpair_t* all = (dpair_t*)malloc((size_t)N * sizeof(dpair_t));
    if (!w || !all) { free(w); free(all); return -1; }
    for (int q = 0; q < B; ++q) {
        const float* phi = queries + (size_t)q * d;
        for (long long i = 0; i < N; ++i) {
            for (int k = 0; k < m; ++k) {                       /* Eq. 2: concatenate */
                int g = codes[i * m + k];
                if (g >= b) { free(w); free(all); return -1; }
                for (int t = 0; t < s; ++t) w[k * s + t] = (double)centroids[((size_t)k * b + g) * s + t];
            }
            double r = 0.0;                                     /* Eq. 3: dot product */
            for (int t = 0; t < d; ++t) r += w[t] * (double)phi[t];
            all[i].score = r;
            all[i].id = (int)i;
        }
        qsort(all, (size_t)N, sizeof(dpair_t), dpair_cmp);
        for (int r = 0; r < K; ++r) {
            out_ids[(size_t)q * K + r] = all[r].id;
            out_scores[(size_t)q * K + r] = all[r].score;
        }
    }
    free(w);
    free(all);
    return 0;
}

/* Eq. 2 (Section 2): the reconstructed item embedding matrix W, float [N][d]: row i is the concatenation of the
 * item's m sub-item embeddings psi_{k, G[i][k]}.  Copies only: exact. */
int pq_oracle_reconstruct(const uint8_t* codes, const float* centroids, long long N, int d, int m, int b, float* W) {
    if (!codes || !centroids || !W || N < 1 || d < 1 || m < 1 || b < 1 || b > 256 || d % m != 0) return -1;
    const int s = d / m;
    for (long long i = 0; i < N; ++i)
        for (int k = 0; k < m; ++k) {
            int g = codes[i * m + k];
            if (g >= b) return -1;
            for (int t = 0; t < s; ++t) W[i * d + (long long)k * s + t] = centroids[((size_t)k * b + g) * s + t];
        }
    return 0;
}

/* Eq. 3 (Section 2), the Transformer's default scoring r = W phi, in float64: scores double [B][N].
 * The paper fixes no evaluation order for this product; float64 is the reference a float32 product is held to. */
int pq_oracle_default_scores(const float* W, const float* queries, long long N, int B, int d, double* scores) {
    if (!W || !queries || !scores || N < 1 || B < 1 || d < 1) return -1;
    for (int q = 0; q < B; ++q) {
        const float* phi = queries + (size_t)q * d;
#pragma omp parallel for schedule(static)
        for (long long i = 0; i < N; ++i) {
            double r = 0.0;
            for (int t = 0; t < d; ++t) r += (double)W[i * d + t] * (double)phi[t];
            scores[(size_t)q * N + i] = r;
        }
    }
    return 0;
}


/* ---- sub-ids wider than a byte (b up to 65536): the same definitions over uint16 codes ---- */

/* Eq. 5 / Algorithm 1, the loop over items, for ONE query (S is [m][b]), codes uint16 [N][m]. */
int pq_oracle_item_scores_u16(const uint16_t* codes, const float* S, float* score, long long N, int m, int b) {
    if (!codes || !S || !score || N < 1 || m < 1 || b < 1 || b > 65536) return -1;
    for (long long i = 0; i < N; ++i)
        for (int k = 0; k < m; ++k)
            if (codes[i * m + k] >= b) return -1;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < N; ++i) {
        const uint16_t* g = codes + i * m;
        float acc = S[g[0]];
        for (int k = 1; k < m; ++k) acc = acc + S[(size_t)k * b + g[k]];
        score[i] = acc + 0.0f;
    }
    return 0;
}

/* Algorithm 1 with V = I for a batch, codes uint16 [N][m]: score all items from the query's S, then TopK. */
int pq_oracle_score_topk_u16(const uint16_t* codes, const float* S, long long N, int B, int m, int b, int K,
                             int* out_ids, float* out_scores) {
    if (!codes || !S || !out_ids || !out_scores || N < 1 || B < 1 || m < 1 || b < 1 || b > 65536 || K < 1 ||
        K > N || N >= 2147483648LL)
        return -1;
    float* score = (float*)malloc((size_t)N * sizeof(float));
    if (!score) return -1;
    int rc = 0;
    for (int q = 0; q < B && rc == 0; ++q) {
        rc = pq_oracle_item_scores_u16(codes, S + (size_t)q * m * b, score, N, m, b);
        if (rc == 0) rc = pq_oracle_topk(score, N, K, out_ids + (size_t)q * K, out_scores + (size_t)q * K);
    }
    free(score);
    return rc;
}

/* Exhaustive scoring by reconstruction in float64 (Eq. 2, Eq. 3, full sort), codes uint16 [N][m]. */
int pq_oracle_bruteforce_topk_u16(const uint16_t* codes, const float* centroids, const float* queries,
                                  long long N, int B, int d, int m, int b, int K, int* out_ids, double* out_scores) {
    if (!codes || !centroids || !queries || !out_ids || !out_scores || N < 1 || B < 1 || d < 1 || m < 1 ||
        b < 1 || b > 65536 || d % m != 0 || K < 1 || K > N || N >= 2147483648LL)
        return -1;
    const int s = d / m;
    dpair_t* all = (dpair_t*)malloc((size_t)N * sizeof(dpair_t));
    if (!all) return -1;
    for (int q = 0; q < B; ++q) {
        const float* phi = queries + (size_t)q * d;
        for (long long i = 0; i < N; ++i) {
            double r = 0.0;                                     /* Eq. 3 over the concatenation of Eq. 2, in place */
            for (int k = 0; k < m; ++k) {
                int g = codes[i * m + k];
                if (g >= b) { free(all); return -1; }
                const float* psi = centroids + ((size_t)k * b + g) * s;
                for (int t = 0; t < s; ++t) r += (double)psi[t] * (double)phi[k * s + t];
            }
            all[i].score = r;
            all[i].id = (int)i;
        }
        qsort(all, (size_t)N, sizeof(dpair_t), dpair_cmp);
        for (int r = 0; r < K; ++r) {
            out_ids[(size_t)q * K + r] = all[r].id;
            out_scores[(size_t)q * K + r] = all[r].score;
        }
    }
    free(all);
    return 0;
}
