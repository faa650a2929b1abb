/* Test infrastructure (like the rest of oracle/): drives every entry point of pq_oracle.c on small seeded inputs, to
 * be compiled together with it under -fsanitize=address,undefined (tests/test_oracle_sanitized.py does so).  It checks
 * memory safety and undefined behaviour only; what the functions compute is pinned by tests/test_oracle_pins.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int pq_oracle_subitem_scores(const float*, const float*, float*, int, int, int, int);
int pq_oracle_item_scores(const uint8_t*, const float*, float*, long long, int, int);
int pq_oracle_item_scores_split_major(const uint8_t*, const float*, float*, long long, int, int);
int pq_oracle_topk_fullsort(const float*, long long, int, int*, float*);
int pq_oracle_topk(const float*, long long, int, int*, float*);
int pq_oracle_score_topk(const uint8_t*, const float*, long long, int, int, int, int, int*, float*);
int pq_oracle_score_topk_subset(const uint8_t*, const float*, const int*, long long, long long, int, int, int, int,
                                int*, float*);
int pq_oracle_pqtopk(const uint8_t*, const float*, const float*, long long, int, int, int, int, int, int*, float*);
int pq_oracle_bruteforce_topk(const uint8_t*, const float*, const float*, long long, int, int, int, int, int, int*,
                              double*);
int pq_oracle_reconstruct(const uint8_t*, const float*, long long, int, int, int, float*);
int pq_oracle_default_scores(const float*, const float*, long long, int, int, double*);
int pq_oracle_item_scores_u16(const uint16_t*, const float*, float*, long long, int, int);
int pq_oracle_score_topk_u16(const uint16_t*, const float*, long long, int, int, int, int, int*, float*);
int pq_oracle_bruteforce_topk_u16(const uint16_t*, const float*, const float*, long long, int, int, int, int, int, int*,
                                  double*);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (uint32_t)(state >> 32);
}
static float rndf(void) { return (float)(rnd() % 2001) / 1000.0f - 1.0f; }

#define CHECK(x) do { if ((x) != 0) { fprintf(stderr, "call failed: %s\n", #x); return 1; } } while (0)

int main(void) {
    for (int round = 0; round < 40; ++round) {
        const int m = 1 + (int)(rnd() % 9), s = 1 + (int)(rnd() % 5), d = m * s, b = 1 + (int)(rnd() % 256);
        const int B = 1 + (int)(rnd() % 3);
        const long long N = 1 + (long long)(rnd() % 300);
        const int K = 1 + (int)(rnd() % N);
        uint8_t* G = malloc((size_t)N * m);
        float* cent = malloc(sizeof(float) * (size_t)m * b * s);
        float* Q = malloc(sizeof(float) * (size_t)B * d);
        float* S = malloc(sizeof(float) * (size_t)B * m * b);
        float* sc = malloc(sizeof(float) * (size_t)N);
        float* W = malloc(sizeof(float) * (size_t)N * d);
        double* r = malloc(sizeof(double) * (size_t)B * N);
        int* ids = malloc(sizeof(int) * (size_t)B * K);
        float* out = malloc(sizeof(float) * (size_t)B * K);
        double* dout = malloc(sizeof(double) * (size_t)B * K);
        int* sub = malloc(sizeof(int) * (size_t)N);
        if (!G || !cent || !Q || !S || !sc || !W || !r || !ids || !out || !dout || !sub) return 2;
        for (long long i = 0; i < N * m; ++i) G[i] = (uint8_t)(rnd() % b);
        for (int i = 0; i < m * b * s; ++i) cent[i] = rndf();
        for (int i = 0; i < B * d; ++i) Q[i] = rndf();
        for (long long i = 0; i < N; ++i) sub[i] = (int)(N - 1 - i);
        CHECK(pq_oracle_subitem_scores(Q, cent, S, B, d, m, b));
        CHECK(pq_oracle_item_scores(G, S, sc, N, m, b));
        CHECK(pq_oracle_item_scores_split_major(G, S, sc, N, m, b));
        CHECK(pq_oracle_topk_fullsort(sc, N, K, ids, out));
        CHECK(pq_oracle_topk(sc, N, K, ids, out));
        CHECK(pq_oracle_score_topk(G, S, N, B, m, b, K, ids, out));
        CHECK(pq_oracle_score_topk_subset(G, S, sub, N, N, B, m, b, K, ids, out));
        CHECK(pq_oracle_pqtopk(G, cent, Q, N, B, d, m, b, K, ids, out));
        CHECK(pq_oracle_bruteforce_topk(G, cent, Q, N, B, d, m, b, K, ids, dout));
        CHECK(pq_oracle_reconstruct(G, cent, N, d, m, b, W));
        CHECK(pq_oracle_default_scores(W, Q, N, B, d, r));
        {   /* the same catalogue with its sub-ids held in 16 bits */
            uint16_t* G16 = malloc(sizeof(uint16_t) * (size_t)N * m);
            if (!G16) return 2;
            for (long long i = 0; i < N * m; ++i) G16[i] = G[i];
            CHECK(pq_oracle_item_scores_u16(G16, S, sc, N, m, b));
            CHECK(pq_oracle_score_topk_u16(G16, S, N, B, m, b, K, ids, out));
            CHECK(pq_oracle_bruteforce_topk_u16(G16, cent, Q, N, B, d, m, b, K, ids, dout));
            free(G16);
        }
        free(G); free(cent); free(Q); free(S); free(sc); free(W); free(r); free(ids); free(out); free(dout); free(sub);
    }
    puts("sanitized oracle run: ok");
    return 0;
}
