/*
 * pqtopk.h -- C ABI of the MI355X (gfx950) PQTopK scoring library.
 *
 * PQTopK (Petrov, Macdonald, Tonellotto, RecSys '24, Section 3) scores every item of a catalogue whose item
 * embeddings are product-quantised (Section 2, "Sub-Id based recommendation"): item i carries m sub-ids
 * G[i] = {g_i1..g_im} (Eq. 1), split k owns b sub-item embeddings psi_{k,j} of length d/m, and for a sequence
 * embedding phi = phi_1 || .. || phi_m
 *
 *     S[k][j] = psi_{k,j} . phi_k                     (Eq. 4, the sub-id score matrix, once per query)
 *     r_i     = sum_{k} S[k][G[i][k]]                 (Eq. 5, m additions per item)
 *     result  = TopK(r, K)                            (Algorithm 1, V = I)
 *
 * Conventions shared by every entry point
 *   - Indices are 0-based.  N = |I| items, d embedding dim, m splits, b sub-ids per split, B queries, K results.
 *   - Every data pointer is a DEVICE pointer (HIP), dense row-major, owned by the caller for the whole call and
 *     until the enqueued work has finished.  `codes` must be 16-byte aligned, every float / int array 4-byte
 *     aligned (16-byte preferred).  The library allocates nothing, frees nothing and never synchronises: it
 *     enqueues kernels on `stream` (a hipStream_t passed as void*; NULL is the default stream) and returns.
 *     (The measurement aids of pqtopk_measure.h, which are not part of the product path, are the exception: they
 *     time their own launches and so create events and wait for the stream.)
 *   - Grids and workspace sizes are laid out for the 256 compute units of an MI355X.  On a GPU with another number
 *     of compute units every result is the same; only the speed differs.
 *   - Return value: PQ_OK (0) or a negative PQ_ERR_* code.  Arguments are validated on the host before any HIP
 *     call; on an argument error nothing is enqueued and no output is touched.
 *   - Arithmetic: fp32, round to nearest even, no flush to zero.  Eq. 4 is a left-to-right chain of fused
 *     multiply-adds over the d/m elements starting from +0; Eq. 5 is a left-to-right chain of fp32 additions
 *     over k = 0..m-1 starting from the k = 0 term; a finished score of -0 is returned as +0.
 *   - TopK order: score descending, then item id ascending.  The result is unique and is returned sorted.
 *   - Inputs must be finite and every sub-id must be < b; otherwise results are unspecified (no out-of-bounds
 *     access happens for any uint8 sub-id).
 */
#ifndef PQTOPK_H
#define PQTOPK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PQ_OK                0
#define PQ_ERR_NULL         -1   /* a required pointer is NULL */
#define PQ_ERR_SHAPE        -2   /* B, d, m, b, K or N < 1; d % m != 0; b > 256 (65536 for 16-bit sub-ids); K > N; N >= 2^31 */
#define PQ_ERR_UNSUPPORTED  -3   /* valid problem, but outside what the kernels cover (see PQ_MAX_*) */
#define PQ_ERR_WORKSPACE    -4   /* workspace smaller than pq_score_topk_workspace_bytes() */
#define PQ_ERR_ALIGN        -5   /* a pointer is not aligned as required */
#define PQ_ERR_HIP          -6   /* a HIP call (kernel launch) failed; pq_strerror() gives HIP's text */
#define PQ_ERR_TOO_LARGE    -7   /* pq_score_topk_static(): the problem needs more than PQ_STATIC_SCRATCH_BYTES of scratch */

#define PQ_MAX_K      512        /* largest K the top-K kernels keep per query */
#define PQ_MAX_M      128        /* largest number of splits (score tables of m*256 floats must fit LDS) */
#define PQ_MAX_B    65535        /* largest batch per call */
#define PQ_STATIC_SCRATCH_BYTES (8u << 20)   /* built-in scratch of pq_score_topk_static(), per GPU */

/*
 * Sub-id score matrix, Eq. 4 (Section 3): S[q][k][j] = psi_{k,j} . phi_{q,k}.
 *   queries    in   float [B][d]        sequence embeddings; chunk k is elements k*d/m .. (k+1)*d/m - 1
 *   centroids  in   float [m][b][d/m]   Psi_k, row j is psi_{k,j}
 *   S          out  float [B][m][b]
 * b may be as large as 65536 here (S does not depend on how the codebook stores its sub-ids).
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED (B > PQ_MAX_B), PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_subitem_scores(const float* queries, const float* centroids, float* S,
                      int B, int d, int m, int b, void* stream);

/*
 * Bytes of device workspace pq_score_topk() needs for this problem.  Pure host arithmetic, no HIP call.
 * Returns 0 for arguments pq_score_topk() would reject.
 */
size_t pq_score_topk_workspace_bytes(long long N, int B, int m, int b, int K);

/*
 * Algorithm 1 with V = I (Section 3): for each of B queries, score all N items by Eq. 5 from that query's S and
 * return the K best <item id, score> pairs.  Item scores are never written to memory.
 *   codes       in   uint8 [N][m]     codebook G (Eq. 1), sub-ids < b
 *   S           in   float [B][m][b]  from pq_subitem_scores() (or any finite table)
 *   out_ids     out  int32 [B][K]     rank r of query q at [q][r]; score descending, id ascending
 *   out_scores  out  float [B][K]     the scores of those items
 *   workspace        scratch of at least pq_score_topk_workspace_bytes(N, B, m, b, K) bytes, 16-byte aligned;
 *                    contents on entry are irrelevant (it receives every workgroup's K best keys, which one or
 *                    more small launches fold into the result); calls sharing a workspace must not overlap in time
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED (K > PQ_MAX_K, m > PQ_MAX_M, B > PQ_MAX_B, or m and K together
 *         too large for the 160 KB of LDS: m KB of score tables plus about 80*nextpow2(K+64) bytes of candidate
 *         lists; every K <= 512 fits with m <= 64, and m = 128 fits with K <= 64),
 *         PQ_ERR_WORKSPACE, PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_score_topk(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                  int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes, void* stream);

/*
 * pq_score_topk() for callers that cannot allocate or pass device scratch: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace), same kernels, same
 * result; the workgroups' partial top-K lists go to an array built into the library (PQ_STATIC_SCRATCH_BYTES = 8 MiB
 * of device memory per GPU the library runs on, held until the process ends) instead of a caller's workspace.  The
 * call allocates and frees nothing.
 *   - A problem whose pq_score_topk_workspace_bytes() exceeds PQ_STATIC_SCRATCH_BYTES is rejected with
 *     PQ_ERR_TOO_LARGE (nothing enqueued).  Every named workload fits (the largest, B = 1024 with K = 100, needs
 *     less than 2 MiB).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race and give unspecified results; calls on one stream are ordered and safe.  Nothing in the array
 *     has to survive from one call to the next.
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED, PQ_ERR_ALIGN, PQ_ERR_TOO_LARGE, PQ_ERR_HIP.
 */
int pq_score_topk_static(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                         int* out_ids, float* out_scores, void* stream);

/*
 * Algorithm 1 with V = I for codebooks whose sub-ids do not fit a byte.  The paper's codebook G holds natural numbers
 * and leaves b, the number of sub-ids per split, open (Section 2, Eq. 1); pq_score_topk() covers b <= 256 with one
 * byte per sub-id, this entry point b <= 65536 with two.  Same arithmetic, order and output as pq_score_topk().
 *   codes       in   uint16 [N][m]    codebook G, sub-ids < b (16-byte aligned)
 *   S           in   float [B][m][b]
 *   workspace        at least pq_score_topk_u16_workspace_bytes(N, B, m, b, K) bytes, 16-byte aligned
 * The query's whole m x b table is held in LDS when m * b * 4 bytes plus the candidate lists (about 80 *
 * nextpow2(K + 64) bytes) fit 160 KB, e.g. m * b <= 36864 at K = 10 (m = 8: b <= 4608); a larger table is read where
 * it lies, in device memory (it stays in L2; several times slower per lookup, sub-ids clamped to b - 1).  Rows of 8,
 * 16 or 32 bytes (m = 4, 8, 16) are scanned as 16-byte vectors; any other m row by row.  Every query of a batch scans
 * the codebook by itself (no shared pass).  A sub-id >= b makes the result unspecified, but no device memory outside the
 * arguments is touched: lookups in device memory are clamped to the table, lookups in LDS stay in LDS.
 * Errors: as pq_score_topk(), with PQ_ERR_SHAPE for b > 65536.
 */
size_t pq_score_topk_u16_workspace_bytes(long long N, int B, int m, int b, int K);
int pq_score_topk_u16(const uint16_t* codes, const float* S, long long N, int B, int m, int b, int K,
                      int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bytes of device workspace pq_score_topk_subset() needs for a candidate list of n_subset items.  Pure host
 * arithmetic, no HIP call.  Returns 0 for arguments pq_score_topk_subset() would reject.
 */
size_t pq_score_topk_subset_workspace_bytes(long long n_subset, int B, int m, int b, int K);

/*
 * Algorithm 1 with its optional argument V, a list of candidate items (Section 3): for each of B queries, score
 * only the items named in `subset` by Eq. 5 and return the K best <item id, score> pairs among them.  The list is
 * shared by the whole batch.  The rows G[V] are gathered from `codes` in place: no sub-matrix is materialised.
 *   codes       in   uint8 [N][m]        codebook G (Eq. 1) of the whole catalogue
 *   S           in   float [B][m][b]
 *   subset      in   int32 [n_subset]    item ids in [0, N), pairwise distinct, in any order (device pointer,
 *                                        4-byte aligned); the result does not depend on their order
 *   out_ids     out  int32 [B][K]        item ids (not positions in the list); score descending, id ascending
 *   out_scores  out  float [B][K]
 *   workspace        at least pq_score_topk_subset_workspace_bytes(n_subset, B, m, b, K) bytes, 16-byte aligned
 * The ids in the list cannot be checked on the host.  An id outside [0, N) is read as item N-1 (never out of
 * bounds); with such an id, or with a repeated id, the result is unspecified.
 * Errors: as pq_score_topk(), with PQ_ERR_SHAPE also for K > n_subset or n_subset > N.
 */
int pq_score_topk_subset(const uint8_t* codes, const float* S, const int* subset, long long n_subset, long long N,
                         int B, int m, int b, int K, int* out_ids, float* out_scores, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * The two scoring methods the paper compares PQTopK with, on the same inputs: the Transformer's default scoring
 * r = W phi over reconstructed item embeddings (Section 2, Eq. 2 and Eq. 3) and RecJPQ's original split-major
 * scoring (Algorithm 2, Section 3).  Both write one score per item to memory; pq_topk_scores() then ranks them.
 * They exist for comparison and cross-checks: pq_score_topk() is the product path and never materialises scores.
 */

/* Bytes of device workspace pq_topk_scores() needs; pure host arithmetic; 0 for arguments it would reject. */
size_t pq_topk_scores_workspace_bytes(long long N, int B, int K);

/*
 * TopK (Algorithm 1's and Algorithm 2's last step) over score rows that sit in memory.
 *   scores      in   float [B][ld]   row q holds query q's N scores (ld >= N; 16-byte aligned; ld % 4 == 0 if B > 1)
 *   out_ids     out  int32 [B][K]    score descending, id ascending;  out_scores float [B][K]  (-0 returned as +0)
 *   workspace        at least pq_topk_scores_workspace_bytes(N, B, K) bytes, 16-byte aligned
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE (N, B, K < 1, K > N, ld < N, N >= 2^31), PQ_ERR_UNSUPPORTED (K > PQ_MAX_K,
 *         B > PQ_MAX_B), PQ_ERR_WORKSPACE, PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_topk_scores(const float* scores, long long ld, long long N, int B, int K, int* out_ids, float* out_scores,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Algorithm 2 (RecJPQScore) without its TopK: for k = 0 .. m-1 in turn, one pass over all items adds split k's sub-id
 * score to the item's running score, scores[q][i] (+)= S[q][k][G[i][k]] (m launches, the score array re-read and
 * re-written by each).  Per item the additions happen in the same order as in pq_score_topk(), so the scores are
 * bit-equal to Eq. 5's as defined above.
 *   codes uint8 [N][m];  S float [B][m][b];  scores out float [B][ld], ld >= N
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED (m > PQ_MAX_M, B > PQ_MAX_B), PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_recjpq_scores(const uint8_t* codes, const float* S, long long N, int B, int m, int b, float* scores,
                     long long ld, void* stream);

/*
 * Eq. 2: the reconstructed item embedding matrix, W[i] = psi_{0,G[i][0]} || ... || psi_{m-1,G[i][m-1]} (copies only).
 *   codes uint8 [N][m];  centroids float [m][b][d/m];  W out float [N][d]  (N*d*4 bytes: 2.6 GB at N = 1.28M, d = 512)
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED (m > PQ_MAX_M), PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_reconstruct_items(const uint8_t* codes, const float* centroids, long long N, int d, int m, int b, float* W,
                         void* stream);

/*
 * Eq. 3, the default scoring: scores[q][i] = W[i] . phi_q in float32.  The paper fixes no order for this product, so
 * results agree with a float64 product to float32 rounding (not bit for bit with any particular order):
 *   - one or two queries: a mat-vec pass over W per query (sixteen lanes share a row of W, each accumulates every
 *     sixteenth 16-byte piece with fused multiply-adds, the partial sums are added across lanes);
 *   - three queries or more (and d a multiple of 16): ONE pass over W for the whole batch on the matrix cores, 32 queries
 *     x 64 items per wave, each score one left-to-right chain of fused multiply-adds over the d elements.
 *   W float [N][d] (16-byte aligned);  queries float [B][d] (16-byte aligned);  scores out float [B][ld], ld >= N
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_UNSUPPORTED (d % 4 != 0, d > 16384, B > PQ_MAX_B), PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_default_scores(const float* W, const float* queries, long long N, int B, int d, float* scores, long long ld,
                      void* stream);

/* Text for a PQ_* code; for PQ_ERR_HIP the text of the most recent HIP error seen by this thread. */
const char* pq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* PQTOPK_H */
