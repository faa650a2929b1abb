// Algorithm 1 with a candidate list V, for lists short enough that a workgroup's share fits its registers and K < 32
// (scan_subset_kernel): lists of up to a couple of million candidates at batch 1.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp,
// scan_batched.hpp, fold.hpp, comparison.hpp.
#pragma once

// Most 16-byte code vectors' worth of gathered rows a thread of the candidate-list kernel holds.
constexpr int kSubsetMaxVecs = 8;

// grid = (list blocks, B); one query per workgroup.  A thread holds R = U * (16 / M) candidates: slot s of thread t of
// workgroup g is position (s * blocks + g) * NT + t of the list (slot s of all workgroups together is one contiguous
// stretch of V: the ids are read coalesced).  Every id is requested first, then every row G[V[p]] (M bytes each,
// gathered where they lie: a random list costs a 32-byte sector per row), then the query's table goes to LDS; the rows
// of 16 / M candidates are packed into one code vector and scored by the scan's own routine (same lookups, same
// left-to-right sums), and the workgroup's K best come out of select_small_k(), keyed by ITEM id: ties go to the lower
// item id wherever it sits in the list.  The general kernel reads a row only when its turn comes and scores row after
// row; here all of a thread's rows are on their way at once, which is what a gather needs.
//   M: bytes of an item's row (4, 8 or 16); U: code vectors' worth of rows per thread (1 .. kSubsetMaxVecs)
// An id outside [0, n_items) is clamped to n_items - 1 (memory-safe; the result is then unspecified, as documented).
template <int M, int U, int NT>
__global__ __launch_bounds__(NT) void scan_subset_kernel(ScanArgs a) {
    constexpr int IPV = 16 / M, WPI = M / 4;                   // candidates per code vector, 4-byte words per row
    constexpr int R = U * IPV;
    static_assert(M == 4 || M == 8 || M == 16, "rows of 4, 8 or 16 bytes");
    static_assert(U >= 1 && U <= kSubsetMaxVecs, "vectors per thread");
    __shared__ __align__(16) float lut[M * kLutStride];
    __shared__ SmallSelectLds<NT> sel;
    const int tid = threadIdx.x;
    const int q = blockIdx.y, nblk = gridDim.x, blk = blockIdx.x, K = a.K, b = a.b;
    const uint32_t n = (uint32_t)a.N;                          // candidates in the list
    const uint32_t first = (uint32_t)blk * NT + (uint32_t)tid, stride = (uint32_t)nblk * NT;

    // ---- the ids (coalesced), then the rows they name
    uint32_t item[R];
#pragma unroll
    for (int s = 0; s < R; ++s) {
        const uint32_t pos = first + (uint32_t)s * stride;
        item[s] = (uint32_t)a.subset[pos < n ? pos : n - 1];  // (past the end: a re-read, never scored)
    }
    uint32_t w[U][4];
#pragma unroll
    for (int s = 0; s < R; ++s) {
        const uint32_t i = item[s] < a.n_items ? item[s] : a.n_items - 1;
        const uint32_t* row = reinterpret_cast<const uint32_t*>(a.codes + (size_t)i * M);
        if constexpr (M == 4) {
            w[s / IPV][s % IPV] = row[0];
        } else if constexpr (M == 8) {
            const uint2 x = *reinterpret_cast<const uint2*>(row);
            w[s / IPV][2 * (s % IPV)] = x.x; w[s / IPV][2 * (s % IPV) + 1] = x.y;
        } else {
            const uint4 x = *reinterpret_cast<const uint4*>(row);
            w[s][0] = x.x; w[s][1] = x.y; w[s][2] = x.z; w[s][3] = x.w;
        }
        item[s] = i;
    }
    static_assert(WPI * IPV == 4, "a code vector is four words");

    // ---- the query's table to LDS (rows padded with zeros to 256 entries), all values requested before the first store
    const float* Sq = a.S + (size_t)q * M * b;
    {
        constexpr int kPer = (M * kLutStride + NT - 1) / NT;
        float tv[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = tid + i * NT, k = e / kLutStride, j = e % kLutStride;
            tv[i] = (e < M * kLutStride && j < b) ? Sq[k * b + j] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i)
            if (tid + i * NT < M * kLutStride) lut[tid + i * NT] = tv[i];
    }
    small_select_clear<NT>(sel, tid);
    __syncthreads();

    // ---- Eq. 5 for every candidate this thread holds
    float sc[R];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float part[IPV];
        score_vector<M, 1>(lut, w[u], part);
#pragma unroll
        for (int e = 0; e < IPV; ++e) {
            const int s = u * IPV + e;
            sc[s] = first + (uint32_t)s * stride < n ? part[e] : empty_score();
        }
    }

    // ---- the workgroup's K best, ranked, straight to the workspace
    uint64_t* const mine_out = a.ws_keys + ((size_t)q * nblk + blk) * K;
    select_small_k<NT, R>(sc, [&](int slot) -> uint32_t { return item[slot]; }, K, sel, tid,
                          [&](int rank, uint64_t key) { mine_out[rank] = key; });
}
