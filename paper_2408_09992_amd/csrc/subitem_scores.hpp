// Eq. 4: the sub-id score matrix S (pq_subitem_scores).
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------------------------
// Eq. 4.  One thread per (split, sub-id) and a tile of queries: the thread keeps its sub-item embedding in
// registers and, per query, runs the left-to-right chain of fused multiply-adds over the d/m elements from +0.
constexpr int kSubThreads = 64;
constexpr int kSubQueryTile = 16;

// STAMP: measurement instance that also records wall-clock stamps (entry and end) per workgroup in `stamps`.
template <int S_ELEMS, bool STAMP = false>   // S_ELEMS: d/m when it is one of the unrolled sizes, else 0 (runtime loop)
__global__ __launch_bounds__(kSubThreads) void subitem_scores_kernel(const float* __restrict__ queries,
                                                                     const float* __restrict__ centroids,
                                                                     float* __restrict__ S, int B, int d, int m, int b,
                                                                     uint64_t* stamps = nullptr) {
    const int s = S_ELEMS ? S_ELEMS : d / m;
    uint64_t* const rec = STAMP ? stamps + ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, threadIdx.x);
    const int kj = blockIdx.x * kSubThreads + threadIdx.x;       // k * b + j
    const int q0 = blockIdx.y * kSubQueryTile;
    if (kj >= m * b) return;
    const int k = kj / b;
    const float* psi = centroids + (size_t)kj * s;
    int q1 = q0 + kSubQueryTile;
    if (q1 > B) q1 = B;
    if (S_ELEMS) {
        float w[S_ELEMS ? S_ELEMS : 1];
        if ((S_ELEMS % 4) == 0 && (((uintptr_t)psi) & 15) == 0) {
            const float4* p4 = reinterpret_cast<const float4*>(psi);
#pragma unroll
            for (int t = 0; t < S_ELEMS / 4; ++t) {
                float4 v = p4[t];
                w[4 * t] = v.x; w[4 * t + 1] = v.y; w[4 * t + 2] = v.z; w[4 * t + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int t = 0; t < S_ELEMS; ++t) w[t] = psi[t];
        }
        for (int q = q0; q < q1; ++q) {
            const float* phi = queries + (size_t)q * d + (size_t)k * S_ELEMS;
            float acc = 0.0f;
#pragma unroll
            for (int t = 0; t < S_ELEMS; ++t) acc = __builtin_fmaf(w[t], phi[t], acc);
            S[(size_t)q * m * b + kj] = acc;
        }
        stamp<STAMP>(rec, kStampEnd, threadIdx.x);
    } else {
        for (int q = q0; q < q1; ++q) {
            const float* phi = queries + (size_t)q * d + (size_t)k * s;
            float acc = 0.0f;
            for (int t = 0; t < s; ++t) acc = __builtin_fmaf(psi[t], phi[t], acc);
            S[(size_t)q * m * b + kj] = acc;
        }
    }
}

// Eq. 4 for batches.  A workgroup (one wave) serves 64 sub-ids of ONE split and a tile of queries, so the query
// chunk it multiplies with is the same for all its lanes (read through the scalar cache), and it runs the chains of
// kSubInterleave queries side by side: the chains are independent, which hides the latency of each chain's
// dependent multiply-adds.  Per query the arithmetic is the same left-to-right chain from +0 as above.
constexpr int kSubInterleave = 8;     // queries whose chains run interleaved
constexpr int kSubBatchTile = 8;      // queries per workgroup

template <int S_ELEMS>   // d/m (a multiple of 4) when it is one of the unrolled sizes, else 0: d/m (a multiple of 4) at run time
__global__ __launch_bounds__(kSubThreads) void subitem_scores_batched_kernel(const float* __restrict__ queries,
                                                                             const float* __restrict__ centroids,
                                                                             float* __restrict__ S, int B, int d, int m, int b) {
    const int s = S_ELEMS ? S_ELEMS : d / m;
    const int jblocks = (b + kSubThreads - 1) / kSubThreads;
    const int k = blockIdx.x / jblocks;                              // the same for the whole workgroup
    const int j = (blockIdx.x % jblocks) * kSubThreads + threadIdx.x;
    const bool live = j < b;
    const int kj = k * b + (live ? j : 0);
    const float4* psi4 = reinterpret_cast<const float4*>(centroids + (size_t)kj * s);
    const int q0 = blockIdx.y * kSubBatchTile;
    int q1 = q0 + kSubBatchTile;
    if (q1 > B) q1 = B;
    for (int q = q0; q < q1; q += kSubInterleave) {
        const float4* phi4[kSubInterleave];
        float acc[kSubInterleave];
#pragma unroll
        for (int i = 0; i < kSubInterleave; ++i) {
            const int qi = (q + i < q1) ? q + i : q1 - 1;            // past the tile: a repeat, computed and not stored
            phi4[i] = reinterpret_cast<const float4*>(queries + (size_t)qi * d + (size_t)k * s);
            acc[i] = 0.0f;
        }
#pragma unroll 4
        for (int t4 = 0; t4 < s / 4; ++t4) {                         // four elements of every chain per step
            const float4 wv = psi4[t4];
#pragma unroll
            for (int i = 0; i < kSubInterleave; ++i) {
                const float4 pv = phi4[i][t4];
                acc[i] = __builtin_fmaf(wv.x, pv.x, acc[i]);
                acc[i] = __builtin_fmaf(wv.y, pv.y, acc[i]);
                acc[i] = __builtin_fmaf(wv.z, pv.z, acc[i]);
                acc[i] = __builtin_fmaf(wv.w, pv.w, acc[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < kSubInterleave; ++i)
            if (live && q + i < q1) S[(size_t)(q + i) * m * b + kj] = acc[i];
    }
}
