// Eq. 4: the sub-id score matrix S (pq_subitem_scores).
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------------------------
// Eq. 4.  One thread per (split, sub-id) and a tile of queries: the thread keeps its sub-item embedding in
// registers and, per query, runs the left-to-right chain of fused multiply-adds over the d/m elements from +0.
constexpr int kSubThreads = 64;
constexpr int kSubQueryTile = 16;

// STAMP: measurement instance that also records wall-clock stamps (entry and end) per workgroup in `stamps`.
// COAL (the host: S_ELEMS a multiple of 4, 64 | m * b, centroids 16-byte aligned): the wave's 64 sub-item embeddings are
// one contiguous block of memory, which the lanes read piece after piece (a load instruction covers 1 KB of whole
// cache lines) and hand to their owners through LDS (rows padded by 16 bytes: conflict-free both ways).  Read row by
// row instead, every load instruction touches 64 lines for 16 bytes each, and the sixteen of them keep the L1's tag
// lookup busy for a good part of this kernel's microsecond.
template <int S_ELEMS, bool STAMP = false, bool COAL = false>   // S_ELEMS: d/m when it is one of the unrolled sizes, else 0 (runtime loop)
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
        if constexpr (COAL) {
            constexpr int PPR = S_ELEMS / 4;                       // 16-byte pieces per row
            constexpr int kRow = S_ELEMS + 4;                      // floats from one row to the next in LDS
            __shared__ __align__(16) float rows[kSubThreads * kRow];
            const float4* blk4 = reinterpret_cast<const float4*>(centroids + (size_t)blockIdx.x * kSubThreads * S_ELEMS);
            float4 v[PPR];
#pragma unroll
            for (int i = 0; i < PPR; ++i) v[i] = blk4[threadIdx.x + i * kSubThreads];
#pragma unroll
            for (int i = 0; i < PPR; ++i) {
                const int piece = threadIdx.x + i * kSubThreads;
                *reinterpret_cast<float4*>(&rows[(piece / PPR) * kRow + 4 * (piece % PPR)]) = v[i];
            }
            __syncthreads();                                       // (a workgroup is one wave)
#pragma unroll
            for (int t = 0; t < PPR; ++t) {
                const float4 x = *reinterpret_cast<const float4*>(&rows[threadIdx.x * kRow + 4 * t]);
                w[4 * t] = x.x; w[4 * t + 1] = x.y; w[4 * t + 2] = x.z; w[4 * t + 3] = x.w;
            }
        } else if ((S_ELEMS % 4) == 0 && (((uintptr_t)psi) & 15) == 0) {
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

// Eq. 4 on the matrix cores, for batches.  Per split, S_k = Phi_k Psi_k^T is a [B x d/m] x [d/m x b] product, and
// the fp32 matrix instruction with an inner dimension of ONE (v_mfma_f32_32x32x1_2b_f32: two independent 32 x 32
// outer products per issue) adds exactly one product to every accumulator, as a fused multiply-add with one
// rounding: a chain of d/m such instructions over t = 0, 1, ... is the same left-to-right chain from +0 as the
// scalar kernels run, bit for bit, denormals included (checked against the CPU's fmaf chain).  The instructions with a
// deeper inner dimension sum several products per issue in an order of their own and are not used.
// A workgroup of four waves owns 64 sub-ids of one split and 128 queries, a wave 32 of the queries: lanes l and
// l + 32 supply query (l % 32)'s chunk, lane l supplies sub-item embedding j0 + l, and block 0 / block 1 of the
// instruction are sub-ids j0 .. j0 + 31 / j0 + 32 .. j0 + 63.  Accumulator register v of lane l is query
// 8 * ((v % 16) / 4) + 4 * (l / 32) + v % 4 and sub-id j0 + 32 * (v / 16) + l % 32.
// Both operands are rows of 64 floats that a lane needs whole, one row per lane: read straight from memory that is one
// cache line per lane and load.  So the workgroup copies its tiles (the 64 sub-item embeddings: 16 KB of consecutive
// memory; each wave's 32 query chunks) to LDS with consecutive lanes on consecutive 16 bytes, rows padded to 68 floats
// (a lane's row then starts four banks after its neighbour's), and lanes read their rows from there.
// grid = (m * ceil(b / 64), ceil(B / 128)).  Rows of queries and centroids must be 16-byte aligned and d/m a multiple
// of 16; chunks of CH elements are staged at a time.  Query q's row of S starts at S + q * ldS (ldS = m * b for Eq. 4).
// The default scoring r = W phi of Section 2 (Eq. 3) is the same product with one split and the items in the place of
// the sub-ids (m = 1, b = |I|, centroids = W): pq_default_scores() runs this kernel for batches.
typedef float floatx32 __attribute__((ext_vector_type(32)));
constexpr int kSubMfmaThreads = 256;
constexpr int kSubMfmaQueries = 32 * (kSubMfmaThreads / kWave);   // queries per workgroup
constexpr int kSubMfmaPad = 4;                                    // floats added to a staged row

template <int CH>   // elements staged at a time: 16, 32 or 64
__global__ __launch_bounds__(kSubMfmaThreads) void subitem_scores_mfma_kernel(const float* __restrict__ queries,
                                                                            const float* __restrict__ centroids,
                                                                            float* __restrict__ S, int B, int d, int m, int b,
                                                                            long long ldS) {
    constexpr int ROW = CH + kSubMfmaPad, NW = kSubMfmaThreads / kWave, C4 = CH / 4;   // C4: 16-byte pieces of a staged row
    __shared__ __align__(16) float psi[64 * ROW];
    __shared__ __align__(16) float phi[NW][32 * ROW];
    const int s = d / m;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int jtiles = (b + 63) / 64;
    const int k = blockIdx.x / jtiles, j0 = (blockIdx.x % jtiles) * 64;
    const int q0 = blockIdx.y * kSubMfmaQueries + wave * 32;
    const bool active = q0 < B;                                // (a wave past the batch only helps staging the embeddings)
    floatx32 acc;
#pragma unroll
    for (int v = 0; v < 32; ++v) acc[v] = 0.0f;
    // (Issuing the next chunk's loads before this chunk's matrix instructions, through registers, was measured and is
    // slower: the extra registers cost more than the overlap gains; two or three workgroups per CU overlap instead.)
    for (int c = 0; c < s; c += CH) {
        if (c != 0) __syncthreads();                           // the previous chunk has been read
        // sub-item embeddings j0 .. j0 + 63, elements c .. c + CH - 1 (rows past b repeat the last one)
#pragma unroll
        for (int p = tid; p < 64 * C4; p += kSubMfmaThreads) {
            const int row = p / C4, piece = p % C4, j = min(j0 + row, b - 1);
            const float4 x = reinterpret_cast<const float4*>(centroids + ((size_t)k * b + j) * s + c)[piece];
            *reinterpret_cast<float4*>(&psi[row * ROW + 4 * piece]) = x;
        }
        // this wave's 32 query chunks
#pragma unroll
        for (int p = lane; active && p < 32 * C4; p += kWave) {
            const int row = p / C4, piece = p % C4, q = min(q0 + row, B - 1);
            const float4 x = reinterpret_cast<const float4*>(queries + (size_t)q * d + (size_t)k * s + c)[piece];
            *reinterpret_cast<float4*>(&phi[wave][row * ROW + 4 * piece]) = x;
        }
        __syncthreads();
        if (!active) continue;
        float av[CH], bv[CH];
#pragma unroll
        for (int i = 0; i < C4; ++i) {
            const float4 x = *reinterpret_cast<const float4*>(&phi[wave][(lane & 31) * ROW + 4 * i]);
            const float4 y = *reinterpret_cast<const float4*>(&psi[lane * ROW + 4 * i]);
            av[4 * i] = x.x; av[4 * i + 1] = x.y; av[4 * i + 2] = x.z; av[4 * i + 3] = x.w;
            bv[4 * i] = y.x; bv[4 * i + 1] = y.y; bv[4 * i + 2] = y.z; bv[4 * i + 3] = y.w;
        }
#pragma unroll
        for (int t = 0; t < CH; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x1f32(av[t], bv[t], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 32; ++v) {
        const int qq = q0 + 8 * ((v % 16) / 4) + 4 * (lane / 32) + v % 4, jj = j0 + 32 * (v / 16) + (lane & 31);
        if (qq < B && jj < b) S[(size_t)qq * ldS + (size_t)k * b + jj] = acc[v];
    }
}
