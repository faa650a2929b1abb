// PQTopK scoring for gfx950 (MI355X): kernels and the C ABI declared in include/pqtopk.h.
//
// Path (paper Section 3): pq_subitem_scores() builds the sub-id score matrix S (Eq. 4); pq_score_topk() streams the
// codebook G once, turns every item's m sub-ids into a score by m table lookups in LDS (Eq. 5), and keeps only the
// K best <id, score> pairs (Algorithm 1, V = I).  Item scores never reach memory.
//
// Total order used everywhere: a 64-bit key  (orderable(score) << 32) | ~id.  A larger key is a better item:
// higher score first, lower id between equal scores.  Keys of distinct items are distinct, key 0 means "empty".
//
// Shape of pq_score_topk(): one scan launch, then a small fold launch.
//   scan_topk_kernel<M, C, NT> (one query per workgroup; grid = (item blocks, B)):
//     1. requests its query's table values and its first rounds of codes, then fills the m x b table into LDS
//        (C copies of it for long scans, so that lanes with different copies never collide on an LDS bank);
//     2. scores a first round of items into registers and derives a floor that at least K of them reach (per wave
//        by bisection with ballots for K <= 64; from a 1024-bucket histogram over the workgroup for larger K):
//        everything below it is out for good;
//     3. streams the rest of its share of G against the floor; code loads are branch-free and counted, so the next
//        round's loads stay in flight; waves take their work units from a counter in LDS; survivors (a handful)
//        go to small per-wave lists in LDS that are pruned exactly (by key) when they fill, which raises the floor;
//     4. selects its exact K best and writes them, sorted, to the workspace.
//   scan_topk_tiled_kernel<M> (m = 8 or 16, B >= 2; a tile of four queries per workgroup, tables interleaved as
//     float4 so one 16-byte LDS read serves the four queries and sub-id extraction is shared): same steps, plus
//     workgroup checkpoints at geometrically spaced rounds that merge the waves' lists and raise all floors.
//   fold_topk_kernel (one workgroup per query) reduces the workgroups' lists to the final sorted K.
// Floors and histograms only ever prune; every decision that picks a winner compares full keys, so the result is
// exact for any input, including heavy ties (which merely take slower paths).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "pqtopk.h"

namespace {

constexpr int kWave = 64;
constexpr int kThreads = 512;                     // scan workgroup: 8 waves
constexpr int kWaves = kThreads / kWave;
constexpr int kBigThreads = 1024;                 // workgroup of the long single-query scan with replicated tables
constexpr int kMaxWaves = kBigThreads / kWave;
constexpr int kLutStride = 256;                   // table entries per split in LDS (a uint8 sub-id never runs past it)
constexpr int kBins = 1024;                       // score buckets of the pruning histogram
// 16-byte code vectors a thread holds per round: 4 for m >= 8, fewer for small m so a thread never holds > 16 items
// Units of work a thread holds per round in the kernels with a compile-time m.  m <= 16: a unit is one 16-byte code
// vector (16/m items); m = 32, 64: a unit is one item (m/16 vectors).  Four vectors per thread from m = 8 on.
__host__ __device__ constexpr int vec_per_thread(int m) { return m == 64 ? 1 : (m == 32 ? 2 : (m >= 8 ? 4 : (m == 4 ? 2 : 1))); }
constexpr int kGenericItemsPerThread = 4;         // items a thread holds per round when m is not 1,2,4,8,16
constexpr int kRing = 2;                          // rounds of codes a thread has loaded or in flight
constexpr int kFoldRegs = 12;                     // keys per thread the fold keeps in registers (6144 per query)
constexpr int kChunkKeys = 2048;                  // keys the grid-level fold takes per pass (4 per thread)
constexpr size_t kMaxLdsBytes = 160 * 1024;       // LDS per workgroup on gfx950
constexpr int kAssumedCUs = 256;                  // MI355X; only used to size grids and the workspace
constexpr int kBlocksPerCU = 2;                   // single-query scan workgroups per CU over the whole grid
constexpr int kTableCopies = 16;                  // copies of the score tables in the long single-query scan
constexpr int kTableCopiesMinRounds = 8;          // rounds per workgroup from which the copies pay for themselves

__device__ __forceinline__ uint32_t orderable_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float score_of_key(uint64_t key) {
    uint32_t u = (uint32_t)(key >> 32);
    u ^= (u >> 31) ? 0x80000000u : 0xFFFFFFFFu;
    return __uint_as_float(u);
}
__device__ __forceinline__ int id_of_key(uint64_t key) { return (int)(~(uint32_t)key); }
__device__ __forceinline__ uint64_t make_key(float score, uint32_t id) {
    return ((uint64_t)orderable_bits(score) << 32) | (uint32_t)(~id);
}

// Ordering point between LDS accesses of the lanes of ONE wave (LDS serves a wave's requests in issue order).
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Cross-lane steps through the DPP data path (no LDS traffic).  Lanes whose source lies outside their row of 16
// keep `identity`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_f32(float identity, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t identity, uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xF, false);
}
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;
constexpr int kDppRowShr = 0x110;        // + n
constexpr int kDppBcast15 = 0x142;
constexpr int kDppBcast31 = 0x143;

// min and max over the wave, returned in every lane
__device__ __forceinline__ void wave_minmax(float& mn, float& mx) {
    mn = fminf(mn, dpp_f32<kDppQuadSwap1>(mn, mn));       mx = fmaxf(mx, dpp_f32<kDppQuadSwap1>(mx, mx));
    mn = fminf(mn, dpp_f32<kDppQuadSwap2>(mn, mn));       mx = fmaxf(mx, dpp_f32<kDppQuadSwap2>(mx, mx));
    mn = fminf(mn, dpp_f32<kDppRowHalfMirror>(mn, mn));   mx = fmaxf(mx, dpp_f32<kDppRowHalfMirror>(mx, mx));
    mn = fminf(mn, dpp_f32<kDppRowMirror>(mn, mn));       mx = fmaxf(mx, dpp_f32<kDppRowMirror>(mx, mx));
    // every row of 16 lanes now holds its own extremes; combine the four rows through scalar reads
    float m0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mn), 0));
    float m1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mn), 16));
    float m2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mn), 32));
    float m3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mn), 48));
    float x0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 0));
    float x1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 16));
    float x2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 32));
    float x3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mx), 48));
    mn = fminf(fminf(m0, m1), fminf(m2, m3));
    mx = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
}

// A floor for a wave's top K (K in 1..64): a value that at least K of the lanes' values v reach, found by bisection
// between the wave's extremes with one ballot per step (so close below the K-th largest, not exactly it).  Lanes
// with nothing to offer pass -inf; if fewer than K lanes have a value the floor is -inf.  Same result in every lane.
__device__ __forceinline__ float wave_floor_for_k(float v, int K) {
    const float ninf = -__builtin_inff();
    if (__popcll(__ballot(v > ninf)) < K) return ninf;
    float lo = v > ninf ? v : __builtin_inff(), hi = v;
    wave_minmax(lo, hi);                                      // at least K lanes reach lo
#pragma unroll
    for (int step = 0; step < 12; ++step) {
        const float mid = lo + (hi - lo) * 0.5f;
        if (__popcll(__ballot(v >= mid)) >= K) lo = mid; else hi = mid;
    }
    return lo;
}

// inclusive prefix sum over the lanes of the wave (lane i gets v[0] + .. + v[i])
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t v) {
    v += dpp_u32<kDppRowShr + 1>(0u, v);
    v += dpp_u32<kDppRowShr + 2>(0u, v);
    v += dpp_u32<kDppRowShr + 4>(0u, v);
    v += dpp_u32<kDppRowShr + 8>(0u, v);
    v += dpp_u32<kDppBcast15, 0xA>(0u, v);               // lane 15 -> lanes 16..31, lane 47 -> lanes 48..63
    v += dpp_u32<kDppBcast31, 0xC>(0u, v);               // lane 31 -> lanes 32..63
    return v;
}

// Bitonic sort of n (a power of two) keys in LDS, descending.  BLOCK: all threads of the workgroup take part and
// stages are separated by workgroup barriers; otherwise one wave sorts its own array.
template <bool BLOCK>
__device__ void bitonic_sort_desc(uint64_t* a, int n, int tid, int nthr) {
    for (int k = 2; k <= n; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < (n >> 1); t += nthr) {
                int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int p = i | j;
                bool desc = (i & k) == 0;
                uint64_t x = a[i], y = a[p];
                if ((x < y) == desc) { a[i] = y; a[p] = x; }
            }
            if (BLOCK) __syncthreads(); else wave_sync();
        }
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Eq. 4.  One thread per (split, sub-id) and a tile of queries: the thread keeps its sub-item embedding in
// registers and, per query, runs the left-to-right chain of fused multiply-adds over the d/m elements from +0.
constexpr int kSubThreads = 64;
constexpr int kSubQueryTile = 16;

template <int S_ELEMS>   // d/m when it is one of the unrolled sizes, else 0 (runtime loop)
__global__ __launch_bounds__(kSubThreads) void subitem_scores_kernel(const float* __restrict__ queries,
                                                                     const float* __restrict__ centroids,
                                                                     float* __restrict__ S, int B, int d, int m, int b) {
    const int s = S_ELEMS ? S_ELEMS : d / m;
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

template <int S_ELEMS>   // d/m, a multiple of 4
__global__ __launch_bounds__(kSubThreads) void subitem_scores_batched_kernel(const float* __restrict__ queries,
                                                                             const float* __restrict__ centroids,
                                                                             float* __restrict__ S, int B, int d, int m, int b) {
    const int jblocks = (b + kSubThreads - 1) / kSubThreads;
    const int k = blockIdx.x / jblocks;                              // the same for the whole workgroup
    const int j = (blockIdx.x % jblocks) * kSubThreads + threadIdx.x;
    const bool live = j < b;
    const int kj = k * b + (live ? j : 0);
    const float4* psi4 = reinterpret_cast<const float4*>(centroids + (size_t)kj * S_ELEMS);
    const int q0 = blockIdx.y * kSubBatchTile;
    int q1 = q0 + kSubBatchTile;
    if (q1 > B) q1 = B;
    for (int q = q0; q < q1; q += kSubInterleave) {
        const float4* phi4[kSubInterleave];
        float acc[kSubInterleave];
#pragma unroll
        for (int i = 0; i < kSubInterleave; ++i) {
            const int qi = (q + i < q1) ? q + i : q1 - 1;            // past the tile: a repeat, computed and not stored
            phi4[i] = reinterpret_cast<const float4*>(queries + (size_t)qi * d + (size_t)k * S_ELEMS);
            acc[i] = 0.0f;
        }
#pragma unroll 4
        for (int t4 = 0; t4 < S_ELEMS / 4; ++t4) {                   // four elements of every chain per step
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

// ---------------------------------------------------------------------------------------------------------------
// Small per-workgroup control block in LDS.
struct Ctl {
    float lo;            // lower end of the score range the histogram covers
    float scale;         // buckets per unit of score (0: range degenerate, histogram off)
    float cut;           // scores <= cut cannot reach this workgroup's top K (valid after a histogram pass)
    int bstar;           // bucket of the K-th best in the histogrammed set
    int ncand;           // candidates collected for an exact selection
    int keep;            // batched kernel: keys currently held in the workgroup's best[] array of this query
    int next_unit;       // single-query kernel: next unit of work to hand to a wave
    int wave_cnt[kMaxWaves];
    float wave_min[kMaxWaves];
    float wave_max[kMaxWaves];
};

template <int BINS = kBins>
__device__ __forceinline__ int bucket_of(float score, float lo, float scale) {
    // monotone non-decreasing in score: subtract, multiply by a non-negative, truncate (negative and NaN give 0)
    float x = (score - lo) * scale;
    int bkt = (x > 0.0f) ? (int)x : 0;
    return bkt > BINS - 1 ? BINS - 1 : bkt;
}

// Range of the scores held by the workgroup -> bucket mapping.  Every thread passes the min / max of its own valid
// scores (+inf / -inf if it has none).  One barrier; lo / scale come back in registers and in ctl.
template <int NW = kWaves>
__device__ __forceinline__ void set_range(float mn, float mx, Ctl* ctl, int tid, float& lo_out, float& scale_out) {
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    wave_minmax(mn, mx);
    if (lane == 0) { ctl->wave_min[wave] = mn; ctl->wave_max[wave] = mx; }
    __syncthreads();
    float lo = ctl->wave_min[0], hi = ctl->wave_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) { lo = fminf(lo, ctl->wave_min[w]); hi = fmaxf(hi, ctl->wave_max[w]); }
    float range = hi - lo;
    float scale = (range > 0.0f) ? (float)kBins / range : 0.0f;
    if (!(scale > 0.0f) || scale > 3.0e38f) scale = 0.0f;
    if (tid == 0) {                                          // read by find_cut / block_select after a later barrier
        ctl->lo = lo;
        ctl->scale = scale;
        ctl->cut = -__builtin_inff();
        ctl->bstar = 0;
        ctl->ncand = 0;
    }
    lo_out = lo;
    scale_out = scale;
}

// One wave: find the highest bucket b* such that buckets >= b* hold at least K entries (0 if there are fewer than K
// in all), and a score cut that every entry of a bucket >= b* exceeds.  hist has BINS counters (a multiple of 256).
template <int BINS = kBins>
__device__ void find_cut(const uint32_t* hist, int K, Ctl* ctl, int lane) {
    constexpr int per = BINS / kWave;                        // buckets per lane; lane 0 owns the TOP ones
    const int first = BINS - per * (lane + 1);               // this lane's lowest bucket
    uint32_t c[per];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < per; i += 4) {
        uint4 v = *reinterpret_cast<const uint4*>(hist + first + i);
        c[i] = v.x; c[i + 1] = v.y; c[i + 2] = v.z; c[i + 3] = v.w;
        mine += v.x + v.y + v.z + v.w;
    }
    const uint32_t upto = wave_prefix_sum(mine);             // entries in this lane's buckets and all higher ones
    const uint64_t has = __ballot(upto >= (uint32_t)K);
    if (has != 0) {
        const int owner = __builtin_ctzll(has);              // lane with the highest buckets that reaches K
        if (lane == owner) {
            uint32_t above = upto - mine;
            int found = -1;
#pragma unroll
            for (int i = per - 1; i >= 0; --i) {
                above += c[i];
                if (found < 0 && above >= (uint32_t)K) found = i;
            }
            ctl->bstar = first + (found < 0 ? 0 : found);
        }
    } else if (lane == 0) {
        ctl->bstar = 0;
    }
    wave_sync();
    const int bstar = ctl->bstar;
    if (lane == 0) {
        // a score cut with bucket_of(cut) < b*: by monotonicity every entry of a bucket >= b* is > cut
        float cut = -__builtin_inff();
        if (bstar > 0 && ctl->scale > 0.0f) {
            float width = 1.0f / ctl->scale;
            cut = ctl->lo + ((float)bstar - 0.5f) * width;
            for (int guard = 0; guard < 64 && bucket_of<BINS>(cut, ctl->lo, ctl->scale) >= bstar; ++guard) cut -= width;
            if (bucket_of<BINS>(cut, ctl->lo, ctl->scale) >= bstar) cut = -__builtin_inff();
        }
        ctl->cut = cut;
    }
}

// Sort a wave's candidate list (cnt of cap slots used) in place, best first.  Returns the K-th best key, or 0 if
// the list holds fewer than K.  Out of line on purpose: it is rare and large.
__device__ __noinline__ uint64_t sort_wave_list(uint64_t* buf, int cap, int cnt, int K, int lane) {
    for (int t = cnt + lane; t < cap; t += kWave) buf[t] = 0;
    wave_sync();
    bitonic_sort_desc<false>(buf, cap, lane, kWave);
    return cnt >= K ? buf[K - 1] : 0ull;
}

// Smallest float above x (x finite or -inf; -inf stays -inf): `s >= next_up(x)` is `s > x`.
__device__ __forceinline__ float next_up(float x) {
    if (x == -__builtin_inff()) return x;
    if (x == 0.0f) return __uint_as_float(1u);
    uint32_t u = __float_as_uint(x);
    return __uint_as_float(x > 0.0f ? u + 1u : u - 1u);
}

// Per-wave candidate list in LDS.  A batch of at most one key per lane is appended by ballot compaction (no LDS
// round trip: positions come from the ballot mask).  When the list passes `prune_at` it is cut back to its K best
// and the wave's private score floor rises; when it would overflow it is sorted and pruned first.  Everything a
// wave drops is beaten by K keys it still holds.
struct WaveTopK {
    uint64_t* buf;       // cap keys
    int cap;             // power of two, >= K + 64
    int K;
    int prune_at;        // list length that triggers a tightening (0: only when full)
    int cnt;             // keys in the list (wave-uniform)
    uint64_t thr;        // K-th best key of the list once known, else 0
    float floor_ge;      // a score must be >= this to be worth appending

    // lanes in `mask` (non-empty, = ballot(take)) append the key of (score, id)
    __device__ __forceinline__ void append(uint64_t mask, bool take, float score, uint32_t id, int lane) {
        const uint64_t key = make_key(score + 0.0f, id);
        int n = __popcll(mask);
        if (cnt + n > cap) {                                  // rare: make room by sorting and keeping the K best
            const uint64_t kth = sort_wave_list(buf, cap, cnt, K, lane);
            if (cnt >= K) { cnt = K; thr = kth; floor_ge = fmaxf(floor_ge, score_of_key(thr)); }
            take = take && key > thr;
            mask = __ballot(take);
            if (mask == 0) return;
            n = __popcll(mask);
        }
        const int pos = cnt + __popcll(mask & ((1ull << lane) - 1ull));
        if (take) buf[pos] = key;
        cnt += n;
    }

    // cut the list back to its K best (sorted), raise thr and the floor
    __device__ void tighten(int lane) {
        wave_sync();
        if (cnt <= kWave) {                                   // one key per lane: rank by counting
            const uint64_t mine = lane < cnt ? buf[lane] : 0ull;
            const int cnt8 = (cnt + 7) & ~7;                  // cap >= 128 > cnt8; pad with zeros (a zero beats nothing)
            if (lane >= cnt && lane < cnt8) buf[lane] = 0ull;
            wave_sync();
            int rank = 0;
            for (int u = 0; u < cnt8; u += 8) {               // eight keys per trip keeps the LDS latency off the path
                const ulonglong2 p0 = *reinterpret_cast<const ulonglong2*>(buf + u);
                const ulonglong2 p1 = *reinterpret_cast<const ulonglong2*>(buf + u + 2);
                const ulonglong2 p2 = *reinterpret_cast<const ulonglong2*>(buf + u + 4);
                const ulonglong2 p3 = *reinterpret_cast<const ulonglong2*>(buf + u + 6);
                rank += (p0.x > mine) + (p0.y > mine) + (p1.x > mine) + (p1.y > mine) + (p2.x > mine) + (p2.y > mine) +
                        (p3.x > mine) + (p3.y > mine);
            }
            wave_sync();
            if (mine != 0ull && rank < K) buf[rank] = mine;
            wave_sync();
            if (cnt >= K) { cnt = K; thr = buf[K - 1]; }
        } else {
            const uint64_t kth = sort_wave_list(buf, cap, cnt, K, lane);
            if (cnt >= K) { cnt = K; thr = kth; }
        }
        if (thr != 0ull) floor_ge = fmaxf(floor_ge, score_of_key(thr));
    }
};

constexpr int kFastCand = 128;   // keys one wave can rank on its own (two per lane)
constexpr double kTiledMinLookups = 2.0e8;   // B * N * m from which the batched kernel takes over (measured crossover)
constexpr int kFilterMin = 64;   // single-query scan: final candidate sets larger than this are first cut by a floor

// One wave: sorted exact K best of the T <= MAXT keys in c[] (LDS; c has room for T rounded up to a multiple of 8,
// zeros allowed anywhere and ignored), written to dst[0..K) (LDS, zero where fewer than K exist).  More than 64 keys
// are first cut down to those that reach a floor at least K of them reach (about K keys, compacted in place); what
// is left is ranked by counting: the position of a key is the number of keys that beat it.  No workgroup barrier;
// every lane of the wave calls it.  wave_floor_for_k() must be declared above.
template <int MAXT = kFastCand>
__device__ __forceinline__ void wave_rank_select(uint64_t* c, int T, int K, uint64_t* dst, int lane) {
    constexpr int PER = MAXT / kWave;
    uint64_t mine[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) mine[j] = (lane + j * kWave < T) ? c[lane + j * kWave] : 0ull;
    for (int t = lane; t < K; t += kWave) dst[t] = 0ull;
    if (T > kWave && K <= kWave) {
        float best = -__builtin_inff();
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (mine[j] != 0ull) best = fmaxf(best, score_of_key(mine[j]));
        const float floor_ge = wave_floor_for_k(best, K);
        wave_sync();                                          // every lane holds its keys: c can be rewritten
        int kept = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const bool take = mine[j] != 0ull && score_of_key(mine[j]) >= floor_ge;
            const uint64_t mask = __ballot(take);
            if (take) c[kept + __popcll(mask & ((1ull << lane) - 1ull))] = mine[j];
            kept += __popcll(mask);
        }
        T = kept;
        wave_sync();
#pragma unroll
        for (int j = 0; j < PER; ++j) mine[j] = (lane + j * kWave < T) ? c[lane + j * kWave] : 0ull;
    }
    const int T8 = (T + 7) & ~7;
    wave_sync();                                              // (the pad below must not overtake the reads above)
    for (int t = T + lane; t < T8; t += kWave) c[t] = 0ull;
    wave_sync();
    int rank[PER];
#pragma unroll
    for (int j = 0; j < PER; ++j) rank[j] = 0;
    for (int u = 0; u < T8; u += 8) {
        const ulonglong2 p0 = *reinterpret_cast<const ulonglong2*>(c + u);
        const ulonglong2 p1 = *reinterpret_cast<const ulonglong2*>(c + u + 2);
        const ulonglong2 p2 = *reinterpret_cast<const ulonglong2*>(c + u + 4);
        const ulonglong2 p3 = *reinterpret_cast<const ulonglong2*>(c + u + 6);
#pragma unroll
        for (int j = 0; j < PER; ++j)
            if (j * kWave < T)
                rank[j] += (p0.x > mine[j]) + (p0.y > mine[j]) + (p1.x > mine[j]) + (p1.y > mine[j]) +
                           (p2.x > mine[j]) + (p2.y > mine[j]) + (p3.x > mine[j]) + (p3.y > mine[j]);
    }
#pragma unroll
    for (int j = 0; j < PER; ++j)
        if (mine[j] != 0ull && rank[j] < K) dst[rank[j]] = mine[j];
    wave_sync();
}

// Sorted exact K best of the C candidates in cand[] by counting: the position of a key is the number of candidates
// that beat it.  cand must have room for C rounded up to a multiple of 8 (the pad is zeroed here; a zero beats
// nothing).  dst[0..K) is zero-filled where fewer than K exist.  When the workgroup has four threads per candidate,
// four adjacent lanes share a key and each counts over a quarter of the candidates: the loop is bound by the latency
// of its LDS reads, so a shorter loop per thread is what makes it faster.
template <int NT = kThreads>
__device__ void rank_select(uint64_t* cand, int C, int K, uint64_t* dst, int tid) {
    const int C8 = (C + 7) & ~7;
    for (int i = tid; i < K; i += NT) dst[i] = 0;
    if (tid < C8 - C) cand[C + tid] = 0;
    __syncthreads();
    auto count8 = [&](int u, uint64_t mine) -> int {
        const ulonglong2 p0 = *reinterpret_cast<const ulonglong2*>(cand + u);
        const ulonglong2 p1 = *reinterpret_cast<const ulonglong2*>(cand + u + 2);
        const ulonglong2 p2 = *reinterpret_cast<const ulonglong2*>(cand + u + 4);
        const ulonglong2 p3 = *reinterpret_cast<const ulonglong2*>(cand + u + 6);
        return (p0.x > mine) + (p0.y > mine) + (p1.x > mine) + (p1.y > mine) + (p2.x > mine) + (p2.y > mine) +
               (p3.x > mine) + (p3.y > mine);
    };
    if (C8 * 4 <= NT) {
        const int t = tid >> 2, part = tid & 3;              // (C8 is a multiple of 8: a wave is all in or all out)
        if (t < C8) {
            const uint64_t mine = cand[t];
            uint32_t rank = 0;
#pragma unroll 2
            for (int u = part * 8; u < C8; u += 32) rank += (uint32_t)count8(u, mine);
            rank += dpp_u32<kDppQuadSwap1>(0u, rank);
            rank += dpp_u32<kDppQuadSwap2>(0u, rank);
            if (part == 0 && mine != 0ull && rank < (uint32_t)K) dst[rank] = mine;
        }
    } else {
        for (int t = tid; t < C; t += NT) {
            const uint64_t mine = cand[t];
            int rank = 0;
            for (int u = 0; u < C8; u += 8) rank += count8(u, mine);
            if (rank < K) dst[rank] = mine;
        }
    }
    __syncthreads();
}

// Exact selection of the K best among the nonzero keys of src[0..n) (LDS, zeros allowed anywhere), written sorted
// to dst[0..K) (zero-filled if fewer than K exist).  All NT threads of the workgroup call it, ctl->lo / scale / ncand = 0 set.
// `cand` holds candmax keys, `hist` kBins counters.  If the histogram cannot narrow the set to candmax keys (ties,
// degenerate range), src is sorted in place instead, which needs n to be a power of two.
template <int NT = kThreads>
__device__ void block_select(uint64_t* src, int n, int K, uint64_t* dst, uint64_t* cand, int candmax, uint32_t* hist,
                             Ctl* ctl, int tid) {
    const int lane = tid & (kWave - 1);
    for (int i = tid; i < kBins; i += NT) hist[i] = 0;
    if (tid == 0) ctl->ncand = 0;
    __syncthreads();
    const float lo = ctl->lo, scale = ctl->scale;
    for (int i = tid; i < n; i += NT) {
        uint64_t key = src[i];
        if (key) atomicAdd(&hist[bucket_of(score_of_key(key), lo, scale)], 1u);
    }
    __syncthreads();
    if (tid < kWave) find_cut(hist, K, ctl, lane);
    __syncthreads();
    const int bstar = ctl->bstar;
    for (int i = tid; i < n; i += NT) {
        uint64_t key = src[i];
        if (key && bucket_of(score_of_key(key), lo, scale) >= bstar) {
            int pos = atomicAdd(&ctl->ncand, 1);
            if (pos < candmax) cand[pos] = key;
        }
    }
    __syncthreads();
    const int C = ctl->ncand;
    if (C <= candmax) {
        rank_select<NT>(cand, C, K, dst, tid);
    } else {
        bitonic_sort_desc<true>(src, n, tid, NT);
        for (int i = tid; i < K; i += NT) dst[i] = src[i];
        __syncthreads();
    }
}

__host__ __device__ inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

// LDS layout of the scan kernel (dynamic): lut | hist | ctl | wave lists | cand | sorted
struct ScanLds {
    float* lut;
    uint32_t* hist;
    Ctl* ctl;
    uint64_t* lists;     // waves * cap
    uint64_t* cand;      // candmax
    uint64_t* sorted;    // K
};

__host__ __device__ inline size_t scan_lds_bytes(size_t lut_floats, int cap, int candmax, int K, int waves = kWaves) {
    return align16(lut_floats * sizeof(float)) + kBins * sizeof(uint32_t) + align16(sizeof(Ctl)) +
           (size_t)waves * cap * sizeof(uint64_t) + (size_t)candmax * sizeof(uint64_t) +
           align16((size_t)K * sizeof(uint64_t));
}

__device__ inline ScanLds carve_scan(unsigned char* smem, size_t lut_floats, int cap, int candmax, int waves = kWaves) {
    ScanLds L;
    size_t off = 0;
    L.lut = reinterpret_cast<float*>(smem + off);        off += align16(lut_floats * sizeof(float));
    L.hist = reinterpret_cast<uint32_t*>(smem + off);    off += kBins * sizeof(uint32_t);
    L.ctl = reinterpret_cast<Ctl*>(smem + off);          off += align16(sizeof(Ctl));
    L.lists = reinterpret_cast<uint64_t*>(smem + off);   off += (size_t)waves * cap * sizeof(uint64_t);
    L.cand = reinterpret_cast<uint64_t*>(smem + off);    off += (size_t)candmax * sizeof(uint64_t);
    L.sorted = reinterpret_cast<uint64_t*>(smem + off);
    return L;
}

struct ScanArgs {
    const uint8_t* codes;
    const float* S;
    long long N;
    int m, b, K;
    int cap;             // keys per wave list (power of two >= K + 64)
    int candmax;         // keys of the exact-selection candidate array
    int prune_at;        // wave list length that triggers a tightening (0: only when full)
    uint64_t* ws_keys;   // [B][nblk][K]
    const int* subset;   // candidate list V (generic kernel only): unit p stands for item subset[p]; nullptr: V = I
    uint32_t n_items;    // items in the catalogue (bounds the ids read from `subset`)
};

// The end of a single-query scan: the waves' lists -> the workgroup's exact K best, sorted, in L.sorted (zero where
// fewer than K exist).  Every thread of the workgroup calls it once its wave has offered everything.
template <int NT>
__device__ __forceinline__ void workgroup_select(const ScanLds& L, Ctl* ctl, WaveTopK& top, int K, int cap, int candmax,
                                                 int tid) {
    constexpr int NW = NT / kWave;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    if (lane == 0) {
        ctl->wave_cnt[wave] = top.cnt;
        ctl->wave_max[wave] = top.thr != 0ull ? score_of_key(top.thr) : -__builtin_inff();   // <= the wave's K-th best
    }
    if (tid == 0) ctl->ncand = 0;
    __syncthreads();
    // lane w of every wave holds wave w's count and floor: totals by cross-lane operations, one LDS round trip
    static_assert(NW <= kWave, "one lane per wave");
    const uint32_t cnt_w = lane < NW ? (uint32_t)ctl->wave_cnt[lane] : 0u;
    float fl_lo = lane < NW ? ctl->wave_max[lane] : -__builtin_inff(), wg_floor = fl_lo;
    const uint32_t upto = wave_prefix_sum(cnt_w);
    int total = __builtin_amdgcn_readlane((int)upto, kWave - 1);
    const int before = __builtin_amdgcn_readlane((int)(upto - cnt_w), wave);
    wave_minmax(fl_lo, wg_floor);
    if (total <= candmax) {
        if (total > kFilterMin) {
            // a long scan leaves every wave with its own K best and more: only keys that reach the best of the waves'
            // K-th scores can be among the workgroup's K best (that score is a lower bound of the workgroup's K-th)
            for (int t0 = 0; t0 < top.cnt; t0 += kWave) {
                const uint64_t key = t0 + lane < top.cnt ? top.buf[t0 + lane] : 0ull;
                const bool take = key != 0ull && score_of_key(key) >= wg_floor;
                const uint64_t mask = __ballot(take);
                int base = 0;
                if (lane == 0 && mask != 0) base = atomicAdd(&ctl->ncand, __popcll(mask));
                base = __builtin_amdgcn_readfirstlane(base);
                if (take) L.cand[base + __popcll(mask & ((1ull << lane) - 1ull))] = key;
            }
            __syncthreads();
            total = ctl->ncand;
        } else {
            for (int t = lane; t < top.cnt; t += kWave) L.cand[before + t] = top.buf[t];
        }
        rank_select<NT>(L.cand, total, K, L.sorted, tid);        // its first barrier orders the copies above
    } else {
        // too many keys for one ranking (long lists, large K): histogram over the listed keys' own range, or a sort
        float mn = __builtin_inff(), mx = -__builtin_inff();
        for (int t = lane; t < top.cnt; t += kWave) {
            const float v = score_of_key(top.buf[t]);
            mn = fminf(mn, v); mx = fmaxf(mx, v);
        }
        float lo, scale;
        set_range<NW>(mn, mx, ctl, tid, lo, scale);
        for (int t = top.cnt + lane; t < cap; t += kWave) top.buf[t] = 0;
        __syncthreads();
        block_select<NT>(L.lists, NW * cap, K, L.sorted, L.cand, candmax, L.hist, ctl, tid);
    }
}

// Items a thread holds per round.  M > 0: m is M and one 16-byte vector carries 16/M items; M == 0: any m, one item
// per slot, row loads sized by m's alignment.
template <int M>
struct Round {
    static constexpr int kUnitsPerThread = M ? vec_per_thread(M) : kGenericItemsPerThread;   // lane-sized units of work
    static constexpr int kVPU = M > 16 ? M / 16 : 1;                                     // 16-byte vectors per unit
    static constexpr int kIPV = (M && M <= 16) ? 16 / M : 1;                             // items per unit
    static constexpr int kVecs = M ? kUnitsPerThread * kVPU : 0;                         // 16-byte loads per round
    static constexpr int kItems = kUnitsPerThread * kIPV;
    static constexpr int kWords = M ? kVecs * 4 : 1;
};

// Eq. 5 for the 16/M items packed in one 16-byte vector (words w[0..3], little-endian): all 16 table reads are
// issued before any sum so they overlap in the LDS pipeline, then each item sums its m values left to right.
// A sum of -0 is left as it is here; it is turned into +0 where a key is made.
// With C > 1 the tables are replicated: entry e of the table array has C copies at words e * C .. e * C + C - 1 and
// `lut` already points at this lane's copy (lane % C), so lanes with different copies never share an LDS bank.
template <int M, int C = 1>
__device__ __forceinline__ void score_vector(const float* lut, const uint32_t* w, float* sc) {
    float v[16];
#pragma unroll
    for (int byte = 0; byte < 16; ++byte) {
        const uint32_t code = (w[byte >> 2] >> ((byte & 3) * 8)) & 0xFFu;
        v[byte] = lut[((byte % M) * kLutStride + code) * C];
    }
    __builtin_amdgcn_sched_barrier(0);                // keep the 16 reads ahead of the sums
#pragma unroll
    for (int e = 0; e < 16 / M; ++e) {
        float acc = v[e * M];
#pragma unroll
        for (int k = 1; k < M; ++k) acc = acc + v[e * M + k];
        sc[e] = acc;
    }
}

// Eq. 5 for one item of M = 32 or 64 sub-ids (M/16 vectors, words w[0 .. M/4)): one left-to-right chain over all M
// values; the 16 table reads of a vector are issued together.
template <int M>
__device__ __forceinline__ float score_wide(const float* lut, const uint32_t* w) {
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < M / 16; ++j) {
        float v[16];
#pragma unroll
        for (int byte = 0; byte < 16; ++byte) {
            const uint32_t code = (w[4 * j + (byte >> 2)] >> ((byte & 3) * 8)) & 0xFFu;
            v[byte] = lut[(j * 16 + byte) * kLutStride + code];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int byte = 0; byte < 16; ++byte) acc = (j == 0 && byte == 0) ? v[0] : acc + v[byte];
    }
    return acc;
}

__device__ float score_row(const float* lut, const uint8_t* row, int m) {
    float acc = 0.0f;
    if ((m & 15) == 0) {
        const uint4* p = reinterpret_cast<const uint4*>(row);
        for (int v = 0; v < (m >> 4); ++v) {
            uint4 x = p[v];
            uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                float t = lut[(v * 16 + k) * kLutStride + ((w[k >> 2] >> ((k & 3) * 8)) & 0xFFu)];
                acc = (v == 0 && k == 0) ? t : acc + t;
            }
        }
    } else if ((m & 3) == 0) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(row);
        for (int v = 0; v < (m >> 2); ++v) {
            uint32_t w = p[v];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float t = lut[(v * 4 + k) * kLutStride + ((w >> (k * 8)) & 0xFFu)];
                acc = (v == 0 && k == 0) ? t : acc + t;
            }
        }
    } else {
        acc = lut[row[0]];
        for (int k = 1; k < m; ++k) acc = acc + lut[k * kLutStride + row[k]];
    }
    return acc;
}

// Unit (code vector, or item in the generic kernel) that thread `tid` of workgroup `blk` owns in slot u of its
// round rr: ((rr * kUnits + u) * nblk + blk) * NT + tid.  Slot u of one round of all workgroups together is one
// contiguous stretch of the catalogue, so the grid sweeps memory front to back.  32-bit arithmetic: there are fewer
// than 2^31 units (N < 2^31, m <= 16 in the vector kernels) and the few rounds a kernel reaches past the end add
// less than 2^24 to that, so nothing wraps.
template <int M, int NT>
__device__ __forceinline__ uint32_t unit_of(uint32_t rr, int u, int nblk, int blk, int tid) {
    return ((rr * Round<M>::kUnitsPerThread + u) * (uint32_t)nblk + (uint32_t)blk) * NT + (uint32_t)tid;
}

// The code vectors this thread owns in round rr (vector kernels only).  Always the same number of plain 16-byte
// loads, with the vector index clamped to `last_vec` (the last vector that lies wholly inside the catalogue): no
// branch, so the compiler knows how many loads are outstanding at any point and lets several rounds stay in
// flight.  A clamped vector's items are masked out by the caller.
template <int M, int NT = kThreads>
__device__ __forceinline__ void load_round(const ScanArgs& a, uint32_t rr, int nblk, int blk, uint32_t last_vec,
                                           uint32_t spare_vec, int tid, uint32_t (&w)[Round<M>::kWords]) {
    if constexpr (M > 0) {
        const uint4* base = reinterpret_cast<const uint4*>(a.codes);
        constexpr int VPU = Round<M>::kVPU;
#pragma unroll
        for (int u = 0; u < Round<M>::kUnitsPerThread; ++u) {
            uint32_t v = unit_of<M, NT>(rr, u, nblk, blk, tid);
            v = v <= last_vec ? v : spare_vec;
#pragma unroll
            for (int j = 0; j < VPU; ++j) {
                const uint4 x = base[(size_t)v * VPU + j];
                const int o = 4 * (u * VPU + j);
                w[o] = x.x; w[o + 1] = x.y; w[o + 2] = x.z; w[o + 3] = x.w;
            }
        }
    }
}

// Scores of the items this thread owns in that round (slots past the catalogue's end get arbitrary finite values).
// `inside`: the round lies wholly inside the scanned units (n_units of them); otherwise vectors past the end are not
// looked up at all (a wave whose lanes are all past the end skips the vector's table reads).
template <int M, int C = 1, int NT = kThreads>
__device__ __forceinline__ void score_round(const ScanArgs& a, const float* lut, uint32_t rr, int nblk, int blk, int tid,
                                            bool inside, uint32_t n_units, const uint32_t (&w)[Round<M>::kWords],
                                            float (&sc)[Round<M>::kItems]) {
    if constexpr (M > 0) {
#pragma unroll
        for (int u = 0; u < Round<M>::kUnitsPerThread; ++u) {
            if (inside || unit_of<M, NT>(rr, u, nblk, blk, tid) < n_units) {
                if constexpr (M > 16) sc[u] = score_wide<M>(lut, &w[4 * Round<M>::kVPU * u]);
                else score_vector<M, C>(lut, &w[4 * u], &sc[u * Round<M>::kIPV]);
            } else {
#pragma unroll
                for (int e = 0; e < Round<M>::kIPV; ++e) sc[u * Round<M>::kIPV + e] = 0.0f;
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < kGenericItemsPerThread; ++u) {
            const uint32_t unit = unit_of<M, NT>(rr, u, nblk, blk, tid);
            float v = 0.0f;
            if (unit < n_units) {
                uint32_t item = unit;
                if (a.subset) {                                // an id past the catalogue is clamped: never out of bounds
                    item = (uint32_t)a.subset[unit];
                    item = item < a.n_items ? item : a.n_items - 1;
                }
                v = score_row(lut, a.codes + (size_t)item * a.m, a.m);
            }
            sc[u] = v;
        }
    }
}

// Id of the item in slot e of this thread's round (may lie past the scanned items in the last round).
template <int M, int NT = kThreads>
__device__ __forceinline__ uint32_t item_of_slot(uint32_t rr, int nblk, int blk, int tid, int e) {
    constexpr int IPV = Round<M>::kIPV;
    return unit_of<M, NT>(rr, e / IPV, nblk, blk, tid) * IPV + (e % IPV);
}

// Catalogue scan: grid = (item blocks, B).  Leaves each workgroup's exact, sorted K best keys in the workspace.
// LDS: the score tables are a static array when m is a template value (their address is then a compile-time
// constant, which lets sub-id extraction and address arithmetic fold into one instruction per lookup); the rest is
// dynamic: [tables if M == 0] | hist | ctl | wave lists | cand | sorted.
// C > 1 (long single-query scans): C copies of the tables, in dynamic LDS, cut the bank conflicts of the lookups.
template <int M, int C = 1, int NT = kThreads>
__global__ __launch_bounds__(NT, 4) void scan_topk_kernel(ScanArgs a) {
    constexpr int NW = NT / kWave;
    static_assert(C == 1 || M > 0, "replicated tables need a compile-time m");
    __shared__ __align__(16) float lut_static[(M && C == 1) ? M * kLutStride : 4];
    extern __shared__ __align__(16) unsigned char smem[];
    const int m = M ? M : a.m;
    const ScanLds L = carve_scan(smem, (M && C == 1) ? 0 : (size_t)m * kLutStride * C, a.cap, a.candmax, NW);
    float* const lut_base = (M && C == 1) ? lut_static : L.lut;
    Ctl* ctl = L.ctl;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x, K = a.K, b = a.b;
    constexpr int kItems = Round<M>::kItems;
    constexpr int kUnits = Round<M>::kUnitsPerThread;
    constexpr int kWords = Round<M>::kWords;

    // Vector kernels scan the code vectors that lie wholly inside the catalogue; the fewer than 16 / M items after
    // them (when N * M is not a multiple of 16) are scored one by one at the end.  The generic kernel scans items.
    const uint32_t total_units = (uint32_t)((M && M <= 16) ? (a.N * M) / 16 : a.N);
    const uint32_t n_scan = M ? total_units * Round<M>::kIPV : total_units;   // items the rounds cover
    const uint32_t last_vec = total_units - 1;                                // (total_units >= 1: the host sees to it)
    const uint32_t round_units = (uint32_t)NT * kUnits * nblk;                // units all workgroups take per round
    const uint32_t rounds = (total_units + round_units - 1) / round_units;    // every workgroup runs them all
    const uint32_t inside_rounds = total_units / round_units;                 // rounds with no ragged end

    // ---- 1. the first kRing rounds' codes on their way, then the query's table into LDS
    uint32_t r = 0;
    const int blk = blockIdx.x;
    uint32_t w[kRing][kWords];
    // (vt: the thread index whose share of round rr is meant; a wave may take over another wave's share)
    // (loads past the end go to a line of this wave's own instead of all to the last one: no single hot line when
    // thousands of waves reach the end of their scan together)
    const uint32_t own_vec = (uint32_t)(blk * NW + wave) * 4u;
    const uint32_t spare_vec = own_vec < last_vec ? own_vec : last_vec;
    auto fetch = [&](uint32_t rr, int vt, uint32_t (&buf)[kWords]) {
        load_round<M, NT>(a, rr, nblk, blk, last_vec, spare_vec, vt, buf);
    };
    // (the host sends catalogues with no whole code vector, N * M < 16, to the generic kernel: rounds >= 1 here)
    auto fetch_first = [&]() {                                // no branch: the loads can be counted, so what follows
#pragma unroll                                                // waits for exactly what it needs
        for (int i = 0; i < kRing; ++i) fetch(r + i, tid, w[i]);
    };
    const float* Sq = a.S + (size_t)q * m * b;
    if constexpr (C > 1) {
        // thread t writes the 16-byte pieces t, t + NT, ... of the replicated tables (piece p is a quarter of the C
        // copies of entry p / (C / 4)): consecutive lanes write consecutive LDS addresses.  Values requested first.
        constexpr int kPieces = M * kLutStride * (C / 4);
        constexpr int kPer = (kPieces + NT - 1) / NT;
        float tv[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = (tid + i * NT) / (C / 4), k = e / kLutStride, j = e % kLutStride;
            tv[i] = (e < M * kLutStride && j < b) ? Sq[k * b + j] : 0.0f;
        }
        fetch_first();
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int piece = tid + i * NT;
            if (piece < kPieces) reinterpret_cast<float4*>(lut_base)[piece] = make_float4(tv[i], tv[i], tv[i], tv[i]);
        }
    } else if (b == kLutStride && ((uintptr_t)Sq & 15) == 0) {
        // b = 256: the query's table is copied as it is, in 16-byte pieces, all requested before the first is stored
        const float4* src = reinterpret_cast<const float4*>(Sq);
        float4* dst = reinterpret_cast<float4*>(lut_base);
        if constexpr (M > 0) {
            constexpr int kPieces = M * kLutStride / 4;
            constexpr int kPer = (kPieces + NT - 1) / NT;
            float4 t4[kPer];
#pragma unroll
            for (int i = 0; i < kPer; ++i)
                t4[i] = (kPieces % NT == 0 || tid + i * NT < kPieces) ? src[tid + i * NT] : make_float4(0, 0, 0, 0);
            fetch_first();
#pragma unroll
            for (int i = 0; i < kPer; ++i)
                if (kPieces % NT == 0 || tid + i * NT < kPieces) dst[tid + i * NT] = t4[i];
        } else {
            fetch_first();
#pragma unroll 4
            for (int e = tid; e < m * (kLutStride / 4); e += NT) dst[e] = src[e];
        }
    } else {
        fetch_first();
        for (int e = tid; e < m * kLutStride; e += NT) {
            int k = e / kLutStride, j = e % kLutStride;
            lut_base[e] = (j < b) ? Sq[k * b + j] : 0.0f;
        }
    }
    for (int i = tid; i < kBins; i += NT) L.hist[i] = 0;
    if (tid == 0) ctl->next_unit = kRing * NW;
    __syncthreads();
    const float* const lut = lut_base + (C > 1 ? lane % C : 0);   // this lane's copy

    WaveTopK top{L.lists + (size_t)wave * a.cap, a.cap, K, a.prune_at, 0, 0ull, -__builtin_inff()};

    // item id of a scanned unit (they differ only under a candidate list)
    auto id_of = [&](uint32_t unit) -> uint32_t {
        if constexpr (M == 0) {
            if (a.subset) {
                const uint32_t item = (uint32_t)a.subset[unit];
                return item < a.n_items ? item : a.n_items - 1;
            }
        }
        return unit;
    };
    // what a round's scores offer to the wave's list: everything at or above its floor
    auto offer = [&](const float (&sc)[kItems], uint32_t rr, int vt) {
        float best = sc[0];
#pragma unroll
        for (int e = 1; e < kItems; ++e) best = fmaxf(best, sc[e]);
        if (__ballot(best >= top.floor_ge) == 0) return;      // nothing in this round can matter
        const bool inside = rr < inside_rounds;
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const uint32_t item = item_of_slot<M, NT>(rr, nblk, blk, vt, e);
            const bool take = sc[e] >= top.floor_ge && (inside || item < n_scan);
            const uint64_t mask = __ballot(take);
            if (mask != 0) top.append(mask, take, sc[e], take ? id_of(item) : 0u, lane);
        }
        if (top.prune_at != 0 && top.cnt >= top.prune_at) top.tighten(lane);
    };
    // one streamed round
    auto process = [&](const uint32_t (&w)[kWords], uint32_t rr, int vt) {
        float sc[kItems];
        score_round<M, C, NT>(a, lut, rr, nblk, blk, vt, rr < inside_rounds, total_units, w, sc);
        offer(sc, rr, vt);
    };

    {
        // ---- 2. first round: scores in registers, histogram over their range, cut
        float sc[kItems];
        score_round<M, C, NT>(a, lut, r, nblk, blk, tid, r < inside_rounds, total_units, w[0], sc);
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int e = 0; e < kItems; ++e)
            if (item_of_slot<M, NT>(r, nblk, blk, tid, e) < n_scan) { mn = fminf(mn, sc[e]); mx = fmaxf(mx, sc[e]); }
        float lo, scale;
        set_range<NW>(mn, mx, ctl, tid, lo, scale);
        int bk[kItems];
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            bk[e] = bucket_of(sc[e], lo, scale);
            if (item_of_slot<M, NT>(r, nblk, blk, tid, e) < n_scan) atomicAdd(&L.hist[bk[e]], 1u);
        }
        __syncthreads();
        if (tid < kWave) find_cut(L.hist, K, ctl, lane);
        __syncthreads();
        const int bstar = ctl->bstar;
        top.floor_ge = next_up(ctl->cut);                     // bucket >= b* implies score > cut
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const uint32_t item = item_of_slot<M, NT>(r, nblk, blk, tid, e);
            const bool take = item < n_scan && bk[e] >= bstar;
            const uint64_t mask = __ballot(take);
            if (mask != 0) top.append(mask, take, sc[e], take ? id_of(item) : 0u, lane);
        }
        if (top.prune_at != 0 && top.cnt >= top.prune_at) top.tighten(lane);
        r += 1;
    }

    // ---- 3. stream the remaining rounds against the wave's floor.  Work is handed out in units of one wave's share
    // of a round: unit j is the share of wave j % NW in round j / NW.  A wave's first kRing units are its own share
    // of the first kRing rounds (already loaded or on their way); after that it takes the next free unit from a
    // counter in LDS, so a wave that falls behind (LDS arbitration, candidate handling) does not hold the workgroup
    // up at the end.  The counter's atomic is issued one step before its result is used, and a unit's loads are
    // unconditional (past the last unit they are clamped re-reads whose data is never used): no wait in the loop
    // is longer than it has to be.
    if (rounds == 2) {
        process(w[1], 1, tid);                                // a short scan: the second round is already loaded
    } else if (rounds > 2) {
        const uint32_t units = rounds * NW;
        int pending = 0;                                      // lane 0: result of the last counter request
        auto request_unit = [&]() { if (lane == 0) pending = atomicAdd(&ctl->next_unit, 1); };
        auto requested_unit = [&]() -> uint32_t { return (uint32_t)__builtin_amdgcn_readfirstlane(pending); };
        uint32_t unit[kRing];                                 // unit held by w[i]
#pragma unroll
        for (int i = 1; i < kRing; ++i) unit[i] = (uint32_t)i * NW + wave;
        request_unit();
        unit[0] = requested_unit();
        request_unit();
        fetch(unit[0] / NW, (int)(unit[0] % NW) * kWave + lane, w[0]);
        while (unit[1 % kRing] < units) {                     // the oldest unit held; a younger one past the end scores nothing
#pragma unroll
            for (int i = 1; i <= kRing; ++i) {
                const int s = i % kRing;
                process(w[s], unit[s] / NW, (int)(unit[s] % NW) * kWave + lane);
                unit[s] = requested_unit();
                request_unit();
                fetch(unit[s] / NW, (int)(unit[s] % NW) * kWave + lane, w[s]);
            }
        }
    }
    if constexpr (M > 0 && M <= 16) {
        // the fewer than 16 / M items after the last whole code vector, one per lane of one wave
        if (blockIdx.x == 0 && wave == 0) {
            const uint32_t item = n_scan + lane;
            float sc = 0.0f;
            bool take = false;
            if (item < (uint32_t)a.N) {
                const uint8_t* row = a.codes + (size_t)item * M;
                sc = lut[(size_t)row[0] * C];
#pragma unroll
                for (int k = 1; k < M; ++k) sc = sc + lut[((size_t)k * kLutStride + row[k]) * C];
                take = sc >= top.floor_ge;
            }
            const uint64_t mask = __ballot(take);
            if (mask != 0) top.append(mask, take, sc, (uint32_t)item, lane);
        }
    }

    // ---- 4. workgroup selection: the waves' lists -> exact K best, sorted
    workgroup_select<NT>(L, ctl, top, K, a.cap, a.candmax, tid);
    uint64_t* mine_out = a.ws_keys + ((size_t)q * nblk + blockIdx.x) * K;
    for (int t = tid; t < K; t += NT) mine_out[t] = L.sorted[t];
}

// ---------------------------------------------------------------------------------------------------------------
// Batched scan: one workgroup serves a tile of kQ = 4 queries with one pass over its share of G.  The four queries'
// tables are interleaved ([split][sub-id] -> float4), so one 16-byte LDS read returns the table values of the four
// queries for one sub-id: random 16-byte gathers move about twice the bytes per clock that 4-byte ones do, and
// sub-id extraction, address arithmetic and the code loads are shared by the whole tile.
// grid = (item blocks, ceil(B / kQ)).  Static LDS: the tile's tables.  Dynamic LDS:
// hist[kQ][kTiledBins] | ctl[kQ] | state[kWaves][kQ] | lists[kQ][kWaves][cap] | cand[candmax] | sorted[K] | best[kQ][kpad].
constexpr int kQ = 4;                    // queries per tile
constexpr int kTileVecs = 2;             // 16-byte code vectors a thread holds per round
constexpr int kTiledBins = kBins / kQ;   // buckets per query; the kQ histograms together serve as one kBins histogram

// One (wave, query) candidate list's state.  It lives in LDS so that the streaming loop keeps none of it in registers.
struct WaveQ {
    unsigned long long thr;
    int cnt;
    float floor_ge;
};

// Workgroup-wide floors of the batched kernel.  Per query a histogram of kFloorBins buckets counts every score the
// workgroup has appended to a list (and all of the first round's scores); its range is fixed after the first
// round.  At least K counted scores lie in the buckets from b* up, so the lower edge of b* is a lower bound of the
// workgroup's K-th best score so far: a floor for all eight waves, a bucket's width away from the exact one, kept up
// to date for the price of one LDS atomic per candidate and a short scan of the histogram every few rounds.
constexpr int kFloorBins = 256;
struct FloorState {
    float lo, scale;     // bucket of score s: (s - lo) * scale, clamped to [0, kFloorBins)
    int dirty;           // a score was counted since the floor was last derived
    int pad;
};
// (the floors themselves are kQ floats of their own, read once per round by kQ lanes of each wave; a racing store may
// lower one briefly, which is still a valid floor)

// One wave: the floor the histogram allows (see above), -inf if it counts fewer than K scores.  Same value in all lanes.
__device__ __forceinline__ float floor_from_hist(const uint32_t* hist, int K, float lo, float scale, int lane) {
    constexpr int per = kFloorBins / kWave;                  // buckets per lane; lane 0 owns the top ones
    const int first = kFloorBins - per * (lane + 1);
    const uint4 v = *reinterpret_cast<const uint4*>(hist + first);
    static_assert(per == 4, "one 16-byte read per lane");
    const uint32_t mine = v.x + v.y + v.z + v.w;
    const uint32_t upto = wave_prefix_sum(mine);
    const uint64_t has = __ballot(upto >= (uint32_t)K);
    if (has == 0 || !(scale > 0.0f)) return -__builtin_inff();
    const int owner = __builtin_ctzll(has);
    uint32_t above = upto - mine;                            // counted in buckets above this lane's
    int found = 0;
    above += v.w; if (above >= (uint32_t)K) found = 3;
    else { above += v.z; if (above >= (uint32_t)K) found = 2;
    else { above += v.y; if (above >= (uint32_t)K) found = 1; } }
    const int bstar = __builtin_amdgcn_readlane(first + found, owner);
    if (bstar <= 0) return -__builtin_inff();
    // a score cut with bucket(cut) < b*: by monotonicity every score counted in a bucket >= b* is > cut
    const float width = 1.0f / scale;
    float cut = lo + ((float)bstar - 0.5f) * width;
    for (int guard = 0; guard < 8 && bucket_of<kFloorBins>(cut, lo, scale) >= bstar; ++guard) cut -= width;
    if (bucket_of<kFloorBins>(cut, lo, scale) >= bstar) return -__builtin_inff();
    return next_up(cut);
}

// keys of room per query in the workgroup's best[] array (a checkpoint may keep a few more than K)
__host__ __device__ inline int tiled_best_keys(int K) { return ((K > 128 ? K : 128) + 1) & ~1; }

__host__ __device__ inline size_t tiled_lds_bytes(int cap, int candmax, int K) {
    return (size_t)kBins * sizeof(uint32_t) + (size_t)kQ * align16(sizeof(Ctl)) +
           (size_t)kWaves * kQ * sizeof(WaveQ) + (size_t)kQ * kWaves * cap * sizeof(uint64_t) +
           (size_t)candmax * sizeof(uint64_t) + align16((size_t)K * sizeof(uint64_t)) +
           (size_t)kQ * tiled_best_keys(K) * sizeof(uint64_t) + (size_t)kQ * kFloorBins * sizeof(uint32_t) +
           (size_t)kQ * sizeof(FloorState) + (size_t)kQ * sizeof(float);
}

// Eq. 5 for the 16/M items of one code vector and the kQ = 4 queries of the tile; sc[q][e], sums left to right.
// The four queries' tables are interleaved ([split][sub-id] -> float4): one 16-byte LDS read per sub-id.
template <int M>
__device__ __forceinline__ void score_vector_quad(const float4* lut4, const uint32_t* w, float (&sc)[kQ][16 / M]) {
    static_assert(kQ == 4, "one float4 per table entry");
    float4 v[16];
#pragma unroll
    for (int byte = 0; byte < 16; ++byte) {
        const uint32_t code = (w[byte >> 2] >> ((byte & 3) * 8)) & 0xFFu;
        v[byte] = lut4[(byte % M) * kLutStride + code];
    }
    __builtin_amdgcn_sched_barrier(0);                    // keep the 16 reads ahead of the sums
#pragma unroll
    for (int e = 0; e < 16 / M; ++e) {
        float4 acc = v[e * M];
#pragma unroll
        for (int k = 1; k < M; ++k) {
            acc.x = acc.x + v[e * M + k].x; acc.y = acc.y + v[e * M + k].y;
            acc.z = acc.z + v[e * M + k].z; acc.w = acc.w + v[e * M + k].w;
        }
        sc[0][e] = acc.x; sc[1][e] = acc.y; sc[2][e] = acc.z; sc[3][e] = acc.w;
    }
}

// What one thread offers to one query's list after a round: NI scores, their item ids, and whether each may enter.
template <int NI>
struct Slots {
    float sc[NI];
    uint32_t id[NI];
    bool ok[NI];
};

// The uncommon half of a round for one query: some lane holds a score at or above the list's floor.  Out of line, with
// the list's state loaded from and stored back to LDS, so the streaming loop stays small.
template <int NI>
__device__ __noinline__ void offer_slow(WaveQ* st, uint64_t* buf, int cap, int K, int prune_at, Slots<NI> s, int lane) {
    WaveTopK top{buf, cap, K, prune_at, st->cnt, st->thr, st->floor_ge};
#pragma unroll
    for (int e = 0; e < NI; ++e) {
        const bool take = s.ok[e] && s.sc[e] >= top.floor_ge;
        const uint64_t mask = __ballot(take);
        if (mask != 0) top.append(mask, take, s.sc[e], s.id[e], lane);
    }
    if (top.prune_at != 0 && top.cnt >= top.prune_at) top.tighten(lane);
    if (lane == 0) { st->cnt = top.cnt; st->thr = top.thr; st->floor_ge = top.floor_ge; }
    wave_sync();
}

// The batched kernel's dynamic LDS, carved.
struct TileLds {
    uint32_t* hist;
    unsigned char* pctl;     // kQ control blocks
    WaveQ* states;           // [kWaves][kQ]
    uint64_t* lists;         // [kQ][kWaves][cap]
    uint64_t* cand;          // candmax (>= kQ * kFastCand)
    uint64_t* sorted;        // K
    uint64_t* best;          // [kQ][kpad]: per query, a superset of the workgroup's K best so far (ctl->keep keys)
    int kpad;
    float* sfloor;           // [kQ] workgroup-wide floors
};

// Final merge of the batched kernel.  Per query it merges the eight waves' lists (and whatever best[q] already holds:
// ctl(q)->keep keys) into best[q]: the exact K best of everything the workgroup scanned, sorted.  Two paths:
//   - few keys everywhere: wave q ranks query q by counting, no workgroup barrier inside;
//   - otherwise: ranking / sorting by the whole workgroup, one query at a time.
// Every thread of the workgroup calls it.  Out of line: the streaming loop stays small.
__device__ __noinline__ void tile_checkpoint(const TileLds& L, int nq, int K, int cap, int candmax, int tid) {
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    auto ctl_of = [&](int q) { return reinterpret_cast<Ctl*>(L.pctl + (size_t)q * align16(sizeof(Ctl))); };
    auto reset_lists = [&](int q, int wv, float floor_ge) {   // one thread per (query, wave)
        WaveQ* st = L.states + wv * kQ + q;
        st->cnt = 0;
        st->thr = 0ull;
        st->floor_ge = fmaxf(st->floor_ge, floor_ge);
        if (wv == 0) L.sfloor[q] = fmaxf(L.sfloor[q], floor_ge);
    };
    __syncthreads();                                          // every wave's list state in LDS is final
    int total[kQ], keep[kQ];
    bool all_small = true;
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
        total[q] = 0;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) total[q] += L.states[wv * kQ + q].cnt;
        keep[q] = ctl_of(q)->keep;
        if (q < nq && total[q] + keep[q] > kFastCand) all_small = false;
    }
    bool exact_needed[kQ];
#pragma unroll
    for (int q = 0; q < kQ; ++q) exact_needed[q] = q < nq;

    if (all_small) {
        if (wave < nq) {
            const int q = wave, T = total[q] + keep[q];
            uint64_t* c = L.cand + (size_t)q * kFastCand;
            uint64_t* bq = L.best + (size_t)q * L.kpad;
            int at = 0;
            for (int wv = 0; wv < kWaves; ++wv) {
                const int n = L.states[wv * kQ + q].cnt;
                const uint64_t* src = L.lists + ((size_t)q * kWaves + wv) * cap;
                for (int t = lane; t < n; t += kWave) c[at + t] = src[t];
                at += n;
            }
            for (int t = lane; t < keep[q]; t += kWave) c[at + t] = bq[t];
            wave_sync();
            wave_rank_select(c, T, K, bq, lane);
            const uint64_t kth = bq[K - 1];
            if (lane < kWaves) reset_lists(q, lane, kth != 0ull ? score_of_key(kth) : -__builtin_inff());
            if (lane == 0) ctl_of(q)->keep = K;
        }
        __syncthreads();
        return;
    }

    for (int q = 0; q < nq; ++q) {
        if (!exact_needed[q]) continue;
        int before = 0;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv)
            if (wv < wave) before += L.states[wv * kQ + q].cnt;
        const int mine = L.states[wave * kQ + q].cnt;
        uint64_t* qlists = L.lists + (size_t)q * kWaves * cap;
        uint64_t* buf = qlists + (size_t)wave * cap;
        uint64_t* bq = L.best + (size_t)q * L.kpad;
        if (total[q] + keep[q] <= candmax) {                  // one ranking of lists and best together
            for (int t = lane; t < mine; t += kWave) L.cand[before + t] = buf[t];
            for (int t = tid; t < keep[q]; t += kThreads) L.cand[total[q] + t] = bq[t];
            rank_select(L.cand, total[q] + keep[q], K, L.sorted, tid);
        } else {                                              // lists first (histogram or sort), then with best
            for (int t = mine + lane; t < cap; t += kWave) buf[t] = 0;
            __syncthreads();
            block_select(qlists, kWaves * cap, K, L.sorted, L.cand, candmax, L.hist, ctl_of(q), tid);
            for (int t = tid; t < K; t += kThreads) L.cand[t] = L.sorted[t];
            for (int t = tid; t < keep[q]; t += kThreads) L.cand[K + t] = bq[t];
            __syncthreads();
            rank_select(L.cand, K + keep[q], K, L.sorted, tid);
        }
        for (int t = tid; t < K; t += kThreads) bq[t] = L.sorted[t];
        const uint64_t kth = L.sorted[K - 1];
        if (tid < kWaves) reset_lists(q, tid, kth != 0ull ? score_of_key(kth) : -__builtin_inff());
        if (tid == 0) ctl_of(q)->keep = K;
        __syncthreads();                                      // sorted / cand are reused by the next query
    }
}

template <int M>
__global__ __launch_bounds__(kThreads) void scan_topk_tiled_kernel(ScanArgs a, int B) {
    constexpr int IPV = 16 / M, kItems = kTileVecs * IPV, kWords = kTileVecs * 4;
    __shared__ __align__(16) float4 lut4[M * kLutStride];
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem);
    unsigned char* pctl = smem + (size_t)kBins * sizeof(uint32_t);
    WaveQ* states = reinterpret_cast<WaveQ*>(pctl + (size_t)kQ * align16(sizeof(Ctl)));
    uint64_t* lists = reinterpret_cast<uint64_t*>(states + kWaves * kQ);
    uint64_t* cand = lists + (size_t)kQ * kWaves * a.cap;
    uint64_t* sorted = cand + a.candmax;
    const int kpad = tiled_best_keys(a.K);
    uint64_t* best = sorted + align16((size_t)a.K * sizeof(uint64_t)) / sizeof(uint64_t);   // [kQ][kpad]
    uint32_t* fhist = reinterpret_cast<uint32_t*>(best + (size_t)kQ * kpad);                 // [kQ][kFloorBins]
    FloorState* fstate = reinterpret_cast<FloorState*>(fhist + kQ * kFloorBins);             // [kQ]
    float* sfloor = reinterpret_cast<float*>(fstate + kQ);                                   // [kQ]
    auto ctl_of = [&](int q) { return reinterpret_cast<Ctl*>(pctl + (size_t)q * align16(sizeof(Ctl))); };
    const TileLds tl{hist, pctl, states, lists, cand, sorted, best, kpad, sfloor};

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q0 = blockIdx.y * kQ, nblk = gridDim.x, K = a.K, b = a.b;
    const int nq = (B - q0 < kQ) ? B - q0 : kQ;               // queries of this tile that exist
    // The rounds cover the code vectors that lie wholly inside the catalogue (at least one: the host sends smaller
    // catalogues elsewhere); the fewer than 16 / M items after them are scored one by one at the end.
    const long long total_units = (a.N * M) / 16;
    const long long n_scan = total_units * IPV;
    const long long last_vec = total_units - 1;
    const long long round_units = (long long)kThreads * kTileVecs;
    const long long rounds = (total_units + round_units - 1) / round_units;
    const long long inside_rounds = total_units / round_units;
    WaveQ* const my_state = states + wave * kQ;
    auto list_of = [&](int q) { return lists + ((size_t)q * kWaves + wave) * a.cap; };

    // a round's code vectors: always kTileVecs plain 16-byte loads, the index clamped to the last whole vector (no
    // branch, so the loads can be counted and a second round stays in flight); clamped items are masked out later
    // (vt: the thread index whose share of the round is meant; a wave may take over another wave's share)
    auto load = [&](long long rr, int vt, uint32_t (&w)[kWords]) {
        const uint4* base = reinterpret_cast<const uint4*>(a.codes);
#pragma unroll
        for (int u = 0; u < kTileVecs; ++u) {
            long long v = rr * round_units + (long long)u * kThreads + vt;
            v = v < last_vec ? v : last_vec;
            const uint4 x = base[v];
            w[4 * u] = x.x; w[4 * u + 1] = x.y; w[4 * u + 2] = x.z; w[4 * u + 3] = x.w;
        }
    };
    auto item_of = [&](long long rr, int vt, int e) {
        return (rr * round_units + (long long)(e / IPV) * kThreads + vt) * IPV + (e % IPV);
    };
    auto score = [&](const uint32_t (&w)[kWords], float (&sc)[kQ][kItems]) {
#pragma unroll
        for (int u = 0; u < kTileVecs; ++u) {
            float part[kQ][IPV];
            score_vector_quad<M>(lut4, &w[4 * u], part);
#pragma unroll
            for (int q = 0; q < kQ; ++q)
#pragma unroll
                for (int e = 0; e < IPV; ++e) sc[q][u * IPV + e] = part[q][e];
        }
    };

    // ---- 1. codes on their way, the tile's tables into LDS (queries past B get zero tables and are never scored)
    long long r = blockIdx.x;
    uint32_t wa[kWords], wb[kWords];
    load(r, tid, wa);
    load(r + nblk, tid, wb);
    {
        float* lutf = reinterpret_cast<float*>(lut4);
        if (b == kLutStride) {                                // whole rows: 16-byte loads, four sub-ids at a time
            for (int e4 = tid; e4 < kQ * M * kLutStride / 4; e4 += kThreads) {
                const int q = e4 / (M * kLutStride / 4), kj4 = e4 % (M * kLutStride / 4);
                float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (q < nq) v = reinterpret_cast<const float4*>(a.S + (size_t)(q0 + q) * M * kLutStride)[kj4];
                float* dst = lutf + (size_t)kj4 * 4 * kQ + q;
                dst[0] = v.x; dst[kQ] = v.y; dst[2 * kQ] = v.z; dst[3 * kQ] = v.w;
            }
        } else {
            for (int e = tid; e < kQ * M * kLutStride; e += kThreads) {
                const int q = e / (M * kLutStride), kj = e % (M * kLutStride), k = kj / kLutStride, j = kj % kLutStride;
                const float v = (q < nq && j < b) ? a.S[((size_t)(q0 + q) * M + k) * b + j] : 0.0f;
                lutf[((size_t)k * kLutStride + j) * kQ + q] = v;
            }
        }
        for (int i = tid; i < kBins; i += kThreads) hist[i] = 0;
        for (int i = tid; i < kQ * kFloorBins; i += kThreads) fhist[i] = 0;
        for (int i = tid; i < kQ * kpad; i += kThreads) best[i] = 0;
        if (tid < kQ) ctl_of(tid)->keep = 0;
        if (tid == 0) ctl_of(0)->next_unit = 3 * kWaves;       // units 0 .. 3 kWaves - 1 are the waves' own (see 3.)
        if (lane < kQ) my_state[lane] = WaveQ{0ull, 0, -__builtin_inff()};
    }
    __syncthreads();

    // One round's scores against the kQ lists of this wave.  The lists' lengths are cached in scalar registers
    // (cnt[q]) while rounds stream: a survivor then costs one ballot-compacted LDS write and no LDS round trip.
    // Anything else (a list that would overflow, or is due for tightening) goes through the out-of-line path, with
    // the length synchronised through the list's state in LDS around the call.
    int cnt[kQ];
#pragma unroll
    for (int q = 0; q < kQ; ++q) cnt[q] = 0;
    auto publish_counts = [&]() {                             // before anything else reads the states
        if (lane == 0) {
#pragma unroll
            for (int q = 0; q < kQ; ++q) my_state[q].cnt = cnt[q];
        }
    };
    auto offer_round = [&](const float (&sc)[kQ][kItems], long long rr, int vt, const int* bk, const int* bstar) {
        const bool inside = rr < inside_rounds;
        // the kQ floors: read by kQ lanes only (an LDS read costs by the lane), then handed to the whole wave
        const int my_floor = lane < kQ ? __float_as_int(sfloor[lane]) : 0;
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            if (q >= nq) continue;
            float best = sc[q][0];
#pragma unroll
            for (int e = 1; e < kItems; ++e) best = fmaxf(best, sc[q][e]);
            const float floor_ge = __int_as_float(__builtin_amdgcn_readlane(my_floor, q));
            if (__ballot(best >= floor_ge) == 0) continue;    // the usual case
            const float flo = fstate[q].lo, fscale = fstate[q].scale;
            uint64_t* const buf = list_of(q);
            int stop = kItems;                                // first item the inline path had to leave
            bool ok[kItems];
#pragma unroll
            for (int e = 0; e < kItems; ++e) {
                const long long item = item_of(rr, vt, e);
                ok[e] = (inside || item < n_scan) && (bk == nullptr || bk[q * kItems + e] >= bstar[q]);
                if (stop < kItems) continue;
                const bool take = ok[e] && sc[q][e] >= floor_ge;
                const uint64_t mask = __ballot(take);
                if (mask == 0) continue;
                const int n = __popcll(mask);
                if (cnt[q] + n > a.cap) { stop = e; continue; }
                const int pos = cnt[q] + __popcll(mask & ((1ull << lane) - 1ull));
                if (take) {
                    buf[pos] = make_key(sc[q][e] + 0.0f, (uint32_t)item);
                    if (bk == nullptr)                            // (the first round's scores are all counted already)
                        atomicAdd(&fhist[q * kFloorBins + bucket_of<kFloorBins>(sc[q][e], flo, fscale)], 1u);
                }
                cnt[q] += n;
                if (bk == nullptr && lane == 0) fstate[q].dirty = 1;
            }
            if (stop < kItems || (a.prune_at != 0 && cnt[q] >= a.prune_at)) {
                Slots<kItems> s;
#pragma unroll
                for (int e = 0; e < kItems; ++e) {
                    s.sc[e] = sc[q][e];
                    s.id[e] = (uint32_t)item_of(rr, vt, e);
                    s.ok[e] = ok[e] && e >= stop;
                }
                if (lane == 0) my_state[q].cnt = cnt[q];
                wave_sync();
                offer_slow<kItems>(&my_state[q], buf, a.cap, K, a.prune_at, s, lane);
                cnt[q] = __builtin_amdgcn_readfirstlane(my_state[q].cnt);
                if (lane == 0 && my_state[q].floor_ge > sfloor[q]) sfloor[q] = my_state[q].floor_ge;   // the wave's K-th best
            }
        }
    };

    // Every eighth round of a wave (the waves take turns): floors of the queries whose histograms have grown.
    auto refresh_floors = [&]() {
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            if (q >= nq || fstate[q].dirty == 0) continue;
            if (lane == 0) fstate[q].dirty = 0;               // before the histogram is read: a count that lands
            wave_sync();                                      // later sets it again
            const float f = floor_from_hist(fhist + q * kFloorBins, K, fstate[q].lo, fstate[q].scale, lane);
            if (lane == 0 && f > sfloor[q]) sfloor[q] = f;
        }
    };
    int turn = wave;                                          // rounds until this wave's next refresh

    {
        // ---- 2. first round: per query a histogram over its own score range gives that query's cut
        float sc[kQ][kItems];
        score(wa, sc);
        load(r + 2 * nblk, tid, wa);
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
            for (int e = 0; e < kItems; ++e)
                if (item_of(r, tid, e) < n_scan) { mn = fminf(mn, sc[q][e]); mx = fmaxf(mx, sc[q][e]); }
            wave_minmax(mn, mx);
            if (lane == 0) { ctl_of(q)->wave_min[wave] = mn; ctl_of(q)->wave_max[wave] = mx; }
        }
        __syncthreads();
        int bk[kQ * kItems], bstar[kQ];
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            Ctl* c = ctl_of(q);
            float lo = c->wave_min[0], hi = c->wave_max[0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) { lo = fminf(lo, c->wave_min[w]); hi = fmaxf(hi, c->wave_max[w]); }
            // (the histogram lives on as the query's floor histogram: a quarter of the range is added on top, for
            // the scores of later rounds that beat everything in this one)
            const float range = (hi - lo) * 1.25f;
            float scale = (range > 0.0f) ? (float)kFloorBins / range : 0.0f;
            if (!(scale > 0.0f) || scale > 3.0e38f) scale = 0.0f;
            if (tid == q) {
                c->lo = lo; c->scale = scale; c->cut = -__builtin_inff(); c->bstar = 0; c->ncand = 0;
                fstate[q].lo = lo; fstate[q].scale = scale; fstate[q].dirty = 0;
            }
#pragma unroll
            for (int e = 0; e < kItems; ++e) {
                bk[q * kItems + e] = bucket_of<kFloorBins>(sc[q][e], lo, scale);
                if (q < nq && item_of(r, tid, e) < n_scan) atomicAdd(&fhist[q * kFloorBins + bk[q * kItems + e]], 1u);
            }
        }
        __syncthreads();
        if (wave < kQ) {
            find_cut<kFloorBins>(fhist + wave * kFloorBins, K, ctl_of(wave), lane);
            if (lane == 0) sfloor[wave] = next_up(ctl_of(wave)->cut);
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            bstar[q] = ctl_of(q)->bstar;
            if (lane == 0) my_state[q].floor_ge = next_up(ctl_of(q)->cut);
        }
        wave_sync();
        offer_round(sc, r, tid, bk, bstar);
    }

    // ---- 3. stream.  Work is handed out in units of one wave's share of one of this workgroup's rounds: unit u is
    // the share of wave u % kWaves in the workgroup's round u / kWaves (catalogue round blockIdx.x + that * nblk).
    // wb and wa hold the wave's own shares of rounds 1 and 2; after those a wave takes the next free unit from a
    // counter in LDS (requested one step before it is needed).  Without this the four waves that were launched first
    // finish their static shares 15-25 % earlier than the other four and the scan ends on half-empty SIMDs.  Loads
    // are unconditional (past the end they are clamped re-reads, never scored): the waits stay exact.
    // No workgroup-wide step in here: the shared floors keep every wave's candidates few, and a list that fills up
    // all the same is sorted and cut back by its own wave.
    {
        const uint32_t my_rounds = (uint32_t)((rounds - blockIdx.x + nblk - 1) / nblk);
        const uint32_t units = my_rounds * kWaves;
        int pending = 0;                                      // lane 0: result of the last counter request
        auto request_unit = [&]() { if (lane == 0) pending = atomicAdd(&ctl_of(0)->next_unit, 1); };
        auto requested_unit = [&]() -> uint32_t { return (uint32_t)__builtin_amdgcn_readfirstlane(pending); };
        auto round_of = [&](uint32_t u) -> long long { return (long long)blockIdx.x + (long long)(u / kWaves) * nblk; };
        auto vt_of = [&](uint32_t u) -> int { return (int)(u % kWaves) * kWave + lane; };
        uint32_t ub = kWaves + wave, ua = 2 * kWaves + wave;  // units held by wb and wa
        request_unit();
        while (ub < units) {                                  // ub is the older of the two
            {
                float sc[kQ][kItems];
                score(wb, sc);
                const uint32_t done = ub;
                ub = requested_unit();
                request_unit();
                load(round_of(ub), vt_of(ub), wb);
                offer_round(sc, round_of(done), vt_of(done), nullptr, nullptr);
            }
            {
                float sc[kQ][kItems];
                const uint32_t done = ua;
                if (done < units) score(wa, sc);
                ua = requested_unit();
                request_unit();
                load(round_of(ua), vt_of(ua), wa);
                if (done < units) offer_round(sc, round_of(done), vt_of(done), nullptr, nullptr);
            }
            turn -= 2;
            if (turn < 0) { turn += kWaves; refresh_floors(); }
        }
    }
    // the fewer than 16 / M items after the last whole code vector: one per lane of one wave, per query
    if (blockIdx.x == 0 && wave == 0 && n_scan < a.N) {
        const long long item = n_scan + lane;
        float tsc[kQ];
#pragma unroll
        for (int q = 0; q < kQ; ++q) tsc[q] = 0.0f;
        if (item < a.N) {
            const uint8_t* row = a.codes + item * M;
#pragma unroll
            for (int p = 0; p < kQ / 2; ++p) {
                const float* lf = reinterpret_cast<const float*>(lut4);
                float2 acc = make_float2(lf[(size_t)row[0] * kQ + 2 * p], lf[(size_t)row[0] * kQ + 2 * p + 1]);
#pragma unroll
                for (int k = 1; k < M; ++k) {
                    const size_t at = ((size_t)k * kLutStride + row[k]) * kQ + 2 * p;
                    acc.x = acc.x + lf[at];
                    acc.y = acc.y + lf[at + 1];
                }
                tsc[2 * p] = acc.x;
                tsc[2 * p + 1] = acc.y;
            }
        }
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            if (q >= nq) continue;
            Slots<kItems> s;
#pragma unroll
            for (int e = 0; e < kItems; ++e) { s.sc[e] = tsc[q]; s.id[e] = (uint32_t)item; s.ok[e] = e == 0 && item < a.N; }
            if (lane == 0) my_state[q].cnt = cnt[q];
            wave_sync();
            offer_slow<kItems>(&my_state[q], list_of(q), a.cap, K, a.prune_at, s, lane);
            cnt[q] = __builtin_amdgcn_readfirstlane(my_state[q].cnt);
        }
    }

    // ---- 4. last checkpoint, then the workgroup's exact K best per query go to the workspace, sorted
    publish_counts();
    tile_checkpoint(tl, nq, K, a.cap, a.candmax, tid);
    for (int i = tid; i < nq * K; i += kThreads) {
        const int q = i / K, t = i % K;
        a.ws_keys[((size_t)(q0 + q) * nblk + blockIdx.x) * K + t] = best[(size_t)q * kpad + t];
    }
}

// Grid-level fold: one workgroup per query turns the nblk sorted lists of K keys into the final K, sorted.
// Dynamic LDS: hist | ctl | stage (stage_keys, a power of two >= 2K) | cand | sorted
struct FoldArgs {
    const uint64_t* ws_keys;   // [B][nblk][K]
    int nblk, K;
    int stage_keys, candmax;
    int* out_ids;
    float* out_scores;
};

__host__ __device__ inline size_t fold_lds_bytes(int stage_keys, int candmax, int K) {
    return kBins * sizeof(uint32_t) + align16(sizeof(Ctl)) + (size_t)stage_keys * sizeof(uint64_t) +
           (size_t)candmax * sizeof(uint64_t) + align16((size_t)K * sizeof(uint64_t));
}

__global__ __launch_bounds__(kThreads) void fold_topk_kernel(FoldArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem);
    Ctl* ctl = reinterpret_cast<Ctl*>(smem + kBins * sizeof(uint32_t));
    uint64_t* stage = reinterpret_cast<uint64_t*>(smem + kBins * sizeof(uint32_t) + align16(sizeof(Ctl)));
    uint64_t* cand = stage + a.stage_keys;
    uint64_t* sorted = cand + a.candmax;
    const int tid = threadIdx.x, q = blockIdx.x, K = a.K;
    const uint64_t* all = a.ws_keys + (size_t)q * a.nblk * K;
    const long long nkeys = (long long)a.nblk * K;
    auto key_at = [&](long long i) { return all[i]; };
    auto emit = [&](const uint64_t* sorted_keys) {
        for (int t = tid; t < K; t += kThreads) {
            const uint64_t key = sorted_keys[t];
            a.out_ids[(size_t)q * K + t] = id_of_key(key);
            a.out_scores[(size_t)q * K + t] = score_of_key(key);
        }
    };

    // score range of all the keys (empty slots of short lists are 0); a modest number of keys stays in registers
    const int lane = tid & (kWave - 1);
    const bool in_regs = nkeys <= (long long)kThreads * kFoldRegs;
    uint64_t keys[kFoldRegs];
    float mn = __builtin_inff(), mx = -__builtin_inff();
    if (in_regs) {
#pragma unroll
        for (int r = 0; r < kFoldRegs; ++r) {
            const long long i = (long long)r * kThreads + tid;
            keys[r] = (i < nkeys) ? key_at(i) : 0ull;
            if (keys[r]) { float s = score_of_key(keys[r]); mn = fminf(mn, s); mx = fmaxf(mx, s); }
        }
    } else {
        for (long long i = tid; i < nkeys; i += kThreads) {
            uint64_t key = key_at(i);
            if (key) { float s = score_of_key(key); mn = fminf(mn, s); mx = fmaxf(mx, s); }
        }
    }
    for (int i = tid; i < kBins; i += kThreads) hist[i] = 0;
    float lo, scale;
    set_range(mn, mx, ctl, tid, lo, scale);

    if (in_regs) {
        // one pass: histogram, cut, collect the few keys at or above the cut, rank them
        int bk[kFoldRegs];
#pragma unroll
        for (int r = 0; r < kFoldRegs; ++r) {
            bk[r] = -1;
            if (keys[r]) { bk[r] = bucket_of(score_of_key(keys[r]), lo, scale); atomicAdd(&hist[bk[r]], 1u); }
        }
        __syncthreads();
        if (tid < kWave) find_cut(hist, K, ctl, lane);
        __syncthreads();
        const int bstar = ctl->bstar;
#pragma unroll
        for (int r = 0; r < kFoldRegs; ++r) {
            if (bk[r] >= bstar) {
                int pos = atomicAdd(&ctl->ncand, 1);
                if (pos < a.candmax) cand[pos] = keys[r];
            }
        }
        __syncthreads();
        const int C = ctl->ncand;
        if (C <= a.candmax) {
            rank_select(cand, C, K, sorted, tid);
            emit(sorted);
            return;
        }
        // too many keys share the cut bucket (heavy ties): take the staged, sorting path below
    }

    int keep = 0;                                            // best-so-far keys carried at the front of stage
    long long done = 0;
    while (done < nkeys) {
        long long take = nkeys - done;
        if (take > a.stage_keys - keep) take = a.stage_keys - keep;
        for (int t = tid; t < a.stage_keys - keep; t += kThreads) stage[keep + t] = (t < take) ? key_at(done + t) : 0ull;
        __syncthreads();
        block_select(stage, a.stage_keys, K, sorted, cand, a.candmax, hist, ctl, tid);
        done += take;
        keep = K;
        if (done < nkeys) {
            for (int t = tid; t < K; t += kThreads) stage[t] = sorted[t];
            __syncthreads();
        }
    }
    emit(sorted);
}

// ---------------------------------------------------------------------------------------------------------------
// host side

thread_local char g_hip_error[256] = "no HIP error recorded";

int record_hip(hipError_t e) {
    if (e == hipSuccess) return PQ_OK;
    strncpy(g_hip_error, hipGetErrorString(e), sizeof(g_hip_error) - 1);
    g_hip_error[sizeof(g_hip_error) - 1] = 0;
    return PQ_ERR_HIP;
}

int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// ---------------------------------------------------------------------------------------------------------------
// The paper's two other scoring methods (Section 2 and Algorithm 2), for comparison on the same inputs.  Both
// materialise a score per item in HBM, which PQTopK never does; TopK over that array is a kernel of its own.

// TopK of score rows that already sit in memory: scores float [B][ld], N of them used per row.  grid = (blocks, B).
// Same lists, keys and final selection as the catalogue scan; a wave's first floor is one that K of its lanes' best
// scores reach.  Leaves each workgroup's K best keys in the workspace for fold_topk_kernel.
struct TopkScoresArgs {
    const float* scores;
    long long ld, N;
    int K, cap, candmax, prune_at;
    uint64_t* ws_keys;   // [B][nblk][K]
};

constexpr int kScoreVecs = 4;            // 16-byte vectors (four scores each) a thread holds per round

__global__ __launch_bounds__(kThreads, 4) void topk_scores_kernel(TopkScoresArgs a) {
    constexpr int NT = kThreads, NW = kWaves;
    extern __shared__ __align__(16) unsigned char smem[];
    const ScanLds L = carve_scan(smem, 0, a.cap, a.candmax, NW);
    Ctl* ctl = L.ctl;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x, K = a.K;
    const float* row = a.scores + (size_t)q * a.ld;
    const float4* row4 = reinterpret_cast<const float4*>(row);
    const uint32_t total_vec = (uint32_t)(a.N / 4);          // whole vectors; the up to three scores after them come last
    const uint32_t round_vecs = (uint32_t)NT * kScoreVecs;
    const uint32_t rounds = (total_vec + round_vecs - 1) / round_vecs;
    const uint32_t last_vec = total_vec ? total_vec - 1 : 0;
    WaveTopK top{L.lists + (size_t)wave * a.cap, a.cap, K, a.prune_at, 0, 0ull, -__builtin_inff()};

    auto vec_of = [&](uint32_t rr, int u) { return rr * round_vecs + (uint32_t)u * NT + (uint32_t)tid; };
    auto load = [&](uint32_t rr, float4 (&w)[kScoreVecs]) {   // branch-free: past the end the last vector is re-read
#pragma unroll
        for (int u = 0; u < kScoreVecs; ++u) {
            const uint32_t v = vec_of(rr, u);
            w[u] = row4[v < last_vec ? v : last_vec];
        }
    };
    bool first = true;
    auto offer = [&](const float4 (&w)[kScoreVecs], uint32_t rr) {
        float sc[kScoreVecs * 4];
        float best = -__builtin_inff();
#pragma unroll
        for (int u = 0; u < kScoreVecs; ++u) {
            sc[4 * u] = w[u].x; sc[4 * u + 1] = w[u].y; sc[4 * u + 2] = w[u].z; sc[4 * u + 3] = w[u].w;
            if (vec_of(rr, u) < total_vec) best = fmaxf(best, fmaxf(fmaxf(w[u].x, w[u].y), fmaxf(w[u].z, w[u].w)));
        }
        if (first && K <= kWave) top.floor_ge = wave_floor_for_k(best, K);
        first = false;
        if (__ballot(best >= top.floor_ge) == 0) return;
#pragma unroll
        for (int e = 0; e < kScoreVecs * 4; ++e) {
            const uint32_t v = vec_of(rr, e / 4);
            const bool take = v < total_vec && sc[e] >= top.floor_ge;
            const uint64_t mask = __ballot(take);
            if (mask != 0) top.append(mask, take, sc[e], v * 4u + (uint32_t)(e % 4), lane);
        }
        if (top.prune_at != 0 && top.cnt >= top.prune_at) top.tighten(lane);
    };

    if (total_vec != 0) {
        float4 wa[kScoreVecs], wb[kScoreVecs];
        uint32_t r = blockIdx.x;                              // this workgroup's rounds: r, r + nblk, ...
        load(r, wa);
        load(r + nblk, wb);
        for (; r < rounds; r += 2 * nblk) {                   // (a round past the end offers nothing)
            offer(wa, r);
            load(r + 2 * nblk, wa);
            offer(wb, r + nblk);
            load(r + 3 * nblk, wb);
        }
    }
    if (blockIdx.x == 0 && wave == 0) {                       // the scores after the last whole vector
        const long long item = (long long)total_vec * 4 + lane;
        const bool have = item < a.N;
        const float sc = have ? row[item] : 0.0f;
        const bool take = have && sc >= top.floor_ge;
        const uint64_t mask = __ballot(take);
        if (mask != 0) top.append(mask, take, sc, (uint32_t)item, lane);
    }
    workgroup_select<NT>(L, ctl, top, K, a.cap, a.candmax, tid);
    uint64_t* mine_out = a.ws_keys + ((size_t)q * nblk + blockIdx.x) * K;
    for (int t = tid; t < K; t += NT) mine_out[t] = L.sorted[t];
}

// Algorithm 2 (RecJPQScore), one pass of its outer loop: split k's sub-id scores are added to every item's running
// score, scores[q][i] (+)= S[q][k][G[i][k]].  The caller runs k = 0 .. m-1 in order, so every item's sum is the
// same left-to-right chain as in Algorithm 1.  grid = (item blocks, B); a thread owns four consecutive items.
constexpr int kRecjpqThreads = 256;
__global__ __launch_bounds__(kRecjpqThreads) void recjpq_pass_kernel(const uint8_t* codes, const float* S, float* scores,
                                                                     long long ld, long long N, int m, int b, int k) {
    __shared__ float row[kLutStride];
    const int q = blockIdx.y;
    for (int j = threadIdx.x; j < kLutStride; j += kRecjpqThreads)
        row[j] = j < b ? S[((size_t)q * m + k) * b + j] : 0.0f;
    __syncthreads();
    float* out = scores + (size_t)q * ld;
    const long long i0 = ((long long)blockIdx.x * kRecjpqThreads + threadIdx.x) * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const long long i = i0 + j;
        if (i < N) {
            const float s = row[codes[i * m + k]];
            out[i] = k == 0 ? s : out[i] + s;
        }
    }
}

// Eq. 2: the reconstructed item embedding matrix, W[i] = psi_{0,G[i][0]} || .. || psi_{m-1,G[i][m-1]}; one element per
// thread, grid-stride.
__global__ __launch_bounds__(256) void reconstruct_kernel(const uint8_t* codes, const float* centroids, float* W,
                                                          long long N, int d, int m, int b) {
    const int s = d / m;
    const long long total = N * d, stride = (long long)gridDim.x * blockDim.x;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        const long long i = idx / d;
        const int t = (int)(idx % d), k = t / s;
        W[idx] = centroids[((size_t)k * b + codes[i * m + k]) * s + (t % s)];
    }
}

// Eq. 3, the default scoring r = W phi for one query per grid row, float32: sixteen lanes share an item's row of W
// (each takes every sixteenth 16-byte piece and multiplies-and-adds it into one accumulator, in order), then their
// sixteen partial sums are added up across the lanes.  d must be a multiple of 4.  Dynamic LDS: the query, d floats.
constexpr int kDefaultThreads = 256;
__global__ __launch_bounds__(kDefaultThreads) void default_scores_kernel(const float* W, const float* queries, float* scores,
                                                                        long long ld, long long N, int d) {
    extern __shared__ __align__(16) unsigned char smem[];
    float4* phi4 = reinterpret_cast<float4*>(smem);
    const int q = blockIdx.y, d4 = d / 4;
    for (int c = threadIdx.x; c < d4; c += kDefaultThreads)
        phi4[c] = reinterpret_cast<const float4*>(queries + (size_t)q * d)[c];
    __syncthreads();
    const int lane = threadIdx.x & (kWave - 1), sub = lane & 15;
    const long long rows_per_pass = (long long)gridDim.x * (kDefaultThreads / 16);
    for (long long row = (long long)blockIdx.x * (kDefaultThreads / 16) + threadIdx.x / 16; row < N; row += rows_per_pass) {
        // (the sixteen lanes of a group share `row`, so they enter and leave the loop together)
        const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)row * d);
        float acc = 0.0f;
        for (int c = sub; c < d4; c += 16) {
            const float4 w = w4[c], p = phi4[c];
            acc = __builtin_fmaf(w.x, p.x, acc);
            acc = __builtin_fmaf(w.y, p.y, acc);
            acc = __builtin_fmaf(w.z, p.z, acc);
            acc = __builtin_fmaf(w.w, p.w, acc);
        }
        acc += dpp_f32<kDppRowShr + 1>(0.0f, acc);
        acc += dpp_f32<kDppRowShr + 2>(0.0f, acc);
        acc += dpp_f32<kDppRowShr + 4>(0.0f, acc);
        acc += dpp_f32<kDppRowShr + 8>(0.0f, acc);            // lane 15 of each group of sixteen holds the sum
        if (sub == 15) scores[(size_t)q * ld + row] = acc;
    }
}

// Measurement aid: a plain streaming read (16-byte loads, nothing else), the yardstick the scan's HBM rate is held to.
constexpr int kReadThreads = 256, kReadUnroll = 8;     // (eight waves per CU with eight loads in flight each read fastest here)
__global__ __launch_bounds__(kReadThreads) void stream_read_kernel(const uint4* src, long long nvec) {
    uint32_t acc = 0;
    const long long stride = (long long)gridDim.x * kReadThreads;
    long long i = (long long)blockIdx.x * kReadThreads + threadIdx.x;
    for (; i + (kReadUnroll - 1) * stride < nvec; i += kReadUnroll * stride) {
        uint4 v[kReadUnroll];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < kReadUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (; i < nvec; i += stride) { const uint4 v = src[i]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    asm volatile("" ::"v"(acc));                              // (the loaded data is used: the loads stay)
}

struct ScanPlan {
    int copies;      // single-query kernel: copies of the score tables in LDS (1 or kTableCopies)
    bool tiled;      // batched kernel: kQ queries per workgroup
    bool big;        // single-query kernel: kBigThreads threads per workgroup, one workgroup per CU
    int nblk;        // item blocks per query
    int cap;         // keys per wave list
    int candmax;     // keys of the candidate array
    int stage_keys;  // keys the fold stages per pass
    size_t scan_dyn_lds;     // dynamic LDS of the scan launch
    size_t scan_lds;         // dynamic + the static score tables of the vector kernels
    size_t fold_lds;
    bool vec;
};

bool is_vec_m(int m) { return m == 1 || m == 2 || m == 4 || m == 8 || m == 16 || m == 32 || m == 64; }

// `generic`: plan for the generic kernel whatever m is (candidate-list scans use it: their rows are gathered)
ScanPlan make_plan(long long N, int B, int m, int K, bool generic = false) {
    ScanPlan p;
    p.vec = !generic && is_vec_m(m) && N * m >= 16;            // (the vector kernels need one whole code vector at least)
    const long long units = (p.vec && m <= 16) ? (N * m) / 16 : N;   // whole code vectors (the few items after them are extra)
    const long long per_round = (long long)kThreads * (p.vec ? vec_per_thread(m) : kGenericItemsPerThread);
    long long rounds = (units + per_round - 1) / per_round;
    long long most = (kBlocksPerCU * (long long)kAssumedCUs) / B;   // workgroups over the whole grid
    if (most < 8) most = 8;
    long long nblk = rounds < most ? rounds : most;
    long long one_per_cu = kAssumedCUs / B;                    // a short scan is spread evenly: one workgroup per CU, which
    if (one_per_cu < 8) one_per_cu = 8;                        // then takes two or three (possibly ragged) rounds
    if (rounds > one_per_cu && rounds <= most) nblk = one_per_cu;
    if (nblk < 1) nblk = 1;
    if (B > 1 && nblk >= 32) nblk &= ~7LL;                     // same item block of every query on the same XCD
    p.nblk = (int)nblk;
    p.cap = next_pow2(K + kWave);
    if (p.cap < 128) p.cap = 128;
    p.candmax = next_pow2(2 * K);
    if (p.candmax < 512) p.candmax = 512;
    p.stage_keys = next_pow2(2 * K);
    if (p.stage_keys < kChunkKeys) p.stage_keys = kChunkKeys;
    p.copies = 1;
    // A long scan for few queries is bound by LDS bank conflicts of the random lookups: with kTableCopies copies of
    // the tables, lanes l and l' collide only if l % kTableCopies == l' % kTableCopies.  Worth its LDS and fill time
    // only when every workgroup streams many rounds; one workgroup per CU then (the tables take 128 KB at m = 8).
    if (p.vec && m <= 8) {
        const long long nb = kAssumedCUs / B;                  // one workgroup (of kBigThreads) per CU over the whole grid
        const long long big_round = (long long)kBigThreads * vec_per_thread(m);
        const long long big_rounds = (units + big_round - 1) / big_round;
        const size_t dyn = scan_lds_bytes((size_t)m * kLutStride * kTableCopies, p.cap, p.candmax, K, kMaxWaves);
        if (nb >= 8 && big_rounds >= kTableCopiesMinRounds * nb && dyn <= kMaxLdsBytes) {   // (nb < 8: more queries than
                                                                                            // the grid has room for)
            p.copies = kTableCopies;
            p.nblk = (int)nb;
        }
    }
    // A generic scan whose tables leave room for only one 512-thread workgroup per CU (m > 36 or so) runs 1024-thread
    // workgroups instead, one per CU: the same tables then serve sixteen waves, which is what hides the latency of
    // the row loads.  Only when there is more than one workgroup's worth of work per CU.
    p.big = p.copies > 1;
    if (!p.vec || m == 64) {
        const size_t small = scan_lds_bytes((size_t)m * kLutStride, p.cap, p.candmax, K, kWaves);
        const size_t big = scan_lds_bytes((size_t)m * kLutStride, p.cap, p.candmax, K, kMaxWaves);
        long long nb = kAssumedCUs / B;
        if (nb < 8) nb = 8;
        if (2 * small > kMaxLdsBytes && big <= kMaxLdsBytes && rounds > nb) {
            const long long big_round = (long long)kBigThreads * (p.vec ? vec_per_thread(m) : kGenericItemsPerThread);
            const long long big_rounds = (units + big_round - 1) / big_round;
            if (big_rounds < nb) nb = big_rounds;
            if (B > 1 && nb >= 8) nb &= ~7LL;
            p.big = true;
            p.nblk = (int)nb;
        }
    }
    const size_t lut_dyn = p.copies > 1 ? (size_t)m * kLutStride * p.copies : (p.vec ? 0 : (size_t)m * kLutStride);
    p.scan_dyn_lds = scan_lds_bytes(lut_dyn, p.cap, p.candmax, K, p.big ? kMaxWaves : kWaves);
    p.scan_lds = p.scan_dyn_lds + ((p.vec && p.copies == 1) ? (size_t)m * kLutStride * sizeof(float) : 0);
    p.tiled = false;
    // (a small batch over a small catalogue is faster as B single-query scans side by side: the batched kernel's
    // fixed costs, about 15 us of table fill, first-round cuts and final merge, are not yet paid back)
    const bool small_job = B <= 2 || (double)B * (double)N * m <= kTiledMinLookups;
    if (!generic && !small_job && (m == 8 || m == 16) && N * m >= 16) {   // batched kernel, if its tables and lists fit in LDS
        const size_t dyn = tiled_lds_bytes(p.cap, p.candmax, K);
        const size_t all = dyn + (size_t)kQ * m * kLutStride * sizeof(float);
        if (all <= kMaxLdsBytes) {
            p.tiled = true;
            p.scan_dyn_lds = dyn;
            p.scan_lds = all;
            const long long tiles = (B + kQ - 1) / kQ;
            const long long t_round = (long long)kThreads * kTileVecs;
            const long long t_rounds = (units + t_round - 1) / t_round;
            long long want = ((long long)kAssumedCUs) / tiles;
            if (want < 1) want = 1;                           // enough tiles to fill the machine: one workgroup each
            long long nb = t_rounds < want ? t_rounds : want;
            if (nb >= 8) nb &= ~7LL;                          // every tile's item block x lands on XCD x % 8
            if (nb < 1) nb = 1;
            p.nblk = (int)nb;
        }
    }
    p.fold_lds = fold_lds_bytes(p.stage_keys, p.candmax, K);
    return p;
}

size_t workspace_bytes(const ScanPlan& p, int B, int K) {
    const size_t bytes = (size_t)B * p.nblk * K * sizeof(uint64_t);
    return (bytes + 255) & ~(size_t)255;
}

int check_topk_args(const void* codes, const void* S, long long N, int B, int m, int b, int K, const void* out_ids,
                    const void* out_scores, const void* workspace, size_t workspace_bytes_given) {
    if (!codes || !S || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    if (N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    const ScanPlan p = make_plan(N, B, m, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)codes & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)S & 3) || ((uintptr_t)out_ids & 3) ||
        ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(p, B, K)) return PQ_ERR_WORKSPACE;
    return PQ_OK;
}

template <typename KernelT>
hipError_t allow_lds(KernelT kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

template <int M>
hipError_t launch_scan(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    if constexpr (M >= 1 && M <= 8) {
        if (p.copies == kTableCopies) {
            hipError_t e = allow_lds(scan_topk_kernel<M, kTableCopies, kBigThreads>, p.scan_dyn_lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((scan_topk_kernel<M, kTableCopies, kBigThreads>), dim3(p.nblk, B), dim3(kBigThreads),
                               p.scan_dyn_lds, st, a);
            return hipGetLastError();
        }
    }
    if constexpr (M == 0 || M == 64) {
        if (p.big) {
            hipError_t e = allow_lds(scan_topk_kernel<M, 1, kBigThreads>, p.scan_dyn_lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((scan_topk_kernel<M, 1, kBigThreads>), dim3(p.nblk, B), dim3(kBigThreads),
                               p.scan_dyn_lds, st, a);
            return hipGetLastError();
        }
    }
    hipError_t e = allow_lds(scan_topk_kernel<M>, p.scan_dyn_lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(scan_topk_kernel<M>, dim3(p.nblk, B), dim3(kThreads), p.scan_dyn_lds, st, a);
    return hipGetLastError();
}

// Enqueue the catalogue scan: every workgroup's K best keys land in the workspace.
// `subset` / `n_items`: candidate list (then N is its length and the plan is a generic one) or nullptr / N
int enqueue_scan(const ScanPlan& p, const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                 void* workspace, hipStream_t st, const int* subset = nullptr, long long n_items = 0) {
    ScanArgs a;
    a.codes = codes; a.S = S; a.N = N; a.m = m; a.b = b; a.K = K;
    a.subset = subset; a.n_items = (uint32_t)(subset ? n_items : N);
    a.cap = p.cap; a.candmax = p.candmax;
    a.prune_at = (K <= 28) ? 2 * K + 8 : 0;                 // small K: keep lists short enough to rank in one pass
    a.ws_keys = static_cast<uint64_t*>(workspace);
    hipError_t e;
    if (p.tiled) {
        const dim3 grid(p.nblk, (B + kQ - 1) / kQ);
        if (m == 8) {
            e = allow_lds(scan_topk_tiled_kernel<8>, p.scan_dyn_lds);
            if (e == hipSuccess) hipLaunchKernelGGL(scan_topk_tiled_kernel<8>, grid, dim3(kThreads), p.scan_dyn_lds, st, a, B);
        } else {
            e = allow_lds(scan_topk_tiled_kernel<16>, p.scan_dyn_lds);
            if (e == hipSuccess) hipLaunchKernelGGL(scan_topk_tiled_kernel<16>, grid, dim3(kThreads), p.scan_dyn_lds, st, a, B);
        }
        return record_hip(e == hipSuccess ? hipGetLastError() : e);
    }
    switch (p.vec ? m : 0) {
        case 1: e = launch_scan<1>(p, a, B, st); break;
        case 2: e = launch_scan<2>(p, a, B, st); break;
        case 4: e = launch_scan<4>(p, a, B, st); break;
        case 8: e = launch_scan<8>(p, a, B, st); break;
        case 16: e = launch_scan<16>(p, a, B, st); break;
        case 32: e = launch_scan<32>(p, a, B, st); break;
        case 64: e = launch_scan<64>(p, a, B, st); break;
        default: e = launch_scan<0>(p, a, B, st); break;
    }
    return record_hip(e);
}

// Enqueue the fold of the workspace's lists into the outputs.
int enqueue_fold(const ScanPlan& p, int B, int K, void* workspace, int* out_ids, float* out_scores, hipStream_t st) {
    FoldArgs f;
    f.ws_keys = static_cast<const uint64_t*>(workspace);
    f.nblk = p.nblk; f.K = K; f.stage_keys = p.stage_keys; f.candmax = p.candmax;
    f.out_ids = out_ids; f.out_scores = out_scores;
    hipError_t e = allow_lds(fold_topk_kernel, p.fold_lds);
    if (e != hipSuccess) return record_hip(e);
    hipLaunchKernelGGL(fold_topk_kernel, dim3(B), dim3(kThreads), p.fold_lds, st, f);
    return record_hip(hipGetLastError());
}

template <int S_ELEMS>
void launch_subitem(const float* queries, const float* centroids, float* S, int B, int d, int m, int b, hipStream_t st) {
    if constexpr (S_ELEMS > 0 && S_ELEMS % 4 == 0) {
        // batches: the interleaved kernel (it needs 16-byte aligned rows of queries and centroids)
        if (B >= kSubInterleave && (((uintptr_t)queries | (uintptr_t)centroids) & 15) == 0 && d % 4 == 0) {
            dim3 grid(m * ((b + kSubThreads - 1) / kSubThreads), (B + kSubBatchTile - 1) / kSubBatchTile);
            hipLaunchKernelGGL(subitem_scores_batched_kernel<S_ELEMS>, grid, dim3(kSubThreads), 0, st, queries, centroids, S,
                               B, d, m, b);
            return;
        }
    }
    dim3 grid((m * b + kSubThreads - 1) / kSubThreads, (B + kSubQueryTile - 1) / kSubQueryTile);
    hipLaunchKernelGGL(subitem_scores_kernel<S_ELEMS>, grid, dim3(kSubThreads), 0, st, queries, centroids, S, B, d, m, b);
}

}  // namespace

extern "C" {

int pq_subitem_scores(const float* queries, const float* centroids, float* S, int B, int d, int m, int b,
                      void* stream) {
    if (!queries || !centroids || !S) return PQ_ERR_NULL;
    if (B < 1 || d < 1 || m < 1 || b < 1 || b > 256 || d % m != 0) return PQ_ERR_SHAPE;
    if (B > PQ_MAX_B || m > PQ_MAX_M) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)queries & 3) || ((uintptr_t)centroids & 3) || ((uintptr_t)S & 3)) return PQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (d / m) {
        case 4: launch_subitem<4>(queries, centroids, S, B, d, m, b, st); break;
        case 8: launch_subitem<8>(queries, centroids, S, B, d, m, b, st); break;
        case 16: launch_subitem<16>(queries, centroids, S, B, d, m, b, st); break;
        case 32: launch_subitem<32>(queries, centroids, S, B, d, m, b, st); break;
        case 64: launch_subitem<64>(queries, centroids, S, B, d, m, b, st); break;
        default: launch_subitem<0>(queries, centroids, S, B, d, m, b, st); break;
    }
    return record_hip(hipGetLastError());
}

size_t pq_score_topk_workspace_bytes(long long N, int B, int m, int b, int K) {
    if (N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > N || N >= 2147483648LL) return 0;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return 0;
    const ScanPlan p = make_plan(N, B, m, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_score_topk(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                  float* out_scores, void* workspace, size_t workspace_bytes_given, void* stream) {
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_plan(N, B, m, K);
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = enqueue_scan(p, codes, S, N, B, m, b, K, workspace, st);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_score_topk_profile(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                          int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes_given,
                          void* stream, int iters, float* scan_ms) {
    if (!scan_ms) return PQ_ERR_NULL;
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given);
    if (rc != PQ_OK) return rc;
    if (iters < 1) return PQ_ERR_SHAPE;
    const ScanPlan p = make_plan(N, B, m, K);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    hipError_t e = hipEventCreate(&ev0);
    if (e != hipSuccess) return record_hip(e);
    e = hipEventCreate(&ev1);
    if (e != hipSuccess) { (void)hipEventDestroy(ev0); return record_hip(e); }
    rc = enqueue_scan(p, codes, S, N, B, m, b, K, workspace, st);           // untimed warm-up launch
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev0, st));
    for (int it = 0; it < iters && rc == PQ_OK; ++it) rc = enqueue_scan(p, codes, S, N, B, m, b, K, workspace, st);
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev1, st));
    if (rc == PQ_OK) rc = enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
    if (rc == PQ_OK) rc = record_hip(hipStreamSynchronize(st));
    float ms = 0.0f;
    if (rc == PQ_OK) rc = record_hip(hipEventElapsedTime(&ms, ev0, ev1));
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    if (rc == PQ_OK) *scan_ms = ms / (float)iters;
    return rc;
}

size_t pq_score_topk_subset_workspace_bytes(long long n_subset, int B, int m, int b, int K) {
    if (n_subset < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > n_subset || n_subset >= 2147483648LL) return 0;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return 0;
    const ScanPlan p = make_plan(n_subset, B, m, K, true);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_score_topk_subset(const uint8_t* codes, const float* S, const int* subset, long long n_subset, long long N,
                         int B, int m, int b, int K, int* out_ids, float* out_scores, void* workspace,
                         size_t workspace_bytes_given, void* stream) {
    if (!codes || !S || !subset || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    if (n_subset < 1 || N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > n_subset || n_subset > N ||
        N >= 2147483648LL)
        return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    const ScanPlan p = make_plan(n_subset, B, m, K, true);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)codes & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)S & 3) || ((uintptr_t)subset & 3) ||
        ((uintptr_t)out_ids & 3) || ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(p, B, K)) return PQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = enqueue_scan(p, codes, S, n_subset, B, m, b, K, workspace, st, subset, N);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_read_bandwidth_profile(const void* data, size_t bytes, void* stream, int iters, float* read_ms) {
    if (!data || !read_ms) return PQ_ERR_NULL;
    if (bytes < 16 || iters < 1) return PQ_ERR_SHAPE;
    if ((uintptr_t)data & 15) return PQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const long long nvec = (long long)(bytes / 16);
    long long blocks = (nvec + kReadThreads - 1) / kReadThreads;
    if (blocks > 2LL * kAssumedCUs) blocks = 2LL * kAssumedCUs;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    hipError_t e = hipEventCreate(&ev0);
    if (e != hipSuccess) return record_hip(e);
    e = hipEventCreate(&ev1);
    if (e != hipSuccess) { (void)hipEventDestroy(ev0); return record_hip(e); }
    auto launch = [&]() {
        hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(kReadThreads), 0, st,
                           static_cast<const uint4*>(data), nvec);
        return record_hip(hipGetLastError());
    };
    int rc = launch();                                       // untimed warm-up launch
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev0, st));
    for (int it = 0; it < iters && rc == PQ_OK; ++it) rc = launch();
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev1, st));
    if (rc == PQ_OK) rc = record_hip(hipStreamSynchronize(st));
    float ms = 0.0f;
    if (rc == PQ_OK) rc = record_hip(hipEventElapsedTime(&ms, ev0, ev1));
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    if (rc == PQ_OK) *read_ms = ms / (float)iters;
    return rc;
}

// ---- the comparison scorers (Section 2's default scoring, Algorithm 2) and TopK over score rows

namespace {
// plan of pq_topk_scores: blocks per query, list and candidate sizes (as for the scan), LDS of the two launches
ScanPlan make_topk_scores_plan(long long N, int B, int K) {
    ScanPlan p = {};
    const long long vecs = N / 4;
    const long long per_round = (long long)kThreads * kScoreVecs;
    long long rounds = (vecs + per_round - 1) / per_round;
    if (rounds < 1) rounds = 1;
    long long most = (kBlocksPerCU * (long long)kAssumedCUs) / B;
    if (most < 8) most = 8;
    p.nblk = (int)(rounds < most ? rounds : most);
    p.cap = next_pow2(K + kWave);
    if (p.cap < 128) p.cap = 128;
    p.candmax = next_pow2(2 * K);
    if (p.candmax < 512) p.candmax = 512;
    p.stage_keys = next_pow2(2 * K);
    if (p.stage_keys < kChunkKeys) p.stage_keys = kChunkKeys;
    p.copies = 1;
    p.scan_dyn_lds = p.scan_lds = scan_lds_bytes(0, p.cap, p.candmax, K, kWaves);
    p.fold_lds = fold_lds_bytes(p.stage_keys, p.candmax, K);
    return p;
}

int check_topk_scores_shape(long long ld, long long N, int B, int K) {
    if (N < 1 || B < 1 || K < 1 || K > N || ld < N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    return PQ_OK;
}
}  // namespace

size_t pq_topk_scores_workspace_bytes(long long N, int B, int K) {
    if (check_topk_scores_shape(N, N, B, K) != PQ_OK) return 0;
    const ScanPlan p = make_topk_scores_plan(N, B, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_topk_scores(const float* scores, long long ld, long long N, int B, int K, int* out_ids, float* out_scores,
                   void* workspace, size_t workspace_bytes_given, void* stream) {
    if (!scores || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    int rc = check_topk_scores_shape(ld, N, B, K);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_topk_scores_plan(N, B, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)scores & 15) || (B > 1 && (ld & 3)) || ((uintptr_t)workspace & 15) || ((uintptr_t)out_ids & 3) ||
        ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(p, B, K)) return PQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TopkScoresArgs a;
    a.scores = scores; a.ld = ld; a.N = N; a.K = K; a.cap = p.cap; a.candmax = p.candmax;
    a.prune_at = (K <= 28) ? 2 * K + 8 : 0;
    a.ws_keys = static_cast<uint64_t*>(workspace);
    hipError_t e = allow_lds(topk_scores_kernel, p.scan_dyn_lds);
    if (e != hipSuccess) return record_hip(e);
    hipLaunchKernelGGL(topk_scores_kernel, dim3(p.nblk, B), dim3(kThreads), p.scan_dyn_lds, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return record_hip(e);
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_recjpq_scores(const uint8_t* codes, const float* S, long long N, int B, int m, int b, float* scores,
                     long long ld, void* stream) {
    if (!codes || !S || !scores) return PQ_ERR_NULL;
    if (N < 1 || B < 1 || m < 1 || b < 1 || b > 256 || ld < N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)S & 3) || ((uintptr_t)scores & 3)) return PQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((N + 4LL * kRecjpqThreads - 1) / (4LL * kRecjpqThreads)), B);
    for (int k = 0; k < m; ++k) {                            // Algorithm 2's outer loop: one pass over the items per split
        hipLaunchKernelGGL(recjpq_pass_kernel, grid, dim3(kRecjpqThreads), 0, st, codes, S, scores, ld, N, m, b, k);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return record_hip(e);
    }
    return PQ_OK;
}

int pq_reconstruct_items(const uint8_t* codes, const float* centroids, long long N, int d, int m, int b, float* W,
                         void* stream) {
    if (!codes || !centroids || !W) return PQ_ERR_NULL;
    if (N < 1 || d < 1 || m < 1 || b < 1 || b > 256 || d % m != 0 || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (m > PQ_MAX_M) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)centroids & 3) || ((uintptr_t)W & 3)) return PQ_ERR_ALIGN;
    const long long total = N * d;
    long long blocks = (total + 255) / 256;
    if (blocks > 64 * kAssumedCUs) blocks = 64 * kAssumedCUs;
    hipLaunchKernelGGL(reconstruct_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), codes,
                       centroids, W, N, d, m, b);
    return record_hip(hipGetLastError());
}

int pq_default_scores(const float* W, const float* queries, long long N, int B, int d, float* scores, long long ld,
                      void* stream) {
    if (!W || !queries || !scores) return PQ_ERR_NULL;
    if (N < 1 || B < 1 || d < 1 || ld < N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (B > PQ_MAX_B || d % 4 != 0 || (size_t)d * sizeof(float) > 64 * 1024) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)W & 15) || ((uintptr_t)queries & 15) || ((uintptr_t)scores & 3)) return PQ_ERR_ALIGN;
    long long blocks = (N + kDefaultThreads / 16 - 1) / (kDefaultThreads / 16);
    if (blocks > 16 * kAssumedCUs) blocks = 16 * kAssumedCUs;
    hipLaunchKernelGGL(default_scores_kernel, dim3((unsigned)blocks, B), dim3(kDefaultThreads), (size_t)d * sizeof(float),
                       static_cast<hipStream_t>(stream), W, queries, scores, ld, N, d);
    return record_hip(hipGetLastError());
}

const char* pq_strerror(int code) {
    switch (code) {
        case PQ_OK: return "ok";
        case PQ_ERR_NULL: return "a required pointer is NULL";
        case PQ_ERR_SHAPE:
            return "bad shape: need B,d,m,b,K,N >= 1, d % m == 0, b <= 256, K <= N (K <= |V| <= N with a candidate list), "
                   "N < 2^31";
        case PQ_ERR_UNSUPPORTED:
            return "unsupported: K > 512, m > 128, B > 65535, or score tables plus candidate lists exceed LDS";
        case PQ_ERR_WORKSPACE: return "workspace smaller than pq_score_topk_workspace_bytes()";
        case PQ_ERR_ALIGN: return "pointer alignment: codes and workspace 16 bytes, float/int arrays 4 bytes";
        case PQ_ERR_HIP: return g_hip_error;
        default: return "unknown pqtopk error code";
    }
}

}  // extern "C"
