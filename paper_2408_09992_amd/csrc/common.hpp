// Constants, cross-lane helpers (DPP), wave-level reductions and the bitonic sort shared by every kernel.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

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
constexpr int kRegisterSelectMinK = 32;           // scans of at most kRing rounds: K from which all scores are selected from registers at once
constexpr int kSharedFloorMinRounds = 6;          // single-query scan: rounds per workgroup from which the waves share a floor
constexpr int kSharedFloorMinRoundsLargeK = 3;    // ... for K >= 32
constexpr int kFoldRegs = 12;                     // keys per thread the fold keeps in registers (6144 per query)
constexpr int kFoldWideRegs = 13;                 // ... and of the 1024-thread fold (13,312 keys)
constexpr int kFoldSmallRegs = 6;                 // keys per thread of the small-K fold (3072 per query) ...
constexpr int kFoldSmallRegsMax = 12;             // ... and of its larger instance (6144)
constexpr int kChunkKeys = 2048;                  // keys the grid-level fold takes per pass (4 per thread)
constexpr size_t kMaxLdsBytes = 160 * 1024;       // LDS per workgroup on gfx950
constexpr int kAssumedCUs = 256;                  // MI355X; only used to size grids and the workspace
constexpr int kBlocksPerCU = 2;                   // single-query scan workgroups per CU over the whole grid
constexpr int kTableCopies = 16;                  // copies of the score tables in the long single-query scan
constexpr int kTableCopiesMinRounds = 4;          // rounds per workgroup from which the copies pay for themselves (measured: 2 to 4)

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

// Words in LDS that one wave writes while other waves of the workgroup read them with no barrier in between (shared
// floors, "something changed" flags, histogram counters that other waves update with atomic adds): relaxed atomic
// accesses at workgroup scope.  They compile to the plain LDS loads and stores, but the compiler may neither tear,
// repeat nor hoist them.  Any value such a read returns is one that was stored at some time, which is all the users
// need (every floor ever stored is a valid floor).
template <typename T>
__device__ __forceinline__ T lds_peek(const T* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
template <typename T>
__device__ __forceinline__ void lds_poke(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }
// four consecutive histogram counters (16-byte aligned) that other waves may be incrementing: two 8-byte atomic loads
__device__ __forceinline__ uint4 lds_peek_counters4(const uint32_t* p) {
    const unsigned long long a = lds_peek(reinterpret_cast<const unsigned long long*>(p));
    const unsigned long long b = lds_peek(reinterpret_cast<const unsigned long long*>(p) + 1);
    return make_uint4((uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32));
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

// min and max over the wave of unsigned values, in every lane
__device__ __forceinline__ void wave_minmax_u32(uint32_t& mn, uint32_t& mx) {
    mn = min(mn, dpp_u32<kDppQuadSwap1>(mn, mn));       mx = max(mx, dpp_u32<kDppQuadSwap1>(mx, mx));
    mn = min(mn, dpp_u32<kDppQuadSwap2>(mn, mn));       mx = max(mx, dpp_u32<kDppQuadSwap2>(mx, mx));
    mn = min(mn, dpp_u32<kDppRowHalfMirror>(mn, mn));   mx = max(mx, dpp_u32<kDppRowHalfMirror>(mx, mx));
    mn = min(mn, dpp_u32<kDppRowMirror>(mn, mn));       mx = max(mx, dpp_u32<kDppRowMirror>(mx, mx));
    // every row of 16 lanes now holds its own extremes; combine the four rows through scalar reads
    const uint32_t m0 = (uint32_t)__builtin_amdgcn_readlane((int)mn, 0), m1 = (uint32_t)__builtin_amdgcn_readlane((int)mn, 16);
    const uint32_t m2 = (uint32_t)__builtin_amdgcn_readlane((int)mn, 32), m3 = (uint32_t)__builtin_amdgcn_readlane((int)mn, 48);
    const uint32_t x0 = (uint32_t)__builtin_amdgcn_readlane((int)mx, 0), x1 = (uint32_t)__builtin_amdgcn_readlane((int)mx, 16);
    const uint32_t x2 = (uint32_t)__builtin_amdgcn_readlane((int)mx, 32), x3 = (uint32_t)__builtin_amdgcn_readlane((int)mx, 48);
    mn = min(min(m0, m1), min(m2, m3));
    mx = max(max(x0, x1), max(x2, x3));
}

__device__ __forceinline__ float float_of_orderable(uint32_t u) { return __uint_as_float(u ^ ((u >> 31) ? 0x80000000u : 0xFFFFFFFFu)); }

// A floor for a wave's top K (K in 1..64): a value that at least K of the lanes' values v reach, found by searching
// between the wave's extremes (so close below the K-th largest, not exactly it).  Each of the STEPS steps cuts the
// interval into four with three thresholds whose ballots are independent of one another: a wave on its own issues an
// instruction only every seven cycles or so, dependent or not, so what counts is the number of instructions, and a
// four-way step yields two bits for less than two halvings cost.  (The extremes are taken on the values'
// order-preserving integer images: integer minima need no NaN handling.)  Lanes with nothing to offer pass -inf; if
// fewer than K lanes have a value the floor is -inf.  Same result in every lane.
template <int STEPS = 6>
__device__ __forceinline__ float wave_floor_for_k(float v, int K) {
    const float ninf = -__builtin_inff();
    if (__popcll(__ballot(v > ninf)) < K) return ninf;
    const uint32_t o = orderable_bits(v);
    uint32_t olo = v > ninf ? o : 0xFFFFFFFFu, ohi = o;
    wave_minmax_u32(olo, ohi);
    float lo = float_of_orderable(olo), hi = float_of_orderable(ohi);   // at least K lanes reach lo
#pragma unroll
    for (int step = 0; step < STEPS; ++step) {
        const float range = hi - lo;
        const float t1 = __builtin_fmaf(range, 0.25f, lo), t2 = __builtin_fmaf(range, 0.5f, lo), t3 = __builtin_fmaf(range, 0.75f, lo);
        const bool r1 = __popcll(__ballot(v >= t1)) >= K, r2 = __popcll(__ballot(v >= t2)) >= K,
                   r3 = __popcll(__ballot(v >= t3)) >= K;        // (t1 <= t2 <= t3, so r3 implies r2 implies r1)
        const float new_lo = r3 ? t3 : (r2 ? t2 : (r1 ? t1 : lo));
        hi = !r1 ? t1 : (!r2 ? t2 : (!r3 ? t3 : hi));
        lo = new_lo;
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

// Slots of a wave's stamp record (measurement instances of the kernels; wall_clock64() ticks, lane 0 of the wave).
// A slot a kernel does not pass stays as the caller left it.
constexpr int kStampSlots = 16;
enum StampSlot {
    kStampEntry = 0,        // first instruction of the wave
    kStampRequested = 1,    // scan: table values and the first rounds of codes requested
    kStampTables = 2,       // scan: tables in LDS (after the workgroup's barrier)
    kStampCodes = 3,        // scan: the first rounds' codes have arrived (the stamped instance waits for them here)
    kStampScored = 4,       // scan: short scans: all items scored; longer ones: first round scored
    kStampOffered = 5,      // scan: short scans: the wave's candidates are in the candidate array; longer: first cut found
    kStampStreamed = 6,     // scan: all rounds streamed (longer scans only)
    kStampSelected = 7,     // scan: the workgroup's K best are ranked
    kStampEnd = 8,          // last instruction before the wave ends
    kStampLoaded = 9,       // fold: the lists' keys are in registers
    kStampCut = 10,         // fold: histogram cut found
    kStampCollected = 11,   // fold: candidates collected
};
template <bool STAMP>
__device__ __forceinline__ void stamp(uint64_t* record, int slot, int lane) {
    if constexpr (STAMP) {
        // (nothing is scheduled across a stamp: what precedes it in the source has been issued, and whatever that needed
        // from memory or LDS has arrived, when the clock is read)
        __builtin_amdgcn_sched_barrier(0);
        if (lane == 0) record[slot] = wall_clock64();
        __builtin_amdgcn_sched_barrier(0);
    }
}
