// TopK for small K straight from registers: the selection shared by the short catalogue scan and the small fold.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
//
// These kernels run for a few microseconds with two to four waves per SIMD, so a wave's time is its instruction count
// (a vector instruction occupies its SIMD for four cycles) plus the latencies it cannot hide: everything here is
// written for few instructions and few LDS round trips, not for throughput.
#pragma once

constexpr int kSmallKMax = kRegisterSelectMinK - 1;   // K up to which select_small_k() is used (a wave's 64 lanes give its floor)
constexpr int kSmallCand = 512;                       // keys of its candidate array
constexpr int kSmallFloorSteps = 3;                   // four-way search steps of a wave's floor: a 64th of the lanes' range (5 % more candidates than the exact floor gives)

// An empty slot's score: a quiet NaN.  It never wins a maximum and no comparison with it holds, so empty slots need
// no flags of their own (scores of items are never NaN: the inputs are finite).
__device__ __forceinline__ float empty_score() { return __uint_as_float(0x7FC00000u); }

// LDS a workgroup needs for select_small_k(): the candidate array (16-byte aligned), one key per wave, a counter.
template <int NT>
struct SmallSelectLds {
    uint64_t cand[kSmallCand];
    uint64_t wave_best[NT / kWave];
    int ncand;
    uint32_t floor_bits;   // order-preserving image of the highest floor a wave has found so far (0: none yet)
};

// Before the workgroup barrier that precedes select_small_k(): an empty candidate array and counter.
template <int NT>
__device__ __forceinline__ void small_select_clear(SmallSelectLds<NT>& L, int tid) {
    static_assert(kSmallCand % 2 == 0, "cleared two keys at a time");
    for (int i = tid; i < kSmallCand / 2; i += NT) reinterpret_cast<ulonglong2*>(L.cand)[i] = make_ulonglong2(0ull, 0ull);
    if (tid == 0) { L.ncand = 0; L.floor_bits = 0u; }
}

// max over the wave of a 64-bit key, in every lane (DPP steps inside quads and rows, readlane across the four rows)
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_max_key(uint64_t k) {
    const uint32_t lo = dpp_u32<CTRL>((uint32_t)k, (uint32_t)k), hi = dpp_u32<CTRL>((uint32_t)(k >> 32), (uint32_t)(k >> 32));
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    return o > k ? o : k;
}
__device__ __forceinline__ uint64_t wave_max_key(uint64_t k) {
    k = dpp_max_key<kDppQuadSwap1>(k);
    k = dpp_max_key<kDppQuadSwap2>(k);
    k = dpp_max_key<kDppRowHalfMirror>(k);
    k = dpp_max_key<kDppRowMirror>(k);
    uint64_t best = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)k, row * 16);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(k >> 32), row * 16);
        const uint64_t o = ((uint64_t)hi << 32) | lo;
        best = o > best ? o : best;
    }
    return best;
}

// Sorted exact K best of the n keys in cand[0..n) (LDS; zero up to the next multiple of 8) by counting: a key's position
// is the number of keys that beat it.  Rank r goes to emit(r, key); ranks from n on (fewer than K keys exist) get 0.
// With four threads per key each counts over a quarter of the keys (the loop is bound by the latency of its LDS reads).
// No barrier inside: the caller's barrier has made cand[] complete.
template <int NT, typename Emit>
__device__ __forceinline__ void rank_emit(const uint64_t* cand, int n, int K, int tid, Emit&& emit) {
    const int n8 = (n + 7) & ~7;
    auto count8 = [&](int u, uint64_t mine) -> uint32_t {
        const ulonglong2 p0 = *reinterpret_cast<const ulonglong2*>(cand + u);
        const ulonglong2 p1 = *reinterpret_cast<const ulonglong2*>(cand + u + 2);
        const ulonglong2 p2 = *reinterpret_cast<const ulonglong2*>(cand + u + 4);
        const ulonglong2 p3 = *reinterpret_cast<const ulonglong2*>(cand + u + 6);
        return (uint32_t)((p0.x > mine) + (p0.y > mine) + (p1.x > mine) + (p1.y > mine) + (p2.x > mine) + (p2.y > mine) +
                          (p3.x > mine) + (p3.y > mine));
    };
    if (n8 * 4 <= NT) {
        const int t = tid >> 2, part = tid & 3;              // (n8 is a multiple of 8: a wave is all in or all out)
        if (t < n8) {
            const uint64_t mine = cand[t];
            uint32_t rank = 0;
#pragma unroll 2
            for (int u = part * 8; u < n8; u += 32) rank += count8(u, mine);
            rank += dpp_u32<kDppQuadSwap1>(0u, rank);
            rank += dpp_u32<kDppQuadSwap2>(0u, rank);
            if (part == 0 && mine != 0ull && rank < (uint32_t)K) emit((int)rank, mine);
        }
    } else {
        for (int t = tid; t < n; t += NT) {
            const uint64_t mine = cand[t];
            uint32_t rank = 0;
            for (int u = 0; u < n8; u += 8) rank += count8(u, mine);
            if (mine != 0ull && rank < (uint32_t)K) emit((int)rank, mine);
        }
    }
    for (int t = n + tid; t < K; t += NT) emit(t, 0ull);
}

// The workgroup's exact, sorted K best (1 <= K <= kSmallKMax) of the items its threads hold in registers: thread-local
// slots i = 0 .. R-1 with score sc[i] (empty_score() where a slot holds nothing) and item id id_of(i).  Rank r goes to
// emit(r, key) (0 for ranks that do not exist).  L: cleared by small_select_clear() before the caller's last barrier.
//
// Every wave finds, with wave operations only, a floor that K of its lanes' best scores reach; every one of the wave's K
// best items reaches it, and few others do (a dozen of a wave's hundreds of scores at K = 10).  One ballot per slot
// marks them.  Usually no lane holds two (the ballots' population counts tell): a lane then picks its one candidate by
// the ballots, positions come from the union of the ballots and ONE counter update per wave, and the wave makes one LDS
// write.  Otherwise lanes count their candidates, positions come from a prefix sum, and each lane writes its j-th
// candidate in the wave's j-th write.  After one barrier the workgroup ranks the candidates by counting.  More
// candidates than the array holds (heavy ties) take a slow path that is exact for any input: K times, the best
// remaining key of the workgroup is found and emitted.
// STAMP / rec: measurement instances record wall-clock stamps (candidates written, K best ranked).
template <int NT, int R, bool STAMP = false, typename IdOf, typename Emit>
__device__ __forceinline__ void select_small_k(const float (&sc)[R], IdOf&& id_of, int K, SmallSelectLds<NT>& L, int tid,
                                               Emit&& emit, uint64_t* rec = nullptr) {
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    float best = -__builtin_inff();
#pragma unroll
    for (int i = 0; i < R; ++i) best = fmaxf(best, sc[i]);    // (an empty slot's NaN never wins)
    // A floor that some wave has found holds for the whole workgroup (that wave alone has K items at or above it), so a
    // wave that gets here later takes it and saves the search.  (In the short scan the second wave of every SIMD
    // finishes its lookups most of a microsecond after the first: its selection is what the workgroup waits for.)
    const uint32_t seen = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_peek(&L.floor_bits));
    float f;
    if (seen != 0u) {
        f = float_of_orderable(seen);
    } else {
        f = wave_floor_for_k<kSmallFloorSteps>(best, K);
        if (lane == 0 && f > -__builtin_inff()) atomicMax(&L.floor_bits, orderable_bits(f));
    }
    bool mine[R];                                             // this lane's slot i is a candidate
    bool any_mine = false;
    uint64_t any = 0ull;
    int total = 0;
#pragma unroll
    for (int i = 0; i < R; ++i) {
        mine[i] = sc[i] >= f;
        const uint64_t mask = __ballot(mine[i]);
        any_mine = any_mine || mine[i];
        any |= mask;
        total += __popcll(mask);
    }
    int base = 0;
    if (lane == 0 && total != 0) base = atomicAdd(&L.ncand, total);
    if (total == __popcll(any)) {
        // no lane holds two candidates: a lane's candidate is its one marked slot
        float s = 0.0f;
        uint32_t item = 0;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            s = mine[i] ? sc[i] : s;
            item = mine[i] ? id_of(i) : item;
        }
        base = __builtin_amdgcn_readfirstlane(base);
        const int pos = base + __popcll(any & ((1ull << lane) - 1ull));
        if (any_mine && pos < kSmallCand) L.cand[pos] = make_key(s + 0.0f, item);
    } else {
        uint32_t c = 0;
#pragma unroll
        for (int i = 0; i < R; ++i) c += mine[i] ? 1u : 0u;
        const uint32_t upto = wave_prefix_sum(c);
        base = __builtin_amdgcn_readfirstlane(base);
        const int pos = base + (int)(upto - c);
        for (uint32_t j = 0; __ballot(c > j) != 0; ++j) {     // the wave's j-th write: every lane's j-th candidate
            float s = 0.0f;
            uint32_t item = 0, seen = 0;
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const bool hit = mine[i] && seen == j;
                s = hit ? sc[i] : s;
                item = hit ? id_of(i) : item;
                seen += mine[i] ? 1u : 0u;
            }
            if (c > j && pos + (int)j < kSmallCand) L.cand[pos + (int)j] = make_key(s + 0.0f, item);
        }
    }
    stamp<STAMP>(rec, kStampOffered, lane);
    __syncthreads();
    const int n = L.ncand;
    if (n <= kSmallCand) {
        rank_emit<NT>(L.cand, n, K, tid, emit);
        stamp<STAMP>(rec, kStampSelected, lane);
        return;
    }
    // heavy ties: more candidates than the array holds
    uint64_t last = ~0ull;                                    // every key is smaller
    for (int r = 0; r < K; ++r) {
        uint64_t mine = 0ull;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const uint64_t key = make_key(sc[i] + 0.0f, id_of(i));
            if (sc[i] == sc[i] && key < last && key > mine) mine = key;   // (sc == sc: the slot holds an item)
        }
        mine = wave_max_key(mine);
        if (lane == 0) L.wave_best[wave] = mine;
        __syncthreads();
        uint64_t top = 0ull;
#pragma unroll
        for (int w = 0; w < NT / kWave; ++w) top = L.wave_best[w] > top ? L.wave_best[w] : top;
        if (tid == 0) emit(r, top);                           // (0 once nothing is left)
        last = top;                                           // (0: no key is smaller, the remaining ranks get 0)
        __syncthreads();
    }
}
