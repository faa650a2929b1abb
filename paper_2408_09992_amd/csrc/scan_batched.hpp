// Eq. 5 + TopK for a tile of four queries per workgroup (scan_topk_tiled_kernel).
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

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
// (the floors themselves are kQ floats of their own, read once per round by kQ lanes of each wave with relaxed atomic
// accesses; a racing store may lower one briefly, which is still a valid floor)

// One wave: the floor the histogram allows (see above), -inf if it counts fewer than K scores.  Same value in all lanes.
__device__ __forceinline__ float floor_from_hist(const uint32_t* hist, int K, float lo, float scale, int lane) {
    constexpr int per = kFloorBins / kWave;                  // buckets per lane; lane 0 owns the top ones
    const int first = kFloorBins - per * (lane + 1);
    const uint4 v = lds_peek_counters4(hist + first);          // (other waves may be counting into the histogram)
    static_assert(per == 4, "four counters per lane");
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
    uint32_t* fhist;         // [kQ][kFloorBins] histograms of the scores appended to the lists
    FloorState* fstate;      // [kQ]
};

// Final merge of the batched kernel.  Per query it merges the eight waves' lists (and whatever best[q] already holds:
// ctl(q)->keep keys) into best[q]: the exact K best of everything the workgroup scanned, sorted.  Two paths:
//   - few keys everywhere: wave q ranks query q by counting, no workgroup barrier inside;
//   - otherwise: ranking / sorting by the whole workgroup, one query at a time.
// Every thread of the workgroup calls it, once, after the streaming loop (inlined: a call would save the caller's registers to
// the stack for a function that returns to nothing but the final store).
__device__ __forceinline__ void tile_checkpoint(const TileLds& L, int nq, int K, int cap, int candmax, bool filter, int tid) {
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
    // `filter` (lists that are only cut back when full: K > 12 in this kernel): the floors once more, from the finished histograms;
    // then every wave drops from its lists what lies below them (keys appended while the floors were still low: with
    // K = 100 they are most of what the lists hold).  At least K scanned items reach a query's floor, so none of
    // its K best is dropped.
    if (filter && wave < nq) {
        const float f = floor_from_hist(L.fhist + wave * kFloorBins, K, L.fstate[wave].lo, L.fstate[wave].scale, lane);
        if (lane == 0 && f > L.sfloor[wave]) L.sfloor[wave] = f;
    }
    if (filter) __syncthreads();
    for (int q = 0; filter && q < nq; ++q) {
        WaveQ* st = L.states + wave * kQ + q;
        uint64_t* buf = L.lists + ((size_t)q * kWaves + wave) * cap;
        const float f = L.sfloor[q];
        const int n = st->cnt;
        int out = 0;
        for (int base = 0; base < n; base += kWave) {         // in place: a chunk is in registers before its survivors
            const uint64_t key = base + lane < n ? buf[base + lane] : 0ull;   // are written at or below its start
            const bool take = key != 0ull && score_of_key(key) >= f;
            const uint64_t mask = __ballot(take);
            if (take) buf[out + __popcll(mask & ((1ull << lane) - 1ull))] = key;
            out += __popcll(mask);
        }
        wave_sync();
        if (lane == 0) st->cnt = out;
    }
    if (filter) __syncthreads();
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

// STAMP: measurement instance that also records wall-clock stamps per wave.
template <int M, bool STAMP = false>
__global__ __launch_bounds__(kThreads) void scan_topk_tiled_kernel(ScanArgs a, int B) {
    constexpr int IPV = 16 / M, kItems = kTileVecs * IPV, kWords = kTileVecs * 4;
    uint64_t* const rec = STAMP ? a.stamps + (((size_t)blockIdx.y * gridDim.x + blockIdx.x) * kWaves + threadIdx.x / kWave) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, threadIdx.x & (kWave - 1));
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
    const TileLds tl{hist, pctl, states, lists, cand, sorted, best, kpad, sfloor, fhist, fstate};

    int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;   // (set again after the streaming loop)
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
    WaveQ* my_state = states + wave * kQ;
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
        // A thread owns table entries (split, sub-id) = tid, tid + kThreads, ...: it reads that entry of each of the
        // tile's four tables (consecutive lanes read consecutive floats) and writes them as one float4, consecutive
        // lanes to consecutive 16-byte slots: no bank conflicts, and every load is on its way before the first store.
        // Sub-ids from b on (tables with fewer than 256 entries per split) and queries past B get zeros.
        constexpr int kPer = M * kLutStride / kThreads;        // entries per thread
        static_assert(M * kLutStride % kThreads == 0, "whole entries per thread");
        float tv[kPer][kQ];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = tid + i * kThreads, k = e / kLutStride, j = e % kLutStride;
#pragma unroll
            for (int q = 0; q < kQ; ++q)
                tv[i][q] = (q < nq && j < b) ? a.S[((size_t)(q0 + q) * M + k) * b + j] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i) lut4[tid + i * kThreads] = make_float4(tv[i][0], tv[i][1], tv[i][2], tv[i][3]);
        for (int i = tid; i < kBins; i += kThreads) hist[i] = 0;
        for (int i = tid; i < kQ * kFloorBins; i += kThreads) fhist[i] = 0;
        for (int i = tid; i < kQ * kpad; i += kThreads) best[i] = 0;
        if (tid < kQ) ctl_of(tid)->keep = 0;
        if (tid == 0) ctl_of(0)->next_unit = 3 * kWaves;       // units 0 .. 3 kWaves - 1 are the waves' own (see 3.)
        if (lane < kQ) my_state[lane] = WaveQ{0ull, 0, -__builtin_inff()};
    }
    stamp<STAMP>(rec, kStampRequested, lane);
    __syncthreads();
    stamp<STAMP>(rec, kStampTables, lane);

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
        const int my_floor = lane < kQ ? __float_as_int(lds_peek(&sfloor[lane])) : 0;
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
                if (bk == nullptr && lane == 0) lds_poke(&fstate[q].dirty, 1);
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
                if (lane == 0 && my_state[q].floor_ge > lds_peek(&sfloor[q])) lds_poke(&sfloor[q], my_state[q].floor_ge);   // the wave's K-th best
            }
        }
    };

    // Floors of the queries whose histograms have grown.  The waves take turns: at first each refreshes every eighth of
    // its rounds, then at intervals that grow by a quarter each time (candidates thin out as 1 / rounds, so the floors
    // move ever more slowly, and a refresh costs a wave some eighty instructions per query).
    auto refresh_floors = [&]() {
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            if (q >= nq || lds_peek(&fstate[q].dirty) == 0) continue;
            if (lane == 0) lds_poke(&fstate[q].dirty, 0);     // before the histogram is read: a count that lands
            wave_sync();                                      // later sets it again
            const float f = floor_from_hist(fhist + q * kFloorBins, K, fstate[q].lo, fstate[q].scale, lane);
            if (lane == 0 && f > lds_peek(&sfloor[q])) lds_poke(&sfloor[q], f);
        }
    };
    int turn = wave;                                          // rounds until this wave's next refresh
    int gap = kWaves;                                         // rounds between two refreshes; grows by a quarter each time

    {
        // ---- 2. first round: per query a histogram over its own score range gives that query's cut
        float sc[kQ][kItems];
        score(wa, sc);
        stamp<STAMP>(rec, kStampScored, lane);
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
        stamp<STAMP>(rec, kStampOffered, lane);
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
            if (turn < 0) { gap += gap >> 2; turn += gap; refresh_floors(); }
        }
    }
    // What the code after the loop needs of the thread's own addresses is derived afresh from the thread index: kept
    // alive over the loop, which has no register to spare, two of them went to scratch memory and back (8 bytes per
    // lane: a megabyte of write-back per launch).
    tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    lane = tid & (kWave - 1);
    wave = tid / kWave;
    my_state = states + wave * kQ;
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
    stamp<STAMP>(rec, kStampStreamed, lane);
    publish_counts();
    tile_checkpoint(tl, nq, K, a.cap, a.candmax, a.prune_at == 0, tid);
    stamp<STAMP>(rec, kStampSelected, lane);
    for (int i = tid; i < nq * K; i += kThreads) {
        const int q = i / K, t = i % K;
        a.ws_keys[((size_t)(q0 + q) * nblk + blockIdx.x) * K + t] = best[(size_t)q * kpad + t];
    }
    stamp<STAMP>(rec, kStampEnd, lane);
}
