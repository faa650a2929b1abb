// What the TopK side of every kernel is made of: keys, histogram cuts, per-wave candidate lists, exact selection.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

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
    float shared_floor;  // single-query kernel, scans of several rounds: workgroup-wide score floor from the running histogram
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
// `extend`: factor on the range (room on top for later scores when the histogram lives on as a running one).
template <int NW = kWaves>
__device__ __forceinline__ void set_range(float mn, float mx, Ctl* ctl, int tid, float& lo_out, float& scale_out,
                                          float extend = 1.0f) {
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    wave_minmax(mn, mx);
    if (lane == 0) { ctl->wave_min[wave] = mn; ctl->wave_max[wave] = mx; }
    __syncthreads();
    float lo = ctl->wave_min[0], hi = ctl->wave_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) { lo = fminf(lo, ctl->wave_min[w]); hi = fmaxf(hi, ctl->wave_max[w]); }
    float range = (hi - lo) * extend;
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

// One wave: the score floor a running histogram allows: at least K counted scores lie in the buckets from b* up, so
// the K-th best of everything counted exceeds every score of a lower bucket.  -inf if fewer than K are counted or the
// range is degenerate.  Same value in all lanes; nothing is written.
template <int BINS = kBins>
__device__ __forceinline__ float floor_of_hist(const uint32_t* hist, int K, float lo, float scale, int lane) {
    constexpr int per = BINS / kWave;                        // buckets per lane; lane 0 owns the top ones
    const int first = BINS - per * (lane + 1);
    uint32_t c[per];
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < per; i += 4) {
        const uint4 v = lds_peek_counters4(hist + first + i);  // (other waves may be counting into the histogram)
        c[i] = v.x; c[i + 1] = v.y; c[i + 2] = v.z; c[i + 3] = v.w;
        mine += v.x + v.y + v.z + v.w;
    }
    const uint32_t upto = wave_prefix_sum(mine);
    const uint64_t has = __ballot(upto >= (uint32_t)K);
    if (has == 0 || !(scale > 0.0f)) return -__builtin_inff();
    const int owner = __builtin_ctzll(has);
    uint32_t above = upto - mine;
    int found = 0;
    bool hit = false;
#pragma unroll
    for (int i = per - 1; i >= 0; --i) {
        above += c[i];
        if (!hit && above >= (uint32_t)K) { found = i; hit = true; }
    }
    const int bstar = __builtin_amdgcn_readlane(first + found, owner);
    if (bstar <= 0) return -__builtin_inff();
    const float width = 1.0f / scale;
    float cut = lo + ((float)bstar - 0.5f) * width;          // a score with bucket(cut) < b*
    for (int guard = 0; guard < 8 && bucket_of<BINS>(cut, lo, scale) >= bstar; ++guard) cut -= width;
    if (bucket_of<BINS>(cut, lo, scale) >= bstar) return -__builtin_inff();
    return next_up(cut);
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

// The end of a single-query scan: the waves' lists -> the workgroup's exact K best, sorted, in L.sorted (zero where
// fewer than K exist).  Every thread of the workgroup calls it once its wave has offered everything.
// `running`: L.hist is the scan's running histogram (range hlo / hscale): its floor joins the waves' own.
template <int NT>
__device__ __forceinline__ void workgroup_select(const ScanLds& L, Ctl* ctl, WaveTopK& top, int K, int cap, int candmax,
                                                 int tid, bool running = false, float hlo = 0.0f, float hscale = 0.0f) {
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
    // (every wave derives the histogram's floor by itself; nothing counts into it any more)
    if (running && total > kFilterMin) wg_floor = fmaxf(wg_floor, floor_of_hist<kBins>(L.hist, K, hlo, hscale, lane));
    bool ranked = false;
    if (total <= candmax || (running && wg_floor > -__builtin_inff())) {
        if (total > kFilterMin) {
            // a long scan leaves every wave with its own K best and more: only keys that reach the best of the waves'
            // K-th scores, or the floor of the running histogram, can be among the workgroup's K best (both are lower
            // bounds of the workgroup's K-th)
            for (int t0 = 0; t0 < top.cnt; t0 += kWave) {
                const uint64_t key = t0 + lane < top.cnt ? top.buf[t0 + lane] : 0ull;
                const bool take = key != 0ull && score_of_key(key) >= wg_floor;
                const uint64_t mask = __ballot(take);
                int base = 0;
                if (lane == 0 && mask != 0) base = atomicAdd(&ctl->ncand, __popcll(mask));
                base = __builtin_amdgcn_readfirstlane(base);
                const int pos = base + __popcll(mask & ((1ull << lane) - 1ull));
                if (take && pos < candmax) L.cand[pos] = key;
            }
            __syncthreads();
            total = ctl->ncand;                                   // (more than candmax: the lists are intact, see below)
        } else {
            for (int t = lane; t < top.cnt; t += kWave) L.cand[before + t] = top.buf[t];
        }
        if (total <= candmax) {
            rank_select<NT>(L.cand, total, K, L.sorted, tid);    // its first barrier orders the copies above
            ranked = true;
        }
    }
    if (!ranked) {
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
