// The second launch of every TopK call: the workgroups' lists -> the final sorted K per query (fold_topk_kernel).
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

// Grid-level fold: one workgroup per query turns the nblk sorted lists of K keys into the final K, sorted.
// Dynamic LDS: hist | ctl | stage (stage_keys, a power of two >= 2K) | cand | sorted
struct FoldArgs {
    const uint64_t* ws_keys;   // [B][nlists][K]: per query, nlists sorted lists of K keys
    int nlists, K;
    int lists_per_group;       // lists one workgroup folds; grid = (ceil(nlists / lists_per_group), B)
    int stage_keys, candmax;
    uint64_t* out_keys;        // intermediate level: [B][groups][K] keys; nullptr at the last level, which writes
    int* out_ids;              // ... the result
    float* out_scores;
    uint64_t* stamps;          // STAMP instances only: wall-clock stamps, kStampSlots per wave
};

__host__ __device__ inline size_t fold_lds_bytes(int stage_keys, int candmax, int K) {
    return kBins * sizeof(uint32_t) + align16(sizeof(Ctl)) + (size_t)stage_keys * sizeof(uint64_t) +
           (size_t)candmax * sizeof(uint64_t) + align16((size_t)K * sizeof(uint64_t));
}

// NT threads, REGS keys per thread held in registers: <kThreads, kFoldRegs> is the usual instance; <kBigThreads,
// kFoldWideRegs> takes a query's lists in one go when they are too many for the first (many workgroups times a
// larger K at a small batch), instead of a level of several smaller folds.
template <int NT, int REGS, bool STAMP = false>
__global__ __launch_bounds__(NT) void fold_topk_kernel(FoldArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t* const rec = STAMP ? a.stamps + (((size_t)blockIdx.y * gridDim.x + blockIdx.x) * (NT / kWave) + threadIdx.x / kWave) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, threadIdx.x & (kWave - 1));
    uint32_t* hist = reinterpret_cast<uint32_t*>(smem);
    Ctl* ctl = reinterpret_cast<Ctl*>(smem + kBins * sizeof(uint32_t));
    uint64_t* stage = reinterpret_cast<uint64_t*>(smem + kBins * sizeof(uint32_t) + align16(sizeof(Ctl)));
    uint64_t* cand = stage + a.stage_keys;
    uint64_t* sorted = cand + a.candmax;
    const int tid = threadIdx.x, q = blockIdx.y, group = blockIdx.x, K = a.K;
    const int first_list = group * a.lists_per_group;
    const int my_lists = a.nlists - first_list < a.lists_per_group ? a.nlists - first_list : a.lists_per_group;
    const uint64_t* all = a.ws_keys + ((size_t)q * a.nlists + first_list) * K;
    const long long nkeys = (long long)my_lists * K;
    auto key_at = [&](long long i) { return all[i]; };
    auto emit = [&](const uint64_t* sorted_keys) {
        for (int t = tid; t < K; t += NT) {
            const uint64_t key = sorted_keys[t];
            if (a.out_keys != nullptr) {
                a.out_keys[((size_t)q * gridDim.x + group) * K + t] = key;
            } else {
                a.out_ids[(size_t)q * K + t] = id_of_key(key);
                a.out_scores[(size_t)q * K + t] = score_of_key(key);
            }
        }
    };

    // score range of all the keys (empty slots of short lists are 0).  The host never gives a workgroup more keys than
    // its registers hold (nkeys <= NT * REGS: fold_lists_per_group()).
    const int lane = tid & (kWave - 1);
    uint64_t keys[REGS];
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int r = 0; r < REGS; ++r) {
        const long long i = (long long)r * NT + tid;
        keys[r] = (i < nkeys) ? key_at(i) : 0ull;
        if (keys[r]) { float s = score_of_key(keys[r]); mn = fminf(mn, s); mx = fmaxf(mx, s); }
    }
    for (int i = tid; i < kBins; i += NT) hist[i] = 0;
    stamp<STAMP>(rec, kStampLoaded, lane);
    float lo, scale;
    set_range<NT / kWave>(mn, mx, ctl, tid, lo, scale);

    {
        // one pass: histogram, cut, collect the few keys at or above the cut, rank them
        int bk[REGS];
#pragma unroll
        for (int r = 0; r < REGS; ++r) {
            bk[r] = -1;
            if (keys[r]) { bk[r] = bucket_of(score_of_key(keys[r]), lo, scale); atomicAdd(&hist[bk[r]], 1u); }
        }
        __syncthreads();
        if (tid < kWave) find_cut(hist, K, ctl, lane);
        __syncthreads();
        stamp<STAMP>(rec, kStampCut, lane);
        const int bstar = ctl->bstar;
#pragma unroll
        for (int r = 0; r < REGS; ++r) {
            if (bk[r] >= bstar) {
                int pos = atomicAdd(&ctl->ncand, 1);
                if (pos < a.candmax) cand[pos] = keys[r];
            }
        }
        __syncthreads();
        stamp<STAMP>(rec, kStampCollected, lane);
        const int C = ctl->ncand;
        if (C <= a.candmax) {
            rank_select<NT>(cand, C, K, sorted, tid);
            stamp<STAMP>(rec, kStampSelected, lane);
            emit(sorted);
            stamp<STAMP>(rec, kStampEnd, lane);
            return;
        }
        // too many keys share the cut bucket (heavy ties): take the staged, sorting path below
    }

    int keep = 0;                                            // best-so-far keys carried at the front of stage
    long long done = 0;
    while (done < nkeys) {
        long long take = nkeys - done;
        if (take > a.stage_keys - keep) take = a.stage_keys - keep;
        for (int t = tid; t < a.stage_keys - keep; t += NT) stage[keep + t] = (t < take) ? key_at(done + t) : 0ull;
        __syncthreads();
        block_select<NT>(stage, a.stage_keys, K, sorted, cand, a.candmax, hist, ctl, tid);
        done += take;
        keep = K;
        if (done < nkeys) {
            for (int t = tid; t < K; t += NT) stage[t] = sorted[t];
            __syncthreads();
        }
    }
    emit(sorted);
}

// The fold for small K (K <= kSmallKMax) when a query's lists fit R keys per thread (nlists * K <= NT * R): the keys go
// straight from memory to registers and through select_small_k(), the selection the short scan uses: per-wave floors
// by wave operations, one barrier, ranking by counting.  grid = (1, B).  A kernel of its own because this launch is all
// latency (a few thousand keys): its time is the two dependent memory round trips it cannot avoid (arguments, keys)
// plus its instruction count, and this one has a fifth of the general fold's instructions and a sixth of its barriers.
template <int NT, int R, bool STAMP = false>
__global__ __launch_bounds__(NT) void fold_small_kernel(FoldArgs a) {
    __shared__ SmallSelectLds<NT> sel;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), q = blockIdx.y, K = a.K;
    uint64_t* const rec = STAMP ? a.stamps + ((size_t)q * (NT / kWave) + tid / kWave) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, lane);
    const int nkeys = a.nlists * K;
    const uint64_t* all = a.ws_keys + (size_t)q * nkeys;
    uint64_t keys[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int i = r * NT + tid;
        keys[r] = i < nkeys ? all[i] : 0ull;
    }
    small_select_clear<NT>(sel, tid);
    __syncthreads();
    float sc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) sc[r] = keys[r] != 0ull ? score_of_key(keys[r]) : empty_score();
    stamp<STAMP>(rec, kStampLoaded, lane);
    int* const out_ids = a.out_ids + (size_t)q * K;
    float* const out_scores = a.out_scores + (size_t)q * K;
    select_small_k<NT, R, STAMP>(sc, [&](int slot) -> uint32_t { return (uint32_t)id_of_key(keys[slot]); }, K, sel, tid,
                                 [&](int rank, uint64_t key) {
                                     out_ids[rank] = id_of_key(key);
                                     out_scores[rank] = score_of_key(key);
                                 }, rec);
    stamp<STAMP>(rec, kStampEnd, lane);
}
