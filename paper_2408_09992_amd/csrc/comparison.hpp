// Kernels of the paper's two comparison scorers, TopK over score rows, and the streaming-read yardstick.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

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
