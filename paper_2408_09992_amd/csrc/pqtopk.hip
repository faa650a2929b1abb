// PQTopK scoring for gfx950 (MI355X): kernels and the C ABI declared in include/pqtopk.h.
//
// Path (paper Section 3): pq_subitem_scores() builds the sub-id score matrix S (Eq. 4); pq_score_topk() streams the
// codebook G once, turns every item's m sub-ids into a score by m table lookups in LDS (Eq. 5), and keeps only the
// K best <id, score> pairs (Algorithm 1, V = I).  Item scores never reach memory.
//
// Total order used everywhere: a 64-bit key  (orderable(score) << 32) | ~id.  A larger key is a better item:
// higher score first, lower id between equal scores.  Keys of distinct items are distinct, key 0 means "empty".
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include "pqtopk.h"

namespace {

constexpr int kWave = 64;
constexpr int kScanThreads = 256;                 // 4 waves per workgroup
constexpr int kScanWaves = kScanThreads / kWave;
constexpr int kLutStride = 256;                   // table entries per split in LDS (uint8 sub-ids never run past it)
constexpr int kMergeThreads = 256;
constexpr size_t kMaxLdsBytes = 160 * 1024;       // LDS per workgroup on gfx950
constexpr int kAssumedCUs = 256;                  // MI355X; only used to size grids and the workspace

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
// Eq. 4.  One thread per (query, split, sub-id): a left-to-right chain of fused multiply-adds over the d/m
// elements, starting from +0.
__global__ __launch_bounds__(256) void subitem_scores_kernel(const float* __restrict__ queries,
                                                             const float* __restrict__ centroids,
                                                             float* __restrict__ S, int d, int m, int b) {
    const int s = d / m;
    const int kj = blockIdx.x * 256 + threadIdx.x;       // k * b + j
    const int q = blockIdx.y;
    if (kj >= m * b) return;
    const int k = kj / b;
    const float* psi = centroids + (size_t)kj * s;
    const float* phi = queries + (size_t)q * d + (size_t)k * s;
    float acc = 0.0f;
    for (int t = 0; t < s; ++t) acc = __builtin_fmaf(psi[t], phi[t], acc);
    S[(size_t)q * m * b + kj] = acc;
}

// ---------------------------------------------------------------------------------------------------------------
// Per-wave candidate list in LDS: `cap` keys, `cnt` of them in use, `thr` = K-th best key once K are known.
struct WaveTopK {
    uint64_t* buf;
    int cap;
    int K;
    int cnt;
    uint64_t thr;

    // sort the list, keep the K best, raise the threshold
    __device__ void prune(int lane) {
        for (int t = cnt + lane; t < cap; t += kWave) buf[t] = 0;
        wave_sync();
        bitonic_sort_desc<false>(buf, cap, lane, kWave);
        if (cnt >= K) { cnt = K; thr = buf[K - 1]; }
    }

    // every lane offers one key (0 = nothing); keys above the threshold are appended
    __device__ void offer(uint64_t key, int lane) {
        bool pass = key > thr;
        uint64_t mask = __ballot(pass);
        if (mask == 0) return;
        int n = __popcll(mask);
        if (cnt + n > cap) {
            prune(lane);
            pass = key > thr;
            mask = __ballot(pass);
            if (mask == 0) return;
            n = __popcll(mask);
        }
        int pos = cnt + __popcll(mask & ((1ull << lane) - 1ull));
        if (pass) buf[pos] = key;
        cnt += n;
    }
};

// Eq. 5 for one item whose m sub-ids sit in `c` (M bytes, little-endian packed): left-to-right fp32 sum.
template <int M>
__device__ __forceinline__ float item_score(const float* lut, const uint32_t* words, int first_byte) {
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < M; ++k) {
        int byte = first_byte + k;
        uint32_t code = (words[byte >> 2] >> ((byte & 3) * 8)) & 0xFFu;
        float v = lut[k * kLutStride + code];
        acc = (k == 0) ? v : acc + v;
    }
    return acc + 0.0f;
}

// Catalogue scan, m in {1,2,4,8,16}: one 16-byte load carries 16/M whole items.
// grid = (item blocks, B).  Dynamic LDS: float lut[M*256]; uint64 wavebuf[kScanWaves][cap].
template <int M>
__global__ __launch_bounds__(kScanThreads) void scan_topk_vec_kernel(const uint8_t* __restrict__ codes,
                                                                     const float* __restrict__ S, long long N,
                                                                     int b, int K, int cap,
                                                                     uint64_t* __restrict__ ws) {
    constexpr int IPV = 16 / M;
    extern __shared__ __align__(16) unsigned char smem[];
    float* lut = reinterpret_cast<float*>(smem);
    uint64_t* bufs = reinterpret_cast<uint64_t*>(smem + (size_t)M * kLutStride * sizeof(float));

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x;

    const float* Sq = S + (size_t)q * M * b;
    for (int e = tid; e < M * kLutStride; e += kScanThreads) {
        int k = e / kLutStride, j = e % kLutStride;
        lut[e] = (j < b) ? Sq[k * b + j] : 0.0f;
    }
    __syncthreads();

    WaveTopK top{bufs + (size_t)wave * cap, cap, K, 0, 0ull};

    const long long total_bytes = N * M;
    const long long total_vecs = (total_bytes + 15) / 16;
    const long long full_vecs = total_bytes / 16;
    const uint4* cvec = reinterpret_cast<const uint4*>(codes);

    for (long long base = (long long)blockIdx.x * kScanThreads + wave * kWave; base < total_vecs;
         base += (long long)nblk * kScanThreads) {
        const long long v = base + lane;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (v < full_vecs) {
            uint4 x = cvec[v];
            w[0] = x.x; w[1] = x.y; w[2] = x.z; w[3] = x.w;
        } else if (v < total_vecs) {                      // ragged last vector: byte loads
            for (long long a = v * 16; a < total_bytes; ++a) {
                int o = (int)(a - v * 16);
                w[o >> 2] |= (uint32_t)codes[a] << ((o & 3) * 8);
            }
        }
#pragma unroll
        for (int e = 0; e < IPV; ++e) {
            const long long item = v * IPV + e;
            float sc = item_score<M>(lut, w, e * M);
            uint64_t key = (item < N) ? make_key(sc, (uint32_t)item) : 0ull;
            top.offer(key, lane);
        }
    }

    // wave -> block: every wave leaves its K best (sorted) at the front of its buffer, zeros behind
    top.prune(lane);
    for (int t = top.cnt + lane; t < cap; t += kWave) top.buf[t] = 0;
    __syncthreads();
    bitonic_sort_desc<true>(bufs, kScanWaves * cap, tid, kScanThreads);
    uint64_t* out = ws + ((size_t)q * nblk + blockIdx.x) * K;
    for (int t = tid; t < K; t += kScanThreads) out[t] = bufs[t];
}

// Catalogue scan for any other m: one lane per item, byte loads.
__global__ __launch_bounds__(kScanThreads) void scan_topk_item_kernel(const uint8_t* __restrict__ codes,
                                                                      const float* __restrict__ S, long long N,
                                                                      int m, int b, int K, int cap,
                                                                      uint64_t* __restrict__ ws) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* lut = reinterpret_cast<float*>(smem);
    uint64_t* bufs = reinterpret_cast<uint64_t*>(smem + (size_t)m * kLutStride * sizeof(float));

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x;

    const float* Sq = S + (size_t)q * m * b;
    for (int e = tid; e < m * kLutStride; e += kScanThreads) {
        int k = e / kLutStride, j = e % kLutStride;
        lut[e] = (j < b) ? Sq[k * b + j] : 0.0f;
    }
    __syncthreads();

    WaveTopK top{bufs + (size_t)wave * cap, cap, K, 0, 0ull};

    for (long long base = (long long)blockIdx.x * kScanThreads + wave * kWave; base < N;
         base += (long long)nblk * kScanThreads) {
        const long long item = base + lane;
        uint64_t key = 0ull;
        if (item < N) {
            const uint8_t* g = codes + item * m;
            float acc = lut[g[0]];
            for (int k = 1; k < m; ++k) acc = acc + lut[k * kLutStride + g[k]];
            key = make_key(acc + 0.0f, (uint32_t)item);
        }
        top.offer(key, lane);
    }

    top.prune(lane);
    for (int t = top.cnt + lane; t < cap; t += kWave) top.buf[t] = 0;
    __syncthreads();
    bitonic_sort_desc<true>(bufs, kScanWaves * cap, tid, kScanThreads);
    uint64_t* out = ws + ((size_t)q * nblk + blockIdx.x) * K;
    for (int t = tid; t < K; t += kScanThreads) out[t] = bufs[t];
}

// Grid-level merge: one workgroup per query folds the nblk*K candidate keys into the final K, sorted.
// Dynamic LDS: uint64 buf[mcap], mcap a power of two >= 2*K.
__global__ __launch_bounds__(kMergeThreads) void merge_topk_kernel(const uint64_t* __restrict__ ws, int nblk, int K,
                                                                   int mcap, int* __restrict__ out_ids,
                                                                   float* __restrict__ out_scores) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint64_t* buf = reinterpret_cast<uint64_t*>(smem);
    const int tid = threadIdx.x, q = blockIdx.x;
    const uint64_t* in = ws + (size_t)q * nblk * K;
    const long long total = (long long)nblk * K;
    int keep = 0;
    long long done = 0;
    while (done < total) {
        long long take = total - done;
        if (take > mcap - keep) take = mcap - keep;
        for (int t = tid; t < mcap - keep; t += kMergeThreads) buf[keep + t] = (t < take) ? in[done + t] : 0ull;
        __syncthreads();
        bitonic_sort_desc<true>(buf, mcap, tid, kMergeThreads);
        done += take;
        keep = K;
    }
    for (int t = tid; t < K; t += kMergeThreads) {
        uint64_t key = buf[t];
        out_ids[(size_t)q * K + t] = id_of_key(key);
        out_scores[(size_t)q * K + t] = score_of_key(key);
    }
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

struct ScanPlan {
    int nblk;        // item blocks per query
    int cap;         // keys per wave buffer
    int mcap;        // keys in the merge buffer
    size_t scan_lds;
    size_t merge_lds;
    bool vec;
};

bool is_vec_m(int m) { return m == 1 || m == 2 || m == 4 || m == 8 || m == 16; }

ScanPlan make_plan(long long N, int B, int m, int K) {
    ScanPlan p;
    p.vec = is_vec_m(m);
    long long units = p.vec ? (N * m + 15) / 16 : N;          // lane-sized pieces of work
    long long want = (units + kScanThreads * 4 - 1) / (kScanThreads * 4);
    long long most = (8LL * kAssumedCUs) / B;
    if (most < 1) most = 1;
    if (want > most) want = most;
    if (want < 1) want = 1;
    p.nblk = (int)want;
    p.cap = next_pow2(K + kWave);
    if (p.cap < 128) p.cap = 128;
    p.mcap = next_pow2(2 * K);
    if (p.mcap < 2048) p.mcap = 2048;
    p.scan_lds = (size_t)m * kLutStride * sizeof(float) + (size_t)kScanWaves * p.cap * sizeof(uint64_t);
    p.merge_lds = (size_t)p.mcap * sizeof(uint64_t);
    return p;
}

int check_topk_args(const void* codes, const void* S, long long N, int B, int m, int b, int K, const void* out_ids,
                    const void* out_scores, const void* workspace, size_t workspace_bytes) {
    if (!codes || !S || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    if (N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    if (make_plan(N, B, m, K).scan_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)codes & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)S & 3) || ((uintptr_t)out_ids & 3) ||
        ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes < pq_score_topk_workspace_bytes(N, B, m, b, K)) return PQ_ERR_WORKSPACE;
    return PQ_OK;
}

template <typename KernelT>
hipError_t allow_lds(KernelT kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

// Enqueue scan + merge.  With ev_start / ev_stop the scan kernel alone is bracketed by the two events.
int enqueue_score_topk(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                       float* out_scores, void* workspace, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
    const ScanPlan p = make_plan(N, B, m, K);
    uint64_t* ws = static_cast<uint64_t*>(workspace);
    dim3 grid(p.nblk, B), block(kScanThreads);
    hipError_t e = hipSuccess;
    if (ev_start) { e = hipEventRecord(ev_start, st); if (e != hipSuccess) return record_hip(e); }
#define PQ_LAUNCH_VEC(MM)                                                                                          \
    case MM:                                                                                                       \
        e = allow_lds(scan_topk_vec_kernel<MM>, p.scan_lds);                                                       \
        if (e == hipSuccess)                                                                                       \
            hipLaunchKernelGGL(scan_topk_vec_kernel<MM>, grid, block, p.scan_lds, st, codes, S, N, b, K, p.cap, ws); \
        break;
    if (p.vec) {
        switch (m) {
            PQ_LAUNCH_VEC(1) PQ_LAUNCH_VEC(2) PQ_LAUNCH_VEC(4) PQ_LAUNCH_VEC(8) PQ_LAUNCH_VEC(16)
            default: break;
        }
    } else {
        e = allow_lds(scan_topk_item_kernel, p.scan_lds);
        if (e == hipSuccess)
            hipLaunchKernelGGL(scan_topk_item_kernel, grid, block, p.scan_lds, st, codes, S, N, m, b, K, p.cap, ws);
    }
#undef PQ_LAUNCH_VEC
    if (e != hipSuccess) return record_hip(e);
    e = hipGetLastError();
    if (e != hipSuccess) return record_hip(e);
    if (ev_stop) { e = hipEventRecord(ev_stop, st); if (e != hipSuccess) return record_hip(e); }
    e = allow_lds(merge_topk_kernel, p.merge_lds);
    if (e != hipSuccess) return record_hip(e);
    hipLaunchKernelGGL(merge_topk_kernel, dim3(B), dim3(kMergeThreads), p.merge_lds, st, ws, p.nblk, K, p.mcap,
                       out_ids, out_scores);
    return record_hip(hipGetLastError());
}

}  // namespace

extern "C" {

int pq_subitem_scores(const float* queries, const float* centroids, float* S, int B, int d, int m, int b,
                      void* stream) {
    if (!queries || !centroids || !S) return PQ_ERR_NULL;
    if (B < 1 || d < 1 || m < 1 || b < 1 || b > 256 || d % m != 0) return PQ_ERR_SHAPE;
    if (B > PQ_MAX_B || m > PQ_MAX_M) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)queries & 3) || ((uintptr_t)centroids & 3) || ((uintptr_t)S & 3)) return PQ_ERR_ALIGN;
    dim3 grid((m * b + 255) / 256, B);
    hipLaunchKernelGGL(subitem_scores_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream), queries,
                       centroids, S, d, m, b);
    return record_hip(hipGetLastError());
}

size_t pq_score_topk_workspace_bytes(long long N, int B, int m, int b, int K) {
    if (N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > N || N >= 2147483648LL) return 0;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return 0;
    const ScanPlan p = make_plan(N, B, m, K);
    if (p.scan_lds > kMaxLdsBytes) return 0;
    size_t bytes = (size_t)B * p.nblk * K * sizeof(uint64_t);
    return (bytes + 255) & ~(size_t)255;
}

int pq_score_topk(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                  float* out_scores, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes);
    if (rc != PQ_OK) return rc;
    return enqueue_score_topk(codes, S, N, B, m, b, K, out_ids, out_scores, workspace,
                              static_cast<hipStream_t>(stream), nullptr, nullptr);
}

int pq_score_topk_profile(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                          int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes, void* stream,
                          int iters, float* scan_ms) {
    if (!scan_ms) return PQ_ERR_NULL;
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes);
    if (rc != PQ_OK) return rc;
    if (iters < 1) return PQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t a = nullptr, z = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e != hipSuccess) return record_hip(e);
    e = hipEventCreate(&z);
    if (e != hipSuccess) { (void)hipEventDestroy(a); return record_hip(e); }
    double sum = 0.0;
    for (int it = 0; it < iters && rc == PQ_OK; ++it) {
        rc = enqueue_score_topk(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, st, a, z);
        if (rc != PQ_OK) break;
        e = hipStreamSynchronize(st);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, z);
        if (e != hipSuccess) { rc = record_hip(e); break; }
        sum += ms;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(z);
    if (rc == PQ_OK) *scan_ms = (float)(sum / iters);
    return rc;
}

const char* pq_strerror(int code) {
    switch (code) {
        case PQ_OK: return "ok";
        case PQ_ERR_NULL: return "a required pointer is NULL";
        case PQ_ERR_SHAPE: return "bad shape: need B,d,m,b,K,N >= 1, d % m == 0, b <= 256, K <= N, N < 2^31";
        case PQ_ERR_UNSUPPORTED: return "unsupported: K > 1024, m > 128, B > 65535, or score tables plus candidate lists exceed LDS";
        case PQ_ERR_WORKSPACE: return "workspace smaller than pq_score_topk_workspace_bytes()";
        case PQ_ERR_ALIGN: return "pointer alignment: codes and workspace 16 bytes, float/int arrays 4 bytes";
        case PQ_ERR_HIP: return g_hip_error;
        default: return "unknown pqtopk error code";
    }
}

}  // extern "C"
