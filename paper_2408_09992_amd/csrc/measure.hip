// Machine yardsticks declared in include/pqtopk_measure.h: an empty launch and random gathers from LDS.
// (The aids that time the library's own kernels live in pqtopk.hip, next to the launches they time.)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pqtopk.h"
#include "pqtopk_measure.h"

namespace {

__global__ void empty_kernel(uint32_t* sink, int never) {
    if (never == 0x7fffffff) sink[0] = 1u;                    // (reads its arguments, writes nothing)
}

constexpr int kGatherOffsets = 16;     // gather offsets a lane keeps in registers and shifts from round to round

// 32-bit finaliser of a multiplicative hash: offsets that differ between lanes in every bit
__device__ __forceinline__ uint32_t mix32(uint32_t h) {
    h ^= h >> 16; h *= 0x7feb352du;
    h ^= h >> 15; h *= 0x846ca68bu;
    h ^= h >> 16;
    return h;
}

template <int W> struct GatherWord;
template <> struct GatherWord<4> { using type = uint32_t; };
template <> struct GatherWord<8> { using type = uint2; };
template <> struct GatherWord<16> { using type = uint4; };
__device__ __forceinline__ uint32_t fold_word(uint32_t v) { return v; }
__device__ __forceinline__ uint32_t fold_word(uint2 v) { return v.x ^ v.y; }
__device__ __forceinline__ uint32_t fold_word(uint4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// Every lane reads `rounds` (a multiple of kGatherOffsets) W-byte words from a table in LDS.  Random case: lane l keeps
// kGatherOffsets hashed, W-aligned offsets and adds the same step to all of them each trip (a common shift of random
// offsets is as random).  With `copies` > 1 the table is read as table_bytes / (W * copies) entries of `copies`
// adjacent words each, and lane l reads word l % copies of its entry (the layout of the scan's replicated tables).
// Conflict-free case: the lanes of a wave read 64 consecutive words of a row that moves from trip to trip.  Two
// address instructions per read either way; the reads of a trip are independent.
template <int W>
__global__ __launch_bounds__(1024) void lds_gather_kernel(int table_bytes, int rounds, int conflict_free, int copies,
                                                          uint32_t* sink) {
    extern __shared__ __align__(16) unsigned char table[];
    using Word = typename GatherWord<W>::type;
    uint32_t* t32 = reinterpret_cast<uint32_t*>(table);
    for (int i = threadIdx.x; i < table_bytes / 4; i += blockDim.x) t32[i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    // (copies > 1: the hashed bits choose the entry, the bits below them are the lane's copy and stay put)
    const uint32_t mask = (uint32_t)(table_bytes - 1) & ~(uint32_t)(W * copies - 1);
    const uint32_t copy_off = (threadIdx.x % (uint32_t)copies) * W;
    const uint32_t gid = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t off[kGatherOffsets];
#pragma unroll
    for (int u = 0; u < kGatherOffsets; ++u) {
        if (conflict_free) off[u] = ((mix32((gid / 64u) * kGatherOffsets + u) * (64u * W)) + (threadIdx.x & 63u) * W) & mask;
        else off[u] = (mix32(gid * kGatherOffsets + u + 0x9E3779B9u) & mask) | copy_off;
    }
    uint32_t acc = 0;
    // (a multiple of the entry size: rows stay rows and copies stay copies)
    const uint32_t step = conflict_free ? 64u * W * 5u : 111u * W * (uint32_t)copies;
    uint32_t shift = 0;
    for (int r = 0; r < rounds; r += kGatherOffsets) {
        Word v[kGatherOffsets];
#pragma unroll
        for (int u = 0; u < kGatherOffsets; ++u)
            v[u] = *reinterpret_cast<const Word*>(table + (((off[u] + shift) & mask) | copy_off));
#pragma unroll
        for (int u = 0; u < kGatherOffsets; ++u) acc ^= fold_word(v[u]);
        shift += step;
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;                    // (practically never: the reads are kept, nothing is written)
}


// ---- what synchronising inside one launch costs, against a launch boundary (pq_measure_sync_variant)
// Stand-ins for the two places where a step could save a launch: folding the workgroups' partial results in the last
// workgroup to finish (instead of a fold launch), and computing Eq. 4 inside the scan launch behind a grid-wide barrier
// (instead of an Eq. 4 launch).  The kernels do the synchronisation and the memory traffic of those schemes and none of
// the arithmetic: what is measured is the mechanism.  All waits are bounded.
constexpr int kSyncThreads = 512;
constexpr int kSyncKeys = 10;          // keys a workgroup hands over
constexpr int kSyncSpinLimit = 4000;   // polls of the grid barrier before a workgroup gives up waiting (never reached)
struct SyncArgs {
    uint32_t* ctl;        // control words, zero between launches: [0] ticket, [64 * (1 + g)] group tickets
    uint32_t* tags;       // [grid] generation tags of the grid barrier
    uint64_t* keys;       // [grid][16]
    float* S;             // [2048]: the Eq. 4 stand-in's table
    const float* cent;    // [2048][64]
    const float* phi;     // [512]
    uint64_t* out;        // [8] results nobody needs
    uint32_t gen;         // launch number (the tag of this launch's barrier)
    int lists;            // lists the separate fold launch reads
};

// reduce the `lists` lists of kSyncKeys keys to their maximum (a stand-in for the fold's work); ATOMIC: agent-scope loads
template <bool ATOMIC>
__device__ __forceinline__ void sync_fold(const SyncArgs& a, int lists) {
    __shared__ unsigned long long red[kSyncThreads / 64];
    unsigned long long mx = 0;
    for (int i = threadIdx.x; i < lists * 16; i += kSyncThreads) {
        unsigned long long v = 0ull;
        if ((i & 15) < kSyncKeys) v = ATOMIC ? __hip_atomic_load(&a.keys[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : a.keys[i];
        mx = v > mx ? v : mx;
    }
    for (int o = 32; o > 0; o >>= 1) { const unsigned long long t = __shfl_xor(mx, o); mx = t > mx ? t : mx; }
    if ((threadIdx.x & 63) == 0) red[threadIdx.x / 64] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kSyncThreads / 64; ++w) mx = red[w] > mx ? red[w] : mx;
        a.out[2] = mx;
    }
}

__global__ __launch_bounds__(kSyncThreads) void sync_write_kernel(SyncArgs a) {
    if (threadIdx.x < kSyncKeys) a.keys[blockIdx.x * 16 + threadIdx.x] = (uint64_t)blockIdx.x * 1000 + threadIdx.x + a.gen;
}
__global__ __launch_bounds__(kSyncThreads) void sync_fold_kernel(SyncArgs a) { sync_fold<false>(a, a.lists); }

// the last workgroup to arrive folds.  FENCED: plain stores, an acquire-release ticket (the memory model's way: the
// release writes the L2 back, the acquire invalidates it); else keys written through and read with agent-scope
// accesses, the stores waited for, relaxed tickets.  LEVELS = 2: sixteen group tickets, then one.
template <bool FENCED, int LEVELS>
__global__ __launch_bounds__(kSyncThreads) void sync_last_folds_kernel(SyncArgs a) {
    __shared__ int last;
    const uint64_t key = (uint64_t)blockIdx.x * 1000 + threadIdx.x + a.gen;
    constexpr int kOrder = FENCED ? __ATOMIC_ACQ_REL : __ATOMIC_RELAXED;
    if (threadIdx.x < kSyncKeys) {
        if (FENCED) a.keys[blockIdx.x * 16 + threadIdx.x] = key;
        else __hip_atomic_store(&a.keys[blockIdx.x * 16 + threadIdx.x], key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (FENCED) __syncthreads();
    if (threadIdx.x < 64) {
        if (!FENCED) __builtin_amdgcn_s_waitcnt(0);           // this wave's stores (all of the workgroup's) have left
        if (threadIdx.x == 0) {
            const int nwg = gridDim.x;
            int is_last = 0;
            if (LEVELS == 1) {
                const uint32_t t = __hip_atomic_fetch_add(&a.ctl[0], 1u, kOrder, __HIP_MEMORY_SCOPE_AGENT);
                is_last = t == (uint32_t)nwg - 1;
            } else {
                const int groups = 16, g = blockIdx.x % groups, in_group = (nwg - g + groups - 1) / groups;
                const uint32_t t = __hip_atomic_fetch_add(&a.ctl[64 * (1 + g)], 1u, kOrder, __HIP_MEMORY_SCOPE_AGENT);
                if (t == (uint32_t)in_group - 1) {
                    __hip_atomic_store(&a.ctl[64 * (1 + g)], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const uint32_t t2 = __hip_atomic_fetch_add(&a.ctl[0], 1u, kOrder, __HIP_MEMORY_SCOPE_AGENT);
                    is_last = t2 == (uint32_t)(nwg < groups ? nwg : groups) - 1;
                }
            }
            if (is_last) __hip_atomic_store(&a.ctl[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // self-resetting
            last = is_last;
        }
    }
    __syncthreads();
    if (!last) return;
    if (FENCED) __atomic_thread_fence(__ATOMIC_ACQUIRE);
    sync_fold<!FENCED>(a, gridDim.x);
}

// Eq. 4 spread over the grid (2048 / grid entries per workgroup, each a chain of 64 fused multiply-adds), a grid-wide
// barrier on generation tags (every workgroup publishes its tag and polls all of them), then every workgroup loads the
// whole table into LDS.  FENCED: release store / acquire fence around plain accesses; else agent-scope relaxed accesses.
template <bool FENCED>
__global__ __launch_bounds__(kSyncThreads) void sync_eq4_barrier_kernel(SyncArgs a) {
    __shared__ float lut[2048];
    const int per = 2048 / gridDim.x, tid = threadIdx.x;
    if (tid < per) {
        const int e = blockIdx.x * per + tid;
        const float4* c4 = reinterpret_cast<const float4*>(a.cent + (size_t)e * 64);
        const float4* p4 = reinterpret_cast<const float4*>(a.phi + (e / 256) * 64);
        float4 c[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) c[i] = c4[i];
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float4 p = p4[i];
            acc = __builtin_fmaf(c[i].x, p.x, acc); acc = __builtin_fmaf(c[i].y, p.y, acc);
            acc = __builtin_fmaf(c[i].z, p.z, acc); acc = __builtin_fmaf(c[i].w, p.w, acc);
        }
        if (FENCED) a.S[e] = acc;
        else __hip_atomic_store(&a.S[e], acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (FENCED) {
        __syncthreads();
        if (tid == 0) __hip_atomic_store(&a.tags[blockIdx.x], a.gen, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    } else if (tid < 64) {                                    // (the producing lanes are all in wave 0)
        __builtin_amdgcn_s_waitcnt(0);
        if (tid == 0) __hip_atomic_store(&a.tags[blockIdx.x], a.gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    int ok = 0;
    for (int spin = 0; spin < kSyncSpinLimit && !ok; ++spin) {
        bool mine = true;
        if (tid < (int)gridDim.x) mine = __hip_atomic_load(&a.tags[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.gen;
        ok = __syncthreads_and(mine ? 1 : 0);
        if (!ok) __builtin_amdgcn_s_sleep(2);
    }
    if (FENCED) __atomic_thread_fence(__ATOMIC_ACQUIRE);
    for (int e = tid; e < 2048; e += kSyncThreads)
        lut[e] = FENCED ? a.S[e] : __hip_atomic_load(&a.S[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const float s = lut[(tid * 7) & 2047] + lut[(tid * 13 + 5) & 2047];
    if (s == 1234.5f || !ok) a.out[3 + (ok ? 0 : 1)] = tid;   // ([4] counts nothing unless a wait ran out)
}
__global__ __launch_bounds__(64) void sync_eq4_kernel(SyncArgs a) {
    const int e = blockIdx.x * 64 + threadIdx.x;
    const float4* c4 = reinterpret_cast<const float4*>(a.cent + (size_t)e * 64);
    const float4* p4 = reinterpret_cast<const float4*>(a.phi + (e / 256) * 64);
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const float4 c = c4[i], p = p4[i];
        acc = __builtin_fmaf(c.x, p.x, acc); acc = __builtin_fmaf(c.y, p.y, acc);
        acc = __builtin_fmaf(c.z, p.z, acc); acc = __builtin_fmaf(c.w, p.w, acc);
    }
    a.S[e] = acc;
}
__global__ __launch_bounds__(kSyncThreads) void sync_load_table_kernel(SyncArgs a) {
    __shared__ float lut[2048];
    const int tid = threadIdx.x;
    for (int e = tid; e < 2048; e += kSyncThreads) lut[e] = a.S[e];
    __syncthreads();
    const float s = lut[(tid * 7) & 2047] + lut[(tid * 13 + 5) & 2047];
    if (s == 1234.5f) a.out[3] = tid;
}

template <typename Launch>
int time_launches(hipStream_t st, int iters, float* out_ms, Launch&& launch) {
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (hipEventCreate(&ev0) != hipSuccess) return PQ_ERR_HIP;
    if (hipEventCreate(&ev1) != hipSuccess) { (void)hipEventDestroy(ev0); return PQ_ERR_HIP; }
    bool ok = true;
    launch();                                                 // untimed warm-up launch
    ok = ok && hipGetLastError() == hipSuccess;
    ok = ok && hipEventRecord(ev0, st) == hipSuccess;
    for (int it = 0; it < iters && ok; ++it) launch();
    ok = ok && hipGetLastError() == hipSuccess;
    ok = ok && hipEventRecord(ev1, st) == hipSuccess;
    ok = ok && hipStreamSynchronize(st) == hipSuccess;
    float ms = 0.0f;
    ok = ok && hipEventElapsedTime(&ms, ev0, ev1) == hipSuccess;
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    if (!ok) return PQ_ERR_HIP;
    *out_ms = ms / (float)iters;
    return PQ_OK;
}

}  // namespace

extern "C" {

int pq_measure_empty_launch(int blocks, int threads, void* stream, int iters, float* launch_ms) {
    if (!launch_ms) return PQ_ERR_NULL;
    if (blocks < 1 || iters < 1 || threads < 64 || threads > 1024 || threads % 64 != 0) return PQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return time_launches(st, iters, launch_ms, [&]() {
        hipLaunchKernelGGL(empty_kernel, dim3((unsigned)blocks), dim3((unsigned)threads), 0, st, (uint32_t*)nullptr, 0);
    });
}

int pq_measure_lds_gather(int width, int table_bytes, int rounds, int conflict_free, int copies, int blocks, int threads,
                          uint32_t* sink, void* stream, int iters, float* gather_ms) {
    if (!sink || !gather_ms) return PQ_ERR_NULL;
    if (conflict_free) copies = 1;
    if ((width != 4 && width != 8 && width != 16) || table_bytes < 1024 || table_bytes > 131072 ||
        copies < 1 || copies > 64 || (copies & (copies - 1)) != 0 || width * copies * 2 > table_bytes ||
        (table_bytes & (table_bytes - 1)) != 0 || rounds < kGatherOffsets || rounds % kGatherOffsets != 0 || blocks < 1 ||
        iters < 1 || threads < 64 || threads > 1024 || threads % 64 != 0)
        return PQ_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (table_bytes > 64 * 1024) {                           // (measurement aid: the limit is simply raised on every call)
        const int lds = table_bytes;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(lds_gather_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(lds_gather_kernel<8>), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(lds_gather_kernel<16>), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
            return PQ_ERR_HIP;
    }
    return time_launches(st, iters, gather_ms, [&]() {
        const dim3 grid((unsigned)blocks), block((unsigned)threads);
        if (width == 4) hipLaunchKernelGGL(lds_gather_kernel<4>, grid, block, (size_t)table_bytes, st, table_bytes, rounds, conflict_free, copies, sink);
        else if (width == 8) hipLaunchKernelGGL(lds_gather_kernel<8>, grid, block, (size_t)table_bytes, st, table_bytes, rounds, conflict_free, copies, sink);
        else hipLaunchKernelGGL(lds_gather_kernel<16>, grid, block, (size_t)table_bytes, st, table_bytes, rounds, conflict_free, copies, sink);
    });
}

int pq_measure_sync_variant(int variant, void* scratch, size_t scratch_bytes, void* stream, int iters, float* variant_ms) {
    if (!scratch || !variant_ms) return PQ_ERR_NULL;
    if (variant < 0 || variant >= PQ_SYNC_VARIANTS || iters < 1) return PQ_ERR_SHAPE;
    if ((uintptr_t)scratch & 255) return PQ_ERR_ALIGN;
    if (scratch_bytes < PQ_SYNC_SCRATCH_BYTES) return PQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int grid = 256;                                     // one workgroup per CU, as the single-query scan launches
    unsigned char* base = static_cast<unsigned char*>(scratch);
    SyncArgs a;
    size_t off = 0;
    a.ctl = reinterpret_cast<uint32_t*>(base + off);   off += 64 * 64 * sizeof(uint32_t);
    a.tags = reinterpret_cast<uint32_t*>(base + off);  off += 4096 * sizeof(uint32_t);
    a.keys = reinterpret_cast<uint64_t*>(base + off);  off += 4096 * 16 * sizeof(uint64_t);
    a.S = reinterpret_cast<float*>(base + off);        off += 2048 * sizeof(float);
    a.phi = reinterpret_cast<const float*>(base + off); off += 512 * sizeof(float);
    a.out = reinterpret_cast<uint64_t*>(base + off);   off += 64 * sizeof(uint64_t);
    a.cent = reinterpret_cast<const float*>(base + off); off += (size_t)2048 * 64 * sizeof(float);
    static_assert(64 * 64 * 4 + 4096 * 4 + 4096 * 16 * 8 + 2048 * 4 + 512 * 4 + 64 * 8 + 2048 * 64 * 4 <= PQ_SYNC_SCRATCH_BYTES, "scratch layout");
    a.lists = grid;
    if (hipMemsetAsync(scratch, 0, PQ_SYNC_SCRATCH_BYTES, st) != hipSuccess) return PQ_ERR_HIP;   // (measurement aid: never captured)
    uint32_t gen = 0;
    const dim3 g(grid), b(kSyncThreads);
    return time_launches(st, iters, variant_ms, [&]() {
        a.gen = ++gen;
        switch (variant) {
            case PQ_SYNC_EMPTY: hipLaunchKernelGGL(empty_kernel, g, b, 0, st, (uint32_t*)nullptr, 0); break;
            case PQ_SYNC_FOLD_LAUNCH:
                hipLaunchKernelGGL(sync_write_kernel, g, b, 0, st, a);
                hipLaunchKernelGGL(sync_fold_kernel, dim3(1), b, 0, st, a);
                break;
            case PQ_SYNC_LAST_FOLDS_FENCED: hipLaunchKernelGGL((sync_last_folds_kernel<true, 1>), g, b, 0, st, a); break;
            case PQ_SYNC_LAST_FOLDS_RELAXED: hipLaunchKernelGGL((sync_last_folds_kernel<false, 1>), g, b, 0, st, a); break;
            case PQ_SYNC_LAST_FOLDS_RELAXED_2LEVEL: hipLaunchKernelGGL((sync_last_folds_kernel<false, 2>), g, b, 0, st, a); break;
            case PQ_SYNC_EQ4_LAUNCH:
                hipLaunchKernelGGL(sync_eq4_kernel, dim3(32), dim3(64), 0, st, a);
                hipLaunchKernelGGL(sync_load_table_kernel, g, b, 0, st, a);
                break;
            case PQ_SYNC_EQ4_BARRIER_FENCED: hipLaunchKernelGGL(sync_eq4_barrier_kernel<true>, g, b, 0, st, a); break;
            default: hipLaunchKernelGGL(sync_eq4_barrier_kernel<false>, g, b, 0, st, a); break;
        }
    });
}

}  // extern "C"
