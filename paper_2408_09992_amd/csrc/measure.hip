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

}  // extern "C"
