// Eq. 5 + TopK for catalogues short enough that a workgroup's share fits its registers (scan_short_kernel): the scan of
// every single-query call over up to a few million items with K < 32, the headline workload among them.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

// Most units (16-byte code vectors for m <= 16, items for m = 32 and 64) a thread of the short kernel holds.
__host__ __device__ constexpr int short_max_units(int m) { return kRing * vec_per_thread(m); }

// grid = (item blocks, B); one query per workgroup; a thread holds U units of its workgroup's share: unit u of thread t
// of workgroup g is number (u * blocks + g) * NT + t of the catalogue's units (slot u of all workgroups together is one
// contiguous stretch of G).  The host picks U = ceil(units / (blocks * NT)), so nothing is loaded or looked up in vain
// but the last, ragged slot.  Same lookups and left-to-right sums as scan_topk_kernel (score_vector, score_wide); what
// differs is everything around them: all codes are requested before anything else happens, no lists, no histogram, one
// barrier after the tables' and one in the selection.  This step is all latency (the code matrix is a few
// microseconds of traffic), and a wave's latency is its instruction count: a kernel of its own, a few KB of code.
//   M: bytes of an item's row (1, 2, 4, 8, 16: 16 / M items per code vector; 32, 64: M / 16 vectors per item)
template <int M, int U, int NT, bool STAMP = false>
__global__ __launch_bounds__(NT) void scan_short_kernel(ScanArgs a) {
    constexpr int NW = NT / kWave;
    constexpr int VPU = Round<M>::kVPU, IPV = Round<M>::kIPV;  // vectors per unit, items per unit
    constexpr bool kTail = M <= 16;                            // items after the last whole code vector exist
    constexpr int R = U * IPV + (kTail ? 1 : 0);
    static_assert(U >= 1 && U <= short_max_units(M), "units per thread");
    __shared__ __align__(16) float lut[M * kLutStride];
    __shared__ SmallSelectLds<NT> sel;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x, blk = blockIdx.x, K = a.K, b = a.b;
    uint64_t* const rec = STAMP ? a.stamps + (((size_t)q * nblk + blk) * NW + wave) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, lane);

    const uint32_t total_units = (uint32_t)(M <= 16 ? (a.N * M) / 16 : a.N);   // whole code vectors (M <= 16) or items; >= 1
    const uint32_t last_unit = total_units - 1;
    const uint32_t first = (uint32_t)blk * NT + (uint32_t)tid, stride = (uint32_t)nblk * NT;   // unit u: first + u * stride

    // ---- table values requested, then all codes, then the tables go to LDS
    uint32_t w[U][4 * VPU];
    auto fetch_codes = [&]() {                                // (branch-free: a unit past the end re-reads the last one)
        const uint4* base = reinterpret_cast<const uint4*>(a.codes);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = min(first + (uint32_t)u * stride, last_unit);
#pragma unroll
            for (int j = 0; j < VPU; ++j) {
                const uint4 x = base[(size_t)v * VPU + j];
                w[u][4 * j] = x.x; w[u][4 * j + 1] = x.y; w[u][4 * j + 2] = x.z; w[u][4 * j + 3] = x.w;
            }
        }
    };
    const float* Sq = a.S + (size_t)q * M * b;
    if (b == kLutStride && ((uintptr_t)Sq & 15) == 0) {
        constexpr int kPieces = M * kLutStride / 4;
        constexpr int kPer = (kPieces + NT - 1) / NT;
        const float4* src = reinterpret_cast<const float4*>(Sq);
        float4 t4[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i)
            t4[i] = (kPieces % NT == 0 || tid + i * NT < kPieces) ? src[tid + i * NT] : make_float4(0, 0, 0, 0);
        fetch_codes();
#pragma unroll
        for (int i = 0; i < kPer; ++i)
            if (kPieces % NT == 0 || tid + i * NT < kPieces) reinterpret_cast<float4*>(lut)[tid + i * NT] = t4[i];
    } else {
        // fewer than 256 sub-ids per split, or a table that is only 4-byte aligned: element by element, rows padded with zeros
        constexpr int kPer = (M * kLutStride + NT - 1) / NT;
        float tv[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = tid + i * NT, k = e / kLutStride, j = e % kLutStride;
            tv[i] = (e < M * kLutStride && j < b) ? Sq[k * b + j] : 0.0f;
        }
        fetch_codes();
#pragma unroll
        for (int i = 0; i < kPer; ++i)
            if (tid + i * NT < M * kLutStride) lut[tid + i * NT] = tv[i];
    }
    small_select_clear<NT>(sel, tid);
    stamp<STAMP>(rec, kStampRequested, lane);
    __syncthreads();
    stamp<STAMP>(rec, kStampTables, lane);
    if constexpr (STAMP) {
        __builtin_amdgcn_s_waitcnt(0);                        // every outstanding load: the codes are here
        stamp<STAMP>(rec, kStampCodes, lane);
    }

    // ---- Eq. 5 for everything this thread holds.  Only the last slot can reach past the end (the host's choice of U
    // makes slots 0 .. U-2 whole); what it holds there is nothing
    float sc[R];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool have = u < U - 1 || first + (uint32_t)u * stride < total_units;
        float part[IPV];
        if (u < U - 1 || __ballot(have) != 0) {               // (a wave wholly past the end looks nothing up)
            if constexpr (M > 16) part[0] = score_wide<M>(lut, w[u]);
            else score_vector<M, 1>(lut, w[u], part);
        } else {
#pragma unroll
            for (int e = 0; e < IPV; ++e) part[e] = 0.0f;
        }
#pragma unroll
        for (int e = 0; e < IPV; ++e) sc[u * IPV + e] = have ? part[e] : empty_score();
    }
    if constexpr (kTail) {
        // the fewer than 16 / M items after the last whole code vector: one per lane of the first wave of block 0
        float tail_sc = empty_score();
        if (blk == 0 && wave == 0) {
            const uint32_t tail_item = total_units * IPV + lane;
            if (tail_item < (uint32_t)a.N) {
                const uint8_t* row = a.codes + (size_t)tail_item * M;
                tail_sc = lut[row[0]];
#pragma unroll
                for (int k = 1; k < M; ++k) tail_sc = tail_sc + lut[k * kLutStride + row[k]];
            }
        }
        sc[R - 1] = tail_sc;
    }
    stamp<STAMP>(rec, kStampScored, lane);

    // ---- the workgroup's K best, ranked, straight to the workspace
    uint64_t* const mine_out = a.ws_keys + ((size_t)q * nblk + blk) * K;
    auto id_of = [&](int slot) -> uint32_t {
        if (kTail && slot == R - 1) return total_units * IPV + (uint32_t)lane;
        return (first + (uint32_t)(slot / IPV) * stride) * IPV + (uint32_t)(slot % IPV);
    };
    select_small_k<NT, R, STAMP>(sc, id_of, K, sel, tid, [&](int rank, uint64_t key) { mine_out[rank] = key; }, rec);
    stamp<STAMP>(rec, kStampEnd, lane);
}
