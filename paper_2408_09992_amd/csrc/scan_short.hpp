// Eq. 5 + TopK for catalogues short enough that a workgroup's share fits its registers (scan_short_kernel): the scan of
// every single-query call over up to a few million items with K < 32, the headline workload among them.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

// Most units (16-byte code vectors for m <= 16, items for m = 32 and 64) a thread of the short kernel holds: as many as
// still beat the general kernel (measured at batch 1, K = 10: m = 8, 2.5M items 14.5 -> 12.3 us, at 16 vectors no gain left;
// m = 16, 1.28M items 14.0 -> 11.6 us; m = 32, 700K items 13.9 -> 11.9 us; m = 64, 500K items 15.6 -> 14.4 us, but
// eight items of four vectors each no longer fit the registers; m = 4, 3M items 13.3 -> 11.3 us).
__host__ __device__ constexpr int short_max_units(int m) {
    return m == 1 ? 2 : m == 2 ? 2 : m == 4 ? 6 : m == 8 ? 12 : m == 16 ? 12 : m == 32 ? 8 : 4;
}
// ... with two-byte sub-ids (rows of 8, 16, 32 bytes: m = 4, 8, 16): code vectors, or items of two vectors for m = 16
__host__ __device__ constexpr int short16_max_units(int m) { return m == 16 ? 6 : 12; }

// grid = (item blocks, B); one query per workgroup; a thread holds U units of its workgroup's share: unit u of thread t
// of workgroup g is number (u * blocks + g) * NT + t of the catalogue's units (slot u of all workgroups together is one
// contiguous stretch of G).  The host picks U = ceil(units / (blocks * NT)), so nothing is loaded or looked up in vain
// but the last, ragged slot.  Same lookups and left-to-right sums as scan_topk_kernel (score_vector, score_wide); what
// differs is everything around them: all codes are requested before anything else happens, no lists, no histogram, one
// barrier after the tables' and one in the selection.  This step is all latency (the code matrix is a few
// microseconds of traffic), and a wave's latency is its instruction count: a kernel of its own, a few KB of code.
//   M: splits; CW: bytes per sub-id.  An item's row takes P = M * CW bytes (1, 2, 4, 8, 16: 16 / P items per code vector;
//   32, 64: P / 16 vectors per item).  CW = 2 (M = 4, 8, 16): the query's m x b table lies in dynamic LDS as in memory.
template <int M, int U, int NT, bool STAMP = false, int CW = 1>
__global__ __launch_bounds__(NT) void scan_short_kernel(ScanArgs a) {
    constexpr int NW = NT / kWave;
    constexpr int P = M * CW;
    constexpr int VPU = Round<P>::kVPU, IPV = Round<P>::kIPV;  // vectors per unit, items per unit
    constexpr bool kTail = P < 16 || (CW == 1 && P == 16);     // items after the last whole code vector may exist (a slot is kept for them)
    constexpr int R = U * IPV + (kTail ? 1 : 0);
    static_assert(CW == 1 || CW == 2, "one- or two-byte sub-ids");
    static_assert(U >= 1 && U <= (CW == 1 ? short_max_units(M) : short16_max_units(M)), "units per thread");
    __shared__ __align__(16) float lut_static[CW == 1 ? M * kLutStride : 4];
    extern __shared__ __align__(16) unsigned char smem[];
    float* const lut = CW == 1 ? lut_static : reinterpret_cast<float*>(smem);
    __shared__ SmallSelectLds<NT> sel;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x, blk = blockIdx.x, K = a.K, b = a.b;
    uint64_t* const rec = STAMP ? a.stamps + (((size_t)q * nblk + blk) * NW + wave) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, lane);

    const uint32_t total_units = (uint32_t)(P <= 16 ? (a.N * P) / 16 : a.N);   // whole code vectors (P <= 16) or items; >= 1
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
    if constexpr (CW == 2) {
        // the m x b table as it lies in memory, in 16-byte pieces when its size and address allow
        const int total = M * b;
        fetch_codes();
        if ((total & 3) == 0 && ((uintptr_t)Sq & 15) == 0) {
            const float4* src = reinterpret_cast<const float4*>(Sq);
            float4* dst = reinterpret_cast<float4*>(lut);
#pragma unroll 4
            for (int e = tid; e < (total >> 2); e += NT) dst[e] = src[e];
        } else {
#pragma unroll 4
            for (int e = tid; e < total; e += NT) lut[e] = Sq[e];
        }
    } else if (b == kLutStride && ((uintptr_t)Sq & 15) == 0) {
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
            if constexpr (CW == 2) {
                if constexpr (P > 16) part[0] = score_wide16<M>(lut, b, w[u]);
                else score_vector16<M>(lut, b, w[u], part);
            } else if constexpr (M > 16) part[0] = score_wide<M>(lut, w[u]);
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
                const uint8_t* row = a.codes + (size_t)tail_item * P;
                if constexpr (CW == 2) {
                    const uint16_t* g = reinterpret_cast<const uint16_t*>(row);
                    tail_sc = lut[g[0]];
#pragma unroll
                    for (int k = 1; k < M; ++k) tail_sc = tail_sc + lut[(size_t)k * b + g[k]];
                } else {
                    tail_sc = lut[row[0]];
#pragma unroll
                    for (int k = 1; k < M; ++k) tail_sc = tail_sc + lut[k * kLutStride + row[k]];
                }
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
