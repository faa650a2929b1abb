// Eq. 5 + TopK for one query per workgroup (scan_topk_kernel): the catalogue scan of pq_score_topk and pq_score_topk_subset.
// Part of kernels.hpp, which includes these parts inside namespace pqk in this order:
// common.hpp, subitem_scores.hpp, topk_parts.hpp, select_small.hpp, scan_single.hpp, scan_short.hpp, scan_subset.hpp, scan_batched.hpp,
// fold.hpp, comparison.hpp.
#pragma once

struct ScanArgs {
    const uint8_t* codes;
    const float* S;
    long long N;
    int m, b, K;
    int cap;             // keys per wave list (power of two >= K + 64)
    int candmax;         // keys of the exact-selection candidate array
    int prune_at;        // wave list length that triggers a tightening (0: only when full)
    uint64_t* ws_keys;   // [B][nblk][K]
    const int* subset;   // candidate list V (generic kernel only): unit p stands for item subset[p]; nullptr: V = I
    uint32_t n_items;    // items in the catalogue (bounds the ids read from `subset`)
    uint64_t* stamps;    // STAMP instances only: wall-clock stamps, kStampSlots per wave (slot names: StampSlot)
};

// Items a thread holds per round.  M > 0: an item's row of sub-ids takes M bytes (m sub-ids of one byte, or m / 2 of
// two bytes) and one 16-byte vector carries 16/M items; M == 0: any row, one item per slot, row loads sized by the
// row's alignment.
template <int M>
struct Round {
    static constexpr int kUnitsPerThread = M ? vec_per_thread(M) : kGenericItemsPerThread;   // lane-sized units of work
    static constexpr int kVPU = M > 16 ? M / 16 : 1;                                     // 16-byte vectors per unit
    static constexpr int kIPV = (M && M <= 16) ? 16 / M : 1;                             // items per unit
    static constexpr int kVecs = M ? kUnitsPerThread * kVPU : 0;                         // 16-byte loads per round
    static constexpr int kItems = kUnitsPerThread * kIPV;
    static constexpr int kWords = M ? kVecs * 4 : 1;
};

// Eq. 5 for the 16/M items packed in one 16-byte vector (words w[0..3], little-endian): all 16 table reads are
// issued before any sum so they overlap in the LDS pipeline, then each item sums its m values left to right.
// A sum of -0 is left as it is here; it is turned into +0 where a key is made.
// With C > 1 the tables are replicated: entry e of the table array has C copies at words e * C .. e * C + C - 1 and
// `lut` already points at this lane's copy (lane % C), so lanes with different copies never share an LDS bank.
template <int M, int C = 1>
__device__ __forceinline__ void score_vector(const float* lut, const uint32_t* w, float* sc) {
    float v[16];
#pragma unroll
    for (int byte = 0; byte < 16; ++byte) {
        const uint32_t code = (w[byte >> 2] >> ((byte & 3) * 8)) & 0xFFu;
        v[byte] = lut[((byte % M) * kLutStride + code) * C];
    }
    __builtin_amdgcn_sched_barrier(0);                // keep the 16 reads ahead of the sums
#pragma unroll
    for (int e = 0; e < 16 / M; ++e) {
        float acc = v[e * M];
#pragma unroll
        for (int k = 1; k < M; ++k) acc = acc + v[e * M + k];
        sc[e] = acc;
    }
}

// Eq. 5 for one item of M = 32 or 64 sub-ids (M/16 vectors, words w[0 .. M/4)): one left-to-right chain over all M
// values; the 16 table reads of a vector are issued together.
template <int M>
__device__ __forceinline__ float score_wide(const float* lut, const uint32_t* w) {
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < M / 16; ++j) {
        float v[16];
#pragma unroll
        for (int byte = 0; byte < 16; ++byte) {
            const uint32_t code = (w[4 * j + (byte >> 2)] >> ((byte & 3) * 8)) & 0xFFu;
            v[byte] = lut[(j * 16 + byte) * kLutStride + code];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int byte = 0; byte < 16; ++byte) acc = (j == 0 && byte == 0) ? v[0] : acc + v[byte];
    }
    return acc;
}

__device__ float score_row(const float* lut, const uint8_t* row, int m) {
    float acc = 0.0f;
    if ((m & 15) == 0) {
        const uint4* p = reinterpret_cast<const uint4*>(row);
        for (int v = 0; v < (m >> 4); ++v) {
            uint4 x = p[v];
            uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                float t = lut[(v * 16 + k) * kLutStride + ((w[k >> 2] >> ((k & 3) * 8)) & 0xFFu)];
                acc = (v == 0 && k == 0) ? t : acc + t;
            }
        }
    } else if ((m & 3) == 0) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(row);
        for (int v = 0; v < (m >> 2); ++v) {
            uint32_t w = p[v];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float t = lut[(v * 4 + k) * kLutStride + ((w >> (k * 8)) & 0xFFu)];
                acc = (v == 0 && k == 0) ? t : acc + t;
            }
        }
    } else {
        // rows that start at any byte: the aligned words covering the row are read (every one of them holds at least
        // one byte of the row, so none lies outside the matrix) and realigned two at a time
        const uintptr_t addr = reinterpret_cast<uintptr_t>(row);
        const uint32_t* p = reinterpret_cast<const uint32_t*>(addr & ~(uintptr_t)3);
        const uint32_t off = (uint32_t)(addr & 3);
        const int last_word = (int)((off + (uint32_t)m - 1) >> 2);
        uint32_t cur = p[0];
        const int full = m >> 2;
        for (int v = 0; v <= full; ++v) {                     // the last trip takes the m % 4 bytes left over
            const uint32_t nxt = (v + 1 <= last_word) ? p[v + 1] : 0u;
            const uint32_t w = __builtin_amdgcn_alignbyte(nxt, cur, off);       // bytes off .. off + 3 of nxt:cur
            const int nbytes = v < full ? 4 : (m & 3);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (k < nbytes) {
                    const float t = lut[(v * 4 + k) * kLutStride + ((w >> (k * 8)) & 0xFFu)];
                    acc = (v == 0 && k == 0) ? t : acc + t;
                }
            }
            cur = nxt;
        }
    }
    return acc;
}

// ---- sub-ids of two bytes (alphabets of up to 65536 sub-ids per split): tables of `stride` = b entries per split

// Eq. 5 for the 8/M items packed in one 16-byte vector of 16-bit sub-ids (M = 1, 2, 4 or 8 splits).
// GL: the tables are read from device memory (they do not fit LDS); a sub-id is then clamped to b - 1, so that no
// value of a code can reach outside the table.
template <int M, bool GL = false>
__device__ __forceinline__ void score_vector16(const float* lut, int stride, const uint32_t* w, float* sc) {
    float v[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        uint32_t code = (h & 1) ? (w[h >> 1] >> 16) : (w[h >> 1] & 0xFFFFu);
        if constexpr (GL) code = code < (uint32_t)stride ? code : (uint32_t)stride - 1u;
        v[h] = lut[(h % M) * stride + code];
    }
    __builtin_amdgcn_sched_barrier(0);                // keep the reads ahead of the sums
#pragma unroll
    for (int e = 0; e < 8 / M; ++e) {
        float acc = v[e * M];
#pragma unroll
        for (int k = 1; k < M; ++k) acc = acc + v[e * M + k];
        sc[e] = acc;
    }
}

// Eq. 5 for one item of M = 16 or 32 sub-ids of 16 bits (M/8 vectors): one left-to-right chain over all M values.
template <int M, bool GL = false>
__device__ __forceinline__ float score_wide16(const float* lut, int stride, const uint32_t* w) {
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < M / 8; ++j) {
        float v[8];
#pragma unroll
        for (int h = 0; h < 8; ++h) {
            const uint32_t word = w[4 * j + (h >> 1)];
            uint32_t code = (h & 1) ? (word >> 16) : (word & 0xFFFFu);
            if constexpr (GL) code = code < (uint32_t)stride ? code : (uint32_t)stride - 1u;
            v[h] = lut[(j * 8 + h) * stride + code];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int h = 0; h < 8; ++h) acc = (j == 0 && h == 0) ? v[0] : acc + v[h];
    }
    return acc;
}

// Eq. 5 for one row of m 16-bit sub-ids that starts at any even address.
template <bool GL = false>
__device__ float score_row16(const float* lut, int stride, const uint8_t* row, int m) {
    float acc = 0.0f;
    auto at = [&](uint32_t code) { return GL ? (code < (uint32_t)stride ? code : (uint32_t)stride - 1u) : code; };
    if ((m & 7) == 0) {
        const uint4* p = reinterpret_cast<const uint4*>(row);
        for (int v = 0; v < (m >> 3); ++v) {
            const uint4 x = p[v];
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int h = 0; h < 8; ++h) {
                const uint32_t code = at((h & 1) ? (w[h >> 1] >> 16) : (w[h >> 1] & 0xFFFFu));
                const float t = lut[(v * 8 + h) * stride + code];
                acc = (v == 0 && h == 0) ? t : acc + t;
            }
        }
    } else if ((m & 1) == 0) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(row);
        for (int v = 0; v < (m >> 1); ++v) {
            const uint32_t w = p[v];
            const float t0 = lut[(2 * v) * stride + at(w & 0xFFFFu)];
            const float t1 = lut[(2 * v + 1) * stride + at(w >> 16)];
            acc = (v == 0) ? t0 : acc + t0;
            acc = acc + t1;
        }
    } else {
        const uint16_t* g = reinterpret_cast<const uint16_t*>(row);
        for (int k = 0; k < m; ++k) {
            const float t = lut[k * stride + at(g[k])];
            acc = (k == 0) ? t : acc + t;
        }
    }
    return acc;
}

// Unit (code vector, or item in the generic kernel) that thread `tid` of workgroup `blk` owns in slot u of its
// round rr: ((rr * kUnits + u) * nblk + blk) * NT + tid.  Slot u of one round of all workgroups together is one
// contiguous stretch of the catalogue, so the grid sweeps memory front to back.  32-bit arithmetic: there are fewer
// than 2^31 units (N < 2^31, m <= 16 in the vector kernels) and the few rounds a kernel reaches past the end add
// less than 2^24 to that, so nothing wraps.
template <int M, int NT>
__device__ __forceinline__ uint32_t unit_of(uint32_t rr, int u, int nblk, int blk, int tid) {
    return ((rr * Round<M>::kUnitsPerThread + u) * (uint32_t)nblk + (uint32_t)blk) * NT + (uint32_t)tid;
}

// The code vectors this thread owns in round rr (vector kernels only).  Always the same number of plain 16-byte
// loads, with the vector index clamped to `last_vec` (the last vector that lies wholly inside the catalogue): no
// branch, so the compiler knows how many loads are outstanding at any point and lets several rounds stay in
// flight.  A clamped vector's items are masked out by the caller.
template <int M, int NT = kThreads>
__device__ __forceinline__ void load_round(const ScanArgs& a, uint32_t rr, int nblk, int blk, uint32_t last_vec,
                                           uint32_t spare_vec, int tid, uint32_t (&w)[Round<M>::kWords]) {
    if constexpr (M > 0) {
        const uint4* base = reinterpret_cast<const uint4*>(a.codes);
        constexpr int VPU = Round<M>::kVPU;
#pragma unroll
        for (int u = 0; u < Round<M>::kUnitsPerThread; ++u) {
            uint32_t v = unit_of<M, NT>(rr, u, nblk, blk, tid);
            v = v <= last_vec ? v : spare_vec;
#pragma unroll
            for (int j = 0; j < VPU; ++j) {
                const uint4 x = base[(size_t)v * VPU + j];
                const int o = 4 * (u * VPU + j);
                w[o] = x.x; w[o + 1] = x.y; w[o + 2] = x.z; w[o + 3] = x.w;
            }
        }
    }
}

// Scores of the items this thread owns in that round (slots past the catalogue's end get arbitrary finite values).
// `inside`: the round lies wholly inside the scanned units (n_units of them); otherwise vectors past the end are not
// looked up at all (a wave whose lanes are all past the end skips the vector's table reads).
// M: splits (0: any, at run time); CW: bytes per sub-id; `stride`: table entries per split in LDS.
template <int M, int C = 1, int NT = kThreads, int CW = 1, bool GL = false>
__device__ __forceinline__ void score_round(const ScanArgs& a, const float* lut, int stride, uint32_t rr, int nblk, int blk,
                                            int tid, bool inside, uint32_t n_units,
                                            const uint32_t (&w)[Round<M * CW>::kWords], float (&sc)[Round<M * CW>::kItems]) {
    constexpr int P = M * CW;                                  // bytes of an item's row
    if constexpr (M > 0) {
#pragma unroll
        for (int u = 0; u < Round<P>::kUnitsPerThread; ++u) {
            if (inside || unit_of<P, NT>(rr, u, nblk, blk, tid) < n_units) {
                if constexpr (CW == 2) {
                    if constexpr (P > 16) sc[u] = score_wide16<M, GL>(lut, stride, &w[4 * Round<P>::kVPU * u]);
                    else score_vector16<M, GL>(lut, stride, &w[4 * u], &sc[u * Round<P>::kIPV]);
                } else {
                    if constexpr (M > 16) sc[u] = score_wide<M>(lut, &w[4 * Round<M>::kVPU * u]);
                    else score_vector<M, C>(lut, &w[4 * u], &sc[u * Round<M>::kIPV]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < Round<P>::kIPV; ++e) sc[u * Round<P>::kIPV + e] = 0.0f;
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < kGenericItemsPerThread; ++u) {
            const uint32_t unit = unit_of<M, NT>(rr, u, nblk, blk, tid);
            float v = 0.0f;
            if (unit < n_units) {
                uint32_t item = unit;
                if (a.subset) {                                // an id past the catalogue is clamped: never out of bounds
                    item = (uint32_t)a.subset[unit];
                    item = item < a.n_items ? item : a.n_items - 1;
                }
                if constexpr (CW == 2) v = score_row16<GL>(lut, stride, a.codes + (size_t)item * a.m * 2, a.m);
                else v = score_row(lut, a.codes + (size_t)item * a.m, a.m);
            }
            sc[u] = v;
        }
    }
}

// Id of the item in slot e of this thread's round (may lie past the scanned items in the last round).
template <int M, int NT = kThreads>
__device__ __forceinline__ uint32_t item_of_slot(uint32_t rr, int nblk, int blk, int tid, int e) {
    constexpr int IPV = Round<M>::kIPV;
    return unit_of<M, NT>(rr, e / IPV, nblk, blk, tid) * IPV + (e % IPV);
}

// Catalogue scan: grid = (item blocks, B).  Leaves each workgroup's exact, sorted K best keys in the workspace.
// LDS: the score tables are a static array when m is a template value (their address is then a compile-time
// constant, which lets sub-id extraction and address arithmetic fold into one instruction per lookup); the rest is
// dynamic: [tables if M == 0] | hist | ctl | wave lists | cand | sorted.
// C > 1 (long single-query scans): C copies of the tables, in dynamic LDS, cut the bank conflicts of the lookups.
// CW: bytes per sub-id.  CW = 2 (alphabets of up to 65536 sub-ids per split): rows of m 16-bit sub-ids, the m x b
// table in dynamic LDS as it lies in memory (b entries per split); the vector instances are those whose rows take
// 8, 16 or 32 bytes (m = 4, 8, 16).
// GL (two-byte sub-ids only): the m x b table does not fit LDS and is read where it lies, in device memory (L2).
// STAMP: measurement instance that also records wall-clock stamps per wave (and waits for the first rounds' codes
// before scoring, so that waiting and scoring can be told apart).
template <int M, int C = 1, int NT = kThreads, int CW = 1, bool GL = false, bool STAMP = false>
__global__ __launch_bounds__(NT, 4) void scan_topk_kernel(ScanArgs a) {
    constexpr int NW = NT / kWave;
    constexpr int P = M * CW;                                  // bytes of an item's row (0: known at run time only)
    constexpr bool kStaticLut = M && C == 1 && CW == 1;
    static_assert(C == 1 || (M > 0 && CW == 1), "replicated tables need a compile-time m and one-byte sub-ids");
    static_assert(!GL || CW == 2, "tables in device memory: two-byte sub-ids only");
    __shared__ __align__(16) float lut_static[kStaticLut ? M * kLutStride : 4];
    extern __shared__ __align__(16) unsigned char smem[];
    const int m = M ? M : a.m;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int q = blockIdx.y, nblk = gridDim.x, K = a.K, b = a.b;
    const int stride = CW == 1 ? kLutStride : b;               // table entries per split in LDS
    const ScanLds L = carve_scan(smem, (kStaticLut || GL) ? 0 : (size_t)m * stride * C, a.cap, a.candmax, NW);
    float* const lut_base = kStaticLut ? lut_static : L.lut;
    Ctl* ctl = L.ctl;
    constexpr int kItems = Round<P>::kItems;
    constexpr int kUnits = Round<P>::kUnitsPerThread;
    constexpr int kWords = Round<P>::kWords;
    uint64_t* const rec = STAMP ? a.stamps + (((size_t)q * nblk + blockIdx.x) * NW + wave) * kStampSlots : nullptr;
    stamp<STAMP>(rec, kStampEntry, lane);

    // Vector kernels scan the code vectors that lie wholly inside the catalogue; the fewer than 16 / M items after
    // them (when N * M is not a multiple of 16) are scored one by one at the end.  The generic kernel scans items.
    const uint32_t total_units = (uint32_t)((P && P <= 16) ? (a.N * P) / 16 : a.N);
    const uint32_t n_scan = M ? total_units * Round<P>::kIPV : total_units;   // items the rounds cover
    const uint32_t last_vec = total_units - 1;                                // (total_units >= 1: the host sees to it)
    const uint32_t round_units = (uint32_t)NT * kUnits * nblk;                // units all workgroups take per round
    const uint32_t rounds = (total_units + round_units - 1) / round_units;    // every workgroup runs them all
    const uint32_t inside_rounds = total_units / round_units;                 // rounds with no ragged end

    // ---- 1. the first kRing rounds' codes on their way, then the query's table into LDS
    uint32_t r = 0;
    const int blk = blockIdx.x;
    uint32_t w[kRing][kWords];
    // (vt: the thread index whose share of round rr is meant; a wave may take over another wave's share)
    // (loads past the end go to a line of this wave's own instead of all to the last one: no single hot line when
    // thousands of waves reach the end of their scan together)
    const uint32_t own_vec = (uint32_t)(blk * NW + wave) * 4u;
    const uint32_t spare_vec = own_vec < last_vec ? own_vec : last_vec;
    auto fetch = [&](uint32_t rr, int vt, uint32_t (&buf)[kWords]) {
        load_round<P, NT>(a, rr, nblk, blk, last_vec, spare_vec, vt, buf);
    };
    // (the host sends catalogues with no whole code vector, N * M < 16, to the generic kernel: rounds >= 1 here)
    auto fetch_first = [&]() {                                // no branch: the loads can be counted, so what follows
#pragma unroll                                                // waits for exactly what it needs
        for (int i = 0; i < kRing; ++i) fetch(r + i, tid, w[i]);
    };
    const float* Sq = a.S + (size_t)q * m * b;
    if constexpr (GL) {
        fetch_first();                                        // (nothing to fill: lookups go to memory)
    } else if constexpr (CW == 2) {
        // the query's m x b table as it lies in memory, in 16-byte pieces when its size and address allow
        const int total = m * b;
        fetch_first();
        if ((total & 3) == 0 && ((uintptr_t)Sq & 15) == 0) {
            const float4* src = reinterpret_cast<const float4*>(Sq);
            float4* dst = reinterpret_cast<float4*>(lut_base);
#pragma unroll 4
            for (int e = tid; e < (total >> 2); e += NT) dst[e] = src[e];
        } else {
#pragma unroll 4
            for (int e = tid; e < total; e += NT) lut_base[e] = Sq[e];
        }
    } else if constexpr (C > 1) {
        // thread t writes the 16-byte pieces t, t + NT, ... of the replicated tables (piece p is a quarter of the C
        // copies of entry p / (C / 4)): consecutive lanes write consecutive LDS addresses.  Values requested first.
        constexpr int kPieces = M * kLutStride * (C / 4);
        constexpr int kPer = (kPieces + NT - 1) / NT;
        float tv[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = (tid + i * NT) / (C / 4), k = e / kLutStride, j = e % kLutStride;
            tv[i] = (e < M * kLutStride && j < b) ? Sq[k * b + j] : 0.0f;
        }
        fetch_first();
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int piece = tid + i * NT;
            if (piece < kPieces) reinterpret_cast<float4*>(lut_base)[piece] = make_float4(tv[i], tv[i], tv[i], tv[i]);
        }
    } else if (b == kLutStride && ((uintptr_t)Sq & 15) == 0) {
        // b = 256: the query's table is copied as it is, in 16-byte pieces, all requested before the first is stored
        const float4* src = reinterpret_cast<const float4*>(Sq);
        float4* dst = reinterpret_cast<float4*>(lut_base);
        if constexpr (M > 0) {
            constexpr int kPieces = M * kLutStride / 4;
            constexpr int kPer = (kPieces + NT - 1) / NT;
            float4 t4[kPer];
#pragma unroll
            for (int i = 0; i < kPer; ++i)
                t4[i] = (kPieces % NT == 0 || tid + i * NT < kPieces) ? src[tid + i * NT] : make_float4(0, 0, 0, 0);
            fetch_first();
#pragma unroll
            for (int i = 0; i < kPer; ++i)
                if (kPieces % NT == 0 || tid + i * NT < kPieces) dst[tid + i * NT] = t4[i];
        } else {
            fetch_first();
#pragma unroll 4
            for (int e = tid; e < m * (kLutStride / 4); e += NT) dst[e] = src[e];
        }
    } else if constexpr (M > 0) {
        // fewer than 256 sub-ids per split (or a table that is not 16-byte aligned): element by element, rows padded
        // with zeros to 256 entries; all values requested before the first is stored
        constexpr int kPer = (M * kLutStride + NT - 1) / NT;
        float tv[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int e = tid + i * NT, k = e / kLutStride, j = e % kLutStride;
            tv[i] = (e < M * kLutStride && j < b) ? Sq[k * b + j] : 0.0f;
        }
        fetch_first();
#pragma unroll
        for (int i = 0; i < kPer; ++i)
            if (tid + i * NT < M * kLutStride) lut_base[tid + i * NT] = tv[i];
    } else {
        fetch_first();
#pragma unroll 4
        for (int e = tid; e < m * kLutStride; e += NT) {
            int k = e / kLutStride, j = e % kLutStride;
            lut_base[e] = (j < b) ? Sq[k * b + j] : 0.0f;
        }
    }
    for (int i = tid; i < kBins; i += NT) L.hist[i] = 0;
    if (tid == 0) { ctl->next_unit = kRing * NW; ctl->shared_floor = -__builtin_inff(); ctl->ncand = 0; }
    stamp<STAMP>(rec, kStampRequested, lane);
    __syncthreads();
    stamp<STAMP>(rec, kStampTables, lane);
    if constexpr (STAMP) {
        __builtin_amdgcn_s_waitcnt(0);                        // every outstanding load: the first rounds' codes are here
        stamp<STAMP>(rec, kStampCodes, lane);
    }
    const float* const lut = [&]() -> const float* {
        if constexpr (GL) return Sq;
        else return lut_base + (C > 1 ? lane % C : 0);        // this lane's copy
    }();

    WaveTopK top{L.lists + (size_t)wave * a.cap, a.cap, K, a.prune_at, 0, 0ull, -__builtin_inff()};

    // item id of a scanned unit (they differ only under a candidate list)
    auto id_of = [&](uint32_t unit) -> uint32_t {
        if constexpr (M == 0) {
            if (a.subset) {
                const uint32_t item = (uint32_t)a.subset[unit];
                return item < a.n_items ? item : a.n_items - 1;
            }
        }
        return unit;
    };
    // In scans of several rounds the waves share a workgroup-wide floor: the first round's histogram
    // lives on, every score appended to a list is counted in it, and the waves take turns deriving the floor it
    // allows (at least K counted scores lie above it).  A wave alone sees a sixteenth of the workgroup's items and
    // its own K-th best is a far lower floor: with K = 100 nearly every round of a long scan would offer something.
    // (In a scan of a few rounds the floor has no time to pay for its counting: 5 % slower at two rounds; a larger K
    // pays it back sooner: K = 100 on 10M items, five rounds, 35 -> 28 us.)
    // (`prune_at`: another kernel that shares these lists cuts them back early instead; never set for this one.)
    const bool wide_floor = a.prune_at == 0 && rounds >= (uint32_t)(K >= 32 ? kSharedFloorMinRoundsLargeK : kSharedFloorMinRounds);
    float hlo = 0.0f, hscale = 0.0f;                          // the histogram's range (set in the first round)
    int turn = wave, gap = NW;                                // units until this wave's next turn; grows by a quarter
    // what a round's scores offer to the wave's list: everything at or above its floor
    auto offer = [&](const float (&sc)[kItems], uint32_t rr, int vt) {
        if (wide_floor) {
            top.floor_ge = fmaxf(top.floor_ge, lds_peek(&ctl->shared_floor));
            if (--turn < 0) {
                gap += gap >> 2;
                turn = gap;
                const float f = floor_of_hist<kBins>(L.hist, K, hlo, hscale, lane);
                if (lane == 0 && f > lds_peek(&ctl->shared_floor)) lds_poke(&ctl->shared_floor, f);   // (a racing lower store is still a floor)
                top.floor_ge = fmaxf(top.floor_ge, f);
            }
        }
        float best = sc[0];
#pragma unroll
        for (int e = 1; e < kItems; ++e) best = fmaxf(best, sc[e]);
        if (__ballot(best >= top.floor_ge) == 0) return;      // nothing in this round can matter
        const bool inside = rr < inside_rounds;
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const uint32_t item = item_of_slot<P, NT>(rr, nblk, blk, vt, e);
            const bool take = sc[e] >= top.floor_ge && (inside || item < n_scan);
            const uint64_t mask = __ballot(take);
            if (mask != 0) {
                if (wide_floor && take) atomicAdd(&L.hist[bucket_of(sc[e], hlo, hscale)], 1u);
                top.append(mask, take, sc[e], take ? id_of(item) : 0u, lane);
            }
        }
        if (top.prune_at != 0 && top.cnt >= top.prune_at) top.tighten(lane);
    };
    // one streamed round
    auto process = [&](const uint32_t (&w)[kWords], uint32_t rr, int vt) {
        float sc[kItems];
        score_round<M, C, NT, CW, GL>(a, lut, stride, rr, nblk, blk, vt, rr < inside_rounds, total_units, w, sc);
        offer(sc, rr, vt);
    };

    // ---- 1b. a scan of at most two rounds (every catalogue up to a few million items at batch 1): both rounds' codes
    // are already loaded, so all of the workgroup's scores fit its registers and are selected from there, without the
    // per-wave lists and their merge.
    //   K < 32: every wave finds a floor that K of its lanes' best scores reach (wave operations only), compacts the
    //   dozen or so scores at or above it into the shared candidate array, and after one barrier the workgroup ranks
    //   them all by counting (three barriers in all, against six of the general path).
    //   K >= 32: one selection by the whole workgroup - range, histogram, cut, the few keys at or above the cut ranked
    //   by counting (1.28M items: K = 100 10.1 -> 9.0 us, K = 512 23.0 -> 18.3 us).
    // Heavy ties (more candidates than the array holds) fall through to the general path below, which starts over
    // from the codes.
    bool done = false;
    if (rounds <= (uint32_t)kRing) {
        float sc2[kRing][kItems];
        bool ok2[kRing][kItems];
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int i = 0; i < kRing; ++i) {
            if ((uint32_t)i < rounds) {
                score_round<M, C, NT, CW, GL>(a, lut, stride, i, nblk, blk, tid, (uint32_t)i < inside_rounds, total_units, w[i], sc2[i]);
#pragma unroll
                for (int e = 0; e < kItems; ++e) {
                    ok2[i][e] = (uint32_t)i < inside_rounds || item_of_slot<P, NT>(i, nblk, blk, tid, e) < n_scan;
                    if (ok2[i][e]) { mn = fminf(mn, sc2[i][e]); mx = fmaxf(mx, sc2[i][e]); }
                }
            } else {
#pragma unroll
                for (int e = 0; e < kItems; ++e) { sc2[i][e] = 0.0f; ok2[i][e] = false; }
            }
        }
        // the fewer than 16 / P items after the last whole code vector: one per lane of the first wave of block 0
        float tail_sc = 0.0f;
        bool tail_ok = false;
        uint32_t tail_item = 0;
        if constexpr (P > 0 && P <= 16) {
            if (blockIdx.x == 0 && wave == 0) {
                tail_item = n_scan + lane;
                if (tail_item < (uint32_t)a.N) {
                    const uint8_t* row = a.codes + (size_t)tail_item * P;
                    if constexpr (CW == 2) {
                        const uint16_t* g = reinterpret_cast<const uint16_t*>(row);
                        auto at = [&](uint32_t code) { return GL ? (code < (uint32_t)stride ? code : (uint32_t)stride - 1u) : code; };
                        tail_sc = lut[at(g[0])];
#pragma unroll
                        for (int k = 1; k < M; ++k) tail_sc = tail_sc + lut[(size_t)k * stride + at(g[k])];
                    } else {
                        tail_sc = lut[(size_t)row[0] * C];
#pragma unroll
                        for (int k = 1; k < M; ++k) tail_sc = tail_sc + lut[((size_t)k * kLutStride + row[k]) * C];
                    }
                    tail_ok = true;
                    mn = fminf(mn, tail_sc); mx = fmaxf(mx, tail_sc);
                }
            }
        }
        stamp<STAMP>(rec, kStampScored, lane);
        int ncand = 0;
        if (K < kRegisterSelectMinK) {
            // (mx: the lane's best score, -inf if it holds no item; at least K of the wave's items reach the floor, and
            // so does every one of the wave's K best)
            const float f = wave_floor_for_k(mx, K);
            uint64_t masks[kRing * kItems + 1];
            int cnt = 0;
#pragma unroll
            for (int i = 0; i < kRing; ++i)
#pragma unroll
                for (int e = 0; e < kItems; ++e) {
                    masks[i * kItems + e] = __ballot(ok2[i][e] && sc2[i][e] >= f);
                    cnt += __popcll(masks[i * kItems + e]);
                }
            masks[kRing * kItems] = __ballot(tail_ok && tail_sc >= f);
            cnt += __popcll(masks[kRing * kItems]);
            int base = 0;
            if (lane == 0 && cnt != 0) base = atomicAdd(&ctl->ncand, cnt);
            base = __builtin_amdgcn_readfirstlane(base);
            const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
            for (int i = 0; i < kRing; ++i)
#pragma unroll
                for (int e = 0; e < kItems; ++e) {
                    const uint64_t mk = masks[i * kItems + e];
                    if (mk == 0) continue;
                    const int pos = base + __popcll(mk & below);
                    if (((mk >> lane) & 1ull) && pos < a.candmax)
                        L.cand[pos] = make_key(sc2[i][e] + 0.0f, id_of(item_of_slot<P, NT>(i, nblk, blk, tid, e)));
                    base += __popcll(mk);
                }
            {
                const uint64_t mk = masks[kRing * kItems];
                const int pos = base + __popcll(mk & below);
                if (((mk >> lane) & 1ull) && pos < a.candmax) L.cand[pos] = make_key(tail_sc + 0.0f, id_of(tail_item));
            }
            stamp<STAMP>(rec, kStampOffered, lane);
            __syncthreads();
            ncand = ctl->ncand;
        } else {
            float lo, scale;
            set_range<NW>(mn, mx, ctl, tid, lo, scale);
#pragma unroll
            for (int i = 0; i < kRing; ++i)
#pragma unroll
                for (int e = 0; e < kItems; ++e)
                    if (ok2[i][e]) atomicAdd(&L.hist[bucket_of(sc2[i][e], lo, scale)], 1u);
            if (tail_ok) atomicAdd(&L.hist[bucket_of(tail_sc, lo, scale)], 1u);
            __syncthreads();
            if (tid < kWave) find_cut(L.hist, K, ctl, lane);
            __syncthreads();
            const int bstar = ctl->bstar;
            auto collect = [&](float score, uint32_t item) {      // few threads get here: a counter update each
                const int pos = atomicAdd(&ctl->ncand, 1);
                if (pos < a.candmax) L.cand[pos] = make_key(score + 0.0f, id_of(item));
            };
#pragma unroll
            for (int i = 0; i < kRing; ++i)
#pragma unroll
                for (int e = 0; e < kItems; ++e)
                    if (ok2[i][e] && bucket_of(sc2[i][e], lo, scale) >= bstar) collect(sc2[i][e], item_of_slot<P, NT>(i, nblk, blk, tid, e));
            if (tail_ok && bucket_of(tail_sc, lo, scale) >= bstar) collect(tail_sc, tail_item);
            __syncthreads();
            ncand = ctl->ncand;
            if (ncand > a.candmax) {
                for (int i = tid; i < kBins; i += NT) L.hist[i] = 0;   // (the general path starts from an empty histogram)
            }
        }
        if (!done) {
            if (ncand <= a.candmax) {
                rank_select<NT>(L.cand, ncand, K, L.sorted, tid);
                done = true;
            } else {
                __syncthreads();                                  // start over with the general path
            }
        }
    }

    if (!done) {
    {
        // ---- 2. first round: scores in registers, histogram over their range, cut
        float sc[kItems];
        score_round<M, C, NT, CW, GL>(a, lut, stride, r, nblk, blk, tid, r < inside_rounds, total_units, w[0], sc);
        stamp<STAMP>(rec, kStampScored, lane);
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int e = 0; e < kItems; ++e)
            if (item_of_slot<P, NT>(r, nblk, blk, tid, e) < n_scan) { mn = fminf(mn, sc[e]); mx = fmaxf(mx, sc[e]); }
        float lo, scale;
        set_range<NW>(mn, mx, ctl, tid, lo, scale, wide_floor ? 1.25f : 1.0f);
        hlo = lo;
        hscale = scale;
        int bk[kItems];
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            bk[e] = bucket_of(sc[e], lo, scale);
            if (item_of_slot<P, NT>(r, nblk, blk, tid, e) < n_scan) atomicAdd(&L.hist[bk[e]], 1u);
        }
        __syncthreads();
        if (tid < kWave) {
            find_cut(L.hist, K, ctl, lane);
            if (lane == 0) ctl->shared_floor = next_up(ctl->cut);
        }
        __syncthreads();
        stamp<STAMP>(rec, kStampOffered, lane);
        const int bstar = ctl->bstar;
        top.floor_ge = next_up(ctl->cut);                     // bucket >= b* implies score > cut
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
            const uint32_t item = item_of_slot<P, NT>(r, nblk, blk, tid, e);
            const bool take = item < n_scan && bk[e] >= bstar;
            const uint64_t mask = __ballot(take);
            if (mask != 0) top.append(mask, take, sc[e], take ? id_of(item) : 0u, lane);
        }
        if (top.prune_at != 0 && top.cnt >= top.prune_at) top.tighten(lane);
        r += 1;
    }

    // ---- 3. stream the remaining rounds against the wave's floor.  Work is handed out in units of one wave's share
    // of a round: unit j is the share of wave j % NW in round j / NW.  A wave's first kRing units are its own share
    // of the first kRing rounds (already loaded or on their way); after that it takes the next free unit from a
    // counter in LDS, so a wave that falls behind (LDS arbitration, candidate handling) does not hold the workgroup
    // up at the end.  The counter's atomic is issued one step before its result is used, and a unit's loads are
    // unconditional (past the last unit they are clamped re-reads whose data is never used): no wait in the loop
    // is longer than it has to be.
    if (rounds == 2) {
        process(w[1], 1, tid);                                // a short scan: the second round is already loaded
    } else if (rounds > 2) {
        const uint32_t units = rounds * NW;
        int pending = 0;                                      // lane 0: result of the last counter request
        auto request_unit = [&]() { if (lane == 0) pending = atomicAdd(&ctl->next_unit, 1); };
        auto requested_unit = [&]() -> uint32_t { return (uint32_t)__builtin_amdgcn_readfirstlane(pending); };
        uint32_t unit[kRing];                                 // unit held by w[i]
#pragma unroll
        for (int i = 1; i < kRing; ++i) unit[i] = (uint32_t)i * NW + wave;
        request_unit();
        unit[0] = requested_unit();
        request_unit();
        fetch(unit[0] / NW, (int)(unit[0] % NW) * kWave + lane, w[0]);
        while (unit[1 % kRing] < units) {                     // the oldest unit held; a younger one past the end scores nothing
#pragma unroll
            for (int i = 1; i <= kRing; ++i) {
                const int s = i % kRing;
                process(w[s], unit[s] / NW, (int)(unit[s] % NW) * kWave + lane);
                unit[s] = requested_unit();
                request_unit();
                fetch(unit[s] / NW, (int)(unit[s] % NW) * kWave + lane, w[s]);
            }
        }
    }
    if constexpr (P > 0 && P <= 16) {
        // the fewer than 16 / P items after the last whole code vector, one per lane of one wave
        if (blockIdx.x == 0 && wave == 0) {
            const uint32_t item = n_scan + lane;
            float sc = 0.0f;
            bool take = false;
            if (item < (uint32_t)a.N) {
                const uint8_t* row = a.codes + (size_t)item * P;
                if constexpr (CW == 2) {
                    const uint16_t* g = reinterpret_cast<const uint16_t*>(row);
                    auto at = [&](uint32_t code) { return GL ? (code < (uint32_t)stride ? code : (uint32_t)stride - 1u) : code; };
                    sc = lut[at(g[0])];
#pragma unroll
                    for (int k = 1; k < M; ++k) sc = sc + lut[(size_t)k * stride + at(g[k])];
                } else {
                    sc = lut[(size_t)row[0] * C];
#pragma unroll
                    for (int k = 1; k < M; ++k) sc = sc + lut[((size_t)k * kLutStride + row[k]) * C];
                }
                take = sc >= top.floor_ge;
            }
            const uint64_t mask = __ballot(take);
            if (mask != 0) top.append(mask, take, sc, (uint32_t)item, lane);
        }
    }

    stamp<STAMP>(rec, kStampStreamed, lane);
    // ---- 4. workgroup selection: the waves' lists -> exact K best, sorted
    // (the running histogram's floor joins the final selection from K = 32 on: below, the waves' own floors leave few
    // enough keys, and deriving it would cost more than it saves)
    workgroup_select<NT>(L, ctl, top, K, a.cap, a.candmax, tid, wide_floor && K >= 32, hlo, hscale);
    }
    stamp<STAMP>(rec, kStampSelected, lane);
    uint64_t* mine_out = a.ws_keys + ((size_t)q * nblk + blockIdx.x) * K;
    for (int t = tid; t < K; t += NT) mine_out[t] = L.sorted[t];
    stamp<STAMP>(rec, kStampEnd, lane);
}
