// PQTopK scoring for gfx950 (MI355X): kernels and the C ABI declared in include/pqtopk.h.
//
// Path (paper Section 3): pq_subitem_scores() builds the sub-id score matrix S (Eq. 4); pq_score_topk() streams the
// codebook G once, turns every item's m sub-ids into a score by m table lookups in LDS (Eq. 5), and keeps only the
// K best <id, score> pairs (Algorithm 1, V = I).  Item scores never reach memory.
//
// Total order used everywhere: a 64-bit key  (orderable(score) << 32) | ~id.  A larger key is a better item:
// higher score first, lower id between equal scores.  Keys of distinct items are distinct, key 0 means "empty".
//
// Shape of pq_score_topk(): one scan launch, then a small fold launch.
//   scan_topk_kernel<M, C, NT> (scan_single.hpp; one query per workgroup; grid = (item blocks, B)):
//     1. requests its query's table values and its first rounds of codes, then fills the m x b table into LDS
//        (C copies of it for long scans, so that lanes with different copies never collide on an LDS bank);
//     2. scores a first round of items into registers and cuts it with a 1024-bucket histogram over the workgroup's
//        scores: a floor that at least K of them exceed; everything below it is out for good;
//     3. streams the rest of its share of G against the floor; code loads are branch-free and counted, so the next
//        round's loads stay in flight; waves take their work units from a counter in LDS; survivors (a handful)
//        go to small per-wave lists in LDS that are pruned exactly (by key) when they fill, which raises the floor;
//     4. selects its exact K best and writes them, sorted, to the workspace.
//   scan_topk_tiled_kernel<M> (scan_batched.hpp; m = 8 or 16, larger batches; a tile of four queries per workgroup,
//     tables interleaved as float4 so one 16-byte LDS read serves the four queries and sub-id extraction is shared):
//     same steps; its floors are workgroup-wide, kept up to date by a running histogram of the candidates' scores.
//   fold_topk_kernel (fold.hpp; one workgroup per query) reduces the workgroups' lists to the final sorted K.
// Floors and histograms only ever prune; every decision that picks a winner compares full keys, so the result is
// exact for any input, including heavy ties (which merely take slower paths).
//
// This file holds the host side (plans, launches, the extern "C" entry points).  The device code is in the .hpp parts
// that kernels.hpp gathers in namespace pqk; the large scan kernels are compiled in the inst_*.hip translation units
// and only launched from here.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "pqtopk.h"
#include "pqtopk_measure.h"
#include "kernels.hpp"

// Built-in scratch of pq_score_topk_static(): device memory, one copy per GPU, held until the process ends.  Host code
// never uses this name as an address (it is a handle for hipGetSymbolAddress(), see static_scratch() below).
constexpr size_t kStaticScratchBytes = PQ_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

using namespace pqk;

// ---------------------------------------------------------------------------------------------------------------
// host side

thread_local char g_hip_error[256] = "no HIP error recorded";

// pq_measure_force_general(): bit 0 keeps calls off scan_short_kernel, bit 1 off fold_small_kernel, bit 2 Eq. 4 off the
// matrix cores (0: the product's choice)
std::atomic<int> g_force_general{0};

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

// Keys per wave list: a power of two (the overflow path sorts it) with room for K kept keys plus a wave's worth of
// new ones, and at least K / 4: a list that holds K of its `cap` keys for good is sorted every cap - K appends
// (K = 448 in 512 slots sorted every 64 keys: twice as slow as K = 449 in 1024).
int list_capacity(int K) {
    const int spare = K / 4 > kWave ? K / 4 : kWave;
    const int cap = next_pow2(K + spare);
    return cap < 128 ? 128 : cap;
}

struct ScanPlan {
    int copies;      // single-query kernel: copies of the score tables in LDS (1 or kTableCopies)
    bool tiled;      // batched kernel: kQ queries per workgroup
    bool big;        // single-query kernel: kBigThreads threads per workgroup, one workgroup per CU
    int nblk;        // item blocks per query
    int cap;         // keys per wave list
    int candmax;     // keys of the candidate array
    int stage_keys;  // keys the fold stages per pass
    size_t scan_dyn_lds;     // dynamic LDS of the scan launch
    size_t scan_lds;         // dynamic + the static score tables of the vector kernels
    size_t fold_lds;
    bool vec;
    bool glut;       // two-byte sub-ids: the m x b table does not fit LDS and is read from device memory
    bool short_scan; // scan_short_kernel: every workgroup's share fits its registers, K small
    int short_units; // ... units (code vectors, or items for m = 32, 64) a thread holds
    bool short_subset; // scan_subset_kernel: a candidate list whose share per thread fits its registers, K small
    int subset_vecs;   // ... code vectors' worth of gathered rows a thread holds
};

bool is_vec_m(int m) { return m == 1 || m == 2 || m == 4 || m == 8 || m == 16 || m == 32 || m == 64; }

bool is_vec_m16(int m) { return m == 4 || m == 8 || m == 16; }   // 16-bit sub-ids: rows of 8, 16 or 32 bytes

// With a multiple of 8 blocks per query, block x of every query runs on XCD x % 8 and the queries share that XCD's L2
// (worth about 5 %): taken when it costs at most a sixteenth of the blocks.
long long xcd_aligned(long long nb, int B) {
    return (B > 1 && (nb & 7) * 16 <= nb) ? (nb & ~7LL) : nb;
}

// Item blocks per query when B single-query scans run side by side on `slots` workgroup slots (CUs times resident
// workgroups) and B is too large for eight blocks each: as many as fill the slots once, or a few times over when one
// filling would leave many idle.  Cost of a choice: (fillings) x (a block's share of the query's streaming time, which
// the table lookups bound at 9.1 per clock and CU, plus some 8 us per workgroup for tables, first cut and selection).
long long blocks_for_many_queries(long long slots, long long B, long long rounds, double lookups_per_query) {
    const double stream_us = lookups_per_query / (9.1 * 2400.0);
    long long best_nb = 1;
    double best_us = 0.0;
    for (int fill = 1; fill <= 8; ++fill) {
        long long nb = slots * fill / B;
        if (nb > rounds) nb = rounds;
        if (nb < 1) nb = 1;
        const long long fillings = (B * nb + slots - 1) / slots;
        const double us = (double)fillings * (stream_us / (double)nb + 8.0);
        if (fill == 1 || us < best_us) { best_us = us; best_nb = nb; }
    }
    return best_nb;
}

// Lookups (B * N * m) from which the batched kernel beats B single-query scans side by side.  Measured on catalogues
// of 3e5 to 2e7 items: its fixed costs (about 15 us of tables, first cuts and final merge, more with K) are paid back
// from 2e8 lookups on at K = 10.  At m = 8 the side-by-side scans run with replicated tables as long as their lists
// leave room for them (K <= 64) and then stay ahead up to 8e8 lookups; for K > 128 their shared floors do.
double tiled_min_lookups(int m, int K) {
    if (m == 8) {
        if (K <= 12) return kTiledMinLookups * (1.0 + K / 400.0);
        if (K <= 64) return 8.5e8;
        if (K <= 128) return 3.5e8;
        return 9.0e8;
    }
    return K <= 128 ? kTiledMinLookups * (1.0 + K / 400.0) : 5.0e8;
}

// `generic`: plan for the generic kernel whatever m is (candidate-list scans use it: their rows are gathered)
// `cw`, `b`: bytes per sub-id (1 or 2) and, for two-byte sub-ids, the alphabet size (it sizes the tables in LDS)
ScanPlan make_plan(long long N, int B, int m, int K, bool generic = false, int cw = 1, int b = kLutStride) {
    ScanPlan p;
    const int row = m * cw;                                    // bytes of an item's row
    size_t lut_floats = cw == 1 ? (size_t)m * kLutStride : (size_t)m * b;
    p.cap = list_capacity(K);
    p.candmax = next_pow2(2 * K);
    if (p.candmax < 512) p.candmax = 512;
    // two-byte sub-ids whose table leaves no room in LDS (even for one 1024-thread workgroup): lookups go to memory
    p.glut = cw == 2 && scan_lds_bytes(lut_floats, p.cap, p.candmax, K, kMaxWaves) > kMaxLdsBytes;
    if (p.glut) lut_floats = 0;
    p.vec = !generic && (cw == 1 ? is_vec_m(m) : is_vec_m16(m)) && N * row >= 16;   // (one whole code vector at least)
    const long long units = (p.vec && row <= 16) ? (N * row) / 16 : N;   // whole code vectors (the few items after them are extra)
    const long long per_round = (long long)kThreads * (p.vec ? vec_per_thread(row) : kGenericItemsPerThread);
    long long rounds = (units + per_round - 1) / per_round;
    const double lookups = (double)N * m;                           // table lookups of one query's scan
    long long most = (kBlocksPerCU * (long long)kAssumedCUs) / B;   // workgroups over the whole grid
    if (most < 8) most = blocks_for_many_queries(kBlocksPerCU * (long long)kAssumedCUs, B, rounds, lookups);
    long long nblk = rounds < most ? rounds : most;
    long long one_per_cu = kAssumedCUs / B;                    // a short scan is spread evenly: one workgroup per CU, which
    if (one_per_cu < 8) one_per_cu = 8;                        // then takes two or three (possibly ragged) rounds
    if (rounds > one_per_cu && rounds <= most) nblk = one_per_cu;
    if (nblk < 1) nblk = 1;
    nblk = xcd_aligned(nblk, B);
    {
        // A fold of one launch instead of two levels is worth a slightly coarser grid (K = 53 .. 69 at batch 1: 256
        // lists of K = 64 take two fold levels, 208 lists one launch: 22.1 -> 19.1 us per call); not a much coarser one
        // (K = 100 on 133 workgroups instead of 256: 24.7 -> 26.9 us).
        const long long one_fold = (long long)kBigThreads * kFoldWideRegs / K;   // lists one fold launch takes
        if (nblk > one_fold && 4 * one_fold >= 3 * nblk) nblk = one_fold;
    }
    p.nblk = (int)nblk;
    p.stage_keys = next_pow2(2 * K);
    if (p.stage_keys < kChunkKeys) p.stage_keys = kChunkKeys;
    p.copies = 1;
    // A long scan for few queries is bound by LDS bank conflicts of the random lookups: with kTableCopies copies of
    // the tables, lanes l and l' collide only if l % kTableCopies == l' % kTableCopies.  Worth its LDS and fill time
    // only when every workgroup streams many rounds; one workgroup per CU then (the tables take 128 KB at m = 8).
    if (cw == 1 && p.vec && m <= 8) {
        const long long big_round = (long long)kBigThreads * vec_per_thread(m);
        const long long big_rounds = (units + big_round - 1) / big_round;
        long long nb = kAssumedCUs / B;                        // one workgroup (of kBigThreads) per CU over the whole grid
        if (nb < 8) nb = blocks_for_many_queries(kAssumedCUs, B, big_rounds, lookups);
        const size_t dyn = scan_lds_bytes((size_t)m * kLutStride * kTableCopies, p.cap, p.candmax, K, kMaxWaves);
        if (big_rounds >= kTableCopiesMinRounds * nb && dyn <= kMaxLdsBytes) {
            p.copies = kTableCopies;
            p.nblk = (int)nb;
        }
    }
    // A scan whose tables leave room for only one 512-thread workgroup per CU (generic: m > 36 or so; m = 64; large
    // alphabets of two-byte sub-ids) runs 1024-thread workgroups instead, one per CU: the same tables then serve
    // sixteen waves, which is what hides the latency of the row loads.  Only when there is more than one workgroup's
    // worth of work per CU.
    p.big = p.copies > 1;
    if (!p.vec || m == 64 || cw == 2) {
        const size_t small = scan_lds_bytes(lut_floats, p.cap, p.candmax, K, kWaves);
        const size_t big = scan_lds_bytes(lut_floats, p.cap, p.candmax, K, kMaxWaves);
        const long long big_round = (long long)kBigThreads * (p.vec ? vec_per_thread(row) : kGenericItemsPerThread);
        const long long big_rounds = (units + big_round - 1) / big_round;
        long long nb = kAssumedCUs / B;
        if (nb < 8) nb = blocks_for_many_queries(kAssumedCUs, B, big_rounds, lookups);
        if (2 * small > kMaxLdsBytes && big <= kMaxLdsBytes && rounds > nb) {
            if (big_rounds < nb) nb = big_rounds;
            nb = xcd_aligned(nb, B);
            p.big = true;
            p.nblk = (int)nb;
        }
    }
    const bool static_lut = p.vec && p.copies == 1 && cw == 1;   // tables in the kernel's static LDS array
    const size_t lut_dyn = p.copies > 1 ? lut_floats * p.copies : (static_lut ? 0 : lut_floats);
    p.scan_dyn_lds = scan_lds_bytes(lut_dyn, p.cap, p.candmax, K, p.big ? kMaxWaves : kWaves);
    p.scan_lds = p.scan_dyn_lds + (static_lut ? lut_floats * sizeof(float) : 0);
    p.tiled = false;
    // (a small batch over a small catalogue is faster as B single-query scans side by side: the batched kernel's
    // fixed costs, about 15 us of table fill, first-round cuts and final merge, are not yet paid back)
    const bool small_job = B <= 2 || (double)B * (double)N * m <= tiled_min_lookups(m, K);
    if (cw == 1 && !generic && !small_job && (m == 8 || m == 16) && N * m >= 16) {   // batched kernel, if its tables and lists fit in LDS
        const size_t dyn = tiled_lds_bytes(p.cap, p.candmax, K);
        const size_t all = dyn + (size_t)kQ * m * kLutStride * sizeof(float);
        if (all <= kMaxLdsBytes) {
            p.tiled = true;
            p.scan_dyn_lds = dyn;
            p.scan_lds = all;
            const long long tiles = (B + kQ - 1) / kQ;
            const long long t_round = (long long)kThreads * kTileVecs;
            const long long t_rounds = (units + t_round - 1) / t_round;
            // Item blocks per tile: as many as fill the CUs once, or twice or three times over when a single filling
            // would leave many CUs idle (96 tiles: 2 blocks = 192 workgroups, 5 blocks = 480).  The LDS is the bound, so
            // L workgroups on a CU take L times a workgroup's streaming time, plus fixed costs per workgroup (tables,
            // first-round cuts, final merge; measured: 28 us, and 20 + 0.75 K us for every further workgroup on the CU;
            // streaming: 1.3 ns per code vector and tile).
            const double stream_us = 1.3e-3 * (double)units;
            double best_us = 0.0;
            long long nb = 1;
            for (int fill = 1; fill <= 3; ++fill) {
                long long cand = ((long long)kAssumedCUs * fill) / tiles;
                if (cand > t_rounds) cand = t_rounds;
                if (cand < 1) cand = 1;
                const long long per_cu = (tiles * cand + kAssumedCUs - 1) / kAssumedCUs;   // workgroups on the busiest CU
                const double us = (double)per_cu * stream_us / (double)cand + 28.0 + (20.0 + 0.75 * K) * (double)(per_cu - 1);
                if (fill == 1 || us < best_us) { best_us = us; nb = cand; }
            }
            p.nblk = (int)nb;
        }
    }
    p.fold_lds = fold_lds_bytes(p.stage_keys, p.candmax, K);
    // Single-query scans (one query per workgroup row) with a small K whose share per thread fits a few registers run
    // the short kernel: scores stay in registers, one selection, a few KB of code.  Its grid is spread as thin as the
    // CUs allow (one workgroup per CU over all queries): a workgroup's time is the lookups of its share plus a fixed
    // selection, so the fewer units a thread holds the better, and the small fold takes the 256 lists in its stride.
    p.short_scan = false;
    p.short_units = 0;
    // (two-byte sub-ids: when the table fits LDS beside the selection's few KB)
    const bool short16 = cw == 2 && !p.glut && lut_floats * sizeof(float) + sizeof(SmallSelectLds<kThreads>) <= kMaxLdsBytes;
    if ((cw == 1 || short16) && p.vec && !generic && !p.tiled && K <= kSmallKMax) {
        long long nb = kAssumedCUs / B;
        if (nb < 1) nb = 1;
        const long long thin = (units + kThreads - 1) / kThreads;          // workgroups if every thread held one unit
        if (nb > thin) nb = thin;
        const long long per_slot = (long long)kThreads * nb;               // units one slot of all threads covers
        const long long slots = (units + per_slot - 1) / per_slot;
        if (slots <= (cw == 1 ? short_max_units(m) : short16_max_units(m))) {
            // (one-byte sub-ids: the general kernel takes the same grid when the measurement hook keeps a call off the
            // short one; two-byte sub-ids: its plan stays as it is)
            const bool forced = (g_force_general.load(std::memory_order_relaxed) & 1) != 0;
            if (cw == 1 || !forced) {
                p.nblk = (int)nb;
                p.copies = 1;
                p.big = false;
            }
            if (cw == 1) {
                p.scan_dyn_lds = scan_lds_bytes(0, p.cap, p.candmax, K, kWaves);
                p.scan_lds = p.scan_dyn_lds + lut_floats * sizeof(float);
            }
            if (!forced) {
                p.short_scan = true;
                p.short_units = (int)slots;
                p.scan_dyn_lds = cw == 1 ? 0 : lut_floats * sizeof(float);
                p.scan_lds = lut_floats * sizeof(float) + sizeof(SmallSelectLds<kThreads>);
            }
        }
    }
    // Candidate lists (the `generic` plans) of rows of 4, 8 or 16 bytes with a small K, short enough for a thread to
    // hold its share: every row of a thread is requested at once and the selection comes straight from registers.
    // Same thin grid as the short scan.
    p.short_subset = false;
    p.subset_vecs = 0;
    if (generic && cw == 1 && (m == 4 || m == 8 || m == 16) && K <= kSmallKMax &&
        !(g_force_general.load(std::memory_order_relaxed) & 1)) {
        long long nb = kAssumedCUs / B;
        if (nb < 1) nb = 1;
        const long long thin = (N + kThreads - 1) / kThreads;              // workgroups if every thread held one candidate
        if (nb > thin) nb = thin;
        const long long per_thread = (N + kThreads * nb - 1) / (kThreads * nb);
        const long long vecs = (per_thread * m + 15) / 16;
        if (vecs <= kSubsetMaxVecs) {
            p.short_subset = true;
            p.subset_vecs = (int)vecs;
            p.nblk = (int)nb;
            p.copies = 1;
            p.big = false;
            p.scan_dyn_lds = 0;
            p.scan_lds = (size_t)m * kLutStride * sizeof(float) + sizeof(SmallSelectLds<kThreads>);
        }
    }
    return p;
}

size_t keys_bytes(const ScanPlan& p, int B, int K) {
    const size_t bytes = (size_t)B * p.nblk * K * sizeof(uint64_t);
    return (bytes + 255) & ~(size_t)255;
}

size_t fold_area_keys(int nblk, int B, int K);

// workspace: [B][nblk][K] keys from the scan | a second, smaller key area for folds that take more than one level
size_t workspace_bytes(const ScanPlan& p, int B, int K) {
    return keys_bytes(p, B, K) + ((fold_area_keys(p.nblk, B, K) * sizeof(uint64_t) + 255) & ~(size_t)255);
}

int check_topk_shape(long long N, int B, int m, int b, int K, int cw) {
    if (N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > (cw == 1 ? 256 : 65536) || K > N || N >= 2147483648LL)
        return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    return PQ_OK;
}

int check_topk_args(const void* codes, const void* S, long long N, int B, int m, int b, int K, const void* out_ids,
                    const void* out_scores, const void* workspace, size_t workspace_bytes_given, int cw = 1) {
    if (!codes || !S || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    const int rc = check_topk_shape(N, B, m, b, K, cw);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_plan(N, B, m, K, false, cw, b);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)codes & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)S & 3) || ((uintptr_t)out_ids & 3) ||
        ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(p, B, K)) return PQ_ERR_WORKSPACE;
    return PQ_OK;
}

constexpr int kMaxDevices = 64;

// Kernels that take more than 64 KB of dynamic LDS need the limit raised, per kernel and device: done the first time a
// kernel asks for that much (and again only if it later asks for more), not on every call.
struct LdsGrant { const void* fn; int dev; size_t bytes; };
hipError_t allow_lds_once(const void* fn, size_t bytes) {
    static std::mutex mu;
    static LdsGrant grants[512];
    static int n_grants = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    LdsGrant* g = nullptr;
    for (int i = 0; i < n_grants && g == nullptr; ++i)
        if (grants[i].fn == fn && grants[i].dev == dev) g = &grants[i];
    if (g != nullptr && g->bytes >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    if (g == nullptr && n_grants < 512) g = &grants[n_grants++];
    if (g != nullptr) *g = LdsGrant{fn, dev, bytes};           // (table full: the attribute is simply set again next time)
    return hipSuccess;
}
template <typename KernelT>
hipError_t allow_lds(KernelT kernel, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    return allow_lds_once(reinterpret_cast<const void*>(kernel), bytes);
}

template <int M, int CW = 1>
hipError_t launch_scan(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    if constexpr (CW == 1 && M >= 1 && M <= 8) {
        if (p.copies == kTableCopies) {
            hipError_t e = allow_lds(scan_topk_kernel<M, kTableCopies, kBigThreads>, p.scan_dyn_lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((scan_topk_kernel<M, kTableCopies, kBigThreads>), dim3(p.nblk, B), dim3(kBigThreads),
                               p.scan_dyn_lds, st, a);
            return hipGetLastError();
        }
    }
    if constexpr (CW == 2) {
        if (p.glut) {
            hipError_t e = allow_lds(scan_topk_kernel<M, 1, kThreads, 2, true>, p.scan_dyn_lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((scan_topk_kernel<M, 1, kThreads, 2, true>), dim3(p.nblk, B), dim3(kThreads), p.scan_dyn_lds,
                               st, a);
            return hipGetLastError();
        }
    }
    if constexpr (M == 0 || M == 64 || CW == 2) {
        if (p.big) {
            hipError_t e = allow_lds(scan_topk_kernel<M, 1, kBigThreads, CW>, p.scan_dyn_lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((scan_topk_kernel<M, 1, kBigThreads, CW>), dim3(p.nblk, B), dim3(kBigThreads),
                               p.scan_dyn_lds, st, a);
            return hipGetLastError();
        }
    }
    hipError_t e = allow_lds(scan_topk_kernel<M, 1, kThreads, CW>, p.scan_dyn_lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((scan_topk_kernel<M, 1, kThreads, CW>), dim3(p.nblk, B), dim3(kThreads), p.scan_dyn_lds, st, a);
    return hipGetLastError();
}

template <int M, int U>
hipError_t launch_short_units(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    if constexpr (U <= short_max_units(M)) {
        if constexpr (M == 8) {
            if (a.stamps != nullptr) {
                hipLaunchKernelGGL((scan_short_kernel<M, U, kThreads, true>), dim3(p.nblk, B), dim3(kThreads), 0, st, a);
                return hipGetLastError();
            }
        }
        hipLaunchKernelGGL((scan_short_kernel<M, U, kThreads, false>), dim3(p.nblk, B), dim3(kThreads), 0, st, a);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;                         // (the plan never asks for it)
    }
}
template <int M>
hipError_t launch_short_m(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    switch (p.short_units) {
        case 1: return launch_short_units<M, 1>(p, a, B, st);
        case 2: return launch_short_units<M, 2>(p, a, B, st);
        case 3: return launch_short_units<M, 3>(p, a, B, st);
        case 4: return launch_short_units<M, 4>(p, a, B, st);
        case 5: return launch_short_units<M, 5>(p, a, B, st);
        case 6: return launch_short_units<M, 6>(p, a, B, st);
        case 7: return launch_short_units<M, 7>(p, a, B, st);
        case 8: return launch_short_units<M, 8>(p, a, B, st);
        case 9: return launch_short_units<M, 9>(p, a, B, st);
        case 10: return launch_short_units<M, 10>(p, a, B, st);
        case 11: return launch_short_units<M, 11>(p, a, B, st);
        case 12: return launch_short_units<M, 12>(p, a, B, st);
        default: return hipErrorInvalidValue;
    }
}
hipError_t launch_short(const ScanPlan& p, const ScanArgs& a, int B, int m, hipStream_t st) {
    switch (m) {
        case 1: return launch_short_m<1>(p, a, B, st);
        case 2: return launch_short_m<2>(p, a, B, st);
        case 4: return launch_short_m<4>(p, a, B, st);
        case 8: return launch_short_m<8>(p, a, B, st);
        case 16: return launch_short_m<16>(p, a, B, st);
        case 32: return launch_short_m<32>(p, a, B, st);
        default: return launch_short_m<64>(p, a, B, st);
    }
}

template <int M, int U>
hipError_t launch_short16_units(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    if constexpr (U <= short16_max_units(M)) {
        hipError_t e = allow_lds(scan_short_kernel<M, U, kThreads, false, 2>, p.scan_dyn_lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((scan_short_kernel<M, U, kThreads, false, 2>), dim3(p.nblk, B), dim3(kThreads), p.scan_dyn_lds, st, a);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;                         // (the plan never asks for it)
    }
}
template <int M>
hipError_t launch_short16_m(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    switch (p.short_units) {
        case 1: return launch_short16_units<M, 1>(p, a, B, st);
        case 2: return launch_short16_units<M, 2>(p, a, B, st);
        case 3: return launch_short16_units<M, 3>(p, a, B, st);
        case 4: return launch_short16_units<M, 4>(p, a, B, st);
        case 5: return launch_short16_units<M, 5>(p, a, B, st);
        case 6: return launch_short16_units<M, 6>(p, a, B, st);
        case 7: return launch_short16_units<M, 7>(p, a, B, st);
        case 8: return launch_short16_units<M, 8>(p, a, B, st);
        case 9: return launch_short16_units<M, 9>(p, a, B, st);
        case 10: return launch_short16_units<M, 10>(p, a, B, st);
        case 11: return launch_short16_units<M, 11>(p, a, B, st);
        case 12: return launch_short16_units<M, 12>(p, a, B, st);
        default: return hipErrorInvalidValue;
    }
}

template <int M>
hipError_t launch_subset_m(const ScanPlan& p, const ScanArgs& a, int B, hipStream_t st) {
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(p.nblk, B), dim3(kThreads), 0, st, a);
        return hipGetLastError();
    };
    switch (p.subset_vecs) {
        case 1: return go(scan_subset_kernel<M, 1, kThreads>);
        case 2: return go(scan_subset_kernel<M, 2, kThreads>);
        case 3: return go(scan_subset_kernel<M, 3, kThreads>);
        case 4: return go(scan_subset_kernel<M, 4, kThreads>);
        case 5: return go(scan_subset_kernel<M, 5, kThreads>);
        case 6: return go(scan_subset_kernel<M, 6, kThreads>);
        case 7: return go(scan_subset_kernel<M, 7, kThreads>);
        case 8: return go(scan_subset_kernel<M, 8, kThreads>);
        default: return hipErrorInvalidValue;
    }
}

// Enqueue the catalogue scan: every workgroup's K best keys land in the workspace.
// `subset` / `n_items`: candidate list (then N is its length and the plan is a generic one) or nullptr / N
// `cw`: bytes per sub-id (2: `codes` holds uint16 values)
int enqueue_scan(const ScanPlan& p, const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                 void* workspace, hipStream_t st, const int* subset = nullptr, long long n_items = 0, int cw = 1,
                 uint64_t* stamps = nullptr) {
    ScanArgs a;
    a.codes = codes; a.S = S; a.N = N; a.m = m; a.b = b; a.K = K;
    a.subset = subset; a.n_items = (uint32_t)(subset ? n_items : N);
    a.stamps = stamps;
    a.cap = p.cap; a.candmax = p.candmax;
    // Batched kernel, small K: lists are cut back to their K best once they pass 2K + 8 keys, short enough to rank in
    // one pass; from K = 13 on its shared floors and final filter do better without (K = 16: 53 -> 48 us, K = 28:
    // 63 -> 52 us at batch 24).  The single-query kernel never cuts early: lists are sorted when full, and the shared
    // floor of long scans keeps them from filling (K = 10: 50M items 79.7 -> 77.5 us, m = 4 at batch 64 57 -> 49 us).
    a.prune_at = (p.tiled && K <= 12) ? 2 * K + 8 : 0;
    a.ws_keys = static_cast<uint64_t*>(workspace);
    hipError_t e;
    if (p.short_scan && cw == 2) {
        if (stamps != nullptr) return PQ_ERR_UNSUPPORTED;
        return record_hip(m == 4 ? launch_short16_m<4>(p, a, B, st) : m == 8 ? launch_short16_m<8>(p, a, B, st) : launch_short16_m<16>(p, a, B, st));
    }
    if (p.short_scan) {
        if (stamps != nullptr && m != 8) return PQ_ERR_UNSUPPORTED;
        return record_hip(launch_short(p, a, B, m, st));
    }
    if (p.short_subset) {
        if (subset == nullptr || stamps != nullptr) return PQ_ERR_UNSUPPORTED;   // (the plan is only made for candidate lists)
        return record_hip(m == 4 ? launch_subset_m<4>(p, a, B, st) : m == 8 ? launch_subset_m<8>(p, a, B, st) : launch_subset_m<16>(p, a, B, st));
    }
    if (p.tiled) {
        const dim3 grid(p.nblk, (B + kQ - 1) / kQ);
        auto launch_tiled = [&](auto kernel) {
            hipError_t err = allow_lds(kernel, p.scan_dyn_lds);
            if (err == hipSuccess) {
                hipLaunchKernelGGL(kernel, grid, dim3(kThreads), p.scan_dyn_lds, st, a, B);
                err = hipGetLastError();
            }
            return err;
        };
        if (stamps != nullptr) e = m == 8 ? launch_tiled(scan_topk_tiled_kernel<8, true>) : launch_tiled(scan_topk_tiled_kernel<16, true>);
        else e = m == 8 ? launch_tiled(scan_topk_tiled_kernel<8, false>) : launch_tiled(scan_topk_tiled_kernel<16, false>);
        return record_hip(e);
    }
    if (stamps != nullptr) {
        // single-query scans: measurement instances exist for m = 8 only
        if (cw != 1 || !p.vec || m != 8 || p.big != (p.copies == kTableCopies)) return PQ_ERR_UNSUPPORTED;
        if (p.copies == kTableCopies) {
            e = allow_lds(scan_topk_kernel<8, kTableCopies, kBigThreads, 1, false, true>, p.scan_dyn_lds);
            if (e == hipSuccess)
                hipLaunchKernelGGL((scan_topk_kernel<8, kTableCopies, kBigThreads, 1, false, true>), dim3(p.nblk, B),
                                   dim3(kBigThreads), p.scan_dyn_lds, st, a);
        } else {
            e = allow_lds(scan_topk_kernel<8, 1, kThreads, 1, false, true>, p.scan_dyn_lds);
            if (e == hipSuccess)
                hipLaunchKernelGGL((scan_topk_kernel<8, 1, kThreads, 1, false, true>), dim3(p.nblk, B), dim3(kThreads),
                                   p.scan_dyn_lds, st, a);
        }
        return record_hip(e == hipSuccess ? hipGetLastError() : e);
    }
    if (cw == 2) {
        switch (p.vec ? m : 0) {
            case 4: e = launch_scan<4, 2>(p, a, B, st); break;
            case 8: e = launch_scan<8, 2>(p, a, B, st); break;
            case 16: e = launch_scan<16, 2>(p, a, B, st); break;
            default: e = launch_scan<0, 2>(p, a, B, st); break;
        }
        return record_hip(e);
    }
    switch (p.vec ? m : 0) {
        case 1: e = launch_scan<1>(p, a, B, st); break;
        case 2: e = launch_scan<2>(p, a, B, st); break;
        case 4: e = launch_scan<4>(p, a, B, st); break;
        case 8: e = launch_scan<8>(p, a, B, st); break;
        case 16: e = launch_scan<16>(p, a, B, st); break;
        case 32: e = launch_scan<32>(p, a, B, st); break;
        case 64: e = launch_scan<64>(p, a, B, st); break;
        default: e = launch_scan<0>(p, a, B, st); break;
    }
    return record_hip(e);
}

// Lists one fold workgroup takes at a level with `nlists` lists per query.  All of them when their keys fit the usual
// fold's registers (kThreads * kFoldRegs keys), or the wide fold's (kBigThreads * kFoldWideRegs keys, `wide` set: one
// launch of one larger workgroup instead of two levels).  More keys than that are split into groups: several small
// folds side by side and one more level beat one workgroup that reads everything (256 lists of K = 100: 12 us in two
// levels, 16-24 us in one workgroup of 1024 threads holding 26 keys each).  A group has about sqrt(nlists) lists, so
// that both levels are small (256 lists of K = 100: 16 folds of 16 lists, then one of 16, instead of 5 folds of 61
// lists and one of 5: 14.4 -> 12.2 us), and never more keys than the usual fold's registers hold.
int fold_lists_per_group(int nlists, int K, bool* wide) {
    const long long nkeys = (long long)nlists * K;
    *wide = nkeys > (long long)kThreads * kFoldRegs && nkeys <= (long long)kBigThreads * kFoldWideRegs;
    if (nkeys <= (long long)kBigThreads * kFoldWideRegs) return nlists;
    const int fit = kThreads * kFoldRegs / K;
    int per = 2;
    while (per * per < nlists) ++per;
    if (per > fit) per = fit;
    return per < 2 ? 2 : per;
}

// Keys of the second key area of the workspace: what the first fold level writes when the lists of a query do not fit
// one workgroup's registers (later levels alternate between the two areas, each needing less than the one before).
size_t fold_area_keys(int nblk, int B, int K) {
    bool wide;
    const int per = fold_lists_per_group(nblk, K, &wide);
    if (nblk <= per) return 0;
    return (size_t)B * ((nblk + per - 1) / per) * K;
}

// Enqueue the fold of the workspace's lists into the outputs: one launch when a query's lists fit one workgroup's
// registers, else levels of launches that each fold groups of lists into one list per group.
int enqueue_fold(const ScanPlan& p, int B, int K, void* workspace, int* out_ids, float* out_scores, hipStream_t st,
                 uint64_t* stamps = nullptr) {
    hipError_t e = allow_lds(fold_topk_kernel<kThreads, kFoldRegs>, p.fold_lds);
    if (e == hipSuccess) e = allow_lds(fold_topk_kernel<kBigThreads, kFoldWideRegs>, p.fold_lds);
    if (e != hipSuccess) return record_hip(e);
    uint64_t* area[2] = {static_cast<uint64_t*>(workspace),
                         reinterpret_cast<uint64_t*>(static_cast<unsigned char*>(workspace) + keys_bytes(p, B, K))};
    int nlists = p.nblk, src = 0;
    for (;;) {
        bool wide;
        const int per = fold_lists_per_group(nlists, K, &wide);
        const int groups = nlists <= per ? 1 : (nlists + per - 1) / per;
        FoldArgs f;
        f.ws_keys = area[src];
        f.nlists = nlists; f.K = K; f.lists_per_group = groups == 1 ? nlists : per;
        f.stage_keys = p.stage_keys; f.candmax = p.candmax;
        f.out_keys = groups == 1 ? nullptr : area[1 - src];
        f.out_ids = out_ids; f.out_scores = out_scores;
        f.stamps = stamps;
        if (groups == 1 && K <= kSmallKMax && (long long)nlists * K <= (long long)kThreads * kFoldSmallRegsMax &&
            !(g_force_general.load(std::memory_order_relaxed) & 2)) {
            // small K, few keys: the lean fold
            const bool few = (long long)nlists * K <= (long long)kThreads * kFoldSmallRegs;
            if (stamps != nullptr) {
                if (few) hipLaunchKernelGGL((fold_small_kernel<kThreads, kFoldSmallRegs, true>), dim3(1, B), dim3(kThreads), 0, st, f);
                else hipLaunchKernelGGL((fold_small_kernel<kThreads, kFoldSmallRegsMax, true>), dim3(1, B), dim3(kThreads), 0, st, f);
            } else {
                if (few) hipLaunchKernelGGL((fold_small_kernel<kThreads, kFoldSmallRegs, false>), dim3(1, B), dim3(kThreads), 0, st, f);
                else hipLaunchKernelGGL((fold_small_kernel<kThreads, kFoldSmallRegsMax, false>), dim3(1, B), dim3(kThreads), 0, st, f);
            }
            return record_hip(hipGetLastError());
        }
        if (stamps != nullptr) {                             // measurement instance: the usual one-launch fold only
            if (wide || groups != 1) return PQ_ERR_UNSUPPORTED;
            e = allow_lds(fold_topk_kernel<kThreads, kFoldRegs, true>, p.fold_lds);
            if (e != hipSuccess) return record_hip(e);
            hipLaunchKernelGGL((fold_topk_kernel<kThreads, kFoldRegs, true>), dim3(1, B), dim3(kThreads), p.fold_lds, st, f);
            return record_hip(hipGetLastError());
        }
        if (wide)
            hipLaunchKernelGGL((fold_topk_kernel<kBigThreads, kFoldWideRegs>), dim3(groups, B), dim3(kBigThreads), p.fold_lds,
                               st, f);
        else
            hipLaunchKernelGGL((fold_topk_kernel<kThreads, kFoldRegs>), dim3(groups, B), dim3(kThreads), p.fold_lds, st, f);
        e = hipGetLastError();
        if (e != hipSuccess) return record_hip(e);
        if (groups == 1) return PQ_OK;
        nlists = groups;
        src = 1 - src;
    }
}

// Batch from which Eq. 4 runs on the matrix cores.  The scalar kernels are faster below: a wave's chain of d/m matrix
// instructions takes as long for one tile of 32 queries as for a GPU full of them (measured at d = 512, m = 8, b = 256:
// 5.8 us against 5.0 us at B = 256, 6.1 against 6.7 at B = 512, 6.7 against 10.8 at B = 1024, 21 against 35 at B = 4096).
constexpr int kSubMfmaMinBatch = 448;
constexpr int kDefaultMfmaMinBatch = 3;    // default scoring: batch from which one matrix-core pass over W beats B mat-vec passes

// Eq. 4 on the matrix cores when the shape allows: rows 16-byte aligned, d/m a multiple of 16.  `ldS`: floats from one
// query's row of S to the next.
bool launch_subitem_mfma(const float* queries, const float* centroids, float* S, int B, int d, int m, long long b, long long ldS,
                         hipStream_t st) {
    const int s = d / m;
    if (s % 16 != 0 || d % 4 != 0 || ((((uintptr_t)queries | (uintptr_t)centroids)) & 15) != 0) return false;
    const long long jtiles = (b + 63) / 64;
    if (m * jtiles > 2147483647LL) return false;
    const dim3 grid((unsigned)(m * jtiles), (B + kSubMfmaQueries - 1) / kSubMfmaQueries);
    if (s % 64 == 0) hipLaunchKernelGGL(subitem_scores_mfma_kernel<64>, grid, dim3(kSubMfmaThreads), 0, st, queries, centroids, S, B, d, m, (int)b, ldS);
    else if (s % 32 == 0) hipLaunchKernelGGL(subitem_scores_mfma_kernel<32>, grid, dim3(kSubMfmaThreads), 0, st, queries, centroids, S, B, d, m, (int)b, ldS);
    else hipLaunchKernelGGL(subitem_scores_mfma_kernel<16>, grid, dim3(kSubMfmaThreads), 0, st, queries, centroids, S, B, d, m, (int)b, ldS);
    return true;
}

template <int S_ELEMS>
void launch_subitem(const float* queries, const float* centroids, float* S, int B, int d, int m, int b, hipStream_t st) {
    if constexpr (S_ELEMS % 4 == 0) {
        // batches, and any sub-dimension that is a multiple of 4 without an unrolled instance (96, 128, ...): the
        // interleaved kernel (it needs 16-byte aligned rows of queries and centroids)
        const bool rows_aligned = (((uintptr_t)queries | (uintptr_t)centroids) & 15) == 0 && d % 4 == 0 && (d / m) % 4 == 0;
        if ((B >= kSubInterleave || S_ELEMS == 0) && rows_aligned) {
            dim3 grid(m * ((b + kSubThreads - 1) / kSubThreads), (B + kSubBatchTile - 1) / kSubBatchTile);
            hipLaunchKernelGGL(subitem_scores_batched_kernel<S_ELEMS>, grid, dim3(kSubThreads), 0, st, queries, centroids, S,
                               B, d, m, b);
            return;
        }
    }
    dim3 grid((m * b + kSubThreads - 1) / kSubThreads, (B + kSubQueryTile - 1) / kSubQueryTile);
    if constexpr (S_ELEMS != 0 && S_ELEMS % 4 == 0 && S_ELEMS <= 128) {
        // whole waves of 16-byte aligned rows: the wave reads its block of sub-item embeddings piece after piece
        if (((long long)m * b) % kSubThreads == 0 && ((uintptr_t)centroids & 15) == 0) {
            hipLaunchKernelGGL((subitem_scores_kernel<S_ELEMS, false, true>), grid, dim3(kSubThreads), 0, st, queries, centroids, S,
                               B, d, m, b, nullptr);
            return;
        }
    }
    hipLaunchKernelGGL(subitem_scores_kernel<S_ELEMS>, grid, dim3(kSubThreads), 0, st, queries, centroids, S, B, d, m, b);
}

// ---- the built-in scratch of pq_score_topk_static(): one array per GPU, held until the process ends
// Device address of `scratch` on the current device.  In host code the array's name is only a handle for
// hipGetSymbolAddress(): every GPU holds its own copy at its own address, looked up once per device and kept.
int static_scratch(void** out) {
    static void* ptr[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return record_hip(e);
    if (dev < 0 || dev >= kMaxDevices) return PQ_ERR_UNSUPPORTED;
    void* p = __atomic_load_n(&ptr[dev], __ATOMIC_ACQUIRE);
    if (p == nullptr) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // (the same answer from every thread that races here)
        if (e != hipSuccess) return record_hip(e);
        if (p == nullptr) return PQ_ERR_HIP;
        __atomic_store_n(&ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return PQ_OK;
}

}  // namespace

extern "C" {

int pq_subitem_scores(const float* queries, const float* centroids, float* S, int B, int d, int m, int b,
                      void* stream) {
    if (!queries || !centroids || !S) return PQ_ERR_NULL;
    if (B < 1 || d < 1 || m < 1 || b < 1 || b > 65536 || d % m != 0) return PQ_ERR_SHAPE;
    if (B > PQ_MAX_B || m > PQ_MAX_M) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)queries & 3) || ((uintptr_t)centroids & 3) || ((uintptr_t)S & 3)) return PQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (B >= kSubMfmaMinBatch && !(g_force_general.load(std::memory_order_relaxed) & 4) &&
        launch_subitem_mfma(queries, centroids, S, B, d, m, b, (long long)m * b, st))
        return record_hip(hipGetLastError());
    switch (d / m) {
        case 4: launch_subitem<4>(queries, centroids, S, B, d, m, b, st); break;
        case 8: launch_subitem<8>(queries, centroids, S, B, d, m, b, st); break;
        case 16: launch_subitem<16>(queries, centroids, S, B, d, m, b, st); break;
        case 32: launch_subitem<32>(queries, centroids, S, B, d, m, b, st); break;
        case 64: launch_subitem<64>(queries, centroids, S, B, d, m, b, st); break;
        default: launch_subitem<0>(queries, centroids, S, B, d, m, b, st); break;
    }
    return record_hip(hipGetLastError());
}

size_t pq_score_topk_workspace_bytes(long long N, int B, int m, int b, int K) {
    if (check_topk_shape(N, B, m, b, K, 1) != PQ_OK) return 0;
    const ScanPlan p = make_plan(N, B, m, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_score_topk(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                  float* out_scores, void* workspace, size_t workspace_bytes_given, void* stream) {
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_plan(N, B, m, K);
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = enqueue_scan(p, codes, S, N, B, m, b, K, workspace, st);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_score_topk_static(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                         float* out_scores, void* stream) {
    if (!codes || !S || !out_ids || !out_scores) return PQ_ERR_NULL;
    int rc = check_topk_shape(N, B, m, b, K, 1);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_plan(N, B, m, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)codes & 15) || ((uintptr_t)S & 3) || ((uintptr_t)out_ids & 3) || ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes(p, B, K) > kStaticScratchBytes) return PQ_ERR_TOO_LARGE;
    void* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != PQ_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = enqueue_scan(p, codes, S, N, B, m, b, K, ws, st);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, ws, out_ids, out_scores, st);
}

}  // extern "C"

namespace {
// scan launches of a pq_score_topk / pq_score_topk_u16 call timed between two events (one untimed launch first)
int profile_scan(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                 float* out_scores, void* workspace, size_t workspace_bytes_given, void* stream, int iters,
                 float* scan_ms, int cw) {
    if (!scan_ms) return PQ_ERR_NULL;
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given, cw);
    if (rc != PQ_OK) return rc;
    if (iters < 1) return PQ_ERR_SHAPE;
    const ScanPlan p = make_plan(N, B, m, K, false, cw, b);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    hipError_t e = hipEventCreate(&ev0);
    if (e != hipSuccess) return record_hip(e);
    e = hipEventCreate(&ev1);
    if (e != hipSuccess) { (void)hipEventDestroy(ev0); return record_hip(e); }
    auto scan = [&]() { return enqueue_scan(p, codes, S, N, B, m, b, K, workspace, st, nullptr, 0, cw); };
    rc = scan();                                                            // untimed warm-up launch
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev0, st));
    for (int it = 0; it < iters && rc == PQ_OK; ++it) rc = scan();
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev1, st));
    if (rc == PQ_OK) rc = enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
    if (rc == PQ_OK) rc = record_hip(hipStreamSynchronize(st));
    float ms = 0.0f;
    if (rc == PQ_OK) rc = record_hip(hipEventElapsedTime(&ms, ev0, ev1));
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    if (rc == PQ_OK) *scan_ms = ms / (float)iters;
    return rc;
}
}  // namespace

extern "C" {

int pq_score_topk_profile(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                          int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes_given,
                          void* stream, int iters, float* scan_ms) {
    return profile_scan(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given, stream, iters,
                        scan_ms, 1);
}

int pq_measure_force_general(int mask) {
    return g_force_general.exchange(mask & 7, std::memory_order_relaxed);
}

int pq_measure_step_stamps(const float* queries, const float* centroids, const uint8_t* codes, long long N, int B,
                           int d, int m, int b, int K, float* S, int* out_ids, float* out_scores, void* workspace,
                           size_t workspace_bytes_given, uint64_t* stamps, size_t stamps_bytes, int* scan_grid,
                           void* stream) {
    if (!queries || !centroids || !S || !stamps) return PQ_ERR_NULL;
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given);
    if (rc != PQ_OK) return rc;
    if (d < 1 || d % m != 0) return PQ_ERR_SHAPE;
    if (((uintptr_t)queries & 3) || ((uintptr_t)centroids & 3) || ((uintptr_t)stamps & 7)) return PQ_ERR_ALIGN;
    if (stamps_bytes < PQ_STAMP_BYTES) return PQ_ERR_WORKSPACE;
    static_assert(PQ_STAMP_SLOTS == kStampSlots, "header and kernels agree on the record size");
    const ScanPlan p = make_plan(N, B, m, K);
    if (!(p.tiled || m == 8)) return PQ_ERR_UNSUPPORTED;       // (scan kernels with a measurement instance)
    const int waves = (!p.tiled && p.big) ? kMaxWaves : kWaves;   // (the batched kernel: always kWaves)
    const long long scan_groups = p.tiled ? (long long)p.nblk * ((B + kQ - 1) / kQ) : (long long)p.nblk * B;
    if (scan_groups * waves > PQ_STAMP_RECORDS || (long long)B * kWaves > PQ_STAMP_RECORDS) return PQ_ERR_UNSUPPORTED;
    if (scan_grid != nullptr) { scan_grid[0] = (int)scan_groups; scan_grid[1] = waves; }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t section = (size_t)PQ_STAMP_RECORDS * PQ_STAMP_SLOTS;
    if (B == 1 && d / m == 64 && (m * b + kSubThreads - 1) / kSubThreads <= PQ_STAMP_RECORDS) {
        if (((long long)m * b) % kSubThreads == 0 && ((uintptr_t)centroids & 15) == 0)
            hipLaunchKernelGGL((subitem_scores_kernel<64, true, true>), dim3(m * b / kSubThreads, 1), dim3(kSubThreads), 0,
                               st, queries, centroids, S, B, d, m, b, stamps);
        else
            hipLaunchKernelGGL((subitem_scores_kernel<64, true>), dim3((m * b + kSubThreads - 1) / kSubThreads, 1), dim3(kSubThreads), 0,
                               st, queries, centroids, S, B, d, m, b, stamps);
        rc = record_hip(hipGetLastError());
    } else {
        rc = pq_subitem_scores(queries, centroids, S, B, d, m, b, stream);   // (no measurement instance: section 0 stays empty)
    }
    if (rc != PQ_OK) return rc;
    rc = enqueue_scan(p, codes, S, N, B, m, b, K, workspace, st, nullptr, 0, 1, stamps + section);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st, stamps + 2 * section);
}

size_t pq_score_topk_u16_workspace_bytes(long long N, int B, int m, int b, int K) {
    if (check_topk_shape(N, B, m, b, K, 2) != PQ_OK) return 0;
    const ScanPlan p = make_plan(N, B, m, K, false, 2, b);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_score_topk_u16(const uint16_t* codes, const float* S, long long N, int B, int m, int b, int K, int* out_ids,
                      float* out_scores, void* workspace, size_t workspace_bytes_given, void* stream) {
    int rc = check_topk_args(codes, S, N, B, m, b, K, out_ids, out_scores, workspace, workspace_bytes_given, 2);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_plan(N, B, m, K, false, 2, b);
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = enqueue_scan(p, reinterpret_cast<const uint8_t*>(codes), S, N, B, m, b, K, workspace, st, nullptr, 0, 2);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_score_topk_u16_profile(const uint16_t* codes, const float* S, long long N, int B, int m, int b, int K,
                              int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes_given,
                              void* stream, int iters, float* scan_ms) {
    return profile_scan(reinterpret_cast<const uint8_t*>(codes), S, N, B, m, b, K, out_ids, out_scores, workspace,
                        workspace_bytes_given, stream, iters, scan_ms, 2);
}

size_t pq_score_topk_subset_workspace_bytes(long long n_subset, int B, int m, int b, int K) {
    if (n_subset < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > n_subset || n_subset >= 2147483648LL) return 0;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return 0;
    const ScanPlan p = make_plan(n_subset, B, m, K, true);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_score_topk_subset(const uint8_t* codes, const float* S, const int* subset, long long n_subset, long long N,
                         int B, int m, int b, int K, int* out_ids, float* out_scores, void* workspace,
                         size_t workspace_bytes_given, void* stream) {
    if (!codes || !S || !subset || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    if (n_subset < 1 || N < 1 || B < 1 || m < 1 || b < 1 || K < 1 || b > 256 || K > n_subset || n_subset > N ||
        N >= 2147483648LL)
        return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    const ScanPlan p = make_plan(n_subset, B, m, K, true);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)codes & 15) || ((uintptr_t)workspace & 15) || ((uintptr_t)S & 3) || ((uintptr_t)subset & 3) ||
        ((uintptr_t)out_ids & 3) || ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(p, B, K)) return PQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = enqueue_scan(p, codes, S, n_subset, B, m, b, K, workspace, st, subset, N);
    if (rc != PQ_OK) return rc;
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_read_bandwidth_profile(const void* data, size_t bytes, void* stream, int iters, float* read_ms) {
    if (!data || !read_ms) return PQ_ERR_NULL;
    if (bytes < 16 || iters < 1) return PQ_ERR_SHAPE;
    if ((uintptr_t)data & 15) return PQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const long long nvec = (long long)(bytes / 16);
    long long blocks = (nvec + kReadThreads - 1) / kReadThreads;
    if (blocks > 2LL * kAssumedCUs) blocks = 2LL * kAssumedCUs;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    hipError_t e = hipEventCreate(&ev0);
    if (e != hipSuccess) return record_hip(e);
    e = hipEventCreate(&ev1);
    if (e != hipSuccess) { (void)hipEventDestroy(ev0); return record_hip(e); }
    auto launch = [&]() {
        hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(kReadThreads), 0, st,
                           static_cast<const uint4*>(data), nvec);
        return record_hip(hipGetLastError());
    };
    int rc = launch();                                       // untimed warm-up launch
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev0, st));
    for (int it = 0; it < iters && rc == PQ_OK; ++it) rc = launch();
    if (rc == PQ_OK) rc = record_hip(hipEventRecord(ev1, st));
    if (rc == PQ_OK) rc = record_hip(hipStreamSynchronize(st));
    float ms = 0.0f;
    if (rc == PQ_OK) rc = record_hip(hipEventElapsedTime(&ms, ev0, ev1));
    (void)hipEventDestroy(ev0);
    (void)hipEventDestroy(ev1);
    if (rc == PQ_OK) *read_ms = ms / (float)iters;
    return rc;
}

// ---- the comparison scorers (Section 2's default scoring, Algorithm 2) and TopK over score rows

namespace {
// plan of pq_topk_scores: blocks per query, list and candidate sizes (as for the scan), LDS of the two launches
ScanPlan make_topk_scores_plan(long long N, int B, int K) {
    ScanPlan p = {};
    const long long vecs = N / 4;
    const long long per_round = (long long)kThreads * kScoreVecs;
    long long rounds = (vecs + per_round - 1) / per_round;
    if (rounds < 1) rounds = 1;
    long long most = (kBlocksPerCU * (long long)kAssumedCUs) / B;
    if (most < 8) most = 8;
    p.nblk = (int)(rounds < most ? rounds : most);
    p.cap = list_capacity(K);
    p.candmax = next_pow2(2 * K);
    if (p.candmax < 512) p.candmax = 512;
    p.stage_keys = next_pow2(2 * K);
    if (p.stage_keys < kChunkKeys) p.stage_keys = kChunkKeys;
    p.copies = 1;
    p.scan_dyn_lds = p.scan_lds = scan_lds_bytes(0, p.cap, p.candmax, K, kWaves);
    p.fold_lds = fold_lds_bytes(p.stage_keys, p.candmax, K);
    return p;
}

int check_topk_scores_shape(long long ld, long long N, int B, int K) {
    if (N < 1 || B < 1 || K < 1 || K > N || ld < N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (K > PQ_MAX_K || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    return PQ_OK;
}
}  // namespace

size_t pq_topk_scores_workspace_bytes(long long N, int B, int K) {
    if (check_topk_scores_shape(N, N, B, K) != PQ_OK) return 0;
    const ScanPlan p = make_topk_scores_plan(N, B, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return 0;
    return workspace_bytes(p, B, K);
}

int pq_topk_scores(const float* scores, long long ld, long long N, int B, int K, int* out_ids, float* out_scores,
                   void* workspace, size_t workspace_bytes_given, void* stream) {
    if (!scores || !out_ids || !out_scores || !workspace) return PQ_ERR_NULL;
    int rc = check_topk_scores_shape(ld, N, B, K);
    if (rc != PQ_OK) return rc;
    const ScanPlan p = make_topk_scores_plan(N, B, K);
    if (p.scan_lds > kMaxLdsBytes || p.fold_lds > kMaxLdsBytes) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)scores & 15) || (B > 1 && (ld & 3)) || ((uintptr_t)workspace & 15) || ((uintptr_t)out_ids & 3) ||
        ((uintptr_t)out_scores & 3))
        return PQ_ERR_ALIGN;
    if (workspace_bytes_given < workspace_bytes(p, B, K)) return PQ_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    TopkScoresArgs a;
    a.scores = scores; a.ld = ld; a.N = N; a.K = K; a.cap = p.cap; a.candmax = p.candmax;
    a.prune_at = (K <= 28) ? 2 * K + 8 : 0;
    a.ws_keys = static_cast<uint64_t*>(workspace);
    hipError_t e = allow_lds(topk_scores_kernel, p.scan_dyn_lds);
    if (e != hipSuccess) return record_hip(e);
    hipLaunchKernelGGL(topk_scores_kernel, dim3(p.nblk, B), dim3(kThreads), p.scan_dyn_lds, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return record_hip(e);
    return enqueue_fold(p, B, K, workspace, out_ids, out_scores, st);
}

int pq_recjpq_scores(const uint8_t* codes, const float* S, long long N, int B, int m, int b, float* scores,
                     long long ld, void* stream) {
    if (!codes || !S || !scores) return PQ_ERR_NULL;
    if (N < 1 || B < 1 || m < 1 || b < 1 || b > 256 || ld < N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (m > PQ_MAX_M || B > PQ_MAX_B) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)S & 3) || ((uintptr_t)scores & 3)) return PQ_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((N + 4LL * kRecjpqThreads - 1) / (4LL * kRecjpqThreads)), B);
    for (int k = 0; k < m; ++k) {                            // Algorithm 2's outer loop: one pass over the items per split
        hipLaunchKernelGGL(recjpq_pass_kernel, grid, dim3(kRecjpqThreads), 0, st, codes, S, scores, ld, N, m, b, k);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return record_hip(e);
    }
    return PQ_OK;
}

int pq_reconstruct_items(const uint8_t* codes, const float* centroids, long long N, int d, int m, int b, float* W,
                         void* stream) {
    if (!codes || !centroids || !W) return PQ_ERR_NULL;
    if (N < 1 || d < 1 || m < 1 || b < 1 || b > 256 || d % m != 0 || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (m > PQ_MAX_M) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)centroids & 3) || ((uintptr_t)W & 3)) return PQ_ERR_ALIGN;
    const long long total = N * d;
    long long blocks = (total + 255) / 256;
    if (blocks > 64 * kAssumedCUs) blocks = 64 * kAssumedCUs;
    hipLaunchKernelGGL(reconstruct_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), codes,
                       centroids, W, N, d, m, b);
    return record_hip(hipGetLastError());
}

int pq_default_scores(const float* W, const float* queries, long long N, int B, int d, float* scores, long long ld,
                      void* stream) {
    if (!W || !queries || !scores) return PQ_ERR_NULL;
    if (N < 1 || B < 1 || d < 1 || ld < N || N >= 2147483648LL) return PQ_ERR_SHAPE;
    if (B > PQ_MAX_B || d % 4 != 0 || (size_t)d * sizeof(float) > 64 * 1024) return PQ_ERR_UNSUPPORTED;
    if (((uintptr_t)W & 15) || ((uintptr_t)queries & 15) || ((uintptr_t)scores & 3)) return PQ_ERR_ALIGN;
    // batches: one pass over W for all queries, on the matrix cores (the same kernel as Eq. 4: one split, the items in
    // the place of the sub-ids); a single query, or a shape that kernel does not take: one mat-vec pass per query
    if (B >= kDefaultMfmaMinBatch && !(g_force_general.load(std::memory_order_relaxed) & 4) &&
        launch_subitem_mfma(queries, W, scores, B, d, 1, N, ld, static_cast<hipStream_t>(stream)))
        return record_hip(hipGetLastError());
    long long blocks = (N + kDefaultThreads / 16 - 1) / (kDefaultThreads / 16);
    if (blocks > 16 * kAssumedCUs) blocks = 16 * kAssumedCUs;
    hipLaunchKernelGGL(default_scores_kernel, dim3((unsigned)blocks, B), dim3(kDefaultThreads), (size_t)d * sizeof(float),
                       static_cast<hipStream_t>(stream), W, queries, scores, ld, N, d);
    return record_hip(hipGetLastError());
}

const char* pq_strerror(int code) {
    switch (code) {
        case PQ_OK: return "ok";
        case PQ_ERR_NULL: return "a required pointer is NULL";
        case PQ_ERR_SHAPE:
            return "bad shape: need B,d,m,b,K,N >= 1, d % m == 0, b <= 256 (65536 with 16-bit sub-ids), K <= N (K <= |V| <= N with a "
                   "candidate list), N < 2^31";
        case PQ_ERR_UNSUPPORTED:
            return "unsupported: K > 512, m > 128, B > 65535, or score tables plus candidate lists exceed LDS";
        case PQ_ERR_WORKSPACE: return "workspace smaller than pq_score_topk_workspace_bytes()";
        case PQ_ERR_ALIGN: return "pointer alignment: codes and workspace 16 bytes, float/int arrays 4 bytes";
        case PQ_ERR_HIP: return g_hip_error;
        case PQ_ERR_TOO_LARGE: return "problem needs more scratch than the library's built-in array holds (PQ_STATIC_SCRATCH_BYTES)";
        default: return "unknown pqtopk error code";
    }
}

}  // extern "C"
