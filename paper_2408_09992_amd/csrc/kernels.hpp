// Device code of the PQTopK library: every kernel template, in namespace pqk, and the list of scan-kernel instances.
//
// The catalogue-scan kernels are large (40-120 KB of code each), so they are compiled in translation units of their
// own (inst_*.hip, each instantiating one group of the list below); every other translation unit sees them as
// `extern template` and only launches them.  The small kernels (Eq. 4, fold, comparison scorers) are instantiated
// where they are launched.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pqk {

#include "common.hpp"
#include "subitem_scores.hpp"
#include "topk_parts.hpp"
#include "select_small.hpp"
#include "scan_single.hpp"
#include "scan_short.hpp"
#include "scan_subset.hpp"
#include "scan_batched.hpp"
#include "fold.hpp"
#ifndef PQ_INSTANCE_TU
#include "comparison.hpp"   // (kernels that are no templates: defined once, in the translation unit that launches them)
#endif

// scan_topk_kernel<M, C, NT, CW, GL> instances, by translation unit.  X(M, C, NT, CW, GL).
// one-byte sub-ids, rows of 1, 2 and 4 bytes (each with and without replicated tables)
#define PQ_SCAN_INSTANCES_U8_NARROW(X) \
    X(1, kTableCopies, kBigThreads, 1, false) X(1, 1, kThreads, 1, false) \
    X(2, kTableCopies, kBigThreads, 1, false) X(2, 1, kThreads, 1, false) \
    X(4, kTableCopies, kBigThreads, 1, false) X(4, 1, kThreads, 1, false)
// one-byte sub-ids, m = 8 and 16 (the named workloads)
#define PQ_SCAN_INSTANCES_U8_MAIN(X) \
    X(8, kTableCopies, kBigThreads, 1, false) X(8, 1, kThreads, 1, false) X(16, 1, kThreads, 1, false)
// one-byte sub-ids, m = 32 and 64
#define PQ_SCAN_INSTANCES_U8_WIDE(X) \
    X(32, 1, kThreads, 1, false) X(64, 1, kBigThreads, 1, false) X(64, 1, kThreads, 1, false)
// any m, row by row (also the candidate-list scan)
#define PQ_SCAN_INSTANCES_GENERIC(X) \
    X(0, 1, kBigThreads, 1, false) X(0, 1, kThreads, 1, false) \
    X(0, 1, kThreads, 2, true) X(0, 1, kBigThreads, 2, false) X(0, 1, kThreads, 2, false)
// two-byte sub-ids, rows of 8, 16 and 32 bytes
#define PQ_SCAN_INSTANCES_U16(X) \
    X(4, 1, kThreads, 2, true) X(4, 1, kBigThreads, 2, false) X(4, 1, kThreads, 2, false) \
    X(8, 1, kThreads, 2, true) X(8, 1, kBigThreads, 2, false) X(8, 1, kThreads, 2, false) \
    X(16, 1, kThreads, 2, true) X(16, 1, kBigThreads, 2, false) X(16, 1, kThreads, 2, false)
// measurement instances (wall-clock stamps per wave) of the two kernels the named single-query workloads run
#define PQ_SCAN_INSTANCES_STAMPED(X) X(8, 1, kThreads, 1, false, true) X(8, kTableCopies, kBigThreads, 1, false, true)
// scan_short_kernel<M, U, NT, STAMP> instances: every number of units per thread up to short_max_units(M), in three
// translation units; measurement instances for m = 8
#define PQ_SHORT_U(X, M, U) X(M, U, kThreads, false)
#define PQ_SHORT_U4(X, M, U) PQ_SHORT_U(X, M, U) PQ_SHORT_U(X, M, U + 1) PQ_SHORT_U(X, M, U + 2) PQ_SHORT_U(X, M, U + 3)
#define PQ_SHORT_INSTANCES_A(X) \
    PQ_SHORT_U4(X, 8, 1) PQ_SHORT_U4(X, 8, 5) PQ_SHORT_U4(X, 8, 9) \
    X(8, 1, kThreads, true) X(8, 2, kThreads, true) X(8, 3, kThreads, true) X(8, 4, kThreads, true) X(8, 5, kThreads, true) \
    X(8, 6, kThreads, true) X(8, 7, kThreads, true) X(8, 8, kThreads, true) \
    PQ_SHORT_U(X, 1, 1) PQ_SHORT_U(X, 1, 2) PQ_SHORT_U(X, 2, 1) PQ_SHORT_U(X, 2, 2) \
    PQ_SHORT_U4(X, 4, 1) PQ_SHORT_U(X, 4, 5) PQ_SHORT_U(X, 4, 6)
#define PQ_SHORT_INSTANCES_B(X) \
    PQ_SHORT_U4(X, 16, 1) PQ_SHORT_U4(X, 16, 5) PQ_SHORT_U4(X, 16, 9)
#define PQ_SHORT_INSTANCES_C(X) \
    PQ_SHORT_U4(X, 32, 1) PQ_SHORT_U4(X, 32, 5) PQ_SHORT_U4(X, 64, 1)
// scan_short_kernel<M, U, NT, false, 2>: two-byte sub-ids, m = 4, 8 (up to 12 code vectors per thread), 16 (up to 6 items)
#define PQ_SHORT16_U(X, M, U) X(M, U, kThreads, false, 2)
#define PQ_SHORT16_INSTANCES(X) \
    PQ_SHORT16_U(X, 4, 1) PQ_SHORT16_U(X, 4, 2) PQ_SHORT16_U(X, 4, 3) PQ_SHORT16_U(X, 4, 4) PQ_SHORT16_U(X, 4, 5) PQ_SHORT16_U(X, 4, 6) \
    PQ_SHORT16_U(X, 4, 7) PQ_SHORT16_U(X, 4, 8) PQ_SHORT16_U(X, 4, 9) PQ_SHORT16_U(X, 4, 10) PQ_SHORT16_U(X, 4, 11) PQ_SHORT16_U(X, 4, 12) \
    PQ_SHORT16_U(X, 8, 1) PQ_SHORT16_U(X, 8, 2) PQ_SHORT16_U(X, 8, 3) PQ_SHORT16_U(X, 8, 4) PQ_SHORT16_U(X, 8, 5) PQ_SHORT16_U(X, 8, 6) \
    PQ_SHORT16_U(X, 8, 7) PQ_SHORT16_U(X, 8, 8) PQ_SHORT16_U(X, 8, 9) PQ_SHORT16_U(X, 8, 10) PQ_SHORT16_U(X, 8, 11) PQ_SHORT16_U(X, 8, 12) \
    PQ_SHORT16_U(X, 16, 1) PQ_SHORT16_U(X, 16, 2) PQ_SHORT16_U(X, 16, 3) PQ_SHORT16_U(X, 16, 4) PQ_SHORT16_U(X, 16, 5) PQ_SHORT16_U(X, 16, 6)
// scan_subset_kernel<M, U, NT>: rows of 4, 8, 16 bytes, every number of vectors per thread
#define PQ_SUBSET_M(X, M) X(M, 1, kThreads) X(M, 2, kThreads) X(M, 3, kThreads) X(M, 4, kThreads) X(M, 5, kThreads) \
    X(M, 6, kThreads) X(M, 7, kThreads) X(M, 8, kThreads)
#define PQ_SUBSET_INSTANCES(X) PQ_SUBSET_M(X, 4) PQ_SUBSET_M(X, 8) PQ_SUBSET_M(X, 16)
// the batched kernel
#define PQ_TILED_INSTANCES(X) X(8, false) X(16, false) X(8, true) X(16, true)

#define PQ_SCAN_DEFINE(M, C, NT, CW, GL) template __global__ void scan_topk_kernel<M, C, NT, CW, GL>(ScanArgs);
#define PQ_SCAN_EXTERN(M, C, NT, CW, GL) extern PQ_SCAN_DEFINE(M, C, NT, CW, GL)
#define PQ_SCAN_DEFINE6(M, C, NT, CW, GL, ST) template __global__ void scan_topk_kernel<M, C, NT, CW, GL, ST>(ScanArgs);
#define PQ_SCAN_EXTERN6(M, C, NT, CW, GL, ST) extern PQ_SCAN_DEFINE6(M, C, NT, CW, GL, ST)
#define PQ_SHORT_DEFINE(M, U, NT, ST) template __global__ void scan_short_kernel<M, U, NT, ST>(ScanArgs);
#define PQ_SHORT_EXTERN(M, U, NT, ST) extern PQ_SHORT_DEFINE(M, U, NT, ST)
#define PQ_SHORT16_DEFINE(M, U, NT, ST, CW) template __global__ void scan_short_kernel<M, U, NT, ST, CW>(ScanArgs);
#define PQ_SHORT16_EXTERN(M, U, NT, ST, CW) extern PQ_SHORT16_DEFINE(M, U, NT, ST, CW)
#define PQ_SUBSET_DEFINE(M, U, NT) template __global__ void scan_subset_kernel<M, U, NT>(ScanArgs);
#define PQ_SUBSET_EXTERN(M, U, NT) extern PQ_SUBSET_DEFINE(M, U, NT)
#define PQ_TILED_DEFINE(M, ST) template __global__ void scan_topk_tiled_kernel<M, ST>(ScanArgs, int);
#define PQ_TILED_EXTERN(M, ST) extern PQ_TILED_DEFINE(M, ST)

#ifndef PQ_INSTANCE_TU
PQ_SCAN_INSTANCES_U8_NARROW(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_U8_MAIN(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_U8_WIDE(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_GENERIC(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_U16(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_STAMPED(PQ_SCAN_EXTERN6)
PQ_SHORT_INSTANCES_A(PQ_SHORT_EXTERN)
PQ_SHORT_INSTANCES_B(PQ_SHORT_EXTERN)
PQ_SHORT_INSTANCES_C(PQ_SHORT_EXTERN)
PQ_SUBSET_INSTANCES(PQ_SUBSET_EXTERN)
PQ_SHORT16_INSTANCES(PQ_SHORT16_EXTERN)
PQ_TILED_INSTANCES(PQ_TILED_EXTERN)
#endif

}  // namespace pqk
