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
#include "scan_single.hpp"
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
// the batched kernel
#define PQ_TILED_INSTANCES(X) X(8) X(16)

#define PQ_SCAN_DEFINE(M, C, NT, CW, GL) template __global__ void scan_topk_kernel<M, C, NT, CW, GL>(ScanArgs);
#define PQ_SCAN_EXTERN(M, C, NT, CW, GL) extern PQ_SCAN_DEFINE(M, C, NT, CW, GL)
#define PQ_TILED_DEFINE(M) template __global__ void scan_topk_tiled_kernel<M>(ScanArgs, int);
#define PQ_TILED_EXTERN(M) extern PQ_TILED_DEFINE(M)

#ifndef PQ_INSTANCE_TU
PQ_SCAN_INSTANCES_U8_NARROW(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_U8_MAIN(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_U8_WIDE(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_GENERIC(PQ_SCAN_EXTERN)
PQ_SCAN_INSTANCES_U16(PQ_SCAN_EXTERN)
PQ_TILED_INSTANCES(PQ_TILED_EXTERN)
#endif

}  // namespace pqk
