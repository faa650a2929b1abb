/*
 * pqtopk_measure.h -- measurement aids of the PQTopK library (libpqtopk.so).
 *
 * None of these is on the product path (include/pqtopk.h is).  They exist so that every figure quoted for the kernels
 * can be re-measured: the scan kernel's own duration, in-kernel wall-clock stamps of the three launches of a step,
 * and the machine yardsticks the figures are held against (an empty launch, a plain streaming read, random gathers
 * from LDS).  Unlike the product entry points they create and destroy HIP events and WAIT for the stream; none
 * allocates device memory.  Pointers are device pointers unless marked (host).  Return values as in pqtopk.h.
 */
#ifndef PQTOPK_MEASURE_H
#define PQTOPK_MEASURE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues the catalogue scan kernel of pq_score_topk() (the kernel that streams `codes`) once
 * untimed and then `iters` times back to back between two HIP events on `stream`, enqueues the fold so the outputs
 * are those of pq_score_topk(), waits for the stream, and stores elapsed / iters in milliseconds in *scan_ms (host
 * pointer): the scan kernel's mean duration including its launch gap.  Like every entry point of this header it synchronises and
 * creates / destroys HIP events.  Same errors as pq_score_topk(); PQ_ERR_SHAPE if iters < 1.
 */
int pq_score_topk_profile(const uint8_t* codes, const float* S, long long N, int B, int m, int b, int K,
                          int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes,
                          void* stream, int iters, float* scan_ms);

/* pq_score_topk_profile() for 16-bit sub-ids: times the scan kernel of pq_score_topk_u16(). */
int pq_score_topk_u16_profile(const uint16_t* codes, const float* S, long long N, int B, int m, int b, int K,
                              int* out_ids, float* out_scores, void* workspace, size_t workspace_bytes,
                              void* stream, int iters, float* scan_ms);

/*
 * A plain streaming-read kernel (16-byte loads and nothing else) over `bytes` bytes at `data`
 * (device pointer, 16-byte aligned), launched once untimed and then `iters` times back to back between two HIP events;
 * *read_ms (host pointer) receives elapsed / iters in milliseconds.  The yardstick for the scan's HBM rate: what this
 * machine delivers to a kernel that does nothing but read.  Synchronises; creates and destroys two HIP events.
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE (bytes < 16, iters < 1), PQ_ERR_ALIGN, PQ_ERR_HIP.
 */
int pq_read_bandwidth_profile(const void* data, size_t bytes, void* stream, int iters, float* read_ms);

/*
 * An empty kernel (it reads its arguments and ends) on a grid of `blocks` workgroups of `threads` threads, launched
 * once untimed and then `iters` times back to back between two HIP events: *launch_ms (host) receives elapsed / iters
 * in milliseconds, the cost of a launch that has nothing to do.  Errors: PQ_ERR_NULL, PQ_ERR_SHAPE (blocks, iters < 1,
 * threads not in 64 .. 1024 or not a multiple of 64), PQ_ERR_HIP.
 */
int pq_measure_empty_launch(int blocks, int threads, void* stream, int iters, float* launch_ms);

/*
 * Random gathers from LDS, the operation that bounds Eq. 5 once a batch shares the code stream: every lane of every
 * wave reads `rounds` times `width` bytes (4, 8 or 16) at a pseudo-random, width-aligned offset inside a table of
 * `table_bytes` bytes (a power of two, 1 KiB .. 128 KiB) that its workgroup has filled in LDS; offsets come from a
 * per-lane hash and do not depend on what was read, so reads overlap as they do in the scan.  `copies` (a power of
 * two, 1 .. 64) reads the table as entries of `copies` adjacent words, lane l reading word l % copies of a random
 * entry: the layout of the scan's replicated tables.  `conflict_free` != 0 makes the lanes of a wave read 64
 * consecutive words instead (the best case the LDS allows; copies is ignored).  Grid: `blocks` workgroups of `threads` threads.  One untimed launch, then `iters` timed back to back;
 * *gather_ms (host) receives elapsed / iters.  The caller derives lane reads per clock and CU from
 * blocks * threads * rounds / time.  `sink` (device, at least 4 bytes) receives a value nobody needs.
 * Errors: PQ_ERR_NULL, PQ_ERR_SHAPE (width, table_bytes, rounds, blocks, threads, iters out of range), PQ_ERR_HIP.
 */
int pq_measure_lds_gather(int width, int table_bytes, int rounds, int conflict_free, int copies, int blocks, int threads,
                          uint32_t* sink, void* stream, int iters, float* gather_ms);

/*
 * What synchronising inside one launch costs on this machine, against a launch boundary: the reason a step stays three
 * launches.  Each variant is launched once untimed and then `iters` times back to back on `stream` between two HIP
 * events; *variant_ms (host) receives elapsed / iters.  The kernels are stand-ins that do the synchronisation and the
 * memory traffic of a scheme and none of its arithmetic (grid of 256 workgroups of 512 threads, as the single-query scan):
 *   PQ_SYNC_EMPTY                      an empty kernel on that grid: the floor
 *   PQ_SYNC_FOLD_LAUNCH                every workgroup writes 10 keys; a second launch of one workgroup reads all 2560
 *   PQ_SYNC_LAST_FOLDS_FENCED          one launch: ... acquire-release ticket, the last workgroup to arrive reads them
 *   PQ_SYNC_LAST_FOLDS_RELAXED         ... keys written through and read with agent-scope accesses, relaxed ticket
 *   PQ_SYNC_LAST_FOLDS_RELAXED_2LEVEL  ... sixteen group tickets, then one (a self-resetting two-level ticket)
 *   PQ_SYNC_EQ4_LAUNCH                 Eq. 4 (2048 chains of 64 multiply-adds) as its own launch, then a launch in which
 *                                      every workgroup loads the 8 KB table into LDS
 *   PQ_SYNC_EQ4_BARRIER_FENCED         one launch: Eq. 4 spread over the grid, a grid-wide barrier on generation tags
 *                                      (release store, acquire fence), then every workgroup loads the table
 *   PQ_SYNC_EQ4_BARRIER_RELAXED        ... with agent-scope relaxed accesses and no fence
 * Every wait in these kernels is bounded.  `scratch`: device memory, 256-byte aligned, at least PQ_SYNC_SCRATCH_BYTES;
 * it is zeroed here.  Errors: PQ_ERR_NULL, PQ_ERR_SHAPE, PQ_ERR_ALIGN, PQ_ERR_WORKSPACE, PQ_ERR_HIP.
 */
#define PQ_SYNC_EMPTY                      0
#define PQ_SYNC_FOLD_LAUNCH                1
#define PQ_SYNC_LAST_FOLDS_FENCED          2
#define PQ_SYNC_LAST_FOLDS_RELAXED         3
#define PQ_SYNC_LAST_FOLDS_RELAXED_2LEVEL  4
#define PQ_SYNC_EQ4_LAUNCH                 5
#define PQ_SYNC_EQ4_BARRIER_FENCED         6
#define PQ_SYNC_EQ4_BARRIER_RELAXED        7
#define PQ_SYNC_VARIANTS                   8
#define PQ_SYNC_SCRATCH_BYTES ((size_t)2 << 20)
int pq_measure_sync_variant(int variant, void* scratch, size_t scratch_bytes, void* stream, int iters, float* variant_ms);

/*
 * Which kernels single-query calls with small K take, for A/B measurement and for tests that must reach the general
 * kernels on shapes the lean ones would serve.  mask bit 0: catalogue scans never take the short kernel (scores in
 * registers, one selection) but the general scan kernel; bit 1: folds never take the small-K fold but the general
 * one; bit 2: Eq. 4 never runs on the matrix cores but in the scalar kernels.  0 restores the library's own choice.  Process-wide, takes effect for calls made after it returns (workspace
 * sizes do not depend on it).  Returns the previous mask.
 */
int pq_measure_force_general(int mask);

/*
 * One whole step (pq_subitem_scores, then pq_score_topk's scan and fold launches) with the measurement instances of
 * the three kernels, which record wall-clock stamps (hipDeviceAttributeWallClockRate ticks, 100 MHz on MI355X) at
 * fixed points: lane 0 of every wave writes PQ_STAMP_SLOTS 64-bit values.  Results (S, ids, scores) are those of the
 * product entry points.  Measurement instances exist for the scans of single-query calls with m = 8 (short and long)
 * and for the batched scan (m = 8 and 16), for both folds, and for Eq. 4 at batch 1 with d / m = 64 (otherwise the
 * product's Eq. 4 kernel runs and section 0 stays as it was); PQ_ERR_UNSUPPORTED for other shapes.
 *   stamps       out  uint64 [3][PQ_STAMP_RECORDS][PQ_STAMP_SLOTS]: section 0 = the Eq. 4 kernel (one record per
 *                     workgroup), section 1 = the scan kernel (record = workgroup * waves + wave, workgroups numbered
 *                     blockIdx.y * gridDim.x + blockIdx.x), section 2 = the fold kernel (record = query * waves + wave).  Slots a kernel does not pass are left as they were: zero the
 *                     buffer first.  Slot meanings: PQ_STAMP_* below.
 *   stamps_bytes      at least PQ_STAMP_BYTES
 *   scan_grid    out  (host, may be NULL) [0] = scan workgroups, [1] = waves per scan workgroup
 * Enqueues on `stream` and returns; does not wait.
 */
#define PQ_STAMP_SLOTS    16
#define PQ_STAMP_RECORDS  8192
#define PQ_STAMP_BYTES    ((size_t)3 * PQ_STAMP_RECORDS * PQ_STAMP_SLOTS * 8)
#define PQ_STAMP_ENTRY      0   /* first instruction of the wave */
#define PQ_STAMP_REQUESTED  1   /* scan: table values and the first two rounds of codes requested */
#define PQ_STAMP_TABLES     2   /* scan: tables in LDS, workgroup barrier passed */
#define PQ_STAMP_CODES      3   /* scan: the first rounds' codes have arrived */
#define PQ_STAMP_SCORED     4   /* scan: all items scored (scans of at most two rounds) / first round scored */
#define PQ_STAMP_OFFERED    5   /* scan: the wave's candidates compacted / first-round cut found */
#define PQ_STAMP_STREAMED   6   /* scan: all rounds streamed (scans of more than two rounds) */
#define PQ_STAMP_SELECTED   7   /* scan and fold: the K best ranked */
#define PQ_STAMP_END        8   /* last instruction of the wave */
#define PQ_STAMP_LOADED     9   /* fold: the lists' keys are in registers */
#define PQ_STAMP_CUT       10   /* fold: histogram cut found */
#define PQ_STAMP_COLLECTED 11   /* fold: candidates collected */
int pq_measure_step_stamps(const float* queries, const float* centroids, const uint8_t* codes, long long N, int B,
                           int d, int m, int b, int K, float* S, int* out_ids, float* out_scores, void* workspace,
                           size_t workspace_bytes, uint64_t* stamps, size_t stamps_bytes, int* scan_grid, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PQTOPK_MEASURE_H */
