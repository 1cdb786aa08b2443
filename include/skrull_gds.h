/*
 * skrull_gds.h -- C ABI of the host-side GDS scheduler: how the global batch of one
 * training iteration is split over the DP ranks and, on each, into micro-batches that
 * DACP can schedule (paper Sec. 4.2 for the joint problem; Sec. 4.3.2, Alg. 2 for the
 * heuristic; App. B.2 for FLOPs(S)).  Each micro-batch it returns, with the DACP
 * decisions already taken, is the input of skrull_dacp_rank_batch and from there of
 * skrull_attn_plan.  Host code only; nothing here touches the GPU.
 *
 * Readings of the listing, which is garbled in places:
 *   - Binpack is not named: longest-processing-time greedy, i.e. sequences by
 *     descending FLOPs(S) (equal costs in the caller's order), each to the DP rank
 *     with the least load so far (lowest rank among equals);
 *   - the first attempt uses ceil(Sum(Subset) / (C*N)) micro-batches (at least one),
 *     the fewest the token limit allows, and every failed attempt adds one;
 *   - an attempt with m micro-batches is Subset[j::m], j = 0..m-1, on the subset sorted
 *     ascending (stable); empty ones (m > |Subset|) are dropped;
 *   - a micro-batch is rejected if its tokens EXCEED C*N (the constraint allows
 *     equality although the listing prints >=) or if DACP reports a scheduling error;
 *   - the run fails when one sequence per micro-batch is still rejected;
 *   - a DP rank whose bin is empty has zero micro-batches.
 */
#ifndef SKRULL_GDS_H
#define SKRULL_GDS_H

#include <stdint.h>

#include "skrull_dacp.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Alg. 2, line 1.  seq_len[K] (each >= 1), K in 1..2^20, dp_world_size ws in 1..65536.
 * dp_bin[k] receives the DP rank (0..ws-1) of sequence k.
 * SKRULL_EINVAL: null pointer or a value outside these ranges.  SKRULL_ENOMEM.
 */
int skrull_gds_binpack(int32_t num_seqs, const int32_t *seq_len, int32_t dp_world_size,
                       const skrull_flops_model_t *model, int32_t *dp_bin);

/*
 * Alg. 2 for DP rank `dp_rank`.  bucket_size C >= 1, cp_degree N in 1..65536.
 * All output arrays have K entries, in the caller's sequence order:
 *   dp_bin[k]      DP rank of sequence k (as skrull_gds_binpack);
 *   micro_batch[k] index 0..*num_micro_batches-1 of its micro-batch if dp_bin[k] ==
 *                  dp_rank, else -1;
 *   ret[k]         DACP's decision for it inside that micro-batch (the CP rank that
 *                  keeps it whole, or -1 = distributed) if dp_bin[k] == dp_rank, else -2.
 * SKRULL_ESCHED: some sequence of this rank exceeds C*N tokens (outputs unspecified).
 * SKRULL_EINVAL: null pointer, dp_rank outside [0, ws), or a value outside the ranges.
 */
int skrull_gds_schedule(int32_t num_seqs, const int32_t *seq_len, int64_t bucket_size,
                        int32_t cp_degree, int32_t dp_world_size, int32_t dp_rank,
                        const skrull_flops_model_t *model, int32_t *dp_bin, int32_t *micro_batch,
                        int32_t *ret, int32_t *num_micro_batches);

/*
 * The members of micro-batch `index` under `micro_batch` (as written by
 * skrull_gds_schedule): their positions in the caller's list, by ascending length
 * (equal lengths in the caller's order), into members[] (room for K); *count receives
 * how many.  SKRULL_EINVAL: null pointer, K < 1 or index < 0.
 */
int skrull_gds_micro_batch(int32_t num_seqs, const int32_t *seq_len, const int32_t *micro_batch,
                           int32_t index, int32_t *members, int32_t *count);

#ifdef __cplusplus
}
#endif
#endif /* SKRULL_GDS_H */
