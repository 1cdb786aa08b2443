/*
 * skrull_dacp.h -- C ABI of the host-side DACP scheduler: which sequences of a
 * micro-batch stay whole on one context-parallel rank and which are cut over all
 * N ranks (paper Sec. 4.1 for the problem, Eq. 1-8; Sec. 4.3.2, Alg. 1 and
 * App. A.1, Alg. 3 for the heuristic; App. B.2 for FLOPs(S)).  Its output is
 * exactly the input of skrull_attn_plan: per rank, a list of sequence lengths
 * with a shard degree (1 or N) and a shard index.
 *
 * Pure host code (no device work, no allocation visible to the caller, no
 * global state); every array is caller-owned HOST memory.
 *
 * How the listing is read where it is silent or inconsistent:
 *   - ret holds ranks 0..N-1, or -1 for a distributed sequence, in the CALLER's
 *     sequence order; the ascending sort is stable; argmin/argmax take the lowest
 *     rank among equals; S/N is exact (no rounding);
 *   - FLOPs(S, N) is FLOPs(S) / N (Eq. 4);
 *   - a roll-back gives the rank S - S/N tokens of capacity back (the listing
 *     prints the opposite sign) and charges S/N tokens and FLOPs(S)/N to every
 *     other rank as well (Eq. 4, Eq. 8);
 *   - a schedule that would leave any rank over its bucket C (Eq. 8) is a
 *     scheduling error, like a roll-back that finds no local sequence.
 */
#ifndef SKRULL_DACP_H
#define SKRULL_DACP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKRULL_ESCHED (-5)  /* DACP scheduling error: the micro-batch does not fit (Alg. 1) */

/* Model constants of FLOPs(S) = 20 b h^2 S + 4 b h h_kv S + 4 b h S^2 (App. B.2). */
typedef struct {
    int64_t hidden;     /* h,    1 .. 2^20 */
    int64_t hidden_kv;  /* h_kv, 1 .. 2^20 */
    int64_t batch;      /* b,    1 .. 2^10 (1 with sequence packing) */
} skrull_flops_model_t;

/*
 * Alg. 1.  seq_len[K] (each >= 1), bucket_size C >= 1 tokens per rank,
 * cp_degree N in 1..65536, K in 1..2^20.  On SKRULL_OK ret[K] holds, for each
 * sequence in the caller's order, the rank that keeps it whole or -1 if it is
 * distributed; the result satisfies Eq. 7 and Eq. 8.  SKRULL_ESCHED: no schedule
 * found (ret is left unspecified).  SKRULL_EINVAL: null pointer or a value
 * outside the ranges above.  SKRULL_ENOMEM: host allocation failed.
 */
int skrull_dacp_schedule(int32_t num_seqs, const int32_t *seq_len, int64_t bucket_size,
                         int32_t cp_degree, const skrull_flops_model_t *model, int32_t *ret);

/*
 * The micro-batch of rank `rank` under schedule `ret`: its local sequences whole
 * (degree 1, index 0) and its slice of every distributed one (degree N, index
 * rank), in the caller's order.  The four output arrays have room for K entries
 * each; *count receives the number written; source[i] is the position of entry
 * i in the caller's list.  These are the seq_len / shard_degree / shard_index
 * arrays of skrull_attn_problem_t.  SKRULL_EINVAL: null pointer, K < 1,
 * rank outside [0, N), or a ret entry outside [-1, N).
 */
int skrull_dacp_rank_batch(int32_t num_seqs, const int32_t *seq_len, const int32_t *ret,
                           int32_t cp_degree, int32_t rank, int32_t *out_seq_len,
                           int32_t *out_shard_degree, int32_t *out_shard_index,
                           int32_t *out_source, int32_t *count);

#ifdef __cplusplus
}
#endif
#endif /* SKRULL_DACP_H */
