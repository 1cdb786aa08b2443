/*
 * skrull_attn.h -- C ABI of the MI355X (gfx950) packed variable-length causal
 * attention library: forward and backward over ONE scheduled micro-batch.
 *
 * The micro-batch is the paper's (Sec. 4.1, Eq. 1-8): context-parallel rank j
 * holds every local sequence assigned to it whole (P_kj = 1) and a 1/N slice
 * of every distributed sequence (D_k = 1; Eq. 8 charges S_k/N of its tokens to
 * each rank).  The caller states it exactly that way: a list of full sequence
 * lengths S[K], and per sequence a shard degree (1 = local, N = distributed),
 * the shard index this GPU holds and, optionally, how the sequence is cut.
 * Sequences are packed without padding (App. B.1) and never attend to one
 * another.  By default a shard is the contiguous query range
 * [floor(r*S/N), floor((r+1)*S/N)) attending to the gathered key/value prefix
 * [0, q_end) at its true positions (the paper leaves the cut open; it only
 * fixes the S/N token count); SKRULL_CUT_TWO_CHUNKS below is the alternative.
 *
 * All tensors are caller-owned DEVICE memory, contiguous, 16-byte aligned,
 * token-major with head_dim innermost:
 *   Q, O, dQ, dO : bf16 [total_q, num_q_heads, head_dim]
 *   K, V, dK, dV : bf16 [total_k, num_kv_heads, head_dim]
 *   LSE          : fp32 [num_q_heads, total_q]   (natural log, scale included)
 * Sequences follow one another in both packings in the caller's order: sequence k
 * owns the next q_len rows of Q/O/dQ/dO (its slice, or its two chunks one after
 * the other) and the next kv_len rows of K/V/dK/dV, which are key positions
 * 0..kv_len-1 of its prefix.
 * Query head h reads key/value head h / (num_q_heads / num_kv_heads).
 *
 * Every function returns 0 (SKRULL_OK) or a negative code; nothing throws or
 * aborts.  State outside the plans: per calling thread, the text of its last error and
 * the opt-in profiling switch at the end of this header; per GPU, the static workspace
 * of skrull_attn_bwd_static.  On failure output pointers written
 * through `out` arguments are left untouched.  Every step runs in HIP kernels;
 * there is no CPU fallback.
 */
#ifndef SKRULL_ATTN_H
#define SKRULL_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKRULL_OK            0
#define SKRULL_EINVAL       (-1)  /* bad argument (see each function)            */
#define SKRULL_ENOMEM       (-2)  /* host or device allocation failed            */
#define SKRULL_EHIP         (-3)  /* a HIP runtime call failed                   */
#define SKRULL_EUNSUPPORTED (-4)  /* no device, or the device is not gfx950      */

typedef struct skrull_attn_plan skrull_attn_plan_t; /* opaque, library-owned */

/* The problem, in the paper's terms (Alg. 1 inputs S[K], N; Eq. 1-8 D_k, P_kj). */
typedef struct {
    int32_t        num_seqs;      /* K >= 1                                                   */
    const int32_t *seq_len;       /* [K] HOST; full (unsharded) length S_k >= 1                */
    const int32_t *shard_degree;  /* [K] HOST; 1 = local (D_k = 0), N > 1 = distributed; <= S_k */
    const int32_t *shard_index;   /* [K] HOST; 0 <= index < degree                             */
    int32_t        num_q_heads;   /* Hq >= 1                                                   */
    int32_t        num_kv_heads;  /* Hkv >= 1, Hq % Hkv == 0                                   */
    int32_t        head_dim;      /* 64 or 128                                                 */
    float          softmax_scale; /* finite, > 0; multiplies Q.K^T inside the kernels          */
    int32_t        block_m;       /* query rows per work item: 64, 128 or 256; 0 = 256          */
    int32_t        block_n;       /* key rows per dK/dV work item: 64, 128, 192 or 256; 0 = library's choice */
    const int32_t *shard_cut;     /* [K] HOST or NULL (= all SKRULL_CUT_CONTIGUOUS)             */
    int32_t        head_split;    /* dK/dV workgroups per KV group, 1..Hq/Hkv; 0 = library's choice */
    int32_t        wg_query_rows; /* query rows per forward / dQ workgroup: 128 or 256; 0 = library's choice */
} skrull_attn_problem_t;

/*
 * How a distributed sequence is cut (the paper fixes only the S_k/N tokens per rank,
 * Eq. 8, and charges every rank FLOPs/N, Eq. 4):
 *  SKRULL_CUT_CONTIGUOUS  the slice [floor(r*S/N), floor((r+1)*S/N)); under the causal
 *                         mask rank r does (2r+1)/N^2 of the work.
 *  SKRULL_CUT_TWO_CHUNKS  the sequence is cut into 2N chunks [floor(i*S/2N),
 *                         floor((i+1)*S/2N)) and rank r holds chunks r and 2N-1-r, so
 *                         every rank does 1/N of the work up to rounding, which is what
 *                         Eq. 4 assumes.  Needs 2N <= S_k.  The rank's rows of
 *                         Q/O/dQ/dO/LSE are chunk r's followed by chunk 2N-1-r's; its
 *                         K/V/dK/dV rows are the prefix [0, end of chunk 2N-1-r).
 * Inside the library such a sequence is two consecutive query SEGMENTS that share one
 * key/value prefix; a contiguous slice or a local sequence is one segment.
 */
#define SKRULL_CUT_CONTIGUOUS 0
#define SKRULL_CUT_TWO_CHUNKS 1

typedef struct {
    int32_t num_seqs, num_q_heads, num_kv_heads, head_dim;
    int32_t block_m, block_n;
    int32_t total_q;              /* sum of q_len  = rows of Q/O/dQ/dO                         */
    int32_t total_k;              /* sum of kv_len = rows of K/V/dK/dV                         */
    int32_t n_fwd_items;          /* entries of the forward / dQ work list                     */
    int32_t n_dkv_items;          /* entries of the dK/dV work list                            */
    int64_t attended_pairs;       /* exact number of (query, key) pairs under the causal mask  */
    int64_t useful_flops_fwd;     /*  4 * pairs * head_dim * Hq                                */
    int64_t useful_flops_bwd;     /* 10 * pairs * head_dim * Hq                                */
    int64_t bwd_workspace_bytes;  /* device scratch skrull_attn_bwd needs (>= 0)               */
    int32_t num_segments;         /* query segments: K + number of two-chunk sequences         */
    int32_t head_split;           /* the dK/dV head split in effect (>= 1)                     */
    int32_t wg_query_rows;        /* query rows per forward / dQ workgroup in effect (128 or 256;
                                     dQ has the 128-row shape at head_dim 64 only)             */
    int32_t reserved;             /* 0                                                         */
} skrull_attn_plan_info_t;

/* Arrays a plan holds on the device, for skrull_attn_plan_export.  They are per
 * query segment (NS = num_segments entries; NS = K when no sequence is cut in two
 * chunks, and then a segment is a sequence). */
enum {
    SKRULL_ARRAY_CU_Q      = 0,   /* int32 [NS+1] first packed Q row of the segment; total     */
    SKRULL_ARRAY_CU_K      = 1,   /* int32 [NS+1] first packed K/V row of its prefix; total    */
    SKRULL_ARRAY_Q_BEGIN   = 2,   /* int32 [NS]   global position of the first local query     */
    SKRULL_ARRAY_Q_LEN     = 3,   /* int32 [NS]                                                */
    SKRULL_ARRAY_KV_LEN    = 4,   /* int32 [NS]   q_begin + q_len: the keys the segment sees   */
    SKRULL_ARRAY_FWD_ITEMS = 5,   /* int32 [n_fwd_items][4] = {segment, q_block, q_row, n_kv}  */
    SKRULL_ARRAY_DKV_ITEMS = 6,   /* int32 [n_dkv_items][4] = {segment, kv_block, m0, n_q}     */
    SKRULL_ARRAY_SHARES_KV = 7    /* int32 [NS]   1 = late chunk: shares the prefix of NS-1    */
};

/*
 * Build the varlen descriptor and the two cost-ordered tile work lists on the
 * device (paper Eq. 8 for the slice sizes; the ordering applies the paper's
 * load-balance rule -- heaviest piece first to the least-loaded worker, Alg. 1
 * argmin(L) and Alg. 2's FLOPs bin-packing -- to compute units: items are
 * stably sorted by descending quadratic cost and dispatched in that order).
 *
 * Forward/dQ list: one item per (segment, block of block_m query rows), cost
 * n_kv = ceil((q_begin + last_row + 1) / block_n).  dK/dV list: one item per
 * (key/value prefix, block of block_n key rows), named by the last segment that
 * reads the prefix; m0 = that segment's first query block that can see the
 * block, cost n_q = number of query blocks that do (of both segments when the
 * prefix is shared).  Ties keep (segment, block) ascending order, so the layout
 * is a pure function of the inputs and of the block sizes in effect.
 *
 * Tuning fields left at 0 are chosen by the library from the head shape, the
 * lengths and the device's compute-unit count, and skrull_attn_plan_info
 * reports what is in effect: block_n is 128, or 192 at head_dim 64 when a
 * sequence of 8,192 tokens or more is present, when the work list is short
 * (its costliest item above an even share per compute unit), or when fewer,
 * larger items still balance (five blocks of 192 key rows x KV heads per
 * compute unit, or a costliest item under 0.7 of the even share; the dK/dV
 * kernel then runs 12 wavefronts over 192 key rows); head_split above 1
 * when the longest dK/dV chain exceeds an even share of the work list;
 * wg_query_rows 128 when the micro-batch holds enough work for the smaller
 * workgroups to pay (head_dim 64: at least 24 blocks of 256 query rows x heads
 * per compute unit or 1.5e9 attended (query, key, head) triples; head_dim 128:
 * at least 16 such blocks and no sequence above 8,192 tokens), else 256.  None
 * of them changes a result beyond the
 * last bit of dK/dV (head_split changes the order of the sum over heads).
 *
 * p and the three arrays it points to are HOST memory, read before return.
 * `hip_stream` (a hipStream_t, may be NULL for the default stream) carries the
 * kernels; the call synchronises that stream because the totals come back to
 * the host.  *out receives a plan that must be released with
 * skrull_attn_plan_destroy.  A plan's descriptor and work lists are immutable and it may
 * be reused by any number of fwd/bwd calls on any stream of the same device.  The kernels
 * are persistent (workgroups take work items from queues until none is left, see
 * skrull_attn_fwd); a backward call keeps its queues in its own workspace, a forward call
 * takes one of the plan's 64 queue slots in turn, so at most 64 forward calls of one plan
 * may be in flight at once, and a forward call captured in a HIP graph (which keeps the
 * slot it was captured with) must not overlap with other forward calls of the same plan.
 * SKRULL_EINVAL: null pointer, K < 1, S_k < 1, degree < 1, index outside
 * [0, degree), more chunks than tokens (degree > S_k, or 2*degree > S_k for a
 * two-chunk cut), a cut other than the two above, head_split outside [0, Hq/Hkv],
 * wg_query_rows other than 0/128/256, Hq % Hkv != 0, head_dim not 64/128, a block size
 * other than 0/64/128/256 (block_n also 192), scale not finite/positive, a total of 2^31 rows or
 * more, more than 2^20 work items in either list, or a sequence too long for
 * the kernels' 32-bit tile offsets: (rows of this rank's longest chunk + 256)
 * * Hq * d * 2 bytes and (S_k + 256) * Hkv * d * 2 bytes must both stay below
 * 2^32 (32 query heads of 128: 524,031 query rows per chunk; 8 KV heads of
 * 128: 2,096,895 tokens per sequence).
 */
int skrull_attn_plan(const skrull_attn_problem_t *p, void *hip_stream, skrull_attn_plan_t **out);

/* Totals of a plan (host struct filled; no device work). */
int skrull_attn_plan_info(const skrull_attn_plan_t *plan, skrull_attn_plan_info_t *info);

/*
 * Copy one of the plan's device arrays to HOST memory `dst` (synchronous).
 * `bytes` must equal the array's exact size in bytes, else SKRULL_EINVAL.
 */
int skrull_attn_plan_export(const skrull_attn_plan_t *plan, int which, void *dst, size_t bytes);

/*
 * Forward: for every sequence k, query head h, local row i at global position
 * p = q_begin[k] + i, with c = h / (Hq/Hkv):
 *     s_j = softmax_scale * q_i . k_j  (j = 0..p),  LSE = log sum_j exp(s_j),
 *     O_i = sum_j exp(s_j - LSE) v_j.
 * This is the O(n^2)-compute / O(n)-memory attention the paper's cost model
 * rests on (Sec. 4.2.1; App. B.2, the 4*b*h*S^2 term).  bf16 MFMA products,
 * fp32 accumulation and softmax, O rounded to bf16 (nearest even), LSE fp32.
 * q, k, v (read) and o, lse (written) are DEVICE pointers in the layout above.
 * Work items go to compute units the way the paper sends sequences to ranks (Alg. 1:
 * the next piece to argmin of the loads): the launch holds as many workgroups as the chip
 * runs at once, each takes the next item of the cost-ordered list of its die until that is
 * empty and then the largest remaining item of the fullest other list (the dies of one chip
 * differ in speed by several percent, which a fixed deal of workgroups to dies cannot even
 * out).  Results do not depend on which workgroup took which item.
 * Only enqueues on `hip_stream` (the attention kernel and, when there are more work items than
 * the chip holds workgroups at once, a small kernel that clears the queue before it); never
 * synchronises.
 * SKRULL_EINVAL on a null or misaligned pointer, or when the current device is
 * not the one the plan was made on.
 */
int skrull_attn_fwd(const skrull_attn_plan_t *plan, const void *q, const void *k, const void *v,
                    void *o, float *lse, void *hip_stream);

/*
 * Backward of the same function, given dO and the forward's O and LSE:
 *     D_i   = dO_i . O_i
 *     P_ij  = exp(softmax_scale * q_i . k_j - LSE_i),  dS_ij = P_ij (dO_i . v_j - D_i)
 *     dQ_i  = softmax_scale * sum_j dS_ij k_j
 *     dK_j  = softmax_scale * sum_{h in group} sum_i dS_ij q_i
 *     dV_j  =                 sum_{h in group} sum_i P_ij dO_i
 * dK/dV of a shard are this rank's partial sums over its own query rows for
 * the whole prefix (a multi-GPU caller would reduce them across ranks; the
 * paper's Eq. 3/Volume(S) is that exchange).  All outputs bf16, rounded once
 * from fp32 accumulators; the group sum is done in registers, or, when the plan's
 * head_split is above 1, over fp32 partial sums in the workspace in a fixed order
 * (no atomics either way, so results are bit-reproducible; two plans with
 * different head_split may differ in the last bit of dK/dV).
 * `workspace` is DEVICE scratch of at least info.bwd_workspace_bytes, 16-byte
 * aligned; contents on entry are ignored and on exit unspecified.
 * Only enqueues on `hip_stream`; never synchronises.
 * SKRULL_EINVAL on a null or misaligned pointer, a workspace that is too small,
 * or when the current device is not the one the plan was made on.
 */
int skrull_attn_bwd(const skrull_attn_plan_t *plan, const void *q, const void *k, const void *v,
                    const void *o, const float *lse, const void *d_o,
                    void *dq, void *dk, void *dv,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * skrull_attn_bwd for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving or training loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and errors as skrull_attn_bwd (bit for bit: the
 * same kernels), but the workspace (-D and LSE*log2(e) per query head and row, and the
 * fp32 partial dK/dV when head_split > 1) is a static device array inside the library of
 * SKRULL_STATIC_SCRATCH_BYTES bytes per GPU, held from library load until the process
 * ends; its address on a device is looked up when the first plan is made on that device.
 * The call allocates and frees nothing, does not synchronise, and only enqueues kernels
 * on `hip_stream`.  Nothing in the array has to start at zero (every word read was
 * written by an earlier kernel of the same call).
 * SKRULL_EINVAL, besides skrull_attn_bwd's cases, when info.bwd_workspace_bytes exceeds
 * SKRULL_STATIC_SCRATCH_BYTES (strerror names both sizes).
 * Every call on one GPU uses the same array: calls that may overlap on one GPU (two
 * streams, two threads) race and must be ordered by the caller.
 */
#define SKRULL_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
int skrull_attn_bwd_static(const skrull_attn_plan_t *plan, const void *q, const void *k, const void *v,
                           const void *o, const float *lse, const void *d_o,
                           void *dq, void *dk, void *dv, void *hip_stream);

/* Release a plan and its device arrays (NULL is ignored). */
void skrull_attn_plan_destroy(skrull_attn_plan_t *plan);

/* Static description of a return code; for SKRULL_EHIP the text of the last
 * HIP error seen by the calling thread is appended. Never NULL. */
const char *skrull_attn_strerror(int code);

/*
 * Measurement aid (not part of the method).  While enabled, skrull_attn_fwd and
 * skrull_attn_bwd bracket each of their kernels with HIP events recorded on
 * the caller's stream.  skrull_attn_profile_read waits for the events of the
 * most recent forward and backward calls and returns the kernel durations in
 * milliseconds: ms[0] forward, ms[1] always 0 (D = rowsum(dO*O) is formed inside
 * the dQ kernel), ms[2] dK/dV with its reduction, ms[3] dQ
 * (an entry is -1 if that call has not been made since enabling).  The switch and its
 * events belong to the CALLING THREAD: it affects only calls that thread makes, any
 * number of threads may profile at once, and a thread reads back what it recorded itself
 * (one stream at a time per thread).  Disabling releases the thread's events;
 * skrull_attn_profile_read returns SKRULL_EINVAL on a thread that has not enabled it.
 */
int skrull_attn_profile(int enable);
int skrull_attn_profile_read(float ms[4]);

/*
 * Measurement aid (not part of the method): how evenly the cost-ordered work lists load the
 * compute units.  After skrull_attn_trace(records, bytes) the calling thread's forward and
 * backward calls make every workgroup write one 32-byte record into the caller's DEVICE
 * buffer `records` (16-byte aligned; the caller zeroes it first):
 *   uint64 t0, t1   the chip-wide 100 MHz counter (s_memrealtime) at its start and end
 *   uint32 hw_id    the HW_ID register (bits 8-11 compute unit, 12 shader array, 13-15 shader engine)
 *   uint32 xcc_id   the XCC_ID register (die)
 *   uint32 block    its blockIdx.x
 *   uint32 one      1
 * Records of the forward kernel come first, then the dQ kernel's, then the dK/dV kernel's;
 * skrull_attn_trace_layout gives, for a plan, the first record and the number of records
 * (= workgroups; those that leave at once write nothing) of the three.  A call whose records
 * do not fit `bytes` returns SKRULL_EINVAL.  skrull_attn_trace(NULL, 0) switches it off.
 * Untraced calls pay one scalar branch per workgroup.  skrull_attn_bwd_static is never traced.
 */
int skrull_attn_trace(void *records, size_t bytes);
int skrull_attn_trace_layout(const skrull_attn_plan_t *plan, int32_t first_record[3], int32_t num_records[3]);

/*
 * Measurement aid (not part of the method).  Runs three launches of about 20 ms of
 * nothing but v_mfma_f32_32x32x16_bf16 on every compute unit (two waves per SIMD,
 * operands in registers) on `hip_stream`, waits, and returns the rate of the last in TFLOP/s: the
 * matrix-pipe ceiling this GPU sustains at the clock it holds under such load, to
 * be read beside the nominal 2.5 PFLOP/s.  Allocates nothing (its 512 KB sink is the start
 * of the static workspace of skrull_attn_bwd_static: do not overlap the two on one GPU).
 */
int skrull_attn_mfma_ceiling(void *hip_stream, float *tflops);

#ifdef __cplusplus
}
#endif
#endif /* SKRULL_ATTN_H */
