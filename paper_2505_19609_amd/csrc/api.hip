// Host side of the C ABI: argument validation, plan construction, launches.
// No arithmetic of the method happens here: the descriptor, the work lists, their costs
// and all attention math are produced by kernels (plan.hip, fwd.hip, bwd.hip).  What the
// host derives from the lengths are upper bounds only (how many work items there can be at
// most, for the allocations and grids) and the tuning choices documented in the header,
// which it takes from the totals that the plan kernels return.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <new>

#include "common.h"
#include "skrull_dacp.h"

namespace {

thread_local char g_err[256] = "";

int hip_fail(hipError_t e, const char *what)
{
    snprintf(g_err, sizeof g_err, "%s: %s", what, hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? SKRULL_ENOMEM : SKRULL_EHIP;
}

#define HIP_TRY(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) { rc = hip_fail(e_, #expr); goto done; } \
    } while (0)

inline bool misaligned(const void *p) { return p == nullptr || ((uintptr_t)p & 15u) != 0; }

inline int64_t align4(int64_t n) { return (n + 3) & ~(int64_t)3; }

// Opt-in kernel timing, per calling thread: events 0/1 bracket the forward kernel, 2..4
// delimit the backward kernels.  A thread that never enables it owns nothing.
struct ProfileState {
    bool on = false, made = false, fwd_seen = false, bwd_seen = false;
    hipEvent_t ev[6];
};
thread_local ProfileState g_prof;

// Opt-in per-workgroup trace, per calling thread: a caller-owned device buffer of WgTrace records.
struct TraceState {
    WgTrace *buf = nullptr;
    size_t records = 0;
};
thread_local TraceState g_trace;

constexpr int32_t kMaxItems = 1 << 20;  // per list (lists above 2,048 items are radix sorted)

// Workspace of skrull_attn_bwd_static, the backward entry point for callers that cannot
// allocate: one array per GPU that the library runs on, held until the process ends.
// In host code the array's name is only a stand-in for the symbol; the device address
// comes from hipGetSymbolAddress, once per device, and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[SKRULL_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on device `dev`, which must be the current device.
int resolve_scratch(int dev, void **out)
{
    if (dev < 0 || dev >= kMaxDevices) return SKRULL_EUNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // (a second thread stores the same address)
    }
    *out = p;
    return SKRULL_OK;
}

int check_device(int *dev_out, int *compute_units)
{
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return SKRULL_EUNSUPPORTED;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SKRULL_EUNSUPPORTED;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return SKRULL_EUNSUPPORTED;
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return SKRULL_EUNSUPPORTED;
    *dev_out = dev;
    *compute_units = prop.multiProcessorCount;
    return SKRULL_OK;
}

// A plan's arrays live on the device it was made on: the calls that use them must run there.
int check_plan_device(const skrull_attn_plan_t *plan)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) {
        snprintf(g_err, sizeof g_err, "plan was made on device %d, current device is %d", plan->device, dev);
        return SKRULL_EINVAL;
    }
    return SKRULL_OK;
}

}  // namespace

extern "C" {

int skrull_attn_plan(const skrull_attn_problem_t *p, void *hip_stream, skrull_attn_plan_t **out)
{
    if (!p || !out || !p->seq_len || !p->shard_degree || !p->shard_index) return SKRULL_EINVAL;
    const int32_t K = p->num_seqs;
    if (K < 1) return SKRULL_EINVAL;
    if (p->num_q_heads < 1 || p->num_kv_heads < 1 || p->num_q_heads % p->num_kv_heads != 0)
        return SKRULL_EINVAL;
    if (p->head_dim != 64 && p->head_dim != 128) return SKRULL_EINVAL;
    if (!(p->softmax_scale > 0.0f) || !isfinite(p->softmax_scale)) return SKRULL_EINVAL;
    const int32_t BM = p->block_m == 0 ? 256 : p->block_m;
    int32_t BN = p->block_n == 0 ? 128 : p->block_n;  // (left open: may become 192 below)
    if ((BM != 64 && BM != 128 && BM != 256) || (BN != 64 && BN != 128 && BN != 192 && BN != 256))
        return SKRULL_EINVAL;
    const int32_t group = p->num_q_heads / p->num_kv_heads;
    if (p->head_split < 0 || p->head_split > group) return SKRULL_EINVAL;
    if (p->wg_query_rows != 0 && p->wg_query_rows != 128 && p->wg_query_rows != 256) return SKRULL_EINVAL;
    // Entry checks are done here so that they work without a device; the kernel repeats
    // them next to the range computation.  The same pass bounds the number of work
    // items from above (chunk lengths differ by at most one row; a prefix is no longer
    // than its sequence), which sizes the allocations and the grids, so that the whole
    // plan is built with one copy in, one copy out and one synchronisation.
    int64_t n_seg = 0;  // query segments: a two-chunk cut contributes two
    int32_t longest_seq = 0;
    const int64_t q_row_bytes = (int64_t)p->num_q_heads * p->head_dim * 2;
    const int64_t kv_row_bytes = (int64_t)p->num_kv_heads * p->head_dim * 2;
    int64_t cap_fwd = 0, cap_dkv = 0;
    for (int32_t k = 0; k < K; ++k) {
        const int32_t s = p->seq_len[k], n = p->shard_degree[k], r = p->shard_index[k];
        const int32_t z = p->shard_cut ? p->shard_cut[k] : SKRULL_CUT_CONTIGUOUS;
        if (z != SKRULL_CUT_CONTIGUOUS && z != SKRULL_CUT_TWO_CHUNKS) return SKRULL_EINVAL;
        if (s < 1 || n < 1 || r < 0 || r >= n || (int64_t)n * (1 + z) > s) return SKRULL_EINVAL;
        n_seg += 1 + z;
        longest_seq = s > longest_seq ? s : longest_seq;
        const int64_t chunks = (int64_t)n * (1 + z), longest = (s + chunks - 1) / chunks;
        // The kernels address a tile as a 32-bit byte offset from the first row of its
        // query segment (rows of Hq*d bf16) or of its key/value prefix (rows of Hkv*d
        // bf16), and prefetch up to four 64-row tiles past the end (those read as zero).
        if ((longest + 256) * q_row_bytes > (int64_t)UINT32_MAX ||
            ((int64_t)s + 256) * kv_row_bytes > (int64_t)UINT32_MAX) {
            snprintf(g_err, sizeof g_err, "sequence %d is too long for 32-bit tile offsets", k);
            return SKRULL_EINVAL;
        }
        cap_fwd += (1 + z) * ((longest + BM - 1) / BM);
        cap_dkv += ((int64_t)s + BN - 1) / BN;
    }
    if (n_seg > INT32_MAX / 2) return SKRULL_EINVAL;
    if (cap_fwd > 8 * (int64_t)kMaxItems || cap_dkv > 8 * (int64_t)kMaxItems) return SKRULL_EINVAL;
    int dev = 0, compute_units = 0;
    int rc = check_device(&dev, &compute_units);
    if (rc != SKRULL_OK) return rc;
    {   // set-up for skrull_attn_bwd_static: this device's address of the static workspace
        void *unused = nullptr;
        if ((rc = resolve_scratch(dev, &unused)) != SKRULL_OK) return rc;
    }

    // dK/dV block size when the caller leaves it open.  At head_dim 64 the kernel has a
    // 12-wavefront shape over 192 key rows; with a sequence of 8,192 tokens or more in the
    // micro-batch it was 3-16 % faster than the 8-wavefront shape over 128 on whole sequences
    // and on slices of distributed ones alike (14 query / 2 KV heads; 2 x 8,192 ... 98,304
    // tokens, both cuts, the benchmark length mixes).  On shorter sequences it wins (7-14 %)
    // exactly where the work list is so short that the heads are split anyway (longest
    // chain above an even share of 128-key items, see head_split below), and loses 2-25 %
    // where it is not: there the fewer, larger workgroups and the split they then need
    // cost more than the third wavefront per SIMD brings.  That second case is decided by the
    // ranges kernel from the costs of the 128-key work list (bn_alt), and comes back in totals.
    int32_t bn_alt = 0;
    if (p->block_n == 0 && p->head_dim == 64) {
        if (longest_seq >= 8192) BN = 192;
        else bn_alt = 192;
    }
    // (cap_dkv counts items of BN key rows; the alternative is larger, so it needs fewer)

    hipStream_t st = (hipStream_t)hip_stream;
    skrull_attn_plan_t *plan = nullptr;
    int32_t *tmp = nullptr, *host_in = nullptr;
    PlanTotals totals;
    // tmp (released before return): S, N, R, cut [K each] | fwd_off, dkv_off [n_seg+1 each] |
    // totals | unsorted items
    const int64_t kin = align4(K), kpad = align4(n_seg + 1);
    const int64_t totals_ints = align4((int64_t)((sizeof(PlanTotals) + 3) / 4));
    // no work item costs more than this many blocks (64 rows is the smallest block; a two-chunk
    // cut adds the query blocks of both chunks)
    const int32_t cost_bound = 2 * (longest_seq / 64 + 2);
    const int64_t radix_ints = plan_radix_ints((int32_t)cap_fwd, (int32_t)cap_dkv, cost_bound);
    const int64_t tmp_ints = 4 * kin + 2 * kpad + totals_ints + 4 * (cap_fwd + cap_dkv) + radix_ints;
    const int64_t desc_ints = 6 * kpad;
    const int64_t queue_ints = SKRULL_FWD_QUEUE_SLOTS * 16;  // 64-byte work queues of the forward launches
    int32_t *fwd_off = nullptr, *dkv_off = nullptr, *scratch = nullptr;
    PlanTotals *totals_d = nullptr;

    plan = new (std::nothrow) skrull_attn_plan_t();
    if (!plan) return SKRULL_ENOMEM;
    memset(plan, 0, sizeof *plan);
    plan->K = K; plan->NS = (int32_t)n_seg; plan->Hq = p->num_q_heads; plan->Hkv = p->num_kv_heads; plan->d = p->head_dim;
    plan->BM = BM; plan->BN = BN; plan->scale = p->softmax_scale; plan->device = dev;

    host_in = (int32_t *)calloc((size_t)(4 * kin), sizeof(int32_t));
    if (!host_in) { rc = SKRULL_ENOMEM; goto done; }
    memcpy(host_in, p->seq_len, (size_t)K * 4);
    memcpy(host_in + kin, p->shard_degree, (size_t)K * 4);
    memcpy(host_in + 2 * kin, p->shard_index, (size_t)K * 4);
    if (p->shard_cut) memcpy(host_in + 3 * kin, p->shard_cut, (size_t)K * 4);

    HIP_TRY(hipMalloc((void **)&tmp, (size_t)tmp_ints * sizeof(int32_t)));
    HIP_TRY(hipMalloc((void **)&plan->pool, (size_t)(queue_ints + desc_ints + 4 * (cap_fwd + cap_dkv)) * sizeof(int32_t)));
    plan->fwd_queues = (WorkQueue *)plan->pool;   // (zeroed by every forward call before its launch)
    plan->cu_q = plan->pool + queue_ints;
    plan->cu_k = plan->cu_q + kpad;
    plan->q_begin = plan->cu_q + 2 * kpad;
    plan->q_len = plan->cu_q + 3 * kpad;
    plan->kv_len = plan->cu_q + 4 * kpad;
    plan->shares_kv = plan->cu_q + 5 * kpad;
    plan->fwd_items = plan->cu_q + desc_ints;
    plan->dkv_items = plan->fwd_items + 4 * cap_fwd;
    fwd_off = tmp + 4 * kin;
    dkv_off = fwd_off + kpad;
    totals_d = (PlanTotals *)(dkv_off + kpad);
    scratch = dkv_off + kpad + totals_ints;
    // a pageable source is staged by the runtime before the call returns
    HIP_TRY(hipMemcpyAsync(tmp, host_in, (size_t)(4 * kin) * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(launch_plan_ranges(tmp, tmp + kin, tmp + 2 * kin, tmp + 3 * kin, K, BM, BN,
                               INT32_MAX / (p->num_q_heads * p->head_dim),
                               INT32_MAX / (p->num_kv_heads * p->head_dim), plan->q_begin,
                               plan->q_len, plan->kv_len, plan->cu_q, plan->cu_k, plan->shares_kv,
                               fwd_off, dkv_off, (int32_t)cap_fwd, (int32_t)cap_dkv, bn_alt, p->num_kv_heads,
                               compute_units, totals_d, st));
    HIP_TRY(launch_plan_items(plan, fwd_off, dkv_off, (int32_t)cap_fwd, (int32_t)cap_dkv, scratch,
                              scratch + 4 * cap_fwd, scratch + 4 * (cap_fwd + cap_dkv), cost_bound, totals_d, st));
    HIP_TRY(hipMemcpyAsync(&totals, totals_d, sizeof totals, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (totals.bad_entry != 0 || totals.n_seg != plan->NS || totals.total_q > INT32_MAX ||
        totals.total_k > INT32_MAX || totals.n_fwd > kMaxItems || totals.n_dkv > kMaxItems ||
        totals.n_fwd > cap_fwd || totals.n_dkv > cap_dkv) {
        snprintf(g_err, sizeof g_err, "micro-batch too large or invalid entry %d", totals.bad_entry - 1);
        rc = SKRULL_EINVAL;
        goto done;
    }
    if (totals.block_n != BN && totals.block_n != bn_alt) { rc = SKRULL_EHIP; snprintf(g_err, sizeof g_err, "plan kernels returned block_n %d", totals.block_n); goto done; }
    plan->BN = totals.block_n;
    plan->total_q = (int32_t)totals.total_q;
    plan->total_k = (int32_t)totals.total_k;
    plan->n_fwd = (int32_t)totals.n_fwd;
    plan->n_dkv = (int32_t)totals.n_dkv;
    plan->pairs = totals.pairs;
    // dK/dV head split.  A workgroup of that kernel walks all query tiles of one key
    // block for every query head of the KV group, one after another; its longest chain
    // is cost_max * group.  Spread evenly, the whole list is cost_sum * group * Hkv over
    // the compute units.  When the longest chain exceeds that share (few KV heads, one
    // long sequence in a small micro-batch) the heads of a group are shared out over
    // several workgroups until it no longer does, with a factor two of slack.
    // Workgroup shape of the forward and dQ kernels.  Several 4-wavefront workgroups per compute
    // unit hide each other's start-up, drain and barriers, but they also stretch each other's
    // work items (three share a unit and its oldest wave is served first), and a launch ends only
    // when its last stretched item does; so the small shape pays once the launch holds enough
    // work to bury that tail.  Measured on 8 to 64 query heads x 16,384 to 32,768 tokens x
    // sequences of 256 to 32,768 tokens: at head_dim 64 the small shape wins (forward by 3-15 %,
    // dQ by 1-6 %) when the micro-batch has at least 24 blocks of 256 query rows x heads per
    // compute unit or at least 1.5e9 attended (query, key, head) triples, and loses by 2-90 %
    // (forward) below that; at head_dim 128 (forward only: the small dQ shape does not fit the LDS
    // twice) it wins by 1-8 % from 16 such blocks per compute unit on while no sequence exceeds
    // 8,192 tokens, where the 8-wavefront workgroup's deeper tile ring and halved tile traffic
    // take over.
    if (p->wg_query_rows != 0) {
        plan->wg_query_rows = p->wg_query_rows;
    } else {
        const double blocks_per_cu = (double)plan->Hq * (double)totals.total_q / (256.0 * (double)compute_units);
        const double triples = (double)totals.pairs * (double)plan->Hq;
        const bool small_shape = p->head_dim == 64 ? (blocks_per_cu >= 24.0 || triples >= 1.5e9)
                                                   : (longest_seq <= 8192 && blocks_per_cu >= 16.0);
        plan->wg_query_rows = small_shape ? 128 : 256;
    }
    plan->head_split = p->head_split;
    if (plan->head_split == 0) {
        // Split only when the longest chain of the work list (its costliest item, all the
        // heads of a group) exceeds an even share of the whole list over the compute units:
        // then that chain bounds the kernel's time and shortening it pays for the fp32
        // partial sums and their reduction; below that the unsplit kernel is 5-40 % faster
        // (measured on 45 micro-batches of three head shapes; the ratio below was the
        // dividing line at 1.0: splits won from 1.27 up, lost or tied up to 0.98).
        // The 12-wavefront shape (fewer, larger workgroups: rounding of workgroups per compute
        // unit weighs more) gains from the split from half that ratio on: at 14/2 heads x 64
        // every batch measured from 2 x 8,192 to 65,536 tokens was 7-50 % faster split 7 ways
        // (65,536 tokens, ratio 0.75: 17.4 -> 16.1 ms; eight 8,192-token sequences, 0.72: equal).
        const double share = (double)totals.dkv_cost_sum * plan->Hkv / (double)compute_units;
        // (that factor of two only where it was measured to pay: a sequence of 8,192 tokens or more
        // and a short list, under five items x KV heads per compute unit; with longer lists of
        // 192-key items, 16-64 heads on ragged 32,768-token micro-batches, a split at ratios of
        // 0.6-0.9 cost 6-16 %, and on short lists of short sequences up to 90 %)
        const bool short_list = (int64_t)totals.n_dkv * plan->Hkv < 5 * (int64_t)compute_units;
        const double scale = (plan->d == 64 && plan->BN == 192 && short_list && longest_seq >= 8192) ? 2.0 : 1.0;
        const double want = share > 0.0 ? scale * (double)totals.dkv_cost_max / share : 1.0;
        int32_t hs = want <= 1.0 ? 1 : (want >= (double)group ? group : (int32_t)ceil(want));
        // only equal shares: workgroups with different numbers of heads walk the query
        // tiles at different paces, stop sharing them in L2 and run 10 % slower (measured
        // with 7 heads per group split 3 + 4), so take the next divisor of the group size
        const int32_t asked = hs;
        while (hs < group && group % hs != 0) ++hs;
        // ... unless that divisor is three times what was asked for and the chain is less than
        // 1.5 even shares (7 heads per group at ratios of 1.0-1.4: split 7 ways 6-14 % slower
        // than unsplit, equal at 1.7)
        if (hs >= 3 * asked && want < 1.5) hs = 1;
        plan->head_split = hs < 1 ? 1 : (hs > group ? group : hs);
    }
    rc = SKRULL_OK;
done:
    free(host_in);
    if (tmp) (void)hipFree(tmp);
    if (rc != SKRULL_OK) {
        if (plan) {
            if (plan->pool) (void)hipFree(plan->pool);
            delete plan;
        }
        return rc;
    }
    *out = plan;
    return SKRULL_OK;
}

int skrull_attn_plan_info(const skrull_attn_plan_t *plan, skrull_attn_plan_info_t *info)
{
    if (!plan || !info) return SKRULL_EINVAL;
    info->num_seqs = plan->K;
    info->num_q_heads = plan->Hq;
    info->num_kv_heads = plan->Hkv;
    info->head_dim = plan->d;
    info->block_m = plan->BM;
    info->block_n = plan->BN;
    info->total_q = plan->total_q;
    info->total_k = plan->total_k;
    info->n_fwd_items = plan->n_fwd;
    info->n_dkv_items = plan->n_dkv;
    info->attended_pairs = plan->pairs;
    info->useful_flops_fwd = 4 * plan->pairs * plan->d * plan->Hq;
    info->useful_flops_bwd = 10 * plan->pairs * plan->d * plan->Hq;
    // -D and LSE*log2(e) per (head, row), then 256 bytes for the work queues of the two kernels
    info->bwd_workspace_bytes = ((((int64_t)plan->Hq * plan->total_q * 8) + 255) & ~(int64_t)255) + 256;
    if (plan->head_split > 1)  // fp32 partial dK and dV of every share of the heads
        info->bwd_workspace_bytes += 2 * (int64_t)plan->head_split * plan->total_k * plan->Hkv * plan->d * 4;
    info->num_segments = plan->NS;
    info->head_split = plan->head_split;
    info->wg_query_rows = plan->wg_query_rows;
    info->reserved = 0;
    return SKRULL_OK;
}

int skrull_attn_plan_export(const skrull_attn_plan_t *plan, int which, void *dst, size_t bytes)
{
    if (!plan || !dst) return SKRULL_EINVAL;
    const int32_t *src = nullptr;
    size_t n = 0;
    switch (which) {
    case SKRULL_ARRAY_CU_Q: src = plan->cu_q; n = (size_t)plan->NS + 1; break;
    case SKRULL_ARRAY_CU_K: src = plan->cu_k; n = (size_t)plan->NS + 1; break;
    case SKRULL_ARRAY_Q_BEGIN: src = plan->q_begin; n = (size_t)plan->NS; break;
    case SKRULL_ARRAY_Q_LEN: src = plan->q_len; n = (size_t)plan->NS; break;
    case SKRULL_ARRAY_KV_LEN: src = plan->kv_len; n = (size_t)plan->NS; break;
    case SKRULL_ARRAY_SHARES_KV: src = plan->shares_kv; n = (size_t)plan->NS; break;
    case SKRULL_ARRAY_FWD_ITEMS: src = plan->fwd_items; n = (size_t)plan->n_fwd * 4; break;
    case SKRULL_ARRAY_DKV_ITEMS: src = plan->dkv_items; n = (size_t)plan->n_dkv * 4; break;
    default: return SKRULL_EINVAL;
    }
    if (bytes != n * sizeof(int32_t)) return SKRULL_EINVAL;
    if (int rc = check_plan_device(plan)) return rc;
    hipError_t e = hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, "hipMemcpy(export)");
    return SKRULL_OK;
}

int skrull_attn_fwd(const skrull_attn_plan_t *plan, const void *q, const void *k, const void *v,
                    void *o, float *lse, void *hip_stream)
{
    if (!plan) return SKRULL_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse))
        return SKRULL_EINVAL;
    if (int rc = check_plan_device(plan)) return rc;
    if (g_prof.on) (void)hipEventRecord(g_prof.ev[0], (hipStream_t)hip_stream);
    WgTrace *trace = nullptr;
    if (g_trace.buf) {
        if ((size_t)grid_fwd(plan) > g_trace.records) return SKRULL_EINVAL;
        trace = g_trace.buf;
    }
    hipError_t e = launch_fwd(plan, q, k, v, o, lse, (hipStream_t)hip_stream, trace);
    if (e != hipSuccess) return hip_fail(e, "forward launch");
    if (g_prof.on) { (void)hipEventRecord(g_prof.ev[1], (hipStream_t)hip_stream); g_prof.fwd_seen = true; }
    return SKRULL_OK;
}

int skrull_attn_bwd(const skrull_attn_plan_t *plan, const void *q, const void *k, const void *v,
                    const void *o, const float *lse, const void *d_o, void *dq, void *dk, void *dv,
                    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!plan) return SKRULL_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
        misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv) ||
        misaligned(workspace))
        return SKRULL_EINVAL;
    skrull_attn_plan_info_t info;
    skrull_attn_plan_info(plan, &info);
    if ((int64_t)workspace_bytes < info.bwd_workspace_bytes) return SKRULL_EINVAL;
    if (int rc = check_plan_device(plan)) return rc;
    WgTrace *trace = nullptr;
    if (g_trace.buf) {  // after the forward's records
        const size_t first = (size_t)grid_fwd(plan);
        if (first + grid_dq(plan) + grid_dkv(plan) > g_trace.records) return SKRULL_EINVAL;
        trace = g_trace.buf + first;
    }
    hipError_t e = launch_bwd(plan, q, k, v, o, lse, d_o, dq, dk, dv, (float *)workspace,
                              (hipStream_t)hip_stream, g_prof.on ? g_prof.ev + 2 : nullptr, trace);
    if (e != hipSuccess) return hip_fail(e, "backward launch");
    if (g_prof.on) g_prof.bwd_seen = true;
    return SKRULL_OK;
}

int skrull_attn_bwd_static(const skrull_attn_plan_t *plan, const void *q, const void *k, const void *v,
                           const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                           void *dv, void *hip_stream)
{
    if (!plan) return SKRULL_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) ||
        misaligned(d_o) || misaligned(dq) || misaligned(dk) || misaligned(dv))
        return SKRULL_EINVAL;
    skrull_attn_plan_info_t info;
    skrull_attn_plan_info(plan, &info);
    if (info.bwd_workspace_bytes > (int64_t)SKRULL_STATIC_SCRATCH_BYTES) {
        snprintf(g_err, sizeof g_err,
                 "this plan needs %lld bytes of backward workspace, the static one holds %lld "
                 "(use skrull_attn_bwd, or a plan with head_split = 1 if the partial sums are what is large)",
                 (long long)info.bwd_workspace_bytes, (long long)SKRULL_STATIC_SCRATCH_BYTES);
        return SKRULL_EINVAL;
    }
    if (int rc = check_plan_device(plan)) return rc;
    void *ws = nullptr;  // resolved when the plan was made; looked up again only if that was another process state
    if (int rc = resolve_scratch(plan->device, &ws)) return rc;
    hipError_t e = launch_bwd(plan, q, k, v, o, lse, d_o, dq, dk, dv, (float *)ws,
                              (hipStream_t)hip_stream, g_prof.on ? g_prof.ev + 2 : nullptr, nullptr);
    if (e != hipSuccess) return hip_fail(e, "backward launch");
    if (g_prof.on) g_prof.bwd_seen = true;
    return SKRULL_OK;
}

void skrull_attn_plan_destroy(skrull_attn_plan_t *plan)
{
    if (!plan) return;
    if (plan->pool) (void)hipFree(plan->pool);
    delete plan;
}

int skrull_attn_mfma_ceiling(void *hip_stream, float *tflops)
{
    if (!tflops) return SKRULL_EINVAL;
    int dev = 0, compute_units = 0;
    int rc = check_device(&dev, &compute_units);
    if (rc != SKRULL_OK) return rc;
    const int blocks = compute_units, iters = 40000;  // ~20 ms of MFMAs
    float ms = 0.0f;
    void *ws = nullptr;  // the probe's sink (blocks x 2 KB) is the static workspace: nothing is allocated
    if ((size_t)blocks * 512 * sizeof(float) > (size_t)SKRULL_STATIC_SCRATCH_BYTES) return SKRULL_EUNSUPPORTED;
    if ((rc = resolve_scratch(dev, &ws)) != SKRULL_OK) return rc;
    hipError_t e = run_mfma_probe(blocks, iters, (float *)ws, (hipStream_t)hip_stream, &ms);
    if (e != hipSuccess) return hip_fail(e, "MFMA probe");
    // blocks x 8 waves x iters x 4 MFMAs x 32*32*16*2 flop
    *tflops = (float)((double)blocks * 8.0 * iters * 4.0 * 32768.0 / (ms * 1e-3) / 1e12);
    return SKRULL_OK;
}

int skrull_attn_trace(void *records, size_t bytes)
{
    if (records && (misaligned(records) || bytes < sizeof(WgTrace))) return SKRULL_EINVAL;
    g_trace.buf = (WgTrace *)records;
    g_trace.records = records ? bytes / sizeof(WgTrace) : 0;
    return SKRULL_OK;
}

int skrull_attn_trace_layout(const skrull_attn_plan_t *plan, int32_t first_record[3], int32_t num_records[3])
{
    if (!plan || !first_record || !num_records) return SKRULL_EINVAL;
    num_records[0] = grid_fwd(plan);
    num_records[1] = grid_dq(plan);
    num_records[2] = grid_dkv(plan);
    first_record[0] = 0;
    first_record[1] = num_records[0];
    first_record[2] = num_records[0] + num_records[1];
    return SKRULL_OK;
}

int skrull_attn_profile(int enable)
{
    ProfileState &ps = g_prof;
    if (enable && !ps.made) {
        for (int i = 0; i < 6; ++i) {
            hipError_t e = hipEventCreate(&ps.ev[i]);
            if (e != hipSuccess) {
                while (i-- > 0) (void)hipEventDestroy(ps.ev[i]);
                return hip_fail(e, "hipEventCreate");
            }
        }
        ps.made = true;
    }
    if (!enable && ps.made) {  // switching off releases the thread's events
        for (int i = 0; i < 6; ++i) (void)hipEventDestroy(ps.ev[i]);
        ps.made = false;
    }
    ps.on = enable != 0;
    ps.fwd_seen = ps.bwd_seen = false;
    return SKRULL_OK;
}

int skrull_attn_profile_read(float ms[4])
{
    ProfileState &ps = g_prof;
    if (!ms || !ps.on) return SKRULL_EINVAL;
    for (int i = 0; i < 4; ++i) ms[i] = -1.0f;
    hipError_t e;
    if (ps.fwd_seen) {
        if ((e = hipEventSynchronize(ps.ev[1])) != hipSuccess) return hip_fail(e, "hipEventSynchronize");
        if ((e = hipEventElapsedTime(&ms[0], ps.ev[0], ps.ev[1])) != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
    }
    if (ps.bwd_seen) {
        // backward events: ev[2] start, ev[3] after dQ (which also forms D), ev[4] after dK/dV
        if ((e = hipEventSynchronize(ps.ev[4])) != hipSuccess) return hip_fail(e, "hipEventSynchronize");
        ms[1] = 0.0f;
        if ((e = hipEventElapsedTime(&ms[3], ps.ev[2], ps.ev[3])) != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
        if ((e = hipEventElapsedTime(&ms[2], ps.ev[3], ps.ev[4])) != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
    }
    return SKRULL_OK;
}

const char *skrull_attn_strerror(int code)
{
    thread_local char buf[320];
    switch (code) {
    case SKRULL_OK: return "ok";
    case SKRULL_EINVAL:
        if (g_err[0]) { snprintf(buf, sizeof buf, "invalid argument (%s)", g_err); return buf; }
        return "invalid argument";
    case SKRULL_ENOMEM: return "out of memory";
    case SKRULL_EHIP: snprintf(buf, sizeof buf, "HIP runtime error (%s)", g_err); return buf;
    case SKRULL_EUNSUPPORTED: return "no gfx950 (MI355X) device available";
    case SKRULL_ESCHED: return "DACP scheduling error: the micro-batch does not fit the buckets";
    default: return "unknown error code";
    }
}

}  // extern "C"
