// Varlen descriptor builder and cost-ordered tile work lists, on the device.
//
// The micro-batch is stated the way the paper states it (Sec. 4.1, Eq. 1-8):
// full lengths S[K] plus, per sequence, local (degree 1) or distributed over N
// ranks with this GPU holding slice `index` (Eq. 8: S_k/N tokens per rank), cut
// either as one contiguous slice or as two chunks that balance the causal work.
// Three small kernels:
//   1. plan_ranges : per-segment query/KV ranges, the packed offsets
//                    (exclusive scans), per-segment work-item offsets, totals
//   2. plan_emit   : one thread per work item writes {seq, block, x, cost}
//   3. plan_sort   : stable descending-cost order by rank counting, so the
//                    hardware dispatcher, which hands out workgroups in grid
//                    order, always gives the heaviest remaining tile to the
//                    first compute unit that frees up -- the paper's
//                    least-loaded-first rule (Alg. 1, argmin over L) applied
//                    to compute units instead of ranks.
#include "common.h"

namespace {

constexpr int kScanThreads = 256;

// Block-wide exclusive scan of one int64 per thread; returns the exclusive
// prefix and writes the block total to *total (same value in every thread).
// Inside a wavefront the scan runs on lane shuffles; the four wavefronts' totals
// meet in LDS (two barriers per scan).
__device__ inline int64_t block_exclusive_scan(int64_t v, int64_t *lds, int64_t *total)
{
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int64_t incl = v;
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    int64_t before = 0, all = 0;
    for (int w = 0; w < kScanThreads / 64; ++w) {
        const int64_t x = lds[w];
        if (w < wave) before += x;
        all += x;
    }
    *total = all;
    __syncthreads();  // lds may be reused by the next scan
    return before + incl - v;
}

__device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// One thread per sequence.  A sequence cut the contiguous way is one query
// segment; one cut the load-balanced way (chunks r and 2N-1-r of 2N) is two
// consecutive segments, early chunk first, that share one key/value prefix (the
// late chunk's).  All per-segment arrays are indexed by segment; fwd_off / dkv_off
// are the work-item offsets (an early chunk owns no dK/dV items: its offset equals
// its partner's).
__global__ __launch_bounds__(kScanThreads) void plan_ranges_kernel(
    const int32_t *__restrict__ S, const int32_t *__restrict__ N, const int32_t *__restrict__ R,
    const int32_t *__restrict__ Z, int32_t K, int32_t BM, int32_t BN, int32_t max_q_rows,
    int32_t max_k_rows, int32_t *__restrict__ q_begin, int32_t *__restrict__ q_len,
    int32_t *__restrict__ kv_len, int32_t *__restrict__ cu_q, int32_t *__restrict__ cu_k,
    int32_t *__restrict__ shares_kv, int32_t *__restrict__ fwd_off, int32_t *__restrict__ dkv_off,
    int32_t cap_fwd, int32_t cap_dkv, int32_t bn_alt, int32_t kv_heads, int32_t compute_units,
    PlanTotals *__restrict__ totals)
{
    __shared__ int64_t lds[kScanThreads];
    __shared__ int32_t first_bad;
    const int t = threadIdx.x;
    if (t == 0) first_bad = 0x7fffffff;
    __syncthreads();
    // Choice between BN and a larger dK/dV block bn_alt (0 = no choice to make).  The larger
    // one is taken when, with blocks of BN key rows, the costliest work item exceeds an even
    // share of the whole list over the compute units (cost_max > cost_sum * Hkv / CUs), the
    // same ratio that decides the head split; the costs are those of the dK/dV items that
    // plan_emit_kernel would write for BN.  It is also taken, given a sequence of at least two
    // of the larger blocks, when their list is still long (at least five x KV heads per compute
    // unit) or when the costliest item stays under 0.7 of that even share.  Fewer, larger
    // workgroups run the rounds 7-18 % faster (measured on 14 to 64 heads x 16,384-65,536 tokens,
    // uniform and ragged lengths) but balance worse: with few items and a costliest one between
    // 0.7 and 1.0 of the even share, ragged micro-batches lost 4-15 % by them.
    if (bn_alt != 0) {
        int64_t c_sum = 0, c_max = 0, n_alt = 0, longest = 0;
        for (int32_t k = t; k < K; k += kScanThreads) {
            const int64_t s = S[k], n = N[k], r = R[k], z = Z[k];
            const int64_t chunks = n * (z ? 2 : 1);
            if (s < 1 || n < 1 || r < 0 || r >= n || (z != 0 && z != 1) || chunks > s) continue;
            const int64_t idx[2] = {r, 2 * n - 1 - r};
            const int nseg = (int)z + 1;
            int64_t qb[2], qe[2];
            for (int part = 0; part < nseg; ++part) {
                qb[part] = (idx[part] * s) / chunks;
                qe[part] = ((idx[part] + 1) * s) / chunks;
            }
            n_alt += ceil_div64(qe[nseg - 1], bn_alt);
            longest = qe[nseg - 1] > longest ? qe[nseg - 1] : longest;
            for (int64_t j0 = 0; j0 < qe[nseg - 1]; j0 += BN) {
                int64_t cost = 0;
                for (int part = 0; part < nseg; ++part) {
                    if (j0 >= qe[part]) continue;
                    const int64_t i0 = j0 > qb[part] ? j0 - qb[part] : 0;
                    cost += ceil_div64(qe[part] - qb[part], BM) - i0 / BM;
                }
                c_sum += cost;
                c_max = cost > c_max ? cost : c_max;
            }
        }
        int64_t tot;
        block_exclusive_scan(c_sum, lds, &tot);
        c_sum = tot;
        // maximum over the block through the same LDS array
        lds[t] = c_max;
        __syncthreads();
        for (int off = kScanThreads / 2; off > 0; off >>= 1) {
            if (t < off && lds[t + off] > lds[t]) lds[t] = lds[t + off];
            __syncthreads();
        }
        c_max = lds[0];
        __syncthreads();
        block_exclusive_scan(n_alt, lds, &tot);
        n_alt = tot;
        lds[t] = longest;
        __syncthreads();
        for (int off = kScanThreads / 2; off > 0; off >>= 1) {
            if (t < off && lds[t + off] > lds[t]) lds[t] = lds[t + off];
            __syncthreads();
        }
        longest = lds[0];
        __syncthreads();
        const bool long_list = n_alt * kv_heads >= 5 * (int64_t)compute_units;
        const bool even_list = 10 * c_max * compute_units <= 7 * c_sum * kv_heads;
        if (c_max * compute_units > c_sum * kv_heads ||
            ((long_list || even_list) && longest >= 2 * (int64_t)bn_alt))
            BN = bn_alt;
    }
    int64_t base_s = 0, base_q = 0, base_k = 0, base_f = 0, base_d = 0, pairs = 0;
    for (int32_t k0 = 0; k0 < K; k0 += kScanThreads) {
        const int32_t k = k0 + t;
        int64_t qb[2] = {0, 0}, ql[2] = {0, 0}, nf[2] = {0, 0};
        int64_t nseg = 0, owned = 0, nd = 0, pr = 0;
        if (k < K) {
            const int64_t s = S[k], n = N[k], r = R[k], z = Z[k];
            const int64_t chunks = n * (z ? 2 : 1);
            if (s < 1 || n < 1 || r < 0 || r >= n || (z != 0 && z != 1) || chunks > s) {
                atomicMin(&first_bad, k);
            } else {
                nseg = z + 1;
                const int64_t idx[2] = {r, 2 * n - 1 - r};
                for (int part = 0; part < nseg; ++part) {
                    const int64_t b = (idx[part] * s) / chunks, e = ((idx[part] + 1) * s) / chunks;
                    qb[part] = b;
                    ql[part] = e - b;
                    nf[part] = ceil_div64(e - b, BM);
                    pr += (e * (e + 1) - b * (b + 1)) / 2;
                    owned = e;  // the late chunk's prefix covers the early one's
                }
                // one sequence of one tensor must span fewer than 2^31 elements
                // (the kernels address inside a sequence with 32-bit offsets)
                if (ql[0] + ql[1] > max_q_rows || owned > max_k_rows) atomicMin(&first_bad, k);
                nd = ceil_div64(owned, BN);
            }
        }
        int64_t tot;
        const int64_t e_s = block_exclusive_scan(nseg, lds, &tot);
        const int64_t seg0 = base_s + e_s;
        base_s += tot;
        const int64_t e_q = block_exclusive_scan(ql[0] + ql[1], lds, &tot);
        const int64_t row0 = base_q + e_q;
        base_q += tot;
        const int64_t e_k = block_exclusive_scan(owned, lds, &tot);
        const int64_t krow0 = base_k + e_k;
        base_k += tot;
        const int64_t e_f = block_exclusive_scan(nf[0] + nf[1], lds, &tot);
        const int64_t f0 = base_f + e_f;
        base_f += tot;
        const int64_t e_d = block_exclusive_scan(nd, lds, &tot);
        const int64_t d0 = base_d + e_d;
        base_d += tot;
        block_exclusive_scan(pr, lds, &tot);
        pairs += tot;
        for (int part = 0; part < nseg; ++part) {
            const int64_t sg = seg0 + part;
            q_begin[sg] = (int32_t)qb[part];
            q_len[sg] = (int32_t)ql[part];
            kv_len[sg] = (int32_t)(qb[part] + ql[part]);
            cu_q[sg] = (int32_t)(row0 + (part ? ql[0] : 0));
            cu_k[sg] = (int32_t)krow0;
            shares_kv[sg] = part;
            fwd_off[sg] = (int32_t)(f0 + (part ? nf[0] : 0));
            dkv_off[sg] = (int32_t)d0;
        }
    }
    __syncthreads();
    if (t == 0) {
        cu_q[base_s] = (int32_t)base_q;
        cu_k[base_s] = (int32_t)base_k;
        fwd_off[base_s] = (int32_t)base_f;
        dkv_off[base_s] = (int32_t)base_d;
        totals->total_q = base_q;
        totals->total_k = base_k;
        totals->n_fwd = base_f;
        totals->n_dkv = base_d;
        totals->pairs = pairs;
        totals->bad_entry = (first_bad == 0x7fffffff) ? 0 : first_bad + 1;
        totals->n_seg = (int32_t)base_s;
        totals->dkv_cost_sum = 0;
        totals->dkv_cost_max = 0;
        totals->cap_fwd = cap_fwd;
        totals->cap_dkv = cap_dkv;
        totals->block_n = BN;
    }
}

// Largest k with off[k] <= item (off is an exclusive scan with off[K] = n).
__device__ inline int32_t owner_of(const int32_t *off, int32_t K, int32_t item)
{
    int32_t lo = 0, hi = K;  // invariant: off[lo] <= item < off[hi]
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (off[mid] <= item) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(256) void plan_emit_kernel(
    int32_t K, int32_t BM, const int32_t *__restrict__ q_begin,
    const int32_t *__restrict__ q_len, const int32_t *__restrict__ kv_len,
    const int32_t *__restrict__ cu_q, const int32_t *__restrict__ shares_kv,
    const int32_t *__restrict__ fwd_off,
    const int32_t *__restrict__ dkv_off, int4 *__restrict__ fwd_items,
    int4 *__restrict__ dkv_items, PlanTotals *__restrict__ totals)
{
    // the grid covers an upper bound of the item counts; the counts themselves are the
    // ranges kernel's (clamped: a count past the limit is rejected by the host afterwards)
    const int32_t n_fwd = (int32_t)min((long long)totals->n_fwd, (long long)totals->cap_fwd);
    const int32_t n_dkv = (int32_t)min((long long)totals->n_dkv, (long long)totals->cap_dkv);
    const int32_t BN = totals->block_n;  // the ranges kernel's choice where the caller left it open
    const int32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n_fwd) {
        const int32_t k = owner_of(fwd_off, K, t);
        const int32_t m = t - fwd_off[k];
        const int64_t row0 = (int64_t)m * BM;
        const int64_t left = q_len[k] - row0;
        const int64_t rows = left < BM ? left : BM;
        fwd_items[t] = make_int4(k, m, (int32_t)(cu_q[k] + row0),
                                 (int32_t)ceil_div64((int64_t)q_begin[k] + row0 + rows, BN));
    }
    if (t < n_dkv) {
        // equal offsets (an early chunk and its partner) resolve to the later segment,
        // the one that owns the shared prefix
        const int32_t k = owner_of(dkv_off, K, t);
        const int32_t b = t - dkv_off[k];
        int64_t i0 = (int64_t)b * BN - q_begin[k];
        if (i0 < 0) i0 = 0;
        const int32_t m0 = (int32_t)(i0 / BM);
        int32_t cost = (int32_t)ceil_div64(q_len[k], BM) - m0;
        if (shares_kv[k] && (int64_t)b * BN < kv_len[k - 1]) {  // query blocks of the early chunk
            int64_t j0 = (int64_t)b * BN - q_begin[k - 1];
            if (j0 < 0) j0 = 0;
            cost += (int32_t)ceil_div64(q_len[k - 1], BM) - (int32_t)(j0 / BM);
        }
        dkv_items[t] = make_int4(k, b, m0, cost);
        atomicAdd(&totals->dkv_cost_sum, (unsigned long long)cost);
        atomicMax(&totals->dkv_cost_max, cost);
    }
}

// Stable sort by descending .w: item a goes to slot
//   #{b : cost_b > cost_a} + #{b < a : cost_b == cost_a}.
// Costs are streamed through LDS in tiles; every thread of a block walks the
// same tile, so the reads are broadcasts.
__global__ __launch_bounds__(256) void plan_sort_kernel(const int4 *__restrict__ in,
                                                        const PlanTotals *__restrict__ totals,
                                                        int which, int4 *__restrict__ out)
{
    __shared__ int32_t tile[1024];
    const int32_t n = which == 0 ? (int32_t)min((long long)totals->n_fwd, (long long)totals->cap_fwd)
                                 : (int32_t)min((long long)totals->n_dkv, (long long)totals->cap_dkv);
    const int32_t a = blockIdx.x * blockDim.x + threadIdx.x;
    const int4 me = (a < n) ? in[a] : make_int4(0, 0, 0, 0);
    int32_t rank = 0;
    for (int32_t b0 = 0; b0 < n; b0 += 1024) {
        __syncthreads();
        for (int32_t i = threadIdx.x; i < 1024; i += blockDim.x)
            tile[i] = (b0 + i < n) ? in[b0 + i].w : -1;
        __syncthreads();
        const int32_t lim = (n - b0 < 1024) ? n - b0 : 1024;
        for (int32_t i = 0; i < lim; ++i) {
            const int32_t cb = tile[i];
            rank += (cb > me.w) || (cb == me.w && b0 + i < a);
        }
    }
    if (a < n) out[rank] = me;
}

// ---------------------------------------------------------------------------
// Long lists: stable least-significant-digit radix sort on key = key_max - cost
// (ascending key = descending cost), 8 bits per pass, 1024 consecutive items per
// block.  Three kernels per pass: per-block digit histogram; exclusive scan of the
// (digit, block) table in digit-major order; scatter, in which an item's offset is
// its digit's start + the items of that digit in earlier blocks + those before it
// in its own block (which keeps equal keys in their order: the sort is stable).
// ---------------------------------------------------------------------------
constexpr int kRadixBlock = 1024;

__device__ inline int32_t list_length(const PlanTotals *totals, int which)
{
    return which == 0 ? (int32_t)min((long long)totals->n_fwd, (long long)totals->cap_fwd)
                      : (int32_t)min((long long)totals->n_dkv, (long long)totals->cap_dkv);
}

__global__ __launch_bounds__(256) void radix_hist_kernel(const int4 *__restrict__ in,
                                                         const PlanTotals *__restrict__ totals, int which,
                                                         int32_t key_max, int shift, int32_t nb,
                                                         int32_t *__restrict__ hist)
{
    __shared__ int32_t h[256];
    const int32_t n = list_length(totals, which);
    h[threadIdx.x] = 0;
    __syncthreads();
    const int32_t base = blockIdx.x * kRadixBlock;
    for (int32_t i = threadIdx.x; i < kRadixBlock; i += 256)
        if (base + i < n) atomicAdd(&h[((key_max - in[base + i].w) >> shift) & 255], 1);
    __syncthreads();
    hist[threadIdx.x * nb + blockIdx.x] = h[threadIdx.x];
}

// one block; thread d scans the counts of digit d over the blocks, then the digits are scanned
__global__ __launch_bounds__(256) void radix_scan_kernel(int32_t *__restrict__ hist, int32_t nb)
{
    __shared__ int64_t lds[kScanThreads];
    const int d = threadIdx.x;
    int32_t run = 0;
    for (int32_t b = 0; b < nb; ++b) {
        const int32_t c = hist[d * nb + b];
        hist[d * nb + b] = run;
        run += c;
    }
    int64_t tot;
    const int32_t start = (int32_t)block_exclusive_scan(run, lds, &tot);
    for (int32_t b = 0; b < nb; ++b) hist[d * nb + b] += start;
}

__global__ __launch_bounds__(256) void radix_scatter_kernel(const int4 *__restrict__ in,
                                                            const PlanTotals *__restrict__ totals, int which,
                                                            int32_t key_max, int shift, int32_t nb,
                                                            const int32_t *__restrict__ hist,
                                                            int4 *__restrict__ out)
{
    __shared__ unsigned char dig[kRadixBlock];
    const int32_t n = list_length(totals, which);
    const int32_t base = blockIdx.x * kRadixBlock;
    const int32_t cnt = min(kRadixBlock, n - base);
    if (cnt <= 0) return;
    // thread t owns the consecutive items 4t .. 4t+3 of the block
    int4 mine[4];
    for (int e = 0; e < 4; ++e) {
        const int32_t i = 4 * threadIdx.x + e;
        if (i < cnt) {
            mine[e] = in[base + i];
            dig[i] = (unsigned char)(((key_max - mine[e].w) >> shift) & 255);
        }
    }
    __syncthreads();
    for (int e = 0; e < 4; ++e) {
        const int32_t i = 4 * threadIdx.x + e;
        if (i >= cnt) break;
        const unsigned char d = dig[i];
        int32_t before = 0;  // items of the same digit earlier in this block
        for (int32_t j = 0; j < i; ++j) before += dig[j] == d;
        out[hist[(int32_t)d * nb + blockIdx.x] + before] = mine[e];
    }
}

}  // namespace

hipError_t launch_plan_ranges(const int32_t *S, const int32_t *N, const int32_t *r,
                              const int32_t *cut, int32_t K, int32_t BM, int32_t BN,
                              int32_t max_q_rows, int32_t max_k_rows, int32_t *q_begin,
                              int32_t *q_len, int32_t *kv_len, int32_t *cu_q, int32_t *cu_k,
                              int32_t *shares_kv, int32_t *fwd_off, int32_t *dkv_off,
                              int32_t cap_fwd, int32_t cap_dkv, int32_t bn_alt, int32_t kv_heads,
                              int32_t compute_units, PlanTotals *totals, hipStream_t st)
{
    plan_ranges_kernel<<<1, kScanThreads, 0, st>>>(S, N, r, cut, K, BM, BN, max_q_rows, max_k_rows,
                                                   q_begin, q_len, kv_len, cu_q, cu_k, shares_kv,
                                                   fwd_off, dkv_off, cap_fwd, cap_dkv, bn_alt, kv_heads,
                                                   compute_units, totals);
    return hipGetLastError();
}

// Above this many items (the host's upper bound) a list is sorted by radix passes instead of
// by rank counting, which is quadratic (measured: 0.25 ms for 5,000 items, 3 ms for 16,000; the
// radix passes take 0.05 ms there).
constexpr int32_t kRankSortMax = 2048;

int plan_radix_passes(int32_t cap, int32_t cost_bound)
{
    if (cap <= kRankSortMax) return 0;
    int bits = 1;
    while (bits < 31 && (1 << bits) <= cost_bound) ++bits;
    return (bits + 7) / 8;
}

int64_t plan_radix_ints(int32_t cap_fwd, int32_t cap_dkv, int32_t cost_bound)
{
    int64_t n = 0;
    if (plan_radix_passes(cap_fwd, cost_bound)) n += 256 * (int64_t)((cap_fwd + kRadixBlock - 1) / kRadixBlock);
    if (plan_radix_passes(cap_dkv, cost_bound)) n += 256 * (int64_t)((cap_dkv + kRadixBlock - 1) / kRadixBlock);
    return n;
}

// Sort one list.  `a` holds the emitted items when the number of passes is odd (or zero), `b`
// when it is even, so that the last pass (or the rank sort) always writes the plan's array `b`.
static hipError_t sort_list(int which, int32_t cap, int32_t cost_bound, int4 *a, int4 *b, int32_t *hist,
                            PlanTotals *totals, hipStream_t st)
{
    const int passes = plan_radix_passes(cap, cost_bound);
    if (passes == 0) {
        plan_sort_kernel<<<(cap + 255) / 256, 256, 0, st>>>(a, totals, which, b);
        return hipGetLastError();
    }
    int key_bits = 8 * passes;
    const int32_t key_max = key_bits >= 31 ? INT32_MAX : (1 << key_bits) - 1;  // >= any cost
    const int32_t nb = (cap + kRadixBlock - 1) / kRadixBlock;
    int4 *src = (passes & 1) ? a : b, *dst = (passes & 1) ? b : a;
    for (int pass = 0; pass < passes; ++pass) {
        radix_hist_kernel<<<nb, 256, 0, st>>>(src, totals, which, key_max, 8 * pass, nb, hist);
        radix_scan_kernel<<<1, 256, 0, st>>>(hist, nb);
        radix_scatter_kernel<<<nb, 256, 0, st>>>(src, totals, which, key_max, 8 * pass, nb, hist, dst);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        int4 *t = src; src = dst; dst = t;
    }
    return hipSuccess;
}

hipError_t launch_plan_items(const skrull_attn_plan_t *p, const int32_t *fwd_off,
                             const int32_t *dkv_off, int32_t cap_fwd, int32_t cap_dkv,
                             int32_t *scratch_fwd, int32_t *scratch_dkv, int32_t *radix_hist,
                             int32_t cost_bound, PlanTotals *totals, hipStream_t st)
{
    // grids are sized by the host's upper bounds of the item counts; the kernels take the
    // counts from `totals` on the device, so no round trip to the host is needed in between
    const int32_t n = cap_fwd > cap_dkv ? cap_fwd : cap_dkv;
    // the emit kernel writes each list where its sort starts from
    const bool fwd_even = plan_radix_passes(cap_fwd, cost_bound) != 0 && plan_radix_passes(cap_fwd, cost_bound) % 2 == 0;
    const bool dkv_even = plan_radix_passes(cap_dkv, cost_bound) != 0 && plan_radix_passes(cap_dkv, cost_bound) % 2 == 0;
    plan_emit_kernel<<<(n + 255) / 256, 256, 0, st>>>(
        p->NS, p->BM, p->q_begin, p->q_len, p->kv_len, p->cu_q, p->shares_kv, fwd_off, dkv_off,
        (int4 *)(fwd_even ? p->fwd_items : scratch_fwd), (int4 *)(dkv_even ? p->dkv_items : scratch_dkv), totals);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int32_t *hist_dkv = radix_hist;
    if (plan_radix_passes(cap_fwd, cost_bound)) hist_dkv += 256 * (int64_t)((cap_fwd + kRadixBlock - 1) / kRadixBlock);
    e = sort_list(0, cap_fwd, cost_bound, (int4 *)scratch_fwd, (int4 *)p->fwd_items, radix_hist, totals, st);
    if (e != hipSuccess) return e;
    return sort_list(1, cap_dkv, cost_bound, (int4 *)scratch_dkv, (int4 *)p->dkv_items, hist_dkv, totals, st);
}
