/*
 * skrull_oracle.c -- plain CPU fp64 oracle for packed variable-length causal
 * attention (forward and analytic backward) over one scheduled micro-batch,
 * plus the integer descriptor / tile work-list layout.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, written-out definition that the
 * GPU library is checked against.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP path and must never be used to produce a product
 * result.
 *
 * What the micro-batch is (paper, Sec. 4.1 "DACP", Eq. 1-8): a context-parallel
 * rank j receives every local sequence assigned to it whole (P_kj = 1) and a
 * 1/N slice of every distributed sequence (D_k = 1; Eq. 8 charges S_k/N tokens
 * to each rank, Eq. 4 charges 1/N of its FLOPs).  The sequences are packed
 * without padding (App. B.1, "sequence packing") and never attend to each
 * other.  The paper treats attention itself as a black box of O(n^2) compute
 * and O(n) memory (Sec. 4.2.1 "Local sequence assignment"); the arithmetic
 * below is the textbook definition of causal softmax attention and of its
 * gradient, evaluated in double precision with no tiling, no online softmax
 * and no reordering.
 *
 * Readings the paper leaves open (each also listed in the design notes):
 *  - the slice of a distributed sequence is the CONTIGUOUS query range
 *    [floor(r*S/N), floor((r+1)*S/N)) of shard index r, attending to the key /
 *    value prefix [0, q_end) at its true global positions; or, as a
 *    load-balanced alternative, chunks r and 2N-1-r of a cut into 2N chunks
 *    (see oracle_ranges);
 *  - query head h reads key/value head h / (Hq/Hkv) (contiguous GQA groups);
 *  - LSE is the natural log of the sum of exp(scale * q.k) over allowed keys.
 *
 * Inputs are float (bf16 values widened exactly); every sum is carried in
 * double.  Parity status: every function here is pinned by tests/test_oracle_*
 * (dense library softmax in fp64, autograd, finite differences, brute-force
 * tile counting, closed forms); nothing is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Integer part                                                        */
/* ------------------------------------------------------------------ */

/* Query segments and packed offsets (paper Eq. 8: a distributed sequence
 * contributes S_k/N tokens to each rank; local ones contribute S_k).
 *
 * cut[k] = 0: ONE segment, the contiguous slice of shard index r:
 *   q_begin = floor(r*S/N), q_end = floor((r+1)*S/N), kv_len = q_end.
 * cut[k] = 1 (load-balanced cut; the paper leaves the cut open and its Eq. 4
 *   assumes every rank does 1/N of the work, which a causal contiguous cut does
 *   not give): the sequence is cut into 2N chunks [floor(i*S/2N), floor((i+1)*S/2N));
 *   the rank holds chunk r and chunk 2N-1-r, as TWO consecutive segments (early
 *   chunk first) whose query rows follow each other in Q/O/dQ/dO and which share
 *   ONE key/value prefix [0, end of the late chunk): cu_k is the same for both,
 *   shares_kv[late segment] = 1.
 * A segment is all the other functions here know: query rows q_begin..q_begin+q_len-1
 * (global positions) at packed rows cu_q.., seeing keys 0..position at packed rows
 * cu_k..; kv_len = q_begin + q_len.
 * Outputs have room for 2K segments (cu_q / cu_k: 2K+1; the entry after the last
 * segment holds the total).  Returns the number of segments, or -1 on an invalid
 * entry (S<1, N<1, r outside [0,N), fewer tokens than chunks, cut not 0/1) or if a
 * total does not fit in int32.  cut may be NULL (all 0). */
int oracle_ranges(int32_t K, const int32_t *S, const int32_t *N, const int32_t *r,
                  const int32_t *cut,
                  int32_t *q_begin, int32_t *q_len, int32_t *kv_len,
                  int32_t *cu_q, int32_t *cu_k, int32_t *shares_kv)
{
    int64_t tq = 0, tk = 0;
    int32_t ns = 0;
    if (K < 1) return -1;
    for (int32_t k = 0; k < K; ++k) {
        const int32_t z = cut ? cut[k] : 0;
        if (z != 0 && z != 1) return -1;
        const int64_t chunks = (int64_t)N[k] * (z ? 2 : 1);
        if (S[k] < 1 || N[k] < 1 || r[k] < 0 || r[k] >= N[k] || chunks > S[k]) return -1;
        const int64_t idx[2] = {r[k], 2 * (int64_t)N[k] - 1 - r[k]};
        int64_t owned = 0;
        for (int32_t part = 0; part <= z; ++part) {
            const int64_t b = (idx[part] * (int64_t)S[k]) / chunks;
            const int64_t e = ((idx[part] + 1) * (int64_t)S[k]) / chunks;
            q_begin[ns] = (int32_t)b;
            q_len[ns] = (int32_t)(e - b);
            kv_len[ns] = (int32_t)e;
            cu_q[ns] = (int32_t)tq;
            cu_k[ns] = (int32_t)tk;
            shares_kv[ns] = part;
            tq += e - b;
            owned = e;              /* the late chunk's prefix covers the early one's */
            ++ns;
        }
        tk += owned;
        if (tq > INT32_MAX || tk > INT32_MAX) return -1;
    }
    cu_q[ns] = (int32_t)tq;
    cu_k[ns] = (int32_t)tk;
    return ns;
}

/* Number of attended (query, key) pairs: query at global position p sees keys
 * 0..p, so a query range [b, e) sees sum_{p=b}^{e-1} (p+1) = (e(e+1) - b(b+1))/2. */
int64_t oracle_attended_pairs(int32_t K, const int32_t *q_begin, const int32_t *q_len)
{
    int64_t a = 0;
    for (int32_t k = 0; k < K; ++k) {
        int64_t b = q_begin[k], e = (int64_t)q_begin[k] + q_len[k];
        a += (e * (e + 1) - b * (b + 1)) / 2;
    }
    return a;
}

static int32_t ceil_div(int64_t a, int64_t b) { return (int32_t)((a + b - 1) / b); }

/* Stable sort of 4-int items by DESCENDING items[.][3] (insertion of each item
 * after all items of greater-or-equal cost that precede it).  O(n^2) on
 * purpose: obviously stable, obviously a permutation. */
static void stable_sort_desc_cost(int32_t *items, int32_t n)
{
    int32_t *tmp = (int32_t *)malloc((size_t)n * 4 * sizeof(int32_t));
    int32_t *rank = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    for (int32_t a = 0; a < n; ++a) {
        int32_t ra = 0;
        for (int32_t b = 0; b < n; ++b) {
            int32_t ca = items[4 * a + 3], cb = items[4 * b + 3];
            if (cb > ca || (cb == ca && b < a)) ++ra;
        }
        rank[a] = ra;
    }
    for (int32_t a = 0; a < n; ++a) memcpy(tmp + 4 * rank[a], items + 4 * a, 4 * sizeof(int32_t));
    memcpy(items, tmp, (size_t)n * 4 * sizeof(int32_t));
    free(tmp);
    free(rank);
}

/* Forward / dQ work list.  One item per (sequence k, query block m of BM rows):
 *   {k, m, cu_q[k] + m*BM, n_kv}, n_kv = ceil((q_begin + min(q_len, (m+1)*BM)) / BN)
 * = how many BN-wide key blocks the block's last row can see (its quadratic
 * cost).  Emitted for k ascending, m ascending, then stably sorted by
 * descending n_kv -- the paper's "give the heaviest piece to the least loaded
 * worker" rule (Alg. 1, argmin over loads; Alg. 2, sorted bin-packing by
 * FLOPs) at the granularity of compute units.
 * `items` must hold 4*sum_k ceil(q_len/BM) ints.  Returns the item count. */
int32_t oracle_fwd_items(int32_t K, const int32_t *q_begin, const int32_t *q_len,
                         const int32_t *cu_q, int32_t BM, int32_t BN, int32_t *items)
{
    int32_t n = 0;
    for (int32_t k = 0; k < K; ++k) {
        int32_t nb = ceil_div(q_len[k], BM);
        for (int32_t m = 0; m < nb; ++m) {
            int64_t row0 = (int64_t)m * BM;
            int64_t rows = q_len[k] - row0 < BM ? q_len[k] - row0 : BM;
            if (items) {
                items[4 * n + 0] = k;
                items[4 * n + 1] = m;
                items[4 * n + 2] = (int32_t)(cu_q[k] + row0);
                items[4 * n + 3] = ceil_div((int64_t)q_begin[k] + row0 + rows, BN);
            }
            ++n;
        }
    }
    if (items) stable_sort_desc_cost(items, n);
    return n;
}

/* dK/dV work list.  One item per (key/value prefix, key block n of BN rows).  A
 * prefix belongs to the LAST segment k that reads it (the only one, or the late chunk
 * of a two-chunk cut); an early chunk (shares_kv[k+1] = 1) emits no items of its own.
 *   {k, n, m0, n_q}: the first local query row of segment k that can see the block is
 *   i0 = max(0, n*BN - q_begin); m0 = floor(i0 / BM) is its first query block that
 *   touches it; n_q (cost) = the number of query blocks that do: ceil(q_len/BM) - m0
 *   of segment k plus, if the prefix is shared and the block starts inside the early
 *   chunk's own prefix, the same count for segment k-1.
 * Same emission order and the same stable descending sort as above. */
int32_t oracle_dkv_items(int32_t K, const int32_t *q_begin, const int32_t *q_len,
                         const int32_t *kv_len, const int32_t *shares_kv,
                         int32_t BM, int32_t BN, int32_t *items)
{
    int32_t n = 0;
    for (int32_t k = 0; k < K; ++k) {
        if (k + 1 < K && shares_kv[k + 1]) continue;
        int32_t nb = ceil_div(kv_len[k], BN);
        for (int32_t b = 0; b < nb; ++b) {
            int32_t m0 = 0, cost = 0;
            for (int32_t s = k; s >= k - (shares_kv[k] ? 1 : 0); --s) {
                if ((int64_t)b * BN >= kv_len[s]) continue;
                int64_t i0 = (int64_t)b * BN - q_begin[s];
                if (i0 < 0) i0 = 0;
                if (s == k) m0 = (int32_t)(i0 / BM);
                cost += ceil_div(q_len[s], BM) - (int32_t)(i0 / BM);
            }
            if (items) {
                items[4 * n + 0] = k;
                items[4 * n + 1] = b;
                items[4 * n + 2] = m0;
                items[4 * n + 3] = cost;
            }
            ++n;
        }
    }
    if (items) stable_sort_desc_cost(items, n);
    return n;
}

/* ------------------------------------------------------------------ */
/* Floating part                                                       */
/* ------------------------------------------------------------------ */

/* Shapes shared by the three functions below ("sequence k" = segment k of
 * oracle_ranges).
 *   Q, dO : [Tq, Hq, d] float, packed; segment k owns rows cu_q[k]..cu_q[k]+q_len[k]-1
 *   K, V  : [Tk, Hkv, d] float, packed; segment k reads rows cu_k[k]..cu_k[k]+kv_len[k]-1,
 *           which are key positions 0..kv_len[k]-1
 * A work entry t names (seq[t], head[t], idx[t]).  Entries are independent and
 * are spread over the host cores. */

static double dotf(const float *a, const float *b, int32_t d)
{
    double s = 0.0;
    for (int32_t t = 0; t < d; ++t) s += (double)a[t] * (double)b[t];
    return s;
}

/* Forward rows.  For entry t: sequence k, query head h, local row i (global
 * position p = q_begin[k] + i), kv head c = h / (Hq/Hkv):
 *   s_j = scale * q_i . k_j for j = 0..p,  LSE = log sum_j exp(s_j),
 *   P_j = exp(s_j - LSE),  O = sum_j P_j v_j.
 * Outputs O[t, 0..d) and LSE[t] (double). */
void oracle_fwd_rows(const float *Q, const float *Kt, const float *V,
                     int32_t Hq, int32_t Hkv, int32_t d, double scale,
                     const int32_t *q_begin, const int32_t *cu_q, const int32_t *cu_k,
                     int64_t n, const int32_t *seq, const int32_t *head, const int32_t *idx,
                     double *O, double *LSE)
{
    const int32_t g = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t t = 0; t < n; ++t) {
        const int32_t k = seq[t], h = head[t], i = idx[t], c = h / g;
        const int64_t p = (int64_t)q_begin[k] + i;
        const float *q = Q + ((int64_t)(cu_q[k] + i) * Hq + h) * d;
        double *s = (double *)malloc((size_t)(p + 1) * sizeof(double));
        double mx = -INFINITY;
        for (int64_t j = 0; j <= p; ++j) {
            const float *kj = Kt + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
            s[j] = scale * dotf(q, kj, d);
            if (s[j] > mx) mx = s[j];
        }
        double z = 0.0;
        for (int64_t j = 0; j <= p; ++j) z += exp(s[j] - mx);
        const double lse = mx + log(z);
        double *o = O + t * d;
        for (int32_t e = 0; e < d; ++e) o[e] = 0.0;
        for (int64_t j = 0; j <= p; ++j) {
            const double pj = exp(s[j] - lse);
            const float *vj = V + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
            for (int32_t e = 0; e < d; ++e) o[e] += pj * (double)vj[e];
        }
        LSE[t] = lse;
        free(s);
    }
}

/* Backward with respect to the queries, row by row.  For entry t (k, h, i),
 * with P and O as in the forward:
 *   D    = sum_e dO_i[e] * O_i[e]
 *   dP_j = dO_i . v_j,   dS_j = P_j * (dP_j - D)
 *   dQ_i = scale * sum_j dS_j k_j
 * Outputs dQ[t, 0..d) and Dout[t]. */
void oracle_bwd_dq_rows(const float *Q, const float *Kt, const float *V, const float *dO,
                        int32_t Hq, int32_t Hkv, int32_t d, double scale,
                        const int32_t *q_begin, const int32_t *cu_q, const int32_t *cu_k,
                        int64_t n, const int32_t *seq, const int32_t *head, const int32_t *idx,
                        double *dQ, double *Dout)
{
    const int32_t g = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t t = 0; t < n; ++t) {
        const int32_t k = seq[t], h = head[t], i = idx[t], c = h / g;
        const int64_t p = (int64_t)q_begin[k] + i;
        const float *q = Q + ((int64_t)(cu_q[k] + i) * Hq + h) * d;
        const float *go = dO + ((int64_t)(cu_q[k] + i) * Hq + h) * d;
        double *P = (double *)malloc((size_t)(p + 1) * sizeof(double));
        double *o = (double *)calloc((size_t)d, sizeof(double));
        double mx = -INFINITY;
        for (int64_t j = 0; j <= p; ++j) {
            const float *kj = Kt + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
            P[j] = scale * dotf(q, kj, d);
            if (P[j] > mx) mx = P[j];
        }
        double z = 0.0;
        for (int64_t j = 0; j <= p; ++j) z += exp(P[j] - mx);
        const double lse = mx + log(z);
        for (int64_t j = 0; j <= p; ++j) {
            P[j] = exp(P[j] - lse);
            const float *vj = V + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
            for (int32_t e = 0; e < d; ++e) o[e] += P[j] * (double)vj[e];
        }
        double D = 0.0;
        for (int32_t e = 0; e < d; ++e) D += (double)go[e] * o[e];
        double *dq = dQ + t * d;
        for (int32_t e = 0; e < d; ++e) dq[e] = 0.0;
        for (int64_t j = 0; j <= p; ++j) {
            const float *kj = Kt + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
            const float *vj = V + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
            const double dS = P[j] * (dotf(go, vj, d) - D);
            for (int32_t e = 0; e < d; ++e) dq[e] += dS * (double)kj[e];
        }
        for (int32_t e = 0; e < d; ++e) dq[e] *= scale;
        Dout[t] = D;
        free(P);
        free(o);
    }
}

/* Backward with respect to keys and values, column by column.  For entry t
 * (sequence k, KV head c, key position j), summing over the g query heads of
 * the group and over the local query rows i whose position q_begin+i >= j:
 *   P_ij  = exp(scale * q_i . k_j - LSE[h, cu_q[k]+i])
 *   dS_ij = P_ij * (dO_i . v_j - Dfull[h, cu_q[k]+i])
 *   dV_j  = sum P_ij dO_i,   dK_j = scale * sum dS_ij q_i
 * LSEfull and Dfull are [Hq, Tq] doubles from the two functions above; only
 * the (head, row) cells the listed columns can see are read.
 * For a shard these are this rank's partial sums over its own query rows.  When two
 * segments share a key/value prefix, the gradient of a key row is the sum of the
 * columns of both (the caller adds them). */
void oracle_bwd_dkv_cols(const float *Q, const float *Kt, const float *V, const float *dO,
                         const double *LSEfull, const double *Dfull, int64_t Tq,
                         int32_t Hq, int32_t Hkv, int32_t d, double scale,
                         const int32_t *q_begin, const int32_t *q_len,
                         const int32_t *cu_q, const int32_t *cu_k,
                         int64_t n, const int32_t *seq, const int32_t *kvhead, const int32_t *col,
                         double *dK, double *dV)
{
    const int32_t g = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t t = 0; t < n; ++t) {
        const int32_t k = seq[t], c = kvhead[t], j = col[t];
        const float *kj = Kt + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
        const float *vj = V + ((int64_t)(cu_k[k] + j) * Hkv + c) * d;
        double *dk = dK + t * d, *dv = dV + t * d;
        for (int32_t e = 0; e < d; ++e) { dk[e] = 0.0; dv[e] = 0.0; }
        int64_t i0 = (int64_t)j - q_begin[k];
        if (i0 < 0) i0 = 0;
        for (int32_t h = c * g; h < (c + 1) * g; ++h) {
            for (int64_t i = i0; i < q_len[k]; ++i) {
                const int64_t row = (int64_t)cu_q[k] + i;
                const float *q = Q + (row * Hq + h) * d;
                const float *go = dO + (row * Hq + h) * d;
                const double P = exp(scale * dotf(q, kj, d) - LSEfull[(int64_t)h * Tq + row]);
                const double dS = P * (dotf(go, vj, d) - Dfull[(int64_t)h * Tq + row]);
                for (int32_t e = 0; e < d; ++e) {
                    dv[e] += P * (double)go[e];
                    dk[e] += dS * (double)q[e];
                }
            }
        }
        for (int32_t e = 0; e < d; ++e) dk[e] *= scale;
    }
}

/* Number of OpenMP threads a parallel region here will use. */
int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
