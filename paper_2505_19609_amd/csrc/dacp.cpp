// Host-side DACP scheduler (paper Sec. 4.3.2, Alg. 1; App. A.1, Alg. 3; App. B.2).
//
// All quantities that the paper divides by N are kept multiplied by N, so the
// whole run is exact integer arithmetic:
//   cap[j]  = N * (remaining bucket of rank j)      tokens * N
//   load[j] = N * (load of rank j)                  FLOPs  * N
// A whole sequence of S tokens costs N*S of cap and N*FLOPs(S) of load on one
// rank; a distributed one costs S of cap and FLOPs(S) of load on every rank.
#include <algorithm>
#include <new>
#include <numeric>
#include <vector>

#include "skrull_attn.h"
#include "skrull_dacp.h"

namespace {

typedef unsigned __int128 u128;
typedef __int128 i128;

struct Scheduler {
    int K, N;
    std::vector<int32_t> len;    // sorted ascending
    std::vector<int32_t> where;  // per sorted position: rank, -1 distributed, -2 not placed yet
    std::vector<u128> cost;      // FLOPs of each sorted sequence
    std::vector<i128> cap;       // may go negative after a roll-back charged other ranks
    std::vector<u128> load;

    int least_loaded() const { return (int)(std::min_element(load.begin(), load.end()) - load.begin()); }
    int roomiest() const { return (int)(std::max_element(cap.begin(), cap.end()) - cap.begin()); }
    int tightest() const { return (int)(std::min_element(cap.begin(), cap.end()) - cap.begin()); }

    bool fits_whole(int rank, int pos) const { return cap[rank] >= (i128)N * len[pos]; }

    void keep_whole(int pos, int rank)
    {
        where[pos] = rank;
        cap[rank] -= (i128)N * len[pos];
        load[rank] += (u128)N * cost[pos];
    }
    void spread(int pos)
    {
        where[pos] = -1;
        for (int j = 0; j < N; ++j) {
            cap[j] -= len[pos];
            load[j] += cost[pos];
        }
    }
    // first (shortest) sequence held whole by `rank` becomes distributed
    bool relieve(int rank)
    {
        for (int pos = 0; pos < K; ++pos) {
            if (where[pos] != rank) continue;
            cap[rank] += (i128)N * len[pos];
            load[rank] -= (u128)N * cost[pos];
            spread(pos);
            return true;
        }
        return false;
    }

    bool run()
    {
        int pos = 0;
        while (pos < K) {
            int r = least_loaded();
            if (!fits_whole(r, pos)) r = roomiest();
            if (fits_whole(r, pos)) {
                keep_whole(pos++, r);
                continue;
            }
            const int t = tightest();
            if (cap[t] >= (i128)len[pos]) {  // every rank can take its S/N slice
                spread(pos++);
                continue;
            }
            if (!relieve(t)) return false;   // then try this sequence again
        }
        return *std::min_element(cap.begin(), cap.end()) >= 0;  // Eq. 8 on every rank
    }
};

bool model_ok(const skrull_flops_model_t *m)
{
    return m && m->hidden >= 1 && m->hidden <= (1 << 20) && m->hidden_kv >= 1 &&
           m->hidden_kv <= (1 << 20) && m->batch >= 1 && m->batch <= (1 << 10);
}

}  // namespace

extern "C" int skrull_dacp_schedule(int32_t num_seqs, const int32_t *seq_len, int64_t bucket_size,
                                    int32_t cp_degree, const skrull_flops_model_t *model, int32_t *ret)
{
    if (!seq_len || !ret || !model_ok(model)) return SKRULL_EINVAL;
    if (num_seqs < 1 || num_seqs > (1 << 20) || cp_degree < 1 || cp_degree > 65536 || bucket_size < 1)
        return SKRULL_EINVAL;
    for (int32_t k = 0; k < num_seqs; ++k)
        if (seq_len[k] < 1) return SKRULL_EINVAL;
    try {
        const int K = num_seqs, N = cp_degree;
        std::vector<int32_t> order(K);
        std::iota(order.begin(), order.end(), 0);
        std::stable_sort(order.begin(), order.end(),
                         [&](int32_t a, int32_t b) { return seq_len[a] < seq_len[b]; });
        Scheduler s;
        s.K = K;
        s.N = N;
        s.len.resize(K);
        s.cost.resize(K);
        s.where.assign(K, -2);
        const u128 b = (u128)model->batch, h = (u128)model->hidden, hkv = (u128)model->hidden_kv;
        for (int p = 0; p < K; ++p) {
            const u128 S = (u128)seq_len[order[p]];
            s.len[p] = seq_len[order[p]];
            s.cost[p] = 20 * b * h * h * S + 4 * b * h * hkv * S + 4 * b * h * S * S;  // App. B.2
        }
        s.cap.assign(N, (i128)bucket_size * N);
        s.load.assign(N, 0);
        if (!s.run()) return SKRULL_ESCHED;
        for (int p = 0; p < K; ++p) ret[order[p]] = s.where[p];
        return SKRULL_OK;
    } catch (const std::bad_alloc &) {
        return SKRULL_ENOMEM;
    }
}

extern "C" int skrull_dacp_rank_batch(int32_t num_seqs, const int32_t *seq_len, const int32_t *ret,
                                      int32_t cp_degree, int32_t rank, int32_t *out_seq_len,
                                      int32_t *out_shard_degree, int32_t *out_shard_index,
                                      int32_t *out_source, int32_t *count)
{
    if (!seq_len || !ret || !out_seq_len || !out_shard_degree || !out_shard_index || !out_source || !count)
        return SKRULL_EINVAL;
    if (num_seqs < 1 || cp_degree < 1 || rank < 0 || rank >= cp_degree) return SKRULL_EINVAL;
    for (int32_t k = 0; k < num_seqs; ++k)
        if (ret[k] < -1 || ret[k] >= cp_degree) return SKRULL_EINVAL;
    int32_t n = 0;
    for (int32_t k = 0; k < num_seqs; ++k) {
        if (ret[k] != -1 && ret[k] != rank) continue;
        out_seq_len[n] = seq_len[k];
        out_shard_degree[n] = ret[k] == -1 ? cp_degree : 1;
        out_shard_index[n] = ret[k] == -1 ? rank : 0;
        out_source[n] = k;
        ++n;
    }
    *count = n;
    return SKRULL_OK;
}
