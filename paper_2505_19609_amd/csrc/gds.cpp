// Host-side GDS scheduler (paper Sec. 4.3.2, Alg. 2; cost function of App. B.2).
// Integer arithmetic throughout; the per-micro-batch DACP run is the library's own
// skrull_dacp_schedule.
#include <algorithm>
#include <new>
#include <numeric>
#include <vector>

#include "skrull_attn.h"
#include "skrull_gds.h"

namespace {

typedef unsigned __int128 u128;

bool model_ok(const skrull_flops_model_t *m)
{
    return m && m->hidden >= 1 && m->hidden <= (1 << 20) && m->hidden_kv >= 1 &&
           m->hidden_kv <= (1 << 20) && m->batch >= 1 && m->batch <= (1 << 10);
}

u128 flops(const skrull_flops_model_t *m, int32_t len)
{
    const u128 b = (u128)m->batch, h = (u128)m->hidden, hkv = (u128)m->hidden_kv, S = (u128)len;
    return 20 * b * h * h * S + 4 * b * h * hkv * S + 4 * b * h * S * S;
}

bool lengths_ok(int32_t K, const int32_t *len)
{
    if (!len || K < 1 || K > (1 << 20)) return false;
    for (int32_t k = 0; k < K; ++k)
        if (len[k] < 1) return false;
    return true;
}

// heaviest first, each to the least-loaded rank
void pack(int32_t K, const int32_t *len, int32_t ws, const skrull_flops_model_t *m, int32_t *bin)
{
    std::vector<u128> cost(K), load(ws, 0);
    for (int32_t k = 0; k < K; ++k) cost[k] = flops(m, len[k]);
    std::vector<int32_t> order(K);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return cost[a] > cost[b]; });
    for (int32_t k : order) {
        const int32_t i = (int32_t)(std::min_element(load.begin(), load.end()) - load.begin());
        bin[k] = i;
        load[i] += cost[k];
    }
}

}  // namespace

extern "C" int skrull_gds_binpack(int32_t num_seqs, const int32_t *seq_len, int32_t dp_world_size,
                                  const skrull_flops_model_t *model, int32_t *dp_bin)
{
    if (!lengths_ok(num_seqs, seq_len) || !model_ok(model) || !dp_bin) return SKRULL_EINVAL;
    if (dp_world_size < 1 || dp_world_size > 65536) return SKRULL_EINVAL;
    try {
        pack(num_seqs, seq_len, dp_world_size, model, dp_bin);
        return SKRULL_OK;
    } catch (const std::bad_alloc &) {
        return SKRULL_ENOMEM;
    }
}

extern "C" int skrull_gds_schedule(int32_t num_seqs, const int32_t *seq_len, int64_t bucket_size,
                                   int32_t cp_degree, int32_t dp_world_size, int32_t dp_rank,
                                   const skrull_flops_model_t *model, int32_t *dp_bin,
                                   int32_t *micro_batch, int32_t *ret, int32_t *num_micro_batches)
{
    if (!lengths_ok(num_seqs, seq_len) || !model_ok(model)) return SKRULL_EINVAL;
    if (!dp_bin || !micro_batch || !ret || !num_micro_batches) return SKRULL_EINVAL;
    if (dp_world_size < 1 || dp_world_size > 65536 || dp_rank < 0 || dp_rank >= dp_world_size)
        return SKRULL_EINVAL;
    if (cp_degree < 1 || cp_degree > 65536 || bucket_size < 1) return SKRULL_EINVAL;
    try {
        const int32_t K = num_seqs;
        pack(K, seq_len, dp_world_size, model, dp_bin);
        std::vector<int32_t> mine;  // this rank's subset, ascending length
        for (int32_t k = 0; k < K; ++k) {
            micro_batch[k] = -1;
            ret[k] = -2;
            if (dp_bin[k] == dp_rank) mine.push_back(k);
        }
        *num_micro_batches = 0;
        if (mine.empty()) return SKRULL_OK;
        std::stable_sort(mine.begin(), mine.end(),
                         [&](int32_t a, int32_t b) { return seq_len[a] < seq_len[b]; });
        const int64_t n = (int64_t)mine.size();
        const u128 limit = (u128)bucket_size * (u128)cp_degree;  // C*N tokens per micro-batch
        u128 total = 0;
        for (int32_t k : mine) total += (u128)seq_len[k];
        int64_t m = (int64_t)((total + limit - 1) / limit);      // fewest the token limit allows
        std::vector<int32_t> lens, decided;
        for (; m <= n; ++m) {
            bool ok = true;
            for (int64_t j = 0; j < m && ok; ++j) {
                lens.clear();
                u128 tokens = 0;
                for (int64_t p = j; p < n; p += m) {
                    lens.push_back(seq_len[mine[p]]);
                    tokens += (u128)seq_len[mine[p]];
                }
                if (tokens > limit) { ok = false; break; }
                decided.resize(lens.size());
                const int rc = skrull_dacp_schedule((int32_t)lens.size(), lens.data(), bucket_size,
                                                    cp_degree, model, decided.data());
                if (rc == SKRULL_ESCHED) { ok = false; break; }
                if (rc != SKRULL_OK) return rc;
                int64_t i = 0;
                for (int64_t p = j; p < n; p += m, ++i) {
                    micro_batch[mine[p]] = (int32_t)j;
                    ret[mine[p]] = decided[i];
                }
            }
            if (ok) {
                *num_micro_batches = (int32_t)m;
                return SKRULL_OK;
            }
        }
        return SKRULL_ESCHED;
    } catch (const std::bad_alloc &) {
        return SKRULL_ENOMEM;
    }
}

extern "C" int skrull_gds_micro_batch(int32_t num_seqs, const int32_t *seq_len,
                                      const int32_t *micro_batch, int32_t index, int32_t *members,
                                      int32_t *count)
{
    if (!seq_len || !micro_batch || !members || !count || num_seqs < 1 || index < 0)
        return SKRULL_EINVAL;
    int32_t n = 0;
    for (int32_t k = 0; k < num_seqs; ++k)
        if (micro_batch[k] == index) members[n++] = k;
    try {
        std::stable_sort(members, members + n, [&](int32_t a, int32_t b) { return seq_len[a] < seq_len[b]; });
    } catch (const std::bad_alloc &) {
        return SKRULL_ENOMEM;
    }
    *count = n;
    return SKRULL_OK;
}
