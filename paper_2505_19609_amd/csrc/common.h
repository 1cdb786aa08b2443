// Internal declarations shared by the HIP translation units of libskrull_attn.
// Nothing here is part of the public ABI (that is include/skrull_attn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skrull_attn.h"

struct WorkQueue;
// forward calls of one plan that may be in flight at once (each takes one queue slot in turn)
#define SKRULL_FWD_QUEUE_SLOTS 64

// Device-resident descriptor + work lists of one micro-batch.
struct skrull_attn_plan {
    int32_t K, NS, Hq, Hkv, d, BM, BN;  // K sequences, NS >= K query segments
    float scale;
    int32_t total_q, total_k, n_fwd, n_dkv;
    int64_t pairs;
    int32_t head_split;  // workgroups that share the query heads of one KV group in dK/dV
    int32_t wg_query_rows;  // query rows per forward / dQ workgroup: 128 (4 wavefronts) or 256 (8)
    int device;
    // one allocation (descriptor arrays, then the two item lists); the pointers below index into it
    int32_t *pool;
    int32_t *cu_q, *cu_k, *q_begin, *q_len, *kv_len, *shares_kv;  // per segment: [NS+1] x2, [NS] x4
    int32_t *fwd_items, *dkv_items;                   // [n][4], sorted
    WorkQueue *fwd_queues;  // [SKRULL_FWD_QUEUE_SLOTS] at the start of the pool: work queues of forward launches
    uint32_t fwd_calls;     // forward calls made so far (atomic): call i uses slot i mod SKRULL_FWD_QUEUE_SLOTS
};

// Totals written by the ranges kernel and read back by the host.
struct PlanTotals {
    int64_t total_q, total_k, n_fwd, n_dkv, pairs;
    int32_t bad_entry;   // index+1 of the first invalid sequence, 0 if none
    int32_t n_seg;       // number of query segments
    // cost (query blocks) of the dK/dV items, accumulated by the emit kernel
    unsigned long long dkv_cost_sum;
    int32_t dkv_cost_max;
    int32_t cap_fwd, cap_dkv;  // room in the item arrays (the host's upper bounds)
    int32_t block_n;           // key rows per dK/dV item in effect (the ranges kernel's choice where open)
};

// Opt-in per-workgroup trace (measurement aid): one record per work item of a launch.
struct WgTrace {
    uint64_t t0, t1;      // s_memrealtime (100 MHz, one counter for the whole chip) at start and end
    uint32_t hw_id;       // HW_ID register: bits 8-11 CU, 12 shader array, 13-15 shader engine
    uint32_t xcc_id;      // XCC_ID register: the die (XCD)
    uint32_t block;       // index of the work item (the block index in a plain grid)
    uint32_t one;         // 1 = record written
};
#ifdef __HIPCC__
__device__ __forceinline__ uint64_t trace_begin(const WgTrace *t)
{
    return t ? __builtin_amdgcn_s_memrealtime() : 0;
}
// every wave of the workgroup calls this at the very end of the kernel (wave-uniform branch)
__device__ __forceinline__ void trace_end(WgTrace *t, uint64_t t0, int work)
{
    if (!t) return;
    __syncthreads();
    if (threadIdx.x == 0) {
        WgTrace r;
        r.t0 = t0;
        r.t1 = __builtin_amdgcn_s_memrealtime();
        r.hw_id = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_REG_HW_ID, all 32 bits
        r.xcc_id = __builtin_amdgcn_s_getreg((31 << 11) | 20);  // HW_REG_XCC_ID
        r.block = work;
        r.one = 1;
        t[work] = r;
    }
}
#endif

// plan.hip
hipError_t launch_plan_ranges(const int32_t *S, const int32_t *N, const int32_t *r,
                              const int32_t *cut, int32_t K, int32_t BM, int32_t BN,
                              int32_t max_q_rows, int32_t max_k_rows, int32_t *q_begin,
                              int32_t *q_len, int32_t *kv_len, int32_t *cu_q, int32_t *cu_k,
                              int32_t *shares_kv, int32_t *fwd_off, int32_t *dkv_off,
                              int32_t cap_fwd, int32_t cap_dkv, int32_t bn_alt, int32_t kv_heads,
                              int32_t compute_units, PlanTotals *totals, hipStream_t st);
// `cost_bound`: no work item costs more (host's bound from the longest sequence); lists whose
// upper bound of items exceeds the rank sort's limit are radix sorted and need
// plan_radix_ints(...) ints of scratch at `radix_hist`
hipError_t launch_plan_items(const skrull_attn_plan_t *p, const int32_t *fwd_off,
                             const int32_t *dkv_off, int32_t cap_fwd, int32_t cap_dkv,
                             int32_t *scratch_fwd, int32_t *scratch_dkv, int32_t *radix_hist,
                             int32_t cost_bound, PlanTotals *totals, hipStream_t st);
int64_t plan_radix_ints(int32_t cap_fwd, int32_t cap_dkv, int32_t cost_bound);

// fwd.hip / bwd.hip
// `trace` (may be null): room for one WgTrace per workgroup of every kernel launched, in
// launch order (launch_bwd: dQ's records, then dK/dV's); grid sizes from the functions below
hipError_t launch_fwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      void *o, float *lse, hipStream_t st, WgTrace *trace);
hipError_t launch_bwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                      void *dv, float *delta, hipStream_t st, hipEvent_t *ev, WgTrace *trace);
int grid_fwd(const skrull_attn_plan_t *p);
int grid_dq(const skrull_attn_plan_t *p);
int grid_dkv(const skrull_attn_plan_t *p);

// probe.hip
hipError_t run_mfma_probe(int blocks, int iters, float *scratch, hipStream_t st, float *ms);
