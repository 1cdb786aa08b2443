// Internal declarations shared by the HIP translation units of libskrull_attn.
// Nothing here is part of the public ABI (that is include/skrull_attn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "skrull_attn.h"

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
    int32_t pad;
};

// plan.hip
hipError_t launch_plan_ranges(const int32_t *S, const int32_t *N, const int32_t *r,
                              const int32_t *cut, int32_t K, int32_t BM, int32_t BN,
                              int32_t max_q_rows, int32_t max_k_rows, int32_t *q_begin,
                              int32_t *q_len, int32_t *kv_len, int32_t *cu_q, int32_t *cu_k,
                              int32_t *shares_kv, int32_t *fwd_off, int32_t *dkv_off,
                              int32_t cap_fwd, int32_t cap_dkv, PlanTotals *totals, hipStream_t st);
hipError_t launch_plan_items(const skrull_attn_plan_t *p, const int32_t *fwd_off,
                             const int32_t *dkv_off, int32_t cap_fwd, int32_t cap_dkv,
                             int32_t *scratch_fwd, int32_t *scratch_dkv, PlanTotals *totals,
                             hipStream_t st);

// fwd.hip / bwd.hip
hipError_t launch_fwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      void *o, float *lse, hipStream_t st);
hipError_t launch_bwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                      void *dv, float *delta, hipStream_t st, hipEvent_t *ev);

// probe.hip
hipError_t run_mfma_probe(int blocks, int iters, float *scratch, hipStream_t st, float *ms);
