// Work queues of a persistent launch.
//
// The hardware deals the workgroups of a grid to the eight dies (XCDs) round-robin, block b
// to die b mod 8, and only balances the load inside a die.  The dies of one chip do not run
// at one speed (on the measured parts the same list of work items took one die 6 % longer
// than another), so a grid with one workgroup per work item ends with the fast dies idle for
// the last 3-5 % of the launch.  Here a launch instead starts as many workgroups as the chip
// holds at once, and each takes work items until none is left: first from its own die's
// queue (work items w = die, die + 8, die + 16, ... in list order, which keeps the heads of
// one KV group on one die and its L2, as the static mapping did), then from the queue with
// the most items left.  The work lists are sorted by descending cost, so what is stolen at
// the end are the smallest items: the paper's rule (Alg. 1: the next piece goes to argmin of
// the loads) applied across dies at run time, since their speeds are not known beforehand.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

struct WorkQueue {
    int32_t next[8];  // per die: how many of its work items have been handed out
    int32_t pad[8];
};

// Next work item for a workgroup on die `xcd`, or -1 when every queue is empty.  Called by
// one lane.  Counters are device-scope atomics (the dies' L2 caches are not coherent with
// each other for plain accesses).
__device__ __forceinline__ int claim_work(WorkQueue *q, int n_work, int xcd)
{
    int k = __hip_atomic_fetch_add(&q->next[xcd], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (8 * k + xcd < n_work) return 8 * k + xcd;
    for (;;) {
        // the queue with the most items left
        int best = -1, best_left = 0;
        for (int y = 0; y < 8; ++y) {
            const int ky = __hip_atomic_load(&q->next[y], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int left = (n_work - y + 7) / 8 - ky;  // items of queue y: ceil((n_work - y) / 8)
            if (left > best_left) { best_left = left; best = y; }
        }
        if (best < 0) return -1;
        k = __hip_atomic_fetch_add(&q->next[best], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (8 * k + best < n_work) return 8 * k + best;
        // someone else took its last item in between: look again (every failed attempt
        // means a queue has run empty, so this ends after at most eight rounds)
    }
}

// Die this wave runs on (XCC_ID register, bits 0-3).
__device__ __forceinline__ int my_xcd() { return __builtin_amdgcn_s_getreg((31 << 11) | 20) & 7; }

// Work loop of a persistent workgroup: `body(w)` for every work item it takes.  Without a
// queue (q == nullptr) the workgroup does the one item of its block index, as in a plain
// grid.  `slot` is one int of LDS.
template <typename F>
__device__ __forceinline__ void work_loop(WorkQueue *q, int n_work, int *slot, F body)
{
    const int xcd = q ? my_xcd() : 0;
    bool first = true;
    for (;;) {
        int w;
        if (q) {
            if (threadIdx.x == 0) *slot = claim_work(q, n_work, xcd);
            __syncthreads();
            w = __builtin_amdgcn_readfirstlane(*slot);
            __syncthreads();  // everyone has read the slot before the next claim overwrites it
        } else {
            w = first ? (int)blockIdx.x : -1;
            first = false;
        }
        if (w < 0 || w >= n_work) return;
        body(w);
    }
}

// Zeroes `n` work queues (a launch's queue must be zero when its kernel starts).
static __global__ void queue_reset_kernel(WorkQueue *q, int n)
{
    int32_t *w = (int32_t *)q;
    for (int i = threadIdx.x; i < n * (int)(sizeof(WorkQueue) / 4); i += blockDim.x) w[i] = 0;
}

// Workgroups of `kernel` that the whole chip holds at once.
template <typename K>
static int resident_workgroups(K kernel, int threads)
{
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess ||
        cus < 1 || per_cu < 1) {
        (void)hipGetLastError();
        return 0;  // unknown: the caller falls back to one workgroup per work item
    }
    return cus * per_cu;
}

// Workgroups of a kernel (a template argument) that the chip holds at once; queried once.
template <auto Kernel>
static int resident_of(int threads)
{
    static const int resident = resident_workgroups(Kernel, threads);
    return resident;
}

// A launch needs its queue only when there are more work items than the chip holds workgroups at
// once; otherwise one workgroup per item, all resident together, is the whole schedule.
template <auto Kernel>
static bool wants_queue(int threads, int n_work)
{
    const int resident = resident_of<Kernel>(threads);
    return resident > 0 && n_work > resident;
}

// Persistent launch when `queued` (as many workgroups as fit the chip at once, each taking work
// items from the queue in `prm` until none is left), else a plain grid of one workgroup per item
// (`prm` then carries no queue).
template <auto Kernel, typename P>
static hipError_t launch_work(int threads, int n_work, bool queued, const P &prm, hipStream_t st)
{
    const int grid = queued ? resident_of<Kernel>(threads) : n_work;
    Kernel<<<grid, threads, 0, st>>>(prm);
    return hipGetLastError();
}
