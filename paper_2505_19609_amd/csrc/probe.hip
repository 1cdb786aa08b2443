// Measurement aid, not part of the method: the rate this GPU sustains on nothing but
// v_mfma_f32_32x32x16_bf16 (two waves per SIMD, four independent accumulators each,
// operands in registers), for bench.py to print beside the nominal 2.5 PFLOP/s.  The
// shader clock under sustained matrix work sits below the boost clock the nominal
// figure assumes, so this is the ceiling a kernel can actually be held against.
#include "common.h"
#include "mfma.h"

namespace {

__global__ __launch_bounds__(512, 2) void mfma_only_kernel(float *out, int iters)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(0.001f * (lane + i));
        b[i] = (__bf16)(0.002f * (lane - i));
    }
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int v = 0; v < 16; ++v) { c0[v] = 0.0f; c1[v] = 0.0f; c2[v] = 0.0f; c3[v] = 0.0f; }
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
        c0 = mfma32(a, b, c0);
        c1 = mfma32(a, b, c1);
        c2 = mfma32(a, b, c2);
        c3 = mfma32(a, b, c3);
    }
    float s = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace

hipError_t run_mfma_probe(int blocks, int iters, float *scratch, hipStream_t st, float *ms)
{
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    // two full-length launches first: the clock takes tens of milliseconds to settle
    mfma_only_kernel<<<blocks, 512, 0, st>>>(scratch, iters);
    mfma_only_kernel<<<blocks, 512, 0, st>>>(scratch, iters);
    (void)hipEventRecord(e0, st);
    mfma_only_kernel<<<blocks, 512, 0, st>>>(scratch, iters);
    (void)hipEventRecord(e1, st);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e;
}
