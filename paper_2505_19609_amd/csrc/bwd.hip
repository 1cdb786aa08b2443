// Backward kernels: D = rowsum(dO * O), dQ, and dK/dV with the GQA head
// reduction, for the packed varlen causal attention of fwd.hip.
//
//   P_ij  = exp(scale * q_i.k_j - LSE_i)          dP_ij = dO_i . v_j
//   dS_ij = P_ij (dP_ij - D_i)
//   dQ_i  = scale * sum_j dS_ij k_j
//   dK_j  = scale * sum_{h in group} sum_i dS_ij q_i
//   dV_j  =         sum_{h in group} sum_i P_ij dO_i
//
// dQ kernel: work items and orientation of the forward kernel (query index on
// the MFMA column, so LSE_i and D_i are per-lane scalars):
//     S^T = K Q^T, dP^T = V dO^T           A = K / V tile rows (LDS), B = Q / dO (registers)
//     dQ^T[t,i] += sum_j K^T[t,j] dS^T[j,i] A = transposed K tile (LDS), B = dS^T (registers)
// dK/dV kernel: one workgroup owns BN key rows of one KV head and walks over
// the g query heads of the group and the query tiles that can see them; the
// key index is on the MFMA column, so the two accumulators of a lane belong to
// one key row and the group sum never leaves registers:
//     S = Q K^T, dP = dO V^T               A = Q / dO tile rows (LDS), B = K / V (registers)
//     dV^T[t,j] += sum_i dO^T[t,i] P[i,j]   A = transposed dO tile (LDS), B = P (registers)
//     dK^T[t,j] += sum_i Q^T[t,i] dS[i,j]   A = transposed Q tile (LDS),  B = dS (registers)
// The paper's FLOPs model counts this quadratic work per sequence (App. B.2);
// the work-list order balances it over compute units (plan.hip).
#include <type_traits>

#include "common.h"
#include "mfma.h"
#include "tiles.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------
// D[h, row] = sum_t dO[row,h,t] * O[row,h,t]
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const uint16_t *__restrict__ o,
                                                    const uint16_t *__restrict__ d_o,
                                                    const float *__restrict__ lse,
                                                    float *__restrict__ delta,
                                                    float *__restrict__ lse2, int64_t n_pairs,
                                                    int32_t Hq, int32_t total_q)
{
    constexpr int CH = D / 8;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t pair = gid / CH;  // (row, head) flattened row-major
    float acc = 0.0f;
    if (pair < n_pairs) {
        const uint4 a = *(const uint4 *)(o + gid * 8);
        const uint4 b = *(const uint4 *)(d_o + gid * 8);
        const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            acc += __builtin_bit_cast(float, aw[w] << 16) * __builtin_bit_cast(float, bw[w] << 16);
            acc += __builtin_bit_cast(float, aw[w] & 0xffff0000u) *
                   __builtin_bit_cast(float, bw[w] & 0xffff0000u);
        }
    }
#pragma unroll
    for (int off = CH / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (pair < n_pairs && (gid % CH) == 0) {
        const int64_t row = pair / Hq;
        const int32_t hh = (int32_t)(pair % Hq);
        delta[(int64_t)hh * total_q + row] = acc;
        // LSE in the exp2 domain, so the main kernels need no extra multiply
        lse2[(int64_t)hh * total_q + row] = lse[(int64_t)hh * total_q + row] * kLog2e;
    }
}

struct BwdParams {
    const uint16_t *q, *k, *v, *d_o;
    const float *lse, *delta, *lse2;
    uint16_t *dq, *dk, *dv;
    const int4 *fwd_items, *dkv_items;
    const int32_t *cu_q, *cu_k, *q_begin, *q_len, *kv_len;
    int32_t Hq, Hkv, total_q, BM, BN;
    float scale, scale_log2;
};

// ---------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------
constexpr int NW = 4;          // wavefronts per workgroup
constexpr int SUB = 32 * NW;   // query (dQ) or key (dK/dV) rows per pass

template <int D>
__global__ __launch_bounds__(64 * NW, 2) void dq_kernel(const BwdParams prm)
{
    constexpr int NT = 64 * NW, KS = D / 16, TT = D / 32, KT = TILE_ROWS;
    constexpr int TILE_BYTES = TileGeom<D>::BYTES;
    // [buffer][K rows | V rows]; one array so that the V operand address is the
    // K operand address plus a constant
    __shared__ __align__(16) unsigned char lds_kv[2][2][TILE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int n = lane & 31, h = lane >> 5;
    const int item_id = blockIdx.x / prm.Hq, hl = blockIdx.x % prm.Hq;
    const int g = prm.Hq / prm.Hkv;
    const int c = hl % prm.Hkv;
    const int head = c * g + hl / prm.Hkv;

    FragAddr<D> fa;
    fa.init(lane);
    TileLoader<D, NT> ld;
    ld.init(tid, (uint32_t)prm.Hkv * D * 2);

    const int4 it = prm.fwd_items[item_id];
    const int seq = it.x;
    const int qb = prm.q_begin[seq], ql = prm.q_len[seq], kvl = prm.kv_len[seq];
    const int kbase = prm.cu_k[seq];
    const int item_rows = min(prm.BM, ql - it.y * prm.BM);

    for (int sub = 0; sub * SUB < item_rows; ++sub) {
    const int row0 = it.y * prm.BM + sub * SUB;
    const int qrow0 = it.z + sub * SUB;
    const int rows = min(SUB, ql - row0);
    const int p0 = qb + row0;
    const int n_tiles = (p0 + rows + KT - 1) / KT;

    const int wrow0 = 32 * wave;
    const bool wave_active = wrow0 < rows;
    const int my_i = wrow0 + n;
    const int my_pos = p0 + my_i;
    const int w_pmin = p0 + wrow0;
    const int w_pmax = p0 + min(wrow0 + 31, rows - 1);
    const int my_row = qrow0 + min(my_i, rows - 1);  // packed row, clamped for loads

    bf16x8 qf[KS], dof[KS];
    {
        int hd = head;
        asm volatile("" : "+s"(hd));  // keep this address arithmetic inside the pass
        const size_t off = ((size_t)my_row * prm.Hq + hd) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = as_bf16x8(*(const uint4 *)(prm.q + off + 16 * ks));
            dof[ks] = as_bf16x8(*(const uint4 *)(prm.d_o + off + 16 * ks));
        }
    }
    const float lse2 = prm.lse2[(size_t)head * prm.total_q + my_row];
    const float dlt = prm.delta[(size_t)head * prm.total_q + my_row];

    const __amdgpu_buffer_rsrc_t rk = ld.rsrc(prm.k + ((size_t)kbase * prm.Hkv + c) * D, kvl);
    const __amdgpu_buffer_rsrc_t rv = ld.rsrc(prm.v + ((size_t)kbase * prm.Hkv + c) * D, kvl);

    f32x16 acc[TT];
    zero_acc(acc);
    const float cs = prm.scale_log2;

    __syncthreads();  // the previous pass is done with both buffers
    ld.load(rk, lds_kv[0][0], 0, tid);
    ld.load(rv, lds_kv[0][1], 0, tid);
    wait_vmem();
    __syncthreads();
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int kv0 = tile * KT;
        const unsigned char *tk = lds_kv[tile & 1][0];
        if (tile + 1 < n_tiles) {  // lands in the other buffer during the math below
            ld.load(rk, lds_kv[(tile + 1) & 1][0], kv0 + KT, tid);
            ld.load(rv, lds_kv[(tile + 1) & 1][1], kv0 + KT, tid);
        }
        if (wave_active && kv0 <= w_pmax) {
            const bool diag = kv0 + KT - 1 > w_pmin;  // some key of the tile is past some query
            // 32 keys at a time: S^T and dP^T stay in 32 registers.  The instruction
            // order inside each half is pinned with scheduling groups so that LDS
            // operand reads run a few MFMAs ahead of their use.
#pragma unroll 1
            for (int jt = 0; jt < 2; ++jt) {
                const unsigned char *th = tk + jt * (32 * TileGeom<D>::ROWB);  // this half's 32 keys
                f32x16 s, dp;
#pragma unroll
                for (int v = 0; v < 16; ++v) { s[v] = 0.0f; dp[v] = 0.0f; }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s = mfma32(fa.rows(th, 0, ks), qf[ks], s);
                    dp = mfma32(fa.rows(th + TILE_BYTES, 0, ks), dof[ks], dp);
                }
                if (diag) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float p = fast_exp2(__builtin_fmaf(s[v], cs, -lse2));
                        p = (kv0 + 32 * jt + acc_row(v, h) > my_pos) ? 0.0f : p;
                        s[v] = p * (dp[v] - dlt);  // dS^T
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        s[v] = fast_exp2(__builtin_fmaf(s[v], cs, -lse2)) * (dp[v] - dlt);
                }
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const bf16x8 ds = acc_to_b(s, kb);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
                        acc[tt] = mfma32(fa.cols(th, tt, kb), ds, acc[tt]);
                }
            }
        }
        wait_vmem();      // my share of the next tile has landed
        __syncthreads();  // ... and everyone's; everyone is done reading this tile
    }
    if (wave_active && my_i < rows) {
        // derived after the loop from opaque copies, so that no part of the
        // output address is kept in registers during the loop
        int row = qrow0 + my_i, hh = h;
        asm volatile("" : "+v"(row), "+v"(hh));
        store_rows_bf16<TT>(prm.dq + ((size_t)row * prm.Hq + head) * D, acc, prm.scale, hh);
    }
    }  // pass
}

// ---------------------------------------------------------------------------
// dK / dV, paired waves.
//
// One wave owning 32 key rows would need K, V, dK and dV of those rows in
// registers (192 of them at d=128), which pins it to one wave per SIMD with
// nothing to hide LDS latency or softmax arithmetic behind.  Here two waves that
// share a SIMD share the 32 key rows instead:
//   role 0 ("S wave"):  S = Q K^T, P = exp2(S*c - LSE'), dV^T += dO^T P;  holds K, dV
//   role 1 ("dP wave"): dP = dO V^T, dS = P (dP - D), dK^T += Q^T dS;     holds V, dK
// P goes from the first to the second through LDS in MFMA operand format (bf16,
// 2 KB per 32x32 tile).  The dP wave runs one step behind, so that it always has
// matrix work of its own (dP of step k) while the S wave does the softmax of
// step k, and one workgroup barrier per step is all the synchronisation needed.
// A step is 32 query rows; query tiles (64 rows) sit in a ring of three buffers
// filled by asynchronous global->LDS loads two tiles ahead.
// ---------------------------------------------------------------------------
constexpr int NWP = 8;  // 4 S waves + 4 dP waves

template <int D>
__global__ __launch_bounds__(64 * NWP, 2) void dkv_pair_kernel(const BwdParams prm)
{
    constexpr int NT = 64 * NWP, KS = D / 16, TT = D / 32, QT = TILE_ROWS;
    constexpr int TILE_BYTES = TileGeom<D>::BYTES;
    __shared__ __align__(16) unsigned char lds_t[3][2][TILE_BYTES];  // [ring][Q | dO] rows
    __shared__ __align__(16) float lds_ld[3][2][QT];                 // [ring][LSE*log2e | D]
    __shared__ __align__(16) unsigned char lds_p[4][2][2][1024];     // [pair][parity][half][lane*16]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wave >> 2, pw = wave & 3;  // waves w and w+4 share a SIMD and 32 key rows
    const int n = lane & 31, h = lane >> 5;
    const int item_id = blockIdx.x / prm.Hkv, c = blockIdx.x % prm.Hkv;
    const int g = prm.Hq / prm.Hkv;
    FragAddr<D> fa;
    fa.init(lane);
    TileLoader<D, NT> ld;
    ld.init(tid, (uint32_t)prm.Hq * D * 2);

    const int4 it = prm.dkv_items[item_id];
    const int seq = it.x;
    const int qb = prm.q_begin[seq], ql = prm.q_len[seq], kvl = prm.kv_len[seq];
    const int kbase = prm.cu_k[seq], qbase = prm.cu_q[seq];
    const int item_rows = min(prm.BN, kvl - it.y * prm.BN);
    const float cs = prm.scale_log2;

    for (int sub = 0; sub * SUB < item_rows; ++sub) {
    const int kv0 = it.y * prm.BN + sub * SUB;  // first key position of the pass
    const int krows = min(SUB, kvl - kv0);
    const int wj0 = kv0 + 32 * pw;              // this pair's first key position
    const bool wave_active = 32 * pw < krows;
    const int my_j = wj0 + n;                   // this lane's key position

    // B operand held for the whole pass: this lane's key row of K (role 0) or V (role 1).
    bf16x8 bf[KS];
    {
        const uint16_t *src = role == 0 ? prm.k : prm.v;
        int hh = h;
        asm volatile("" : "+v"(hh));  // keep this address arithmetic inside the pass
        const size_t off = ((size_t)(kbase + min(my_j, kvl - 1)) * prm.Hkv + c) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bf[ks] = as_bf16x8(*(const uint4 *)(src + off + 16 * ks));
    }

    const int i_first = (max(0, kv0 - qb) / QT) * QT;  // first query tile that can see key kv0
    const int n_qt = (ql - i_first + QT - 1) / QT;
    const int n_iter = n_qt * g;     // (head, query tile) pairs
    const int n_steps = 2 * n_iter;  // 32-row steps

    f32x16 acc[TT];  // dV^T (role 0) or dK^T (role 1) of this lane's key
    zero_acc(acc);

    auto fetch = [&](int T) __attribute__((always_inline)) {
        const int head = c * g + T / n_qt;
        const int i0 = i_first + (T % n_qt) * QT;
        const int buf = T % 3;
        const size_t hoff = ((size_t)qbase * prm.Hq + head) * D;
        // query rows past the end of the sequence read as zero (and are masked)
        ld.load(ld.rsrc(prm.q + hoff, ql), lds_t[buf][0], i0, tid);
        ld.load(ld.rsrc(prm.d_o + hoff, ql), lds_t[buf][1], i0, tid);
        if (wave < 2) {
            typedef void __attribute__((address_space(3))) * lds_void_t;
            const float *src = (wave == 0 ? prm.lse2 : prm.delta) + (size_t)head * prm.total_q +
                               qbase + min(i0 + lane, ql - 1);
            __builtin_amdgcn_global_load_lds((const void *)src, (lds_void_t)lds_ld[buf][wave], 4, 0, 0);
        }
    };

    __syncthreads();  // the previous pass is done with every buffer
    fetch(0);
    if (n_iter > 1) fetch(1);
    wait_vmem();
    __syncthreads();

    f32x16 dp_prev;  // role 1: dP of the previous step
#pragma unroll
    for (int v = 0; v < 16; ++v) dp_prev[v] = 0.0f;
    bool prev_act = false;
    int prev_buf = 0, prev_half = 0;

    for (int k = 0; k <= n_steps; ++k) {  // the extra step drains the dP waves
        const int T = k >> 1, half = k & 1, buf = T % 3;
        if (half == 1 && T + 2 < n_iter) fetch(T + 2);  // into the buffer tile T-1 has left
        const int i0 = i_first + (T % n_qt) * QT + 32 * half;  // first query row of the step
        // skip steps whose last query still precedes this pair's first key
        const bool act = k < n_steps && wave_active && qb + i0 + 31 >= wj0;
        const unsigned char *tq = lds_t[buf][0], *tdo = lds_t[buf][1];
        unsigned char *px = lds_p[pw][k & 1][0];

        if (role == 0) {
            if (act) {
                f32x16 s;
#pragma unroll
                for (int v = 0; v < 16; ++v) s[v] = 0.0f;
                bf16x8 fr[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) fr[ks] = fa.rows(tq, half, ks);
                __builtin_amdgcn_sched_barrier(0);  // all operand reads in flight before the MFMAs
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) s = mfma32(fr[ks], bf[ks], s);
                bf16x8 ft[2][TT];  // transposed dO fragments, fetched behind the softmax
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) ft[kb][tt] = fa.cols(tdo, tt, 2 * half + kb);
                __builtin_amdgcn_sched_barrier(0);
                const float *t_lse = lds_ld[buf][0] + 32 * half;
                // masked pairs: key past the query (causal) or query row past the end
                const bool need_mask = (qb + i0 < wj0 + 31) || (i0 + 32 > ql);
#pragma unroll
                for (int vb = 0; vb < 4; ++vb) {
                    const float4 l4 = *(const float4 *)(t_lse + 8 * vb + 4 * h);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        s[4 * vb + e] = fast_exp2(__builtin_fmaf(s[4 * vb + e], cs, -lv[e]));
                }
                if (need_mask) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int i = i0 + acc_row(v, h);
                        s[v] = (my_j > qb + i || i >= ql) ? 0.0f : s[v];
                    }
                }
                const bf16x8 pb0 = acc_to_b(s, 0), pb1 = acc_to_b(s, 1);
                *(bf16x8 *)(px + lane * 16) = pb0;
                *(bf16x8 *)(px + 1024 + lane * 16) = pb1;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(ft[0][tt], pb0, acc[tt]);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(ft[1][tt], pb1, acc[tt]);
            }
        } else {
            if (prev_act) {
                // dS and dK of the previous step: P as the S wave of this pair left it
                const unsigned char *tqp = lds_t[prev_buf][0];
                bf16x8 ft[2][TT];  // transposed Q fragments of the previous step
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) ft[kb][tt] = fa.cols(tqp, tt, 2 * prev_half + kb);
                const unsigned char *pp = lds_p[pw][(k - 1) & 1][0];
                const uint4 p0 = *(const uint4 *)(pp + lane * 16);
                const uint4 p1 = *(const uint4 *)(pp + 1024 + lane * 16);
                const uint32_t pw32[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                const float *t_dlt = lds_ld[prev_buf][1] + 32 * prev_half;
#pragma unroll
                for (int vb = 0; vb < 4; ++vb) {
                    const float4 d4 = *(const float4 *)(t_dlt + 8 * vb + 4 * h);
                    const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * vb + e;
                        const uint32_t w = pw32[v >> 1];
                        const float p = __builtin_bit_cast(float, (v & 1) ? (w & 0xffff0000u) : (w << 16));
                        dp_prev[v] = p * (dp_prev[v] - dd[e]);  // dS
                    }
                }
                const bf16x8 db0 = acc_to_b(dp_prev, 0), db1 = acc_to_b(dp_prev, 1);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(ft[0][tt], db0, acc[tt]);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(ft[1][tt], db1, acc[tt]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int v = 0; v < 16; ++v) dp_prev[v] = 0.0f;
            if (act) {  // dP of this step, consumed in the next one
                bf16x8 fr[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) fr[ks] = fa.rows(tdo, half, ks);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) dp_prev = mfma32(fr[ks], bf[ks], dp_prev);
            }
            prev_act = act;
            prev_buf = buf;
            prev_half = half;
        }
        if (half == 0) wait_vmem();  // the tile fetched one step ago has had a full step to land
        __syncthreads();
    }
    if (wave_active && my_j < kvl) {
        // the output address is derived here, after the loop, from an opaque copy
        // of the row index so that nothing of it occupies registers during the loop
        int row = kbase + my_j, hh = h;
        asm volatile("" : "+v"(row), "+v"(hh));
        const size_t off = ((size_t)row * prm.Hkv + c) * D;
        if (role == 0) store_rows_bf16<TT>(prm.dv + off, acc, 1.0f, hh);
        else store_rows_bf16<TT>(prm.dk + off, acc, prm.scale, hh);
    }
    }  // pass
}

template <int D>
hipError_t launch_d(const skrull_attn_plan_t *p, const BwdParams &prm, const void *o, float *delta,
                    hipStream_t st, hipEvent_t *ev)
{
    if (ev) (void)hipEventRecord(ev[0], st);
    const int64_t n_pairs = (int64_t)p->total_q * p->Hq;
    const int64_t threads = n_pairs * (D / 8);
    delta_kernel<D><<<(unsigned)((threads + 255) / 256), 256, 0, st>>>(
        (const uint16_t *)o, prm.d_o, prm.lse, delta, (float *)prm.lse2, n_pairs, p->Hq, p->total_q);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[1], st);
    const int gq = p->n_fwd * p->Hq, gk = p->n_dkv * p->Hkv;
    dkv_pair_kernel<D><<<gk, 64 * NWP, 0, st>>>(prm);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[2], st);
    dq_kernel<D><<<gq, 64 * NW, 0, st>>>(prm);
    if (ev) (void)hipEventRecord(ev[3], st);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_bwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                      void *dv, float *delta, hipStream_t st, hipEvent_t *ev)
{
    BwdParams prm;
    prm.q = (const uint16_t *)q; prm.k = (const uint16_t *)k; prm.v = (const uint16_t *)v;
    prm.d_o = (const uint16_t *)d_o; prm.lse = lse; prm.delta = delta;
    prm.lse2 = delta + (size_t)p->Hq * p->total_q;
    prm.dq = (uint16_t *)dq; prm.dk = (uint16_t *)dk; prm.dv = (uint16_t *)dv;
    prm.fwd_items = (const int4 *)p->fwd_items; prm.dkv_items = (const int4 *)p->dkv_items;
    prm.cu_q = p->cu_q; prm.cu_k = p->cu_k; prm.q_begin = p->q_begin; prm.q_len = p->q_len;
    prm.kv_len = p->kv_len;
    prm.Hq = p->Hq; prm.Hkv = p->Hkv; prm.total_q = p->total_q; prm.BM = p->BM; prm.BN = p->BN;
    prm.scale = p->scale; prm.scale_log2 = p->scale * kLog2e;
    if (p->d == 128) return launch_d<128>(p, prm, o, delta, st, ev);
    if (p->d == 64) return launch_d<64>(p, prm, o, delta, st, ev);
    return hipErrorInvalidValue;
}
