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
    // Two [K rows | V rows] buffers, each its own LDS object, and a tile loop
    // unrolled by two: every access names its buffer statically, so the compiler
    // knows that operand reads never touch the buffer an asynchronous load is
    // filling.  K and V share an object so that the V operand address is the K
    // operand address plus a constant.
    __shared__ __align__(16) unsigned char lds_kv0[2][TILE_BYTES], lds_kv1[2][TILE_BYTES];

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

    auto do_tile = [&](int tile, const unsigned char *tk, unsigned char *nxt) __attribute__((always_inline)) {
        const int kv0 = tile * KT;
        if (tile + 1 < n_tiles) {  // lands in the other buffer during the math below
            ld.load(rk, nxt, kv0 + KT, tid);
            ld.load(rv, nxt + TILE_BYTES, kv0 + KT, tid);
        }
        if (wave_active && kv0 <= w_pmax) {
            const bool diag = kv0 + KT - 1 > w_pmin;  // some key of the tile is past some query
            // 32 keys at a time: S^T and dP^T stay in 32 registers.
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
    };

    __syncthreads();  // the previous pass is done with both buffers
    ld.load(rk, lds_kv0[0], 0, tid);
    ld.load(rv, lds_kv0[1], 0, tid);
    wait_vmem();
    __syncthreads();
    for (int tile = 0; tile < n_tiles; tile += 2) {
        do_tile(tile, lds_kv0[0], lds_kv1[0]);
        if (tile + 1 < n_tiles) do_tile(tile + 1, lds_kv1[0], lds_kv0[0]);
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
// nothing to hide LDS latency or softmax arithmetic behind.  Here two waves
// share the 32 key rows instead:
//   role 0 ("S wave"):  S = Q K^T, P = exp2(S*c - LSE'), dV^T += dO^T P;  holds K, dV
//   role 1 ("dP wave"): dP = dO V^T, dS = P (dP - D), dK^T += Q^T dS;     holds V, dK
// P goes from the first to the second through LDS in MFMA operand format (bf16,
// 4 KB per 64x32 tile).  The unit of work is a tile of 64 query rows; the dP
// wave finishes a tile (dS, dK) one round after the S wave produced its P, so
// one workgroup barrier per round is all the synchronisation there is, and in
// every round both waves of a pair have 32 MFMAs of their own.
// Query tiles (Q, dO, LSE', D) sit in a ring of three LDS slots: a round reads
// the current slot (both waves) and the previous one (dP wave) while the
// asynchronous fetch of the next tile fills the third.
// ---------------------------------------------------------------------------
constexpr int NWP = 8;  // 4 S waves + 4 dP waves

template <int D>
__global__ __launch_bounds__(64 * NWP, 2) void dkv_kernel(const BwdParams prm)
{
    constexpr int KS = D / 16, TT = D / 32, QT = TILE_ROWS;
    constexpr int TB = TileGeom<D>::BYTES;
    constexpr int SLOT = 2 * TB + 2 * QT * 4;  // Q rows | dO rows | LSE*log2e | D
    __shared__ __align__(16) unsigned char lds_ring[3][SLOT];
    __shared__ __align__(16) unsigned char lds_p[4][2][4][1024];  // [pair][round parity][16-row block][lane*16]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wave >> 2, pw = wave & 3;  // waves w and w+4 share 32 key rows
    const int n = lane & 31, h = lane >> 5;
    const int item_id = blockIdx.x / prm.Hkv, c = blockIdx.x % prm.Hkv;
    const int g = prm.Hq / prm.Hkv;
    FragAddr<D> fa;
    fa.init(lane);
    RingLoader<D, NWP> ld;
    ld.init(lane, wave, (uint32_t)prm.Hq * D * 2);
    const uint32_t ring0 = lds_addr(&lds_ring[0][0]);

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
        const size_t off = ((size_t)(kbase + min(my_j, kvl - 1)) * prm.Hkv + c) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bf[ks] = as_bf16x8(*(const uint4 *)(src + off + 16 * ks));
    }

    const int i_first = (max(0, kv0 - qb) / QT) * QT;  // first query tile that can see key kv0
    const int n_qt = (ql - i_first + QT - 1) / QT;
    const int n_iter = n_qt * g;  // (head, query tile) pairs

    f32x16 acc[TT];  // dV^T (role 0) or dK^T (role 1) of this lane's key
    zero_acc(acc);

    // fetch of tile (head th of the group, query tile tq_idx) into ring slot `slot`
    auto fetch = [&](int th, int tq_idx, int slot) __attribute__((always_inline)) {
        const int head = c * g + th;
        const int i0 = i_first + tq_idx * QT;
        const uint32_t base = ring0 + (uint32_t)slot * SLOT;
        const size_t hoff = ((size_t)qbase * prm.Hq + head) * D;
        // rows past the end of the sequence read as zero (and are masked)
        ld.load(ld.rsrc(prm.q + hoff, ql), base, i0, wave);
        ld.load(ld.rsrc(prm.d_o + hoff, ql), base + TB, i0, wave);
        const size_t soff = (size_t)head * prm.total_q + qbase;
        if (wave == 2) dma_b32(rsrc_words(prm.lse2 + soff, (uint32_t)ql * 4), base + 2 * TB, lane * 4, i0 * 4);
        if (wave == 3) dma_b32(rsrc_words(prm.delta + soff, (uint32_t)ql * 4), base + 2 * TB + QT * 4, lane * 4, i0 * 4);
    };

    __syncthreads();  // the previous pass is done with every buffer
    fetch(0, 0, 0);
    wait_vmem();
    __syncthreads();

    // The two roles run the same round structure (same fetches, same barriers)
    // in separate loops, so that each keeps only its own values in registers.
    // Round T: ring slot T % 3 holds tile T = (head ch, query tile cq); the fetch
    // of tile T+1 = (nh, nq) goes to the next slot.
    if (role == 0) {
        int nh = 0, nq = 1, cq = 0, slot = 0;
        if (nq == n_qt) { nq = 0; nh = 1; }
        for (int T = 0; T <= n_iter; ++T) {
            const int slot_next = slot == 2 ? 0 : slot + 1;
            if (T + 1 < n_iter) fetch(nh, nq, slot_next);
            const unsigned char *cur = lds_ring[slot];
            const int i0 = i_first + cq * QT;  // first query row of the tile
            // a tile is skipped when its last query still precedes this pair's first key
            const bool act = T < n_iter && wave_active && qb + i0 + QT - 1 >= wj0;
            if (act) {
                const unsigned char *tq = cur, *tdo = cur + TB;
                const float *t_lse = (const float *)(cur + 2 * TB);
                unsigned char *px = lds_p[pw][T & 1][0];
                f32x16 s[2];
                zero_acc(s);
                // operand reads go out in two groups, each ahead of the MFMAs that use it;
                // the two 32-row blocks give two independent accumulation chains
#pragma unroll
                for (int kh = 0; kh < 2; ++kh) {
                    bf16x8 f0[KS / 2], f1[KS / 2];
#pragma unroll
                    for (int x = 0; x < KS / 2; ++x) {
                        f0[x] = fa.rows(tq, 0, kh * (KS / 2) + x);
                        f1[x] = fa.rows(tq, 1, kh * (KS / 2) + x);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < KS / 2; ++x) {
                        s[0] = mfma32(f0[x], bf[kh * (KS / 2) + x], s[0]);
                        s[1] = mfma32(f1[x], bf[kh * (KS / 2) + x], s[1]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                bf16x8 ft[TT];  // transposed dO fragments of the first 16 rows, fetched behind the softmax
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) ft[tt] = fa.cols(tdo, tt, 0);
                // masked pairs: key past the query (causal) or query row past the end
                const bool need_mask = (qb + i0 < wj0 + 31) || (i0 + QT > ql);
#pragma unroll
                for (int b = 0; b < 2; ++b) {
#pragma unroll
                    for (int vb = 0; vb < 4; ++vb) {
                        const float4 l4 = *(const float4 *)(t_lse + 32 * b + 8 * vb + 4 * h);
                        const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            s[b][4 * vb + e] = fast_exp2(__builtin_fmaf(s[b][4 * vb + e], cs, -lv[e]));
                    }
                }
                if (need_mask) {
#pragma unroll
                    for (int b = 0; b < 2; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int i = i0 + 32 * b + acc_row(v, h);
                            s[b][v] = (my_j > qb + i || i >= ql) ? 0.0f : s[b][v];
                        }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kbg = 0; kbg < 4; ++kbg) {
                    const bf16x8 pb = acc_to_b(s[kbg >> 1], kbg & 1);
                    *(bf16x8 *)(px + kbg * 1024 + lane * 16) = pb;
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(ft[tt], pb, acc[tt]);
                    if (kbg < 3) {
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) ft[tt] = fa.cols(tdo, tt, kbg + 1);
                    }
                }
            }
            wait_vmem();      // my share of the next tile has landed
            __syncthreads();  // ... and everyone's; P of this round is visible; the previous slot is free
            slot = slot_next;
            cq = nq;
            if (++nq == n_qt) { nq = 0; ++nh; }
        }
    } else {
        f32x16 dp[2];  // dP of the previous round's tile
        zero_acc(dp);
        bool prev_act = false;
        int nh = 0, nq = 1, cq = 0, slot = 0;
        if (nq == n_qt) { nq = 0; nh = 1; }
        for (int T = 0; T <= n_iter; ++T) {  // the extra round finishes the last tile
            const int slot_next = slot == 2 ? 0 : slot + 1, slot_prev = slot == 0 ? 2 : slot - 1;
            if (T + 1 < n_iter) fetch(nh, nq, slot_next);
            const unsigned char *cur = lds_ring[slot], *prv = lds_ring[slot_prev];
            const int i0 = i_first + cq * QT;
            const bool act = T < n_iter && wave_active && qb + i0 + QT - 1 >= wj0;
            if (prev_act) {
                // dS and dK of the previous round's tile: P as the S wave of this pair left it
                const float *t_dlt = (const float *)(prv + 2 * TB) + QT;
                const unsigned char *pp = lds_p[pw][(T - 1) & 1][0];
                bf16x8 ft[TT];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) ft[tt] = fa.cols(prv, tt, 0);
#pragma unroll
                for (int kbg = 0; kbg < 4; ++kbg) {
                    const int b = kbg >> 1, kb = kbg & 1;
                    const uint4 p4 = *(const uint4 *)(pp + kbg * 1024 + lane * 16);
                    const uint32_t pw32[4] = {p4.x, p4.y, p4.z, p4.w};
                    f32x16 &dpb = dp[b];
#pragma unroll
                    for (int vb = 0; vb < 2; ++vb) {
                        const float4 d4 = *(const float4 *)(t_dlt + 32 * b + 16 * kb + 8 * vb + 4 * h);
                        const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int v = 8 * kb + 4 * vb + e;
                            const uint32_t w = pw32[(4 * vb + e) >> 1];
                            const float pv = __builtin_bit_cast(float, (e & 1) ? (w & 0xffff0000u) : (w << 16));
                            dpb[v] = pv * (dpb[v] - dd[e]);  // dS
                        }
                    }
                    const bf16x8 db = acc_to_b(dpb, kb);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(ft[tt], db, acc[tt]);
                    if (kbg < 3) {
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) ft[tt] = fa.cols(prv, tt, kbg + 1);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (act) {  // dP of this round's tile, consumed in the next round
                const unsigned char *tdo = cur + TB;
                zero_acc(dp);
#pragma unroll
                for (int kh = 0; kh < 2; ++kh) {
                    bf16x8 f0[KS / 2], f1[KS / 2];
#pragma unroll
                    for (int x = 0; x < KS / 2; ++x) {
                        f0[x] = fa.rows(tdo, 0, kh * (KS / 2) + x);
                        f1[x] = fa.rows(tdo, 1, kh * (KS / 2) + x);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < KS / 2; ++x) {
                        dp[0] = mfma32(f0[x], bf[kh * (KS / 2) + x], dp[0]);
                        dp[1] = mfma32(f1[x], bf[kh * (KS / 2) + x], dp[1]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            prev_act = act;
            wait_vmem();
            __syncthreads();
            slot = slot_next;
            cq = nq;
            if (++nq == n_qt) { nq = 0; ++nh; }
        }
    }
    if (wave_active && my_j < kvl) {
        const size_t off = ((size_t)(kbase + my_j) * prm.Hkv + c) * D;
        if (role == 0) store_rows_bf16<TT>(prm.dv + off, acc, 1.0f, h);
        else store_rows_bf16<TT>(prm.dk + off, acc, prm.scale, h);
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
    dkv_kernel<D><<<gk, 64 * NWP, 0, st>>>(prm);
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
