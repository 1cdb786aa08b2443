// Backward kernels: D = rowsum(dO * O), dQ, and dK/dV with the GQA head
// reduction, for the packed varlen causal attention of fwd.hip.
//
//   P_ij  = exp(scale * q_i.k_j - LSE_i)          dP_ij = dO_i . v_j
//   dS_ij = P_ij (dP_ij - D_i)
//   dQ_i  = scale * sum_j dS_ij k_j
//   dK_j  = scale * sum_{h in group} sum_i dS_ij q_i
//   dV_j  =         sum_{h in group} sum_i P_ij dO_i
//
// dQ kernel: work items, workgroup shape and orientation of the forward kernel
// (query index on the MFMA column, so LSE_i and D_i are per-lane scalars):
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
#include "queue.h"
#include "tiles.h"

namespace {

constexpr float kLog2e = 1.4426950408889634f;

struct BwdParams {
    const uint16_t *q, *k, *v, *d_o, *o;
    const float *lse;
    float *delta, *lse2;  // workspace [Hq, total_q] each: -D and LSE * log2(e), written by the dQ kernel
    uint16_t *dq, *dk, *dv;
    const int4 *fwd_items, *dkv_items;
    const int32_t *cu_q, *cu_k, *q_begin, *q_len, *kv_len, *shares_kv;
    int32_t Hq, Hkv, total_q, BM, BN;
    float scale, scale_log2;
    // dK/dV head split: the query heads of a KV group are shared out over `head_split`
    // workgroups, which leave unrounded partial sums in dk_part / dv_part
    // ([head_split][total_k][Hkv][D] fp32) for dkv_reduce_kernel; 1 = no split
    int32_t head_split, total_k;
    float *dk_part, *dv_part;
    WgTrace *trace_dq, *trace_dkv;  // null, or one record per work item (measurement aid)
    WorkQueue *queue_dq, *queue_dkv;  // work queues of the persistent launches (workspace), zeroed before use
    int32_t n_work_dq, n_work_dkv;    // work items: what a plain grid would have as workgroups
};

// ---------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------
// The dQ kernel comes in two shapes, like the forward: 8 wavefronts (256 query rows) with a
// five-slot K ring and a four-slot V ring, one workgroup per compute unit; and, where two of
// them fit the LDS together (head_dim 64), 4 wavefronts (128 rows) with three K slots and two
// V slots, fetching one tile ahead with a barrier per tile.
constexpr int NWQ_LARGE = 8, NWQ_SMALL = 4;

// Two scores and two (dP - D) values -> one packed bf16 pair of dS, in two parts so
// that each part can sit behind one MFMA of a pipelined step (plain arithmetic would
// be moved by the compiler to its first use, behind all the MFMAs of the step).
// Part one: p = exp2(s * c - lse'); part two: p * (dP - D), packed.  Each exponential
// has an instruction between it and the first use of its result.
__device__ __forceinline__ void ds_exp2(float s0, float s1, float c, float l, float &t0, float &t1)
{
    asm volatile("v_fma_f32 %0, %2, %4, -%5\n\t"
                 "v_fma_f32 %1, %3, %4, -%5\n\t"
                 "v_exp_f32 %0, %0\n\t"
                 "v_exp_f32 %1, %1"
                 : "=&v"(t0), "=&v"(t1)
                 : "v"(s0), "v"(s1), "s"(c), "v"(l));
}
__device__ __forceinline__ uint32_t ds_mul_pack(float t0, float t1, float g0, float g1)
{
    uint32_t pk;
    float u0, u1;
    asm volatile("v_mul_f32 %1, %3, %5\n\t"
                 "v_mul_f32 %2, %4, %6\n\t"
                 "v_cvt_pk_bf16_f32 %0, %1, %2"
                 : "=&v"(pk), "=&v"(u0), "=&v"(u1)
                 : "v"(t0), "v"(t1), "v"(g0), "v"(g1));
    return pk;
}

// One workgroup = one forward work item (at most 256 query rows) x one query head;
// each of the 8 waves owns 32 query rows, two waves per SIMD.  K and V stream in
// 64-row tiles through LDS rings (K: five slots, V: four), fetched two tiles ahead by
// buffer loads that write LDS directly; fetches are issued, and the workgroup meets
// at a barrier, every second tile.  Half-tile j (32 keys) goes through
//   A(j): S^T = K Q^T and dP^T - D = V dO^T with -D as the accumulator's start,
//   V(j): dS^T = exp2(S^T c - LSE') (dP^T - D), rounded to bf16,
//   B(j): dQ^T += K^T dS^T,
// and step j issues A(j+1) with the vector work V(j) spread between its MFMAs, then
// B(j).  B(j) reads the transposed K of the half tile BEFORE the one A(j+1) reads,
// which is why the K ring has one slot more than the V ring.  Steps at the start, the
// end and the causal diagonal of a wave's range take a plain path with guards.
template <int D, int NWQ>
__device__ __forceinline__ void dq_work(const BwdParams &prm, const int bid)
{
    constexpr bool SMALL = NWQ == NWQ_SMALL;
    constexpr int KSL = SMALL ? 3 : 5, VSL = SMALL ? 2 : 4;  // ring slots
    constexpr int KS = D / 16, TT = D / 32, KT = TILE_ROWS;
    typedef TileGeom<D> G;
    constexpr int TB = G::BYTES;
    constexpr int HALF = 32 * G::ROWB;  // byte offset of a tile's second 32 rows
    typedef RingLoader<D, NWQ> Loader;
    static_assert(KS == 2 * TT, "B(j) has half as many MFMAs as A(j+1)");

    __shared__ __align__(16) unsigned char lds_k[KSL][TB];
    __shared__ __align__(16) unsigned char lds_v[VSL][TB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int n = lane & 31, h = lane >> 5;
    // an item of more rows than the workgroup covers is split over `subs` workgroups
    const int subs = (prm.BM + 32 * NWQ - 1) / (32 * NWQ);
    const int item_id = bid / (prm.Hq * subs), sub = (bid / prm.Hq) % subs;
    const int hl = bid % prm.Hq;
    const int g = prm.Hq / prm.Hkv;
    const int c = hl % prm.Hkv;
    const int head = c * g + hl / prm.Hkv;

    FragAddr<D> fa;
    fa.init(lane);
    Loader ld;
    ld.init(lane, wave, (uint32_t)prm.Hkv * D * 2);
    const uint32_t ring_k = lds_addr(&lds_k[0][0]), ring_v = lds_addr(&lds_v[0][0]);

    const int4 it = prm.fwd_items[item_id];
    const int seq = it.x;
    const int qb = prm.q_begin[seq], ql = prm.q_len[seq], kvl = prm.kv_len[seq];
    const int kbase = prm.cu_k[seq];
    const int row0 = it.y * prm.BM + sub * 32 * NWQ;
    const int qrow0 = it.z + sub * 32 * NWQ;
    const int rows = min(32 * NWQ, min(prm.BM, ql - it.y * prm.BM) - sub * 32 * NWQ);
    if (rows <= 0) return;  // the item ends before this part (the whole workgroup leaves)
    const uint64_t trace_t0 = trace_begin(prm.trace_dq);
    const int p0 = qb + row0;  // global position of the item's first query
    const int n_tiles = (p0 + rows + KT - 1) / KT;
    const float cs = prm.scale_log2;

    const int wrow0 = 32 * wave;
    const bool wave_active = wrow0 < rows;
    const int my_i = wrow0 + n;
    const int w_pmin = p0 + wrow0;
    const int w_pmax = p0 + min(wrow0 + 31, rows - 1);
    // half tiles (32 keys) of this wave: 0..L hold a visible key, those below n_full only visible keys
    const int L = wave_active ? w_pmax / 32 : -1;
    const int n_full = wave_active ? (w_pmin + 1) / 32 : 0;

    const i32x4 rk = ld.rsrc(prm.k + ((size_t)kbase * prm.Hkv + c) * D, kvl);
    const i32x4 rv = ld.rsrc(prm.v + ((size_t)kbase * prm.Hkv + c) * D, kvl);

    // Large shape: the fetch group issued at the start of an even period t is K and V tiles
    // t+2, t+3 (tiles past the end read as zero).  Small shape: every period t fetches K
    // and V tile t+1.
    int kslot = 0;  // slot of K tile t (t mod KSL), advanced at the end of every period
    auto fetch = [&](int t) __attribute__((always_inline)) {
        if (SMALL) {
            ld.load(rk, ring_k + (uint32_t)(kslot == 2 ? 0 : kslot + 1) * TB, (t + 1) * KT, wave);
            ld.load(rv, ring_v + (uint32_t)((t + 1) & 1) * TB, (t + 1) * KT, wave);
        } else {
            const int k2 = kslot >= 3 ? kslot - 3 : kslot + 2, k3 = kslot >= 2 ? kslot - 2 : kslot + 3;
            ld.load(rk, ring_k + (uint32_t)k2 * TB, (t + 2) * KT, wave);
            ld.load(rv, ring_v + (uint32_t)((t + 2) & 3) * TB, (t + 2) * KT, wave);
            ld.load(rk, ring_k + (uint32_t)k3 * TB, (t + 3) * KT, wave);
            ld.load(rv, ring_v + (uint32_t)((t + 3) & 3) * TB, (t + 3) * KT, wave);
        }
    };
    // start-up: the tiles of the first period(s).  The fetch group of period 0 follows after the
    // barrier below, because until then its slots stage this item's rows of Q, dO and O.
    ld.load(rk, ring_k, 0, wave);
    ld.load(rv, ring_v, 0, wave);
    if (!SMALL) {
        ld.load(rk, ring_k + TB, KT, wave);
        ld.load(rv, ring_v + TB, KT, wave);
    }
    // this wave's staging region: half a ring slot that holds no tile yet (large shape: K slots
    // 2-4 for waves 0-5 and V slots 2-3 for waves 6-7; small shape: K slots 1-2)
    typedef WaveStage<D> Stage;
    static_assert(2 * Stage::BYTES == TB, "two staging regions per ring slot");
    const uint32_t stage = SMALL ? ring_k + TB + (uint32_t)wave * Stage::BYTES
                                 : (wave < 6 ? ring_k + 2 * TB + (uint32_t)wave * Stage::BYTES
                                             : ring_v + 2 * TB + (uint32_t)(wave - 6) * Stage::BYTES);

    // B operands held for the whole item: this lane's query row of Q and dO
    bf16x8 qf[KS], dof[KS];
    float lse2, nd;
    {
        Stage st;
        st.init(lane);
        const uint32_t pitch = (uint32_t)prm.Hq * D * 2;
        const size_t hoff = ((size_t)qrow0 * prm.Hq + head) * D;
        u32x4 vq[Stage::N], vg[Stage::N], vo[Stage::N];
        st.load(vq, prm.q + hoff, pitch, wrow0, rows);
        st.load(vg, prm.d_o + hoff, pitch, wrow0, rows);
        st.load(vo, prm.o + hoff, pitch, wrow0, rows);
        const int my_row = qrow0 + min(my_i, rows - 1);  // packed row, clamped for loads
        lse2 = prm.lse[(size_t)head * prm.total_q + my_row] * kLog2e;
        st.put(stage, vq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = fa.rows_at(stage, ks);
        st.put(stage, vg);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dof[ks] = fa.rows_at(stage, ks);
        st.put(stage, vo);
        // D = rowsum(dO * O) of this lane's row (each half of the wave holds half of the
        // head dims) and LSE in the exp2 domain; both are stored at the end of the item for the
        // dK/dV kernel, launched after this one (it takes -D as the start of its dP accumulator)
        float dsum = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint4 ow = __builtin_bit_cast(uint4, fa.rows_at(stage, ks));
            const uint4 gw = __builtin_bit_cast(uint4, dof[ks]);
            const uint32_t a[4] = {ow.x, ow.y, ow.z, ow.w}, b[4] = {gw.x, gw.y, gw.z, gw.w};
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                dsum += __builtin_bit_cast(float, a[w] << 16) * __builtin_bit_cast(float, b[w] << 16);
                dsum += __builtin_bit_cast(float, a[w] & 0xffff0000u) * __builtin_bit_cast(float, b[w] & 0xffff0000u);
            }
        }
        nd = -add_other_half(dsum);
    }
    // Everything issued so far has to land here: the compiler's own count of
    // outstanding loads must be zero before the loops, or the waits it places
    // for these fragments would also wait for the tile fetches in flight.
    wait_vmem();
    __syncthreads();
    if ((SMALL ? 1 : 2) < n_tiles) fetch(0);  // the staging regions are free again

    f32x16 acc[TT];
    zero_acc(acc);

    // ---- pipelined step j: A(j+1) from kp / vp with V(j) on s_in / g_in between its
    // MFMAs, then B(j) on the transposed K at kt.  FIRST: first step of a period (reads
    // its first operands itself and, at the end, those of the second step from kp2 / vp2);
    // otherwise they are already in fr.
    auto steady = [&](auto first_tag, const unsigned char *kp, const unsigned char *vp,
                      const unsigned char *kt, const unsigned char *kp2, const unsigned char *vp2,
                      const f32x16 &s_in, const f32x16 &g_in, f32x16 &s_out, f32x16 &g_out,
                      bf16x8 (&fr)[4]) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_tag)::value;
        // operand stream of the step: 2*KS reads for A (K rows, V rows alternating), then 2*TT for B
        auto operand = [&](int x) __attribute__((always_inline)) {
            if (x < 2 * KS) return (x & 1) ? fa.rows(vp, 0, x >> 1) : fa.rows(kp, 0, x >> 1);
            const int y = x - 2 * KS;
            return fa.cols(kt, y % TT, y / TT);
        };
        if (FIRST) {
#pragma unroll
            for (int x = 0; x < 3; ++x) fr[x] = operand(x);
        }
        SB();
        uint32_t pw[8];
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            constexpr int EPS = 16 / KS;  // dS values per step of the loop (2 or 4)
            float t[EPS];
            if (i == 0) {
                f32x16 z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                s_out = mfma32(fr[0], qf[0], z);
            } else {
                s_out = mfma32(fr[(2 * i) % 4], qf[i], s_out);
            }
#pragma unroll
            for (int e = 0; e < EPS; e += 2)
                ds_exp2(s_in[EPS * i + e], s_in[EPS * i + e + 1], cs, lse2, t[e], t[e + 1]);
            fr[(2 * i + 3) % 4] = operand(2 * i + 3);
            SB();
            if (i == 0) {
                f32x16 z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = nd;
                g_out = mfma32(fr[1], dof[0], z);
            } else {
                g_out = mfma32(fr[(2 * i + 1) % 4], dof[i], g_out);
            }
#pragma unroll
            for (int e = 0; e < EPS; e += 2)
                pw[(EPS * i + e) >> 1] = ds_mul_pack(t[e], t[e + 1], g_in[EPS * i + e], g_in[EPS * i + e + 1]);
            fr[(2 * i + 4) % 4] = operand(2 * i + 4);
            SB();
        }
        const bf16x8 ds0 = as_bf16x8(make_uint4(pw[0], pw[1], pw[2], pw[3]));
        const bf16x8 ds1 = as_bf16x8(make_uint4(pw[4], pw[5], pw[6], pw[7]));
#pragma unroll
        for (int y = 0; y < 2 * TT; ++y) {
            acc[y % TT] = mfma32(fr[(2 * KS + y) % 4], y < TT ? ds0 : ds1, acc[y % TT]);
            const int nx = y + 3;  // of this step's B stream, then of the next step's A stream
            if (nx < 2 * TT) {
                fr[(2 * KS + nx) % 4] = operand(2 * KS + nx);
            } else if (FIRST) {
                const int x = nx - 2 * TT;
                fr[x] = (x & 1) ? fa.rows(vp2, 0, x >> 1) : fa.rows(kp2, 0, x >> 1);
            }
            SB();
        }
    };

    // ---- plain step j with run-time guards (start, end and diagonal of the wave's range)
    auto generic = [&](int j, const unsigned char *kp, const unsigned char *vp, const unsigned char *kt,
                       const f32x16 &s_in, const f32x16 &g_in, f32x16 &s_out, f32x16 &g_out)
                       __attribute__((always_inline)) {
        if (j + 1 <= L) {  // A(j+1)
#pragma unroll
            for (int v = 0; v < 16; ++v) { s_out[v] = 0.0f; g_out[v] = nd; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s_out = mfma32(fa.rows(kp, 0, ks), qf[ks], s_out);
                g_out = mfma32(fa.rows(vp, 0, ks), dof[ks], g_out);
                if (ks % 4 == 3) SB();
            }
        }
        if (j >= 0 && j <= L) {  // V(j), B(j)
            f32x16 ds;
#pragma unroll
            for (int v = 0; v < 16; ++v) ds[v] = fast_exp2(__builtin_fmaf(s_in[v], cs, -lse2)) * g_in[v];
            if (j >= n_full) {  // half tile touches the diagonal for this wave
                // relative position from an opaque copy of the lane index: the sixteen
                // per-register thresholds are formed here rather than kept for the whole kernel
                int li = lane;
                asm volatile("" : "+v"(li));
                const int rel = p0 + wrow0 + (li & 31) - 32 * j - 4 * (li >> 5);  // my_pos - 32j - 4h
#pragma unroll
                for (int v = 0; v < 16; ++v) ds[v] = (8 * (v >> 2) + (v & 3) > rel) ? 0.0f : ds[v];
            }
            SB();
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 b = acc_to_b(ds, kb);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(fa.cols(kt, tt, kb), b, acc[tt]);
                SB();
            }
        }
    };

    f32x16 sx, sy, gx, gy;  // S and dP - D of the current / next half tile, ping-pong
#pragma unroll
    for (int v = 0; v < 16; ++v) { sx[v] = 0.0f; sy[v] = 0.0f; gx[v] = 0.0f; gy[v] = 0.0f; }

    // Period t: steps 2t-1 and 2t, i.e. A of both halves of tile t (K and V rows), B of
    // the second half of K tile t-1 and of the first half of K tile t.  K tile t sits in
    // slot t mod KSL, V tile t in slot t mod VSL.  Large shape: an even period starts by
    // fetching the tiles of the next two periods into slots that the periods before the
    // last barrier have left; an odd period ends with the wait for them and the barrier.
    // Small shape: every period fetches the next tile (into the slot of K tile t-2, whose
    // second half period t-1 was the last to read, and of V tile t-1) and ends with the
    // wait and the barrier.
    auto period_begin = [&](int t) __attribute__((always_inline)) {
        if (t == 0) return;  // period 0's group went out at start-up
        if (SMALL) {
            if (t + 1 < n_tiles) fetch(t);
        } else {
            if ((t & 1) == 0 && t + 2 < n_tiles) fetch(t);
        }
    };
    auto period_end = [&](int t) __attribute__((always_inline)) {
        if (SMALL || (t & 1)) {
            wait_vmem();      // my share of the tiles of the next period(s) has landed
            __syncthreads();  // ... and everyone's; everyone is done with the tiles they replace
        }
        kslot = kslot == KSL - 1 ? 0 : kslot + 1;
    };
    // periods whose two steps are fully inside the wave's unmasked range
    const int t_steady_end = min((L - 1) / 2, (n_full - 1) / 2);  // last t with 2t+1 <= L and 2t < n_full
    auto plain_period = [&](int t) __attribute__((always_inline)) {
        period_begin(t);
        const unsigned char *tk = lds_k[kslot], *tv = lds_v[t & (VSL - 1)];
        const unsigned char *tkp = lds_k[kslot == 0 ? KSL - 1 : kslot - 1] + HALF;  // second half of K tile t-1
#pragma unroll 1
        for (int hh = 0; hh < 2; ++hh) {
            generic(2 * t - 1 + hh, tk + hh * HALF, tv + hh * HALF, hh ? tk : tkp, sx, gx, sy, gy);
            sx = sy;
            gx = gy;
        }
        period_end(t);
    };
    plain_period(0);
    int t = 1;
    for (; t <= t_steady_end; ++t) {
        period_begin(t);
        const unsigned char *tk = lds_k[kslot], *tv = lds_v[t & (VSL - 1)];
        const unsigned char *tkp = lds_k[kslot == 0 ? KSL - 1 : kslot - 1] + HALF;
        bf16x8 fr[4];  // operand fragments in flight
        steady(std::true_type{}, tk, tv, tkp, tk + HALF, tv + HALF, sx, gx, sy, gy, fr);
        steady(std::false_type{}, tk + HALF, tv + HALF, tk, tk, tv, sy, gy, sx, gx, fr);
        period_end(t);
    }
#pragma unroll 1
    for (; t <= n_tiles; ++t) plain_period(t);

    __syncthreads();  // nobody reads a tile any more: the staging regions are free
    if (wave_active) {
        // derived after the loop from opaque copies, so that no part of the
        // output addresses is kept in registers during the loop
        int li = lane;
        asm volatile("" : "+v"(li));
        const int on = li & 31, oh = li >> 5, oi = wrow0 + on;
        Stage st;
        st.init(li);
        st.put_acc(stage, acc, prm.scale, on, oh);
        st.store(stage, prm.dq + ((size_t)qrow0 * prm.Hq + head) * D, (uint32_t)prm.Hq * D * 2, wrow0, rows);
        if (oh == 0 && oi < rows) {
            prm.delta[(size_t)head * prm.total_q + qrow0 + oi] = nd;
            prm.lse2[(size_t)head * prm.total_q + qrow0 + oi] = lse2;
        }
    }
    trace_end(prm.trace_dq, trace_t0, bid);
}

template <int D, int NWQ>
__global__ __launch_bounds__(64 * NWQ, 2) void dq_kernel(const BwdParams prm)
{
    __shared__ int work_slot;
    work_loop(prm.queue_dq, prm.n_work_dq, &work_slot,
              [&](int w) __attribute__((always_inline)) { dq_work<D, NWQ>(prm, w); });
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
// Vector-ALU pieces of the dK/dV kernel, written out so that they stay where the
// kernel puts them: between the MFMAs of the next block (plain arithmetic would be
// moved to its first use, behind all of them, and a wave that issues nothing but
// vector instructions for a long stretch slows the MFMAs of the wave it shares a
// SIMD with).
// Four scores -> four probabilities exp2(s * c - l), packed twice: to two bf16 pairs (w0, w1:
// the S wave's own MFMA operand) and to two fp16 pairs (h0, h1: what the dP wave gets).  The
// dP wave only multiplies P element by element, and a mixed-precision multiply takes an fp16
// operand as it is, where a bf16 one costs an instruction to widen first: the extra packing
// here is on the wave of the pair that waits at the barrier, the widening was on the one that
// does not.  (Probabilities are at most 1; fp16 keeps three bits more of them than bf16 and
// goes to zero below 6e-8.)  Every exponential has an instruction between it and the first use
// of its result.
__device__ __forceinline__ void p_quad(const float (&sv)[4], float c, const float4 &l, uint32_t &w0, uint32_t &w1,
                                       uint32_t &h0, uint32_t &h1)
{
    float t0, t1, t2, t3;
    asm volatile("v_fma_f32 %0, %8, %12, -%13\n\t"
                 "v_fma_f32 %1, %9, %12, -%14\n\t"
                 "v_fma_f32 %2, %10, %12, -%15\n\t"
                 "v_fma_f32 %3, %11, %12, -%16\n\t"
                 "v_exp_f32 %0, %0\n\t"
                 "v_exp_f32 %1, %1\n\t"
                 "v_exp_f32 %2, %2\n\t"
                 "v_exp_f32 %3, %3\n\t"
                 "v_cvt_pk_bf16_f32 %4, %0, %1\n\t"
                 "v_cvt_pk_bf16_f32 %5, %2, %3\n\t"
                 "v_cvt_pk_f16_f32 %6, %0, %1\n\t"
                 "v_cvt_pk_f16_f32 %7, %2, %3"
                 : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(w0), "=&v"(w1), "=&v"(h0), "=&v"(h1)
                 : "v"(sv[0]), "v"(sv[1]), "v"(sv[2]), "v"(sv[3]), "s"(c), "v"(l.x), "v"(l.y), "v"(l.z), "v"(l.w));
}
// Two packed fp16 P pairs times four (dP - D) values -> two packed bf16 dS pairs.
__device__ __forceinline__ void ds_quad(uint32_t p01, uint32_t p23, const float (&g)[4], uint32_t &w0, uint32_t &w1)
{
    float t0, t1, t2, t3;
    asm volatile("v_fma_mix_f32 %0, %6, %8, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]\n\t"
                 "v_fma_mix_f32 %1, %6, %9, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
                 "v_fma_mix_f32 %2, %7, %10, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]\n\t"
                 "v_fma_mix_f32 %3, %7, %11, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]\n\t"
                 "v_cvt_pk_bf16_f32 %4, %0, %1\n\t"
                 "v_cvt_pk_bf16_f32 %5, %2, %3"
                 : "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3), "=&v"(w0), "=&v"(w1)
                 : "v"(p01), "v"(p23), "v"(g[0]), "v"(g[1]), "v"(g[2]), "v"(g[3]));
}

// PAIRS wave pairs per workgroup: 4 (8 wavefronts, 128 key rows, two wavefronts per SIMD), or,
// at head_dim 64 where 136 registers and 106 KB of LDS allow it, 6 (12 wavefronts, 192 key
// rows, three per SIMD): more wavefronts to overlap with and a third fewer fetches of each
// query tile.  The 12-wavefront shape serves work items of block_n = 192.
constexpr int PAIRS_8W = 4, PAIRS_12W = 6;

template <int D, int PAIRS>
__device__ __forceinline__ void dkv_work(const BwdParams &prm, const int bid)
{
    constexpr int NWP = 2 * PAIRS;   // wavefronts: PAIRS S waves, then PAIRS dP waves
    constexpr int SUB = 32 * PAIRS;  // key rows per workgroup
    constexpr int KS = D / 16, TT = D / 32, QT = TILE_ROWS;
    constexpr int TB = TileGeom<D>::BYTES;
    constexpr int SLOT = 2 * TB + 2 * QT * 4;  // Q rows | dO rows | LSE*log2e | D
    __shared__ __align__(16) unsigned char lds_ring[3][SLOT];
    __shared__ __align__(16) unsigned char lds_p[PAIRS][2][4][1024];  // [pair][round parity][16-row block][lane*16]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int role = wave / PAIRS, pw = wave % PAIRS;  // waves w and w+PAIRS share 32 key rows
    const int n = lane & 31, h = lane >> 5;
    // blockIdx -> (item, SUB-key pass of the item, KV head); an item of more key rows
    // than SUB is several workgroups
    const int passes = (prm.BN + SUB - 1) / SUB;
    const int sub = bid % passes;
    const int hs = prm.head_split;
    const int hp = (bid / passes) % hs;  // which share of the group's query heads
    const int c = (bid / passes / hs) % prm.Hkv, item_id = bid / passes / hs / prm.Hkv;
    const int g_all = prm.Hq / prm.Hkv;
    const int head_lo = (hp * g_all) / hs;
    const int g = ((hp + 1) * g_all) / hs - head_lo;  // >= 1 since head_split <= g_all
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

    if (sub * SUB >= item_rows) return;  // (whole workgroup) this item has no second pass
    const uint64_t trace_t0 = trace_begin(prm.trace_dkv);
    const int kv0 = it.y * prm.BN + sub * SUB;  // first key position of the pass
    const int krows = min(SUB, kvl - kv0);
    const int wj0 = kv0 + 32 * pw;              // this pair's first key position
    const bool wave_active = 32 * pw < krows;
    const int my_j = wj0 + n;                   // this lane's key position

    // this wave's staging region: ring slots 1 and 2 hold no tile at the start and the end of a
    // pass (eight regions); the waves beyond the eighth use the P exchange area
    typedef WaveStage<D> Stage;
    static_assert(8 * Stage::BYTES <= 2 * SLOT && (NWP - 8) * Stage::BYTES <= (int)sizeof(lds_p),
                  "staging regions do not fit the idle part of the LDS");
    const uint32_t stage = wave < 8 ? ring0 + SLOT + (uint32_t)wave * Stage::BYTES
                                    : lds_addr(&lds_p[0][0][0][0]) + (uint32_t)(wave - 8) * Stage::BYTES;
    // B operand held for the whole pass: this lane's key row of K (role 0) or V (role 1).
    bf16x8 bf[KS];
    {
        Stage st;
        st.init(lane);
        u32x4 vk[Stage::N];
        st.load(vk, (role == 0 ? prm.k : prm.v) + ((size_t)kbase * prm.Hkv + c) * D, (uint32_t)prm.Hkv * D * 2, wj0, kvl);
        st.put(stage, vk);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bf[ks] = fa.rows_at(stage, ks);
    }

    // Query tiles that can see key kv0, numbered 0 .. n_qt-1 in position order: those of
    // the early chunk (segment seq-1, when this prefix is shared by two chunks and the
    // pass starts inside the early chunk's own prefix) and then those of segment seq.
    const int i_first = (max(0, kv0 - qb) / QT) * QT;
    const int n_qt_own = (ql - i_first + QT - 1) / QT;
    int qb_e = 0, ql_e = 0, qbase_e = 0, i_first_e = 0, n_qt_e = 0;
    if (prm.shares_kv[seq] && kv0 < prm.kv_len[seq - 1]) {
        qb_e = prm.q_begin[seq - 1];
        ql_e = prm.q_len[seq - 1];
        qbase_e = prm.cu_q[seq - 1];
        i_first_e = (max(0, kv0 - qb_e) / QT) * QT;
        n_qt_e = (ql_e - i_first_e + QT - 1) / QT;
    }
    const int n_qt = n_qt_e + n_qt_own;
    const int n_iter = n_qt * g;  // (head, query tile) pairs
    // tile t -> first global position of its segment, rows of the segment, first row of the tile
    auto tile_qb = [&](int t) __attribute__((always_inline)) { return t < n_qt_e ? qb_e : qb; };
    auto tile_ql = [&](int t) __attribute__((always_inline)) { return t < n_qt_e ? ql_e : ql; };
    auto tile_i0 = [&](int t) __attribute__((always_inline)) {
        return t < n_qt_e ? i_first_e + t * QT : i_first + (t - n_qt_e) * QT;
    };

    f32x16 acc[TT];  // dV^T (role 0) or dK^T (role 1) of this lane's key
    zero_acc(acc);

    // fetch of tile (head th of the group, query tile tq_idx) into ring slot `slot`
    auto fetch = [&](int th, int tq_idx, int slot) __attribute__((always_inline)) {
        const int head = c * g_all + head_lo + th;
        const int i0 = tile_i0(tq_idx);
        const int rows = tile_ql(tq_idx);
        const int first_row = tq_idx < n_qt_e ? qbase_e : qbase;
        const uint32_t base = ring0 + (uint32_t)slot * SLOT;
        const size_t hoff = ((size_t)first_row * prm.Hq + head) * D;
        // rows past the end of the segment read as zero (and are masked)
        ld.load(ld.rsrc(prm.q + hoff, rows), base, i0, wave);
        ld.load(ld.rsrc(prm.d_o + hoff, rows), base + TB, i0, wave);
        const size_t soff = (size_t)head * prm.total_q + first_row;
        if (wave == 2) dma_b32(rsrc_words(prm.lse2 + soff, (uint32_t)rows * 4), base + 2 * TB, lane * 4, i0 * 4);
        if (wave == 3) dma_b32(rsrc_words(prm.delta + soff, (uint32_t)rows * 4), base + 2 * TB + QT * 4, lane * 4, i0 * 4);
    };

    fetch(0, n_qt - 1, 0);
    wait_vmem();
    __syncthreads();

    // Round T: ring slot T % 3 holds (head T % g, query tile n_qt - 1 - T / g): heads
    // innermost, query tiles from the end of the sequence down to the block's
    // diagonal.  Every workgroup of a sequence then starts at the same tile and the
    // ones running together walk the same tiles at the same time, which is what
    // lets the XCD's L2 serve most of their fetches.
    // A pair's LIVE rounds are a prefix of the sequence: the tiles whose last query still
    // precedes the pair's first key are the lowest ones, walked last.  Each role runs its
    // live rounds in ONE loop with ONE sequence of MFMAs (masks, where a tile needs them,
    // only change scores before the exponentials), then idles through the rest with the
    // fetches and barriers every wave must take part in.  With alternative MFMA paths
    // inside one loop the compiler reconciled their register assignments with ~100
    // register copies per round.
    auto tile_live = [&](int t) __attribute__((always_inline)) {
        return tile_qb(t) + tile_i0(t) + QT - 1 >= wj0;
    };
    int n_live = 0;  // live rounds of this pair
    if (wave_active) {
        int dead_tiles = 0;
        if (n_qt_e > 0) {  // the early chunk's lowest tile may be dead; the late chunk's never is
            if (!tile_live(0)) dead_tiles = 1;
        } else {
            while (dead_tiles < n_qt && !tile_live(dead_tiles)) ++dead_tiles;
        }
        n_live = (n_qt - dead_tiles) * g;
    }
    int nh = 1, nq = n_qt - 1, cq = n_qt - 1, slot = 0;  // cq: tile of this round; (nh, nq): head, tile of the next
    if (nh == g) { nh = 0; --nq; }
    // start of a round: fetch the next round's tile; end: wait, barrier, advance
    auto round_begin = [&](int T) __attribute__((always_inline)) {
        if (T + 1 < n_iter) fetch(nh, nq, slot == 2 ? 0 : slot + 1);
    };
    auto round_end = [&]() __attribute__((always_inline)) {
        wait_vmem();      // my share of the next tile has landed
        __syncthreads();  // ... and everyone's; P of this round is visible; the previous slot is free
        slot = slot == 2 ? 0 : slot + 1;
        cq = nq;
        if (++nh == g) { nh = 0; --nq; }
    };
    int T = 0;
    if (role == 0) {
#pragma unroll 1
        for (; T < n_live; ++T) {
            round_begin(T);
            const unsigned char *cur = lds_ring[slot];
            const int i0 = tile_i0(cq);  // first query row of the tile inside its segment
            const int qb_t = tile_qb(cq), ql_t = tile_ql(cq);
            const unsigned char *tq = cur, *tdo = cur + TB;
            const float *t_lse = (const float *)(cur + 2 * TB);
            unsigned char *px = lds_p[pw][T & 1][0];
            // masked pairs: key past the query (causal) or query row past the end
            const bool need_mask = (qb_t + i0 < wj0 + 31) || (i0 + QT > ql_t);
            // scores of masked pairs become -inf (probability 0) before the exponentials
            auto mask_block = [&](f32x16 &sb, int b) __attribute__((always_inline)) {
                // (the asm also keeps this block behind its branch: turned into selects it
                // would run in every round)
                int li = lane;
                asm volatile("" : "+v"(li));  // thresholds formed here, not kept across rounds
                const int row0 = i0 + 32 * b + 4 * (li >> 5);            // + 8*vb + e = query row
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = row0 + 8 * (v >> 2) + (v & 3);
                    sb[v] = (wj0 + (li & 31) > qb_t + i || i >= ql_t) ? -INFINITY : sb[v];
                }
            };
            f32x16 s[2];
            bf16x8 fr[4];
            // S of the first 32 rows; operand reads run three MFMAs ahead
#pragma unroll
            for (int x = 0; x < 3; ++x) fr[x] = fa.rows(tq, 0, x);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == 0) {
                    f32x16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                    s[0] = mfma32(fr[0], bf[0], z);
                } else {
                    s[0] = mfma32(fr[ks % 4], bf[ks], s[0]);
                }
                const int nx = ks + 3;
                fr[nx % 4] = nx < KS ? fa.rows(tq, 0, nx) : fa.rows(tq, 1, nx - KS);
                SB();
            }
            if (need_mask) mask_block(s[0], 0);
            // S of the second 32 rows with the probabilities of the first behind its
            // MFMAs, then dV of the first with the probabilities of the second
            uint32_t w[2][8];
            uint32_t hw[4];  // fp16 copies of two quads at a time, on their way to the dP wave
            bf16x8 ft[4];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == 0) {
                    f32x16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                    s[1] = mfma32(fr[(KS + 0) % 4], bf[0], z);
                } else {
                    s[1] = mfma32(fr[(KS + ks) % 4], bf[ks], s[1]);
                }
                const int nx = ks + 3;
                if (nx < KS) fr[(KS + nx) % 4] = fa.rows(tq, 1, nx);
                if (KS == 8 ? (ks % 2 == 1) : true) {
                    const int vb = KS == 8 ? ks / 2 : ks;
                    const float4 l4 = *(const float4 *)(t_lse + 8 * vb + 4 * h);
                    const float sv[4] = {s[0][4 * vb], s[0][4 * vb + 1], s[0][4 * vb + 2], s[0][4 * vb + 3]};
                    p_quad(sv, cs, l4, w[0][2 * vb], w[0][2 * vb + 1], hw[2 * (vb & 1)], hw[2 * (vb & 1) + 1]);
                    if (vb & 1) *(uint4 *)(px + (vb >> 1) * 1024 + lane * 16) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                }
                if (ks >= KS - 3) ft[(ks - (KS - 3))] = fa.cols(tdo, (ks - (KS - 3)) % TT, (ks - (KS - 3)) / TT);
                SB();
            }
            if (need_mask) mask_block(s[1], 1);
            const bf16x8 pb0 = as_bf16x8(make_uint4(w[0][0], w[0][1], w[0][2], w[0][3]));
            const bf16x8 pb1 = as_bf16x8(make_uint4(w[0][4], w[0][5], w[0][6], w[0][7]));
            // dV of rows 0..31 (2 x TT MFMAs); probabilities of rows 32..63 behind them
#pragma unroll
            for (int m = 0; m < 2 * TT; ++m) {
                acc[m % TT] = mfma32(ft[m % 4], m < TT ? pb0 : pb1, acc[m % TT]);
                const int nx = m + 3;
                ft[nx % 4] = fa.cols(tdo, nx % TT, nx / TT);  // runs on into rows 32..63
                if (TT == 4 ? (m % 2 == 1) : true) {
                    const int vb = TT == 4 ? m / 2 : m;
                    const float4 l4 = *(const float4 *)(t_lse + 32 + 8 * vb + 4 * h);
                    const float sv[4] = {s[1][4 * vb], s[1][4 * vb + 1], s[1][4 * vb + 2], s[1][4 * vb + 3]};
                    p_quad(sv, cs, l4, w[1][2 * vb], w[1][2 * vb + 1], hw[2 * (vb & 1)], hw[2 * (vb & 1) + 1]);
                    if (vb & 1) *(uint4 *)(px + (2 + (vb >> 1)) * 1024 + lane * 16) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                }
                SB();
            }
            const bf16x8 pb2 = as_bf16x8(make_uint4(w[1][0], w[1][1], w[1][2], w[1][3]));
            const bf16x8 pb3 = as_bf16x8(make_uint4(w[1][4], w[1][5], w[1][6], w[1][7]));
            // dV of rows 32..63
#pragma unroll
            for (int m = 2 * TT; m < 4 * TT; ++m) {
                acc[m % TT] = mfma32(ft[m % 4], m < 3 * TT ? pb2 : pb3, acc[m % TT]);
                const int nx = m + 3;
                if (nx < 4 * TT) ft[nx % 4] = fa.cols(tdo, nx % TT, nx / TT);
                SB();
            }
            round_end();
        }
    } else {
        f32x16 dp[2];  // dP - D of the previous round's tile
        zero_acc(dp);
        // first live round: dP - D of its tile only
        if (n_live > 0) {
            round_begin(T);
            const unsigned char *cur = lds_ring[slot];
            const unsigned char *tdo = cur + TB;
            const float *t_nd = (const float *)(cur + 2 * TB) + QT;  // -D of this round's tile
            // accumulator start of a 32-row block of dP: -D of its rows
            auto neg_d = [&](int b) __attribute__((always_inline)) {
                f32x16 z;
#pragma unroll
                for (int vb = 0; vb < 4; ++vb) {
                    const float4 d4 = *(const float4 *)(t_nd + 32 * b + 8 * vb + 4 * h);
                    z[4 * vb] = d4.x; z[4 * vb + 1] = d4.y; z[4 * vb + 2] = d4.z; z[4 * vb + 3] = d4.w;
                }
                return z;
            };
            {
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    dp[b] = neg_d(b);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        dp[b] = mfma32(fa.rows(tdo, b, ks), bf[ks], dp[b]);
                        if (ks % 4 == 3) SB();
                    }
                }
            }
            round_end();
            ++T;
        }
#pragma unroll 1
        for (; T < n_live; ++T) {
            round_begin(T);
            const int slot_prev = slot == 0 ? 2 : slot - 1;
            const unsigned char *cur = lds_ring[slot], *prv = lds_ring[slot_prev];
            const unsigned char *tdo = cur + TB;
            const float *t_nd = (const float *)(cur + 2 * TB) + QT;  // -D of this round's tile
            const unsigned char *pp = lds_p[pw][(T - 1) & 1][0];
            // accumulator start of a 32-row block of dP: -D of its rows
            auto neg_d = [&](int b) __attribute__((always_inline)) {
                f32x16 z;
#pragma unroll
                for (int vb = 0; vb < 4; ++vb) {
                    const float4 d4 = *(const float4 *)(t_nd + 32 * b + 8 * vb + 4 * h);
                    z[4 * vb] = d4.x; z[4 * vb + 1] = d4.y; z[4 * vb + 2] = d4.z; z[4 * vb + 3] = d4.w;
                }
                return z;
            };
            // dS of 16 rows (block b, half kb) of the previous tile from its P and dP - D
            auto ds_half = [&](const uint4 &p4, const f32x16 &g, int kb, uint32_t (&w)[4]) __attribute__((always_inline)) {
                const float g0[4] = {g[8 * kb], g[8 * kb + 1], g[8 * kb + 2], g[8 * kb + 3]};
                const float g1[4] = {g[8 * kb + 4], g[8 * kb + 5], g[8 * kb + 6], g[8 * kb + 7]};
                ds_quad(p4.x, p4.y, g0, w[0], w[1]);
                ds_quad(p4.z, p4.w, g1, w[2], w[3]);
            };
            // Both tiles live: dP of this tile's first 32 rows with dS of the previous
            // tile's first 32 rows behind its MFMAs; dK of those rows with the second dS
            // behind; then dK of the second rows and dP of this tile's second rows.
            f32x16 dpn;
            bf16x8 fr[4], ft[4];
            uint32_t w[4][4];
            // what the first MFMA waits for is asked for first (when the barrier opens all eight
            // waves queue their reads at once): -D, the start of its accumulator, and dO
            dpn = neg_d(0);
#pragma unroll
            for (int x = 0; x < 3; ++x) fr[x] = fa.rows(tdo, 0, x);
            SB();
            const uint4 p0 = *(const uint4 *)(pp + 0 * 1024 + lane * 16);
            const uint4 p1 = *(const uint4 *)(pp + 1 * 1024 + lane * 16);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                dpn = mfma32(fr[ks % 4], bf[ks], dpn);
                const int nx = ks + 3;
                if (nx < KS) fr[nx % 4] = fa.rows(tdo, 0, nx);
                if (ks == (KS == 8 ? 1 : 0)) ds_half(p0, dp[0], 0, w[0]);
                if (ks == (KS == 8 ? 4 : 2)) ds_half(p1, dp[0], 1, w[1]);
                if (ks >= KS - 3) ft[ks - (KS - 3)] = fa.cols(prv, (ks - (KS - 3)) % TT, (ks - (KS - 3)) / TT);
                SB();
            }
            const uint4 p2 = *(const uint4 *)(pp + 2 * 1024 + lane * 16);
            const uint4 p3 = *(const uint4 *)(pp + 3 * 1024 + lane * 16);
            const bf16x8 db0 = as_bf16x8(make_uint4(w[0][0], w[0][1], w[0][2], w[0][3]));
            const bf16x8 db1 = as_bf16x8(make_uint4(w[1][0], w[1][1], w[1][2], w[1][3]));
#pragma unroll
            for (int m = 0; m < 2 * TT; ++m) {
                acc[m % TT] = mfma32(ft[m % 4], m < TT ? db0 : db1, acc[m % TT]);
                const int nx = m + 3;
                ft[nx % 4] = fa.cols(prv, nx % TT, nx / TT);  // runs on into rows 32..63
                if (m == (TT == 4 ? 1 : 0)) ds_half(p2, dp[1], 0, w[2]);
                if (m == (TT == 4 ? 4 : 2)) ds_half(p3, dp[1], 1, w[3]);
                SB();
            }
            const bf16x8 db2 = as_bf16x8(make_uint4(w[2][0], w[2][1], w[2][2], w[2][3]));
            const bf16x8 db3 = as_bf16x8(make_uint4(w[3][0], w[3][1], w[3][2], w[3][3]));
            // dS of the previous tile is complete: its dP - D registers take the start of this
            // tile's second block (-D) now, eight MFMAs before the products that need it
            dp[1] = neg_d(1);
#pragma unroll
            for (int x = 0; x < 3; ++x) fr[x] = fa.rows(tdo, 1, x);
            SB();
#pragma unroll
            for (int m = 2 * TT; m < 4 * TT; ++m) {
                acc[m % TT] = mfma32(ft[m % 4], m < 3 * TT ? db2 : db3, acc[m % TT]);
                const int nx = m + 3;
                if (nx < 4 * TT) ft[nx % 4] = fa.cols(prv, nx % TT, nx / TT);
                SB();
            }
            dp[0] = dpn;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                dp[1] = mfma32(fr[ks % 4], bf[ks], dp[1]);
                const int nx = ks + 3;
                if (nx < KS) fr[nx % 4] = fa.rows(tdo, 1, nx);
                SB();
            }
            round_end();
        }
        // the round after the last live one: dS and dK of the last live tile
        if (n_live > 0) {
            round_begin(T);
            const int slot_prev = slot == 0 ? 2 : slot - 1;
            const unsigned char *prv = lds_ring[slot_prev];
            const unsigned char *pp = lds_p[pw][(T - 1) & 1][0];
            // dS of 16 rows (block b, half kb) of the previous tile from its P and dP - D
            auto ds_half = [&](const uint4 &p4, const f32x16 &g, int kb, uint32_t (&w)[4]) __attribute__((always_inline)) {
                const float g0[4] = {g[8 * kb], g[8 * kb + 1], g[8 * kb + 2], g[8 * kb + 3]};
                const float g1[4] = {g[8 * kb + 4], g[8 * kb + 5], g[8 * kb + 6], g[8 * kb + 7]};
                ds_quad(p4.x, p4.y, g0, w[0], w[1]);
                ds_quad(p4.z, p4.w, g1, w[2], w[3]);
            };
            {
#pragma unroll
                for (int kbg = 0; kbg < 4; ++kbg) {
                    const uint4 p4 = *(const uint4 *)(pp + kbg * 1024 + lane * 16);
                    uint32_t w[4];
                    ds_half(p4, dp[kbg >> 1], kbg & 1, w);
                    const bf16x8 db = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) acc[tt] = mfma32(fa.cols(prv, tt, kbg), db, acc[tt]);
                    SB();
                }
            }
            round_end();
            ++T;
        }
    }
    // rounds without work for this pair: keep fetching and meeting the others
#pragma unroll 1
    for (; T <= n_iter; ++T) {
        round_begin(T);
        round_end();
    }
    // (the last round ended with a barrier: nobody reads a tile or P any more)
    if (wave_active) {
        if (hs == 1) {
            Stage st;
            st.init(lane);
            st.put_acc(stage, acc, role == 0 ? 1.0f : prm.scale, n, h);
            st.store(stage, (role == 0 ? prm.dv : prm.dk) + ((size_t)kbase * prm.Hkv + c) * D,
                     (uint32_t)prm.Hkv * D * 2, wj0, kvl);
        } else if (my_j < kvl) {
            const size_t off = ((size_t)(kbase + my_j) * prm.Hkv + c) * D;
            const size_t part = (size_t)hp * prm.total_k * prm.Hkv * D;
            store_rows_f32<TT>((role == 0 ? prm.dv_part : prm.dk_part) + part + off, acc, h);
        }
    }
    trace_end(prm.trace_dkv, trace_t0, bid);
}

template <int D, int PAIRS>
__global__ __launch_bounds__(128 * PAIRS, PAIRS == PAIRS_12W ? 3 : 2) void dkv_kernel(const BwdParams prm)
{
    __shared__ int work_slot;
    work_loop(prm.queue_dkv, prm.n_work_dkv, &work_slot,
              [&](int w) __attribute__((always_inline)) { dkv_work<D, PAIRS>(prm, w); });
}

// Sum of the head-split partial gradients, rounded once: out = bf16(mul * sum_p part[p]).
__global__ __launch_bounds__(256) void dkv_reduce_kernel(const float *__restrict__ part, int32_t parts,
                                                         int64_t n4, float mul, uint16_t *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    float4 a = ((const float4 *)part)[i];
    for (int32_t p = 1; p < parts; ++p) {
        const float4 b = ((const float4 *)part)[(int64_t)p * n4 + i];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    uint2 w;
    w.x = pack_bf16(a.x * mul, a.y * mul);
    w.y = pack_bf16(a.z * mul, a.w * mul);
    ((uint2 *)out)[i] = w;
}

// true when the dQ kernel runs in its 4-wavefront shape (it fits the LDS twice only at head_dim 64)
bool small_dq_shape(const skrull_attn_plan_t *p) { return p->d == 64 && p->wg_query_rows == 32 * NWQ_SMALL; }
int dkv_pairs(const skrull_attn_plan_t *p) { return (p->d == 64 && p->BN == 32 * PAIRS_12W) ? PAIRS_12W : PAIRS_8W; }

template <auto KernelQ, auto KernelKV>
hipError_t launch_pair(const skrull_attn_plan_t *p, BwdParams prm, int threads_q, int threads_kv, hipStream_t st,
                       hipEvent_t *ev)
{
    // dQ first: it also leaves -D and LSE*log2(e) of every (head, row) in the workspace,
    // which dK/dV reads.  Events: ev[0] start, ev[1] after dQ, ev[2] after dK/dV.
    if (ev) (void)hipEventRecord(ev[0], st);
    const bool queued_q = wants_queue<KernelQ>(threads_q, prm.n_work_dq);
    const bool queued_kv = wants_queue<KernelKV>(threads_kv, prm.n_work_dkv);
    if (queued_q || queued_kv) {
        queue_reset_kernel<<<1, 64, 0, st>>>(prm.queue_dq, 2);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (!queued_q) prm.queue_dq = nullptr;
    if (!queued_kv) prm.queue_dkv = nullptr;
    hipError_t e = launch_work<KernelQ>(threads_q, prm.n_work_dq, queued_q, prm, st);
    if (e != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[1], st);
    e = launch_work<KernelKV>(threads_kv, prm.n_work_dkv, queued_kv, prm, st);
    if (e != hipSuccess) return e;
    if (p->head_split > 1) {
        const int64_t n4 = (int64_t)p->total_k * p->Hkv * p->d / 4;
        const unsigned blocks = (unsigned)((n4 + 255) / 256);
        dkv_reduce_kernel<<<blocks, 256, 0, st>>>(prm.dk_part, p->head_split, n4, prm.scale, prm.dk);
        dkv_reduce_kernel<<<blocks, 256, 0, st>>>(prm.dv_part, p->head_split, n4, 1.0f, prm.dv);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (ev) (void)hipEventRecord(ev[2], st);
    return hipGetLastError();
}

template <int D>
hipError_t launch_d(const skrull_attn_plan_t *p, const BwdParams &prm, hipStream_t st, hipEvent_t *ev)
{
    if constexpr (D == 64) {  // the small dQ shape fits the LDS twice, and dK/dV has its 12-wavefront shape, only here
        const bool small_q = small_dq_shape(p), wide_kv = dkv_pairs(p) == PAIRS_12W;
        if (small_q && wide_kv)
            return launch_pair<dq_kernel<D, NWQ_SMALL>, dkv_kernel<D, PAIRS_12W>>(p, prm, 64 * NWQ_SMALL, 128 * PAIRS_12W, st, ev);
        if (small_q)
            return launch_pair<dq_kernel<D, NWQ_SMALL>, dkv_kernel<D, PAIRS_8W>>(p, prm, 64 * NWQ_SMALL, 128 * PAIRS_8W, st, ev);
        if (wide_kv)
            return launch_pair<dq_kernel<D, NWQ_LARGE>, dkv_kernel<D, PAIRS_12W>>(p, prm, 64 * NWQ_LARGE, 128 * PAIRS_12W, st, ev);
    }
    return launch_pair<dq_kernel<D, NWQ_LARGE>, dkv_kernel<D, PAIRS_8W>>(p, prm, 64 * NWQ_LARGE, 128 * PAIRS_8W, st, ev);
}

}  // namespace

int grid_dq(const skrull_attn_plan_t *p)
{
    const int subs = small_dq_shape(p) ? (p->BM + 32 * NWQ_SMALL - 1) / (32 * NWQ_SMALL) : 1;
    return p->n_fwd * p->Hq * subs;
}

int grid_dkv(const skrull_attn_plan_t *p)
{
    const int pairs = dkv_pairs(p);
    return p->n_dkv * p->Hkv * p->head_split * ((p->BN + 32 * pairs - 1) / (32 * pairs));
}

hipError_t launch_bwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      const void *o, const float *lse, const void *d_o, void *dq, void *dk,
                      void *dv, float *delta, hipStream_t st, hipEvent_t *ev, WgTrace *trace)
{
    BwdParams prm;
    prm.trace_dq = trace;
    prm.trace_dkv = trace ? trace + grid_dq(p) : nullptr;
    prm.q = (const uint16_t *)q; prm.k = (const uint16_t *)k; prm.v = (const uint16_t *)v;
    prm.d_o = (const uint16_t *)d_o; prm.o = (const uint16_t *)o; prm.lse = lse; prm.delta = delta;
    prm.lse2 = delta + (size_t)p->Hq * p->total_q;
    prm.dq = (uint16_t *)dq; prm.dk = (uint16_t *)dk; prm.dv = (uint16_t *)dv;
    prm.fwd_items = (const int4 *)p->fwd_items; prm.dkv_items = (const int4 *)p->dkv_items;
    prm.cu_q = p->cu_q; prm.cu_k = p->cu_k; prm.q_begin = p->q_begin; prm.q_len = p->q_len;
    prm.kv_len = p->kv_len; prm.shares_kv = p->shares_kv;
    prm.Hq = p->Hq; prm.Hkv = p->Hkv; prm.total_q = p->total_q; prm.BM = p->BM; prm.BN = p->BN;
    prm.scale = p->scale; prm.scale_log2 = p->scale * kLog2e;
    prm.head_split = p->head_split; prm.total_k = p->total_k;
    prm.n_work_dq = grid_dq(p);
    prm.n_work_dkv = grid_dkv(p);
    {
        // workspace: -D | LSE*log2e | (256-byte aligned) two work queues in 256 bytes | dK partials | dV partials
        const size_t rows = (((size_t)p->Hq * p->total_q * 8) + 255) & ~(size_t)255;
        prm.queue_dq = (WorkQueue *)((char *)delta + rows);
        prm.queue_dkv = prm.queue_dq + 1;
        prm.dk_part = (float *)((char *)delta + rows + 256);
        prm.dv_part = prm.dk_part + (size_t)p->head_split * p->total_k * p->Hkv * p->d;
    }
    if (p->d == 128) return launch_d<128>(p, prm, st, ev);
    if (p->d == 64) return launch_d<64>(p, prm, st, ev);
    return hipErrorInvalidValue;
}
